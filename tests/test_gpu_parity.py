"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
byte for byte, on the same seeded inputs.  Integer / byte work: bit-exact."""

import numpy as np
import pytest

from oracle.kv_oracle import AllocChecker
from paper_2411_18424_amd import synth

pytestmark = pytest.mark.gpu

MiB = 1 << 20


@pytest.fixture
def harness():
    made = []

    def make(shape, cfg=1, host_bytes=64 * MiB, **kw):
        from gpu_util import Harness
        h = Harness(shape, cfg, host_bytes, **kw)
        made.append(h)
        return h

    yield make
    for h in made:
        h.close()


def _tiny_requests(cfg=1):
    rng = synth.rng_for(cfg)
    lens = synth.lengths_uniform(rng, 8, 16, 256)
    nblk = synth.blocks_for(lens, synth.TINY.block_size)
    tables = synth.deal_tables(rng, synth.TINY.n_blocks, nblk, run=1)
    tables2 = synth.deal_tables(rng, synth.TINY.n_blocks, nblk, run=1)
    return lens, tables, tables2


def test_tiny_pool_swap_all_out_then_in(harness):
    """Config 1: 8 requests out to pinned host, then back through a fresh permutation."""
    h = harness(synth.TINY)
    lens, tables, tables2 = _tiny_requests()
    before = [h.oracle.token_kv(t, int(n)) for t, n in zip(tables, lens)]
    for r, t in enumerate(tables):
        h.pool.swap_out(r, t)
        h.oracle.swap_out(r, t)
    for r in range(len(tables)):
        h.assert_image_equal(r)
    h.assert_pool_equal()  # a swap-out changes nothing on the GPU
    # the preempted requests' blocks get reused by others
    junk = np.full((int(sum(len(t) for t in tables)), h.shape.P, h.shape.C), 0xEE, np.uint8)
    h.overwrite_blocks(np.concatenate(tables), junk)
    for r, t in enumerate(tables2):
        h.pool.swap_in(r, t)
        h.oracle.swap_in(r, t)
    h.pool.kv_wait_all()
    h.assert_pool_equal()
    for r, (t, n) in enumerate(zip(tables2, lens)):
        assert np.array_equal(h.oracle.token_kv(t, int(n)), before[r])
    st = h.pool.kv_stats()
    assert st["bytes_out"] == h.oracle.bytes_out and st["bytes_in"] == h.oracle.bytes_in


def test_batched_calls_match_oracle(harness):
    h = harness(synth.TINY, cfg=2)
    _, tables, tables2 = _tiny_requests(cfg=2)
    reqs = list(range(100, 100 + len(tables)))
    h.pool.swap_out_batch(reqs, tables)
    for r, t in zip(reqs, tables):
        h.oracle.swap_out(r, t)
    for r in reqs:
        h.assert_image_equal(r)
    h.pool.swap_in_batch(reqs, tables2)
    for r, t in zip(reqs, tables2):
        h.oracle.swap_in(r, t)
    h.pool.kv_wait_all()
    h.assert_pool_equal()


@pytest.mark.parametrize("L,H,D,B,e,N", [
    (1, 1, 8, 1, 2, 64),       # C = 16 bytes: one vector per chunk
    (3, 3, 40, 16, 2, 96),     # C = 3840: ragged tail inside a tile
    (2, 5, 24, 16, 2, 128),    # C = 3840*... = 3840? (5*24*16*2 = 3840)
    (2, 7, 72, 16, 2, 64),     # C = 16128: several tiles + ragged tail
    (4, 8, 128, 16, 2, 64),    # C = 32 KiB: full-tile fast path, 8 vectors per lane
    (2, 40, 128, 16, 2, 24),   # C = 160 KiB: 5 tiles per chunk
    (2, 4, 64, 16, 1, 64),     # 1-byte elements (fp8 KV): C = 4 KiB
    (1, 2, 96, 16, 4, 48),     # 4-byte elements: C = 12 KiB
])
def test_shapes_and_ragged_chunks(harness, L, H, D, B, e, N):
    shape = synth.KVShape("s", L, H, D, B, e, N, "fp16")
    h = harness(shape, cfg=3, fill="random")  # random bytes: NaN / Inf patterns included
    rng = synth.rng_for(3, stream=L * 1000 + H)
    nblk = [1, 2, 5, N // 4]
    tables = synth.deal_tables(rng, N, nblk)
    tables2 = synth.deal_tables(rng, N, nblk)
    for r, t in enumerate(tables):
        h.pool.swap_out(r, t)
        h.oracle.swap_out(r, t)
        h.assert_image_equal(r)
    for r, t in enumerate(tables2):
        h.pool.swap_in(r, t)
        h.oracle.swap_in(r, t)
    h.pool.kv_wait_all()
    h.assert_pool_equal()


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 7])
@pytest.mark.parametrize("unroll", [0, 1, 2, 4, 8])
def test_every_tile_width_and_kernel_variant(harness, unroll, variant):
    shape = synth.KVShape("s", 2, 6, 80, 16, 2, 80, "bf16")  # C = 30720: full for U<=2, ragged for 4, 8
    h = harness(shape, cfg=4, fill="random", tile_unroll=unroll, pack_variant=variant)
    rng = synth.rng_for(4)
    t = rng.permutation(80)[:33].astype(np.int32)
    t2 = rng.permutation(80)[:33].astype(np.int32)
    h.pool.swap_out(0, t)
    h.oracle.swap_out(0, t)
    h.assert_image_equal(0)
    h.pool.swap_in(0, t2)
    h.oracle.swap_in(0, t2)
    h.pool.kv_wait_all()
    h.assert_pool_equal()


@pytest.mark.parametrize("m", [64, 65, 79, 80, 111])
@pytest.mark.parametrize("L,H,D", [(2, 4, 64), (3, 3, 40), (1, 40, 128)])  # C = 8 KiB, 3840 B, 160 KiB
def test_xcd_aware_order_with_short_last_groups(harness, L, H, D, m):
    """Launches of 64 blocks or more walk the tiles in XCD-aware order (groups of 16 blocks);
    block counts that are not a multiple of 16 leave the last group short."""
    shape = synth.KVShape("s", L, H, D, 16, 2, 160, "fp16")
    for variant in (0, 2):  # XCD-aware order, plain 3-D grid
        h = harness(shape, cfg=35, fill="random", pack_variant=variant, host_bytes=128 * MiB)
        rng = synth.rng_for(35, stream=m)
        t = rng.permutation(160)[:m].astype(np.int32)
        t2 = rng.permutation(160)[:m].astype(np.int32)
        h.pool.swap_out(0, t)
        h.oracle.swap_out(0, t)
        h.assert_image_equal(0)
        h.pool.swap_in(0, t2)
        h.oracle.swap_in(0, t2)
        h.pool.kv_wait_all()
        h.assert_pool_equal()


def test_ring_wraps_when_request_exceeds_staging(harness):
    shape = synth.TINY
    # rings of 7 block records, pieces of 3: a 16-block request wraps the ring twice and
    # has to interleave gathers with copies
    h = harness(shape, cfg=5, staging_out_bytes=7 * shape.R, staging_in_bytes=7 * shape.R,
                max_piece_bytes=3 * shape.R, copy_chunk_bytes=40000)
    rng = synth.rng_for(5)
    tables = synth.deal_tables(rng, shape.n_blocks, [16, 7, 16, 1])
    tables2 = synth.deal_tables(rng, shape.n_blocks, [16, 7, 16, 1])
    for r, t in enumerate(tables):
        h.pool.swap_out(r, t)
        h.oracle.swap_out(r, t)
    for r in range(4):
        h.assert_image_equal(r)
    for r, t in enumerate(tables2):
        h.pool.swap_in(r, t)
        h.oracle.swap_in(r, t)
    h.pool.kv_wait_all()
    h.assert_pool_equal()
    st = h.pool.kv_stats()
    assert st["gather_launches"] == 6 + 3 + 6 + 1
    assert st["d2h_copies"] > st["gather_launches"]  # copies are also cut at 40000 bytes


@pytest.mark.parametrize("variant", [0, 1])
def test_more_blocks_than_one_launch_carries(harness, variant):
    """A launch carries at most 896 table entries: 2500 blocks need 3 launches."""
    shape = synth.KVShape("s", 1, 1, 32, 16, 2, 4096, "fp16")  # C = 1 KiB, R = 2 KiB
    h = harness(shape, cfg=6, fill="random", pack_variant=variant)
    rng = synth.rng_for(6)
    t = rng.permutation(4096)[:2500].astype(np.int32)
    t2 = rng.permutation(4096)[:2500].astype(np.int32)
    h.pool.swap_out(0, t)
    h.oracle.swap_out(0, t)
    h.assert_image_equal(0)
    h.pool.swap_in(0, t2)
    h.oracle.swap_in(0, t2)
    h.pool.kv_wait_all()
    h.assert_pool_equal()
    assert h.pool.kv_stats()["gather_launches"] >= 3


def test_multi_turn_delta_and_contamination(harness):
    """Section 3.3 flow: keep the host copy, move only dirty / invalid blocks, grow the image."""
    shape = synth.TINY
    h = harness(shape, cfg=7, host_slack_blocks=4)
    rng = synth.rng_for(7)
    B = shape.block_size
    tokens = 5 * B - 3
    perm = rng.permutation(shape.n_blocks).astype(np.int32)
    cursor = 5
    table = perm[:5].copy()
    h.pool.swap_out(0, table)
    h.oracle.swap_out(0, table)
    h.assert_image_equal(0)
    for turn in range(6):
        # resume into fresh blocks
        new_table = perm[cursor:cursor + len(table)].copy()
        cursor += len(table)
        h.pool.swap_in(0, new_table)
        h.oracle.swap_in(0, new_table)
        h.pool.kv_wait(0)
        h.assert_pool_equal()
        # the turn appends tokens: tail block changes, new blocks appear
        new_tokens = int(rng.integers(1, 4 * B))
        n_old = len(new_table)
        dirty = synth.turn_dirty_mask(n_old, tokens, new_tokens, B)
        extra = len(dirty) - n_old
        grown = np.concatenate([new_table, perm[cursor:cursor + extra]]).astype(np.int32)
        cursor += extra
        touched = np.flatnonzero(dirty)
        h.overwrite_blocks(grown[touched], synth.fresh_tokens(rng, shape, len(touched)))
        tokens += new_tokens
        if turn % 2 == 1:  # part of the host copy was reclaimed meanwhile
            inval = synth.random_mask(rng, n_old, 0.3)
            h.pool.kv_host_invalidate(0, inval)
            h.oracle.host_invalidate(0, inval)
        moved = h.pool.swap_out_delta(0, grown, dirty)
        want = h.oracle.swap_out_delta(0, grown, dirty)
        assert moved == len(want)
        h.assert_image_equal(0)
        table = grown
    st = h.pool.kv_stats()
    assert st["bytes_out"] == h.oracle.bytes_out
    assert st["bytes_in"] == h.oracle.bytes_in
    assert st["host_new_extents"] >= 1 or st["host_arena_used"] > 0


@pytest.mark.parametrize("flags", [0, 256], ids=["strided_copies", "one_copy_per_run"])
def test_scattered_dirty_blocks_and_scattered_swap_in(harness, flags):
    """Random 20 % dirty masks over a 200-block image, three turns, and swap-ins that skip a
    random resident set: the scattered records travel as rows of 2-D copies (or one by one),
    the image and the pool must match the oracle byte for byte either way."""
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 512, "bf16")  # R = 512 KiB
    h = harness(shape, cfg=37, host_bytes=256 * MiB, fill="random", flags=flags, host_slack_blocks=8)
    rng = synth.rng_for(37)
    t = rng.permutation(512)[:200].astype(np.int32)
    h.pool.swap_out(0, t)
    h.oracle.swap_out(0, t)
    # a second image right behind the first one, so that growth opens a second extent
    other = np.setdiff1d(np.arange(512), t)[:20].astype(np.int32)
    h.pool.swap_out(1, other)
    h.oracle.swap_out(1, other)
    h.assert_image_equal(0)
    spare = np.setdiff1d(np.arange(512), np.concatenate([t, other])).astype(np.int32)
    for turn in range(3):
        grow = spare[turn * 15:(turn + 1) * 15]
        t = np.concatenate([t, grow]).astype(np.int32)
        dirty = synth.random_mask(rng, t.size, 0.2)
        dirty[-15:] = 1
        touched = np.flatnonzero(dirty)
        h.overwrite_blocks(t[touched], synth.fresh_tokens(rng, shape, touched.size))
        moved = h.pool.swap_out_delta(0, t, dirty)
        want = h.oracle.swap_out_delta(0, t, dirty)
        assert moved == len(want)
        h.assert_image_equal(0)
        # scramble the request's GPU blocks, keep a random resident set, bring the rest back
        resident = synth.random_mask(rng, t.size, 0.6)
        lost = np.flatnonzero(resident == 0)
        h.overwrite_blocks(t[lost], np.full((lost.size, shape.P, shape.C), 0xDD, np.uint8))
        assert h.pool.swap_in_delta(0, t, resident) == len(h.oracle.swap_in(0, t, resident=resident))
        h.pool.kv_wait(0)
        h.assert_pool_equal()
    st = h.pool.kv_stats()
    assert (st["strided_copies"] > 0) == (flags == 0)
    assert st["bytes_out"] == h.oracle.bytes_out and st["bytes_in"] == h.oracle.bytes_in


@pytest.mark.parametrize("flags", [1024, 1024 | 8], ids=["two_streams", "four_streams"])
def test_scattered_records_over_both_copy_streams(harness, flags):
    """KV_FLAG_SECOND_LANE: the scattered 1 MiB records of a delta swap-out travel as plain copies,
    every other one on the host-to-device stream, unless a swap-in is in flight; images and pool
    must match the oracle byte for byte, also when a swap-in follows at once on that stream."""
    shape = synth.KVShape("s", 16, 8, 128, 16, 2, 512, "bf16")  # R = 1 MiB
    h = harness(shape, cfg=39, host_bytes=400 * MiB, fill="random", flags=flags, host_slack_blocks=8)
    rng = synth.rng_for(39)
    perm = rng.permutation(512).astype(np.int32)
    t, other, spare = perm[:200], perm[200:260], perm[260:320]
    h.pool.swap_out(0, t)
    h.oracle.swap_out(0, t)
    h.pool.swap_out(1, other)
    h.oracle.swap_out(1, other)
    h.pool.kv_wait_all()
    for turn in range(4):
        dirty = synth.random_mask(rng, t.size, 0.25)
        touched = np.flatnonzero(dirty)
        h.overwrite_blocks(t[touched], synth.fresh_tokens(rng, shape, touched.size))
        if turn == 2:      # a swap-in is in flight: the host-to-device stream is not idle
            h.pool.swap_in(1, spare)
            h.oracle.swap_in(1, spare)
        moved = h.pool.swap_out_delta(0, t, dirty)
        assert moved == len(h.oracle.swap_out_delta(0, t, dirty))
        if turn == 1:      # a swap-in right behind the swap-out, on the stream that carries half of its copies
            h.pool.swap_in(1, spare)
            h.oracle.swap_in(1, spare)
        h.pool.kv_wait_all()
        h.assert_image_equal(0)
        h.assert_pool_equal()
        if turn in (1, 2):
            h.pool.swap_out(1, spare)
            h.oracle.swap_out(1, spare)
            h.pool.kv_wait(1)
            other, spare = spare, other
    st = h.pool.kv_stats()
    assert st["second_lane_copies"] > 0 and st["bytes_out"] == h.oracle.bytes_out


def test_partial_swap_in_moves_only_non_resident_blocks(harness):
    h = harness(synth.TINY, cfg=8)
    rng = synth.rng_for(8)
    t, t2 = synth.deal_tables(rng, 256, [12])[0], synth.deal_tables(rng, 256, [12])[0]
    h.pool.swap_out(0, t)
    h.oracle.swap_out(0, t)
    res = synth.random_mask(rng, 12, 0.5)
    res[0], res[1] = 1, 0
    moved = h.pool.swap_in_delta(0, t2, res)
    want = h.oracle.swap_in(0, t2, resident=res)
    assert moved == len(want)
    h.pool.kv_wait(0)
    h.assert_pool_equal()


def test_swap_in_over_blocks_still_being_gathered(harness):
    """Conflict (Section 3.2): request B resumes into the blocks request A is leaving."""
    shape = synth.KVShape("s", 4, 8, 128, 16, 2, 96, "bf16")
    h = harness(shape, cfg=9, host_bytes=256 * MiB)
    rng = synth.rng_for(9)
    ta, tb = synth.deal_tables(rng, 96, [40, 40])
    h.pool.swap_out(1, tb)
    h.oracle.swap_out(1, tb)
    h.pool.kv_wait(1)
    for rep in range(3):
        h.pool.swap_out(0, ta)            # A's blocks are being read ...
        h.pool.swap_in(1, ta[::-1].copy())  # ... while B is written into them
        h.oracle.swap_out(0, ta)
        h.oracle.swap_in(1, ta[::-1].copy())
        h.assert_image_equal(0)
        h.pool.kv_wait(1)
        h.assert_pool_equal()
        # and the reverse hazard: gather blocks whose scatter is still in flight
        h.pool.swap_in(0, tb)
        h.pool.swap_out(1, tb)
        h.oracle.swap_in(0, tb)
        h.oracle.swap_out(1, tb)
        h.assert_image_equal(1)
        h.pool.kv_wait_all()
        h.assert_pool_equal()
        ta, tb = tb, ta


def test_allocator_driven_flow(harness):
    """Tables come from alloc_block_group; blocks are freed right after swap_out is enqueued
    and may be handed out again only once their gather has finished."""
    shape = synth.KVShape("s", 4, 8, 128, 16, 2, 128, "bf16")
    h = harness(shape, cfg=10, host_bytes=512 * MiB)
    chk = AllocChecker(shape.n_blocks)
    rng = synth.rng_for(10)
    live = {}
    for r in range(6):
        ids, runs = h.pool.alloc_block_group(r, 20, 8)
        rl = chk.on_alloc(r, ids)
        assert runs == len(rl)
        live[r] = ids
        h.overwrite_blocks(ids, synth.fresh_tokens(rng, shape, len(ids)))
    # preempt 0..2, resume them later into whatever the allocator returns
    for r in range(3):
        h.pool.swap_out(r, live[r])
        h.oracle.swap_out(r, live[r])
        h.pool.free_block_group(r, live[r])
        chk.on_free(r, live[r])
    for r in range(3):
        ids, _ = h.pool.alloc_block_group(r, 20, 8)
        chk.on_alloc(r, ids)
        h.pool.swap_in(r, ids)
        h.oracle.swap_in(r, ids)
        live[r] = ids
    h.pool.kv_wait_all()
    for r in range(3):
        h.assert_image_equal(r)
    h.assert_pool_equal()
    free, _ = h.pool.kv_free_blocks()
    assert free + chk.n_used() == shape.n_blocks


def test_blocks_freed_during_a_swap_in_are_held_back(harness):
    """A request is resumed and its blocks are given up at once (it is preempted again before
    anything ran, or it ends): the allocator must not hand them out while the scatter still
    writes them, or the next owner's KV would be overwritten."""
    import torch
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 1024, "bf16")  # R = 512 KiB, 512 MiB pool
    h = harness(shape, cfg=33, host_bytes=512 * MiB, fill="random")
    ids, _ = h.pool.alloc_block_group(0, 600, 8)
    h.pool.swap_out(0, ids)
    h.oracle.swap_out(0, ids)
    h.pool.kv_wait(0)
    h.pool.free_block_group(0, ids)
    stream = torch.cuda.Stream()
    view = h.gpu.view(shape.P, shape.n_blocks, shape.C)
    for rep in range(3):
        ids, _ = h.pool.alloc_block_group(0, 600, 8)
        h.pool.swap_in(0, ids)                 # 300 MiB over the link: several milliseconds
        h.pool.free_block_group(0, ids)        # ... and the blocks are given up at once
        other, _ = h.pool.alloc_block_group(1, 900, 8)   # needs most of them back
        idx = torch.from_numpy(other.astype(np.int64)).to(h.dev)
        with torch.cuda.stream(stream):
            view[:, idx, :] = 0x30 + rep       # the next owner writes its KV right away
        stream.synchronize()
        h.oracle.swap_in(0, ids)
        h.oracle.G[:, other.astype(np.int64), :] = 0x30 + rep
        h.pool.kv_wait_all()
        h.assert_pool_equal()
        h.pool.free_block_group(1, other)
    assert h.pool.kv_stats()["conflict_waits"] >= 3


@pytest.mark.parametrize("flags", [0, 8, 128], ids=["two_streams", "four_streams", "three_streams"])
def test_swap_ins_into_the_same_blocks_land_in_call_order(harness, flags):
    """Raw tables, no allocator in between: two requests are swapped in to the same blocks by
    different paths (staged scatter, then 2-D copies on the copy stream); the later call wins."""
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 512, "bf16")  # R = 512 KiB
    h = harness(shape, cfg=34, host_bytes=512 * MiB, fill="random", flags=flags)
    rng = synth.rng_for(34)
    ta, tb, target = (rng.permutation(512)[:200].astype(np.int32) for _ in range(3))
    for r, t in ((0, ta), (1, tb)):
        h.pool.swap_out(r, t)
        h.oracle.swap_out(r, t)
    h.pool.kv_wait_all()
    for rep in range(3):
        h.pool.swap_in(0, target)
        h.pool.swap_in_direct(1, target[::-1].copy())
        h.pool.swap_in(0, target)
        h.pool.swap_in_direct(1, target)
        h.oracle.swap_in(0, target)
        h.oracle.swap_in(1, target[::-1].copy())
        h.oracle.swap_in(0, target)
        h.oracle.swap_in(1, target)
        h.pool.kv_wait_all()
        h.assert_pool_equal()


@pytest.mark.parametrize("flags", [0, 8, 128], ids=["two_streams", "four_streams", "three_streams"])
def test_older_writer_on_another_stream_is_waited_for(harness, flags):
    """Three swap-ins, no host wait between them: a slow one by per-block copies on the copy
    stream into blocks Ta, a small staged one into Tb, then one over Ta and Tb together.  The
    last call's scatter must land after BOTH earlier writers although conflict detection waits
    for the newest of them only: completion events of a direction fire in issue order."""
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 512, "bf16")  # R = 512 KiB
    h = harness(shape, cfg=35, host_bytes=512 * MiB, fill="random", flags=flags)
    rng = synth.rng_for(35)
    perm = rng.permutation(512).astype(np.int32)
    src_a, src_b, src_c = perm[:200], perm[200:204], perm[204:408]
    ta, tb = perm[408:508][:96], perm[508:512]
    ta = np.concatenate([ta, perm[:104]])          # 200 blocks for request 0
    for r, t in ((0, src_a), (1, src_b), (2, src_c)):
        h.pool.swap_out(r, t)
        h.oracle.swap_out(r, t)
    h.pool.kv_wait_all()
    for rep in range(2):
        h.pool.swap_in_direct(0, ta, per_block=True)   # 3200 small copies: slow
        h.pool.swap_in(1, tb)
        h.pool.swap_in(2, np.concatenate([ta, tb]))
        h.oracle.swap_in(0, ta)
        h.oracle.swap_in(1, tb)
        h.oracle.swap_in(2, np.concatenate([ta, tb]))
        h.pool.kv_wait(2)
        h.assert_pool_equal()
        ta = ta[::-1].copy()


def test_full_swap_out_of_a_grown_request_while_its_swap_in_is_in_flight(harness):
    """A request is swapped in and, before that has finished, swapped out in full with a table
    that no longer fits its old host image: the old image must not be given back under the
    running swap-in, and the new op must not be reported done before it has run."""
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 1024, "bf16")  # R = 512 KiB
    h = harness(shape, cfg=36, host_bytes=600 * MiB, fill="random")
    rng = synth.rng_for(36)
    perm = rng.permutation(1024).astype(np.int32)
    t1, t2, extra = perm[:300], perm[300:600], perm[600:700]
    h.pool.swap_out(7, t1)
    h.oracle.swap_out(7, t1)
    h.pool.kv_wait(7)
    for rep in range(2):
        grown = np.concatenate([t2, extra])   # 400 blocks > 300 + 32 of slack: the image is rebuilt
        h.pool.swap_in(7, t2)                 # 150 MiB, about 3 ms on the link
        h.pool.swap_out(7, grown)             # 200 MiB, issued at once
        done_at_once = h.pool.kv_query(7)
        h.oracle.swap_in(7, t2)
        h.oracle.swap_out(7, grown)
        assert not done_at_once, "a 200 MiB swap-out cannot be complete microseconds after the call"
        h.pool.kv_wait_packed(7)
        h.assert_image_equal(7)
        h.assert_pool_equal()
        # back to 300 blocks through a different table for the second round
        h.pool.kv_host_release(7)
        h.oracle.host_release(7)
        h.pool.swap_out(7, t1)
        h.oracle.swap_out(7, t1)
        h.pool.kv_wait(7)
        t2 = perm[700:1000]


@pytest.mark.parametrize("flags", [0, 8, 128], ids=["two_streams", "four_streams", "three_streams"])
def test_swap_out_copies_held_back_until_the_gathers_are_done(harness, flags):
    """A swap-out of 16 MiB or more returns with its gathers enqueued and its copies in the
    hands of the pool's copy thread.  Whatever is called next - a swap-in of another request, a
    swap-in of the same request, a stream wait, a host read, another swap-out, the release of
    the image - must see the same bytes as with KV_FLAG_NO_DEFER_COPIES, and completion is not reported
    before the copies have run."""
    import torch
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 1024, "bf16")  # R = 512 KiB
    h = harness(shape, cfg=37, host_bytes=700 * MiB, fill="random", flags=flags,
                staging_out_bytes=96 * MiB, max_piece_bytes=16 * MiB)
    rng = synth.rng_for(37)
    perm = rng.permutation(1024).astype(np.int32)
    ta, tb, tc, td = perm[:300], perm[300:500], perm[500:800], perm[800:1000]
    h.pool.swap_out(2, tb)
    h.oracle.swap_out(2, tb)
    h.pool.kv_wait(2)
    side = torch.cuda.Stream()
    for rep in range(3):
        # request 1 leaves (150 MiB: larger than the out ring, so the call also drains pieces itself),
        # request 2 comes back into other blocks at once, then request 1 follows it back in
        h.pool.swap_out(1, ta)
        done_at_once = h.pool.kv_query(1)
        h.pool.swap_in(2, td)
        h.oracle.swap_out(1, ta)
        h.oracle.swap_in(2, td)
        assert not done_at_once  # 150 MiB take 2.6 ms on the link
        if rep == 0:
            h.pool.kv_stream_wait(1, side.cuda_stream)   # needs the completion event to exist
            side.synchronize()
            assert h.pool.kv_query(1)
        elif rep == 1:
            h.assert_image_equal(1)                      # a host read right behind the call
        h.pool.swap_in(1, tc)                            # follows the swap-out of the same request
        h.oracle.swap_in(1, tc)
        h.pool.swap_out(2, td)                           # the next swap-out waits for the hand-over
        h.oracle.swap_out(2, td)
        h.pool.kv_wait(1)
        h.pool.kv_wait(2)
        h.assert_pool_equal()
        h.assert_image_equal(1)
        h.assert_image_equal(2)
        ta, tc = tc, ta
        tb, td = td, tb
    st = h.pool.kv_stats()
    assert st["blocks_out"] == 200 + 3 * 500 and st["blocks_in"] == 3 * 500
    h.pool.swap_out(1, ta)
    h.pool.kv_host_release(1)   # gives the image back: only after the held-back copies have run
    h.pool.swap_out(2, tb)      # and the pool is destroyed (by the fixture) with a swap-out just handed over


def test_several_swap_outs_held_back_at_once(harness):
    """Swap-outs of different requests issued back to back: each is enqueued behind the ones whose
    copies are still held back as long as the out ring has room for it, and waits for their
    hand-over when it has not; a small swap-out (copies enqueued inside the call) overtakes them,
    and so does another request's swap-in."""
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 1024, "bf16")  # R = 512 KiB, out ring 128 MiB
    h = harness(shape, cfg=38, host_bytes=600 * MiB, fill="random")
    rng = synth.rng_for(38)
    perm = rng.permutation(1024).astype(np.int32)
    tabs = [perm[i * 44:(i + 1) * 44] for i in range(8)]           # 22 MiB each: held back
    spare = [perm[500 + i * 44:500 + (i + 1) * 44] for i in range(8)]
    small = perm[400:404]                                           # 2 MiB: not held back
    here, there = perm[900:944], perm[950:994]
    h.pool.swap_out(100, here)
    h.oracle.swap_out(100, here)
    h.pool.kv_wait(100)
    for rep in range(2):
        for r in range(8):                     # 176 MiB in all: the later calls wait for ring room
            h.pool.swap_out(r, tabs[r])
            h.oracle.swap_out(r, tabs[r])
            if r == 2:
                h.pool.swap_out(50, small)
                h.oracle.swap_out(50, small)
            if r == 4:
                h.pool.swap_in(100, there)     # another request's swap-in goes ahead
                h.oracle.swap_in(100, there)
        h.pool.kv_wait_all()
        for r in list(range(8)) + [50, 100]:
            assert h.pool.kv_query(r)
            h.assert_image_equal(r)
        h.assert_pool_equal()
        for r in range(8):                     # and back, into other blocks
            h.pool.swap_in(r, spare[r])
            h.oracle.swap_in(r, spare[r])
        h.pool.swap_out(100, there)
        h.oracle.swap_out(100, there)
        h.pool.kv_wait_all()
        h.assert_pool_equal()
        h.assert_image_equal(100)
        tabs, spare = spare, tabs
        here, there = there, here


def test_a_c_caller_reads_host_images_in_the_contract_layout():
    """tests/host/host_read_check.cpp (built by paper_2411_18424_amd.build): kv_host_read and
    kv_host_view from a C++ program, including an image that continues in a second extent."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "host", "host_read_check.bin")
    if not os.path.exists(exe):
        pytest.skip("tests/host/host_read_check.bin is not built (python -m paper_2411_18424_amd.build)")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert run.returncode == 0 and "host_read_check: 0 failures" in run.stdout, run.stdout[-3000:]


def test_empty_request_and_queries(harness):
    h = harness(synth.TINY, cfg=11)
    h.pool.swap_out(0, np.zeros(0, np.int32))
    h.oracle.swap_out(0, [])
    h.pool.kv_wait(0)
    assert h.pool.kv_query(0)
    assert h.pool.kv_host_view(0).shape[0] == 0 and h.pool.kv_host_read(0).shape[0] == 0
    h.pool.swap_in(0, np.zeros(0, np.int32))
    h.pool.kv_wait(0)
    h.assert_pool_equal()


def test_rejected_calls_have_no_effect(harness):
    h = harness(synth.TINY, cfg=12, host_bytes=20 * synth.TINY.R, host_slack_blocks=0)
    kv = h.kv
    t = np.arange(10, 20, dtype=np.int32)
    h.pool.swap_out(0, t)
    h.oracle.swap_out(0, t)
    h.assert_image_equal(0)
    for bad in ([1, 2, 2], [0, 256], [-1, 3]):
        with pytest.raises(kv.KVError) as ei:
            h.pool.swap_out(1, np.array(bad, np.int32))
        assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError) as ei:
        h.pool.swap_in(5, t)
    assert ei.value.status == kv.KV_ENOENT
    with pytest.raises(kv.KVError) as ei:
        h.pool.swap_in(0, t[:5])
    assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError) as ei:
        h.pool.swap_out(2, np.arange(0, 11, dtype=np.int32))  # arena holds 20 records, 10 in use
    assert ei.value.status == kv.KV_ENOMEM_HOST
    h.pool.kv_host_invalidate(0, [1] + [0] * 9)
    h.oracle.host_invalidate(0, [1] + [0] * 9)
    with pytest.raises(kv.KVError) as ei:
        h.pool.swap_in(0, t)
    assert ei.value.status == kv.KV_ENOENT
    h.pool.kv_wait_all()
    h.assert_pool_equal()
    h.assert_image_equal(0)
    st = h.pool.kv_stats()
    assert st["bytes_out"] == 10 * h.shape.R and st["bytes_in"] == 0


def test_ordering_with_the_compute_stream(harness):
    """KV written on the caller's stream just before swap_out must be what gets swapped, and
    a stream made to wait by kv_stream_wait sees the swapped-in bytes."""
    import torch
    shape = synth.KVShape("s", 4, 8, 128, 16, 2, 64, "bf16")
    stream = torch.cuda.Stream()
    from gpu_util import Harness
    h = Harness(shape, 13, 256 * MiB, fill="random",
                flags=4, compute_stream=stream.cuda_stream)  # KV_FLAG_ORDER_COMPUTE
    try:
        rng = synth.rng_for(13)
        t, t2 = synth.deal_tables(rng, 64, [24, 24])
        view = h.gpu.view(shape.P, shape.n_blocks, shape.C)
        idx = torch.from_numpy(t.astype(np.int64)).to(h.dev)
        payload = synth.fresh_tokens(rng, shape, 24)
        dev_payload = torch.from_numpy(np.ascontiguousarray(payload.transpose(1, 0, 2))).to(h.dev)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            for _ in range(20):  # keep the stream busy, last write wins
                view[:, idx, :] = 0
            view[:, idx, :] = dev_payload
        h.pool.swap_out(0, t)  # no host synchronisation in between
        h.oracle.G[:, t.astype(np.int64), :] = payload.transpose(1, 0, 2)
        h.oracle.swap_out(0, t)
        h.assert_image_equal(0)
        h.pool.swap_in(0, t2)
        h.oracle.swap_in(0, t2)
        h.pool.kv_stream_wait(0, stream.cuda_stream)
        with torch.cuda.stream(stream):
            idx2 = torch.from_numpy(t2.astype(np.int64)).to(h.dev)
            got = view[:, idx2, :].clone()
        stream.synchronize()
        assert np.array_equal(got.cpu().numpy(), h.oracle.G[:, t2.astype(np.int64), :])
    finally:
        h.close()


def test_profile_records(harness):
    h = harness(synth.TINY, cfg=14, flags=2)  # KV_FLAG_PROFILE
    t = np.arange(16, dtype=np.int32)
    h.pool.swap_out(0, t)
    h.pool.swap_in(0, t[::-1].copy())
    recs = h.pool.kv_profile_read()
    kinds = sorted(k for k, _, _ in recs)
    assert kinds == [0, 1, 2, 3]
    for k, nbytes, ms in recs:
        assert nbytes == 16 * h.shape.R and ms > 0
    tl = h.pool.kv_profile_timeline()
    assert [(k, b) for k, b, _, _ in tl] == [(k, b) for k, b, _ in recs]
    starts = {k: t0 for k, _, t0, _ in tl}
    assert tl[0][2] == 0 and all(t0 >= 0 for t0 in starts.values())
    assert starts[0] <= starts[2] <= starts[3] <= starts[1]   # gather, its copy, copy back, scatter
    h.pool.kv_profile_reset()
    assert h.pool.kv_profile_read() == []


def test_probes_report_plausible_rates():
    from paper_2411_18424_amd import kvswap
    hbm = kvswap.kv_hbm_probe(256 * MiB, 3)
    d2h = kvswap.kv_link_probe(64 * MiB, 0, 2)
    h2d = kvswap.kv_link_probe(64 * MiB, 1, 2)
    assert 100 < hbm < 8000
    assert 1 < d2h < 200 and 1 < h2d < 200


@pytest.mark.parametrize("per_block", [False, True])
def test_direct_copy_comparison_path(harness, per_block):
    """The paper-style path (one copy per block group and plane, no pack kernel) must give
    the same bytes as the packed path."""
    shape = synth.KVShape("s", 3, 4, 64, 16, 2, 128, "fp16")
    h = harness(shape, cfg=15, fill="random")
    rng = synth.rng_for(15)
    tables = synth.deal_tables(rng, 128, [20, 7, 1], run=4)
    tables2 = synth.deal_tables(rng, 128, [20, 7, 1], run=1)
    for r, t in enumerate(tables):
        h.pool.swap_out_direct(r, t, per_block)
        h.oracle.swap_out(r, t)
        h.assert_image_equal(r)
    for r, t in enumerate(tables2):
        h.pool.swap_in_direct(r, t, per_block)
        h.oracle.swap_in(r, t)
    h.pool.kv_wait_all()
    h.assert_pool_equal()
    st = h.pool.kv_stats()
    assert st["gather_launches"] == 0 and st["scatter_launches"] == 0
    runs_out = (5 + 2 + 1) if not per_block else 28
    assert st["d2h_copies"] == runs_out * shape.P
    assert st["h2d_copies"] == 28 * shape.P  # fully fragmented resume tables: one copy per block and plane


def test_swap_manager_path_matches_oracle(harness):
    """Swaps submitted through the manager's dispatcher thread give the same bytes; a resume
    into blocks that a queued swap-out is still to read is kept in order."""
    shape = synth.KVShape("s", 4, 8, 128, 16, 2, 128, "bf16")
    h = harness(shape, cfg=16, host_bytes=512 * MiB)
    kv = h.kv
    m = kv.KVManager(h.pool)
    try:
        rng = synth.rng_for(16)
        ta, tb, tc = synth.deal_tables(rng, 128, [30, 30, 20])
        tickets = [m.kv_manager_submit(kv.KV_TASK_SWAP_OUT, 1, tb)]
        h.oracle.swap_out(1, tb)
        for rep in range(4):
            tickets.append(m.kv_manager_submit(kv.KV_TASK_SWAP_OUT, 0, ta))
            tickets.append(m.kv_manager_submit(kv.KV_TASK_SWAP_IN, 1, ta[::-1].copy()))  # into A's blocks
            h.oracle.swap_out(0, ta)
            h.oracle.swap_in(1, ta[::-1].copy())
            tickets.append(m.kv_manager_submit(kv.KV_TASK_SWAP_OUT, 1, ta[::-1].copy()))
            tickets.append(m.kv_manager_submit(kv.KV_TASK_SWAP_IN, 0, tb))
            h.oracle.swap_out(1, ta[::-1].copy())
            h.oracle.swap_in(0, tb)
            ta, tb = tb, ta
        dirty = synth.random_mask(rng, 30, 0.4)
        tickets.append(m.kv_manager_submit(kv.KV_TASK_SWAP_OUT_DELTA, 0, ta, dirty))
        h.oracle.swap_out_delta(0, ta, dirty)
        assert m.kv_manager_wait(tickets[-1]) == kv.KV_OK
        m.kv_manager_drain()
        done = dict(m.kv_manager_poll(64))
        assert set(done) == set(tickets[:-1]) and all(s == kv.KV_OK for s in done.values())
        h.assert_image_equal(0)
        h.assert_image_equal(1)
        h.assert_pool_equal()
    finally:
        m.kv_manager_destroy()


@pytest.mark.parametrize("flags", [0, 128], ids=["two_streams", "three_streams"])
def test_algorithm_1_iterations_match_oracle(harness, flags):
    """A scheduler loop through kv_manager_iterate: every iteration preempts one running request
    and resumes one swapped request - into the very blocks the victim leaves (a KV cache
    conflict, step 3.1) or into spare blocks - asynchronously or synchronously (step 4).  The
    oracle replays every iteration with the conflicting swap-out first; nothing is waited for
    except through the manager."""
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 512, "bf16")  # R = 512 KiB, 30 MiB per request
    h = harness(shape, cfg=38, host_bytes=512 * MiB, fill="random", flags=flags)
    kv = h.kv
    m = kv.KVManager(h.pool)
    try:
        rng = synth.rng_for(38)
        perm = rng.permutation(512).astype(np.int32)
        table = {r: perm[r * 60:(r + 1) * 60] for r in range(6)}
        spare = list(perm[360:])
        running, swapped, ongoing = set(range(6)), [], set()
        stats = {"conflicts": 0, "async": 0, "sync": 0}
        # two requests leave first
        m.kv_manager_iterate(swap_out=[(0, table[0]), (1, table[1])])
        for r in (0, 1):
            h.oracle.swap_out(r, table[r])
            running.discard(r)
            swapped.append(r)
            spare.extend(table.pop(r))
        for k in range(14):
            v = sorted(running)[int(rng.integers(0, len(running)))]
            u = swapped.pop(0)
            n = 60
            if k % 2 == 0:   # the resumed request takes over the victim's blocks
                new = table[v][::-1].copy()
            else:            # or blocks that have been free for a while
                new = np.array(spare[:n], dtype=np.int32)
                del spare[:n]
                spare.extend(int(b) for b in table[v])
            mode = (0, 1, 2)[k % 3]
            resumed, r = m.kv_manager_iterate(swap_in=[(u, new)], swap_out=[(v, table[v])], force_mode=mode)
            h.oracle.swap_out(v, table[v])   # a conflicting swap-out is dispatched first; otherwise
            h.oracle.swap_in(u, new)         # the two touch different blocks and the order is free
            assert r["conflicts"] == (1 if k % 2 == 0 else 0)
            stats["conflicts"] += r["conflicts"]
            stats["async" if r["async"] else "sync"] += 1
            running.discard(v)
            swapped.append(v)
            table.pop(v)
            table[u] = new
            ongoing.add(u)
            for q in resumed:
                assert q in ongoing
                ongoing.discard(q)
                running.add(q)
            if not running:  # the scheduler has nothing to run: it waits for a swap-in (an empty iteration polls)
                while not running:
                    resumed, _ = m.kv_manager_iterate()
                    for q in resumed:
                        ongoing.discard(q)
                        running.add(q)
        m.kv_manager_drain()
        resumed, r = m.kv_manager_iterate()
        for q in resumed:
            ongoing.discard(q)
            running.add(q)
        assert not ongoing and r["ongoing_swap_ins"] == 0 and r["failures"] == 0
        assert stats["conflicts"] == 7 and stats["sync"] >= 4 and stats["async"] >= 4
        for q in swapped:
            h.assert_image_equal(q)
        h.assert_pool_equal()
        st = h.pool.kv_stats()
        assert st["bytes_out"] == h.oracle.bytes_out and st["bytes_in"] == h.oracle.bytes_in
    finally:
        m.kv_manager_destroy()


def test_algorithm_1_with_the_allocator_and_blocks_freed_by_the_dispatcher(harness):
    """The scheduler loop of the benchmark's config 3 in small: tables come from the block-group
    allocator, kv_manager_iterate preempts with KV_IT_FREE_OUT_BLOCKS (the dispatcher frees the
    victim's blocks right after its swap-out is enqueued, so the allocator parks them until the
    gather has read them) and resumes into freshly allocated blocks - often the ones just vacated.
    New KV is written into every request before it leaves; the oracle replays the same calls."""
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 256, "bf16")  # R = 512 KiB; the pool is tight on purpose
    h = harness(shape, cfg=39, host_bytes=400 * MiB, fill="random")
    kv = h.kv
    m = kv.KVManager(h.pool)
    checker = AllocChecker(shape.n_blocks)
    try:
        rng = synth.rng_for(39)
        n_req, lag = 24, 2
        nblk = rng.integers(20, 90, size=n_req)
        out_tab, in_tab, waiting = {}, {}, set()
        for i in range(n_req + lag):
            j = i - lag
            swap_in, swap_out = [], []
            if i < n_req:
                ids, _ = h.pool.alloc_block_group(i, int(nblk[i]), 8)   # waits for parked blocks if it must
                checker.on_alloc(i, ids)
                h.overwrite_blocks(ids, synth.fresh_tokens(rng, shape, len(ids)))  # the request's KV
                out_tab[i] = ids
                swap_out = [(i, ids)]
            if j >= 0:
                ids2, _ = h.pool.alloc_block_group(10**6 + j, int(nblk[j]), 8)
                checker.on_alloc(10**6 + j, ids2)
                in_tab[j] = ids2
                swap_in = [(j, ids2)]
                waiting.add(j)
            resumed, r = m.kv_manager_iterate(swap_in=swap_in, swap_out=swap_out, free_out_blocks=True,
                                              force_mode=1 + i % 2)
            assert r["conflicts"] == 0   # the allocator never hands out a block the iteration's swap-out still owns
            if swap_out:
                h.oracle.swap_out(i, out_tab[i])
                checker.on_free(i, out_tab[i])    # freed by the dispatcher
            if swap_in:
                h.oracle.swap_in(j, in_tab[j])
            while True:                            # the scheduler has nothing else to do: poll (step 1)
                for q in resumed:
                    waiting.discard(q)
                    h.pool.kv_host_release(q)
                    h.oracle.host_release(q)
                    h.pool.free_block_group(10**6 + q, in_tab[q])
                    checker.on_free(10**6 + q, in_tab.pop(q))
                if j < 0 or j not in waiting:
                    break
                resumed, _ = m.kv_manager_iterate()
        m.kv_manager_drain()
        assert not waiting and m.kv_manager_failures() == []
        h.pool.kv_wait_all()
        h.assert_pool_equal()
        st = h.pool.kv_stats()
        assert st["bytes_out"] == h.oracle.bytes_out and st["bytes_in"] == h.oracle.bytes_in
        free, largest = h.pool.kv_free_blocks()
        assert free == shape.n_blocks == largest and checker.n_used() == 0
    finally:
        m.kv_manager_destroy()


def test_concurrent_host_threads(harness):
    """The pool may be driven from several host threads: four threads swap disjoint requests
    out and back in at the same time."""
    import threading
    shape = synth.KVShape("s", 4, 8, 128, 16, 2, 256, "bf16")
    h = harness(shape, cfg=17, host_bytes=1024 * MiB)
    rng = synth.rng_for(17)
    tables = synth.deal_tables(rng, 256, [24] * 8)
    tables2 = synth.deal_tables(synth.rng_for(17, stream=1), 256, [24] * 8)
    # resume tables overlap other requests' current tables: keep each thread's pair disjoint
    # from the others by resuming into a permutation of its own blocks
    errors = []

    def worker(k):
        try:
            for rep in range(5):
                for r in (2 * k, 2 * k + 1):
                    h.pool.swap_out(r, tables[r])
                for r in (2 * k, 2 * k + 1):
                    h.pool.kv_wait(r)
                    h.pool.swap_in(r, tables[r][::-1].copy() if rep % 2 == 0 else tables[r])
                for r in (2 * k, 2 * k + 1):
                    h.pool.kv_wait(r)
        except Exception as e:  # pragma: no cover
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors
    for r in range(8):
        for rep in range(5):
            h.oracle.swap_out(r, tables[r])
            h.oracle.swap_in(r, tables[r][::-1].copy() if rep % 2 == 0 else tables[r])
    del tables2
    h.pool.kv_wait_all()
    for r in range(8):
        h.assert_image_equal(r)
    h.assert_pool_equal()


@pytest.mark.parametrize("L,H,D,B,e,N", [
    (2, 4, 64, 16, 2, 256),    # tiny config: C = 8 KiB (bounds-checked 32 KiB tiles)
    (4, 8, 128, 16, 2, 96),    # C = 32 KiB: exactly one tile per chunk
    (2, 40, 128, 16, 2, 24),   # C = 160 KiB: 5 tiles per chunk
    (3, 3, 40, 16, 2, 96),     # C = 3840: ragged
    (1, 1, 32, 16, 2, 2048),   # many small blocks: more than 440 per swap-in -> several launches
])
@pytest.mark.parametrize("out_too", [0, 64], ids=["in", "in_and_out"])
def test_mapped_swaps_touch_the_host_image_directly(harness, L, H, D, B, e, N, out_too):
    """KV_FLAG_MAPPED_SWAP_IN (and KV_FLAG_MAPPED_SWAP_OUT): swaps by kernels that read / write
    pinned host memory; same bytes as the staged path, for full, partial, delta and
    multi-extent images."""
    shape = synth.KVShape("s", L, H, D, B, e, N, "fp16")
    h = harness(shape, cfg=18, fill="random", flags=16 | out_too, host_slack_blocks=2)
    rng = synth.rng_for(18, stream=N)
    n = min(N // 3, 700)
    t = rng.permutation(N)[:n].astype(np.int32)
    u = rng.permutation(N)[:5].astype(np.int32)
    n0 = n - 9 if n > 18 else n // 2     # first image; it later grows by more than its slack
    h.pool.swap_out(0, t[:n0])
    h.oracle.swap_out(0, t[:n0])
    h.pool.swap_out(1, u)                     # takes the arena space right behind request 0
    h.oracle.swap_out(1, u)
    dirty = np.zeros(n, np.uint8)
    h.pool.swap_out_delta(0, t, dirty)        # grows past its slack: the image gets a second extent
    h.oracle.swap_out_delta(0, t, dirty)
    assert h.pool.kv_host_len(0) == (n, 2)
    h.assert_image_equal(0)
    t2 = rng.permutation(N)[:n].astype(np.int32)
    res = synth.random_mask(rng, n, 0.3)
    assert h.pool.swap_in_delta(0, t2, res) == len(h.oracle.swap_in(0, t2, resident=res))
    h.pool.kv_wait(0)
    h.assert_pool_equal()
    t3 = rng.permutation(N)[:n].astype(np.int32)
    h.pool.swap_in(0, t3)
    h.oracle.swap_in(0, t3)
    h.pool.swap_out(0, t3)                    # and straight out again: gather after mapped scatter
    h.oracle.swap_out(0, t3)
    h.assert_image_equal(0)
    h.assert_pool_equal()
    st = h.pool.kv_stats()
    assert st["h2d_copies"] == 0 and st["bytes_in"] == h.oracle.bytes_in
    assert (st["d2h_copies"] == 0) == bool(out_too) and st["bytes_out"] == h.oracle.bytes_out


@pytest.mark.parametrize("mapped", [0, 16], ids=["copy_engine", "mapped_reads"])
def test_layerwise_swap_in_lands_layer_by_layer(harness, mapped):
    """Layer-wise swap-in (the alternative of Section 2.2, Challenge #2): same bytes as swap_in,
    and a stream that waits for layer l sees that layer's K and V complete."""
    import torch
    shape = synth.KVShape("lw", 6, 4, 64, 16, 2, 160, "bf16")  # C = 8 KiB, R = 96 KiB
    stream = torch.cuda.Stream()
    h = harness(shape, cfg=31, host_bytes=64 * MiB, fill="random", host_slack_blocks=2,
                staging_in_bytes=1 * MiB, copy_chunk_bytes=256 * 1024,
                flags=4 | mapped, compute_stream=stream.cuda_stream)  # KV_FLAG_ORDER_COMPUTE [| MAPPED_SWAP_IN]
    rng = synth.rng_for(31)
    view = h.gpu.view(shape.P, shape.n_blocks, shape.C)
    n = 37
    perm = rng.permutation(shape.n_blocks).astype(np.int32)
    t = perm[:n].copy()
    # an image in two extents: 30 blocks, a neighbour behind its slack, then 7 more
    h.pool.swap_out(0, t[:30])
    h.oracle.swap_out(0, t[:30])
    h.pool.swap_out(1, perm[100:105].copy())
    h.oracle.swap_out(1, perm[100:105].copy())
    dirty = np.zeros(n, np.uint8)
    assert h.pool.swap_out_delta(0, t, dirty) == 7
    h.oracle.swap_out_delta(0, t, dirty)
    assert h.pool.kv_host_len(0) == (n, 2)
    h.assert_image_equal(0)
    cursor = 37
    for step, partial in ((1, False), (2, False), (4, False), (6, False), (3, True)):
        t2 = perm[cursor:cursor + n].copy()
        cursor = 37 + (cursor - 37 + n) % 60
        idx = torch.from_numpy(t2.astype(np.int64)).to(h.dev)
        with torch.cuda.stream(stream):
            view[:, idx, :] = 0xEE  # stale bytes, written on the compute stream just before
        h.oracle.G[:, t2.astype(np.int64), :] = 0xEE
        res = synth.random_mask(rng, n, 0.4) if partial else None
        moved = h.pool.swap_in_layerwise(0, t2, step, res)
        assert moved == len(h.oracle.swap_in(0, t2, resident=res))
        seen = []
        for layer in range(shape.n_layers):
            h.pool.kv_stream_wait_layer(0, layer, stream.cuda_stream)
            with torch.cuda.stream(stream):
                seen.append(view[2 * layer:2 * layer + 2, idx, :].clone())
        h.pool.kv_wait_layer(0, 0)
        stream.synchronize()
        for layer, got in enumerate(seen):
            want = h.oracle.G[2 * layer:2 * layer + 2, t2.astype(np.int64), :]
            assert np.array_equal(got.cpu().numpy(), want), (step, layer)
        h.pool.kv_wait(0)
        h.assert_pool_equal()
    st = h.pool.kv_stats()
    assert st["bytes_in"] == h.oracle.bytes_in


def test_growing_requests_through_block_groups(harness):
    """Requests grow through the block-group manager, are preempted (swap-out, groups closed
    while the gather may still be reading them) and resumed into whatever groups are free."""
    shape = synth.KVShape("s", 2, 4, 64, 16, 2, 160, "fp16")
    h = harness(shape, cfg=19, host_bytes=256 * MiB)
    h.pool.kv_bg_configure(16, 3)
    rng = synth.rng_for(19)
    chk = AllocChecker(shape.n_blocks)
    n_of = {}
    for r in range(6):
        ids = h.pool.kv_bg_append(r, int(rng.integers(4, 20)), 4)
        chk.on_alloc(r, ids)
        h.overwrite_blocks(ids, synth.fresh_tokens(rng, shape, len(ids)))
        n_of[r] = len(ids)
    for rnd in range(4):
        for r in range(6):                     # everybody decodes: one more block each
            ids = h.pool.kv_bg_append(r, 1)
            chk.on_alloc(r, ids)
            h.overwrite_blocks(ids, synth.fresh_tokens(rng, shape, 1))
            n_of[r] += 1
        victims = [int(v) for v in rng.permutation(6)[:3]]
        for v in victims:                      # preempt three of them
            t = h.pool.kv_bg_table(v)
            assert len(t) == n_of[v]
            h.pool.swap_out(v, t)
            h.oracle.swap_out(v, t)
            h.pool.kv_bg_close(v)
            chk.on_free(v, t)
        for v in victims:                      # ... and resume them right away
            ids = h.pool.kv_bg_append(v, n_of[v], 2)
            chk.on_alloc(v, ids)
            h.pool.swap_in(v, ids)
            h.oracle.swap_in(v, ids)
        h.pool.kv_wait_all()
        for v in victims:
            h.assert_image_equal(v)
        h.assert_pool_equal()
    st = h.pool.kv_bg_stats()
    assert st["used_blocks"] == chk.n_used() == sum(n_of.values())


def test_host_arena_eviction_keeps_data_exact(harness):
    """A small host arena with KV_FLAG_HOST_EVICT: which blocks get reclaimed is the policy's
    choice (any lower-priority, idle victim is valid), so the oracle is told which bits the
    library cleared; every byte that remains valid, and every later re-send, must be exact."""
    shape = synth.KVShape("s", 2, 4, 64, 16, 2, 200, "fp16")
    h = harness(shape, cfg=20, host_bytes=60 * synth.KVShape("s", 2, 4, 64, 16, 2, 200, "fp16").R,
                flags=32, host_slack_blocks=2)
    rng = synth.rng_for(20)
    sizes, tables = {}, {}
    prio = {r: int(rng.integers(0, 4)) for r in range(8)}
    for r in range(8):
        h.pool.kv_host_set_priority(r, prio[r])

    def sync_evictions():
        for r in sizes:
            lib_valid = h.pool.kv_host_valid(r, sizes[r]).astype(bool)
            ora = h.oracle.host[r].host_valid
            assert not (lib_valid & ~ora).any()           # the library never validates on its own
            gone = ora & ~lib_valid
            if gone.any():
                assert all(prio[r] <= prio[o] for o in [last_caller])  # only lower or equal priority
                h.oracle.host_invalidate(r, gone.astype(np.uint8))

    evicted_total = 0
    for step in range(60):
        r = int(rng.integers(0, 8))
        last_caller = r
        n = sizes.get(r, 0) + int(rng.integers(1, 10))
        n = min(n, 24)
        t = rng.permutation(200)[:n].astype(np.int32)
        payload = synth.fresh_tokens(rng, shape, n)
        h.overwrite_blocks(t, payload)
        dirty = synth.random_mask(rng, n, 0.3)
        try:
            if r in sizes:
                moved = h.pool.swap_out_delta(r, t, dirty)
            else:
                h.pool.swap_out(r, t)
                moved = n
        except h.kv.KVError as e:
            assert e.status == h.kv.KV_ENOMEM_HOST
            sync_evictions()                               # a failed call must have evicted nothing
            continue
        if r in sizes:
            want = h.oracle.swap_out_delta(r, t, dirty)
            # blocks evicted from r itself earlier are already invalid in the oracle
            assert moved == len(want)
        else:
            h.oracle.swap_out(r, t)
        sizes[r], tables[r] = n, t
        h.pool.kv_wait(r)
        sync_evictions()
        for q in sizes:
            h.assert_image_equal(q)
        evicted_total = h.pool.kv_stats()["host_evicted_blocks"]
    assert evicted_total > 0
    # everything still valid can be swapped back in exactly
    for r in sizes:
        valid = h.pool.kv_host_valid(r, sizes[r])
        t2 = rng.permutation(200)[:sizes[r]].astype(np.int32)
        h.pool.swap_in_delta(r, t2, 1 - valid)
        h.oracle.swap_in(r, t2, resident=1 - valid)
        h.pool.kv_wait(r)
        h.assert_pool_equal()
