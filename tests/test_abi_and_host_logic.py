"""CPU-only tests of the boundary and the host logic.

The library is loaded (no GPU needed for that), every function the header declares
must be exported, and pools created with KV_FLAG_PLAN_ONLY exercise validation, the
block-group allocator, the host arena and the reuse map without a single HIP call.
Plan-only pools move no bytes, so nothing here is a parity claim about data."""

import os
import re

import numpy as np
import pytest

from oracle.kv_oracle import AllocChecker, KVOracle
from paper_2411_18424_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def kv():
    from paper_2411_18424_amd import kvswap
    return kvswap


def plan_pool(kv, shape, host_blocks=64, flags_extra=0, **kw):
    return kv.KVPool(n_layers=shape.n_layers, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                     block_size=shape.block_size, elt_bytes=shape.elt_bytes,
                     n_gpu_blocks=shape.n_blocks, host_bytes=host_blocks * shape.R,
                     flags=kv.KV_FLAG_PLAN_ONLY | flags_extra, **kw)


def test_header_symbols_are_exported(kv):
    text = open(os.path.join(ROOT, "include", "kvswap.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:int32_t|char\s*\*|void)\s+\**\s*(\w+)\s*\(", text, flags=re.M)
    assert {"kv_pool_create", "alloc_block_group", "swap_out", "swap_in", "swap_out_delta"} <= set(names)
    assert len(names) >= 25
    for n in names:
        assert hasattr(kv.lib, n), "library does not export %s" % n
    assert set(names) == set(kv.lib._signatures), "binding and header disagree"


def test_create_rejects_bad_configs(kv):
    s = synth.TINY
    with pytest.raises(kv.KVError) as ei:
        kv.KVPool(n_layers=0, n_kv_heads=1, head_dim=8, block_size=16, elt_bytes=2, n_gpu_blocks=4,
                  flags=kv.KV_FLAG_PLAN_ONLY)
    assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError):  # chunk of 6 bytes is not a multiple of 16
        kv.KVPool(n_layers=1, n_kv_heads=1, head_dim=3, block_size=1, elt_bytes=2, n_gpu_blocks=4,
                  flags=kv.KV_FLAG_PLAN_ONLY)
    with pytest.raises(kv.KVError):  # a device pool needs a device pointer
        kv.KVPool(n_layers=s.n_layers, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim,
                  block_size=s.block_size, elt_bytes=s.elt_bytes, n_gpu_blocks=s.n_blocks)
    with pytest.raises(kv.KVError):  # a ring slot must hold one block record
        plan_pool(kv, s, staging_out_bytes=1024)


def test_validation_errors_and_no_effect(kv):
    p = plan_pool(kv, synth.TINY, host_blocks=20, host_slack_blocks=0)
    p.swap_out(0, np.arange(10, dtype=np.int32))
    st0 = p.kv_stats()
    for bad, code in (([3, 3], kv.KV_EINVAL), ([256], kv.KV_EINVAL), ([-2], kv.KV_EINVAL)):
        with pytest.raises(kv.KVError) as ei:
            p.swap_out(1, np.array(bad, np.int32))
        assert ei.value.status == code
    with pytest.raises(kv.KVError) as ei:
        p.swap_in(9, np.arange(3, dtype=np.int32))
    assert ei.value.status == kv.KV_ENOENT
    with pytest.raises(kv.KVError) as ei:
        p.swap_in(0, np.arange(3, dtype=np.int32))
    assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError) as ei:
        p.swap_out_delta(0, np.arange(4, dtype=np.int32), np.ones(4, np.uint8))  # shorter than image
    assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError) as ei:
        p.swap_out(2, np.arange(11, dtype=np.int32))
    assert ei.value.status == kv.KV_ENOMEM_HOST
    with pytest.raises(kv.KVError) as ei:
        p.swap_out_batch([4, 4], [[1], [2]])
    assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError) as ei:
        p.swap_out_batch([4, 5], [[1, 2], [2, 3]])  # a block in two tables
    assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError) as ei:
        p.kv_host_view(0)
    assert ei.value.status == kv.KV_ENODEV
    with pytest.raises(kv.KVError) as ei:
        p.kv_host_read(0)
    assert ei.value.status == kv.KV_ENODEV
    with pytest.raises(kv.KVError) as ei:
        p.kv_host_read(0, 8, 3)  # past the end of the 10-block image
    assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError):
        p.kv_wait(12345)
    assert p.kv_stats() == st0
    assert p.kv_host_valid(0, 10).all()


def test_moved_sets_follow_the_reuse_map(kv):
    """Bookkeeping only: the number of blocks each call moves equals the oracle's moved set
    over a random multi-turn history with contamination and partial swap-in."""
    shape = synth.KVShape("s", 1, 1, 8, 1, 2, 512, "fp16")
    p = plan_pool(kv, shape, host_blocks=4096)
    o = KVOracle(1, 1, 8, 1, 2, 512)
    rng = synth.rng_for(21)
    sizes = {}
    for step in range(300):
        r = int(rng.integers(0, 8))
        n_old = sizes.get(r, 0)
        kind = rng.integers(0, 5)
        if n_old == 0 or kind == 0:
            n = int(rng.integers(1, 40))
            t = rng.permutation(512)[:n].astype(np.int32)
            p.swap_out(r, t)
            o.swap_out(r, t)
            sizes[r] = n
        elif kind in (1, 2):
            n = n_old + int(rng.integers(0, 12))
            t = rng.permutation(512)[:n].astype(np.int32)
            dirty = synth.random_mask(rng, n, 0.2)
            assert p.swap_out_delta(r, t, dirty) == len(o.swap_out_delta(r, t, dirty))
            sizes[r] = n
        elif kind == 3:
            m = synth.random_mask(rng, n_old, 0.25)
            p.kv_host_invalidate(r, m)
            o.host_invalidate(r, m)
        else:
            t = rng.permutation(512)[:n_old].astype(np.int32)
            res = 1 - o.host[r].host_valid.astype(np.uint8)  # invalid blocks must be resident
            res |= synth.random_mask(rng, n_old, 0.3)
            assert p.swap_in_delta(r, t, res) == len(o.swap_in(r, t, resident=res))
        assert np.array_equal(p.kv_host_valid(r, sizes[r]).astype(bool), o.host[r].host_valid)
    st = p.kv_stats()
    assert st["bytes_out"] == o.bytes_out and st["bytes_in"] == o.bytes_in
    assert st["host_new_extents"] > 0


def test_allocator_never_double_assigns(kv):
    shape = synth.KVShape("s", 1, 1, 8, 1, 2, 1000, "fp16")
    p = plan_pool(kv, shape)
    chk = AllocChecker(1000)
    rng = synth.rng_for(22)
    live = {}
    for step in range(2000):
        if live and (rng.random() < 0.45 or chk.n_used() > 900):
            r = list(live)[int(rng.integers(0, len(live)))]
            ids = live.pop(r)
            if rng.random() < 0.3 and len(ids) > 1:  # free in two parts, any order
                cut = int(rng.integers(1, len(ids)))
                sh = rng.permutation(len(ids))
                p.free_block_group(r, ids[sh[:cut]])
                p.free_block_group(r, ids[sh[cut:]])
            else:
                p.free_block_group(r, ids)
            chk.on_free(r, ids)
        else:
            n = int(rng.integers(1, 80))
            free, largest = p.kv_free_blocks()
            assert free == 1000 - chk.n_used()
            if n > free:
                with pytest.raises(kv.KVError) as ei:
                    p.alloc_block_group(step, n, 8)
                assert ei.value.status == kv.KV_ENOMEM_GPU
                continue
            ids, runs = p.alloc_block_group(step, n, 8)
            rl = chk.on_alloc(step, ids)
            assert runs == len(rl)
            if largest >= n:
                assert runs == 1, "a free run of %d could hold %d blocks" % (largest, n)
            live[step] = ids
    for r, ids in live.items():
        p.free_block_group(r, ids)
    assert p.kv_free_blocks() == (1000, 1000)  # everything merged back into one group


def test_allocator_rejects_bad_frees(kv):
    p = plan_pool(kv, synth.TINY)
    ids, _ = p.alloc_block_group(1, 8, 1)
    for bad in ([ids[0], ids[0]], [300], [200]):
        with pytest.raises(kv.KVError) as ei:
            p.free_block_group(1, np.array(bad, np.int32))
        assert ei.value.status == kv.KV_EINVAL
    assert p.kv_free_blocks()[0] == 256 - 8
    p.free_block_group(1, ids)
    with pytest.raises(kv.KVError):
        p.free_block_group(1, ids)  # double free


def test_fragmented_pool_yields_few_long_runs(kv):
    """Block groups (Section 3.1): when the pool is fragmented the allocator still returns
    the longest free runs first."""
    shape = synth.KVShape("s", 1, 1, 8, 1, 2, 256, "fp16")
    p = plan_pool(kv, shape)
    all_ids, _ = p.alloc_block_group(0, 256, 1)
    # free runs of length 16, 8, 4, 2 at known places
    for start, ln in ((0, 16), (32, 8), (64, 4), (96, 2)):
        p.free_block_group(0, np.arange(start, start + ln, dtype=np.int32))
    ids, runs = p.alloc_block_group(1, 26, 8)
    assert AllocChecker.run_lengths(ids) == [16, 8, 2]
    assert runs == 3
    ids2, runs2 = p.alloc_block_group(2, 3, 1)
    assert AllocChecker.run_lengths(ids2) == [3] and ids2[0] == 64


def test_min_run_keeps_short_fragments_out_of_a_split_request(kv):
    """alloc_block_group's min_run: when a request has to be split, its remainder is carved from
    a free run of at least min_run blocks while one exists; without the preference it takes the
    best fit, which is a short fragment here."""
    shape = synth.TINY
    for min_run, want_tail_start in ((8, 100), (1, 64), (0, 64)):
        p = plan_pool(kv, shape)
        p.alloc_block_group(0, 256, 1)
        for start, ln in ((0, 40), (64, 5), (100, 30), (200, 5)):
            p.free_block_group(0, np.arange(start, start + ln, dtype=np.int32))
        ids, runs = p.alloc_block_group(1, 45, min_run)
        assert AllocChecker.run_lengths(ids) == [40, 5] and runs == 2
        assert ids[0] == 0 and ids[40] == want_tail_start, (min_run, ids[40])
        # a request that fits one run takes the best fit whatever min_run says
        ids2, runs2 = p.alloc_block_group(2, 5, min_run)
        assert runs2 == 1 and ids2[0] == (64 if want_tail_start == 100 else 200)
        p.close()
    # every longer run used up: the short fragments are the fallback
    p = plan_pool(kv, shape)
    p.alloc_block_group(0, 256, 1)
    for start, ln in ((0, 40), (64, 5), (200, 5)):
        p.free_block_group(0, np.arange(start, start + ln, dtype=np.int32))
    ids, runs = p.alloc_block_group(1, 44, 8)
    assert AllocChecker.run_lengths(ids) == [40, 4] and ids[40] == 64
    with pytest.raises(kv.KVError) as ei:
        p.alloc_block_group(2, 1, -1)
    assert ei.value.status == kv.KV_EINVAL
    p.close()


def test_plan_counts_copies_and_launches(kv):
    """Host-side plan of one swap: launches per ring slot, one copy per run of adjacent host
    records, copies cut at copy_chunk_bytes."""
    shape = synth.TINY  # R = 32 KiB
    p = plan_pool(kv, shape, host_blocks=256, staging_out_bytes=8 * shape.R,
                  staging_in_bytes=8 * shape.R, copy_chunk_bytes=3 * shape.R)
    t = np.arange(10, dtype=np.int32)
    p.swap_out(0, t)
    st = p.kv_stats()
    assert st["gather_launches"] == 3          # pieces of 4 blocks (half the ring): 4 + 4 + 2
    assert st["d2h_copies"] == 2 + 2 + 1       # 4 records -> 3 + 1, 2 records -> 1
    dirty = np.array([1, 0, 1, 1, 0, 0, 0, 1, 1, 1], np.uint8)
    assert p.swap_out_delta(0, t, dirty) == 6
    st2 = p.kv_stats()
    # moved j = 0 | 2 3 | 7 8 9 -> piece A holds 0,2,3,7 (runs 0 | 2-3 | 7), piece B holds 8,9
    assert st2["gather_launches"] - st["gather_launches"] == 2
    assert st2["d2h_copies"] - st["d2h_copies"] == 3 + 1


def test_scattered_records_travel_as_rows_of_strided_copies(kv):
    """Equal runs of host records a constant stride apart become one 2-D copy: the dirty blocks
    {1, 5, 9, 13} (stride 4) and {20, 22} of a 40-block image cost two copies instead of six, a
    run of three next to them one more; the same for a partial swap-in."""
    shape = synth.TINY
    for flags, want_out, want_in in ((0, 3, 3), (kv.KV_FLAG_NO_STRIDED_COPIES, 7, 7)):
        p = plan_pool(kv, shape, host_blocks=128, flags_extra=flags)
        t = np.arange(40, dtype=np.int32)
        p.swap_out(0, t)
        base = p.kv_stats()
        dirty = np.zeros(40, np.uint8)
        dirty[[1, 5, 9, 13, 20, 22, 30, 31, 32]] = 1
        assert p.swap_out_delta(0, t, dirty) == 9
        st = p.kv_stats()
        assert st["d2h_copies"] - base["d2h_copies"] == want_out
        assert st["strided_copies"] == (2 if flags == 0 else 0)
        assert st["bytes_out"] - base["bytes_out"] == 9 * shape.R
        assert p.swap_in_delta(0, t, 1 - dirty) == 9
        st2 = p.kv_stats()
        assert st2["h2d_copies"] - st["h2d_copies"] == want_in
        p.close()
    # rows may not be cut: a chain is limited by copy_chunk_bytes
    p = plan_pool(kv, shape, host_blocks=128, copy_chunk_bytes=2 * shape.R)
    t = np.arange(40, dtype=np.int32)
    p.swap_out(0, t)
    base = p.kv_stats()
    dirty = np.zeros(40, np.uint8)
    dirty[[1, 5, 9, 13]] = 1
    p.swap_out_delta(0, t, dirty)
    assert p.kv_stats()["d2h_copies"] - base["d2h_copies"] == 2  # two copies of two rows
    p.close()


def test_layerwise_swap_in_plan(kv):
    """Layer-wise swap-in: per step of layers one 2-D copy per run of adjacent host records
    (rows cut at copy_chunk_bytes) and one scatter per ring piece; pieces hold more blocks
    because a step moves only a slice of each record."""
    shape = synth.TINY  # 2 layers, C = 8 KiB, R = 32 KiB
    p = plan_pool(kv, shape, host_blocks=256, staging_out_bytes=8 * shape.R,
                  staging_in_bytes=8 * shape.R, copy_chunk_bytes=3 * shape.R)
    t = np.arange(10, dtype=np.int32)
    p.swap_out(0, t)
    st0 = p.kv_stats()
    assert p.swap_in_layerwise(0, t[::-1].copy(), 1) == 10
    st1 = p.kv_stats()
    # slice = R/2: pieces of 8 blocks (8 + 2), copies of at most 6 rows -> (2 + 1) per step
    assert st1["h2d_copies"] - st0["h2d_copies"] == 2 * 3
    assert st1["scatter_launches"] - st0["scatter_launches"] == 2 * 2
    assert st1["bytes_in"] - st0["bytes_in"] == 10 * shape.R
    assert p.swap_in_layerwise(0, t, 2) == 10
    st2 = p.kv_stats()
    # one step of both layers = the whole record: pieces 4 + 4 + 2, copies of at most 3 rows
    assert st2["h2d_copies"] - st1["h2d_copies"] == 2 + 2 + 1
    assert st2["scatter_launches"] - st1["scatter_launches"] == 3
    res = np.array([1, 0, 0, 1, 1, 1, 0, 1, 1, 1], np.uint8)
    assert p.swap_in_layerwise(0, t, 1, res) == 3          # j = 1 2 | 6 -> two runs per step
    st3 = p.kv_stats()
    assert st3["h2d_copies"] - st2["h2d_copies"] == 2 * 2
    p.kv_wait_layer(0, 1)
    p.kv_stream_wait_layer(0, 0, 0)
    for bad in (0, 3, -1):
        with pytest.raises(kv.KVError) as ei:
            p.swap_in_layerwise(0, t, bad)
        assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError) as ei:
        p.kv_wait_layer(0, 2)
    assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError) as ei:
        p.kv_wait_layer(5, 0)
    assert ei.value.status == kv.KV_ENOENT
    assert p.kv_stats()["bytes_in"] == st3["bytes_in"]
    # reading the pinned image directly: a step is one kernel launch, there are no copies
    q = plan_pool(kv, shape, host_blocks=256, flags_extra=kv.KV_FLAG_MAPPED_SWAP_IN)
    q.swap_out(0, t)
    assert q.swap_in_layerwise(0, t, 1) == 10
    assert q.kv_stats()["scatter_launches"] == 2 and q.kv_stats()["h2d_copies"] == 0


def test_mapped_swap_out_takes_small_moved_sets_only(kv):
    shape = synth.TINY
    p = plan_pool(kv, shape, host_blocks=256, flags_extra=kv.KV_FLAG_MAPPED_SWAP_OUT, mapped_out_max_blocks=4)
    t = np.arange(10, dtype=np.int32)
    p.swap_out(0, t[:4])                     # 4 blocks: one kernel, no copy
    st = p.kv_stats()
    assert (st["gather_launches"], st["d2h_copies"], st["bytes_out"]) == (1, 0, 4 * shape.R)
    p.swap_out(1, t[:5])                     # 5 blocks: staged
    st = p.kv_stats()
    assert (st["gather_launches"], st["d2h_copies"]) == (2, 1)
    dirty = np.array([0, 0, 1, 0, 1], np.uint8)
    assert p.swap_out_delta(1, t[:5], dirty) == 2   # the moved set counts, not the request
    st = p.kv_stats()
    assert (st["gather_launches"], st["d2h_copies"]) == (3, 1)
    with pytest.raises(kv.KVError) as ei:
        plan_pool(kv, shape, mapped_out_max_blocks=-1)
    assert ei.value.status == kv.KV_EINVAL
    with pytest.raises(kv.KVError) as ei:
        plan_pool(kv, shape, defer_min_bytes=-1)
    assert ei.value.status == kv.KV_EINVAL


def test_copy_scheduling_options_do_not_change_what_moves(kv):
    """Holding copies back, never holding them back, the second copy lane: options of how copies
    are enqueued.  The plan (what moves, how many launches and copies, where the records land)
    is the same under each of them; a plan-only pool starts no thread."""
    shape = synth.TINY
    rng = synth.rng_for(77)
    t = rng.permutation(shape.n_blocks)[:40].astype(np.int32)
    dirty = synth.random_mask(rng, 40, 0.3)
    seen = []
    for flags, kw in ((0, {}), (kv.KV_FLAG_NO_DEFER_COPIES, {}), (kv.KV_FLAG_SECOND_LANE, dict(defer_min_bytes=1)),
                      (0, dict(defer_min_bytes=1))):
        p = plan_pool(kv, shape, host_blocks=256, flags_extra=flags, **kw)
        p.swap_out(3, t)
        assert p.kv_query(3)
        moved = p.swap_out_delta(3, t, dirty)
        p.swap_in(3, t[::-1].copy())
        p.kv_wait_all()
        st = p.kv_stats()
        rec = p.kv_host_blocks(3)[1]
        seen.append((moved, st["gather_launches"], st["d2h_copies"], st["h2d_copies"], st["strided_copies"],
                     st["second_lane_copies"], st["bytes_out"], st["bytes_in"], tuple(int(r) for r in rec)))
        p.kv_pool_destroy()
    assert all(s == seen[0] for s in seen), seen
    assert seen[0][0] == int(dirty.sum()) and seen[0][5] == 0


def test_host_images_grow_by_extents_and_give_everything_back(kv):
    """Section 3.3: room behind a new image is reserved for the next turn; when it is used up
    the image continues in a further extent (it is never moved)."""
    shape = synth.TINY
    p = plan_pool(kv, shape, host_blocks=64, host_slack_blocks=4)
    t = np.arange(100, dtype=np.int32)
    p.swap_out(0, t[:10])                       # [0,14): 10 used + 4 slack
    p.swap_out(1, t[10:20])                     # [14,28)
    assert p.kv_host_len(0) == (10, 1)
    assert p.swap_out_delta(0, t[:13], np.zeros(13, np.uint8)) == 3      # fits the slack
    assert p.kv_host_len(0) == (13, 1) and p.kv_stats()["host_new_extents"] == 0
    assert p.swap_out_delta(0, t[:20], np.zeros(20, np.uint8)) == 7      # neighbour is taken: new extent
    assert p.kv_host_len(0) == (20, 2) and p.kv_stats()["host_new_extents"] == 1
    # request 1 is the last image in the arena: it grows in place
    assert p.swap_out_delta(1, t[30:50], np.zeros(20, np.uint8)) == 10
    assert p.kv_host_len(1)[1] == 1
    used = p.kv_stats()["host_arena_used"]
    # a full swap-out that fits the room already held reuses it
    p.swap_out(0, t[:18])
    assert p.kv_host_len(0) == (18, 2) and p.kv_stats()["host_arena_used"] == used
    # exhausting the arena is an error without effect
    with pytest.raises(kv.KVError) as ei:
        p.swap_out(2, t[50:100])
    assert ei.value.status == kv.KV_ENOMEM_HOST
    assert p.kv_stats()["host_arena_used"] == used
    for r in (0, 1):
        p.kv_host_release(r)
    assert p.kv_stats()["host_arena_used"] == 0
    p.swap_out(3, t[:60])                       # the whole arena is one run again
    assert p.kv_host_len(3) == (60, 1)


def test_fragmented_arena_serves_an_image_in_several_extents(kv):
    shape = synth.TINY
    p = plan_pool(kv, shape, host_blocks=40, host_slack_blocks=0)
    t = np.arange(200, dtype=np.int32)
    for r in range(4):
        p.swap_out(r, t[10 * r:10 * r + 10])    # four images of 10 records fill the arena
    p.kv_host_release(0)
    p.kv_host_release(2)                        # two holes of 10
    p.swap_out(9, t[100:118])                   # 18 records: no single run holds them
    assert p.kv_host_len(9) == (18, 2)
    st = p.kv_stats()
    assert st["host_arena_used"] == 38 * shape.R
    assert st["d2h_copies"] == 4 + 2            # the split image is copied as two runs


def test_swap_manager_dispatches_in_order_and_reports_each_task_once(kv):
    """Algorithm 1 primitives on a plan-only pool: submit returns tickets, the dispatcher
    applies tasks in submission order, poll / wait report every task exactly once with the
    status the entry point returned."""
    shape = synth.KVShape("s", 1, 1, 8, 1, 2, 512, "fp16")
    p = plan_pool(kv, shape, host_blocks=2048)
    m = kv.KVManager(p)
    o = KVOracle(1, 1, 8, 1, 2, 512)
    rng = synth.rng_for(31)
    tickets, expect_fail = [], set()
    for r in range(20):
        t = rng.permutation(512)[:int(rng.integers(1, 30))].astype(np.int32)
        tickets.append(m.kv_manager_submit(kv.KV_TASK_SWAP_OUT, r, t))
        o.swap_out(r, t)
        t2 = rng.permutation(512)[:len(t)].astype(np.int32)
        tickets.append(m.kv_manager_submit(kv.KV_TASK_SWAP_IN, r, t2))   # must follow its swap-out
        o.swap_in(r, t2)
    bad = m.kv_manager_submit(kv.KV_TASK_SWAP_IN, 999, np.arange(3, dtype=np.int32))  # no host copy
    expect_fail.add(bad)
    tickets.append(bad)
    d = rng.permutation(512)[:25].astype(np.int32)
    tickets.append(m.kv_manager_submit(kv.KV_TASK_SWAP_OUT_DELTA, 0, np.concatenate([d]), np.ones(25, np.uint8)))
    first = tickets[0]
    assert m.kv_manager_wait(first) == kv.KV_OK
    m.kv_manager_drain()
    seen = {}
    while True:
        got = m.kv_manager_poll(7)
        if not got:
            break
        for tk, st in got:
            assert tk not in seen
            seen[tk] = st
    assert set(seen) == set(tickets) - {first}
    for tk, st in seen.items():
        if tk in expect_fail:
            assert st == kv.KV_ENOENT
        elif tk == tickets[-1]:
            assert st in (kv.KV_OK, kv.KV_EINVAL)  # request 0 had fewer or more than 25 blocks
        else:
            assert st == kv.KV_OK
    with pytest.raises(kv.KVError):
        m.kv_manager_wait(first)  # already reported
    st = p.kv_stats()
    ms = m.kv_manager_stats()
    assert ms["submitted"] == ms["dispatched"] == len(tickets) and ms["failed"] >= 1
    assert ms["queued"] == 0 and ms["in_flight"] == 0
    assert st["bytes_in"] == o.bytes_in  # every swap-in found its swap-out dispatched before it
    m.kv_manager_destroy()


def test_algorithm_1_iterations_move_requests_between_the_queues(kv):
    """kv_manager_iterate on a plan-only pool: running -> swapped by a swap-out, swapped ->
    ongoing_swap_in -> running by an asynchronous swap-in (reported by a later iteration's
    step 1), swapped -> running at once by a synchronous one; conflicts between the two sets of
    an iteration are counted and the conflicting swap-out is dispatched first (the moved bytes
    then equal the oracle's, which applies the swap-out first); illegal transitions are
    refused; a failed swap is booked by the next iteration."""
    shape = synth.KVShape("s", 1, 1, 8, 1, 2, 512, "fp16")
    p = plan_pool(kv, shape, host_blocks=600)
    m = kv.KVManager(p, sync_below_ms=1e-9)  # the strategy always answers asynchronous
    W = (kv.KV_WHERE_RUNNING, kv.KV_WHERE_SWAPPED, kv.KV_WHERE_ONGOING_SWAP_IN)
    ta, tb, tc = (np.arange(i * 40, i * 40 + 30, dtype=np.int32) for i in range(3))
    # iteration 1: A and B leave
    resumed, r = m.kv_manager_iterate(swap_out=[(1, ta), (2, tb)])
    assert resumed == [] and r["conflicts"] == 0 and r["ongoing_swap_ins"] == 0
    assert m.kv_manager_where(1) == W[1] and m.kv_manager_where(2) == W[1]
    with pytest.raises(kv.KVError) as ei:
        m.kv_manager_iterate(swap_out=[(1, ta)])          # not running
    assert ei.value.status == kv.KV_EBUSY
    with pytest.raises(kv.KVError) as ei:
        m.kv_manager_iterate(swap_in=[(3, tc)])           # never swapped out
    assert ei.value.status == kv.KV_ENOENT
    # iteration 2: A resumes asynchronously into the blocks C vacates in the same iteration
    resumed, r = m.kv_manager_iterate(swap_in=[(1, tc)], swap_out=[(3, tc)])
    assert r["async"] == 1 and r["conflicts"] == 1 and resumed == []
    assert m.kv_manager_where(1) == W[2] and m.kv_manager_where(3) == W[1]
    m.kv_manager_drain()
    assert p.kv_stats()["conflict_waits"] == 0  # plan-only: nothing is in flight, but the order held:
    assert p.kv_host_len(3)[0] == 30            # C's swap-out was accepted (its table was still C's)
    # iteration 3: step 1 finds A's swap-in complete; B resumes synchronously
    resumed, r = m.kv_manager_iterate(swap_in=[(2, ta)], force_mode=2)
    assert sorted(resumed) == [1, 2] and r["completed_swap_ins"] == 1 and r["waited_swap_ins"] == 1
    assert r["async"] == 0 and r["ongoing_swap_ins"] == 0
    assert m.kv_manager_where(1) == W[0] and m.kv_manager_where(2) == W[0]
    # a swap-out that fails when it is dispatched (arena full) returns the request to running
    big = np.arange(0, 500, dtype=np.int32)
    m.kv_manager_iterate(swap_out=[(7, big)])
    m.kv_manager_drain()
    resumed, r = m.kv_manager_iterate()
    assert r["failures"] == 1 and m.kv_manager_failures() == [(7, kv.KV_ENOMEM_HOST)]
    assert m.kv_manager_where(7) == W[0]
    # preemption that gives the victim's blocks up: the dispatcher frees them once the swap-out is enqueued
    ids, _ = p.alloc_block_group(50, 40, 8)
    assert p.kv_free_blocks()[0] == 512 - 40
    m.kv_manager_iterate(swap_out=[(50, ids)], free_out_blocks=True)
    m.kv_manager_drain()
    assert p.kv_free_blocks()[0] == 512 and p.kv_host_len(50)[0] == 40
    # delta swap-outs through the iteration
    resumed, r = m.kv_manager_iterate(swap_out=[(1, tc, np.ones(30, np.uint8))])
    m.kv_manager_drain()
    st = m.kv_manager_iteration_stats()
    assert st["iterations"] == 7 and st["swap_outs"] == 6 and st["swap_ins"] == 2 and st["conflicts"] == 1
    assert st["async_iterations"] == 1 and st["sync_iterations"] == 1 and st["resumed"] == 2
    assert p.kv_stats()["blocks_out"] == 30 * 4 + 40 and p.kv_stats()["blocks_in"] == 60
    m.kv_manager_destroy()


def test_swap_manager_strategy_follows_swap_in_size(kv):
    """Step 4: short swap-ins are waited for, long ones proceed asynchronously; the recent
    window damps single outliers."""
    shape = synth.LLAMA3_8B  # R = 2 MiB: 0.5 ms of link time at 55 GB/s is about 13 blocks
    p = plan_pool(kv, shape.with_blocks(4096), host_blocks=4096)
    m = kv.KVManager(p, link_gbps=55.0, sync_below_ms=0.5)
    assert m.kv_manager_strategy(0, 0) is False
    assert m.kv_manager_strategy(4, 4 * 2) is False        # four swap-ins of 2 blocks: 0.08 ms each
    assert m.kv_manager_strategy(4, 4 * 200) is True       # 7.6 ms each
    # a window full of long swap-ins keeps the mode asynchronous for one short request ...
    for r in range(8):
        m.kv_manager_submit(kv.KV_TASK_SWAP_OUT, r, np.arange(r * 300, r * 300 + 300, dtype=np.int32))
        m.kv_manager_submit(kv.KV_TASK_SWAP_IN, r, np.arange(r * 300, r * 300 + 300, dtype=np.int32))
    m.kv_manager_drain()
    assert m.kv_manager_strategy(1, 2) is True
    # ... and a window full of short ones makes it synchronous
    m2 = kv.KVManager(p, window=8, link_gbps=55.0, sync_below_ms=0.5)
    for r in range(100, 108):
        m2.kv_manager_submit(kv.KV_TASK_SWAP_OUT, r, np.arange(3500 + (r - 100) * 2, 3502 + (r - 100) * 2, dtype=np.int32))
        m2.kv_manager_submit(kv.KV_TASK_SWAP_IN, r, np.arange(3500 + (r - 100) * 2, 3502 + (r - 100) * 2, dtype=np.int32))
    m2.kv_manager_drain()
    assert m2.kv_manager_strategy(1, 20) is False  # (0.76 + 0.08) / 2 = 0.42 ms < 0.5 ms
    s = m.kv_manager_stats()
    assert s["strategy_calls"] == 4 and s["strategy_async"] == 2
    m.kv_manager_destroy()
    m2.kv_manager_destroy()


def test_block_groups_grow_steal_and_return(kv):
    """Section 3.1: a request grows inside its active group; when no free group is left the
    tail of another request's active group is split off; closing returns everything."""
    shape = synth.KVShape("s", 1, 1, 8, 1, 2, 96, "fp16")
    p = plan_pool(kv, shape)
    p.kv_bg_configure(32, 1)
    chk = AllocChecker(96)
    a = p.kv_bg_append(1, 5)                       # opens a group of 32, uses 5
    assert a.tolist() == [0, 1, 2, 3, 4]
    chk.on_alloc(1, a)
    b = p.kv_bg_append(2, 3)                       # second request: its own group of 32
    assert b.tolist() == [32, 33, 34]
    chk.on_alloc(2, b)
    for k in range(5, 32):                         # request 1 grows one block at a time, contiguously
        x = p.kv_bg_append(1, 1)
        assert x.tolist() == [k]
        chk.on_alloc(1, x)
    x = p.kv_bg_append(1, 1)                       # active group full and its neighbour taken: new group
    assert x.tolist() == [64]
    chk.on_alloc(1, x)
    st = p.kv_bg_stats()
    assert (st["n_requests"], st["used_blocks"], st["tail_blocks"], st["steals"]) == (2, 36, 60, 0)
    assert p.kv_free_blocks()[0] == 0              # every block is used or reserved as a tail
    c = p.kv_bg_append(3, 10)                      # no free group: steals from an active tail
    chk.on_alloc(3, c)
    assert AllocChecker.run_lengths(c) == [10]
    st = p.kv_bg_stats()
    assert st["steals"] == 1 and st["used_blocks"] == 46
    assert np.array_equal(p.kv_bg_table(1), np.concatenate([np.arange(32), [64]]))
    assert np.array_equal(p.kv_bg_table(3), c)
    with pytest.raises(kv.KVError) as ei:
        p.kv_bg_append(4, 60)                      # more than free blocks + other requests' tails
    assert ei.value.status == kv.KV_ENOMEM_GPU
    assert p.kv_bg_stats()["used_blocks"] == 46
    for r in (1, 2, 3):
        p.kv_bg_close(r)
    assert p.kv_free_blocks() == (96, 96)
    with pytest.raises(kv.KVError):
        p.kv_bg_close(1)


def test_block_groups_never_double_assign_under_churn(kv):
    shape = synth.KVShape("s", 1, 1, 8, 1, 2, 600, "fp16")
    p = plan_pool(kv, shape)
    p.kv_bg_configure(24, 5)
    chk = AllocChecker(600)
    rng = synth.rng_for(33)
    owned = {}
    for step in range(3000):
        r = int(rng.integers(0, 24))
        if r in owned and rng.random() < 0.08:
            assert np.array_equal(p.kv_bg_table(r), np.concatenate(owned[r]))
            p.kv_bg_close(r)
            chk.on_free(r, np.concatenate(owned.pop(r)))
            continue
        n = int(rng.integers(1, 4)) if r in owned else int(rng.integers(1, 60))
        try:
            ids = p.kv_bg_append(r, n, int(rng.integers(0, 8)))
        except kv.KVError as e:
            assert e.status == kv.KV_ENOMEM_GPU
            continue
        chk.on_alloc(r, ids)
        owned.setdefault(r, []).append(ids)
    st = p.kv_bg_stats()
    assert st["used_blocks"] == chk.n_used() and st["steals"] > 0
    assert st["used_blocks"] + st["tail_blocks"] + p.kv_free_blocks()[0] == 600
    for r in list(owned):
        p.kv_bg_close(r)
    assert p.kv_free_blocks() == (600, 600)


def test_granularity_grows_with_the_first_group_size():
    """The synthetic serving loop: larger first groups give fewer, longer groups per swap-out
    (Section 5.3.1 measures this on its traces; here only the direction is checked)."""
    from paper_2411_18424_amd import granularity
    small = granularity.simulate(first_group=1, pattern="markov", n_iters=1500)
    large = granularity.simulate(first_group=64, pattern="markov", n_iters=1500)
    assert small["swap_outs"] > 50 and large["swap_outs"] > 50
    assert large["avg_blocks_per_group"] > 1.5 * small["avg_blocks_per_group"]
    assert large["avg_groups_per_swap"] < small["avg_groups_per_swap"]
    assert granularity.run_lengths([3, 4, 5, 9, 10, 2]) == [3, 2, 1]


def test_host_eviction_by_priority_and_recency(kv):
    """KV_FLAG_HOST_EVICT (Section 3.3, contamination): a full arena reclaims the host copies of
    lower-priority requests - reserved room first, then their last logical blocks - never of
    higher-priority ones; all or nothing."""
    shape = synth.TINY
    p = plan_pool(kv, shape, host_blocks=40, host_slack_blocks=2, flags_extra=kv.KV_FLAG_HOST_EVICT)
    t = np.arange(200, dtype=np.int32)
    for r, prio in ((0, 5), (1, 1), (2, 1), (3, 9)):
        p.kv_host_set_priority(r, prio)
        p.swap_out(r, t[10 * r:10 * r + 8])          # 8 records + 2 of room each: arena full
    assert p.kv_stats()["host_arena_used"] == 40 * shape.R
    p.swap_in(2, t[100:108])                         # request 2 was used more recently than 1
    # request 0 (priority 5) needs 12 records more than it has room for
    moved = p.swap_out_delta(0, t[40:60], np.zeros(20, np.uint8))
    assert moved == 12
    st = p.kv_stats()
    # 10 + 2 slack wanted -> falls back to what can be had; victims: request 1 first (LRU), then 2
    v1, v2, v3 = p.kv_host_valid(1, 8), p.kv_host_valid(2, 8), p.kv_host_valid(3, 8)
    assert v3.all(), "a higher-priority request must never be evicted"
    lost1, lost2 = int(8 - v1.sum()), int(8 - v2.sum())
    assert lost1 > 0 and lost1 >= lost2
    assert st["host_evicted_blocks"] == lost1 + lost2
    assert (v1[:8 - lost1] == 1).all() and (v1[8 - lost1:] == 0).all()   # the tail goes first
    assert st["host_arena_used"] <= 40 * shape.R
    # the evicted request gets its blocks back on its next swap-out (it may evict in turn)
    p.kv_host_set_priority(1, 7)
    assert p.swap_out_delta(1, t[110:118], np.zeros(8, np.uint8)) == lost1
    assert p.kv_host_valid(1, 8).all()
    # a request that outranks nobody cannot evict: error without effect
    p.kv_host_set_priority(7, 0)
    before = (p.kv_stats(), p.kv_host_valid(0, 20).tolist(), p.kv_host_valid(2, 8).tolist())
    with pytest.raises(kv.KVError) as ei:
        p.swap_out(7, t[150:190])
    assert ei.value.status == kv.KV_ENOMEM_HOST
    assert (p.kv_stats(), p.kv_host_valid(0, 20).tolist(), p.kv_host_valid(2, 8).tolist()) == before
    # swap-in of a block that lost its copy is refused unless it is resident
    if lost2:
        with pytest.raises(kv.KVError) as ei:
            p.swap_in(2, t[120:128])
        assert ei.value.status == kv.KV_ENOENT
        res = 1 - p.kv_host_valid(2, 8)
        assert p.swap_in_delta(2, t[120:128], res) == 8 - lost2


def test_host_records_never_overlap_under_growth_and_eviction(kv):
    """Arena invariants over a random multi-request history with growth, release and eviction:
    every record belongs to at most one logical block of one image, lies inside the arena, and
    a block has a record exactly while it can be valid."""
    shape = synth.KVShape("s", 1, 1, 8, 1, 2, 4096, "fp16")
    arena = 600
    p = plan_pool(kv, shape, host_blocks=arena, flags_extra=kv.KV_FLAG_HOST_EVICT, host_slack_blocks=5)
    rng = synth.rng_for(41)
    live = {}
    for step in range(600):
        r = int(rng.integers(0, 12))
        kind = int(rng.integers(0, 6))
        try:
            if r not in live or kind == 0:
                n = int(rng.integers(1, 90))
                p.kv_host_set_priority(r, int(rng.integers(0, 3))) if r in live else None
                p.swap_out(r, rng.permutation(4096)[:n].astype(np.int32))
                live[r] = n
            elif kind in (1, 2, 3):
                n = live[r] + int(rng.integers(0, 25))
                p.swap_out_delta(r, rng.permutation(4096)[:n].astype(np.int32), synth.random_mask(rng, n, 0.2))
                live[r] = n
            elif kind == 4:
                p.kv_host_release(r)
                del live[r]
            else:
                p.kv_host_set_priority(r, int(rng.integers(0, 3)))
        except kv.KVError as err:
            assert err.status == kv.KV_ENOMEM_HOST, err      # refused calls change nothing
        seen = {}
        for q, n in live.items():
            base, rec = p.kv_host_blocks(q)
            assert base is None and rec.size == n == p.kv_host_len(q)[0]
            valid = p.kv_host_valid(q, n).astype(bool)
            assert not valid[rec < 0].any(), "a block without a record cannot be valid"
            for j in np.flatnonzero(rec >= 0):
                x = int(rec[j])
                assert 0 <= x < arena, x
                assert x not in seen, "record %d holds block %d of request %d and %s" % (x, j, q, seen[x])
                seen[x] = (q, int(j))
        st = p.kv_stats()
        assert len(seen) * shape.R <= st["host_arena_used"] <= arena * shape.R
    assert p.kv_stats()["host_evicted_blocks"] > 0
    for q in list(live):
        p.kv_host_release(q)
    assert p.kv_stats()["host_arena_used"] == 0


def test_reuse_cuts_swap_out_volume_and_small_host_memory_erodes_it():
    """Direction of the paper's microbenchmark (Section 5.3.3): with reuse far fewer blocks are
    swapped out than when the whole context leaves every time; a smaller host arena means more
    contaminated copies and more blocks sent again."""
    from paper_2411_18424_amd import reuse_sim
    base = reuse_sim.simulate(1 << 20, reuse=False, n_preempt=300)
    big = reuse_sim.simulate(1 << 20, reuse=True, n_preempt=300)
    small = reuse_sim.simulate(4000, reuse=True, n_preempt=300)
    assert big["blocks_out"] < 0.5 * base["blocks_out"]
    assert big["evicted_blocks"] == 0 and small["evicted_blocks"] > 0
    assert big["blocks_out"] < small["blocks_out"] < base["blocks_out"]


def test_device_pool_fails_loudly_without_a_gpu(kv):
    """No CPU fallback: without a device a real (non plan-only) pool cannot be created."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    s = synth.TINY
    with pytest.raises(kv.KVError) as ei:
        kv.KVPool(n_layers=s.n_layers, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim, block_size=s.block_size,
                  elt_bytes=s.elt_bytes, n_gpu_blocks=s.n_blocks, gpu_base=0x1000, host_bytes=1 << 20)
    assert ei.value.status in (kv.KV_EHIP, kv.KV_ENOMEM_HOST, kv.KV_ENOMEM_GPU)
    with pytest.raises(kv.KVError):
        kv.kv_link_probe(1 << 20, 0, 1)
