"""GPU parity on long seeded random operation streams: a small serving loop (requests grow,
get preempted, resume into whatever the allocator returns, lose parts of their host copy,
finish) drives the library with no host synchronisation between calls, and the CPU oracle
replays the same calls in program order.  Pool and host images must agree byte for byte at
every checkpoint (Sections 3.2 and 3.3: asynchronous swapping, conflict handling, reuse)."""

import numpy as np
import pytest

from oracle.kv_oracle import AllocChecker
from paper_2411_18424_amd import synth

pytestmark = pytest.mark.gpu

KiB, MiB = 1 << 10, 1 << 20
SHAPE = synth.KVShape("stream", 2, 2, 64, 16, 2, 512, "fp16")  # C = 4 KiB, R = 16 KiB, 8 MiB pool

ORDER_COMPUTE, FOUR_STREAMS, MAPPED_SWAP_IN, MAPPED_SWAP_OUT = 4, 8, 16, 64


class Loop:
    """The serving loop's own state: which requests run (and where), which are swapped out."""

    def __init__(self, h, stream, rng, n_req):
        self.h, self.stream, self.rng = h, stream, rng
        self.chk = AllocChecker(SHAPE.n_blocks)
        self.view = h.gpu.view(SHAPE.P, SHAPE.n_blocks, SHAPE.C)
        self.table = {}      # running request -> physical table
        self.tokens = {}     # every live request -> tokens so far
        self.dirty = {}      # running request -> blocks written since its last swap-out
        self.swapped = set()
        self.has_image = set()
        self.free_ids = list(range(n_req))
        self.next_id = n_req
        self.tight = False   # host arena smaller than the swapped set can get
        self.refused = 0

    # -- both sides get the same bytes; the GPU write goes on the compute stream, unsynchronised
    def write(self, blocks, payload):
        torch = self.h.torch
        blocks = np.asarray(blocks, dtype=np.int64)
        if blocks.size == 0:
            return
        planes = np.ascontiguousarray(payload.transpose(1, 0, 2))
        self.h.oracle.G[:, blocks, :] = planes
        with torch.cuda.stream(self.stream):
            idx = torch.from_numpy(blocks).to(self.h.dev, non_blocking=False)
            self.view[:, idx, :] = torch.from_numpy(planes).to(self.h.dev)

    def alloc(self, req, n):
        free, _ = self.h.pool.kv_free_blocks()
        if n > free:
            return None
        ids, runs = self.h.pool.alloc_block_group(req, n, 4)
        assert runs == len(self.chk.on_alloc(req, ids))
        return ids

    def free(self, req, ids):
        self.h.pool.free_block_group(req, ids)
        self.chk.on_free(req, ids)

    # -- operations
    def start(self):
        if not self.free_ids:
            return
        n = int(self.rng.integers(1, 41))
        req = self.free_ids[-1]
        ids = self.alloc(req, n)
        if ids is None:
            return
        self.free_ids.pop()
        self.table[req] = ids
        self.tokens[req] = n * SHAPE.block_size - int(self.rng.integers(0, SHAPE.block_size))
        self.dirty[req] = np.ones(n, np.uint8)
        self.write(ids, synth.fresh_tokens(self.rng, SHAPE, n))

    def grow(self, req):
        B = SHAPE.block_size
        new_tokens = int(self.rng.integers(1, 6 * B))
        n_old = len(self.table[req])
        mask = synth.turn_dirty_mask(n_old, self.tokens[req], new_tokens, B)
        extra = len(mask) - n_old
        ids = self.alloc(req, extra) if extra else np.zeros(0, np.int32)
        if ids is None:
            return
        # the request's blocks may still be receiving its swap-in: order the write after it
        if req in self.has_image:
            self.h.pool.kv_stream_wait(req, self.stream.cuda_stream)
        table = np.concatenate([self.table[req], ids]).astype(np.int32)
        touched = np.flatnonzero(mask)
        self.write(table[touched], synth.fresh_tokens(self.rng, SHAPE, len(touched)))
        self.table[req] = table
        self.tokens[req] += new_tokens
        self.dirty[req] = np.concatenate([self.dirty[req], np.zeros(extra, np.uint8)]) | mask

    def preempt(self, req):
        table, dirty = self.table[req], self.dirty[req]
        delta = req in self.has_image and self.rng.random() < 0.8
        try:
            if delta:
                moved = self.h.pool.swap_out_delta(req, table, dirty)
            else:
                self.h.pool.swap_out(req, table)
        except self.h.kv.KVError as err:
            # a full host arena refuses the call; a refused call has no effect (checked by the
            # next checkpoint), so the request just keeps running
            assert self.tight and err.status == self.h.kv.KV_ENOMEM_HOST, err
            self.refused += 1
            return
        if delta:
            assert moved == len(self.h.oracle.swap_out_delta(req, table, dirty))
        else:
            self.h.oracle.swap_out(req, table)
        del self.table[req], self.dirty[req]
        self.has_image.add(req)
        self.swapped.add(req)
        self.free(req, table)  # right away: the allocator holds them back until the gather is done

    def resume(self, req):
        n, _ = self.h.pool.kv_host_len(req)
        ids = self.alloc(req, n)
        if ids is None:
            return
        self.h.pool.swap_in(req, ids)
        self.h.oracle.swap_in(req, ids)
        self.swapped.discard(req)
        self.table[req] = ids
        self.dirty[req] = np.zeros(n, np.uint8)

    def contaminate(self, req):
        n, _ = self.h.pool.kv_host_len(req)
        mask = synth.random_mask(self.rng, n, 0.3)
        self.h.pool.kv_host_invalidate(req, mask)
        self.h.oracle.host_invalidate(req, mask)

    def finish(self, req):
        """A request ends: its blocks and its host copy go back."""
        if req in self.table:
            if req in self.has_image:
                self.h.pool.kv_stream_wait(req, self.stream.cuda_stream)
            self.free(req, self.table.pop(req))
            self.dirty.pop(req)
        if req in self.has_image:
            self.h.pool.kv_host_release(req)
            self.h.oracle.host_release(req)
            self.has_image.discard(req)
        self.swapped.discard(req)
        del self.tokens[req]
        self.free_ids.append(self.next_id)  # a fresh id: nothing of the old request may linger
        self.next_id += 1

    def drop_host_copy(self, req):
        """A running request loses its whole host copy (memory pressure): next swap-out is full."""
        self.h.pool.kv_host_release(req)
        self.h.oracle.host_release(req)
        self.has_image.discard(req)
        self.dirty[req][:] = 1

    def step(self):
        r = self.rng.random()
        running = sorted(self.table)
        swapped = sorted(self.swapped)
        pick = lambda xs: xs[int(self.rng.integers(0, len(xs)))]
        if r < 0.15 or not self.tokens:
            self.start()
        elif r < 0.35 and running:
            self.grow(pick(running))
        elif r < 0.60 and running:
            self.preempt(pick(running))
        elif r < 0.85 and swapped:
            self.resume(pick(swapped))
        elif r < 0.93 and running:
            # only a request that is back on the GPU can lose host blocks (Section 3.3): part of
            # the copy (contamination) or all of it
            with_copy = [q for q in running if q in self.has_image]
            if with_copy and r < 0.90:
                self.contaminate(pick(with_copy))
            elif with_copy:
                self.drop_host_copy(pick(with_copy))
        elif r < 0.97 and self.tokens:
            self.finish(pick(sorted(self.tokens)))
        else:
            self.start()

    def checkpoint(self):
        self.h.pool.kv_wait_all()
        self.stream.synchronize()
        self.h.assert_pool_equal()
        for req in sorted(self.has_image):
            self.h.assert_image_equal(req)
        st = self.h.pool.kv_stats()
        assert st["bytes_out"] == self.h.oracle.bytes_out
        assert st["bytes_in"] == self.h.oracle.bytes_in
        free, _ = self.h.pool.kv_free_blocks()
        assert free + self.chk.n_used() == SHAPE.n_blocks


CASES = {
    # name: (seed, flags, pool keywords)
    "two_streams_small_rings": (101, ORDER_COMPUTE, dict(staging_out_bytes=1 * MiB, staging_in_bytes=512 * KiB,
                                                         max_piece_bytes=128 * KiB, host_slack_blocks=4)),
    "four_streams_default_rings": (102, ORDER_COMPUTE | FOUR_STREAMS, dict(host_slack_blocks=0)),
    "persistent_pack_kernel": (103, ORDER_COMPUTE, dict(pack_variant=1, staging_out_bytes=2 * MiB,
                                                        staging_in_bytes=2 * MiB, copy_chunk_bytes=64 * KiB)),
    "mapped_swap_in": (104, ORDER_COMPUTE | MAPPED_SWAP_IN, dict(host_slack_blocks=8)),
    # small swap-outs store to the host from a kernel, larger ones go through staging and copies
    "mapped_small_swap_outs": (106, ORDER_COMPUTE | MAPPED_SWAP_OUT, dict(mapped_out_max_blocks=12,
                                                                           host_slack_blocks=4)),
    "tight_host_arena": (105, ORDER_COMPUTE, dict(host_slack_blocks=2)),
}


@pytest.mark.parametrize("case", sorted(CASES))
def test_random_serving_loop_matches_oracle(case):
    import torch
    from gpu_util import Harness
    seed, flags, kw = CASES[case]
    host_bytes = 2 * MiB if case == "tight_host_arena" else 64 * MiB
    stream = torch.cuda.Stream()
    h = Harness(SHAPE, seed, host_bytes, fill="random", flags=flags,
                compute_stream=stream.cuda_stream, **kw)
    try:
        rng = synth.rng_for(seed)
        loop = Loop(h, stream, rng, n_req=14)
        loop.tight = case == "tight_host_arena"
        for i in range(1500):
            loop.step()
            if i % 150 == 149:
                loop.checkpoint()
        loop.checkpoint()
        assert h.oracle.bytes_out > 50 * SHAPE.R and h.oracle.bytes_in > 50 * SHAPE.R
        assert (loop.refused > 0) == loop.tight
    finally:
        h.close()
