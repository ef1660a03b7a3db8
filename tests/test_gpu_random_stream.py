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
# transfers that take milliseconds, so calls really overlap: C = 32 KiB, R = 512 KiB, 2 GiB pool
BIG = synth.KVShape("stream_big", 8, 8, 128, 16, 2, 4096, "bf16")

ORDER_COMPUTE, FOUR_STREAMS, MAPPED_SWAP_IN, MAPPED_SWAP_OUT, SCATTER_STREAM = 4, 8, 16, 64, 128
NO_DEFER_COPIES = 512
SECOND_LANE = 1024


class Loop:
    """The serving loop's own state: which requests run (and where), which are swapped out."""

    def __init__(self, h, stream, rng, n_req, max_blocks=40):
        self.h, self.stream, self.rng = h, stream, rng
        self.shape = h.shape
        self.max_blocks = max_blocks
        self.chk = AllocChecker(self.shape.n_blocks)
        self.view = h.gpu.view(self.shape.P, self.shape.n_blocks, self.shape.C)
        self.table = {}      # running request -> physical table
        self.tokens = {}     # every live request -> tokens so far
        self.dirty = {}      # running request -> blocks written since its last swap-out
        self.swapped = set()
        self.kept = {}       # swapped-out request -> its blocks that stayed on the GPU
        self.has_image = set()
        self.free_ids = list(range(n_req))
        self.next_id = n_req
        self.tight = False   # host arena smaller than the swapped set can get
        self.refused = 0
        # The oracle replays the calls later, at the checkpoint: nothing slow may sit between
        # two library calls, or each would have finished before the next one is made.
        self.pending = []
        self.log = []        # (request, what) in program order, for failure reports
        # new KV comes from a resident base of 256 random blocks (same bytes on both sides)
        torch = h.torch
        self.base_host = rng.integers(0, 256, size=(self.shape.P, 256, self.shape.C), dtype=np.uint8)
        self.base_dev = torch.from_numpy(self.base_host).to(h.dev)
        torch.cuda.synchronize()

    def payload(self, n):
        """New KV of n blocks: which base blocks they copy."""
        return self.rng.integers(0, 256, size=n)

    # -- both sides get the same bytes; the GPU write goes on the compute stream, unsynchronised
    def write(self, blocks, sel):
        torch = self.h.torch
        blocks = np.asarray(blocks, dtype=np.int64)
        if blocks.size == 0:
            return
        sel = np.asarray(sel, dtype=np.int64)
        G, base = self.h.oracle.G, self.base_host

        def on_oracle():
            G[:, blocks, :] = base[:, sel, :]
        self.pending.append(on_oracle)
        with torch.cuda.stream(self.stream):
            idx = torch.from_numpy(blocks).to(self.h.dev)
            src = torch.from_numpy(sel).to(self.h.dev)
            self.view[:, idx, :] = self.base_dev[:, src, :]

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
        n = int(self.rng.integers(1, self.max_blocks + 1))
        req = self.free_ids[-1]
        ids = self.alloc(req, n)
        if ids is None:
            return
        self.free_ids.pop()
        self.table[req] = ids
        self.tokens[req] = n * self.shape.block_size - int(self.rng.integers(0, self.shape.block_size))
        self.dirty[req] = np.ones(n, np.uint8)
        self.write(ids, self.payload(n))
        self.note(req, "start %d blocks %s.." % (n, ids[:4].tolist()))

    def grow(self, req):
        B = self.shape.block_size
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
        self.write(table[touched], self.payload(len(touched)))
        self.table[req] = table
        self.tokens[req] += new_tokens
        self.dirty[req] = np.concatenate([self.dirty[req], np.zeros(extra, np.uint8)]) | mask
        self.note(req, "grow +%d blocks, touched %s" % (extra, table[touched].tolist()[:6]))

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
        oracle = self.h.oracle
        if delta:
            def on_oracle(moved=moved, table=table.copy(), dirty=dirty.copy()):
                assert moved == len(oracle.swap_out_delta(req, table, dirty))
        else:
            def on_oracle(table=table.copy()):
                oracle.swap_out(req, table)
        self.pending.append(on_oracle)
        self.note(req, "preempt %s n=%d" % ("delta" if delta else "full", len(table)))
        del self.table[req], self.dirty[req]
        self.has_image.add(req)
        self.swapped.add(req)
        # sometimes the first blocks stay on the GPU (a partly resident request); the rest is
        # freed right away: the allocator holds them back until the gather is done
        keep = int(self.rng.integers(0, len(table))) if self.rng.random() < 0.3 else 0
        self.kept[req] = table[:keep]
        self.free(req, table[keep:])

    def resume(self, req):
        n, _ = self.h.pool.kv_host_len(req)
        kept = self.kept[req]
        rest = self.alloc(req, n - len(kept)) if n > len(kept) else np.zeros(0, np.int32)
        if rest is None:
            return
        del self.kept[req]
        ids = np.concatenate([kept, rest]).astype(np.int32)
        resident = np.zeros(n, np.uint8)
        resident[:len(kept)] = 1
        how = int(self.rng.integers(0, 3))
        if len(kept):
            moved = self.h.pool.swap_in_delta(req, ids, resident)
        elif how == 0:
            moved = self.h.pool.swap_in_layerwise(req, ids, int(self.rng.integers(1, self.shape.n_layers + 1)))
        else:
            self.h.pool.swap_in(req, ids)
            moved = n
        oracle = self.h.oracle

        def on_oracle(ids=ids.copy(), moved=moved):
            assert moved == len(oracle.swap_in(req, ids, resident=resident))
        self.pending.append(on_oracle)
        self.note(req, "resume (%d kept) into %s.." % (len(kept), ids[:4].tolist()))
        self.swapped.discard(req)
        self.table[req] = ids
        self.dirty[req] = np.zeros(n, np.uint8)

    def preempt_batch(self, reqs):
        """Several victims leave in one call (full swap-outs; all or none on a full arena)."""
        tables = [self.table[q] for q in reqs]
        try:
            self.h.pool.swap_out_batch(reqs, tables)
        except self.h.kv.KVError as err:
            assert self.tight and err.status == self.h.kv.KV_ENOMEM_HOST, err
            self.refused += 1
            return
        oracle = self.h.oracle
        for q, t in zip(reqs, tables):
            self.pending.append(lambda q=q, t=t.copy(): oracle.swap_out(q, t))
            self.note(q, "preempt in a batch n=%d" % len(t))
            del self.table[q], self.dirty[q]
            self.has_image.add(q)
            self.swapped.add(q)
            self.kept[q] = t[:0]
            self.free(q, t)

    def resume_batch(self, reqs):
        tables = []
        for q in reqs:
            n, _ = self.h.pool.kv_host_len(q)
            ids = self.alloc(q, n)
            if ids is None:
                for q2, t2 in zip(reqs, tables):
                    self.free(q2, t2)
                return
            tables.append(ids)
        self.h.pool.swap_in_batch(reqs, tables)
        oracle = self.h.oracle
        for q, t in zip(reqs, tables):
            self.pending.append(lambda q=q, t=t.copy(): oracle.swap_in(q, t))
            self.note(q, "resume in a batch into %s.." % t[:4].tolist())
            del self.kept[q]
            self.swapped.discard(q)
            self.table[q] = t
            self.dirty[q] = np.zeros(len(t), np.uint8)

    def contaminate(self, req):
        n, _ = self.h.pool.kv_host_len(req)
        mask = synth.random_mask(self.rng, n, 0.3)
        self.h.pool.kv_host_invalidate(req, mask)
        self.pending.append(lambda: self.h.oracle.host_invalidate(req, mask))
        self.note(req, "contaminate %d" % int(mask.sum()))

    def finish(self, req):
        """A request ends: its blocks and its host copy go back."""
        if req in self.table:
            if req in self.has_image:
                self.h.pool.kv_stream_wait(req, self.stream.cuda_stream)
            self.free(req, self.table.pop(req))
            self.dirty.pop(req)
        if req in self.has_image:
            self.h.pool.kv_host_release(req)
            self.pending.append(lambda: self.h.oracle.host_release(req))
            self.has_image.discard(req)
        self.swapped.discard(req)
        if req in self.kept:
            self.free(req, self.kept.pop(req))
        del self.tokens[req]
        self.note(req, "finish")
        self.free_ids.append(self.next_id)  # a fresh id: nothing of the old request may linger
        self.next_id += 1

    def drop_host_copy(self, req):
        """A running request loses its whole host copy (memory pressure): next swap-out is full."""
        self.h.pool.kv_host_release(req)
        self.pending.append(lambda: self.h.oracle.host_release(req))
        self.has_image.discard(req)
        self.dirty[req][:] = 1
        self.note(req, "drop host copy")

    def note(self, req, what):
        self.log.append((req, what))

    def step(self):
        r = self.rng.random()
        running = sorted(self.table)
        swapped = sorted(self.swapped)
        pick = lambda xs: xs[int(self.rng.integers(0, len(xs)))]
        if r < 0.15 or not self.tokens:
            self.start()
        elif r < 0.35 and running:
            self.grow(pick(running))
        elif r < 0.55 and running:
            self.preempt(pick(running))
        elif r < 0.60 and len(running) >= 3:
            k = int(self.rng.integers(2, 4))
            self.preempt_batch([int(q) for q in self.rng.choice(running, size=k, replace=False)])
        elif r < 0.80 and swapped:
            self.resume(pick(swapped))
        elif r < 0.85 and swapped:
            whole = [q for q in swapped if len(self.kept[q]) == 0]   # nothing of them stayed on the GPU
            if len(whole) >= 2:
                self.resume_batch([int(q) for q in self.rng.choice(whole, size=2, replace=False)])
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

    def diagnose(self):
        """Who owns the blocks that differ, what was done to them, and what they hold instead."""
        got, want = self.h.gpu_pool(), self.h.oracle.G
        bad = np.flatnonzero((got != want).any(axis=(0, 2)))
        owner = {int(b): q for q, t in self.table.items() for b in t}
        lines = ["%d blocks differ: %s" % (bad.size, bad[:24].tolist())]
        owners = sorted({owner.get(int(b), -1) for b in bad})
        lines.append("owners (-1 = free): %s" % owners)
        for q in owners:
            if q >= 0:
                lines.append("request %d table %s" % (q, self.table[q].tolist()))
                lines.append("  history: " + "; ".join(w for r, w in self.log if r == q))
        b = int(bad[0])
        planes_bad = np.flatnonzero((got[:, b] != want[:, b]).any(axis=1))
        lines.append("block %d: planes that differ %s" % (b, planes_bad.tolist()[:16]))
        p0 = int(planes_bad[0])
        holds = [s for s in range(256) if np.array_equal(got[p0, b], self.base_host[p0, s])]
        lines.append("  GPU holds base block(s) %s of that plane" % holds)
        wants = [s for s in range(256) if np.array_equal(want[p0, b], self.base_host[p0, s])]
        lines.append("  oracle holds base block(s) %s" % wants)
        same_as = [int(x) for x in range(want.shape[1]) if np.array_equal(got[p0, b], want[p0, x])][:8]
        lines.append("  GPU bytes equal the oracle's block(s) %s of that plane" % same_as)
        lines.append("last 30 calls: " + "; ".join("%d %s" % rw for rw in self.log[-30:]))
        return "\n".join(lines)

    def checkpoint(self):
        for fn in self.pending:  # the oracle catches up, in program order
            fn()
        self.pending.clear()
        self.h.pool.kv_wait_all()
        self.stream.synchronize()
        try:
            self.h.assert_pool_equal()
        except AssertionError as err:
            raise AssertionError(str(err) + "\n" + self.diagnose()) from None
        for req in sorted(self.has_image):
            self.h.assert_image_equal(req)
        st = self.h.pool.kv_stats()
        assert st["bytes_out"] == self.h.oracle.bytes_out
        assert st["bytes_in"] == self.h.oracle.bytes_in
        free, _ = self.h.pool.kv_free_blocks()
        assert free + self.chk.n_used() == self.shape.n_blocks


CASES = {
    # name: (seed, flags, pool keywords)
    "two_streams_small_rings": (101, ORDER_COMPUTE, dict(staging_out_bytes=1 * MiB, staging_in_bytes=512 * KiB,
                                                         max_piece_bytes=128 * KiB, host_slack_blocks=4)),
    "four_streams_default_rings": (102, ORDER_COMPUTE | FOUR_STREAMS, dict(host_slack_blocks=0)),
    "three_streams_small_rings": (107, ORDER_COMPUTE | SCATTER_STREAM, dict(staging_out_bytes=1 * MiB, staging_in_bytes=512 * KiB,
                                                                         max_piece_bytes=64 * KiB)),
    "persistent_pack_kernel": (103, ORDER_COMPUTE, dict(pack_variant=1, staging_out_bytes=2 * MiB,
                                                        staging_in_bytes=2 * MiB, copy_chunk_bytes=64 * KiB)),
    "mapped_swap_in": (104, ORDER_COMPUTE | MAPPED_SWAP_IN, dict(host_slack_blocks=8)),
    # small swap-outs store to the host from a kernel, larger ones go through staging and copies
    "mapped_small_swap_outs": (106, ORDER_COMPUTE | MAPPED_SWAP_OUT, dict(mapped_out_max_blocks=12,
                                                                           host_slack_blocks=4)),
    "tight_host_arena": (105, ORDER_COMPUTE, dict(host_slack_blocks=2)),
    # every swap-out's copies enqueued by the pool's copy thread once its gathers have finished (the default does
    # that for swap-outs of 16 MiB or more only, which this small shape never reaches)
    "deferred_copies_two_streams": (108, ORDER_COMPUTE, dict(staging_out_bytes=1 * MiB, staging_in_bytes=512 * KiB,
                                                             max_piece_bytes=128 * KiB, defer_min_bytes=1)),
    "deferred_copies_three_streams": (109, ORDER_COMPUTE | SCATTER_STREAM, dict(host_slack_blocks=4, defer_min_bytes=1)),
    "deferred_copies_tight_host_arena": (110, ORDER_COMPUTE, dict(host_slack_blocks=2, defer_min_bytes=1)),
    "deferred_copies_four_streams_small_rings": (111, ORDER_COMPUTE | FOUR_STREAMS,
                                                 dict(staging_out_bytes=1 * MiB, staging_in_bytes=512 * KiB,
                                                      max_piece_bytes=64 * KiB, defer_min_bytes=1)),
    "deferred_copies_mapped_swap_in": (112, ORDER_COMPUTE | MAPPED_SWAP_IN, dict(host_slack_blocks=8, defer_min_bytes=1)),
}


@pytest.mark.parametrize("case", sorted(CASES))
def test_random_serving_loop_matches_oracle(case):
    import torch
    from gpu_util import Harness
    seed, flags, kw = CASES[case]
    host_bytes = 2 * MiB if case.endswith("tight_host_arena") else 64 * MiB
    stream = torch.cuda.Stream()
    h = Harness(SHAPE, seed, host_bytes, fill="random", flags=flags,
                compute_stream=stream.cuda_stream, **kw)
    try:
        rng = synth.rng_for(seed)
        loop = Loop(h, stream, rng, n_req=14)
        loop.tight = case.endswith("tight_host_arena")
        for i in range(1500):
            loop.step()
            if i % 150 == 149:
                loop.checkpoint()
        loop.checkpoint()
        assert h.oracle.bytes_out > 50 * SHAPE.R and h.oracle.bytes_in > 50 * SHAPE.R
        assert (loop.refused > 0) == loop.tight
    finally:
        h.close()


BIG_CASES = {
    # rings smaller than most requests: pieces wrap, gathers interleave with copies
    "small_rings": (201, ORDER_COMPUTE, dict(staging_out_bytes=48 * MiB, staging_in_bytes=24 * MiB,
                                            max_piece_bytes=8 * MiB, copy_chunk_bytes=4 * MiB)),
    "four_streams": (202, ORDER_COMPUTE | FOUR_STREAMS, dict(staging_out_bytes=256 * MiB, staging_in_bytes=64 * MiB)),
    "three_streams": (204, ORDER_COMPUTE | SCATTER_STREAM, dict(staging_out_bytes=128 * MiB, staging_in_bytes=32 * MiB,
                                                             max_piece_bytes=8 * MiB)),
    "mapped_both_ways": (203, ORDER_COMPUTE | MAPPED_SWAP_IN | MAPPED_SWAP_OUT, dict(mapped_out_max_blocks=64)),
    "second_lane": (207, ORDER_COMPUTE | SECOND_LANE, dict(staging_out_bytes=256 * MiB, staging_in_bytes=64 * MiB)),
    # the cases above hold back the copies of swap-outs of 16 MiB or more (the default); these hold back all, or none
    "all_copies_held_back_small_rings": (205, ORDER_COMPUTE, dict(staging_out_bytes=48 * MiB, staging_in_bytes=24 * MiB,
                                                                 max_piece_bytes=8 * MiB, defer_min_bytes=1)),
    "no_copies_held_back_three_streams": (206, ORDER_COMPUTE | SCATTER_STREAM | NO_DEFER_COPIES,
                                          dict(staging_out_bytes=128 * MiB, staging_in_bytes=32 * MiB)),
}


@pytest.mark.parametrize("case", sorted(BIG_CASES))
def test_random_serving_loop_with_millisecond_transfers(case):
    """The same loop with requests of up to 100 MiB: swaps take milliseconds, so unsynchronised
    calls overlap on the device for real and ordering mistakes would show in the bytes."""
    import torch
    from gpu_util import Harness
    seed, flags, kw = BIG_CASES[case]
    stream = torch.cuda.Stream()
    h = Harness(BIG, seed, 3 * 1024 * MiB, fill="random", flags=flags, compute_stream=stream.cuda_stream,
                host_slack_blocks=8, **kw)
    try:
        loop = Loop(h, stream, synth.rng_for(seed), n_req=12, max_blocks=200)
        for i in range(240):
            loop.step()
            if i % 80 == 79:
                loop.checkpoint()
        assert h.oracle.bytes_out > 2000 * BIG.R and h.oracle.bytes_in > 1000 * BIG.R
        assert h.pool.kv_stats()["conflict_waits"] > 0
    finally:
        h.close()
