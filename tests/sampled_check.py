"""Oracle side of the GPU parity runs at the workloads' stated counts, where the data is far too
large for the CPU oracle to move all of it (hundreds of GiB per run).

Two KVOracle instances see every call the library sees:

* ``heads``: a pool whose chunks ARE the first 16 bytes of the real chunks, same planes, same
  number of physical blocks, the full block tables.  Gather and scatter move chunks as opaque
  bytes, so they commute with taking a byte range of every chunk: the first 16 bytes of every
  chunk of every host image and of the whole GPU pool must equal what this oracle holds.  The
  synthetic content stamps those bytes with (plane, content id), so a chunk that lands in the
  wrong place anywhere in a run is identified.
* ``full``: real chunk size, but a compact pool that holds only a sample of each request's
  logical blocks (the moved bytes of logical block j do not depend on any other block, so the
  oracle can compute sampled outputs one by one).  All bytes of the sampled blocks are compared.

Expected values come from these oracles only; the GPU side is written through the same
generator (paper_2411_18424_amd.synth.PoolContent) by content id.
"""

from __future__ import annotations

import numpy as np

from oracle.kv_oracle import KVOracle
from paper_2411_18424_amd import synth


class SampledCheck:
    def __init__(self, shape: synth.KVShape, cfg: int, host_bytes: int, slots: int, **pool_kw):
        import torch
        from paper_2411_18424_amd import kvswap

        self.torch, self.kv, self.shape = torch, kvswap, shape
        self.dev = torch.device("cuda:0")
        self.content = synth.PoolContent(shape, cfg)
        self.heads = KVOracle(shape.n_layers, 1, 1, 8, 2, shape.n_blocks)  # C = 16 bytes
        assert self.heads.C == 16
        self.full = KVOracle(shape.n_layers, shape.n_kv_heads, shape.head_dim, shape.block_size,
                             shape.elt_bytes, slots)
        self.free_slots = list(range(slots))[::-1]
        self.slot_of: dict[int, int] = {}      # physical block -> slot of the compact pool
        self.sample: dict[int, np.ndarray] = {}  # request -> sampled logical indices, ascending
        self.no_heads: set[int] = set()  # requests followed by the sampled-block oracle only (the heads
                                         # oracle loops over every chunk of a request in Python)
        self.gpu = torch.zeros(shape.R * shape.n_blocks, dtype=torch.uint8, device=self.dev)
        self.view = self.gpu.view(shape.P, shape.n_blocks, shape.C)
        self.pool = kvswap.KVPool(
            n_layers=shape.n_layers, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
            block_size=shape.block_size, elt_bytes=shape.elt_bytes, n_gpu_blocks=shape.n_blocks,
            gpu_base=self.gpu.data_ptr(), host_bytes=host_bytes, **pool_kw)

    # ------------------------------------------------------------------ sampled blocks
    def set_sample(self, req: int, js) -> None:
        self.sample[req] = np.unique(np.asarray(js, dtype=np.int64))

    def extend_sample(self, req: int, js) -> None:
        """New sampled indices must lie behind the old ones (the request grew)."""
        old = self.sample[req]
        js = np.unique(np.asarray(js, dtype=np.int64))
        assert js.size == 0 or old.size == 0 or js.min() > old.max()
        self.sample[req] = np.concatenate([old, js])

    def _slots(self, blocks, create: bool) -> np.ndarray:
        out = np.empty(len(blocks), dtype=np.int64)
        for k, b in enumerate(blocks):
            b = int(b)
            if b not in self.slot_of:
                assert create, "sampled block %d has no slot" % b
                self.slot_of[b] = self.free_slots.pop()
            out[k] = self.slot_of[b]
        return out

    def drop_blocks(self, blocks) -> None:
        """The request no longer owns these physical blocks (freed): their slots are recycled."""
        for b in blocks:
            s = self.slot_of.pop(int(b), None)
            if s is not None:
                self.free_slots.append(s)

    # ------------------------------------------------------------------ content
    def write(self, req: int, table, js, ids) -> None:
        """Logical blocks js of the request (physical table[js]) receive content `ids` (one content
        id per block) on the GPU and in both oracles."""
        table = np.asarray(table, dtype=np.int64)
        js = np.asarray(js, dtype=np.int64)
        ids = np.asarray(ids, dtype=np.int64)
        if js.size == 0:
            return
        self.content.fill_device_payload(self.gpu, table[js], ids)
        self.heads.G[:, table[js], :] = self.content.heads(ids).transpose(1, 0, 2)
        sel = np.isin(js, self.sample.get(req, np.zeros(0, np.int64)))
        if sel.any():
            slots = self._slots(table[js[sel]], create=True)
            self.full.G[:, slots, :] = self.content.payload(ids[sel]).transpose(1, 0, 2)

    def scribble(self, blocks, value: int) -> None:
        """Blocks that belong to nobody get a constant byte (a later owner must overwrite it)."""
        blocks = np.asarray(blocks, dtype=np.int64)
        if blocks.size == 0:
            return
        idx = self.torch.from_numpy(blocks).to(self.dev)
        self.view[:, idx, :] = value
        self.heads.G[:, blocks, :] = value
        for b in blocks:
            if int(b) in self.slot_of:
                self.full.G[:, self.slot_of[int(b)], :] = value

    # ------------------------------------------------------------------ the calls, oracle side
    def _sub(self, req: int, table, create: bool):
        S = self.sample[req]
        S = S[S < len(table)]
        return S, self._slots(np.asarray(table, dtype=np.int64)[S], create)

    def oracle_swap_out(self, req: int, table) -> None:
        if req not in self.no_heads:
            self.heads.swap_out(req, table)
        _, slots = self._sub(req, table, create=False)
        self.full.swap_out(req, slots)

    def oracle_swap_out_delta(self, req: int, table, dirty) -> list:
        moved = self.heads.swap_out_delta(req, table, dirty)
        S, slots = self._sub(req, table, create=False)
        self.full.swap_out_delta(req, slots, np.asarray(dirty)[S])
        return moved

    def oracle_swap_in(self, req: int, table, resident=None) -> list:
        moved = None
        if req not in self.no_heads:
            moved = self.heads.swap_in(req, table, resident=resident)
        S, slots = self._sub(req, table, create=True)  # fresh blocks get slots of their own
        self.full.swap_in(req, slots, resident=None if resident is None else np.asarray(resident)[S])
        return moved

    def oracle_invalidate(self, req: int, mask) -> None:
        self.heads.host_invalidate(req, mask)
        S = self.sample[req]
        self.full.host_invalidate(req, np.asarray(mask)[S[S < len(mask)]])

    def oracle_release(self, req: int) -> None:
        if req not in self.no_heads:
            self.heads.host_release(req)
        self.full.host_release(req)
        self.sample.pop(req, None)

    # ------------------------------------------------------------------ comparisons
    def check_image(self, req: int, rows=None) -> None:
        """Host image of req: first 16 bytes of every chunk of every valid block, and all bytes of
        the sampled blocks, against the oracles.  rows: when the image sits in several extents
        (no zero-copy view), compare the chunk heads of these logical blocks only."""
        pool, s = self.pool, self.shape
        pool.kv_wait(req)
        n = pool.kv_host_len(req)[0]
        view = pool.kv_host_view(req)
        want = self.heads.host.get(req)
        if want is not None:
            assert n == want.n_blocks, (n, want.n_blocks)
            assert np.array_equal(pool.kv_host_valid(req, n).astype(bool), want.host_valid)
        if want is not None and view is None and rows is not None:
            for j in np.unique(np.asarray(rows, dtype=np.int64)):
                if want.host_valid[j]:
                    got = pool.kv_host_read(req, int(j), 1)[0]
                    assert np.array_equal(got[:, :16], want.Hq[j]), \
                        "host image of req %d: chunk heads of logical block %d differ" % (req, j)
            want = None  # done
        for lo in range(0, n if want is not None else 0, 512):
            hi = min(n, lo + 512)
            got = view[lo:hi] if view is not None else pool.kv_host_read(req, lo, hi - lo)
            v = want.host_valid[lo:hi]
            if not np.array_equal(got[:, :, :16][v], want.Hq[lo:hi][v]):
                bad = np.argwhere((got[:, :, :16] != want.Hq[lo:hi]).any(axis=2) & v[:, None])
                raise AssertionError("host image of req %d: chunk heads differ at (block, plane) %s ..."
                                     % (req, (bad[:6] + [lo, 0]).tolist()))
        S = self.sample[req]
        S = S[S < n]
        fw = self.full.host[req]
        assert fw.n_blocks == S.size
        for k, j in enumerate(S):
            if not fw.host_valid[k]:
                continue
            got = view[j] if view is not None else pool.kv_host_read(req, int(j), 1)[0]
            if not np.array_equal(got, fw.Hq[k]):
                bad = np.flatnonzero((got != fw.Hq[k]).any(axis=1))
                raise AssertionError("host image of req %d: logical block %d differs in planes %s ..."
                                     % (req, j, bad[:6].tolist()))

    def check_blocks(self, req: int, table) -> None:
        """GPU blocks of a table: chunk heads of all of them, all bytes of the sampled ones."""
        table = np.asarray(table, dtype=np.int64)
        self.torch.cuda.synchronize()
        idx = self.torch.from_numpy(table).to(self.dev)
        got = self.view[:, idx, :16].cpu().numpy() if req not in self.no_heads else None
        if got is not None and not np.array_equal(got, self.heads.G[:, table, :]):
            bad = np.argwhere((got != self.heads.G[:, table, :]).any(axis=2))
            raise AssertionError("req %d: GPU chunk heads differ at (plane, index in table) %s ..."
                                 % (req, bad[:6].tolist()))
        S, slots = self._sub(req, table, create=False)
        if S.size:
            gidx = self.torch.from_numpy(table[S]).to(self.dev)
            gotf = self.view[:, gidx, :].cpu().numpy()
            if not np.array_equal(gotf, self.full.G[:, slots, :]):
                bad = np.argwhere((gotf != self.full.G[:, slots, :]).any(axis=2))
                raise AssertionError("req %d: sampled GPU blocks differ at (plane, sample index) %s ..."
                                     % (req, bad[:6].tolist()))

    def check_pool_heads(self) -> None:
        """First 16 bytes of every chunk of the whole GPU pool."""
        self.torch.cuda.synchronize()
        s = self.shape
        for p0 in range(0, s.P, 16):
            got = self.view[p0:p0 + 16, :, :16].cpu().numpy()
            if not np.array_equal(got, self.heads.G[p0:p0 + 16]):
                bad = np.argwhere((got != self.heads.G[p0:p0 + 16]).any(axis=2))
                raise AssertionError("GPU pool: chunk heads differ at (plane, block) %s ..."
                                     % ((bad[:6] + [p0, 0]).tolist()))

    def close(self) -> None:
        self.pool.kv_pool_destroy()
        del self.view, self.gpu
        self.torch.cuda.empty_cache()
