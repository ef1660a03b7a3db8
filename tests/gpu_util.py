"""Shared helpers of the GPU parity tests: a pool on the device (torch owns the
memory), the same bytes in a CPU oracle, and whole-pool comparison."""

from __future__ import annotations

import numpy as np

from oracle.kv_oracle import KVOracle
from paper_2411_18424_amd import synth


def host_image(pool, req: int) -> np.ndarray:
    """The request's host image [n][P][C]: the library's zero-copy view when it offers one,
    else a copy made by kv_host_read."""
    v = pool.kv_host_view(req)
    return v if v is not None else pool.kv_host_read(req)


class Harness:
    """A KVPool on cuda:0 and a KVOracle holding identical bytes."""

    def __init__(self, shape: synth.KVShape, cfg: int, host_bytes: int, fill: str = "content", **pool_kw):
        import torch
        from paper_2411_18424_amd import kvswap

        self.torch = torch
        self.kv = kvswap
        self.shape = shape
        self.oracle = KVOracle(shape.n_layers, shape.n_kv_heads, shape.head_dim, shape.block_size,
                               shape.elt_bytes, shape.n_blocks)
        if fill == "content":
            synth.PoolContent(shape, cfg).fill(self.oracle.G)
        elif fill == "random":
            rng = synth.rng_for(cfg, stream=7)
            self.oracle.G[:] = rng.integers(0, 256, size=self.oracle.G.shape, dtype=np.uint8)
        self.dev = torch.device("cuda:0")
        self.gpu = torch.from_numpy(self.oracle.G.reshape(-1)).to(self.dev)
        torch.cuda.synchronize()
        self.pool = kvswap.KVPool(
            n_layers=shape.n_layers, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
            block_size=shape.block_size, elt_bytes=shape.elt_bytes, n_gpu_blocks=shape.n_blocks,
            gpu_base=self.gpu.data_ptr(), host_bytes=host_bytes, **pool_kw)

    def gpu_pool(self) -> np.ndarray:
        self.torch.cuda.synchronize()
        return self.gpu.cpu().numpy().reshape(self.oracle.G.shape)

    def overwrite_blocks(self, blocks, payload: np.ndarray) -> None:
        """Write payload [n][P][C] into physical blocks on both sides (new tokens' KV)."""
        blocks = np.asarray(blocks, dtype=np.int64)
        self.oracle.G[:, blocks, :] = payload.transpose(1, 0, 2)
        view = self.gpu.view(self.shape.P, self.shape.n_blocks, self.shape.C)
        idx = self.torch.from_numpy(blocks).to(self.dev)
        view[:, idx, :] = self.torch.from_numpy(np.ascontiguousarray(payload.transpose(1, 0, 2))).to(self.dev)
        self.torch.cuda.synchronize()

    def assert_pool_equal(self) -> None:
        got = self.gpu_pool()
        if not np.array_equal(got, self.oracle.G):
            bad = np.argwhere((got != self.oracle.G).any(axis=2))
            raise AssertionError("pool differs at (plane, block): %s ..." % bad[:8].tolist())

    def assert_image_equal(self, req: int) -> None:
        self.pool.kv_wait(req)
        got = host_image(self.pool, req)
        want = self.oracle.host[req]
        assert got.shape == want.Hq.shape, (got.shape, want.Hq.shape)
        valid = want.host_valid
        # bytes of blocks without a valid host copy are unspecified on both sides
        if not np.array_equal(got[valid], want.Hq[valid]):
            bad = np.argwhere((got != want.Hq).any(axis=2) & valid[:, None])
            raise AssertionError("host image of req %d differs at (logical block, plane): %s ..."
                                 % (req, bad[:8].tolist()))
        assert np.array_equal(self.pool.kv_host_valid(req, got.shape[0]).astype(bool), valid)

    def close(self) -> None:
        self.pool.kv_pool_destroy()


class SparseHarness:
    """Full-size pools: the GPU pool has the real N (addresses beyond 4 GiB, up to 0.8 of HBM),
    the oracle holds only the live blocks in a compact pool and sees every block table through
    an id map.  What a swap moves does not depend on N, only where it sits does, and that is
    the GPU side's business; expected bytes always come from the oracle."""

    def __init__(self, shape: synth.KVShape, cfg: int, host_bytes: int, live_blocks, **pool_kw):
        import torch
        from paper_2411_18424_amd import kvswap

        self.torch = torch
        self.kv = kvswap
        self.shape = shape
        self.dev = torch.device("cuda:0")
        live = np.unique(np.asarray(live_blocks, dtype=np.int64))
        self.live = live
        self.remap = np.full(shape.n_blocks, -1, dtype=np.int64)
        self.remap[live] = np.arange(live.size)
        self.oracle = KVOracle(shape.n_layers, shape.n_kv_heads, shape.head_dim, shape.block_size,
                               shape.elt_bytes, live.size)
        self.content = synth.PoolContent(shape, cfg)
        self.gpu = torch.empty(shape.R * shape.n_blocks, dtype=torch.uint8, device=self.dev)
        self.view = self.gpu.view(shape.P, shape.n_blocks, shape.C)
        self.pool = kvswap.KVPool(
            n_layers=shape.n_layers, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
            block_size=shape.block_size, elt_bytes=shape.elt_bytes, n_gpu_blocks=shape.n_blocks,
            gpu_base=self.gpu.data_ptr(), host_bytes=host_bytes, **pool_kw)

    def t(self, table) -> np.ndarray:
        """A physical block table as the compact oracle sees it."""
        ids = self.remap[np.asarray(table, dtype=np.int64)]
        assert (ids >= 0).all(), "table uses a block that was not declared live"
        return ids

    def load(self, blocks) -> None:
        """Give these physical blocks their seeded content on both sides."""
        blocks = np.asarray(blocks, dtype=np.int64)
        self.content.fill_device_blocks(self.gpu, blocks)
        for p in range(self.shape.P):
            self.oracle.G[p, self.remap[blocks], :] = self.content.plane(p, blocks)

    def stamp_canaries(self, blocks, value: int) -> None:
        blocks = np.asarray(blocks, dtype=np.int64)
        idx = self.torch.from_numpy(blocks).to(self.dev)
        self.view[:, idx, :] = value
        self.oracle.G[:, self.remap[blocks], :] = value
        self.torch.cuda.synchronize()

    def gpu_blocks(self, blocks) -> np.ndarray:
        """Bytes [P][len][C] of physical blocks, downloaded."""
        idx = self.torch.from_numpy(np.asarray(blocks, dtype=np.int64)).to(self.dev)
        self.torch.cuda.synchronize()
        return self.view[:, idx, :].cpu().numpy()

    def assert_blocks_equal(self, blocks, what="") -> None:
        blocks = np.asarray(blocks, dtype=np.int64)
        for lo in range(0, blocks.size, 256):  # bounded host memory
            part = blocks[lo:lo + 256]
            got = self.gpu_blocks(part)
            want = self.oracle.G[:, self.remap[part], :]
            if not np.array_equal(got, want):
                bad = np.argwhere((got != want).any(axis=2))
                raise AssertionError("%s pool differs at (plane, index in list): %s ..." % (what, bad[:8].tolist()))

    def assert_image_equal(self, req: int, sample=None) -> None:
        self.pool.kv_wait(req)
        want = self.oracle.host[req]
        n = self.pool.kv_host_len(req)[0]
        assert n == want.Hq.shape[0], (n, want.Hq.shape)
        view = self.pool.kv_host_view(req)  # None for an image in several extents

        def blocks(js):
            if view is not None:
                return view[js]
            return np.concatenate([self.pool.kv_host_read(req, int(j), 1) for j in js]) if len(js) else \
                np.zeros((0, self.shape.P, self.shape.C), np.uint8)

        js = np.arange(n) if sample is None else np.asarray(sample)
        js = js[want.host_valid[js]]
        for lo in range(0, js.size, 128):
            part = js[lo:lo + 128]
            got = blocks(part)
            if not np.array_equal(got, want.Hq[part]):
                bad = np.argwhere((got != want.Hq[part]).any(axis=2))
                raise AssertionError("host image of req %d differs at (index, plane): %s ..." % (req, bad[:8].tolist()))
        # first 16 bytes of every chunk (the stamp or whatever the block holds): whole image
        valid = want.host_valid
        for lo in range(0, n, 256):
            hi = min(n, lo + 256)
            got = view[lo:hi] if view is not None else self.pool.kv_host_read(req, lo, hi - lo)
            v = valid[lo:hi]
            assert np.array_equal(got[:, :, :16][v], want.Hq[lo:hi, :, :16][v]), "chunk heads differ"

    def close(self) -> None:
        self.pool.kv_pool_destroy()
        del self.view, self.gpu
        self.torch.cuda.empty_cache()
