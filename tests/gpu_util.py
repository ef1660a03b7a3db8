"""Shared helpers of the GPU parity tests: a pool on the device (torch owns the
memory), the same bytes in a CPU oracle, and whole-pool comparison."""

from __future__ import annotations

import numpy as np

from oracle.kv_oracle import KVOracle
from paper_2411_18424_amd import synth


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
        got = self.pool.kv_host_view(req)
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
