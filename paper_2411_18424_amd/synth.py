"""Seeded synthetic inputs for the KV-swap path.

Shared by the tests, the benchmark and the CPU oracle's callers.  It holds no
part of the method itself: only shapes, random payloads, request lengths,
block tables and dirty masks.  The paper evaluates on the multi-round ShareGPT
conversations with offline Random / Markov priority traces (Section 4); neither
is available here, so seeded synthetic length mixes of the same scale stand in.

Everything is a pure function of (shape, seed): numpy's Philox generator.
"""

from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_BASE = 20241127


@dataclass(frozen=True)
class KVShape:
    """Shape of a paged KV pool: P = 2*n_layers planes of n_blocks chunks."""
    name: str
    n_layers: int
    n_kv_heads: int
    head_dim: int
    block_size: int
    elt_bytes: int
    n_blocks: int
    dtype: str  # "fp16" | "bf16": only decides how N(0,1) samples are rounded

    @property
    def P(self) -> int:
        return 2 * self.n_layers

    @property
    def C(self) -> int:
        return self.block_size * self.n_kv_heads * self.head_dim * self.elt_bytes

    @property
    def R(self) -> int:
        return self.P * self.C

    def with_blocks(self, n_blocks: int) -> "KVShape":
        return KVShape(self.name, self.n_layers, self.n_kv_heads, self.head_dim,
                       self.block_size, self.elt_bytes, int(n_blocks), self.dtype)


# The five workload shapes of the build (model shapes as the paper's Section 4
# names them: LLaMA-8B class, plus MHA and long-context GQA variants).
TINY = KVShape("tiny", 2, 4, 64, 16, 2, 256, "fp16")
LLAMA3_8B = KVShape("llama3-8b", 32, 8, 128, 16, 2, 8192, "bf16")
LLAMA2_13B = KVShape("llama2-13b", 40, 40, 128, 16, 2, 17578, "fp16")
QWEN2_72B = KVShape("qwen2-72b", 80, 8, 128, 16, 2, 2048 * 22, "bf16")


def rng_for(cfg: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=SEED_BASE + cfg, counter=[0, 0, 0, stream]))


# ------------------------------------------------------------------ payload
def normal_elements(rng: np.random.Generator, n_elts: int, dtype: str) -> np.ndarray:
    """n_elts samples of N(0,1) rounded to fp16 or bf16, returned as uint16."""
    x = rng.standard_normal(n_elts, dtype=np.float32)
    if dtype == "fp16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = x.view(np.uint32)
        # round-to-nearest-even truncation of fp32 to its top 16 bits
        u = u + 0x7FFF + ((u >> 16) & 1)
        return (u >> 16).astype(np.uint16)
    raise ValueError(dtype)


class PoolContent:
    """Deterministic content of every chunk of a pool.

    A base buffer of W random chunks (16 MiB) is drawn once; chunk (plane p, block b)
    is base window ``(p*2654435761 + b*40503 + seed) % W`` with its first 16
    bytes replaced by a stamp (magic, seed, plane, block) so that a chunk that
    lands in the wrong place is identified, not merely detected.
    """

    MAGIC = 0x4B565357  # "KVSW"

    def __init__(self, shape: KVShape, cfg: int, base_bytes: int = 16 << 20):
        self.shape = shape
        self.seed = SEED_BASE + cfg
        C = shape.C
        assert C % 16 == 0
        self.W = max(1, min(base_bytes // C, shape.P * shape.n_blocks))
        rng = rng_for(cfg, stream=1)
        elts = normal_elements(rng, self.W * C // shape.elt_bytes, shape.dtype)
        self.base = elts.view(np.uint8).reshape(self.W, C)

    def window(self, p, b):
        p = np.asarray(p, dtype=np.uint64)
        b = np.asarray(b, dtype=np.uint64)
        return ((p * np.uint64(2654435761) + b * np.uint64(40503) + np.uint64(self.seed))
                % np.uint64(self.W)).astype(np.int64)

    def stamp(self, p, b) -> np.ndarray:
        """16-byte stamps for arrays of planes / blocks: uint32[...,4]."""
        p = np.asarray(p, dtype=np.uint32)
        b = np.asarray(b, dtype=np.uint32)
        s = np.empty(p.shape + (4,), dtype=np.uint32)
        s[..., 0] = self.MAGIC
        s[..., 1] = np.uint32(self.seed & 0xFFFFFFFF)
        s[..., 2] = p
        s[..., 3] = b
        return s

    def plane(self, p: int, blocks=None) -> np.ndarray:
        """Bytes [len(blocks)][C] of plane p for the given physical blocks."""
        if blocks is None:
            blocks = np.arange(self.shape.n_blocks)
        blocks = np.asarray(blocks, dtype=np.int64)
        out = self.base[self.window(np.full(blocks.shape, p), blocks)]
        out[:, :16] = self.stamp(np.full(blocks.shape, p), blocks).view(np.uint8).reshape(-1, 16)
        return out

    def block(self, b: int) -> np.ndarray:
        """Bytes [P][C] of physical block b (all planes)."""
        ps = np.arange(self.shape.P)
        out = self.base[self.window(ps, np.full(ps.shape, b))]
        out[:, :16] = self.stamp(ps, np.full(ps.shape, b)).view(np.uint8).reshape(-1, 16)
        return out

    def payload(self, ids) -> np.ndarray:
        """Bytes [len(ids)][P][C] for arbitrary integer ids (fresh KV of appended tokens):
        the same windows-plus-stamp construction, cheap enough for GiB-sized payloads."""
        ids = np.asarray(ids, dtype=np.int64)
        out = np.empty((ids.size, self.shape.P, self.shape.C), dtype=np.uint8)
        for p in range(self.shape.P):
            out[:, p, :] = self.plane(p, ids)
        return out

    def fill(self, G: np.ndarray) -> None:
        """Fill a whole pool array G[P][N][C] (uint8) in place."""
        for p in range(self.shape.P):
            G[p] = self.plane(p)

    def fill_device(self, gpu_flat) -> None:
        """Same bytes as fill(), written into a flat uint8 torch tensor on the GPU.

        Only the small base buffer, window indices and stamps cross the host link; the
        pool itself is materialised by an index_select on the device.
        """
        import torch
        s = self.shape
        dev = gpu_flat.device
        view = gpu_flat.view(s.P, s.n_blocks, s.C)
        base = torch.from_numpy(self.base).to(dev)
        blocks = np.arange(s.n_blocks)
        for p in range(s.P):
            idx = torch.from_numpy(self.window(np.full(blocks.shape, p), blocks)).to(dev)
            torch.index_select(base, 0, idx, out=view[p])
            st = self.stamp(np.full(blocks.shape, p), blocks).view(np.uint8).reshape(-1, 16)
            view[p, :, :16] = torch.from_numpy(st).to(dev)
        torch.cuda.synchronize()

    def fill_device_blocks(self, gpu_flat, blocks) -> None:
        """As fill_device(), but only the given physical blocks (pools too large to fill)."""
        import torch
        s = self.shape
        dev = gpu_flat.device
        view = gpu_flat.view(s.P, s.n_blocks, s.C)
        base = torch.from_numpy(self.base).to(dev)
        blocks = np.asarray(blocks, dtype=np.int64)
        bidx = torch.from_numpy(blocks).to(dev)
        for p in range(s.P):
            idx = torch.from_numpy(self.window(np.full(blocks.shape, p), blocks)).to(dev)
            chunk = torch.index_select(base, 0, idx)
            st = self.stamp(np.full(blocks.shape, p), blocks).view(np.uint8).reshape(-1, 16)
            chunk[:, :16] = torch.from_numpy(st).to(dev)
            view[p, bidx, :] = chunk
        torch.cuda.synchronize()


    def fill_device_payload(self, gpu_flat, blocks, ids) -> None:
        """payload(ids) written into the physical blocks `blocks` of a flat uint8 torch tensor on
        the GPU, generated there (only window indices and stamps cross the host link)."""
        import torch
        s = self.shape
        dev = gpu_flat.device
        view = gpu_flat.view(s.P, s.n_blocks, s.C)
        if not hasattr(self, "_base_dev") or self._base_dev.device != dev:
            self._base_dev = torch.from_numpy(self.base).to(dev)
        blocks = np.asarray(blocks, dtype=np.int64)
        ids = np.asarray(ids, dtype=np.int64)
        assert blocks.shape == ids.shape
        bidx = torch.from_numpy(blocks).to(dev)
        ps = np.arange(s.P)
        win = torch.from_numpy(self.window(ps[:, None], ids[None, :])).to(dev)      # [P][n]
        st = torch.from_numpy(self.stamp(np.broadcast_to(ps[:, None], win.shape), np.broadcast_to(ids[None, :], win.shape))
                              .view(np.uint8).reshape(s.P, ids.size, 16)).to(dev)
        for p in range(s.P):
            chunk = torch.index_select(self._base_dev, 0, win[p])
            chunk[:, :16] = st[p]
            view[p, bidx, :] = chunk

    def heads(self, ids) -> np.ndarray:
        """First 16 bytes of every chunk of payload(ids): uint8 [len(ids)][P][16] (the stamps)."""
        ids = np.asarray(ids, dtype=np.int64)
        ps = np.arange(self.shape.P)
        st = self.stamp(np.broadcast_to(ps[None, :], (ids.size, ps.size)),
                        np.broadcast_to(ids[:, None], (ids.size, ps.size)))
        return st.view(np.uint8).reshape(ids.size, self.shape.P, 16)


def fresh_tokens(rng: np.random.Generator, shape: KVShape, n_blocks: int) -> np.ndarray:
    """Random replacement payload for n_blocks whole blocks: uint8 [n][P][C]."""
    elts = normal_elements(rng, n_blocks * shape.R // shape.elt_bytes, shape.dtype)
    return elts.view(np.uint8).reshape(n_blocks, shape.P, shape.C)


# ------------------------------------------------------------ request mixes
def blocks_for(tokens, block_size: int):
    return (np.asarray(tokens) + block_size - 1) // block_size


def lengths_uniform(rng, n_req: int, lo: int, hi: int) -> np.ndarray:
    return rng.integers(lo, hi + 1, size=n_req)


def lengths_lognormal(rng, n_req: int, median: float, sigma: float, lo: int, hi: int,
                      block_size: int, max_total_blocks: int) -> np.ndarray:
    """Lognormal token counts clipped to [lo, hi]; redrawn until they fit the pool."""
    while True:
        x = np.exp(rng.normal(np.log(median), sigma, size=n_req))
        t = np.clip(np.rint(x), lo, hi).astype(np.int64)
        if blocks_for(t, block_size).sum() <= max_total_blocks:
            return t


def lengths_loguniform(rng, n_req: int, lo: int, hi: int) -> np.ndarray:
    return np.rint(np.exp(rng.uniform(np.log(lo), np.log(hi), size=n_req))).astype(np.int64)


# -------------------------------------------------------------- block tables
def deal_tables(rng, n_pool_blocks: int, n_blocks_per_req, run: int = 1):
    """Deal physical blocks to requests from one seeded permutation.

    ``run`` = 1 gives fully fragmented tables.  ``run`` = g permutes g-aligned
    runs of the pool and each request takes whole runs (its last run may be
    partial), i.e. block groups of g contiguous blocks.
    Returns a list of int32 arrays; ids are never shared between requests.
    """
    n_runs = n_pool_blocks // run
    order = rng.permutation(n_runs)
    tables, cursor = [], 0
    for n in n_blocks_per_req:
        n = int(n)
        need = (n + run - 1) // run
        if cursor + need > n_runs:
            raise ValueError("pool too small for the requested tables")
        starts = order[cursor:cursor + need].astype(np.int64) * run
        cursor += need
        ids = (starts[:, None] + np.arange(run)[None, :]).reshape(-1)[:n]
        tables.append(ids.astype(np.int32))
    return tables


def random_mask(rng, n: int, frac: float) -> np.ndarray:
    m = (rng.random(n) < frac).astype(np.uint8)
    return m


def turn_dirty_mask(n_old_blocks: int, old_tokens: int, new_tokens: int, block_size: int) -> np.ndarray:
    """Dirty mask of a conversation turn that appended new_tokens.

    Dirty = the previous tail block if it was partly filled and received
    tokens, plus every newly appended block.
    """
    n_new_blocks = int(blocks_for(old_tokens + new_tokens, block_size))
    m = np.zeros(n_new_blocks, dtype=np.uint8)
    if new_tokens > 0 and old_tokens % block_size != 0 and n_old_blocks > 0:
        m[n_old_blocks - 1] = 1
    m[n_old_blocks:] = 1
    return m


# ------------------------------------------------------------ named workloads
@dataclass
class PreemptWorkload:
    """A pool full of requests, a set of victims to preempt, and fresh tables to resume into."""
    shape: KVShape
    cfg: int
    tokens: np.ndarray          # per request
    tables: list                # per request, current block table
    victims: list               # request ids to preempt
    resume_tables: list         # per victim, disjoint from every current table


def llama3_8b_preempt_workload(n_req: int = 64, n_victims: int = 16, run: int = 8,
                               shape: KVShape = LLAMA3_8B, cfg: int = 2) -> PreemptWorkload:
    """Config 2: lognormal request lengths (median 1k, max 8k tokens) in block groups of
    `run` contiguous blocks; 16 seeded victims; resume tables dealt from the free groups."""
    rng = rng_for(cfg)
    while True:
        tokens = lengths_lognormal(rng, n_req, 1024, 0.8, 16, 8192, shape.block_size, shape.n_blocks)
        nblk = blocks_for(tokens, shape.block_size)
        victims = sorted(int(v) for v in rng.permutation(n_req)[:n_victims])
        try:
            dealt = deal_tables(rng, shape.n_blocks, list(nblk) + [nblk[v] for v in victims], run=run)
        except ValueError:
            continue  # victims' resume tables did not fit the free space: redraw
        return PreemptWorkload(shape, cfg, tokens, dealt[:n_req], victims, dealt[n_req:])
