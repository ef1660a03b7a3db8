"""Brute force on tiny pools: every injective block table, every dirty mask and
every contamination mask, checked against a flat-address formulation that
shares nothing with the oracle's array indexing.  CPU only."""

import itertools

import numpy as np

from oracle.kv_oracle import KVOracle


def flat_pool_addr(P, N, C, p, b, c):
    """Byte address of byte c of chunk (plane p, physical block b): planes are
    outermost, then blocks, then the bytes of the chunk."""
    return (p * N + b) * C + c


def flat_image_addr(P, C, j, p, c):
    """Byte address inside a host image: logical blocks outermost, then planes."""
    return (j * P + p) * C + c


def brute_swap_out(Gflat, P, N, C, T, sel, image_flat):
    out = list(image_flat)
    for j in sel:
        for p in range(P):
            for c in range(C):
                out[flat_image_addr(P, C, j, p, c)] = Gflat[flat_pool_addr(P, N, C, p, T[j], c)]
    return out


def brute_swap_in(Gflat, P, N, C, T, sel, image_flat):
    out = list(Gflat)
    for j in sel:
        for p in range(P):
            for c in range(C):
                out[flat_pool_addr(P, N, C, p, T[j], c)] = image_flat[flat_image_addr(P, C, j, p, c)]
    return out


def _oracle(L, N, seed):
    # C = 16 bytes: block_size 1, 1 head, head_dim 8, 2-byte elements
    o = KVOracle(L, 1, 8, 1, 2, N)
    rng = np.random.default_rng(seed)
    o.G[:] = rng.integers(0, 256, size=o.G.shape, dtype=np.uint8)
    return o, rng


def test_exhaustive_full_swap_round_trip():
    N = 4
    for L in (1, 2):
        for n in range(0, 4):
            for T in itertools.permutations(range(N), n):
                for T2 in itertools.permutations(range(N), n):
                    o, _ = _oracle(L, N, seed=n)
                    g0 = o.G.reshape(-1).tolist()
                    o.swap_out(0, list(T))
                    want_img = brute_swap_out(g0, o.P, N, o.C, T, range(n), [0] * (n * o.R))
                    assert o.host[0].Hq.reshape(-1).tolist() == want_img
                    o.swap_in(0, list(T2))
                    want_g = brute_swap_in(g0, o.P, N, o.C, T2, range(n), want_img)
                    assert o.G.reshape(-1).tolist() == want_g


def test_exhaustive_delta_masks():
    N, L = 4, 2
    checked = 0
    for n in range(1, 4):
        for T in itertools.permutations(range(N), n):
            for dirty in itertools.product((0, 1), repeat=n):
                for inval in itertools.product((0, 1), repeat=n):
                    o, rng = _oracle(L, N, seed=7)
                    o.swap_out(0, list(T))
                    img0 = o.host[0].Hq.reshape(-1).tolist()
                    o.G[:] = rng.integers(0, 256, size=o.G.shape, dtype=np.uint8)
                    g1 = o.G.reshape(-1).tolist()
                    o.host_invalidate(0, list(inval))
                    moved = o.swap_out_delta(0, list(T), list(dirty))
                    sel = [j for j in range(n) if dirty[j] or inval[j]]
                    assert moved == sel
                    assert o.host[0].Hq.reshape(-1).tolist() == \
                        brute_swap_out(g1, o.P, N, o.C, T, sel, img0)
                    assert o.bytes_out == (n + len(sel)) * o.R
                    checked += 1
    assert checked > 1000


def test_exhaustive_partial_swap_in():
    N, L = 4, 1
    for n in range(1, 4):
        for T2 in itertools.permutations(range(N), n):
            for res in itertools.product((0, 1), repeat=n):
                o, rng = _oracle(L, N, seed=3)
                T = list(range(n))
                o.swap_out(0, T)
                img = o.host[0].Hq.reshape(-1).tolist()
                o.G[:] = rng.integers(0, 256, size=o.G.shape, dtype=np.uint8)
                g1 = o.G.reshape(-1).tolist()
                moved = o.swap_in(0, list(T2), resident=list(res))
                sel = [j for j in range(n) if not res[j]]
                assert moved == sel
                assert o.G.reshape(-1).tolist() == brute_swap_in(g1, o.P, N, o.C, T2, sel, img)
