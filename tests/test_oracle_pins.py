"""Pins for the CPU oracle: closed forms, a second formulation through numpy's
own gather / scatter routines, a hand-worked fixture, invariants, and planted
mistakes that at least one pin must catch.  CPU only."""

import os

import numpy as np
import pytest

from oracle.kv_oracle import AllocChecker, KVOracle, OracleError
from paper_2411_18424_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make(shape=None, seed=1, **kw):
    shape = shape or synth.KVShape("t", 2, 2, 8, 4, 2, 24, "fp16")
    o = KVOracle(shape.n_layers, shape.n_kv_heads, shape.head_dim, shape.block_size,
                 shape.elt_bytes, shape.n_blocks)
    rng = np.random.default_rng(seed)
    o.G[:] = rng.integers(0, 256, size=o.G.shape, dtype=np.uint8)
    return o, rng


# ------------------------------------------------------------- hand-worked
def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split(":")
            out[k.strip()] = [int(x) for x in v.split()]
    return out


def test_handworked_fixture():
    g = _read_golden("handworked_swap.txt")
    L, H, D, B, e, N = g["shape"]
    o = KVOracle(L, H, D, B, e, N)
    for p in range(o.P):
        for b in range(N):
            for c in range(o.C):
                o.G[p, b, c] = 100 * p + 10 * b + c
    moved = o.swap_out(7, g["table_out"])
    assert moved == [0, 1]
    assert o.host[7].Hq.reshape(-1).tolist() == g["image"]
    o.swap_in(7, g["table_in"])
    assert o.G.reshape(-1).tolist() == g["pool_after"]


# ------------------------------------------------------------ closed forms
def test_identity_table_single_layer_is_memcpy():
    shape = synth.KVShape("t", 1, 2, 8, 4, 2, 16, "fp16")
    o, _ = make(shape)
    n = 5
    o.swap_out(0, np.arange(n))
    Hq = o.host[0].Hq
    for p in range(o.P):
        assert np.array_equal(Hq[:, p, :], o.G[p, 0:n, :])


def test_swap_in_to_same_table_is_noop_on_pool():
    o, rng = make()
    T = rng.permutation(o.N)[:9]
    before = o.G.copy()
    o.swap_out(3, T)
    o.swap_in(3, T)
    assert np.array_equal(o.G, before)


def test_delta_zero_mask_full_valid_moves_nothing():
    o, rng = make()
    T = rng.permutation(o.N)[:7]
    o.swap_out(1, T)
    img = o.host[1].Hq.copy()
    o.G[:] = rng.integers(0, 256, size=o.G.shape, dtype=np.uint8)  # GPU changed, nothing marked dirty
    out0 = o.bytes_out
    moved = o.swap_out_delta(1, T, np.zeros(7, np.uint8))
    assert moved == []
    assert o.bytes_out == out0
    assert np.array_equal(o.host[1].Hq, img)


def test_delta_all_ones_equals_full_swap_out():
    o1, rng = make(seed=5)
    o2, _ = make(seed=5)
    T = rng.permutation(o1.N)[:11]
    o1.swap_out(1, T)
    o2.swap_out(1, T)
    newG = rng.integers(0, 256, size=o1.G.shape, dtype=np.uint8)
    o1.G[:] = newG
    o2.G[:] = newG
    o1.swap_out(1, T)
    moved = o2.swap_out_delta(1, T, np.ones(11, np.uint8))
    assert moved == list(range(11))
    assert np.array_equal(o1.host[1].Hq, o2.host[1].Hq)
    assert o1.bytes_out == o2.bytes_out


def test_delta_without_prior_image_moves_all():
    o, rng = make()
    T = rng.permutation(o.N)[:6]
    moved = o.swap_out_delta(9, T, np.zeros(6, np.uint8))
    assert moved == list(range(6))
    assert o.host[9].host_valid.all()


# ------------------------------------------- second formulation (library)
def test_gather_equals_numpy_take():
    o, rng = make()
    for n in (1, 2, 9, o.N):
        T = rng.permutation(o.N)[:n]
        o.swap_out(n, T)
        want = np.take(o.G, T, axis=1).transpose(1, 0, 2)
        assert np.array_equal(o.host[n].Hq, want)


def test_scatter_equals_fancy_assignment():
    o, rng = make()
    T = rng.permutation(o.N)[:10]
    o.swap_out(0, T)
    T2 = rng.permutation(o.N)[:10]
    want = o.G.copy()
    want[:, T2, :] = o.host[0].Hq.transpose(1, 0, 2)
    o.swap_in(0, T2)
    assert np.array_equal(o.G, want)


def test_delta_equals_masked_take():
    o, rng = make()
    n = 12
    T = rng.permutation(o.N)[:n]
    o.swap_out(0, T)
    old = o.host[0].Hq.copy()
    o.G[:] = rng.integers(0, 256, size=o.G.shape, dtype=np.uint8)
    dirty = synth.random_mask(rng, n, 0.4)
    inval = synth.random_mask(rng, n, 0.3)
    o.host_invalidate(0, inval)
    moved = o.swap_out_delta(0, T, dirty)
    sel = (dirty | inval).astype(bool)
    assert moved == np.flatnonzero(sel).tolist()
    want = old.copy()
    want[sel] = np.take(o.G, T[sel], axis=1).transpose(1, 0, 2)
    assert np.array_equal(o.host[0].Hq, want)
    assert o.host[0].host_valid.all()


# --------------------------------------------------------------- invariants
def test_round_trip_preserves_every_token():
    shape = synth.KVShape("t", 3, 2, 4, 4, 2, 40, "fp16")
    o, rng = make(shape)
    perm = rng.permutation(o.N)
    n_tok = 4 * 7 - 2  # ragged tail block
    T = perm[:7]
    T2 = rng.permutation(o.N)[:7]
    before = o.token_kv(T, n_tok)
    o.swap_out(0, T)
    o.G[:, T, :] = 0xEE  # the preempted request's blocks are reused by others
    o.swap_in(0, T2)
    after = o.token_kv(T2, n_tok)
    assert np.array_equal(before, after)


def test_token_view_layout():
    # element (t,h,d) of layer l, K|V sits at chunk element (s*H+h)*D+d of block T[t//B]
    shape = synth.KVShape("t", 2, 3, 4, 2, 2, 6, "fp16")
    o, rng = make(shape)
    T = np.array([4, 1, 5])
    kv = o.token_kv(T, 5)
    flat = o.G.reshape(-1)
    for l, k, t, h, d, byte in [(0, 0, 0, 0, 0, 0), (1, 1, 4, 2, 3, 1), (0, 1, 3, 1, 2, 0), (1, 0, 2, 0, 1, 1)]:
        p = 2 * l + k
        j, s = divmod(t, o.B)
        addr = ((p * o.N + T[j]) * o.C) + (((s * o.H + h) * o.D + d) * o.e) + byte
        assert kv[l, k, t, h, d, byte] == flat[addr]


def test_block_record_multiset_preserved_and_others_untouched():
    o, rng = make()
    T = rng.permutation(o.N)[:8]
    T2 = rng.permutation(o.N)[:8]
    o.swap_out(0, T)
    rec_before = sorted(o.G[:, b, :].tobytes() for b in T)
    pool_before = o.G.copy()
    o.swap_in(0, T2)
    rec_after = sorted(o.G[:, b, :].tobytes() for b in T2)
    assert rec_before == rec_after
    others = np.setdiff1d(np.arange(o.N), T2)
    assert np.array_equal(o.G[:, others, :], pool_before[:, others, :])


def test_bytes_moved_counter():
    o, rng = make()
    n = 10
    T = rng.permutation(o.N)[:n]
    o.swap_out(0, T)
    assert o.bytes_out == n * o.R
    dirty = np.array([1, 0, 0, 1, 0, 0, 0, 0, 0, 1], np.uint8)
    inval = np.array([0, 1, 0, 1, 0, 0, 0, 0, 0, 0], np.uint8)
    o.host_invalidate(0, inval)
    moved = o.swap_out_delta(0, T, dirty)
    assert len(moved) == 4
    assert o.bytes_out == (n + 4) * o.R
    res = np.array([1, 1, 1, 0, 0, 0, 0, 0, 0, 0], np.uint8)
    moved = o.swap_in(0, T, resident=res)
    assert moved == list(range(3, 10))
    assert o.bytes_in == 7 * o.R


def test_partial_swap_in_leaves_resident_blocks_alone():
    o, rng = make()
    T = rng.permutation(o.N)[:6]
    o.swap_out(0, T)
    T2 = rng.permutation(o.N)[:6]
    res = np.array([1, 0, 1, 0, 0, 1], np.uint8)
    before = o.G.copy()
    o.swap_in(0, T2, resident=res)
    for j in range(6):
        if res[j]:
            assert np.array_equal(o.G[:, T2[j]], before[:, T2[j]])
        else:
            assert np.array_equal(o.G[:, T2[j]], o.host[0].Hq[j])


def test_growth_appends_blocks():
    o, rng = make()
    perm = rng.permutation(o.N)
    T = perm[:5]
    o.swap_out(0, T)
    old = o.host[0].Hq.copy()
    T_grown = perm[:8]
    o.G[:, T_grown[4:], :] = rng.integers(0, 256, size=(o.P, 4, o.C), dtype=np.uint8)
    dirty = synth.turn_dirty_mask(5, 5 * o.B - 1, 2 * o.B + 3, o.B)
    assert dirty.tolist() == [0, 0, 0, 0, 1, 1, 1, 1]
    moved = o.swap_out_delta(0, T_grown, dirty)
    assert moved == [4, 5, 6, 7]
    assert np.array_equal(o.host[0].Hq[:4], old[:4])
    assert np.array_equal(o.host[0].Hq[4:], np.take(o.G, T_grown[4:], axis=1).transpose(1, 0, 2))


def test_stamped_content_identifies_misrouted_chunk():
    shape = synth.TINY
    content = synth.PoolContent(shape, cfg=1)
    o = KVOracle(shape.n_layers, shape.n_kv_heads, shape.head_dim, shape.block_size,
                 shape.elt_bytes, shape.n_blocks)
    content.fill(o.G)
    rng = synth.rng_for(1)
    T = rng.permutation(shape.n_blocks)[:16]
    o.swap_out(0, T)
    stamps = o.host[0].Hq[:, :, :16].copy().view(np.uint32)  # [n][P][4]
    assert (stamps[..., 0] == content.MAGIC).all()
    assert np.array_equal(stamps[..., 2], np.broadcast_to(np.arange(shape.P)[None, :], (16, shape.P)))
    assert np.array_equal(stamps[..., 3], np.broadcast_to(T[:, None], (16, shape.P)))


# -------------------------------------------------------------- error paths
def test_rejects_bad_calls():
    o, rng = make()
    with pytest.raises(OracleError):
        o.swap_out(0, [0, 1, 1])
    with pytest.raises(OracleError):
        o.swap_out(0, [0, o.N])
    with pytest.raises(OracleError):
        o.swap_out(0, [-1])
    with pytest.raises(OracleError):
        o.swap_in(5, [0, 1])
    o.swap_out(0, [3, 4, 5])
    with pytest.raises(OracleError):
        o.swap_in(0, [0, 1])
    with pytest.raises(OracleError):
        o.swap_out_delta(0, [3, 4], [1, 1])
    with pytest.raises(OracleError):
        o.swap_out_delta(0, [3, 4, 5], [1, 1])
    o.host_invalidate(0, [0, 1, 0])
    before = o.G.copy()
    with pytest.raises(OracleError):
        o.swap_in(0, [6, 7, 8])
    assert np.array_equal(o.G, before)  # a rejected call has no effect
    o.swap_in(0, [6, 7, 8], resident=[0, 1, 0])
    o.host_release(0)
    with pytest.raises(OracleError):
        o.host_release(0)


def test_empty_request():
    o, _ = make()
    assert o.swap_out(0, []) == []
    assert o.swap_in(0, []) == []
    assert o.bytes_out == 0 and o.bytes_in == 0


# ------------------------------------------------------- allocator checker
def test_alloc_checker():
    c = AllocChecker(16)
    assert c.on_alloc(1, [0, 1, 2, 8, 9, 5]) == [3, 2, 1]
    with pytest.raises(AssertionError):
        c.on_alloc(2, [2])
    with pytest.raises(AssertionError):
        c.on_alloc(2, [16])
    with pytest.raises(AssertionError):
        c.on_alloc(2, [3, 3])
    with pytest.raises(AssertionError):
        c.on_free(2, [0])
    c.on_free(1, [0, 1, 2])
    assert c.n_used() == 3
    assert c.on_alloc(2, [2, 1, 0]) == [1, 1, 1]


# -------------------------------------------------------- planted mistakes
# Each mutant makes one plausible mistake in the oracle; the pins above, run
# against it, must fail.  This shows the pins have teeth.
class _DropLastPlane(KVOracle):
    def _move_out(self, img, T, moved):
        for j in moved:
            for p in range(self.P - 1):
                img.Hq[j, p, :] = self.G[p, T[j], :]
            img.host_valid[j] = True
        self.bytes_out += len(moved) * self.R
        return moved


class _SwapKV(KVOracle):
    def _move_out(self, img, T, moved):
        for j in moved:
            for p in range(self.P):
                img.Hq[j, p ^ 1, :] = self.G[p, T[j], :]
            img.host_valid[j] = True
        self.bytes_out += len(moved) * self.R
        return moved


class _LogicalInsteadOfPhysical(KVOracle):
    def _move_out(self, img, T, moved):
        for j in moved:
            for p in range(self.P):
                img.Hq[j, p, :] = self.G[p, j, :]
            img.host_valid[j] = True
        self.bytes_out += len(moved) * self.R
        return moved


class _InverseTable(KVOracle):
    def _move_out(self, img, T, moved):
        for j in moved:
            for p in range(self.P):
                img.Hq[j, p, :] = self.G[p, T[len(T) - 1 - j], :]
            img.host_valid[j] = True
        self.bytes_out += len(moved) * self.R
        return moved


class _IgnoresInvalid(KVOracle):
    def swap_out_delta(self, req, T, dirty):
        T = self._check_table(T)
        dirty = np.asarray(dirty).reshape(-1) != 0
        img = self.host[req]
        img.grow(T.size)
        moved = [j for j in range(T.size) if dirty[j]]
        return self._move_out(img, T, moved)


def _pins_against(cls):
    """Run the library-formulation pins against an oracle class; True if all pass."""
    shape = synth.KVShape("t", 2, 2, 8, 4, 2, 24, "fp16")
    rng = np.random.default_rng(11)
    o = cls(shape.n_layers, shape.n_kv_heads, shape.head_dim, shape.block_size,
            shape.elt_bytes, shape.n_blocks)
    o.G[:] = rng.integers(0, 256, size=o.G.shape, dtype=np.uint8)
    n = 9
    T = rng.permutation(o.N)[:n]
    o.swap_out(0, T)
    if not np.array_equal(o.host[0].Hq, np.take(o.G, T, axis=1).transpose(1, 0, 2)):
        return False
    old = o.host[0].Hq.copy()
    o.G[:] = rng.integers(0, 256, size=o.G.shape, dtype=np.uint8)
    dirty = np.array([1, 0, 0, 0, 1, 0, 0, 0, 0], np.uint8)
    inval = np.array([0, 0, 1, 0, 0, 0, 0, 1, 0], np.uint8)
    o.host_invalidate(0, inval)
    o.swap_out_delta(0, T, dirty)
    sel = (dirty | inval).astype(bool)
    want = old.copy()
    want[sel] = np.take(o.G, T[sel], axis=1).transpose(1, 0, 2)
    return bool(np.array_equal(o.host[0].Hq, want))


def test_pins_pass_on_the_real_oracle():
    assert _pins_against(KVOracle)


@pytest.mark.parametrize("mutant", [_DropLastPlane, _SwapKV, _LogicalInsteadOfPhysical,
                                    _InverseTable, _IgnoresInvalid])
def test_pins_catch_planted_mistakes(mutant):
    assert not _pins_against(mutant)
