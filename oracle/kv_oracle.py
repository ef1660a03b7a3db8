"""CPU oracle for the KV-cache swap path (TEST INFRASTRUCTURE ONLY).

This module is the plain, slow, obviously-correct definition of what a
preemption-driven KV-cache context switch moves.  It exists so that the HIP
library can be compared with it byte for byte.  Only tests, the smoke check and
the benchmark's ``cpu_baseline`` leg may import it; the product path never
does, and this module imports nothing from the product package.

What is modelled (FastSwitch, arXiv 2411.18424):

* A swap moves a request's KV cache between GPU memory and CPU memory so that
  it need not be recomputed (Section 1; Section 2.1 "Preemption").  The result
  is an exact copy, so the oracle is the definition of that copy, written as
  nested loops over logical blocks and planes.
* KV memory is paged in fixed blocks of ``block_size`` tokens, the unit of
  allocation and of transfer (Section 2.2, Challenge #1; Section 3.1).
* A copy of the KV cache is kept in CPU memory after swap-in; on the next
  swap-out only what that copy lacks is moved, and parts of the copy that were
  contaminated (reclaimed) are tracked and sent again (Section 3.3).

Layouts (the paper fixes neither; these are this build's readings):

* GPU pool  ``G[P][N][C]`` bytes, ``P = 2*n_layers`` planes with plane index
  ``p = 2*layer + kv`` (kv 0 = K, 1 = V), ``N`` physical blocks, chunk size
  ``C = block_size * n_kv_heads * head_dim * elt_bytes``.  Inside a chunk the
  element of token ``t``, head ``h``, dim ``d`` is number ``(t*H + h)*D + d``.
* Host image of a request with ``n`` logical blocks: ``Hq[n][P][C]`` bytes
  (block-major), plus one ``host_valid`` bit per logical block.

Parity pins: every function here is pinned by tests/test_oracle_pins.py and
tests/test_oracle_bruteforce.py (closed forms, a second formulation through
numpy.take / fancy assignment, flat-address brute force on tiny pools, a hand
worked fixture, invariants, and planted-mistake checks).  Nothing is unpinned.
"""

from __future__ import annotations

import numpy as np


class OracleError(ValueError):
    """Raised for a call the swap path must reject (bad table, no host copy)."""


class HostImage:
    """CPU-side copy of one request's KV cache (Section 3.3)."""

    def __init__(self, n_blocks: int, P: int, C: int):
        self.Hq = np.zeros((n_blocks, P, C), dtype=np.uint8)
        self.host_valid = np.zeros(n_blocks, dtype=bool)

    @property
    def n_blocks(self) -> int:
        return self.Hq.shape[0]

    def grow(self, n_blocks: int) -> None:
        """Append room for new logical blocks; their bits start invalid."""
        old = self.n_blocks
        if n_blocks < old:
            raise OracleError("a host image never shrinks")
        if n_blocks == old:
            return
        Hq = np.zeros((n_blocks,) + self.Hq.shape[1:], dtype=np.uint8)
        Hq[:old] = self.Hq
        valid = np.zeros(n_blocks, dtype=bool)
        valid[:old] = self.host_valid
        self.Hq, self.host_valid = Hq, valid


class KVOracle:
    """Paged KV pool + per-request host images, moved by plain loops."""

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int,
                 block_size: int, elt_bytes: int, n_blocks: int):
        self.L, self.H, self.D = int(n_layers), int(n_kv_heads), int(head_dim)
        self.B, self.e, self.N = int(block_size), int(elt_bytes), int(n_blocks)
        self.P = 2 * self.L
        self.C = self.B * self.H * self.D * self.e
        self.R = self.P * self.C
        self.G = np.zeros((self.P, self.N, self.C), dtype=np.uint8)
        self.host: dict[int, HostImage] = {}
        self.bytes_out = 0
        self.bytes_in = 0

    # ------------------------------------------------------------------ checks
    def _check_table(self, T) -> np.ndarray:
        T = np.asarray(T, dtype=np.int64).reshape(-1)
        if T.size and (T.min() < 0 or T.max() >= self.N):
            raise OracleError("block id out of range")
        if np.unique(T).size != T.size:
            raise OracleError("duplicate block id in table")
        return T

    # --------------------------------------------------------------- swap out
    def swap_out(self, req: int, T) -> list[int]:
        """Full swap-out: every logical block j of the request goes to the host.

        ``Hq[j][p] = G[p][T[j]]`` for all j, p.  Any earlier host copy of the
        request is discarded first (Section 2.1: the whole KV cache of the
        preempted request is transferred).
        """
        T = self._check_table(T)
        img = HostImage(T.size, self.P, self.C)
        self.host[req] = img
        return self._move_out(img, T, list(range(T.size)))

    def swap_out_delta(self, req: int, T, dirty) -> list[int]:
        """Swap-out with reuse of the CPU copy (Section 3.3).

        Moves exactly the logical blocks j with ``dirty[j]`` set or with no
        valid host copy; all other bytes of the image stay as they are.  A
        request that grew since its last swap-out gets its image extended.
        Returns the moved set, ascending.
        """
        T = self._check_table(T)
        dirty = np.asarray(dirty).reshape(-1) != 0
        if dirty.size != T.size:
            raise OracleError("dirty mask length differs from table length")
        img = self.host.get(req)
        if img is None:
            img = HostImage(T.size, self.P, self.C)
            self.host[req] = img
        elif T.size < img.n_blocks:
            raise OracleError("table shorter than the host image")
        else:
            img.grow(T.size)
        moved = [j for j in range(T.size) if dirty[j] or not img.host_valid[j]]
        return self._move_out(img, T, moved)

    def _move_out(self, img: HostImage, T: np.ndarray, moved: list[int]) -> list[int]:
        for j in moved:
            for p in range(self.P):
                img.Hq[j, p, :] = self.G[p, T[j], :]
            img.host_valid[j] = True
        self.bytes_out += len(moved) * self.R
        return moved

    # ---------------------------------------------------------------- swap in
    def swap_in(self, req: int, T_new, resident=None) -> list[int]:
        """Swap-in into freshly allocated blocks (Section 3.2, swap-in path).

        ``G[p][T_new[j]] = Hq[j][p]`` for every logical block j that is not
        already resident on the GPU (all of them when ``resident`` is None,
        which is the paper's flow: a preempted request holds no GPU blocks).
        The host image is kept, unchanged, for later reuse (Section 3.3).
        """
        T_new = self._check_table(T_new)
        img = self.host.get(req)
        if img is None:
            raise OracleError("request has no host copy")
        if T_new.size != img.n_blocks:
            raise OracleError("table length differs from the host image")
        if resident is None:
            resident = np.zeros(T_new.size, dtype=bool)
        resident = np.asarray(resident).reshape(-1) != 0
        if resident.size != T_new.size:
            raise OracleError("resident mask length differs from table length")
        moved = [j for j in range(T_new.size) if not resident[j]]
        for j in moved:
            if not img.host_valid[j]:
                raise OracleError("logical block %d has no valid host copy" % j)
        for j in moved:
            for p in range(self.P):
                self.G[p, T_new[j], :] = img.Hq[j, p, :]
        self.bytes_in += len(moved) * self.R
        return moved

    # ------------------------------------------------------------- reuse map
    def host_invalidate(self, req: int, mask) -> None:
        """Mark blocks of the CPU copy contaminated (Section 3.3): their bytes
        may no longer be trusted and the next swap-out sends them again."""
        img = self.host.get(req)
        if img is None:
            raise OracleError("request has no host copy")
        mask = np.asarray(mask).reshape(-1) != 0
        if mask.size != img.n_blocks:
            raise OracleError("mask length differs from the host image")
        img.host_valid[mask] = False

    def host_release(self, req: int) -> None:
        if req not in self.host:
            raise OracleError("request has no host copy")
        del self.host[req]

    # ---------------------------------------------------------- logical view
    def token_kv(self, T, n_tokens: int) -> np.ndarray:
        """K and V of the first ``n_tokens`` tokens read through table ``T``.

        Returns bytes shaped ``[L][2][n_tokens][H][D][e]``: what attention
        would read for this request, independent of where the blocks sit.
        """
        T = self._check_table(T)
        if n_tokens > T.size * self.B:
            raise OracleError("more tokens than the table holds")
        out = np.zeros((self.L, 2, n_tokens, self.H, self.D, self.e), dtype=np.uint8)
        for layer in range(self.L):
            for kv in range(2):
                p = 2 * layer + kv
                for t in range(n_tokens):
                    j, s = divmod(t, self.B)
                    chunk = self.G[p, T[j]].reshape(self.B, self.H, self.D, self.e)
                    out[layer, kv, t] = chunk[s]
        return out


class AllocChecker:
    """Invariant checker for a block-group allocator (Section 3.1).

    Many allocations are correct, so this is not an allocator: it replays the
    ids an allocator returned and fails on any id out of range, handed out
    twice, or freed while not owned, and it reports contiguous-run lengths.
    """

    def __init__(self, n_blocks: int):
        self.N = int(n_blocks)
        self.owner: dict[int, int] = {}

    def on_alloc(self, req: int, ids) -> list[int]:
        ids = [int(b) for b in ids]
        if len(set(ids)) != len(ids):
            raise AssertionError("allocator returned an id twice in one call")
        for b in ids:
            if not 0 <= b < self.N:
                raise AssertionError("allocator returned id %d out of range" % b)
            if b in self.owner:
                raise AssertionError("block %d double-assigned (owner %d, new %d)"
                                     % (b, self.owner[b], req))
        for b in ids:
            self.owner[b] = req
        return self.run_lengths(ids)

    def on_free(self, req: int, ids) -> None:
        for b in ids:
            b = int(b)
            if self.owner.get(b) != req:
                raise AssertionError("block %d freed by %d but not owned by it" % (b, req))
            del self.owner[b]

    def n_used(self) -> int:
        return len(self.owner)

    @staticmethod
    def run_lengths(ids) -> list[int]:
        """Lengths of the maximal runs of consecutive ascending ids, in order."""
        runs: list[int] = []
        prev = None
        for b in ids:
            b = int(b)
            if prev is not None and b == prev + 1:
                runs[-1] += 1
            else:
                runs.append(1)
            prev = b
        return runs
