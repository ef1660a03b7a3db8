"""ctypes binding over libkvswap.so: argument marshalling only.

Every function of include/kvswap.h is exposed under its own name on ``lib``;
``KVPool`` is a thin convenience object around a ``kv_pool_t*`` with methods of the
same names.  Nothing here moves, gathers or computes a byte (host images are read through
kv_host_read / kv_host_view of the library): if the shared library is missing
the import fails loudly (build it with ``python -m paper_2411_18424_amd.build``).
"""

from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvswap.so")

KV_OK, KV_EINVAL, KV_ENOMEM_GPU, KV_ENOMEM_HOST = 0, -1, -2, -3
KV_ENOENT, KV_EBUSY, KV_EHIP, KV_ENODEV = -4, -5, -6, -7
KV_FLAG_PLAN_ONLY, KV_FLAG_PROFILE, KV_FLAG_ORDER_COMPUTE, KV_FLAG_FOUR_STREAMS = 1, 2, 4, 8
KV_FLAG_MAPPED_SWAP_IN, KV_FLAG_HOST_EVICT, KV_FLAG_MAPPED_SWAP_OUT, KV_FLAG_SCATTER_STREAM = 16, 32, 64, 128
KV_FLAG_NO_STRIDED_COPIES = 256
KV_FLAG_NO_DEFER_COPIES = 512
KV_FLAG_SECOND_LANE = 1024
KV_FLAG_NO_LAUNCH_EVENTS = 2048
KV_TASK_SWAP_OUT, KV_TASK_SWAP_IN, KV_TASK_SWAP_OUT_DELTA, KV_TASK_SWAP_IN_DELTA = 0, 1, 2, 3
KV_WHERE_RUNNING, KV_WHERE_SWAPPED, KV_WHERE_ONGOING_SWAP_IN = 0, 1, 2
KV_IT_FREE_OUT_BLOCKS = 1

_STATUS_NAMES = {0: "KV_OK", -1: "KV_EINVAL", -2: "KV_ENOMEM_GPU", -3: "KV_ENOMEM_HOST",
                 -4: "KV_ENOENT", -5: "KV_EBUSY", -6: "KV_EHIP", -7: "KV_ENODEV"}


class KVError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("%s: %s" % (_STATUS_NAMES.get(status, status), text))
        self.status = status


class kv_pool_config_t(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("block_size", C.c_int32), ("elt_bytes", C.c_int32), ("flags", C.c_int32),
        ("n_gpu_blocks", C.c_int64), ("gpu_base", C.c_void_p), ("host_bytes", C.c_int64),
        ("staging_base", C.c_void_p), ("staging_out_bytes", C.c_int64),
        ("staging_in_bytes", C.c_int64), ("max_piece_bytes", C.c_int64),
        ("copy_chunk_bytes", C.c_int64), ("compute_stream", C.c_void_p),
        ("host_slack_blocks", C.c_int32), ("gather_grid", C.c_int32),
        ("tile_unroll", C.c_int32), ("pack_variant", C.c_int32),
        ("mapped_in_grid", C.c_int32), ("mapped_out_max_blocks", C.c_int32),
        ("defer_min_bytes", C.c_int64),
    ]


class kv_stats_t(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "bytes_out", "bytes_in", "blocks_out", "blocks_in", "gather_launches",
        "scatter_launches", "d2h_copies", "h2d_copies", "conflict_waits",
        "host_new_extents", "host_evicted_blocks", "host_arena_used", "host_arena_bytes",
        "strided_copies", "second_lane_copies")]


class kv_bg_stats_t(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("n_requests", "n_groups", "used_blocks", "tail_blocks",
                                         "steals", "opened", "appended_groups", "grown_in_place")]


class kv_manager_config_t(C.Structure):
    _fields_ = [("window", C.c_int32), ("reserved", C.c_int32), ("link_gbps", C.c_double),
                ("sync_below_ms", C.c_double)]


class kv_manager_stats_t(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("submitted", "dispatched", "failed", "queued", "in_flight",
                                         "strategy_calls", "strategy_async")] + \
               [("dispatch_us_sum", C.c_double), ("queue_wait_us_sum", C.c_double)]


class kv_iteration_t(C.Structure):
    _fields_ = [("n_swap_in", C.c_int32), ("n_swap_out", C.c_int32),
                ("in_reqs", C.POINTER(C.c_int64)), ("in_tables", C.POINTER(C.c_int32)),
                ("in_n_blocks", C.POINTER(C.c_int32)),
                ("out_reqs", C.POINTER(C.c_int64)), ("out_tables", C.POINTER(C.c_int32)),
                ("out_n_blocks", C.POINTER(C.c_int32)), ("out_dirty", C.POINTER(C.c_uint8)),
                ("force_mode", C.c_int32), ("flags", C.c_int32)]


class kv_iteration_result_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("completed_swap_ins", "waited_swap_ins", "async", "conflicts",
                                         "ongoing_swap_ins", "failures")]


class kv_iteration_stats_t(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("iterations", "swap_ins", "swap_outs", "async_iterations",
                                         "sync_iterations", "conflicts", "resumed")]


class kv_prof_record_t(C.Structure):
    _fields_ = [("kind", C.c_int32), ("reserved", C.c_int32), ("bytes", C.c_int64), ("ms", C.c_double),
                ("start_ms", C.c_double)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libkvswap.so is not built (%s). Run `python -m paper_2411_18424_amd.build`; "
            "there is no fallback path." % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    P = C.POINTER
    pool_p = C.c_void_p
    i32p, i64p, u8p = P(C.c_int32), P(C.c_int64), P(C.c_uint8)
    sig = {
        "kv_pool_create": (C.c_int32, [P(kv_pool_config_t), P(pool_p)]),
        "kv_pool_destroy": (C.c_int32, [pool_p]),
        "alloc_block_group": (C.c_int32, [pool_p, C.c_int64, C.c_int32, C.c_int32, i32p, i32p]),
        "free_block_group": (C.c_int32, [pool_p, C.c_int64, i32p, C.c_int32]),
        "kv_free_blocks": (C.c_int32, [pool_p, i64p, i64p]),
        "kv_bg_configure": (C.c_int32, [pool_p, C.c_int32, C.c_uint64]),
        "kv_bg_append": (C.c_int32, [pool_p, C.c_int64, C.c_int32, C.c_int32, i32p]),
        "kv_bg_table": (C.c_int32, [pool_p, C.c_int64, i32p, C.c_int32, i32p]),
        "kv_bg_close": (C.c_int32, [pool_p, C.c_int64]),
        "kv_bg_stats": (C.c_int32, [pool_p, P(kv_bg_stats_t)]),
        "swap_out": (C.c_int32, [pool_p, C.c_int64, i32p, C.c_int32]),
        "swap_out_delta": (C.c_int32, [pool_p, C.c_int64, i32p, C.c_int32, u8p, i32p]),
        "swap_out_static": (C.c_int32, [pool_p, i32p, C.c_int32, C.c_void_p, C.c_void_p]),
        "swap_in": (C.c_int32, [pool_p, C.c_int64, i32p, C.c_int32]),
        "swap_in_delta": (C.c_int32, [pool_p, C.c_int64, i32p, C.c_int32, u8p, i32p]),
        "swap_out_direct": (C.c_int32, [pool_p, C.c_int64, i32p, C.c_int32, C.c_int32]),
        "swap_in_direct": (C.c_int32, [pool_p, C.c_int64, i32p, C.c_int32, C.c_int32]),
        "swap_in_layerwise": (C.c_int32, [pool_p, C.c_int64, i32p, C.c_int32, u8p, C.c_int32, i32p]),
        "kv_stream_wait_layer": (C.c_int32, [pool_p, C.c_int64, C.c_int32, C.c_void_p]),
        "kv_wait_layer": (C.c_int32, [pool_p, C.c_int64, C.c_int32]),
        "swap_out_batch": (C.c_int32, [pool_p, C.c_int32, i64p, i32p, i32p]),
        "swap_in_batch": (C.c_int32, [pool_p, C.c_int32, i64p, i32p, i32p]),
        "kv_wait": (C.c_int32, [pool_p, C.c_int64]),
        "kv_query": (C.c_int32, [pool_p, C.c_int64, i32p]),
        "kv_wait_packed": (C.c_int32, [pool_p, C.c_int64]),
        "kv_stream_wait": (C.c_int32, [pool_p, C.c_int64, C.c_void_p]),
        "kv_wait_all": (C.c_int32, [pool_p]),
        "kv_host_len": (C.c_int32, [pool_p, C.c_int64, i32p, i32p]),
        "kv_host_blocks": (C.c_int32, [pool_p, C.c_int64, P(C.c_void_p), i64p, C.c_int32]),
        "kv_host_read": (C.c_int32, [pool_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p]),
        "kv_host_view": (C.c_int32, [pool_p, C.c_int64, P(C.c_void_p), i64p]),
        "kv_host_valid": (C.c_int32, [pool_p, C.c_int64, u8p, C.c_int32]),
        "kv_host_invalidate": (C.c_int32, [pool_p, C.c_int64, u8p, C.c_int32]),
        "kv_host_release": (C.c_int32, [pool_p, C.c_int64]),
        "kv_host_set_priority": (C.c_int32, [pool_p, C.c_int64, C.c_int32]),
        "kv_stats": (C.c_int32, [pool_p, P(kv_stats_t)]),
        "kv_profile_read": (C.c_int32, [pool_p, P(kv_prof_record_t), C.c_int32, i32p]),
        "kv_profile_reset": (C.c_int32, [pool_p]),
        "kv_link_probe": (C.c_int32, [C.c_int64, C.c_int32, C.c_int32, P(C.c_double)]),
        "kv_hbm_probe": (C.c_int32, [C.c_int64, C.c_int32, P(C.c_double)]),
        "kv_record_bytes": (C.c_int32, [pool_p, i64p]),
        "kv_manager_create": (C.c_int32, [pool_p, P(kv_manager_config_t), P(C.c_void_p)]),
        "kv_manager_destroy": (C.c_int32, [C.c_void_p]),
        "kv_manager_submit": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int64, i32p, C.c_int32, u8p,
                                          P(C.c_uint64)]),
        "kv_manager_poll": (C.c_int32, [C.c_void_p, P(C.c_uint64), i32p, C.c_int32, i32p]),
        "kv_manager_wait": (C.c_int32, [C.c_void_p, C.c_uint64, i32p]),
        "kv_manager_drain": (C.c_int32, [C.c_void_p]),
        "kv_manager_strategy": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int64, i32p]),
        "kv_manager_stats": (C.c_int32, [C.c_void_p, P(kv_manager_stats_t)]),
        "kv_manager_iterate": (C.c_int32, [C.c_void_p, P(kv_iteration_t), i64p, C.c_int32, i32p,
                                           P(kv_iteration_result_t)]),
        "kv_manager_failures": (C.c_int32, [C.c_void_p, i64p, i32p, C.c_int32, i32p]),
        "kv_manager_where": (C.c_int32, [C.c_void_p, C.c_int64, i32p]),
        "kv_manager_iteration_stats": (C.c_int32, [C.c_void_p, P(kv_iteration_stats_t)]),
        "kv_last_error": (C.c_char_p, []),
        "kv_version": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    lib._signatures = sig
    return lib


lib = _load()


def _check(status: int) -> int:
    if status != KV_OK:
        raise KVError(status, (lib.kv_last_error() or b"").decode())
    return status


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _u8(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data_as(C.POINTER(C.c_uint8))


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(C.POINTER(C.c_int64))


def kv_link_probe(n_bytes: int, direction: int, reps: int = 10) -> float:
    out = C.c_double()
    _check(lib.kv_link_probe(n_bytes, direction, reps, C.byref(out)))
    return out.value


def kv_hbm_probe(n_bytes: int, reps: int = 10) -> float:
    out = C.c_double()
    _check(lib.kv_hbm_probe(n_bytes, reps, C.byref(out)))
    return out.value


class KVPool:
    """Owner of one ``kv_pool_t*``.  Methods carry the C functions' names."""

    def __init__(self, *, n_layers, n_kv_heads, head_dim, block_size, elt_bytes, n_gpu_blocks,
                 gpu_base=0, host_bytes=0, staging_base=0, staging_out_bytes=0, staging_in_bytes=0,
                 max_piece_bytes=0,
                 host_slack_blocks=-1, copy_chunk_bytes=0, compute_stream=0, flags=0,
                 gather_grid=0, tile_unroll=0, pack_variant=0, mapped_in_grid=0,
                 mapped_out_max_blocks=0, defer_min_bytes=0):
        cfg = kv_pool_config_t(
            n_layers=n_layers, n_kv_heads=n_kv_heads, head_dim=head_dim, block_size=block_size,
            elt_bytes=elt_bytes, flags=flags, n_gpu_blocks=n_gpu_blocks, gpu_base=gpu_base or None,
            host_bytes=host_bytes, staging_base=staging_base or None,
            staging_out_bytes=staging_out_bytes, staging_in_bytes=staging_in_bytes,
            max_piece_bytes=max_piece_bytes, copy_chunk_bytes=copy_chunk_bytes,
            compute_stream=compute_stream or None, host_slack_blocks=host_slack_blocks,
            gather_grid=gather_grid, tile_unroll=tile_unroll, pack_variant=pack_variant,
            mapped_in_grid=mapped_in_grid, mapped_out_max_blocks=mapped_out_max_blocks,
            defer_min_bytes=defer_min_bytes)
        self._h = C.c_void_p()
        _check(lib.kv_pool_create(C.byref(cfg), C.byref(self._h)))
        self.P = 2 * n_layers
        self.C = block_size * n_kv_heads * head_dim * elt_bytes
        self.R = self.P * self.C
        self.N = n_gpu_blocks

    # -- lifetime
    def kv_pool_destroy(self):
        if self._h:
            _check(lib.kv_pool_destroy(self._h))
            self._h = C.c_void_p()

    close = kv_pool_destroy

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.kv_pool_destroy()

    def __del__(self):
        try:
            self.kv_pool_destroy()
        except Exception:
            pass

    # -- allocator
    def alloc_block_group(self, req: int, n_blocks: int, min_run: int = 1):
        out = np.empty(n_blocks, dtype=np.int32)
        runs = C.c_int32()
        _check(lib.alloc_block_group(self._h, req, n_blocks, min_run,
                                     out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(runs)))
        return out, runs.value

    def free_block_group(self, req: int, blocks):
        a, p = _i32(blocks)
        _check(lib.free_block_group(self._h, req, p, a.size))

    def kv_free_blocks(self):
        f, l = C.c_int64(), C.c_int64()
        _check(lib.kv_free_blocks(self._h, C.byref(f), C.byref(l)))
        return f.value, l.value

    # -- block groups of growing requests
    def kv_bg_configure(self, first_group_blocks: int = 0, seed: int = 20241127):
        _check(lib.kv_bg_configure(self._h, first_group_blocks, seed))

    def kv_bg_append(self, req: int, n_blocks: int, reserve_tail: int = 0) -> np.ndarray:
        out = np.empty(n_blocks, dtype=np.int32)
        _check(lib.kv_bg_append(self._h, req, n_blocks, reserve_tail,
                                out.ctypes.data_as(C.POINTER(C.c_int32))))
        return out

    def kv_bg_table(self, req: int) -> np.ndarray:
        n = C.c_int32()
        _check(lib.kv_bg_table(self._h, req, None, 0, C.byref(n)))
        out = np.empty(n.value, dtype=np.int32)
        _check(lib.kv_bg_table(self._h, req, out.ctypes.data_as(C.POINTER(C.c_int32)), n.value, C.byref(n)))
        return out

    def kv_bg_close(self, req: int):
        _check(lib.kv_bg_close(self._h, req))

    def kv_bg_stats(self) -> dict:
        st = kv_bg_stats_t()
        _check(lib.kv_bg_stats(self._h, C.byref(st)))
        return {n: getattr(st, n) for n, _ in kv_bg_stats_t._fields_}

    # -- swaps
    def swap_out(self, req: int, block_table):
        a, p = _i32(block_table)
        _check(lib.swap_out(self._h, req, p, a.size))

    def swap_out_delta(self, req: int, block_table, dirty_mask) -> int:
        a, p = _i32(block_table)
        m, mp = _u8(dirty_mask)
        if m.size != a.size:
            raise KVError(KV_EINVAL, "dirty mask length differs from table length")
        n = C.c_int32()
        _check(lib.swap_out_delta(self._h, req, p, a.size, mp, C.byref(n)))
        return n.value

    def swap_out_static(self, block_table, host_dst: int, stream: int = 0):
        """host_dst: address of caller-owned (pinned) host memory of len(block_table) * R bytes."""
        a, p = _i32(block_table)
        _check(lib.swap_out_static(self._h, p, a.size, host_dst or None, stream or None))

    def swap_in(self, req: int, new_block_table):
        a, p = _i32(new_block_table)
        _check(lib.swap_in(self._h, req, p, a.size))

    def swap_in_delta(self, req: int, new_block_table, resident_mask) -> int:
        a, p = _i32(new_block_table)
        m, mp = _u8(resident_mask)
        if m.size != a.size:
            raise KVError(KV_EINVAL, "resident mask length differs from table length")
        n = C.c_int32()
        _check(lib.swap_in_delta(self._h, req, p, a.size, mp, C.byref(n)))
        return n.value

    def swap_in_layerwise(self, req: int, new_block_table, layers_per_step: int, resident_mask=None) -> int:
        a, p = _i32(new_block_table)
        mp = None
        if resident_mask is not None:
            m, mp = _u8(resident_mask)
            if m.size != a.size:
                raise KVError(KV_EINVAL, "resident mask length differs from table length")
        n = C.c_int32()
        _check(lib.swap_in_layerwise(self._h, req, p, a.size, mp, layers_per_step, C.byref(n)))
        return n.value

    def kv_stream_wait_layer(self, req: int, layer: int, stream: int):
        _check(lib.kv_stream_wait_layer(self._h, req, layer, stream or None))

    def kv_wait_layer(self, req: int, layer: int):
        _check(lib.kv_wait_layer(self._h, req, layer))

    def swap_out_direct(self, req: int, block_table, per_block: bool = False):
        a, p = _i32(block_table)
        _check(lib.swap_out_direct(self._h, req, p, a.size, int(per_block)))

    def swap_in_direct(self, req: int, new_block_table, per_block: bool = False):
        a, p = _i32(new_block_table)
        _check(lib.swap_in_direct(self._h, req, p, a.size, int(per_block)))

    def _batch(self, fn, reqs, tables):
        r, rp = _i64(reqs)
        nb, nbp = _i32([len(t) for t in tables])
        cat = np.concatenate([np.asarray(t, dtype=np.int32) for t in tables]) if len(tables) else \
            np.zeros(0, np.int32)
        cat, cp = _i32(cat)
        _check(fn(self._h, r.size, rp, cp, nbp))

    def swap_out_batch(self, reqs, tables):
        self._batch(lib.swap_out_batch, reqs, tables)

    def swap_in_batch(self, reqs, tables):
        self._batch(lib.swap_in_batch, reqs, tables)

    # -- completion
    def kv_wait(self, req: int):
        _check(lib.kv_wait(self._h, req))

    def kv_wait_packed(self, req: int):
        _check(lib.kv_wait_packed(self._h, req))

    def kv_query(self, req: int) -> bool:
        d = C.c_int32()
        _check(lib.kv_query(self._h, req, C.byref(d)))
        return bool(d.value)

    def kv_stream_wait(self, req: int, stream: int):
        _check(lib.kv_stream_wait(self._h, req, stream or None))

    def kv_wait_all(self):
        _check(lib.kv_wait_all(self._h))

    # -- reuse map
    def kv_host_len(self, req: int):
        n, e = C.c_int32(), C.c_int32()
        _check(lib.kv_host_len(self._h, req, C.byref(n), C.byref(e)))
        return n.value, e.value

    def kv_host_blocks(self, req: int):
        """(arena base address, int64 record index of every logical block)."""
        n, _ = self.kv_host_len(req)
        idx = np.zeros(n, dtype=np.int64)
        base = C.c_void_p()
        _check(lib.kv_host_blocks(self._h, req, C.byref(base), idx.ctypes.data_as(C.POINTER(C.c_int64)), n))
        return base.value, idx

    def kv_host_read(self, req: int, first_block: int = 0, n_blocks: int | None = None) -> np.ndarray:
        """uint8 [n_blocks][P][C]: a copy of those logical blocks of the host image, made by the
        library (it waits for the request first)."""
        if n_blocks is None:
            n_blocks = self.kv_host_len(req)[0] - first_block
        out = np.empty((max(0, n_blocks), self.P, self.C), dtype=np.uint8)
        _check(lib.kv_host_read(self._h, req, first_block, n_blocks, out.ctypes.data_as(C.c_void_p)))
        return out

    def kv_host_view(self, req: int):
        """The library's zero-copy view of the image as uint8 [n][P][C], or None when the image
        is not one run of consecutive arena records (use kv_host_read then)."""
        ptr, nbytes = C.c_void_p(), C.c_int64()
        _check(lib.kv_host_view(self._h, req, C.byref(ptr), C.byref(nbytes)))
        if nbytes.value == 0:
            return np.zeros((0, self.P, self.C), dtype=np.uint8)
        if not ptr.value:
            return None
        buf = (C.c_uint8 * nbytes.value).from_address(ptr.value)
        return np.frombuffer(buf, dtype=np.uint8).reshape(-1, self.P, self.C)

    def kv_host_valid(self, req: int, n: int) -> np.ndarray:
        out = np.zeros(n, dtype=np.uint8)
        _check(lib.kv_host_valid(self._h, req, out.ctypes.data_as(C.POINTER(C.c_uint8)), n))
        return out

    def kv_host_invalidate(self, req: int, mask):
        m, mp = _u8(mask)
        _check(lib.kv_host_invalidate(self._h, req, mp, m.size))

    def kv_host_release(self, req: int):
        _check(lib.kv_host_release(self._h, req))

    def kv_host_set_priority(self, req: int, priority: int):
        _check(lib.kv_host_set_priority(self._h, req, priority))

    # -- stats / profiling
    def kv_stats(self) -> dict:
        st = kv_stats_t()
        _check(lib.kv_stats(self._h, C.byref(st)))
        return {n: getattr(st, n) for n, _ in kv_stats_t._fields_}

    def kv_profile_read(self):
        n = C.c_int32()
        _check(lib.kv_profile_read(self._h, None, 0, C.byref(n)))
        recs = (kv_prof_record_t * max(1, n.value))()
        _check(lib.kv_profile_read(self._h, recs, n.value, C.byref(n)))
        return [(recs[i].kind, recs[i].bytes, recs[i].ms) for i in range(n.value)]

    def kv_profile_timeline(self):
        """(kind, bytes, start_ms, ms) of every launch and copy, in issue order."""
        n = C.c_int32()
        _check(lib.kv_profile_read(self._h, None, 0, C.byref(n)))
        recs = (kv_prof_record_t * max(1, n.value))()
        _check(lib.kv_profile_read(self._h, recs, n.value, C.byref(n)))
        return [(recs[i].kind, recs[i].bytes, recs[i].start_ms, recs[i].ms) for i in range(n.value)]

    def kv_profile_reset(self):
        _check(lib.kv_profile_reset(self._h))


class KVManager:
    """Owner of one ``kv_manager_t*`` over a KVPool (destroy it before the pool)."""

    def __init__(self, pool: KVPool, window: int = 0, link_gbps: float = 0.0, sync_below_ms: float = 0.0):
        cfg = kv_manager_config_t(window=window, reserved=0, link_gbps=link_gbps, sync_below_ms=sync_below_ms)
        self._m = C.c_void_p()
        self._pool = pool  # keeps the pool alive
        _check(lib.kv_manager_create(pool._h, C.byref(cfg), C.byref(self._m)))

    def kv_manager_destroy(self):
        if self._m:
            _check(lib.kv_manager_destroy(self._m))
            self._m = C.c_void_p()

    close = kv_manager_destroy

    def __del__(self):
        try:
            self.kv_manager_destroy()
        except Exception:
            pass

    def kv_manager_submit(self, kind: int, req: int, table, mask=None) -> int:
        a, p = _i32(table)
        mp = None
        if mask is not None:
            m, mp = _u8(mask)
            if m.size != a.size:
                raise KVError(KV_EINVAL, "mask length differs from table length")
        t = C.c_uint64()
        _check(lib.kv_manager_submit(self._m, kind, req, p, a.size, mp, C.byref(t)))
        return t.value

    def kv_manager_poll(self, cap: int = 64):
        tickets = (C.c_uint64 * cap)()
        status = (C.c_int32 * cap)()
        n = C.c_int32()
        _check(lib.kv_manager_poll(self._m, tickets, status, cap, C.byref(n)))
        return [(tickets[i], status[i]) for i in range(n.value)]

    def kv_manager_wait(self, ticket: int) -> int:
        st = C.c_int32()
        _check(lib.kv_manager_wait(self._m, ticket, C.byref(st)))
        return st.value

    def kv_manager_drain(self):
        _check(lib.kv_manager_drain(self._m))

    def kv_manager_strategy(self, n_swap_in: int, swap_in_blocks: int) -> bool:
        a = C.c_int32()
        _check(lib.kv_manager_strategy(self._m, n_swap_in, swap_in_blocks, C.byref(a)))
        return bool(a.value)

    def kv_manager_iterate(self, swap_in=(), swap_out=(), force_mode: int = 0, cap: int = 256,
                           free_out_blocks: bool = False):
        """swap_in: [(req, new_table)]; swap_out: [(req, table)] or [(req, table, dirty_mask)] (all or
        none with masks).  Returns (resumed request ids, result dict)."""
        def pack(items):
            reqs, rp = _i64([it[0] for it in items])
            nb, nbp = _i32([len(it[1]) for it in items])
            cat = np.concatenate([np.asarray(it[1], dtype=np.int32) for it in items]) if len(items) else \
                np.zeros(0, np.int32)
            cat, cp = _i32(cat)
            return (reqs, nb, cat), rp, cp, nbp
        keep_in, irp, icp, inbp = pack(swap_in)
        keep_out, orp, ocp, onbp = pack(swap_out)
        dirty, dp = None, None
        if len(swap_out) and len(swap_out[0]) > 2:
            dirty, dp = _u8(np.concatenate([np.asarray(it[2], dtype=np.uint8) for it in swap_out]))
            if dirty.size != keep_out[2].size:
                raise KVError(KV_EINVAL, "dirty masks do not match the tables")
        it = kv_iteration_t(n_swap_in=len(swap_in), n_swap_out=len(swap_out), in_reqs=irp, in_tables=icp,
                            in_n_blocks=inbp, out_reqs=orp, out_tables=ocp, out_n_blocks=onbp,
                            out_dirty=dp, force_mode=force_mode, flags=KV_IT_FREE_OUT_BLOCKS if free_out_blocks else 0)
        resumed = np.zeros(max(1, cap), dtype=np.int64)
        n = C.c_int32()
        res = kv_iteration_result_t()
        _check(lib.kv_manager_iterate(self._m, C.byref(it), resumed.ctypes.data_as(C.POINTER(C.c_int64)), cap,
                                      C.byref(n), C.byref(res)))
        return ([int(x) for x in resumed[:min(n.value, cap)]],
                {k: getattr(res, k) for k, _ in kv_iteration_result_t._fields_})

    def kv_manager_failures(self, cap: int = 64):
        reqs = (C.c_int64 * cap)()
        status = (C.c_int32 * cap)()
        n = C.c_int32()
        _check(lib.kv_manager_failures(self._m, reqs, status, cap, C.byref(n)))
        return [(reqs[i], status[i]) for i in range(n.value)]

    def kv_manager_where(self, req: int) -> int:
        w = C.c_int32()
        _check(lib.kv_manager_where(self._m, req, C.byref(w)))
        return w.value

    def kv_manager_iteration_stats(self) -> dict:
        st = kv_iteration_stats_t()
        _check(lib.kv_manager_iteration_stats(self._m, C.byref(st)))
        return {n: getattr(st, n) for n, _ in kv_iteration_stats_t._fields_}

    def kv_manager_stats(self) -> dict:
        st = kv_manager_stats_t()
        _check(lib.kv_manager_stats(self._m, C.byref(st)))
        return {n: getattr(st, n) for n, _ in kv_manager_stats_t._fields_}
