"""The other workload configs of the build (1, 3, 4, 5), run as `python bench.py --config N`.

They are parity-test cases first (tests/test_gpu_full_size.py); here they are timed, for the
results table.  Each function returns a dict that bench.py prints as one JSON line.  Pools
are left uninitialised where content does not matter to a copy path.
"""

from __future__ import annotations

import time

import numpy as np

GiB = 1 << 30
MiB = 1 << 20


def _pct(xs, q):
    return round(float(np.percentile(np.asarray(xs, dtype=np.float64), q)), 3) if len(xs) else None


def _rates(recs):
    out = {}
    for kind, name, mult in ((0, "gather", 2), (1, "scatter", 2), (2, "d2h", 1), (3, "h2d", 1), (4, "mapped_in", 1)):
        rs = [r for r in recs if r[0] == kind]
        ms = sum(r[2] for r in rs)
        out[name + "_gbps"] = round(mult * sum(r[1] for r in rs) / ms / 1e6, 1) if ms > 0 else None
        out[name + "_n"] = len(rs)
    return out


def _flags(args, kv, base=0):
    return (base | (kv.KV_FLAG_FOUR_STREAMS if args.four_streams else 0)
            | (kv.KV_FLAG_SCATTER_STREAM if getattr(args, "scatter_stream", False) else 0)
            | (kv.KV_FLAG_MAPPED_SWAP_IN if args.mapped_swap_in else 0)
            | (kv.KV_FLAG_MAPPED_SWAP_OUT if getattr(args, "mapped_swap_out", False) else 0)
            | (kv.KV_FLAG_NO_STRIDED_COPIES if getattr(args, "no_strided_copies", False) else 0)
            | (kv.KV_FLAG_NO_DEFER_COPIES if getattr(args, "no_defer_copies", False) else 0)
            | (kv.KV_FLAG_SECOND_LANE if getattr(args, "second_lane", False) else 0)
            | (kv.KV_FLAG_NO_LAUNCH_EVENTS if getattr(args, "no_launch_events", False) else 0))


def _variant_note():
    """What the environment changed in the timed kernels (development aids), for the JSON line."""
    import os
    return {"KVSWAP_PACK_VARIANT": int(os.environ.get("KVSWAP_PACK_VARIANT", "0")),
            "KVSWAP_MAPPED_GRID": int(os.environ.get("KVSWAP_MAPPED_GRID", "0"))}


def settle(torch, max_s=60.0, quiet_s=3.0):
    """Waits until small swap-outs run at their normal rate, steadily.  When a process that held
    much device memory has just ended (the previous benchmark or test on this machine), the kernel
    driver is still busy with that memory, and for several seconds the device-to-host copies of a
    few MiB behind a gather take several times as long (measured: 98 of 120 delta swap-outs slow
    right after a process with 214 GiB exited, 1 of 120 after 20 s of sleep; large copies lose a
    few per cent).  That is the machine's state, not the workload's: timing starts when every
    probe of the last quiet_s seconds was back to normal.  The probe is the library's own path on a
    small pool of its own: a delta swap-out of 11 scattered 2 MiB block records (gather, then one
    copy per record or pair), and the same records swapped back in.  Returns what it saw."""
    from paper_2411_18424_amd import kvswap as kv, synth
    s = synth.LLAMA3_8B.with_blocks(64)
    gpu = torch.zeros(s.R * s.n_blocks, dtype=torch.uint8, device="cuda:0")
    pool = kv.KVPool(n_layers=s.n_layers, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim, block_size=s.block_size,
                     elt_bytes=s.elt_bytes, n_gpu_blocks=s.n_blocks, gpu_base=gpu.data_ptr(), host_bytes=128 * s.R,
                     staging_out_bytes=64 * s.R, staging_in_bytes=32 * s.R)
    t = np.arange(64, dtype=np.int32)
    pool.swap_out(0, t)
    pool.kv_wait(0)
    dirty = np.zeros(64, np.uint8)
    dirty[[0, 1, 3, 6, 10, 15, 21, 28, 36, 45, 55]] = 1  # gaps 1, 2, 3, ...: no arithmetic progression beyond pairs
    resident = (1 - dirty).astype(np.uint8)
    rates, rates_in, t0 = [], [], time.perf_counter()
    quiet_since = None
    while True:
        a = time.perf_counter()
        moved = pool.swap_out_delta(0, t, dirty)
        pool.kv_wait(0)
        now = time.perf_counter()
        rates.append(round(moved * s.R / (now - a) / 1e9, 1))
        pool.swap_in_delta(0, t, resident)  # the same records back: small host-to-device copies, then a scatter
        pool.kv_wait(0)
        back = time.perf_counter()
        rates_in.append(round(moved * s.R / (back - now) / 1e9, 1))
        now = back
        if rates[-1] < 28.0 or rates_in[-1] < 28.0:
            quiet_since = None
        elif quiet_since is None:
            quiet_since = a
        if (quiet_since is not None and now - quiet_since >= quiet_s) or now - t0 > max_s:
            break
        time.sleep(0.02)
    pool.kv_pool_destroy()
    del gpu
    return {"what": "delta swap-outs of 11 scattered 2 MiB records on a small pool (and the same records swapped back in), "
                    "GB/s call to done, repeated until every probe of the last %g s reached 28 (normal: about 40)" % quiet_s,
            "waited_s": round(time.perf_counter() - t0, 2), "first": rates[0], "min": min(rates), "last": rates[-1],
            "slow_probes": sum(1 for r in rates if r < 28.0), "probes": len(rates),
            "back_in": {"first": rates_in[0], "min": min(rates_in), "last": rates_in[-1],
                        "slow_probes": sum(1 for r in rates_in if r < 28.0)}}


def _pool(kv, torch, s, host_bytes, **kw):
    import os
    if "KVSWAP_PACK_VARIANT" in os.environ:  # development aid: force a kernel variant (echoed in the JSON line)
        kw["pack_variant"] = int(os.environ["KVSWAP_PACK_VARIANT"])
    if "KVSWAP_MAPPED_GRID" in os.environ:  # development aid: workgroups of the mapped kernels (echoed)
        kw["mapped_in_grid"] = int(os.environ["KVSWAP_MAPPED_GRID"])
    gpu = torch.empty(s.R * s.n_blocks, dtype=torch.uint8, device="cuda:0")
    pool = kv.KVPool(n_layers=s.n_layers, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim,
                     block_size=s.block_size, elt_bytes=s.elt_bytes, n_gpu_blocks=s.n_blocks,
                     gpu_base=gpu.data_ptr(), host_bytes=host_bytes, **kw)
    return gpu, pool


def config1(args):
    """Tiny pool: 8 requests of 1..16 blocks (32..512 KiB): small-message latency."""
    import torch
    from paper_2411_18424_amd import kvswap as kv, synth
    s = synth.TINY
    rng = synth.rng_for(1)
    nblk = synth.blocks_for(synth.lengths_uniform(rng, 8, 16, 256), s.block_size)
    tables = synth.deal_tables(rng, s.n_blocks, nblk)
    tables2 = synth.deal_tables(rng, s.n_blocks, nblk)
    gpu, pool = _pool(kv, torch, s, 64 * MiB, flags=_flags(args, kv))
    gpu.random_(0, 256)
    torch.cuda.synchronize()
    settled = settle(torch)
    out_us, in_us, all_ms = [], [], []
    for rep in range(args.warmup + args.steps * 5):
        t0 = time.perf_counter()
        for r, t in enumerate(tables):
            a = time.perf_counter()
            pool.swap_out(r, t)
            pool.kv_wait(r)
            if rep >= args.warmup:
                out_us.append((time.perf_counter() - a) * 1e6)
        for r, t in enumerate(tables2):
            a = time.perf_counter()
            pool.swap_in(r, t)
            pool.kv_wait(r)
            if rep >= args.warmup:
                in_us.append((time.perf_counter() - a) * 1e6)
        if rep >= args.warmup:
            all_ms.append((time.perf_counter() - t0) * 1e3)
        tables, tables2 = tables2, tables
    payload = int(nblk.sum()) * s.R
    # all eight in two batched calls
    b_ms = []
    reqs = list(range(8))
    for rep in range(args.warmup + args.steps * 5):
        t0 = time.perf_counter()
        pool.swap_out_batch(reqs, tables)
        pool.kv_wait_all()
        pool.swap_in_batch(reqs, tables2)
        pool.kv_wait_all()
        if rep >= args.warmup:
            b_ms.append((time.perf_counter() - t0) * 1e3)
        tables, tables2 = tables2, tables
    pool.kv_pool_destroy()
    return {"metric": "KV swap GB/s (out+in) and per-preemption switch latency, 1 MI355X", "unit": "GB/s",
            "value": round(2 * payload / (np.median(all_ms) * 1e-3) / 1e9, 3),
            "config": {"workload": "config 1: tiny pool (2 layers, 4 KV heads, head_dim 64, fp16, 256 blocks), "
                                   "8 requests of 1..16 blocks, one call per request, each waited for"},
            "payload_bytes_each_way": payload,
            "per_request_out_us": {"median": _pct(out_us, 50), "p99": _pct(out_us, 99)},
            "per_request_in_us": {"median": _pct(in_us, 50), "p99": _pct(in_us, 99)},
            "batched_all8_out_in_ms": {"median": _pct(b_ms, 50), "p99": _pct(b_ms, 99)},
            "batched_gbps": round(2 * payload / (np.median(b_ms) * 1e-3) / 1e9, 3),
            "mapped_swap_in": bool(args.mapped_swap_in), "mapped_swap_out": bool(args.mapped_swap_out),
            "settle": settled}


def _copy_fairness(kv, torch, s, gpu):
    """Section 3.2, order of dispatches: how long a small copy of the inference stream (a 4 KiB
    result going to the host, a 4 KiB input coming in) takes while a 3 GiB swap uses the link in
    the same direction, with the swap's copies cut at copy_chunk_bytes or issued whole."""
    comp = torch.cuda.Stream()
    dev = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    host = torch.zeros(4096, dtype=torch.uint8).pin_memory()

    def one(to_host):
        t0 = time.perf_counter()
        with torch.cuda.stream(comp):
            (host if to_host else dev).copy_(dev if to_host else host, non_blocking=True)
        comp.synchronize()
        return (time.perf_counter() - t0) * 1e6

    def stats(xs):
        return {"n": len(xs), "median": _pct(xs, 50), "p99": _pct(xs, 99), "max": _pct(xs, 100)}

    for _ in range(50):
        one(True), one(False)
    out = {"what": "4 KiB pinned copy on another stream, call -> synchronised, host clock; alone and while a "
                   "256-block (3.1 GiB) swap moves in the same direction",
           "alone_d2h": stats([one(True) for _ in range(300)]),
           "alone_h2d": stats([one(False) for _ in range(300)])}
    ids = np.arange(256, dtype=np.int32)
    for name, chunk in (("chunks_of_8_MiB", 8 * MiB), ("chunks_of_64_MiB", 64 * MiB), ("chunks_of_256_MiB_default", 0), ("whole_copies", 1 << 40)):
        pool = kv.KVPool(n_layers=s.n_layers, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim,
                         block_size=s.block_size, elt_bytes=s.elt_bytes, n_gpu_blocks=s.n_blocks,
                         gpu_base=gpu.data_ptr(), host_bytes=(256 + 40) * s.R, copy_chunk_bytes=chunk)
        pool.swap_out(0, ids)
        pool.kv_wait(0)
        d2h, h2d = [], []
        for _ in range(4):
            pool.swap_out(0, ids)
            while not pool.kv_query(0):
                d2h.append(one(True))
            pool.swap_in(0, ids)
            while not pool.kv_query(0):
                h2d.append(one(False))
        pool.kv_pool_destroy()
        out[name] = {"d2h_beside_swap_out": stats(d2h), "h2d_beside_swap_in": stats(h2d)}
    return out


def config3(args):
    """Llama-2-13B MHA shape, pool at 80 % of 288 GB, a stream of preemptions: request i leaves
    while request i-2 resumes, both on side streams, with a compute kernel running beside.
    Run twice: the scheduler calls swap_in / swap_out itself, and the same stream through
    kv_manager_iterate (Algorithm 1: dispatcher thread, step-1 polling, strategy)."""
    import torch
    from paper_2411_18424_amd import kvswap as kv, synth
    s = synth.LLAMA2_13B
    n_pre, lag = args.preemptions, 2
    rng = synth.rng_for(3)
    nblk = synth.blocks_for(rng.integers(512, 4097, size=n_pre), s.block_size)
    host_bytes = int((lag + 2) * (256 + 40)) * s.R
    # 1 GiB each way at once, nothing else running - and not while the driver still clears the device memory of a
    # process that has just ended (the probe then reads 60 GB/s, less than the swaps below reach): wait first
    two_way_peak = getattr(args, "two_way_peak", 0)
    if not two_way_peak:
        settle(torch)
        two_way_peak = kv.kv_link_probe(GiB, 2, 5)
    profiled = not getattr(args, "no_profile", False)  # timing events on every launch and copy, for the rates below
    gpu, pool = _pool(kv, torch, s, host_bytes, copy_chunk_bytes=args.copy_chunk_mib << 20,
                      flags=_flags(args, kv, kv.KV_FLAG_PROFILE if profiled else 0))
    a = torch.randn(8192, 8192, device="cuda:0", dtype=torch.bfloat16)
    comp = torch.cuda.Stream()
    settled = settle(torch)

    def compute(n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(comp):
            e0.record()
            x = a
            for _ in range(n):
                x = torch.mm(x, a) * 1e-2
            e1.record()
        return e0, e1

    e0, e1 = compute(20)
    comp.synchronize()
    e0, e1 = compute(200)
    comp.synchronize()
    alone_ms = e0.elapsed_time(e1) / 200
    # about as much compute per iteration as the median swap takes on the link
    per_iter = max(1, int(float(np.median(nblk)) * s.R / 57e9 * 1e3 / alone_ms))

    def stream(mgr):
        """The 200-preemption stream; tables from the library's block-group allocator (groups of >= 8
        where the pool allows).  mgr None: direct calls; else through kv_manager_iterate."""
        lat, evs, in_tables, moved = [], [], {}, 0
        if profiled:
            pool.kv_profile_reset()
        t_start = time.perf_counter()
        for i in range(n_pre + lag):
            evs.append(compute(per_iter))  # keeps the compute stream busy for about one iteration
            t0 = time.perf_counter()
            j = i - lag
            ids = ids2 = None
            if j >= 0:
                ids2, _ = pool.alloc_block_group(10**6 + j, int(nblk[j]), 8)
                in_tables[j] = ids2
                moved += int(nblk[j]) * s.R
            if i < n_pre:
                ids, _ = pool.alloc_block_group(i, int(nblk[i]), 8)
                moved += int(nblk[i]) * s.R
            if mgr is None:
                # by default the swap-in the scheduler will wait for goes first (Algorithm 1's order);
                # --out-first issues the swap-out of the iteration before it
                if i < n_pre and out_first:
                    pool.swap_out(i, ids)
                    pool.free_block_group(i, ids)  # parked until the gather has read them
                if j >= 0:
                    pool.swap_in(j, ids2)      # ordered after request j's own swap-out by the library
                if i < n_pre and not out_first:
                    pool.swap_out(i, ids)
                    pool.free_block_group(i, ids)
                if j >= 0:
                    # the scheduler only has to wait for the request it resumes (Algorithm 1, step 1);
                    # the swap-out of request i drains in the background
                    pool.kv_wait(j)
            else:
                resumed, _ = mgr.kv_manager_iterate(swap_in=[(j, ids2)] if j >= 0 else [],
                                                    swap_out=[(i, ids)] if i < n_pre else [],
                                                    free_out_blocks=True)
                while j >= 0 and j not in resumed:   # the scheduler has nothing else to run: step 1 until j is back
                    resumed, _ = mgr.kv_manager_iterate()
            if j >= 0:
                lat.append((time.perf_counter() - t0) * 1e3)
                pool.kv_host_release(j)  # the resumed request runs again; copy and blocks are recycled
                pool.free_block_group(10**6 + j, in_tables.pop(j))
        if mgr is not None:
            mgr.kv_manager_drain()
        pool.kv_wait_all()
        total_s = time.perf_counter() - t_start
        comp.synchronize()
        busy_ms = sum(x.elapsed_time(y) for x, y in evs) / (per_iter * len(evs))
        return {"gbps": round(moved / total_s / 1e9, 3),
                "switch_latency_ms": {"median": _pct(lat, 50), "p99": _pct(lat, 99), "max": _pct(lat, 100)},
                "kernels_and_copies": _rates(pool.kv_profile_read()) if profiled else None,
                "compute_slowdown": round(busy_ms / alone_ms, 4), "compute_ms_beside_swaps": round(busy_ms, 4)}

    out_first = bool(getattr(args, "out_first", False))
    direct = stream(None)
    st = pool.kv_stats()
    via = {}
    if not getattr(args, "no_manager_pass", False):
        mgr = kv.KVManager(pool)
        via = stream(mgr)
        via["iteration_stats"] = mgr.kv_manager_iteration_stats()
        ms = mgr.kv_manager_stats()
        via["strategy_async_fraction"] = round(ms["strategy_async"] / max(1, ms["strategy_calls"]), 3)
        via["dispatcher_us_per_task"] = round(ms["dispatch_us_sum"] / max(1, ms["dispatched"]), 1)
        via["queue_wait_us_per_task"] = round(ms["queue_wait_us_sum"] / max(1, ms["dispatched"]), 1)
        mgr.kv_manager_destroy()
    pool.kv_pool_destroy()
    fairness = _copy_fairness(kv, torch, s, gpu) if not getattr(args, "no_fairness", False) else None
    return {"metric": "KV swap GB/s (out+in) and per-preemption switch latency, 1 MI355X", "unit": "GB/s",
            "value": direct["gbps"],
            "link": {"measured_peak_two_way_gbps": round(two_way_peak, 2),
                     "frac_of_measured": round(direct["gbps"] / two_way_peak, 4)},
            "config": {"workload": "config 3: Llama-2-13B-shaped MHA KV (40 layers, 40 KV heads, head_dim 128, fp16), "
                                   "pool %d blocks = %.1f GB, %d preemptions of 512..4096 tokens, one out while one in, "
                                   "compute running on a third stream" % (s.n_blocks, s.n_blocks * s.R / 1e9, n_pre)},
            "switch_latency_ms": {"what": "swap_in(i-2) and swap_out(i) issued together -> the resumed request i-2 is back",
                                  **direct["switch_latency_ms"]},
            "request_MiB": {"median": round(float(np.median(nblk)) * s.R / MiB, 1),
                            "max": round(float(nblk.max()) * s.R / MiB, 1)},
            "kernels_and_copies": direct["kernels_and_copies"], "pool_has_timing_events": profiled,
            "compute_matmul_ms": {"what": "8192^3 bf16 matmul on the compute stream, %d per iteration" % per_iter,
                                  "alone": round(alone_ms, 4), "beside_swaps": direct["compute_ms_beside_swaps"],
                                  "slowdown": direct["compute_slowdown"]},
            "via_manager": {"what": "the same stream through kv_manager_iterate (Algorithm 1): swaps dispatched by the "
                                    "manager's thread, victims' blocks freed by the dispatcher, the resumed request "
                                    "picked up by step-1 polling or by the synchronous branch of step 4", **via},
            "streams": 4 if args.four_streams else 3 if args.scatter_stream else 2, "mapped_swap_in": bool(args.mapped_swap_in),
            "call_order": "swap-out first" if out_first else "swap-in first", "pack_variant": _variant_note(),
            "swap_out_copies": "enqueued inside the call" if getattr(args, "no_defer_copies", False)
                               else "held back until their gathers are done (copy thread)",
            "conflict_waits": st["conflict_waits"], "host_arena_bytes": st["host_arena_bytes"],
            "settle": settled, "small_copy_latency_us": fairness}


def config4(args):
    """Multi-turn delta swap on the Llama-3-8B shape: conversations with a host copy return,
    append 64..512 tokens and leave; only dirty blocks move out.  The stated 128 conversations
    need about 110 GiB of pinned memory at once, more than a process gets on these machines
    (64 GiB was granted, 72 GiB refused, a second 48 GiB beside a first refused too): they go
    through an arena of --arena-gib in waves."""
    import torch
    from paper_2411_18424_amd import kvswap as kv, synth
    s = synth.LLAMA3_8B
    rng = synth.rng_for(4)
    n_conv = args.conversations
    B = s.block_size
    ctx = synth.lengths_loguniform(rng, n_conv, 1024, 16384)
    nb0 = synth.blocks_for(ctx, B)
    arena_blocks = (args.arena_gib << 30) // s.R
    waves, cur, used = [], [], 0
    for c in range(n_conv):  # greedy waves that fit the arena (context + room for two turns)
        need = int(nb0[c]) + 180
        if cur and used + need > arena_blocks:
            waves.append(cur)
            cur, used = [], 0
        cur.append(c)
        used += need
    waves.append(cur)
    host_bytes = arena_blocks * s.R
    gpu, pool = _pool(kv, torch, s, host_bytes, flags=_flags(args, kv, kv.KV_FLAG_PROFILE))
    gpu.random_(0, 256)
    torch.cuda.synchronize()
    settled = settle(torch)
    work = rng.permutation(s.n_blocks)[:1200].astype(np.int32)
    full_ms, delta_ms, in_ms, fracs, delta_bytes, full_bytes = [], [], [], [], 0, 0
    delta_op_gbps, full_recs, probes = [], [], []
    new_ms, new_fracs, new_bytes = [], [], 0  # third turn: the new turn's blocks only, no scattered ones

    def probe():  # is the link itself disturbed right now?  (a 256 MiB device-to-host copy, best of 3)
        probes.append(round(kv.kv_link_probe(256 * MiB, 0, 3), 2))

    for wave in waves:
        probe()
        tok = {}
        for c in wave:
            pool.swap_out(c, rng.permutation(work)[:int(nb0[c])])
            tok[c] = int(ctx[c])
        pool.kv_wait_all()
        for turn in range(3):
            for c in wave:
                n_old = int(synth.blocks_for(tok[c], B))
                t = rng.permutation(work)[:n_old]
                a0 = time.perf_counter()
                pool.swap_in(c, t)
                pool.kv_wait(c)
                in_ms.append((time.perf_counter() - a0) * 1e3)
                new_tokens = int(rng.integers(64, 513))
                dirty = synth.turn_dirty_mask(n_old, tok[c], new_tokens, B)
                if turn < 2:  # top the mask up with scattered blocks of the old context (contaminated copies)
                    target = rng.uniform(0.05, 0.30)
                    dirty[:n_old] |= synth.random_mask(rng, n_old, max(0.0, target - dirty.mean()))
                grown = np.concatenate([t, np.setdiff1d(work, t)[:len(dirty) - n_old]]).astype(np.int32)
                a0 = time.perf_counter()
                moved = pool.swap_out_delta(c, grown, dirty)
                pool.kv_wait(c)
                ms = (time.perf_counter() - a0) * 1e3
                assert moved == int(dirty.sum()), (moved, int(dirty.sum()))
                if turn == 2:
                    new_ms.append(ms)
                    new_bytes += moved * s.R
                    new_fracs.append(moved / len(dirty))
                    tok[c] += new_tokens
                    continue
                delta_ms.append(ms)
                delta_bytes += moved * s.R
                delta_op_gbps.append(moved * s.R / ms / 1e6)
                fracs.append(moved / len(dirty))
                tok[c] += new_tokens
                if turn == 1:  # the same conversation swapped out in full, for comparison
                    n_rec = len(pool.kv_profile_read())
                    a0 = time.perf_counter()
                    pool.swap_out(c, grown)
                    pool.kv_wait(c)
                    full_ms.append((time.perf_counter() - a0) * 1e3)
                    full_bytes += len(grown) * s.R
                    full_recs += pool.kv_profile_read()[n_rec:]
            probe()
        for c in wave:
            pool.kv_host_release(c)
    st = pool.kv_stats()
    pool_recs = pool.kv_profile_read()
    pool.kv_pool_destroy()
    return {"metric": "KV swap GB/s (out+in) and per-preemption switch latency, 1 MI355X", "unit": "GB/s",
            "value": round(delta_bytes / (sum(delta_ms) * 1e-3) / 1e9, 3),
            "value_is": "payload rate of the delta swap-outs alone (all of them: bytes / summed call-to-done times)",
            "config": {"workload": "config 4: Llama-3-8B shape, %d conversations with 1k..16k tokens on the host, in %d wave(s) "
                                   "through a %.0f GiB pinned arena, 2 turns of +64..512 tokens with the mask topped up by "
                                   "scattered blocks to a dirty fraction of 5..30 %% (the value), then a turn of new blocks only"
                                   % (n_conv, len(waves), host_bytes / GiB)},
            "dirty_fraction": {"min": round(min(fracs), 3), "median": _pct(fracs, 50), "max": round(max(fracs), 3)},
            "delta_swap_out_ms": {"median": _pct(delta_ms, 50), "p99": _pct(delta_ms, 99)},
            "delta_swap_out_gbps_per_op": {"what": "payload rate of each delta swap-out, call to done; the spread shows "
                                                   "how steady the small device-to-host copies were in this run",
                                           "p10": _pct(delta_op_gbps, 10), "median": _pct(delta_op_gbps, 50),
                                           "p90": _pct(delta_op_gbps, 90)},
            "link_probe_d2h_gbps": {"what": "256 MiB pinned copies between the phases of the run: is the link itself steady",
                                    "min": min(probes), "median": _pct(probes, 50), "max": max(probes)},
            "new_blocks_only": {"what": "a third turn per conversation whose mask holds the turn's own blocks only (the tail "
                                        "block it wrote into and the appended ones: adjacent records on the host), "
                                        "no scattered blocks of the old context",
                                "gbps": round(new_bytes / (sum(new_ms) * 1e-3) / 1e9, 3),
                                "ms": {"median": _pct(new_ms, 50), "p99": _pct(new_ms, 99)},
                                "dirty_fraction": {"min": round(min(new_fracs), 3), "median": _pct(new_fracs, 50),
                                                   "max": round(max(new_fracs), 3)},
                                "mean_MiB": round(new_bytes / len(new_ms) / MiB, 1)},
            "full_swap_out_ms": {"median": _pct(full_ms, 50), "p99": _pct(full_ms, 99)},
            "full_swap_out_gbps": round(full_bytes / (sum(full_ms) * 1e-3) / 1e9, 3),
            "swap_in_ms": {"median": _pct(in_ms, 50), "p99": _pct(in_ms, 99)},
            "full_swap_out_kernels_and_copies": _rates(full_recs),
            "all_kernels_and_copies": _rates(pool_recs),
            "bytes_moved_equals_dirty_blocks": True, "mapped_swap_in": bool(args.mapped_swap_in),
            "strided_copies": not getattr(args, "no_strided_copies", False), "pack_variant": _variant_note(),
            "second_lane": bool(getattr(args, "second_lane", False)), "second_lane_copies": st["second_lane_copies"],
            "host_new_extents": st["host_new_extents"], "d2h_copies": st["d2h_copies"],
            "d2h_copies_strided": st["strided_copies"], "settle": settled}


def config5(args):
    """Qwen2-72B shape (80 layers), 32k-token requests (2048 blocks, 10 GiB): fully fragmented
    tables vs block groups of 16; packed path vs the paper-style direct per-group copies."""
    import torch
    from paper_2411_18424_amd import kvswap as kv, synth
    s = synth.QWEN2_72B
    n_req = args.requests
    out = {"metric": "KV swap GB/s (out+in) and per-preemption switch latency, 1 MI355X", "unit": "GB/s",
           "config": {"workload": "config 5: Qwen2-72B-shaped GQA KV (80 layers, 8 KV heads, head_dim 128, bf16), pool %d blocks "
                                  "= %.1f GB, %d requests of 2048 blocks (10 GiB) per run length, one at a time"
                                  % (s.n_blocks, s.n_blocks * s.R / 1e9, n_req)}}
    gpu, pool = _pool(kv, torch, s, (2048 + 40) * s.R, flags=_flags(args, kv, kv.KV_FLAG_PROFILE))
    out["settle"] = settle(torch)
    payload = 2048 * s.R
    for run in (1, 16):
        rng = synth.rng_for(5, stream=run)
        tables = synth.deal_tables(rng, s.n_blocks, [2048] * (2 * n_req), run=run)
        pool.kv_profile_reset()
        ms = []
        for r in range(n_req):
            t0 = time.perf_counter()
            pool.swap_out(r, tables[2 * r])
            pool.kv_wait(r)
            t1 = time.perf_counter()
            pool.swap_in(r, tables[2 * r + 1])
            pool.kv_wait(r)
            t2 = time.perf_counter()
            pool.kv_host_release(r)
            if r > 0 or n_req == 1:
                ms.append(((t1 - t0) * 1e3, (t2 - t1) * 1e3))
        rates = _rates(pool.kv_profile_read())
        o = np.array(ms)
        res = {"out_gbps": round(payload / (np.median(o[:, 0]) * 1e-3) / 1e9, 2),
               "in_gbps": round(payload / (np.median(o[:, 1]) * 1e-3) / 1e9, 2),
               "out_ms": _pct(o[:, 0], 50), "in_ms": _pct(o[:, 1], 50), **rates}
        if getattr(args, "no_direct_path", False):  # e.g. under a profiler, where its 327 680 copies take minutes
            out["run_%d" % run] = res
            continue
        # the paper-style direct path on the same tables (one request is enough to see it)
        t0 = time.perf_counter()
        pool.swap_out_direct(99, tables[0], False)
        pool.kv_wait(99)
        t1 = time.perf_counter()
        pool.swap_in_direct(99, tables[1], False)
        pool.kv_wait(99)
        t2 = time.perf_counter()
        pool.kv_host_release(99)
        n_copies = s.P * (2048 // run)
        res["direct_per_group"] = {"copies_each_way": n_copies, "copy_KiB": run * s.C // 1024,
                                   "out_gbps": round(payload / (t1 - t0) / 1e9, 2),
                                   "in_gbps": round(payload / (t2 - t1) / 1e9, 2)}
        out["run_%d" % run] = res
    # the paper's argument in one table: rate of per-group copies against the length of the
    # groups (20 blocks is the average granularity the paper reports for its block groups);
    # the packed path is flat across all of them
    sweep = {}
    for run in (() if getattr(args, "no_group_sweep", False) or getattr(args, "no_direct_path", False)
                else (4, 20, 64, 256, 2048)):
        rng = synth.rng_for(5, stream=1000 + run)
        ta, tb = synth.deal_tables(rng, s.n_blocks, [2048, 2048], run=run)
        t0 = time.perf_counter()
        pool.swap_out_direct(98, ta, False)
        pool.kv_wait(98)
        t1 = time.perf_counter()
        pool.swap_in_direct(98, tb, False)
        pool.kv_wait(98)
        t2 = time.perf_counter()
        pool.kv_host_release(98)
        t3 = time.perf_counter()
        pool.swap_out(97, ta)
        pool.kv_wait(97)
        t4 = time.perf_counter()
        pool.kv_host_release(97)
        sweep["run_%d" % run] = {"copy_KiB": run * s.C // 1024,
                                 "direct_out_gbps": round(payload / (t1 - t0) / 1e9, 2),
                                 "direct_in_gbps": round(payload / (t2 - t1) / 1e9, 2),
                                 "packed_out_gbps": round(payload / (t4 - t3) / 1e9, 2)}
    if sweep:
        out["direct_by_group_length"] = sweep
    pool.kv_pool_destroy()
    out["value"] = round(2 * payload / ((out["run_16"]["out_ms"] + out["run_16"]["in_ms"]) * 1e-3) / 1e9, 3)
    return out


def other_configs(args):
    """Configs 1, 3, 4 and 5 in short form, for the default benchmark run: the stated counts (200
    preemptions, 128 conversations), fewer repetitions and none of the side measurements.  Each
    runs in pools of its own, after waiting for the copy engines to be quiet."""
    import copy
    import torch
    a = copy.copy(args)
    a.warmup, a.steps = 2, 4
    a.preemptions, a.no_fairness, a.out_first, a.no_manager_pass = 200, True, False, False
    a.conversations, a.arena_gib = 128, 56
    a.requests, a.no_group_sweep = 2, True
    a.mapped_swap_in = a.mapped_swap_out = a.four_streams = a.scatter_stream = a.no_strided_copies = False
    a.copy_chunk_mib = 0
    a.second_lane = False
    a.no_profile = True  # config 3 in a pool as an application creates it: no timing events beyond the launches' own
    lane = copy.copy(a)
    lane.second_lane = True  # config 4 once more with KV_FLAG_SECOND_LANE
    out = {}
    for name, fn, arg in (("config_1", config1, a), ("config_4", config4, a), ("config_4_second_lane", config4, lane),
                          ("config_5", config5, a), ("config_3", config3, a)):
        t0 = time.perf_counter()
        try:
            r = fn(arg)
            r.pop("metric", None)
        except Exception as e:  # e.g. not enough free device or pinned memory for this config's pool: say so, go on
            r = {"error": "%s: %s" % (type(e).__name__, str(e)[:300])}
        r["seconds"] = round(time.perf_counter() - t0, 1)
        out[name] = r
        torch.cuda.empty_cache()
    return out
