#!/usr/bin/env python3
"""KV-swap benchmark on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: the 16
victims of the Llama-3-8B-shaped workload (config 2) are swapped out of a 16 GiB paged
KV pool to pinned host memory (gather kernels + device-to-host copies) and swapped back
in through fresh block tables (host-to-device copies + scatter kernels).  The pool is
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
GiB = 1 << 30


def dist3(v):
    v = sorted(v)
    return {"min": round(v[0], 3), "median": round(v[len(v) // 2], 3), "max": round(v[-1], 3)}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def percentile(xs, q):
    import numpy as np
    if len(xs) == 0:
        return None
    return round(float(np.percentile(np.asarray(xs, dtype=np.float64), q)), 3)


def device_state():
    """Clocks and power state of the GPU as the kernel driver reports them (best effort)."""
    import glob
    out = {}
    try:
        import torch
        out["name"] = torch.cuda.get_device_name(0)
    except Exception:
        pass
    for dev in sorted(glob.glob("/sys/class/drm/card*/device")):
        try:
            if open(os.path.join(dev, "vendor")).read().strip() != "0x1002":
                continue
        except OSError:
            continue
        for key, fname in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk"), ("fclk", "pp_dpm_fclk"),
                           ("performance_level", "power_dpm_force_performance_level")):
            try:
                text = open(os.path.join(dev, fname)).read().strip()
            except OSError:
                continue
            lines = text.splitlines()
            cur = [l for l in lines if l.rstrip().endswith("*")]
            out[key] = (cur[0].split(":", 1)[-1].strip(" *") if cur else lines[0]) if lines else ""
            if key != "performance_level" and lines:
                out[key + "_max"] = lines[-1].split(":", 1)[-1].strip(" *")
        break
    return out


def _oracle_for(work, victims):
    """A CPU oracle that holds the seeded content of these victims' blocks (the rest of its pool
    stays untouched zero pages)."""
    import numpy as np
    from oracle.kv_oracle import KVOracle
    from paper_2411_18424_amd import synth

    s = work.shape
    o = KVOracle(s.n_layers, s.n_kv_heads, s.head_dim, s.block_size, s.elt_bytes, s.n_blocks)
    content = synth.PoolContent(s, work.cfg)
    for v in victims:
        blocks = work.tables[v].astype(np.int64)
        for p in range(s.P):
            o.G[p, blocks, :] = content.plane(p, blocks)
    return o


def _oracle_steps(work, o, victims, budget_s, max_steps, start=None):
    """Swap the victims out, then in through the resume tables, repeatedly: (bytes, seconds, steps)."""
    resume = {v: t for v, t in zip(work.victims, work.resume_tables)}
    cur = {v: work.tables[v] for v in victims}
    nxt = {v: resume[v] for v in victims}
    s = work.shape
    if start is not None:
        start.wait()
    steps, moved = 0, 0
    t0 = time.perf_counter()
    while True:
        for v in victims:
            moved += len(o.swap_out(v, cur[v])) * s.R
        for v in victims:
            moved += len(o.swap_in(v, nxt[v])) * s.R
        cur, nxt = nxt, cur
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or steps >= max_steps:
            return moved, dt, steps


def _oracle_worker(args):
    work, victims, budget_s, start, q = args
    o = _oracle_for(work, victims)
    q.put((victims, _oracle_steps(work, o, victims, budget_s, 10**6, start)))


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(work, budget_s=12.0, all_cores_budget_s=8.0):
    """The CPU oracle, as it stands, on the same victims: swap all out, then in through the
    resume tables, repeated until about budget_s seconds of work.  (i) one thread; (ii) all the
    cores of this machine's share, one process per core, the victims dealt to them (one request
    per process where there are as many cores as victims), started together; the aggregate is
    total bytes over the time of the slowest.  Runs before this process has touched the GPU."""
    import multiprocessing as mp

    s = work.shape
    o = _oracle_for(work, work.victims)
    moved, dt, steps = _oracle_steps(work, o, work.victims, budget_s, 50)
    del o
    nb = sum(len(work.tables[v]) for v in work.victims)
    out = {"value": moved / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle", "cpu": cpu_model(),
           "sample": "same 16 victims (%d blocks, %.2f GiB each way), %d full out+in steps, %.1f s"
                     % (nb, nb * s.R / GiB, steps, dt)}
    try:
        n_cpu = len(os.sched_getaffinity(0))
    except AttributeError:
        n_cpu = os.cpu_count() or 1
    n_proc = max(1, min(16, n_cpu, len(work.victims)))
    ctx = mp.get_context("fork")
    start, q = ctx.Barrier(n_proc), ctx.Queue()
    # victims dealt largest first to the least loaded process
    loads, groups = [0] * n_proc, [[] for _ in range(n_proc)]
    for v in sorted(work.victims, key=lambda v: -len(work.tables[v])):
        k = loads.index(min(loads))
        groups[k].append(v)
        loads[k] += len(work.tables[v])
    procs = [ctx.Process(target=_oracle_worker, args=((work, g, all_cores_budget_s, start, q),)) for g in groups]
    for p in procs:
        p.start()
    res = [q.get() for _ in procs]
    for p in procs:
        p.join()
    tot = sum(r[1][0] for r in res)
    slowest = max(r[1][1] for r in res)
    out["all_cores"] = {"value": tot / slowest / 1e9, "unit": "GB/s", "cores": n_proc,
                        "sample": "the same victims dealt to %d processes (largest first), each repeating its own "
                                  "out+in steps for %.0f s; total bytes / %.1f s" % (n_proc, all_cores_budget_s, slowest)}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="config 2 only: leave the short runs of configs 1, 3, 4 and 5 out of the JSON line")
    ap.add_argument("--latency-reps", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5],
                    help="workload config; 2 is the headline (default), the others print their own JSON line")
    ap.add_argument("--preemptions", type=int, default=200, help="config 3: length of the stream")
    ap.add_argument("--conversations", type=int, default=128, help="config 4: conversations (in waves that fit the arena)")
    ap.add_argument("--arena-gib", type=int, default=56, help="config 4: pinned host arena (one allocation)")
    ap.add_argument("--no-strided-copies", action="store_true",
                    help="one copy per run of adjacent host records (KV_FLAG_NO_STRIDED_COPIES), for comparison")
    ap.add_argument("--no-fairness", action="store_true", help="config 3: skip the small-copy latency measurement")
    ap.add_argument("--no-manager-pass", action="store_true", help="config 3: skip the pass through kv_manager_iterate")
    ap.add_argument("--no-defer-copies", action="store_true",
                    help="KV_FLAG_NO_DEFER_COPIES: every swap-out's copies are enqueued inside the call and wait for "
                         "their gathers on the device (default: the pool's copy thread enqueues them once the gathers "
                         "have finished)")
    ap.add_argument("--no-direct-path", action="store_true",
                    help="config 5: leave out the per-group direct copies (the comparison path with hundreds of thousands of copies)")
    ap.add_argument("--second-lane", action="store_true",
                    help="KV_FLAG_SECOND_LANE: scattered records of a held-back swap-out as plain copies over both copy streams")
    ap.add_argument("--no-profile", action="store_true",
                    help="config 3: a pool without KV_FLAG_PROFILE, as an application would create it (no per-launch rates)")
    ap.add_argument("--no-launch-events", action="store_true",
                    help="KV_FLAG_NO_LAUNCH_EVENTS: plain pack launches also for large swaps (with --no-profile)")
    ap.add_argument("--out-first", action="store_true",
                    help="config 3: issue the swap-out of an iteration before its swap-in (default: swap-in first)")
    ap.add_argument("--requests", type=int, default=4, help="config 5: 10 GiB requests per run length")
    ap.add_argument("--mapped-swap-in", action="store_true",
                    help="swap-in by a kernel that reads the pinned host image directly (KV_FLAG_MAPPED_SWAP_IN)")
    ap.add_argument("--mapped-swap-out", action="store_true",
                    help="config 1: swap-out by a kernel that stores into the pinned image (KV_FLAG_MAPPED_SWAP_OUT)")
    ap.add_argument("--copy-chunk-mib", type=int, default=0,
                    help="configs 2 and 3: cut host-link copies at this many MiB (0 = the library's default)")
    ap.add_argument("--max-piece-mib", type=int, default=0,
                    help="config 2: most MiB one piece of a swap carries (0 = the library's default)")
    ap.add_argument("--scatter-stream", action="store_true",
                    help="three streams: scatter kernels on a stream of their own (KV_FLAG_SCATTER_STREAM)")
    ap.add_argument("--four-streams", action="store_true",
                    help="give kernels and copies of each direction their own streams (KV_FLAG_FOUR_STREAMS)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only (the swap path has no cross-GPU step); "
            "--gpus %d is not supported" % args.gpus)
        return 2

    import numpy as np
    from paper_2411_18424_amd import synth

    # The CPU oracle is timed first, in this process, before anything has touched the GPU (its
    # all-cores leg forks workers); the GPU is idle meanwhile and the timed region below has
    # the host to itself.
    cpu = None
    if args.config == 2 and not args.no_cpu_baseline:
        log("timing the CPU oracle (one thread, then all cores) ...")
        cpu = cpu_baseline(synth.llama3_8b_preempt_workload())
        log("cpu oracle: %.2f GB/s on one core, %.2f GB/s on %d (%s)"
            % (cpu["value"], cpu["all_cores"]["value"], cpu["all_cores"]["cores"], cpu["cpu"]))

    import torch
    from paper_2411_18424_amd import kvswap as kv

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.config != 2:
        import bench_configs
        result = {1: bench_configs.config1, 3: bench_configs.config3, 4: bench_configs.config4,
                  5: bench_configs.config5}[args.config](args)
        print(json.dumps(result), flush=True)
        return 0
    work = synth.llama3_8b_preempt_workload()
    s = work.shape
    victims = work.victims
    nb = sum(len(work.tables[v]) for v in victims)
    payload = nb * s.R  # bytes each way per step
    log("workload: %s, pool %d blocks (%.1f GiB), %d requests, %d victims = %d blocks = %.2f GiB each way"
        % (s.name, s.n_blocks, s.n_blocks * s.R / GiB, len(work.tables), len(victims), nb, payload / GiB))

    # ---- measured ceilings (before anything else is resident; not while the driver still clears the device memory
    #      of a process that has just ended: the two-way probe then reads 60 GB/s instead of 97)
    import bench_configs
    settled_first = bench_configs.settle(torch)
    log("settle (before the probes):", settled_first)
    link_d2h = kv.kv_link_probe(GiB, 0, 10)
    link_h2d = kv.kv_link_probe(GiB, 1, 10)
    link_duplex = kv.kv_link_probe(GiB, 2, 5)
    hbm_copy = kv.kv_hbm_probe(2 * GiB, 10)
    log("measured: link d2h %.2f h2d %.2f duplex %.2f GB/s; device copy kernel %.0f GB/s"
        % (link_d2h, link_h2d, link_duplex, hbm_copy))

    # ---- pool resident in HBM
    gpu = torch.empty(s.R * s.n_blocks, dtype=torch.uint8, device=dev)
    content = synth.PoolContent(s, work.cfg)
    content.fill_device(gpu)
    pool = kv.KVPool(n_layers=s.n_layers, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim,
                     block_size=s.block_size, elt_bytes=s.elt_bytes, n_gpu_blocks=s.n_blocks,
                     gpu_base=gpu.data_ptr(), host_bytes=payload + 64 * len(victims) * s.R,
                     flags=kv.KV_FLAG_PROFILE | (kv.KV_FLAG_FOUR_STREAMS if args.four_streams else 0)
                     | (kv.KV_FLAG_SCATTER_STREAM if args.scatter_stream else 0)
                     | (kv.KV_FLAG_NO_DEFER_COPIES if args.no_defer_copies else 0)
                     | (kv.KV_FLAG_SECOND_LANE if args.second_lane else 0)
                     | (kv.KV_FLAG_MAPPED_SWAP_IN if args.mapped_swap_in else 0),
                     pack_variant=int(os.environ.get("KVSWAP_PACK_VARIANT", "0")),
                     copy_chunk_bytes=args.copy_chunk_mib << 20, max_piece_bytes=args.max_piece_mib << 20)
    cur = [work.tables[v] for v in victims]
    nxt = list(work.resume_tables)
    settled = bench_configs.settle(torch)  # not while the driver still clears a previous process's device memory
    log("settle:", settled)

    phase_s = [0.0, 0.0]  # time in the swap-out and the swap-in half of the steps (host clock)
    step_ms = []  # (swap-out half, swap-in half) of every step

    def step():
        nonlocal cur, nxt
        t_a = time.perf_counter()
        pool.swap_out_batch(victims, cur)
        pool.kv_wait_all()
        t_b = time.perf_counter()
        pool.swap_in_batch(victims, nxt)
        pool.kv_wait_all()
        t_c = time.perf_counter()
        phase_s[0] += t_b - t_a
        phase_s[1] += t_c - t_b
        step_ms.append(((t_b - t_a) * 1e3, (t_c - t_b) * 1e3))
        cur, nxt = nxt, cur

    for _ in range(args.warmup):
        step()
    n_warm = len(pool.kv_profile_read())  # also waits for the warm-up to finish
    dev_state = device_state()  # right after the warm-up steps, before the timed region
    torch.cuda.synchronize()
    phase_s[0] = phase_s[1] = 0.0
    del step_ms[:]
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    recs = pool.kv_profile_read()[n_warm:]  # launches and copies of the timed region only

    def agg(kind):
        rs = [r for r in recs if r[0] == kind]
        nbytes = sum(r[1] for r in rs)
        ms = sum(r[2] for r in rs)
        return len(rs), nbytes, ms

    n_g, b_g, ms_g = agg(0)
    n_s, b_s, ms_s = agg(4 if args.mapped_swap_in else 1)
    n_o, b_o, ms_o = agg(2)
    n_i, b_i, ms_i = agg(3)
    gather_gbps = 2 * b_g / ms_g / 1e6
    scatter_gbps = 2 * b_s / ms_s / 1e6
    d2h_gbps = b_o / ms_o / 1e6
    h2d_gbps = b_i / ms_i / 1e6 if ms_i > 0 else b_s / ms_s / 1e6  # mapped swap-in: the kernel is the transfer

    # ---- sampled check against the content definition (outside the timed region)
    pool.swap_out_batch(victims, cur)
    pool.kv_wait_all()
    rng = synth.rng_for(work.cfg, stream=99)
    # a logical block keeps the bytes it was created with, wherever it has been moved since
    origin = [work.tables[v] for v in victims]
    ok = True
    for i in rng.integers(0, len(victims), size=8):
        j = int(rng.integers(0, len(origin[i])))
        ok &= bool(np.array_equal(pool.kv_host_read(victims[i], j, 1)[0], content.block(int(origin[i][j]))))
    pool.swap_in_batch(victims, cur)
    pool.kv_wait_all()

    # ---- per-preemption switch latency: one victim out, one in, call -> completion
    out_ms, in_ms, sw_ms, call_us = [], [], [], []
    for _ in range(args.latency_reps):
        for i, v in enumerate(victims):
            t_a = time.perf_counter()
            pool.swap_out(v, cur[i])
            call_us.append((time.perf_counter() - t_a) * 1e6)
            pool.kv_wait(v)
            t_b = time.perf_counter()
            pool.swap_in(v, nxt[i])
            pool.kv_wait(v)
            t_c = time.perf_counter()
            out_ms.append((t_b - t_a) * 1e3)
            in_ms.append((t_c - t_b) * 1e3)
            sw_ms.append((t_c - t_a) * 1e3)
        cur, nxt = nxt, cur
    # overlapped switch: victim i leaves while victim i-1 resumes (both directions at once)
    ov_ms = []
    if args.latency_reps > 0:
        pool.swap_out(victims[0], cur[0])
        pool.kv_wait(victims[0])
    for i in range(1, len(victims) if args.latency_reps > 0 else 0):
        t_a = time.perf_counter()
        pool.swap_out(victims[i], cur[i])
        pool.swap_in(victims[i - 1], nxt[i - 1])
        pool.kv_wait(victims[i])
        pool.kv_wait(victims[i - 1])
        ov_ms.append((time.perf_counter() - t_a) * 1e3)
    if args.latency_reps > 0:
        pool.swap_in(victims[-1], nxt[-1])
    pool.kv_wait_all()
    # the same swaps submitted through the swap manager: what the scheduler's thread pays
    submit_us, mgr_stats = [], None
    if args.latency_reps > 0:
        mgr = kv.KVManager(pool)
        for _ in range(args.latency_reps):
            for i, v in enumerate(victims):
                t_a = time.perf_counter()
                tk = mgr.kv_manager_submit(kv.KV_TASK_SWAP_OUT, v, cur[i])
                submit_us.append((time.perf_counter() - t_a) * 1e6)
                t_a = time.perf_counter()
                mgr.kv_manager_submit(kv.KV_TASK_SWAP_IN, v, nxt[i])
                submit_us.append((time.perf_counter() - t_a) * 1e6)
            mgr.kv_manager_drain()
            cur, nxt = nxt, cur
        mgr_stats = mgr.kv_manager_stats()
        mgr.kv_manager_destroy()
    all_recs = pool.kv_profile_read()  # every launch and copy of this process
    stats = pool.kv_stats()
    pool.kv_pool_destroy()

    # layer-wise swap-in (the alternative the paper discusses): when does the first step of
    # layers land, when the last, against whole-request swap-in.  A pool of its own without
    # per-launch timing events, which would cost more than the steps themselves.
    lw = {}
    if args.latency_reps > 0:
        pool = kv.KVPool(n_layers=s.n_layers, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim,
                         block_size=s.block_size, elt_bytes=s.elt_bytes, n_gpu_blocks=s.n_blocks,
                         gpu_base=gpu.data_ptr(), host_bytes=payload + 64 * len(victims) * s.R,
                         flags=(kv.KV_FLAG_FOUR_STREAMS if args.four_streams else 0)
                         | (kv.KV_FLAG_MAPPED_SWAP_IN if args.mapped_swap_in else 0))
        pool.swap_out_batch(victims, cur)
        pool.kv_wait_all()
        for lps in (0, s.n_layers, 4, 1):
            call, first, last = [], [], []
            for i, v in enumerate(victims):
                t_a = time.perf_counter()
                if lps:
                    pool.swap_in_layerwise(v, nxt[i], lps)
                    t_b = time.perf_counter()
                    pool.kv_wait_layer(v, 0)
                else:
                    pool.swap_in(v, nxt[i])
                    t_b = time.perf_counter()
                    pool.kv_wait(v)
                t_c = time.perf_counter()
                pool.kv_wait(v)
                t_d = time.perf_counter()
                call.append((t_b - t_a) * 1e3)
                first.append((t_c - t_a) * 1e3)
                last.append((t_d - t_a) * 1e3)
            cur, nxt = nxt, cur
            lw["layers_per_step_%d" % lps if lps else "whole_request_swap_in"] = {
                "call_median": percentile(call, 50), "first_step_median": percentile(first, 50),
                "all_layers_median": percentile(last, 50), "all_victims_sum": round(sum(last), 3)}
        pool.kv_pool_destroy()
    del gpu
    torch.cuda.empty_cache()

    # HBM bytes per launch as the rocprofv3 counters read them (FETCH_SIZE and WRITE_SIZE passes of
    # this same command, scaled by what they read for a plain copy of known size).  The counters
    # cannot be read from inside this process: the figures are those of the committed summary,
    # labelled as such; null when the summary is not there.
    def profiled_traffic(fname):
        tpath = os.path.join(ROOT, "profiles", fname)
        if os.path.exists(tpath):
            with open(tpath) as f:
                for line in f:
                    if line.startswith("hbm_bytes_per_launch:"):
                        return (int(line.split(":")[1].split()[0]),
                                "profiles/%s (rocprofv3 --pmc runs of this command; a stored figure, not measured in this run)" % fname)
        return None, None

    g_traffic, g_src = profiled_traffic("gather_llama3_8b_cfg2_pmc.txt")
    s_traffic, s_src = profiled_traffic("scatter_llama3_8b_cfg2_pmc.txt")
    pack = {
        "gather": {"kernel": "kv_pack_xcd_kernel<256,1,true,false,true> (kv_pack_tile_kernel below 64 blocks per launch)",
                   "achieved": round(gather_gbps, 1), "frac": round(gather_gbps / HBM_PEAK_GBPS, 4),
                   "launches": n_g, "avg_launch_ms": round(ms_g / max(1, n_g), 4),
                   "algorithmic_bytes_per_launch": int(2 * b_g / max(1, n_g)),
                   "traffic": g_traffic, "traffic_source": g_src},
        "scatter": {"kernel": "kv_pack_xcd_kernel<256,1,true,true,true> (kv_pack_tile_kernel below 64 blocks per launch)",
                    "achieved": round(scatter_gbps, 1), "frac": round(scatter_gbps / HBM_PEAK_GBPS, 4),
                    "launches": n_s, "avg_launch_ms": round(ms_s / max(1, n_s), 4),
                    "algorithmic_bytes_per_launch": int(2 * b_s / max(1, n_s)),
                    "traffic": s_traffic, "traffic_source": s_src},
    }
    low = "scatter" if scatter_gbps < gather_gbps else "gather"  # the headline fraction is the lower of the two

    result = {
        "metric": "KV swap GB/s (out+in) and per-preemption switch latency, 1 MI355X",
        "value": round(2 * payload * args.steps / dt / 1e9, 3),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {
            "workload": "config 2: Llama-3-8B-shaped KV (32 layers, 8 KV heads, head_dim 128, block 16, bf16), "
                        "8192-block pool, 64 lognormal requests in block groups of 8, 16 victims swapped out "
                        "(batched) then in through fresh tables",
            "payload_bytes_each_way": payload,
            "victim_blocks": nb,
        },
        "out_gbps": round(payload * args.steps / phase_s[0] / 1e9, 3),
        "in_gbps": round(payload * args.steps / phase_s[1] / 1e9, 3),
        "step_halves_ms": {"what": "host clock, swap-out call -> all done and swap-in call -> all done, over the timed steps",
                           "out": dist3([a for a, _ in step_ms]), "in": dist3([b for _, b in step_ms])},
        "roofline": {
            "bound": "hbm",
            "kernel": "%s direction of the pack kernel (the slower of the two): %s" % (low, pack[low]["kernel"]),
            "achieved": pack[low]["achieved"],
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": pack[low]["frac"],
            "traffic": pack[low]["traffic"],
            "traffic_source": pack[low]["traffic_source"],
            "launches": pack[low]["launches"],
            "avg_launch_ms": pack[low]["avg_launch_ms"],
            "algorithmic_bytes_per_launch": pack[low]["algorithmic_bytes_per_launch"],
            "gather": pack["gather"],
            "scatter": pack["scatter"],
            "device_copy_kernel_gbps": round(hbm_copy, 1),
            # every launch of this process (warm-up, timed region, sampled check and the
            # per-request latency phases): the population a kernel trace of this command sees
            "gather_calls_whole_process": len([r for r in all_recs if r[0] == 0]),
            "gather_avg_ms_whole_process": round(
                sum(r[2] for r in all_recs if r[0] == 0) / max(1, len([r for r in all_recs if r[0] == 0])), 4),
            "scatter_calls_whole_process": len([r for r in all_recs if r[0] == 1]),
            "scatter_avg_ms_whole_process": round(
                sum(r[2] for r in all_recs if r[0] == 1) / max(1, len([r for r in all_recs if r[0] == 1])), 4),
        },
        "link": {
            "measured_peak_d2h_gbps": round(link_d2h, 2),
            "measured_peak_h2d_gbps": round(link_h2d, 2),
            "measured_peak_duplex_gbps": round(link_duplex, 2),
            "d2h_copies_gbps": round(d2h_gbps, 2),
            "h2d_copies_gbps": round(h2d_gbps, 2),
            "d2h_frac_of_measured": round(d2h_gbps / link_d2h, 4),
            "h2d_frac_of_measured": round(h2d_gbps / link_h2d, 4),
        },
        "switch_latency_ms": {
            "what": "one victim: swap_out call -> done, then swap_in call -> done (sequential), host clock",
            "n": len(sw_ms),
            "median": percentile(sw_ms, 50), "p99": percentile(sw_ms, 99),
            "max": percentile(sw_ms, 100),
            "out_median": percentile(out_ms, 50), "in_median": percentile(in_ms, 50),
            "overlapped_median": percentile(ov_ms, 50),
            "overlapped_p99": percentile(ov_ms, 99),
            "median_request_MiB": round(float(np.median([len(t) for t in cur])) * s.R / (1 << 20), 1),
        },
        "layerwise_swap_in_ms": {
            "what": "swap_in_layerwise per victim: host time of the call, call -> first step of layers landed "
                    "(not before the call has returned), call -> all landed; host clock",
            **lw,
        },
        "dispatch_us": {
            "what": "host time of one swap_out per victim: direct call vs submit to the swap manager "
                    "(Python + ctypes included in both)",
            "direct_call_median": percentile(call_us, 50),
            "manager_submit_median": percentile(submit_us, 50),
            "manager_dispatcher_avg": (round(mgr_stats["dispatch_us_sum"] / max(1, mgr_stats["dispatched"]), 2)
                                       if mgr_stats else None),
        },
        "device_state": dev_state,
        "settle": settled, "settle_before_probes": {k: settled_first[k] for k in ("waited_s", "slow_probes", "probes")},
        "streams": 4 if args.four_streams else 3 if args.scatter_stream else 2,
        "swap_out_copies": "enqueued inside the call" if args.no_defer_copies
                           else "held back until their gathers are done (copy thread)",
        "pack_variant": int(os.environ.get("KVSWAP_PACK_VARIANT", "0")),  # development aid; 0 = the default kernels
        "swap_in_path": "mapped host reads" if args.mapped_swap_in else "staged copies + scatter",
        "verified_samples_ok": ok,
        "stats": {k: stats[k] for k in ("gather_launches", "scatter_launches", "d2h_copies", "h2d_copies")},
    }
    if cpu is not None:
        result["cpu_baseline"] = cpu
    if not args.headline_only:
        # the other workload configs in short form (after the headline's timed region; each waits for
        # the copy engines to be quiet first); `python bench.py --config N` is the long form of each
        log("running configs 1, 4, 5, 3 in short form ...")
        args.two_way_peak = link_duplex  # measured above, at the start of the process
        result["other_configs"] = bench_configs.other_configs(args)
    print(json.dumps(result), flush=True)
    return 0 if ok else 1


if __name__ == "__main__":
    sys.exit(main())
