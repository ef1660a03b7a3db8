"""Granularity of block groups under a synthetic preemption stream (CPU only).

FastSwitch's Dynamic Block Group Manager (Section 3.1) is judged by its transfer granularity:
the average number of blocks per contiguous group at swap time (Section 5.3.1 reports about 20
blocks per group on its traces and little sensitivity to the initial group size).  This module
drives the library's block-group manager (on a plan-only pool: bookkeeping only, no GPU) with a
synthetic serving loop - requests decode one token per iteration, priorities are redrawn every
1/f iterations with a Random or a Markov-like pattern (Section 4), the lowest-priority running
requests are preempted and the highest-priority waiting ones resumed - and reports the
granularity seen by the swap-outs.  It stands in for the paper's ShareGPT traces, which are not
available here; only the mechanism is exercised, the absolute figure is not comparable.
"""

from __future__ import annotations

import numpy as np

from . import kvswap as kv
from . import synth


def run_lengths(ids) -> list:
    ids = np.asarray(ids, dtype=np.int64)
    if ids.size == 0:
        return []
    cuts = np.flatnonzero(np.diff(ids) != 1) + 1
    return np.diff(np.concatenate([[0], cuts, [ids.size]])).tolist()


def simulate(first_group: int = 64, pattern: str = "markov", f: float = 0.02, n_iters: int = 4000,
             n_blocks: int = 4096, n_conv: int = 96, block_size: int = 16, seed: int = 7,
             reserve_tail: int = 0) -> dict:
    """Returns average blocks per group over all swap-outs, and manager statistics."""
    shape = synth.KVShape("sim", 1, 1, 8, 1, 2, n_blocks, "fp16")  # tiny records: bookkeeping only
    pool = kv.KVPool(n_layers=1, n_kv_heads=1, head_dim=8, block_size=1, elt_bytes=2,
                     n_gpu_blocks=n_blocks, host_bytes=8 * n_blocks * shape.R, flags=kv.KV_FLAG_PLAN_ONLY)
    pool.kv_bg_configure(first_group, seed)
    rng = synth.rng_for(40 + seed)
    tokens = np.clip(np.rint(np.exp(rng.normal(np.log(400), 0.9, size=n_conv))), 16, 4096).astype(np.int64)
    limit = tokens + np.clip(np.rint(np.exp(rng.normal(np.log(300), 0.8, size=n_conv))), 16, 2048).astype(np.int64)
    running, swapped, waiting = set(), set(), set(range(n_conv))
    prio = rng.random(n_conv)
    last_served = np.zeros(n_conv)
    group_sizes, groups_per_swap = [], []
    period = max(1, int(round(1.0 / f)))

    def blocks_of(c):
        return int(-(-tokens[c] // block_size))

    def free_for_new():
        return pool.kv_free_blocks()[0]

    def try_start(c):
        need = blocks_of(c)
        if need + 8 > free_for_new():
            return False
        pool.kv_bg_append(c, need, reserve_tail)
        if c in swapped:
            pool.swap_in(c, pool.kv_bg_table(c))
            swapped.discard(c)
        waiting.discard(c)
        running.add(c)
        return True

    def preempt(c):
        t = pool.kv_bg_table(c)
        rl = run_lengths(t)
        group_sizes.extend(rl)
        groups_per_swap.append(len(rl))
        pool.swap_out(c, t)
        pool.kv_bg_close(c)
        running.discard(c)
        swapped.add(c)

    for it in range(n_iters):
        if it % period == 0:
            if pattern == "random":
                prio = rng.random(n_conv)
            else:  # recently served requests tend to keep a high priority
                prio = 0.7 * (last_served > it - 2 * period) + 0.3 * rng.random(n_conv)
            order = np.argsort(-prio)
            keep_n = max(1, len(running) // 2)
            keep = set(int(c) for c in order[:n_conv] if int(c) in running)
            low = sorted(running, key=lambda c: prio[c])[:max(0, len(running) - keep_n)]
            for c in low:
                preempt(c)
            for c in order:
                c = int(c)
                if c in running:
                    continue
                if c in swapped or c in waiting:
                    if not try_start(c):
                        break
        # one decode iteration: every running request gets a token; a finished one leaves
        for c in list(running):
            tokens[c] += 1
            last_served[c] = it
            if tokens[c] % block_size == 1 and tokens[c] > 1:
                try:
                    pool.kv_bg_append(c, 1, reserve_tail)
                except kv.KVError:
                    tokens[c] -= 1  # the token was not produced
                    preempt(c)      # out of memory: the request itself is swapped out
                    continue
            if tokens[c] >= limit[c]:
                pool.kv_bg_close(c)
                running.discard(c)
                # the conversation comes back later as a new, longer turn
                limit[c] = tokens[c] + int(np.clip(np.rint(np.exp(rng.normal(np.log(300), 0.8))), 16, 2048))
                waiting.add(c)
        if not running and (waiting or swapped):
            for c in sorted(waiting | swapped, key=lambda c: -prio[c]):
                if not try_start(int(c)):
                    break
    st = pool.kv_bg_stats()
    pool.kv_pool_destroy()
    gs = np.asarray(group_sizes, dtype=np.float64)
    return {"first_group": first_group, "pattern": pattern, "f": f,
            "swap_outs": len(groups_per_swap),
            "avg_blocks_per_group": float(gs.mean()) if gs.size else 0.0,
            "avg_groups_per_swap": float(np.mean(groups_per_swap)) if groups_per_swap else 0.0,
            "avg_blocks_per_swap": float(gs.sum() / max(1, len(groups_per_swap))),
            "steals": st["steals"], "grown_in_place": st["grown_in_place"],
            "appended_groups": st["appended_groups"]}


if __name__ == "__main__":
    for pattern in ("random", "markov"):
        for fg in (1, 4, 16, 64, 187):
            r = simulate(first_group=fg, pattern=pattern)
            print("%-6s first_group %3d: %5.1f blocks/group, %4.1f groups/swap, %5.1f blocks/swap, "
                  "%d swap-outs, %d steals" % (pattern, fg, r["avg_blocks_per_group"], r["avg_groups_per_swap"],
                                               r["avg_blocks_per_swap"], r["swap_outs"], r["steals"]))
