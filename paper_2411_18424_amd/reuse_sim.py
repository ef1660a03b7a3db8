"""Swap-out volume with and without reuse of the CPU copy, against host memory size (CPU only).

FastSwitch's KV Cache Reuse Mechanism (Section 3.3) keeps the CPU copy of a conversation and
sends only what it lacks; its microbenchmark (Section 5.3.3) reports 53 % fewer swapped-out
blocks, and less benefit when CPU memory is small because copies get contaminated.  This module
replays a synthetic multi-turn stream (stand-in for the multi-round ShareGPT traces, which are
not available) on a plan-only pool - bookkeeping only, no GPU - and counts the blocks each
policy moves: `traditional` swaps the whole context out at every preemption, `reuse` uses
swap_out_delta with the turn's dirty mask on a host arena of a given size with
KV_FLAG_HOST_EVICT, where a full arena reclaims the copies of lower-priority conversations.
"""

from __future__ import annotations

import numpy as np

from . import kvswap as kv
from . import synth


def simulate(arena_blocks: int, reuse: bool, n_conv: int = 64, n_preempt: int = 600, seed: int = 3,
             n_blocks: int = 4096, block_size: int = 16) -> dict:
    pool = kv.KVPool(n_layers=1, n_kv_heads=1, head_dim=8, block_size=1, elt_bytes=2,
                     n_gpu_blocks=n_blocks, host_bytes=arena_blocks * 32,
                     flags=kv.KV_FLAG_PLAN_ONLY | kv.KV_FLAG_HOST_EVICT, host_slack_blocks=8)
    rng = synth.rng_for(50 + seed)
    tokens = np.clip(np.rint(np.exp(rng.normal(np.log(600), 0.8, size=n_conv))), 32, 6000).astype(np.int64)
    failed = 0
    for step in range(n_preempt):
        c = int(rng.integers(0, n_conv))
        pool.kv_host_set_priority(c, int(rng.integers(0, 8)))      # priorities are redrawn all the time
        old = int(tokens[c])
        new = int(np.clip(np.rint(np.exp(rng.normal(np.log(150), 0.7))), 8, 1500))
        n_old = int(synth.blocks_for(old, block_size))
        # the conversation ran a turn on the GPU (resumed from its host copy when it has one) ...
        tokens[c] = min(old + new, n_blocks * block_size // 2)
        n = int(synth.blocks_for(tokens[c], block_size))
        table = rng.permutation(n_blocks)[:n].astype(np.int32)
        # ... and is preempted: its KV goes to the host
        try:
            if reuse:
                try:
                    have, _ = pool.kv_host_len(c)
                except kv.KVError:
                    have = 0
                dirty = synth.turn_dirty_mask(min(n_old, n), old, int(tokens[c]) - old, block_size)
                if have == 0 or len(dirty) != n or have > n:
                    pool.swap_out(c, table)
                else:
                    pool.swap_out_delta(c, table, dirty)
            else:
                pool.swap_out(c, table)
        except kv.KVError as e:
            if e.status != kv.KV_ENOMEM_HOST:
                raise
            failed += 1   # no room even after eviction: this preemption would fall back to recomputation
    st = pool.kv_stats()
    pool.kv_pool_destroy()
    return {"arena_blocks": arena_blocks, "reuse": reuse, "blocks_out": st["blocks_out"],
            "evicted_blocks": st["host_evicted_blocks"], "failed": failed}


if __name__ == "__main__":
    base = simulate(1 << 20, reuse=False)
    print("traditional swap-out (whole context every time): %d blocks" % base["blocks_out"])
    for arena in (1 << 20, 8000, 4000, 2000, 1000):
        r = simulate(arena, reuse=True)
        print("reuse, host arena %7d records: %6d blocks (%.1f %% of traditional), %d evicted, %d could not be placed"
              % (arena, r["blocks_out"], 100.0 * r["blocks_out"] / base["blocks_out"], r["evicted_blocks"], r["failed"]))
