"""swap_out_static, the entry point that allocates nothing, against swap_out (and the oracle):
two calls in a row, the second with a smaller input, through the C ABI; and recorded into a HIP
graph by stream capture (it allocates nothing, so it can be), every replay checked."""

import numpy as np
import pytest

from paper_2411_18424_amd import synth

pytestmark = pytest.mark.gpu

MiB = 1 << 20


def test_swap_out_static_matches_swap_out():
    import torch
    from gpu_util import Harness
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 512, "bf16")  # C = 32 KiB, R = 512 KiB
    h = Harness(shape, 71, 256 * MiB, fill="random")
    try:
        kv, pool = h.kv, h.pool
        rng = synth.rng_for(71)
        dst = torch.empty(128 * shape.R, dtype=torch.uint8).pin_memory()
        dst.fill_(0xEE)
        side = torch.cuda.Stream()
        for call, (req, n) in enumerate(((0, 128), (1, 37))):   # 64 MiB (the limit), then 18.5 MiB
            table = rng.permutation(shape.n_blocks)[:n].astype(np.int32)
            # the existing entry point and the definition
            pool.swap_out(req, table)
            h.oracle.swap_out(req, table)
            want = pool.kv_host_read(req)
            assert np.array_equal(want, h.oracle.host[req].Hq)
            # the allocation-free variant: on the caller's stream, then on the library's
            for stream in (side.cuda_stream, 0):
                dst.fill_(0xEE)
                pool.swap_out_static(table, dst.data_ptr(), stream)
                if stream:
                    side.synchronize()
                got = dst.numpy()[:n * shape.R].reshape(n, shape.P, shape.C)
                assert np.array_equal(got, want), "call %d differs from swap_out" % call
                assert (dst.numpy()[n * shape.R:] == 0xEE).all(), "wrote past n_blocks * R"
        h.assert_pool_equal()  # a swap-out changes nothing on the GPU
        # limits and validation: nothing is enqueued
        dst.fill_(0x11)
        for bad in (np.arange(129, dtype=np.int32), np.array([3, 3], np.int32), np.array([512], np.int32)):
            with pytest.raises(kv.KVError) as ei:
                pool.swap_out_static(bad, dst.data_ptr(), 0)
            assert ei.value.status == kv.KV_EINVAL
        pool.swap_out_static(np.zeros(0, np.int32), dst.data_ptr(), 0)
        torch.cuda.synchronize()
        assert (dst.numpy() == 0x11).all()
    finally:
        h.close()


@pytest.mark.parametrize("L,H,D,N,n", [(3, 3, 40, 300, 200),    # chunk of 3840 bytes: not a multiple of the tile
                                       (2, 4, 64, 256, 63),     # 63 blocks: the 3-D grid (below 64 blocks)
                                       (1, 40, 128, 200, 150)]) # one layer, 160 KiB chunks, XCD-aware order
def test_swap_out_static_on_other_shapes(L, H, D, N, n):
    import torch
    from gpu_util import Harness
    shape = synth.KVShape("s", L, H, D, 16, 2, N, "fp16")
    h = Harness(shape, 73, 8 * MiB, fill="random")
    try:
        rng = synth.rng_for(73)
        table = rng.permutation(N)[:n].astype(np.int32)
        dst = torch.empty(n * shape.R, dtype=torch.uint8).pin_memory()
        dst.fill_(0xEE)
        h.pool.swap_out_static(table, dst.data_ptr(), 0)
        h.oracle.swap_out(0, table)
        assert np.array_equal(dst.numpy().reshape(n, shape.P, shape.C), h.oracle.host[0].Hq)
    finally:
        h.close()


def test_swap_out_static_in_a_captured_graph():
    import torch
    from gpu_util import Harness
    shape = synth.KVShape("s", 8, 8, 128, 16, 2, 512, "bf16")  # R = 512 KiB
    h = Harness(shape, 72, 64 * MiB, fill="random")
    try:
        rng = synth.rng_for(72)
        n = 90
        table = rng.permutation(shape.n_blocks)[:n].astype(np.int32)
        dst = torch.empty(n * shape.R, dtype=torch.uint8).pin_memory()
        side = torch.cuda.Stream()
        # eager call first (loads the code object, proves the path)
        h.pool.swap_out_static(table, dst.data_ptr(), side.cuda_stream)
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            h.pool.swap_out_static(table, dst.data_ptr(), torch.cuda.current_stream().cuda_stream)
        for rep in range(3):
            # eager work between the replays: the blocks get new content on both sides
            h.overwrite_blocks(table, synth.fresh_tokens(rng, shape, n))
            dst.fill_(0xEE)
            g.replay()
            torch.cuda.synchronize()
            h.oracle.swap_out(100 + rep, table)
            got = dst.numpy().reshape(n, shape.P, shape.C)
            assert np.array_equal(got, h.oracle.host[100 + rep].Hq), "replay %d delivered other bytes" % rep
    finally:
        h.close()
