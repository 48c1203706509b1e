"""The entry point that allocates nothing: cmp_compress_static against cmp_compress.

For callers that cannot call hipMalloc (graph capture, serving loops): same kernels, scratch in a
static device array.  Checked through the C ABI: the container is byte for byte that of
cmp_compress, on two calls in a row (the second with a smaller input, so stale scratch of the
first would show), and sizes beyond the stated maximum are refused.
"""
import numpy as np
import pytest
import torch

from paper_2011_09017_amd.workloads import activation

pytestmark = pytest.mark.gpu


def test_static_entry_point_matches_cmp_compress(orc):
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2011_09017_amd import binding as gpu
    gpu.lib()
    dev = torch.device("cuda", 0)
    stream = torch.cuda.current_stream(dev).cuda_stream
    for sub in (32, 128):
        cfg = gpu.cmp_config(512, 4096, sub, 7, 0)
        ctx = gpu.Context(sub=sub, max_numel=gpu.CMP_STATIC_MAX_NUMEL)
        # the largest size the entry point takes, with outliers; then smaller inputs, one of them ragged
        cases = [((4, 64, 128, 128), 1e-2, 5), ((2, 16, 56, 56), 1e-2, 0), ((3, 5, 55, 55), 1e-3, 3), ((1, 1, 1, 1), 1e-2, 0)]
        for shape, eb, spikes in cases:
            xh = activation(shape, 5, 0.5, seed=77 + shape[1]).numpy() if np.prod(shape) > 1 else np.full(shape, 0.25, np.float32)
            for k in range(spikes):
                xh.reshape(-1)[(k + 1) * xh.size // (spikes + 1)] = 25000.0 * eb
            x = torch.from_numpy(xh).to(dev)
            ref, rsize, rc = ctx.compress(x, eb)
            assert rc == 0
            out = torch.full((ctx.bound(shape),), 0xCD, dtype=torch.uint8, device=dev)
            rc = gpu.cmp_compress_static(0, cfg, x.data_ptr(), shape, eb, out.data_ptr(), out.numel(), stream)
            assert rc == 0, gpu.cmp_strerror(rc)
            rc, size = gpu.cmp_compressed_size(None, out.data_ptr(), stream)
            assert rc == 0 and size == rsize
            assert torch.equal(out[:size], ref[:rsize]), (shape, sub)
            assert bool((out[size:] == 0xCD).all())                     # nothing written past the container
            # and it is the oracle's container
            orc_rc, obuf, osize, _ = orc.compress(xh, eb, orc.Config(sub=sub))
            assert orc_rc == 0 and osize == size and np.array_equal(out[:size].cpu().numpy(), obuf)
        # beyond the maximum, bad arguments, too little room
        big = torch.zeros((1, 1, 2049, 2048), device=dev)
        out = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
        assert gpu.cmp_compress_static(0, cfg, big.data_ptr(), big.shape, 1e-2, out.data_ptr(), out.numel(), stream) == gpu.CMP_E_ARG
        small = torch.zeros((1, 1, 64, 64), device=dev)
        assert gpu.cmp_compress_static(0, cfg, small.data_ptr(), small.shape, 0.0, out.data_ptr(), out.numel(), stream) == gpu.CMP_E_ARG
        assert gpu.cmp_compress_static(9, cfg, small.data_ptr(), small.shape, 1e-2, out.data_ptr(), out.numel(), stream) == gpu.CMP_E_ARG
        assert gpu.cmp_compress_static(0, cfg, small.data_ptr(), small.shape, 1e-2, out.data_ptr(), 64, stream) == gpu.CMP_E_NOSPACE
        # a container that does not fit is reported by its header
        x = torch.from_numpy(activation((2, 16, 56, 56), 5, 0.5, seed=5).numpy()).to(dev)
        _, need, _ = ctx.compress(x, 1e-2)
        tight = torch.zeros(need - 16, dtype=torch.uint8, device=dev)
        assert gpu.cmp_compress_static(0, cfg, x.data_ptr(), x.shape, 1e-2, tight.data_ptr(), tight.numel(), stream) == 0
        rc, size = gpu.cmp_compressed_size(None, tight.data_ptr(), stream)
        assert rc == gpu.CMP_E_NOSPACE and size == need
        ctx.close()
