"""The measuring aids of the C ABI: per-kernel timers, the calibration kernels, the copy helper."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2411_01611_amd import binding, synth
from gpu_harness import GpuCase


def test_kernel_timers_count_every_launch_of_a_step():
    wl = synth.workload("multi_hot", scale=0.004, batch=333)
    c = GpuCase(wl)
    c.build()
    s = c.s
    d_idx, d_off = c.dev_batch()
    grad = c.sampler.grads(0).to(c.dev)
    assert s.profile_read() == {}                                 # nothing is timed until asked
    s.profile_enable(True)
    for _ in range(2):
        rm = s.remap(d_idx, d_off, wl.batch)
        s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
        s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad, 0.01, 1e-8)
    prof = s.profile_read()
    passes = -(-int(np.ceil(np.log2(wl.total_rows + 1))) // 9)   # 9 bits per radix pass
    want = {"remap_probe": 2, "remap_write": 2, "stage_misses": 2, "sort_hist": 2 * passes, "sort_scan": 2 * passes,
            "sort_scatter": 2 * passes, "seg_count": 2, "seg_write": 2, "seg_rows_long": 2, "seg_combine": 2}
    for name, n in want.items():
        assert prof[name]["launches"] == n, (name, prof)
        assert prof[name]["total_ms"] > 0.0
    assert sum(1 for k in prof if k.startswith("pool_")) == 1     # one pooling kernel, whichever fits the bag lengths
    assert "bwd_pairs" not in prof                                # remap wrote the pairs
    assert s.profile_read() == {}                                 # reading empties the list
    s.profile_enable(False)
    s.remap(d_idx, d_off, wl.batch)
    assert s.profile_read() == {}
    assert s.sync_status() == 0
    c.close()


def test_calibration_kernels_and_copy_helper():
    dev = torch.device("cuda:0")
    src = torch.randint(0, 2 ** 31 - 1, (1 << 20,), dtype=torch.int32, device=dev)
    dst = torch.zeros_like(src)
    binding.calibration_copy(dst, src)
    assert torch.equal(dst, src)
    sink = torch.zeros(binding.CALIB_SINK_BYTES // 4, dtype=torch.int32, device=dev)
    binding.calibration_read(src, sink)
    torch.cuda.synchronize()
    host = binding.PinnedArray((1 << 20,), np.int32)
    binding.memcpy(host.ptr, src.data_ptr(), src.numel() * 4, 2)
    torch.cuda.synchronize()
    assert np.array_equal(host.np, src.cpu().numpy())
    back = torch.empty_like(src)
    binding.memcpy(back.data_ptr(), host.ptr, src.numel() * 4, 1)
    torch.cuda.synchronize()
    assert torch.equal(back, src)
    host.free()
    L = binding.lib()
    assert L.scars_calibration_copy(dst.data_ptr(), src.data_ptr(), 24, None) == binding.ERR_INVALID_ARG   # not 16-byte units
    assert L.scars_memcpy(None, src.data_ptr(), 16, 1, None) == binding.ERR_INVALID_ARG
