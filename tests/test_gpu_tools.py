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


def test_per_table_sort_replaces_the_radix_passes_when_the_caller_states_the_limit():
    wl = synth.workload("dlrm_onehot", scale=0.004, batch=1500)
    c = GpuCase(wl)
    c.build()
    s = c.s
    d_idx, d_off = c.dev_batch()
    grad = c.sampler.grads(0).to(c.dev)
    s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, wl.batch)
    s.profile_enable(True)
    rm = s.remap(d_idx, d_off, wl.batch)
    s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
    s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad, 0.01, 0.0)
    prof = s.profile_read()
    # remap wrote the pairs, rows can be cold: the forward pass's fetch carried the sort, the backward pass found it
    # done, with each run's length and row at the run's first position, and updated by position: one launch
    assert prof["stage_misses+small_sort"]["launches"] == 1 and prof["small_update"]["launches"] == 1
    assert "small_sort" not in prof and "stage_misses" not in prof
    assert not any(k in prof for k in ("small_segments", "seg_rows_long", "seg_rows", "seg_long", "seg_combine")), prof
    assert not any(k.startswith("sort_") or k in ("seg_count", "seg_scan", "seg_write", "bwd_pairs") for k in prof), prof
    assert s.get_counter(binding.COUNTER_SORTED_IN_FWD_USED) == 1
    # a backward pass that does not follow its own forward pass sorts for itself
    rm = s.remap(d_idx, d_off, wl.batch)
    s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad, 0.01, 0.0)
    prof = s.profile_read()
    assert prof["small_sort"]["launches"] == 1 and prof["small_update"]["launches"] == 1 and "bwd_pairs" not in prof
    assert s.get_counter(binding.COUNTER_SORTED_IN_FWD_USED) == 1
    # asked for the sorted segments, it lists the runs and updates run by run (long runs whole, in the same launch)
    rm = s.remap(d_idx, d_off, wl.batch)
    s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm)
    s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, grad, 0.01, 0.0, s.new_bwd_out(int(d_idx.numel())))
    prof = s.profile_read()
    assert prof["small_segments"]["launches"] == 1 and prof["seg_rows_long"]["launches"] == 1, prof
    assert "seg_combine" not in prof and "small_update" not in prof and "small_sort" not in prof, prof
    assert s.get_counter(binding.COUNTER_SORTED_IN_FWD_USED) == 2
    s.profile_enable(False)
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


def test_link_calibration_moves_the_granules_it_says():
    """The host-link calibration kernel: sequential reads copy the host buffer, scattered reads fetch whole granules
    of it, writes land whole granules; the arguments are checked."""
    dev = torch.device("cuda:0")
    n_words = 1 << 18                                             # 1 MiB of host memory
    host = binding.PinnedArray((n_words,), np.int32)
    host.np[...] = np.arange(n_words, dtype=np.int32)
    for granule in (64, 128, 512):
        gw = granule // 4
        n_gran = n_words // gw
        d = torch.full((n_words + 7 * gw,), -1, dtype=torch.int32, device=dev)
        binding.calibration_link(host, d, n_gran, granule, scattered=False, to_host=False)
        torch.cuda.synchronize()
        assert np.array_equal(d.cpu().numpy()[:n_words], host.np) and int(d[n_words]) == -1
        # scattered: more granules than the host holds; every fetched granule is a whole, aligned host granule
        n2 = n_gran + 7
        d.fill_(-1)
        binding.calibration_link(host, d, n2, granule, scattered=True, to_host=False, workgroups=7)
        torch.cuda.synchronize()
        got = d.cpu().numpy()[: n2 * gw].reshape(n2, gw)
        assert (got[:, 0] % gw == 0).all() and (np.diff(got, axis=1) == 1).all()
        assert np.unique(got[:, 0]).size > n_gran // 4               # spread over the buffer, not one granule
        # scattered writes: the host buffer ends up holding whole granules of the device buffer
        src = torch.arange(n_gran * gw, dtype=torch.int32, device=dev) + (1 << 24)
        binding.calibration_link(host, src, n_gran, granule, scattered=True, to_host=True)
        torch.cuda.synchronize()
        # (two device granules may land on one host granule, each 16-byte piece then comes from either of them)
        h = host.np.reshape(-1, 4)
        written = h[:, 0] >= (1 << 24)
        assert written.sum() > n_gran // 4 and ((h[written, 0] - (1 << 24)) % 4 == 0).all()
        assert (np.diff(h[written], axis=1) == 1).all()
        piece = np.arange(h.shape[0]) % (gw // 4)                      # a piece keeps its place inside the granule
        assert (((h[written, 0] - (1 << 24)) // 4) % (gw // 4) == piece[written]).all()
        host.np[...] = np.arange(n_words, dtype=np.int32)
    L = binding.lib()
    d = torch.zeros(1024, dtype=torch.int32, device=dev)
    assert L.scars_calibration_link(host.ptr, host.nbytes, d.data_ptr(), 4, 48, 1, 0, 16, None) == binding.ERR_INVALID_ARG
    assert L.scars_calibration_link(None, host.nbytes, d.data_ptr(), 4, 64, 1, 0, 16, None) == binding.ERR_INVALID_ARG
    assert L.scars_calibration_link(host.ptr, host.nbytes, d.data_ptr(), 4, 64, 1, 0, 0, None) == binding.ERR_INVALID_ARG
    host.free()
