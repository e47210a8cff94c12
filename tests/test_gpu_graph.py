"""The three per-batch calls allocate nothing and never wait on the host, so a step can be captured into a HIP
graph and replayed.  Each replay is checked against eager results, with eager work between the replays."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle
from paper_2411_01611_amd import binding, synth
from gpu_harness import GpuCase, assert_close


def test_graph_replay_of_remap_and_forward_matches_eager():
    wl = synth.workload("multi_hot", scale=0.004, batch=333)
    c = GpuCase(wl)
    c.build()
    d_idx, d_off = c.dev_batch()
    rm = c.s.new_remap_out()
    out = torch.zeros(wl.num_bags, wl.dim, device=c.dev)
    # eager reference
    c.s.remap(d_idx, d_off, wl.batch, rm)
    c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm, out)
    torch.cuda.synchronize()
    ref_out, ref_loc, ref_n = out.clone(), rm.loc.clone(), rm.n_hit_miss.clone()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            c.s.remap(d_idx, d_off, wl.batch, rm)
            c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm, out)
    torch.cuda.current_stream().wait_stream(side)
    other = c.sampler.batch(1)
    for rep in range(3):
        out.fill_(-1.0)
        rm.loc.fill_(-7)
        # eager work on another batch between replays (disturbs the shared workspace on purpose)
        o_idx, o_off = other[0].to(c.dev), other[1].to(c.dev)
        rm2 = c.s.remap(o_idx, o_off, wl.batch)
        c.s.embedding_bag_fwd(o_idx, o_off, wl.batch, rm2)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out), f"replay {rep}"
        L = d_idx.numel()
        assert torch.equal(rm.loc[:L], ref_loc[:L]) and torch.equal(rm.n_hit_miss, ref_n)
    assert c.s.sync_status() == 0
    c.close()


@pytest.mark.parametrize("presort,name", [(0, "multi_hot"), (1, "multi_hot"), (1, "host_spill"), (0, "host_spill/small")])
def test_graph_replay_of_a_training_step_matches_oracle(presort, name):
    """presort: remap starts the backward sort on the library's side stream, which joins the capture and is joined
    back by bwd_update before the capture ends; with one index per bag the forward pass also pools the cached bags on
    a stream of its own, forked and joined inside the call.  "/small": the caller states the lookups per table, so the
    forward pass's fetch launch carries the per-table sort and the backward pass finds it done, replay after replay."""
    name, _, small = name.partition("/")
    wl = synth.workload("multi_hot", scale=0.004, batch=333) if name == "multi_hot" else synth.workload("host_spill", scale=0.0005, batch=3000)
    c = GpuCase(wl)
    c.s.set_tuning(binding.TUNE_PRESORT, presort)
    if small:
        c.s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, wl.batch)
    c.build()
    d_idx, d_off = c.dev_batch()
    idx, off = c.batch
    grad = c.sampler.grads(0)
    d_grad = grad.to(c.dev)
    rm = c.s.new_remap_out()
    out = torch.zeros(wl.num_bags, wl.dim, device=c.dev)
    opt = 1 if wl.optimizer == "adagrad" else 0
    lr, eps = np.float32(wl.lr), np.float32(wl.eps if opt else 0.0)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            c.s.remap(d_idx, d_off, wl.batch, rm)
            c.s.embedding_bag_fwd(d_idx, d_off, wl.batch, rm, out)
            c.s.embedding_bag_bwd_update(d_idx, d_off, wl.batch, rm, d_grad, float(lr), float(eps))
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        rc, want = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, idx.numpy(), off.numpy(), wl.batch)
        oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, opt, idx.numpy(), off.numpy(), wl.batch,
                                        grad.numpy(), lr, eps)
        g.replay()
        torch.cuda.synchronize()
        assert_close(out.cpu().numpy(), want, f"forward of replay {rep}")
    c.s.flush_cache()
    assert c.s.sync_status() == 0
    assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows after three replayed steps")
    if opt:
        assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "state after three replayed steps")
    assert c.s.get_counter(binding.COUNTER_PREPARED_USED) == presort     # decided once, at capture time
    assert c.s.get_counter(binding.COUNTER_SORTED_IN_FWD_USED) == (1 if small else 0)
    c.close()


def test_graph_replay_of_two_steps_in_the_look_ahead_order_matches_oracle():
    """remap(next) -> bwd_update_ahead(this, next) -> fwd(next), twice, over two batches that share rows: the fetch on
    the library's third stream joins the capture and is joined back by the forward pass.  Each replay is two training
    steps; the state at the end of the capture is the one at its start, so replays chain."""
    from test_gpu_lookahead import _share_rows
    wl = synth.workload("multi_hot", scale=0.004, batch=333)
    c = GpuCase(wl, max_L=int(wl.num_bags * 20 * 1.6))
    s = c.s
    s.set_tuning(binding.TUNE_LOOKAHEAD, 1)
    c.build()
    b0 = c.sampler.batch(0)
    b1 = _share_rows(wl, b0, c.sampler.batch(1), 0.3, np.random.default_rng(3))
    bs = [b0, b1]
    dev = [(b[0].to(c.dev), b[1].to(c.dev)) for b in bs]
    grads = [c.sampler.grads(0), c.sampler.grads(1)]
    dgr = [g.to(c.dev) for g in grads]
    rms = [s.new_remap_out(), s.new_remap_out()]
    outs = [torch.zeros(wl.num_bags, wl.dim, device=c.dev) for _ in range(2)]
    lr, eps = np.float32(wl.lr), np.float32(wl.eps)
    nL = [int(b[0].numel()) for b in bs]
    s.remap(dev[0][0], dev[0][1], wl.batch, rms[0])
    s.embedding_bag_fwd(dev[0][0], dev[0][1], wl.batch, rms[0], outs[0])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for e in (0, 1):
                n = 1 - e
                s.remap(dev[n][0], dev[n][1], wl.batch, rms[n])
                s.embedding_bag_bwd_update_ahead(dev[e][0], dev[e][1], wl.batch, rms[e], dgr[e], float(lr), float(eps),
                                                 rms[n], dev[n][0], dev[n][1], wl.batch)
                s.embedding_bag_fwd(dev[n][0], dev[n][1], wl.batch, rms[n], outs[n])
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        outs[0].fill_(-1.0)
        outs[1].fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        for e in (0, 1):
            n = 1 - e
            oracle.embedding_bag_bwd_update(wl.rows, c.ora_tables, c.ora_state, 1, bs[e][0].numpy(), bs[e][1].numpy(), wl.batch,
                                            grads[e].numpy(), lr, eps)
            if e == 0:      # outs[1] is still the forward pass of batch 1 after batch 0's update
                rc, want1 = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, bs[1][0].numpy(), bs[1][1].numpy(), wl.batch)
        rc, want0 = oracle.embedding_bag_fwd(wl.rows, c.ora_tables, bs[0][0].numpy(), bs[0][1].numpy(), wl.batch)
        assert_close(outs[1].cpu().numpy(), want1, f"forward of batch 1 in replay {rep}")
        assert_close(outs[0].cpu().numpy(), want0, f"forward of batch 0 in replay {rep}")
    s.flush_cache()
    assert s.sync_status() == 0
    assert_close(c.pinned_rows(), np.concatenate(c.ora_tables), "rows after three replays")
    assert_close(c.pinned_state_rows(), np.concatenate(c.ora_state), "accumulators after three replays")
    c.close()
