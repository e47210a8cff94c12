"""A complete use of the library on a small problem: `python -m paper_2411_01611_amd.example` (needs an MI355X).

Two tables in pinned host memory, a profile stream to rank the rows (Section III), a cache budget (Section IV),
then one training step of the embedding layer: remap, pooled forward, backward with the SGD update.  The forward
result is compared with a plain torch sum over the same rows, so the script doubles as an installation check.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding


def main(seed: int = 0) -> float:
    rng = np.random.default_rng(seed)
    rows, D, B = [5000, 300], 32, 512                     # two tables, 32 fp32 columns, 512 samples per batch
    T = len(rows)

    # the tables live in pinned host memory the caller owns
    tables = [binding.PinnedArray((n, D), np.float32) for n in rows]
    for t in tables:
        t.np[...] = rng.uniform(-0.01, 0.01, t.shape).astype(np.float32)
    s = binding.Scars(rows, D, binding.DTYPE_F32, [t.ptr for t in tables], binding.OPT_SGD)

    def batch():
        """Jagged, table-major: bag g = t * B + b; skewed ids so that a small cache catches most lookups."""
        lens = rng.integers(0, 6, T * B)
        off = np.zeros(T * B + 1, dtype=np.int32)
        off[1:] = np.cumsum(lens)
        idx = np.concatenate([np.minimum((rng.pareto(1.2, int(off[(t + 1) * B] - off[t * B])) * 20).astype(np.int64),
                                         rows[t] - 1) for t in range(T)]).astype(np.int32)
        return torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()

    budget = 400 * D * 4                                  # room for 400 rows on the device
    s.bind_buffers(budget, max_L=T * B * 5, max_G=T * B)  # allocates what scars_query_sizes asks for and binds it
    # optional: bags hold at most 5 lookups here, so no table gets more than 5 B per batch; stated, the backward pass
    # of so small a batch sorts each table's lookups in LDS instead of by radix passes over the whole batch
    s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, 5 * B)
    p_idx, p_off = batch()
    s.build_cache(p_idx, p_off, B, budget)                # histogram of the profile stream, top-k, cache fill

    idx, off = batch()
    rm = s.remap(idx, off, B)                             # index -> cache slot, ordered hit / miss lists
    n_hit, n_miss = rm.n_hit_miss.tolist()
    out = s.embedding_bag_fwd(idx, off, B, rm)            # [T * B, D] pooled sums, hits from HBM, misses over the link

    # the same sums with plain torch on the host copies of the tables
    base = np.concatenate([[0], np.cumsum(rows)])[:-1]
    off_c, idx_c = off.cpu().numpy(), idx.cpu().numpy().astype(np.int64)
    bag = np.repeat(np.arange(T * B), np.diff(off_c))
    gid = idx_c + base[bag // B]
    all_rows = torch.from_numpy(np.concatenate([t.np for t in tables]))
    want = torch.zeros(T * B, D).index_add_(0, torch.from_numpy(bag), all_rows[torch.from_numpy(gid)])
    err = float((out.cpu() - want).abs().max())

    grad = torch.randn(T * B, D, device="cuda")
    s.embedding_bag_bwd_update(idx, off, B, rm, grad, lr=0.01)   # sorted segments, summed gradients, rows updated
    s.flush_cache()                                       # cached rows back to the host tables
    status = s.sync_status()
    print(f"cached rows {s.cache_rows()}, lookups {idx.numel()}: {n_hit} hits, {n_miss} misses; "
          f"forward max |difference| from torch {err:.2e}; status {status}")
    s.close()
    for t in tables:
        t.free()
    assert status == 0 and err < 1e-5
    return err


def lookahead_loop(seed: int = 1, steps: int = 4) -> float:
    """A training loop that knows its next batch: remap(next) -> bwd_update_ahead(this, next) -> fwd(next), so that the
    next batch's cold rows cross the host link while this batch's updated rows go back.  The tables after the loop are
    compared with plain torch SGD applied batch after batch."""
    rng = np.random.default_rng(seed)
    rows, D, B, lr = [4000, 700], 32, 256, 0.05
    T = len(rows)
    tables = [binding.PinnedArray((n, D), np.float32) for n in rows]
    for t in tables:
        t.np[...] = rng.uniform(-0.01, 0.01, t.shape).astype(np.float32)
    ref = torch.from_numpy(np.concatenate([t.np for t in tables])).double()
    base = np.concatenate([[0], np.cumsum(rows)])[:-1]
    s = binding.Scars(rows, D, binding.DTYPE_F32, [t.ptr for t in tables], binding.OPT_SGD)
    s.set_tuning(binding.TUNE_LOOKAHEAD, 1)
    s.set_tuning(binding.TUNE_MAX_TABLE_LOOKUPS, 4 * B)    # (bags of at most 4 lookups: see main)

    def batch():
        lens = rng.integers(0, 5, T * B)
        off = np.zeros(T * B + 1, dtype=np.int32)
        off[1:] = np.cumsum(lens)
        idx = np.concatenate([np.minimum((rng.pareto(1.1, int(off[(t + 1) * B] - off[t * B])) * 30).astype(np.int64),
                                         rows[t] - 1) for t in range(T)]).astype(np.int32)
        return torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()

    budget = 200 * D * 4
    s.bind_buffers(budget, max_L=T * B * 4, max_G=T * B)
    s.build_cache(*batch(), B, budget)
    batches = [batch() for _ in range(steps + 1)]
    grads = [torch.randn(T * B, D, device="cuda") for _ in range(steps)]
    rms = [s.new_remap_out(), s.new_remap_out()]           # two sets of remap outputs: this batch's and the next one's
    s.remap(*batches[0], B, rms[0])
    s.embedding_bag_fwd(*batches[0], B, rms[0])
    for e in range(steps):
        (idx, off), (nidx, noff) = batches[e], batches[e + 1]
        s.remap(nidx, noff, B, rms[(e + 1) % 2])
        s.embedding_bag_bwd_update_ahead(idx, off, B, rms[e % 2], grads[e], lr, 0.0, rms[(e + 1) % 2], nidx, noff, B)
        s.embedding_bag_fwd(nidx, noff, B, rms[(e + 1) % 2])
        # the same step in plain torch: every lookup of a row adds its bag's gradient, one SGD step per row
        off_c, idx_c = off.cpu().numpy(), idx.cpu().numpy().astype(np.int64)
        bag = np.repeat(np.arange(T * B), np.diff(off_c))
        gid = torch.from_numpy(idx_c + base[bag // B])
        dw = torch.zeros_like(ref).index_add_(0, gid, grads[e].cpu().double()[torch.from_numpy(bag)])
        ref -= lr * dw
    s.flush_cache()
    status = s.sync_status()
    got = torch.from_numpy(np.concatenate([t.np for t in tables])).double()
    err = float((got - ref).abs().max())
    print(f"look-ahead loop of {steps} steps: {s.get_counter(binding.COUNTER_AHEAD_USED)} forward passes found their rows "
          f"fetched ahead; max |difference| of the tables from plain torch SGD {err:.2e}; status {status}")
    s.close()
    for t in tables:
        t.free()
    assert status == 0 and err < 1e-6
    return err


if __name__ == "__main__":
    main()
    lookahead_loop()
