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


if __name__ == "__main__":
    main()
