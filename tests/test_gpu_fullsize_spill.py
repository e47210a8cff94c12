"""The `host_spill` workload at the size bench.py runs it (a module of its own: its pinned tables do not fit beside the
pinned tables the other full-size tests keep for their module).

The workload asks for 200M rows x 512 B = 102.4 GB of pinned host memory.  The test tries that first; when the box
refuses to pin it, it prints what was refused and steps the rows (and the budget with them) down by 0.05 of the full
size until the tables can be pinned -- the rule bench.py follows -- and says which size it ran."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2411_01611_amd import binding, synth
from test_gpu_fullsize import _full_size_sgd_step


def _pin(wl):
    tabs = []
    try:
        for t in range(wl.num_tables):
            tabs.append(binding.PinnedArray((wl.rows[t], wl.dim), np.float32))
    except binding.ScarsError as e:
        done = sum(p.nbytes for p in tabs)
        for p in tabs:
            p.free()
        return None, f"table {len(tabs)} after {done / 1e9:.1f} GB pinned: {e}"
    return tabs, None


@pytest.mark.timeout(1500)
def test_host_spill_at_the_largest_size_the_box_pins_matches_oracle():
    """26 fp32 tables x dim 128, batch 65536 one-hot, Zipf 1.2, 16 GB cached at the full 200M rows (102.4 GB)."""
    scale = 1.0
    while True:
        wl = synth.workload("host_spill", row_scale=scale)
        tabs, why = _pin(wl)
        if tabs is not None:
            break
        print(f"host_spill: cannot pin {wl.total_rows * wl.row_bytes / 1e9:.1f} GB at row_scale {scale:.2f}: {why}", flush=True)
        assert scale > 0.05 + 1e-9, "not even a twentieth of the workload's tables can be pinned"
        scale = round(scale - 0.05, 2)
    print(f"host_spill: running at row_scale {scale:.2f}: {wl.total_rows} rows, {wl.total_rows * wl.row_bytes / 1e9:.1f} GB pinned, "
          f"budget {wl.budget_bytes / 1e9:.2f} GB", flush=True)
    _full_size_sgd_step(wl, 4, tabs)
