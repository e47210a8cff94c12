"""The `host_spill` workload at the size bench.py runs it (a module of its own: its 51 GB of pinned tables do not fit
beside the pinned tables the other full-size tests keep for their module)."""
import pytest

pytestmark = pytest.mark.gpu

from paper_2411_01611_amd import synth
from test_gpu_fullsize import _full_size_sgd_step


@pytest.mark.timeout(1200)
def test_half_size_host_spill_matches_oracle():
    """26 fp32 tables, 100M rows x dim 128 (half the workload's rows, 51 GB: what one process can pin on these boxes),
    batch 65536 one-hot, Zipf 1.2, 8 GB cached -- the size bench.py runs it at."""
    _full_size_sgd_step(synth.workload("host_spill", row_scale=0.5), 4)
