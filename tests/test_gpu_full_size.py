"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.
The oracle evaluates a seeded sample of the selected rows (every output row depends on no
other query, so sampled rows are checked exactly) plus the whole fused K/V cache."""
import numpy as np
import pytest
import torch

from paper_2605_24022_amd import workloads as W
from tests.gpu_util import say
from tests.test_gpu_parity import _check_layer, _run_layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)


@pytest.mark.parametrize("ratio", [15, 5])
def test_layer_config3_sampled_rows(ratio):
    """32768-token context; r = 15 % is the headline point, r = 5 % exercises key-range splits."""
    wl = W.make_workload(W.spec(3, ratio))
    out, kb, vb = _run_layer(wl)
    rows = W.sample_rows(wl.spec.n_sel, 192, seed=ratio)
    say(f"oracle on {len(rows)} sampled rows of {wl.spec.n_sel}")
    _check_layer(wl, out, kb, vb, rows=rows)


def test_layer_config3_full_recompute_equals_full_prefill():
    """r = 100 %: every row is recomputed; the cache pool is poisoned and must not matter."""
    wl = W.make_workload(W.spec(3, 100))
    out, kb, vb = _run_layer(wl)
    rows = W.sample_rows(wl.spec.n_sel, 96, seed=100)
    _check_layer(wl, out, kb, vb, rows=rows)


def test_layer_config4_pinned_host_chunks_clustered_rows():
    """131072-token context streamed from pinned host memory on a second stream, clustered rows."""
    wl = W.make_workload(W.spec(4))
    out, kb, vb = _run_layer(wl, pinned=True)
    rows = W.sample_rows(wl.spec.n_sel, 64, seed=4)
    _check_layer(wl, out, kb, vb, rows=rows)
