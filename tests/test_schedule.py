"""Ratio scheduler (Sec. 4.3): the C-ABI host functions against the oracle, probe by probe.
Host code on both sides, so these run without a GPU."""
import math

import numpy as np
import pytest

from oracle import ct_oracle as O
from paper_2605_24022_amd import binding as B


def test_latency_model_and_prior_match_the_oracle():
    rng = np.random.default_rng(11)
    for _ in range(200):
        r, n = rng.uniform(0, 1), float(rng.integers(1, 1 << 18))
        t_c, t_i, t_o = rng.uniform(1e-4, 1e-2), rng.uniform(1e-5, 1e-2), rng.uniform(0, 1)
        assert B.ct_layer_latency_model(r, n, t_c, t_i, t_o) == pytest.approx(
            O.layer_latency_model(r, n, t_c, t_i, t_o), rel=1e-14)
        lo = rng.uniform(0, 0.5)
        hi = rng.uniform(lo, 1.0)
        assert B.ct_ratio_prior(t_c, t_i, lo, hi) == pytest.approx(O.ratio_prior(t_c, t_i, lo, hi), rel=1e-14)
    assert B.ct_ratio_prior(0.0, 0.0, 0.15, 0.6) == O.ratio_prior(0.0, 0.0, 0.15, 0.6) == 0.15


@pytest.mark.parametrize("seed", range(4))
def test_search_visits_the_oracles_probes(seed):
    rng = np.random.default_rng(100 + seed)
    for case in range(60):
        r_min = rng.uniform(0.0, 0.4)
        r_max = rng.uniform(r_min + 0.05, 1.0)
        m = rng.uniform(r_min - 0.1, r_max + 0.1)      # minimisers outside the bracket as well
        eps = 10.0 ** rng.uniform(-5, -1)
        shape = case % 4
        t_c, t_i = rng.uniform(1e-4, 1e-3), rng.uniform(1e-5, 1e-3)
        f = [lambda r: (r - m) ** 2,
             lambda r: abs(r - m) ** 0.5,
             lambda r: (m - r) * 3.0 if r < m else (r - m) * 0.2,
             lambda r: O.layer_latency_model(r, 32768, t_c, t_i, 0.05)][shape]
        r0 = [r_min, r_max, m, rng.uniform(r_min, r_max), O.ratio_prior(t_c, t_i, r_min, r_max)][case % 5]
        want, probes = O.ratio_search(f, r0, r_min, r_max, eps)
        seen = []
        got, n = B.ct_ratio_search(lambda r: seen.append(r) or f(r), r0, r_min, r_max, eps)
        assert n == len(probes) == len(seen)
        np.testing.assert_allclose(seen, probes, rtol=0, atol=1e-13)
        assert got == pytest.approx(want, abs=1e-13)


def test_search_limits_and_errors():
    f = lambda r: (r - 0.3) ** 2
    got, n = B.ct_ratio_search(f, 0.3, 0.1, 0.9, 1e-6, max_evals=5)
    want, probes = O.ratio_search(f, 0.3, 0.1, 0.9, 1e-6, max_evals=5)
    assert n == 5 == len(probes) and got == pytest.approx(want, abs=1e-13)
    assert B.ct_ratio_search(f, 0.2, 0.2, 0.2, 1e-3) == (0.2, 0)
    for args, code in (((0.3, 0.6, 0.5, 1e-3), B.CT_ERR_RATIO), ((0.3, -0.1, 0.5, 1e-3), B.CT_ERR_RATIO),
                       ((0.3, 0.1, 1.5, 1e-3), B.CT_ERR_RATIO), ((0.3, 0.1, 0.5, 0.0), B.CT_ERR_SHAPE)):
        with pytest.raises(B.CacheTuneError) as e:
            B.ct_ratio_search(f, *args)
        assert e.value.status == code
    with pytest.raises(B.CacheTuneError) as e:
        B.ct_ratio_search(f, 0.3, 0.1, 0.5, 1e-3, max_evals=1)
    assert e.value.status == B.CT_ERR_SHAPE
    lib = B.load()
    assert lib.ct_ratio_search(B.TTFT_FN(), None, 0.3, 0.1, 0.5, 1e-3, 10, None, None) == B.CT_ERR_NULL
