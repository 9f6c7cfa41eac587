"""The entry point that allocates nothing (qsr_clip_factors_static: partial sums in an array inside
the library's device image) against the entry point it is a variant of (qsr_clip_factors, workspace
brought in by the caller): same bits, on two calls in a row, the second with a smaller input, so that
what the first call left in the shared array is there when the second runs."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _pair(K, P, seed):
    import torch
    rng = np.random.default_rng(seed)
    scale = rng.choice([0.02, 2.0, 60.0], size=(K, 1)) / np.sqrt(P)
    return torch.from_numpy((rng.standard_normal((K, P)) * scale).astype(np.float32)).cuda()


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    import paper_2310_14423_amd as qsr
    first = _pair(16, 3_000_000 + 4, 1)       # 184 partial sums per row
    second = _pair(3, 4099, 2)                # smaller in both K and P, rows not 16-byte aligned
    coef = torch.full((64,), -1.0, device="cuda")
    norm = torch.full((64,), -1.0, device="cuda")
    for g in (first, second, first):
        K = g.shape[0]
        want_coef, want_norm = qsr.clip_factors(g, 2.0)
        coef.fill_(-1.0); norm.fill_(-1.0)
        qsr.clip_factors_static(g, 2.0, coef, norm)
        assert torch.equal(coef[:K], want_coef) and torch.equal(norm[:K], want_norm)
        assert bool((coef[K:] == -1.0).all()) and bool((norm[K:] == -1.0).all())
        assert float(norm[:K].min()) > 0.0 and 0.0 < float(coef[:K].min()) <= 1.0


def test_static_scratch_entry_point_limits():
    import torch
    import paper_2310_14423_amd as qsr
    g = torch.zeros((65, 8), device="cuda")
    out = torch.zeros(65, device="cuda")
    with pytest.raises(qsr.QSRError) as e:
        qsr.clip_factors_static(g, 1.0, out, out.clone())
    assert e.value.code == -7
    g64 = _pair(64, 20_000_000, 3)            # the largest case: 64 rows x 1024 partial sums fill the array
    coef = torch.empty(64, device="cuda"); norm = torch.empty(64, device="cuda")
    qsr.clip_factors_static(g64, 2.0, coef, norm)
    want_coef, want_norm = qsr.clip_factors(g64, 2.0)
    assert torch.equal(coef, want_coef) and torch.equal(norm, want_norm)
