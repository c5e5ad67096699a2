"""Pins of oracle/rse_oracle.py (the influence metric of Sec. 3.4.1) against things other than itself."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import rse_oracle as R

HERE = os.path.dirname(os.path.abspath(__file__))


def golden_cases():
    for line in open(os.path.join(HERE, "golden", "rse_hand_values.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        shape, yo, ym, want = (p.strip() for p in line.split("|"))
        n, d = (int(x) for x in shape.split())
        yield (n, d, np.array([float(x) for x in yo.split()]), np.array([float(x) for x in ym.split()]),
               Fraction(want))


def test_hand_worked_values():
    cases = list(golden_cases())
    assert len(cases) >= 6
    for n, d, yo, ym, want in cases:
        got = R.head_rse(ym.reshape(1, 1, n, d), yo.reshape(1, 1, n, d))
        assert got.shape == (1,)
        assert abs(got[0] - float(want)) <= 1e-15 * max(1.0, float(want)), (yo, ym, got, want)


def rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def test_equals_one_minus_r2_of_a_library():
    # the metric is 1 - R^2 (coefficient of determination) of y_m as a prediction of y_o
    from sklearn.metrics import r2_score
    yo, ym = rand((2, 3, 17, 8), 1) + 0.7, rand((2, 3, 17, 8), 2)
    got = R.head_rse(ym, yo)
    for h in range(3):
        want = 1.0 - r2_score(yo[:, h].reshape(-1), ym[:, h].reshape(-1))
        assert abs(got[h] - want) <= 1e-12 * abs(want)


def test_perfect_method_scores_zero_and_the_mean_scores_one():
    yo = rand((1, 4, 33, 16), 3) * 2.0 + 5.0
    assert np.all(R.head_rse(yo.copy(), yo) == 0.0)
    ym = np.empty_like(yo)
    for h in range(4):
        ym[:, h] = yo[:, h].mean()
    np.testing.assert_allclose(R.head_rse(ym, yo), 1.0, rtol=1e-12)


def test_error_is_against_the_original_not_against_its_mean():
    # the reading of Eq. 1: with the mean in the numerator, y_m = y_o would score 1
    yo = rand((1, 1, 8, 4), 4)
    assert R.head_rse(yo, yo)[0] == 0.0


def test_invariances():
    yo, ym = rand((2, 2, 19, 8), 5), rand((2, 2, 19, 8), 6)
    base = R.head_rse(ym, yo)
    np.testing.assert_allclose(R.head_rse(3.5 * ym, 3.5 * yo), base, rtol=1e-12)          # common scale
    np.testing.assert_allclose(R.head_rse(ym + 11.0, yo + 11.0), base, rtol=1e-10)        # common shift
    np.testing.assert_allclose(R.head_rse(-ym, -yo), base, rtol=1e-12)                    # sign
    # the error term is quadratic in the error: doubling the error quadruples the metric
    np.testing.assert_allclose(R.head_rse(yo + 2.0 * (ym - yo), yo), 4.0 * base, rtol=1e-12)


def test_heads_are_independent_and_the_batch_is_pooled():
    yo, ym = rand((2, 3, 11, 4), 7), rand((2, 3, 11, 4), 8)
    base = R.head_rse(ym, yo)
    ym2 = ym.copy()
    ym2[:, 1] += 1.0                       # touching head 1 changes head 1 only
    got = R.head_rse(ym2, yo)
    assert got[0] == base[0] and got[2] == base[2] and got[1] != base[1]
    # pooling: a head's batch entries are one population (B,N) -> (1, B*N)
    pooled = R.head_rse(ym.transpose(1, 0, 2, 3).reshape(1, 3, 22, 4), yo.transpose(1, 0, 2, 3).reshape(1, 3, 22, 4))
    np.testing.assert_allclose(pooled, base, rtol=1e-12)
    # and a permutation of a head's elements, applied to both tensors, changes nothing
    perm = np.random.Generator(np.random.PCG64(9)).permutation(11)
    np.testing.assert_allclose(R.head_rse(ym[:, :, perm], yo[:, :, perm]), base, rtol=1e-12)


def test_large_common_offset_does_not_disturb_it():
    # two-pass mean: spread of y_o is computed about the mean, not as E[y^2] - E[y]^2
    yo, ym = rand((1, 1, 64, 32), 10), rand((1, 1, 64, 32), 11)
    base = R.head_rse(ym, yo)
    np.testing.assert_allclose(R.head_rse(ym + 1.0e6, yo + 1.0e6), base, rtol=1e-8)


def test_accepts_bf16_torch_tensors_exactly():
    import torch
    yo = torch.randn(1, 2, 9, 8, generator=torch.Generator().manual_seed(0)).to(torch.bfloat16)
    ym = torch.randn(1, 2, 9, 8, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16)
    got = R.head_rse(ym, yo)
    want = R.head_rse(ym.double().numpy(), yo.double().numpy())
    assert np.array_equal(got, want)
