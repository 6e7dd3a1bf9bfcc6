"""CPU tests of the latency-model tooling (App. A of the paper): the oracle's regressors and fit
against closed forms and a textbook special case, then the package's host code against the oracle."""
import numpy as np
import pytest

from oracle import latency_model_oracle as orc
from paper_2401_09670_amd import latency_model as lm

H, M = 5120, 20480


# ---------------- oracle pins ----------------
def test_oracle_prefill_regressors_equal_lengths_closed_form():
    # B equal prompts of length l: t = B l, t2 = B l^2 (App. A.1)
    B, l, b = 4, 512, 16
    r = orc.prefill_regressors([l] * B, H, M, b)
    t, t2 = B * l, B * l * l
    assert r[0] == 4 * t * H * H + 2 * t * H * M
    assert r[1] == 3 * H * t2 / b
    assert r[2] == 1.0
    # hand-computed: 4*2048*5120^2 + 2*2048*5120*20480 = 644245094400 ; 3*5120*1048576/16 = 1006632960
    assert r[0] == 644245094400.0 and r[1] == 1006632960.0


def test_oracle_prefill_regressors_depend_on_squares():
    a = orc.prefill_regressors([1000, 24], H, M, 32)
    b = orc.prefill_regressors([512, 512], H, M, 32)
    assert a[0] == b[0]            # same token count, same GEMM work
    assert a[1] > b[1]             # more skewed lengths, more attention work
    assert a[1] == 3 * H * (1000 ** 2 + 24 ** 2) / 32


def test_oracle_decode_regressors():
    r = orc.decode_regressors([100, 200, 300], H, M)
    assert r[0] == 4 * H * H + 2 * H * M == 314572800
    assert r[1] == 3 * H * 600


def test_oracle_fit_recovers_planted_constants():
    rng = np.random.default_rng(0)
    rows = [orc.prefill_regressors(rng.integers(1, 2048, size=rng.integers(1, 9)), H, M, 64) for _ in range(40)]
    c_true = np.array([1.7e-15, 3.1e-13, 2.5e-5])
    t = orc.predict(rows, c_true)
    c = orc.fit(rows, t)
    assert np.allclose(c, c_true, rtol=1e-6)


def test_oracle_fit_is_simple_linear_regression_for_decode():
    # The first decoding regressor is a constant, so the fit is the textbook line through (x, y):
    # slope = cov(x, y) / var(x), intercept = mean(y) - slope mean(x), and C4 = intercept / constant.
    rng = np.random.default_rng(1)
    tot = rng.integers(64, 200000, size=30).astype(np.float64)
    rows = [orc.decode_regressors([t], H, M) for t in tot]
    y = 4e-5 + 2.0e-14 * 3 * H * tot + rng.normal(0, 1e-6, size=30)
    c = orc.fit(rows, y)
    x = 3 * H * tot
    slope = ((x - x.mean()) * (y - y.mean())).sum() / ((x - x.mean()) ** 2).sum()
    icpt = y.mean() - slope * x.mean()
    assert np.isclose(c[1], slope, rtol=1e-8)
    assert np.isclose(c[0] * rows[0][0], icpt, rtol=1e-8)


def test_oracle_fit_residual_is_orthogonal_to_regressors():
    rng = np.random.default_rng(2)
    rows = np.array([orc.prefill_regressors(rng.integers(1, 1024, size=4), H, M, 64) for _ in range(25)])
    y = rng.uniform(1e-4, 1e-2, size=25)
    c = orc.fit(rows, y)
    resid = rows @ c - y
    scaled = rows / np.linalg.norm(rows, axis=0)
    assert np.abs(scaled.T @ resid).max() < 1e-9 * np.linalg.norm(y)


# ---------------- package host code against the oracle ----------------
def test_features_match_oracle():
    rng = np.random.default_rng(3)
    for _ in range(20):
        lens = rng.integers(1, 4096, size=rng.integers(1, 17)).tolist()
        b = int(rng.choice([16, 32, 64]))
        assert np.allclose(lm.prefill_features(lens, H, M, b), orc.prefill_regressors(lens, H, M, b), rtol=1e-13)
        assert np.allclose(lm.decode_features(lens, H, M), orc.decode_regressors(lens, H, M), rtol=1e-13)


def test_fit_matches_oracle_on_noisy_data():
    rng = np.random.default_rng(4)
    rows = [orc.prefill_regressors(rng.integers(1, 2048, size=rng.integers(1, 9)), H, M, 64) for _ in range(50)]
    y = orc.predict(rows, [1.6e-15, 2.0e-13, 3e-5]) * rng.normal(1.0, 0.03, size=50)
    assert np.allclose(lm.fit_least_squares(rows, y), orc.fit(rows, y), rtol=1e-7)
    rows = [orc.decode_regressors(rng.integers(1, 2048, size=rng.integers(1, 257)), H, M) for _ in range(50)]
    y = orc.predict(rows, [1.2e-13, 2.5e-14]) * rng.normal(1.0, 0.03, size=50)
    assert np.allclose(lm.fit_least_squares(rows, y), orc.fit(rows, y), rtol=1e-7)
    res = lm.relative_residuals(rows, y, lm.fit_least_squares(rows, y))
    assert np.allclose(res, (orc.predict(rows, orc.fit(rows, y)) - y) / y, atol=1e-9)


def test_fit_rejects_bad_input():
    with pytest.raises(ValueError):
        lm.fit_least_squares([[1.0, 2.0, 3.0]], [1.0])          # fewer measurements than coefficients
    with pytest.raises(ValueError):
        lm.fit_least_squares([[1.0, 0.0], [2.0, 0.0], [3.0, 0.0]], [1.0, 2.0, 3.0])  # a zero regressor


def test_saturation_length():
    lengths = [16, 32, 64, 128, 256, 512, 1024]
    rate = [10, 20, 40, 75, 92, 99, 100]
    assert lm.saturation_length(lengths, rate) == 256
    assert lm.saturation_length(lengths, rate, frac=0.95) == 512
    assert lm.saturation_length(lengths[::-1], rate[::-1]) == 256   # order of the sweep does not matter
