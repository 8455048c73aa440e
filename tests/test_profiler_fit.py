"""The Profiler's linear model of Attention time (Section 5.1, Eq. (3)): pins of the checker's
fit, and the library's fit (host C ABI) against the checker.  No GPU needed."""
import ctypes as C

import numpy as np
import pytest

import oracle
import paper_2509_08309_amd as H
from paper_2509_08309_amd import binding


def grid(nh=8, ng=8):
    h = np.array([64, 128, 256, 512, 768, 1024, 1536, 2048][:nh], dtype=np.float64)
    g = np.array([32, 64, 128, 256, 512, 1024, 1536, 2048][:ng], dtype=np.float64) * 1024
    hh, gg = np.meshgrid(h, g, indexing="ij")
    return hh.ravel(), gg.ravel()


# ---------------------------------------------------------------- pins of the checker

def test_checker_recovers_exact_coefficients():
    h, g = grid()
    a, b, c = 3.25e-3, 9.5e-5, 7.0
    abc, acc = oracle.profiler_fit(h, g, a * h + b * g + c)
    assert np.allclose(abc, [a, b, c], rtol=1e-9, atol=1e-12) and abs(acc - 1.0) < 1e-12


def test_checker_three_points_by_cramers_rule():
    h = np.array([1.0, 2.0, 4.0])
    g = np.array([10.0, 5.0, 7.0])
    tau = np.array([3.0, 8.0, 6.0])
    M = np.stack([h, g, np.ones(3)], axis=1)
    det = np.linalg.det(M)
    by_hand = []
    for k in range(3):
        Mk = M.copy()
        Mk[:, k] = tau
        by_hand.append(np.linalg.det(Mk) / det)
    abc, acc = oracle.profiler_fit(h, g, tau)
    assert np.allclose(abc, by_hand, rtol=1e-10) and abs(acc - 1.0) < 1e-10


def test_checker_residual_is_orthogonal_to_the_regressors():
    rng = np.random.default_rng(71)
    h, g = grid()
    tau = 0.004 * h + 1e-4 * g + 9 + rng.normal(0, 3, size=h.shape)
    abc, acc = oracle.profiler_fit(h, g, tau)
    res = abc[0] * h + abc[1] * g + abc[2] - tau
    # normal equations; the bound is relative to |regressor| * |residual|
    for col in (h, g, np.ones_like(h)):
        assert abs(res @ col) <= 1e-9 * np.linalg.norm(col) * np.linalg.norm(res)
    # any other coefficient vector has a larger squared error
    base = res @ res
    for d in np.eye(3):
        for eps in (1e-4, -1e-4):
            other = abc * (1 + eps * d)
            r2 = other[0] * h + other[1] * g + other[2] - tau
            assert r2 @ r2 >= base
    assert 0.5 < acc < 1.0


def test_checker_accuracy_formula_by_hand():
    # a = 0, b = 0 by symmetry of the sample; predictions are the mean of tau
    h = np.array([0.0, 1.0, 0.0, 1.0])
    g = np.array([0.0, 0.0, 1.0, 1.0])
    tau = np.array([10.0, 20.0, 20.0, 10.0])
    abc, acc = oracle.profiler_fit(h, g, tau)
    assert np.allclose(abc, [0.0, 0.0, 15.0], atol=1e-12)
    assert abs(acc - (1 - np.mean([5 / 10, 5 / 20, 5 / 20, 5 / 10]))) < 1e-12


def test_checker_rejects_degenerate_samples():
    with pytest.raises(ValueError):
        oracle.profiler_fit([1, 2, 3, 4], [2, 4, 6, 8], [1, 2, 3, 5])      # g = 2h


# ---------------------------------------------------------------- library against the checker

def lib_fit(h, g, tau, want_acc=True):
    lib = binding.load(build_if_missing=True)
    arr = lambda x: np.ascontiguousarray(x, dtype=np.float64)
    h, g, tau = arr(h), arr(g), arr(tau)
    abc = np.zeros(3)
    acc = C.c_double(0)
    rc = H.hetis_profiler_fit(h, g, tau, len(h), abc, acc if want_acc else None)
    return rc, abc, acc.value


@pytest.mark.parametrize("noise", [0.0, 0.5, 5.0])
def test_library_fit_matches_checker(noise):
    rng = np.random.default_rng(72)
    h, g = grid()
    tau = 0.0031 * h + 9.1e-5 * g + 6.5 + rng.normal(0, noise, size=h.shape)
    rc, abc, acc = lib_fit(h, g, tau)
    ref, ref_acc = oracle.profiler_fit(h, g, tau)
    assert rc == 0
    assert np.allclose(abc, ref, rtol=1e-8, atol=1e-10)
    assert abs(acc - ref_acc) < 1e-10
    pred = np.zeros_like(h)
    assert H.hetis_profiler_predict(abc, h, g, len(h), pred) == 0
    assert np.allclose(pred, abc[0] * h + abc[1] * g + abc[2], rtol=1e-15)


def test_library_fit_irregular_samples_and_no_accuracy_pointer():
    rng = np.random.default_rng(73)
    h = rng.integers(1, 3000, size=37).astype(np.float64)
    g = rng.integers(1000, 3_000_000, size=37).astype(np.float64)
    tau = 0.002 * h + 1.2e-4 * g + 4 + rng.normal(0, 1, size=37)
    rc, abc, _ = lib_fit(h, g, tau, want_acc=False)
    ref, _ = oracle.profiler_fit(h, g, tau)
    assert rc == 0 and np.allclose(abc, ref, rtol=1e-8, atol=1e-10)


def test_library_fit_errors():
    h, g = grid(3, 3)
    tau = h + g
    assert lib_fit(h[:2], g[:2], tau[:2])[0] == binding.HETIS_ERR_BAD_SHAPE          # n < 3
    assert lib_fit(h, 2 * h, tau)[0] == binding.HETIS_ERR_BAD_SHAPE                   # dependent
    assert lib_fit(np.full(9, 5.0), g, tau)[0] == binding.HETIS_ERR_BAD_SHAPE         # all h equal
    bad = tau.copy()
    bad[4] = 0.0
    assert lib_fit(h, g, bad)[0] == binding.HETIS_ERR_BAD_SHAPE                       # tau <= 0
    bad[4] = np.nan
    assert lib_fit(h, g, bad)[0] == binding.HETIS_ERR_BAD_SHAPE
    lib = binding.load()
    assert lib.hetis_profiler_fit(None, None, None, 9, None, None) == binding.HETIS_ERR_NULL
    assert H.hetis_profiler_predict(np.zeros(3), None, None, 0, None) == 0
    assert H.hetis_profiler_predict(np.zeros(3), None, None, 4, None) == binding.HETIS_ERR_NULL
