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


# ---------------------------------------------------------------- fit under a >= 0, b >= 0

def lib_fit_nonneg(h, g, tau):
    binding.load(build_if_missing=True)
    arr = lambda x: np.ascontiguousarray(x, dtype=np.float64)
    h, g, tau = arr(h), arr(g), arr(tau)
    abc, acc = np.zeros(3), C.c_double(0)
    rc = H.hetis_profiler_fit_nonneg(h, g, tau, len(h), abc, acc)
    return rc, abc, acc.value


def test_checker_nonneg_equals_plain_fit_when_both_slopes_are_positive():
    rng = np.random.default_rng(74)
    h, g = grid()
    tau = 0.004 * h + 1e-4 * g + 9 + rng.normal(0, 1, size=h.shape)
    plain, acc = oracle.profiler_fit(h, g, tau)
    con, acc2 = oracle.profiler_fit_nonneg(h, g, tau)
    assert plain[0] > 0 and plain[1] > 0
    assert np.allclose(con, plain, rtol=1e-7, atol=1e-10) and abs(acc - acc2) < 1e-9


def test_checker_nonneg_by_hand_on_a_balanced_design():
    # tau = -h + 2 g + 5 on the 2 x 2 design: with a held at 0 the regressors stay orthogonal,
    # so b keeps its value and c absorbs the mean of -h: (0, 2, 4.5)
    h = np.array([0.0, 1.0, 0.0, 1.0])
    g = np.array([0.0, 0.0, 1.0, 1.0])
    abc, _ = oracle.profiler_fit_nonneg(h, g, -h + 2 * g + 5)
    assert np.allclose(abc, [0.0, 2.0, 4.5], atol=1e-9)
    # both slopes negative: the mean
    abc, _ = oracle.profiler_fit_nonneg(h, g, -h - 3 * g + 9)
    assert np.allclose(abc, [0.0, 0.0, 7.0], atol=1e-9)


def test_checker_nonneg_satisfies_the_optimality_conditions():
    """At the constrained optimum the gradient of the squared error is zero in every free
    direction and points into the feasible side for a parameter held at its bound."""
    rng = np.random.default_rng(75)
    h, g = grid()
    tau = -6e-4 * h + 8.8e-5 * g + 27 + rng.normal(0, 2, size=h.shape)
    assert oracle.profiler_fit(h, g, tau)[0][0] < 0
    abc, _ = oracle.profiler_fit_nonneg(h, g, tau)
    assert abc[0] == 0.0 and abc[1] > 0
    res = abc[0] * h + abc[1] * g + abc[2] - tau
    scale = np.linalg.norm(res)
    assert abs(res @ g) <= 1e-8 * np.linalg.norm(g) * scale and abs(res.sum()) <= 1e-8 * 8 * scale
    assert res @ h >= 0          # raising a from 0 would raise the error


@pytest.mark.parametrize("a_true,b_true", [(3e-3, 9e-5), (-6e-4, 8.8e-5), (2e-3, -1e-6), (-1e-3, -1e-6)])
def test_library_nonneg_fit_matches_checker(a_true, b_true):
    rng = np.random.default_rng(76)
    h, g = grid()
    tau = a_true * h + b_true * g + 30 + rng.normal(0, 0.5, size=h.shape)
    rc, abc, acc = lib_fit_nonneg(h, g, tau)
    ref, ref_acc = oracle.profiler_fit_nonneg(h, g, tau)
    assert rc == 0 and abc[0] >= 0 and abc[1] >= 0
    assert np.allclose(abc, ref, rtol=1e-6, atol=1e-9)
    assert abs(acc - ref_acc) < 1e-8
    assert (abc[0] == 0) == (a_true < 0) and (abc[1] == 0) == (b_true < 0)
