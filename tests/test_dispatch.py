"""The Dispatcher's head-wise division (Section 5.2.2, Eq. (7)): pins of the checker, then the
library's solver (host C ABI) against the checker.  No GPU needed."""
import itertools

import numpy as np
import pytest

from oracle import dispatch_oracle as DO


def dev(a=0.001, b=1e-4, c=10.0, h=0.0, g=0.0, capacity=1e9, primary=True, gamma=0.0, beta=0.0):
    return dict(a=a, b=b, c=c, h=h, g=g, capacity=capacity, primary=primary, gamma=gamma, beta=beta)


# ---------------------------------------------------------------- pins of the checker

def test_single_device_takes_everything():
    d = [dev(h=100, g=5000)]
    l = [300, 50]
    z, x, xh, zr = DO.dispatch(d, l, 32, 1)
    want = 0.001 * (100 + 64) + 1e-4 * (5000 + 2 * (300 + 50) * 32) + 10
    assert abs(z - want) < 1e-9 and abs(zr - want) < 1e-9
    assert np.array_equal(xh, [[32], [32]])


def test_identical_idle_devices_split_evenly():
    N, H, r = 4, 32, 1
    d = [dev() for _ in range(N)]
    l = [1000.0]
    z, x, xh, zr = DO.dispatch(d, l, H, r)
    want = 0.001 * H / N + 1e-4 * 2 * 1000 * H / N + 10
    assert abs(z - want) < 1e-9
    assert np.array_equal(xh, [[8, 8, 8, 8]]) and abs(zr - want) < 1e-9


def test_two_devices_equalise_their_times():
    """One request, ample capacity: the optimum puts both devices at the same time; solved by
    hand from K1 + s1 x = K2 + s2 (H - x)."""
    d = [dev(b=1e-4, c=5.0, h=50, g=2e5), dev(b=3e-4, c=8.0, h=10, g=1e4)]
    H, r, l = 64, 1, 2000.0
    A, b, K, _ = DO.device_terms(d, r)
    s = A + b * 2 * l
    x1 = (K[1] - K[0] + s[1] * H) / (s[0] + s[1])
    assert 0 < x1 < H
    z, x, xh, zr = DO.dispatch(d, [l], H, r)
    assert abs(z - (K[0] + s[0] * x1)) < 1e-8
    assert abs(x[0, 0] - x1) < 1e-6
    assert xh.sum() == H and zr >= z - 1e-12
    # rounding moved at most one head: the rounded time is within one head's cost
    assert zr - z <= s.max() + 1e-9


def test_attention_worker_pays_for_the_transfer():
    """Same device parameters, one is an Attention worker with a link cost: it gets fewer heads."""
    d = [dev(primary=True), dev(primary=False, gamma=0.01, beta=3.0)]
    z, x, xh, zr = DO.dispatch(d, [500.0], 40, 1)
    assert x[0, 0] > x[0, 1]
    A, b, K, _ = DO.device_terms(d, 1)
    assert abs(A[1] - (0.001 + 4 * 0.01)) < 1e-15 and abs(K[1] - 13.0) < 1e-12


def test_capacity_binds_and_infeasible():
    # device 0 is much faster but can hold only 1/4 of the request
    l, H, r = 1000.0, 32, 1
    d = [dev(b=1e-5, capacity=2 * l * 8), dev(b=1e-3)]
    z, x, xh, zr = DO.dispatch(d, [l], H, r)
    assert abs(x[0, 0] - 8) < 1e-7 and np.array_equal(xh, [[8, 24]])
    # existing cache counts against the capacity
    d[0]["g"] = 2 * l * 4
    z2, x2, _, _ = DO.dispatch(d, [l], H, r)
    assert abs(x2[0, 0] - 4) < 1e-7 and z2 > z
    # nothing fits
    assert DO.dispatch([dev(capacity=10.0), dev(capacity=10.0)], [l], H, r) is None


def test_groups_of_r_and_brute_force_on_a_tiny_instance():
    """r = 4, two requests, two devices: the rounded division is whole groups; the LP value is
    a lower bound of, and close to, the best whole-group division found by enumeration."""
    r, H = 4, 16
    d = [dev(a=0.002, b=2e-4, c=4.0, h=16, g=3000), dev(a=0.001, b=5e-4, c=6.0)]
    l = [700.0, 150.0]
    z, x, xh, zr = DO.dispatch(d, l, H, r)
    assert (xh % r == 0).all() and (xh.sum(axis=1) == H).all() and (xh >= 0).all()
    best = min(DO.times(d, l, r, [[4 * u0, H - 4 * u0], [4 * u1, H - 4 * u1]]).max()
               for u0, u1 in itertools.product(range(5), repeat=2))
    assert z <= best + 1e-9
    assert zr >= best - 1e-9
    A, b, K, _ = DO.device_terms(d, r)
    one_group = (A + b * (2 / r) * max(l)).max() * r
    assert zr - z <= 2 * one_group            # at most one group per request moved by rounding


def test_rounding_repairs_capacity():
    r, H = 1, 8
    l = [100.0, 100.0]
    # LP optimum fills device 0 exactly with 4.5 + 4.5 heads; rounding up both would overflow
    d = [dev(b=1e-5, capacity=2 * 100 * 9), dev(b=1e-3)]
    z, x, xh, zr = DO.dispatch(d, l, H, r)
    assert abs(x[:, 0].sum() - 9) < 1e-6
    assert (2 * 100 * xh[:, 0]).sum() <= 2 * 100 * 9 + 1e-9
    assert (xh.sum(axis=1) == H).all()


def random_instance(rng, N, J, r):
    H = r * int(rng.integers(2, 9))
    d = [dev(a=float(rng.uniform(0, 0.01)), b=float(rng.uniform(5e-5, 5e-4)),
             c=float(rng.uniform(2, 30)), h=float(rng.integers(0, 500)),
             g=float(rng.integers(0, 200000)), capacity=float(rng.integers(300000, 2000000)),
             primary=bool(i == 0), gamma=float(rng.uniform(0, 0.005)), beta=float(rng.uniform(0, 5)))
         for i in range(N)]
    l = rng.integers(16, 8000, size=J).astype(np.float64)
    return d, l, H


def test_lp_value_is_a_lower_bound_of_any_feasible_division():
    rng = np.random.default_rng(81)
    for _ in range(20):
        N, J, r = int(rng.integers(2, 5)), int(rng.integers(1, 6)), int(rng.choice([1, 2, 8]))
        d, l, H = random_instance(rng, N, J, r)
        sol = DO.solve_lp(d, l, H, r)
        if sol is None:
            continue
        z, x = sol
        assert np.allclose(x.sum(axis=1), H, atol=1e-7) and (x >= -1e-9).all()
        assert abs(DO.times(d, l, r, x).max() - z) < 1e-7 * max(1.0, abs(z))
        _, _, _, cap = DO.device_terms(d, r)
        for _ in range(30):                      # random feasible points are never better
            w = rng.dirichlet(np.ones(N), size=J) * H
            if ((2 / r) * (l[:, None] * w).sum(axis=0) <= cap).all():
                assert DO.times(d, l, r, w).max() >= z - 1e-7 * max(1.0, abs(z))


# ---------------------------------------------------------------- library against the checker

import ctypes as C

import paper_2509_08309_amd as H
from paper_2509_08309_amd import binding


def lib_dispatch(devices, lengths, n_heads, r):
    binding.load(build_if_missing=True)
    N, J = len(devices), len(lengths)
    arr = (H.hetis_dispatch_device * N)()
    for i, d in enumerate(devices):
        arr[i] = H.hetis_dispatch_device(d["a"], d["b"], d["c"], d.get("gamma", 0.0),
                                         d.get("beta", 0.0), d.get("h", 0.0), d.get("g", 0.0),
                                         d["capacity"], 1 if d.get("primary", False) else 0, 0)
    l = np.ascontiguousarray(lengths, dtype=np.float64)
    xf = np.zeros((J, N))
    xh = np.zeros((J, N), dtype=np.int32)
    z, zr = C.c_double(0), C.c_double(0)
    rc = H.hetis_dispatch_solve(arr, N, l, J, n_heads, r, xf, xh, z, zr)
    return rc, z.value, xf, xh, zr.value


def check_against_checker(d, l, H_, r):
    rc, z, xf, xh, zr = lib_dispatch(d, l, H_, r)
    ref = DO.solve_lp(d, l, H_, r)
    if ref is None:
        assert rc == binding.HETIS_ERR_INFEASIBLE
        return None
    assert rc == 0
    z_ref, _ = ref
    tol = 1e-7 * max(1.0, abs(z_ref))
    assert abs(z - z_ref) <= tol, (z, z_ref)
    # the library's fractional division is feasible and attains its own optimum
    _, _, _, cap = DO.device_terms(d, r)
    l = np.asarray(l, dtype=np.float64)
    assert (xf >= -1e-9).all() and np.allclose(xf.sum(axis=1), H_, atol=1e-6)
    assert ((2 / r) * (l[:, None] * xf).sum(axis=0) <= cap * (1 + 1e-9) + 1e-6).all()
    assert abs(DO.times(d, l, r, xf).max() - z) <= 10 * tol
    # rounding: the stated rule applied by the checker to the same fractional division
    want = DO.round_to_groups(d, l, H_, r, xf)
    assert want is not None and np.array_equal(xh, want)
    assert (xh % r == 0).all() and (xh.sum(axis=1) == H_).all()
    assert abs(zr - DO.times(d, l, r, xh).max()) <= 1e-9 * max(1.0, abs(zr))
    return z


def test_library_on_the_pinned_cases():
    check_against_checker([dev(h=100, g=5000)], [300, 50], 32, 1)
    check_against_checker([dev() for _ in range(4)], [1000.0], 32, 1)
    check_against_checker([dev(b=1e-4, c=5.0, h=50, g=2e5), dev(b=3e-4, c=8.0, h=10, g=1e4)],
                          [2000.0], 64, 1)
    check_against_checker([dev(primary=True), dev(primary=False, gamma=0.01, beta=3.0)], [500.0], 40, 1)
    check_against_checker([dev(b=1e-5, capacity=2 * 1000.0 * 8), dev(b=1e-3)], [1000.0], 32, 1)
    check_against_checker([dev(a=0.002, b=2e-4, c=4.0, h=16, g=3000), dev(a=0.001, b=5e-4, c=6.0)],
                          [700.0, 150.0], 16, 4)
    check_against_checker([dev(b=1e-5, capacity=2 * 100 * 9), dev(b=1e-3)], [100.0, 100.0], 8, 1)
    assert check_against_checker([dev(capacity=10.0), dev(capacity=10.0)], [1000.0], 32, 1) is None


@pytest.mark.parametrize("seed", range(12))
def test_library_on_random_instances(seed):
    rng = np.random.default_rng(900 + seed)
    for _ in range(6):
        N, J, r = int(rng.integers(1, 7)), int(rng.integers(1, 25)), int(rng.choice([1, 2, 4, 8]))
        d, l, H_ = random_instance(rng, N, J, r)
        check_against_checker(d, l, H_, r)


def test_library_with_the_fitted_mi355x_parameters():
    """Four devices with the coefficients fitted on this kernel (one of them a Primary worker,
    one half as fast, one almost full): 16 new requests of a 40-head model."""
    fit = dict(a=0.00064, b=9.32e-5, c=15.4)
    d = [dev(**fit, h=640, g=4e5, capacity=4e6, primary=True),
         dev(**fit, h=320, g=1e5, capacity=4e6, primary=False, gamma=0.002, beta=8.0),
         dev(a=0.0013, b=1.9e-4, c=20.0, h=0, g=0, capacity=2e6, primary=False, gamma=0.002, beta=8.0),
         dev(**fit, h=900, g=3.7e6, capacity=4e6, primary=False, gamma=0.002, beta=8.0)]
    rng = np.random.default_rng(82)
    l = np.clip(np.round(np.exp(rng.normal(np.log(800), 0.8, size=16))), 32, 4096)
    z = check_against_checker(d, l, 40, 1)
    assert z is not None


def test_library_argument_errors():
    lib = binding.load(build_if_missing=True)
    d = [dev(), dev()]
    ok = lib_dispatch(d, [100.0], 8, 1)
    assert ok[0] == 0
    assert lib_dispatch(d, [100.0], 9, 2)[0] == binding.HETIS_ERR_BAD_SHAPE        # H % r
    assert lib_dispatch(d, [0.0], 8, 1)[0] == binding.HETIS_ERR_BAD_SHAPE          # length <= 0
    assert lib_dispatch(d, [np.nan], 8, 1)[0] == binding.HETIS_ERR_BAD_SHAPE
    assert lib_dispatch([dev(capacity=-1.0)], [100.0], 8, 1)[0] == binding.HETIS_ERR_BAD_SHAPE
    assert lib_dispatch([dev(g=50.0, capacity=10.0)], [100.0], 8, 1)[0] == binding.HETIS_ERR_INFEASIBLE
    assert lib.hetis_dispatch_solve(None, 1, None, 1, 8, 1, None, None, None, None) == binding.HETIS_ERR_NULL


def test_library_refuses_negative_model_parameters():
    """A cost per head or per cache unit below zero (a fit dominated by noise) would make a
    device look faster the more it is given; the solver refuses it."""
    import ctypes as C
    import paper_2509_08309_amd as H
    from paper_2509_08309_amd import binding
    binding.load(build_if_missing=True)
    for field in ("a", "b", "c", "gamma", "beta"):
        devs = (H.hetis_dispatch_device * 2)()
        for i in range(2):
            devs[i] = H.hetis_dispatch_device(0.001, 1e-4, 10.0, 0.0, 0.0, 0.0, 0.0, 1e9, 1, 0)
        setattr(devs[1], field, -1e-6)
        l = np.array([500.0])
        xh = np.zeros((1, 2), dtype=np.int32)
        assert H.hetis_dispatch_solve(devs, 2, l, 1, 8, 1, None, xh) == binding.HETIS_ERR_BAD_SHAPE
