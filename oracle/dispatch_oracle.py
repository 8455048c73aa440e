"""CPU checker for the Dispatcher's head-wise division (TEST INFRASTRUCTURE ONLY).

What is computed (Section 5.2.2, Eq. (7)): new requests j = 1..J with context lengths l_j each
bring H query heads; x[j][i] of them go to device i.  Device i already serves h_i query heads
over g_i cache units and has a linear time model (Section 5.1, Eq. (3)), so after dispatching
    f_i(x) = A_i * (h_i + sum_j x[j][i]) + b_i * (g_i + (2/r) * sum_j l_j * x[j][i]) + C_i
with A_i = a_i and C_i = c_i on a Primary worker, A_i = a_i + (2 + 2/r) * gamma_i and
C_i = c_i + beta_i on an Attention worker that exchanges q/k/v/out rows with it (Eq. (4)).
The division minimises max_i f_i subject to sum_i x[j][i] = H for every request and to the
cache capacity of every device; it is a linear programme.  Heads move in groups of r
(Section 5.2.1: x / r must be an integer), which the paper leaves to the implementation.

Readings where the paper is silent or at odds with itself:
  - capacity: Eq. (6) bounds sum_j x l by r * M_i / 2 with M_i the AVAILABLE capacity, Eq. (7b)
    adds g_i on the left with the same right-hand side.  Taken here: M_i is the device's total
    capacity in the units of g (one unit = the K or V vector of one token of one KV head), so
    the new heads may use what is left:  (2/r) * sum_j l_j x[j][i] <= M_i - g_i.
  - rounding to groups: per request, the fractional group counts x[j][i] / r are floored and
    the groups still missing go to the devices with the largest fractional parts (ties: lower
    device index); then, while a device exceeds its capacity, one group of the request with the
    longest context on that device moves to the device that has room for it and ends up with
    the smallest f_i (ties: lower index).  If no device has room the problem is infeasible.

This file follows those steps with scipy's LP solver and plain Python loops; it shares no
code with the library.
"""
from __future__ import annotations

import numpy as np
from scipy.optimize import linprog


def device_terms(devices, r):
    """(A, b, K, cap): per device the head coefficient, the cache coefficient, the time before
    dispatching and the cache units still free."""
    A = np.array([d["a"] + (0.0 if d.get("primary", False) else (2 + 2 / r) * d.get("gamma", 0.0))
                  for d in devices])
    b = np.array([d["b"] for d in devices], dtype=np.float64)
    C = np.array([d["c"] + (0.0 if d.get("primary", False) else d.get("beta", 0.0))
                  for d in devices])
    h = np.array([d.get("h", 0.0) for d in devices], dtype=np.float64)
    g = np.array([d.get("g", 0.0) for d in devices], dtype=np.float64)
    cap = np.array([d["capacity"] for d in devices], dtype=np.float64) - g
    return A, b, A * h + b * g + C, cap


def times(devices, lengths, r, x):
    """f_i for a division x[j][i] (fractional or whole heads)."""
    A, b, K, _ = device_terms(devices, r)
    x = np.asarray(x, dtype=np.float64)
    l = np.asarray(lengths, dtype=np.float64)
    return K + A * x.sum(axis=0) + b * (2 / r) * (l[:, None] * x).sum(axis=0)


def solve_lp(devices, lengths, n_heads, r):
    """Optimal max_i f_i of the relaxed problem and one optimal x[j][i]; None if infeasible."""
    A, b, K, cap = device_terms(devices, r)
    l = np.asarray(lengths, dtype=np.float64)
    N, J = len(devices), len(l)
    nv = J * N + 1                                   # x[j][i] at j * N + i, then z
    cost = np.zeros(nv)
    cost[-1] = 1.0
    A_ub, b_ub = [], []
    for i in range(N):
        row = np.zeros(nv)
        for j in range(J):
            row[j * N + i] = A[i] + b[i] * (2 / r) * l[j]
        row[-1] = -1.0
        A_ub.append(row)
        b_ub.append(-K[i])
        row = np.zeros(nv)
        for j in range(J):
            row[j * N + i] = (2 / r) * l[j]
        A_ub.append(row)
        b_ub.append(cap[i])
    A_eq = np.zeros((J, nv))
    for j in range(J):
        A_eq[j, j * N:(j + 1) * N] = 1.0
    res = linprog(cost, A_ub=np.array(A_ub), b_ub=np.array(b_ub), A_eq=A_eq,
                  b_eq=np.full(J, float(n_heads)),
                  bounds=[(0, None)] * (J * N) + [(None, None)], method="highs")
    if res.status == 2:
        return None
    assert res.status == 0, res.message
    return float(res.x[-1]), res.x[:-1].reshape(J, N)


def round_to_groups(devices, lengths, n_heads, r, x_frac):
    """Whole groups of r heads per (request, device) following the rounding rule above.
    Returns an int array [J][N] of head counts, or None if the capacities cannot be met."""
    A, b, K, cap = device_terms(devices, r)
    l = np.asarray(lengths, dtype=np.float64)
    J, N = np.asarray(x_frac).shape
    groups = n_heads // r
    u = np.zeros((J, N), dtype=np.int64)
    for j in range(J):
        frac = np.asarray(x_frac[j], dtype=np.float64) / r
        base = np.floor(frac + 1e-9).astype(np.int64)
        rest = frac - base
        missing = groups - int(base.sum())
        order = sorted(range(N), key=lambda i: (-rest[i], i))
        for i in order[:max(missing, 0)]:
            base[i] += 1
        u[j] = base
    used = lambda: (2 / r) * (l[:, None] * u * r).sum(axis=0)
    for _ in range(J * N * groups + 1):
        over = [i for i in range(N) if used()[i] > cap[i] * (1 + 1e-12) + 1e-9]
        if not over:
            return u * r
        i = over[0]
        cands = [j for j in range(J) if u[j, i] > 0]
        j = max(cands, key=lambda jj: (l[jj], -jj))
        need = (2 / r) * l[j] * r
        best = None
        for k in range(N):
            if k == i or used()[k] + need > cap[k] * (1 + 1e-12) + 1e-9:
                continue
            trial = u.copy()
            trial[j, i] -= 1
            trial[j, k] += 1
            fk = times(devices, lengths, r, trial * r)[k]
            if best is None or fk < best[0]:
                best = (fk, k)
        if best is None:
            return None
        u[j, i] -= 1
        u[j, best[1]] += 1
    return None


def dispatch(devices, lengths, n_heads, r):
    """(z_lp, x_frac, x_heads, z_rounded), or None if infeasible."""
    sol = solve_lp(devices, lengths, n_heads, r)
    if sol is None:
        return None
    z, x = sol
    xh = round_to_groups(devices, lengths, n_heads, r, x)
    if xh is None:
        return None
    return z, x, xh, float(times(devices, lengths, r, xh).max())
