// Host side of the Dispatcher (Section 5.2.2, Eq. (7)): the min-max head-wise division as a
// linear programme, solved by a dense two-phase simplex, then rounded to whole head groups.
// No device code.
#include "../../include/hetis_dispatch.h"

#include <cmath>
#include <vector>

namespace {

constexpr double kEps = 1e-9;

// Dense simplex tableau for  min cost.y  s.t.  A y = rhs, y >= 0  with rhs >= 0.
struct Tableau {
    int m, n;                       // rows, columns (without the right-hand side)
    std::vector<double> t;          // m x (n + 1), row-major; column n is the right-hand side
    std::vector<double> obj;        // n + 1 reduced costs; obj[n] = -(objective value)
    std::vector<int> basis;         // basic column of every row
    std::vector<char> allowed;      // columns that may enter

    double &at(int r, int c) { return t[(size_t)r * (n + 1) + c]; }

    void pivot(int pr, int pc)
    {
        const double inv = 1.0 / at(pr, pc);
        for (int c = 0; c <= n; ++c) at(pr, c) *= inv;
        at(pr, pc) = 1.0;
        for (int r = 0; r < m; ++r) {
            if (r == pr) continue;
            const double f = at(r, pc);
            if (f == 0.0) continue;
            for (int c = 0; c <= n; ++c) at(r, c) -= f * at(pr, c);
            at(r, pc) = 0.0;
        }
        const double f = obj[pc];
        if (f != 0.0) {
            for (int c = 0; c <= n; ++c) obj[c] -= f * at(pr, c);
            obj[pc] = 0.0;
        }
        basis[pr] = pc;
    }

    // reduced costs of `cost` for the current basis
    void price(const std::vector<double> &cost)
    {
        obj.assign(n + 1, 0.0);
        for (int c = 0; c < n; ++c) obj[c] = cost[c];
        for (int r = 0; r < m; ++r) {
            const double cb = cost[basis[r]];
            if (cb == 0.0) continue;
            for (int c = 0; c <= n; ++c) obj[c] -= cb * at(r, c);
        }
    }

    // true: optimal; false: unbounded or iteration limit.  The entering column is the one with
    // the most negative reduced cost; after a run of pivots that did not lower the objective
    // (degenerate vertex) Bland's rule takes over until it does, which rules out cycling.
    bool run()
    {
        const long limit = 200L * (m + n) + 1000;
        int stalled = 0;
        for (long it = 0; it < limit; ++it) {
            int pc = -1;
            if (stalled < 40) {
                double most = -kEps;
                for (int c = 0; c < n; ++c)
                    if (allowed[c] && obj[c] < most) {
                        most = obj[c];
                        pc = c;
                    }
            } else {
                for (int c = 0; c < n; ++c)
                    if (allowed[c] && obj[c] < -kEps) {
                        pc = c;
                        break;
                    }
            }
            if (pc < 0) return true;
            int pr = -1;
            double best = 0.0;
            for (int r = 0; r < m; ++r) {
                const double a = at(r, pc);
                if (a <= kEps) continue;
                const double ratio = at(r, n) / a;
                if (pr < 0 || ratio < best - 1e-12 ||
                    (ratio <= best + 1e-12 && basis[r] < basis[pr])) {
                    pr = r;
                    best = ratio;
                }
            }
            if (pr < 0) return false;
            const double before = obj[n];
            pivot(pr, pc);
            stalled = obj[n] > before + 1e-13 * (1.0 + std::fabs(before)) ? 0 : stalled + 1;
        }
        return false;
    }
};

struct Terms {
    std::vector<double> A, b, K, cap;
};

Terms device_terms(const hetis_dispatch_device *d, int N, int r)
{
    Terms t;
    t.A.resize(N);
    t.b.resize(N);
    t.K.resize(N);
    t.cap.resize(N);
    for (int i = 0; i < N; ++i) {
        const bool prim = d[i].is_primary != 0;
        t.A[i] = d[i].a + (prim ? 0.0 : (2.0 + 2.0 / r) * d[i].gamma);
        t.b[i] = d[i].b;
        const double C = d[i].c + (prim ? 0.0 : d[i].beta);
        t.K[i] = t.A[i] * d[i].h + t.b[i] * d[i].g + C;
        t.cap[i] = d[i].capacity - d[i].g;
    }
    return t;
}

// f_i of a division x[j][i]
template <class X>
double device_time(const Terms &t, const double *len, int J, int N, int r, const X *x, int i)
{
    double heads = 0.0, cache = 0.0;
    for (int j = 0; j < J; ++j) {
        heads += (double)x[(size_t)j * N + i];
        cache += len[j] * (double)x[(size_t)j * N + i];
    }
    return t.K[i] + t.A[i] * heads + t.b[i] * (2.0 / r) * cache;
}

}  // namespace

extern "C" int hetis_dispatch_solve(const hetis_dispatch_device *devices, int32_t n_devices,
                                    const double *lengths, int32_t n_requests, int32_t n_heads,
                                    int32_t group, double *x_frac, int32_t *x_heads,
                                    double *z_lp, double *z_rounded)
{
    if (!devices || !lengths || !x_heads) return HETIS_ERR_NULL;
    const int N = n_devices, J = n_requests, r = group;
    if (N <= 0 || N > 64 || J <= 0 || J > 4096 || r <= 0 || n_heads <= 0 || n_heads % r != 0)
        return HETIS_ERR_BAD_SHAPE;
    for (int i = 0; i < N; ++i) {
        const hetis_dispatch_device &d = devices[i];
        const double v[8] = {d.a, d.b, d.c, d.gamma, d.beta, d.h, d.g, d.capacity};
        for (double q : v)
            if (!std::isfinite(q)) return HETIS_ERR_BAD_SHAPE;
        // a negative cost per head or per cache unit would make a device look faster the more it
        // is given: such a model (e.g. a fit dominated by noise) is refused, not optimised
        for (double q : v)
            if (q < 0) return HETIS_ERR_BAD_SHAPE;
    }
    for (int j = 0; j < J; ++j)
        if (!std::isfinite(lengths[j]) || !(lengths[j] > 0)) return HETIS_ERR_BAD_SHAPE;
    const Terms tm = device_terms(devices, N, r);
    for (int i = 0; i < N; ++i)
        if (tm.cap[i] < 0) return HETIS_ERR_INFEASIBLE;

    // ---- linear programme.  Columns: x[j][i] at j*N + i; z = zp - zm; surplus s_i of the
    // time rows; slack t_i of the capacity rows; one artificial per time row and per request
    // row.  Rows: (time i)  z - sum_j s_ij x_ji - s_i = K_i;  (capacity i)  sum_j (2/r) l_j
    // x_ji + t_i = cap_i;  (request j)  sum_i x_ji = H.  Every row is scaled by its largest
    // coefficient and given a non-negative right-hand side.
    const int nx = J * N, zp = nx, zm = nx + 1, s0 = nx + 2, t0 = s0 + N, a0 = t0 + N;
    const int n = a0 + N + J, m = 2 * N + J;
    Tableau T;
    T.m = m;
    T.n = n;
    T.t.assign((size_t)m * (n + 1), 0.0);
    T.basis.assign(m, -1);
    T.allowed.assign(n, 1);
    for (int i = 0; i < N; ++i) {
        // time row i
        double scale = 1.0;
        for (int j = 0; j < J; ++j)
            scale = std::fmax(scale, std::fabs(tm.A[i] + tm.b[i] * (2.0 / r) * lengths[j]));
        const double sign = tm.K[i] < 0 ? -1.0 : 1.0;
        const double f = sign / scale;
        const int row = i;
        for (int j = 0; j < J; ++j)
            T.at(row, j * N + i) = -f * (tm.A[i] + tm.b[i] * (2.0 / r) * lengths[j]);
        T.at(row, zp) = f;
        T.at(row, zm) = -f;
        T.at(row, s0 + i) = -f;
        T.at(row, n) = f * tm.K[i];
        T.at(row, a0 + i) = 1.0;
        T.basis[row] = a0 + i;
        // capacity row i
        const int crow = N + i;
        double cs = 1.0;
        for (int j = 0; j < J; ++j) cs = std::fmax(cs, (2.0 / r) * lengths[j]);
        for (int j = 0; j < J; ++j) T.at(crow, j * N + i) = (2.0 / r) * lengths[j] / cs;
        T.at(crow, t0 + i) = 1.0;
        T.at(crow, n) = tm.cap[i] / cs;
        T.basis[crow] = t0 + i;
    }
    for (int j = 0; j < J; ++j) {
        const int row = 2 * N + j;
        for (int i = 0; i < N; ++i) T.at(row, j * N + i) = 1.0;
        T.at(row, n) = (double)n_heads;
        T.at(row, a0 + N + j) = 1.0;
        T.basis[row] = a0 + N + j;
    }
    // phase 1: drive the artificials to zero
    std::vector<double> cost(n, 0.0);
    for (int c = a0; c < n; ++c) cost[c] = 1.0;
    T.price(cost);
    if (!T.run()) return HETIS_ERR_INFEASIBLE;
    double rhs_scale = 1.0;
    for (int rr = 0; rr < m; ++rr) rhs_scale = std::fmax(rhs_scale, std::fabs(T.at(rr, n)));
    if (-T.obj[n] > 1e-7 * rhs_scale) return HETIS_ERR_INFEASIBLE;
    for (int c = a0; c < n; ++c) T.allowed[c] = 0;
    for (int rr = 0; rr < m; ++rr) {
        if (T.basis[rr] < a0) continue;
        // an artificial left in the basis at level zero: swap it for any structural column
        int pc = -1;
        for (int c = 0; c < a0; ++c)
            if (std::fabs(T.at(rr, c)) > 1e-7) {
                pc = c;
                break;
            }
        if (pc >= 0) T.pivot(rr, pc);        // otherwise the row is redundant and stays inert
    }
    // phase 2: minimise z
    std::fill(cost.begin(), cost.end(), 0.0);
    cost[zp] = 1.0;
    cost[zm] = -1.0;
    T.price(cost);
    if (!T.run()) return HETIS_ERR_INFEASIBLE;
    std::vector<double> x((size_t)nx, 0.0);
    double z = 0.0;
    for (int rr = 0; rr < m; ++rr) {
        const int c = T.basis[rr];
        const double v = T.at(rr, n);
        if (c < nx)
            x[c] = v > 0 ? v : 0.0;
        else if (c == zp)
            z += v;
        else if (c == zm)
            z -= v;
    }
    if (x_frac)
        for (int k = 0; k < nx; ++k) x_frac[k] = x[k];
    if (z_lp) *z_lp = z;

    // ---- whole groups: largest remainders per request, then capacity repair
    const int groups = n_heads / r;
    std::vector<int> u((size_t)nx, 0);
    for (int j = 0; j < J; ++j) {
        std::vector<double> rest(N);
        int have = 0;
        for (int i = 0; i < N; ++i) {
            const double frac = x[(size_t)j * N + i] / r;
            const int base = (int)std::floor(frac + 1e-9);
            u[(size_t)j * N + i] = base;
            rest[i] = frac - base;
            have += base;
        }
        // fewer than N groups are missing (the fractional parts sum to that many)
        std::vector<char> taken(N, 0);
        for (int k = have; k < groups; ++k) {
            int best = -1;
            for (int i = 0; i < N; ++i)
                if (!taken[i] && (best < 0 || rest[i] > rest[best])) best = i;
            if (best < 0) break;
            taken[best] = 1;
            ++u[(size_t)j * N + best];
        }
    }
    auto used = [&](int i) {
        double s = 0.0;
        for (int j = 0; j < J; ++j) s += lengths[j] * u[(size_t)j * N + i];
        return 2.0 * s;                     // (2/r) * l * (groups * r)
    };
    auto fits = [&](double amount, int i) { return amount <= tm.cap[i] * (1 + 1e-12) + 1e-9; };
    const long repair_limit = (long)J * N * groups + 1;
    for (long it = 0;; ++it) {
        int over = -1;
        for (int i = 0; i < N && over < 0; ++i)
            if (!fits(used(i), i)) over = i;
        if (over < 0) break;
        if (it >= repair_limit) return HETIS_ERR_INFEASIBLE;
        int jmove = -1;
        for (int j = 0; j < J; ++j)
            if (u[(size_t)j * N + over] > 0 && (jmove < 0 || lengths[j] > lengths[jmove])) jmove = j;
        if (jmove < 0) return HETIS_ERR_INFEASIBLE;
        const double need = 2.0 * lengths[jmove];
        int kbest = -1;
        double fbest = 0.0;
        for (int k = 0; k < N; ++k) {
            if (k == over || !fits(used(k) + need, k)) continue;
            --u[(size_t)jmove * N + over];
            ++u[(size_t)jmove * N + k];
            std::vector<int> heads((size_t)nx);
            for (int q = 0; q < nx; ++q) heads[q] = u[q] * r;
            const double fk = device_time(tm, lengths, J, N, r, heads.data(), k);
            ++u[(size_t)jmove * N + over];
            --u[(size_t)jmove * N + k];
            if (kbest < 0 || fk < fbest) {
                kbest = k;
                fbest = fk;
            }
        }
        if (kbest < 0) return HETIS_ERR_INFEASIBLE;
        --u[(size_t)jmove * N + over];
        ++u[(size_t)jmove * N + kbest];
    }
    for (int k = 0; k < nx; ++k) x_heads[k] = u[k] * r;
    if (z_rounded) {
        double zr = -INFINITY;
        for (int i = 0; i < N; ++i)
            zr = std::fmax(zr, device_time(tm, lengths, J, N, r, x_heads, i));
        *z_rounded = zr;
    }
    return HETIS_OK;
}
