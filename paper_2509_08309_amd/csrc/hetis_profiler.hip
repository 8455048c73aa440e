// Host side of the Profiler's Attention-time model (Section 5.1, Eq. (3)): least-squares fit
// of tau = a*h + b*g + c and prediction.  No device code.
#include "../../include/hetis_profiler.h"

#include <cmath>

namespace {

// Solves the 3x3 system M x = y in place by Gaussian elimination with partial pivoting.
// Returns false when a pivot is negligible against the matrix scale (singular system).
bool solve3(double M[3][3], double y[3], double x[3])
{
    double scale = 0.0;
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j) scale = std::fmax(scale, std::fabs(M[i][j]));
    if (!(scale > 0.0)) return false;
    for (int col = 0; col < 3; ++col) {
        int piv = col;
        for (int r = col + 1; r < 3; ++r)
            if (std::fabs(M[r][col]) > std::fabs(M[piv][col])) piv = r;
        if (std::fabs(M[piv][col]) <= 1e-12 * scale) return false;
        if (piv != col) {
            for (int j = 0; j < 3; ++j) std::swap(M[piv][j], M[col][j]);
            std::swap(y[piv], y[col]);
        }
        for (int r = col + 1; r < 3; ++r) {
            const double f = M[r][col] / M[col][col];
            for (int j = col; j < 3; ++j) M[r][j] -= f * M[col][j];
            y[r] -= f * y[col];
        }
    }
    for (int i = 2; i >= 0; --i) {
        double s = y[i];
        for (int j = i + 1; j < 3; ++j) s -= M[i][j] * x[j];
        x[i] = s / M[i][i];
    }
    return true;
}

}  // namespace

extern "C" {

int hetis_profiler_fit(const double *h, const double *g, const double *tau, int32_t n,
                       double *abc, double *accuracy)
{
    if (!h || !g || !tau || !abc) return HETIS_ERR_NULL;
    if (n < 3) return HETIS_ERR_BAD_SHAPE;
    // centre and scale the two regressors: the normal equations of raw (h, g, 1) columns
    // with g in the millions are needlessly ill-conditioned
    double mh = 0.0, mg = 0.0, mt = 0.0;
    for (int i = 0; i < n; ++i) {
        if (!std::isfinite(h[i]) || !std::isfinite(g[i]) || !std::isfinite(tau[i]) || !(tau[i] > 0.0))
            return HETIS_ERR_BAD_SHAPE;
        mh += h[i];
        mg += g[i];
        mt += tau[i];
    }
    mh /= n;
    mg /= n;
    mt /= n;
    double sh = 0.0, sg = 0.0;
    for (int i = 0; i < n; ++i) {
        sh = std::fmax(sh, std::fabs(h[i] - mh));
        sg = std::fmax(sg, std::fabs(g[i] - mg));
    }
    if (!(sh > 0.0) || !(sg > 0.0)) return HETIS_ERR_BAD_SHAPE;
    double M[3][3] = {{0, 0, 0}, {0, 0, 0}, {0, 0, 0}}, y[3] = {0, 0, 0};
    for (int i = 0; i < n; ++i) {
        const double row[3] = {(h[i] - mh) / sh, (g[i] - mg) / sg, 1.0};
        for (int r = 0; r < 3; ++r) {
            for (int c = 0; c < 3; ++c) M[r][c] += row[r] * row[c];
            y[r] += row[r] * (tau[i] - mt);
        }
    }
    double x[3];
    if (!solve3(M, y, x)) return HETIS_ERR_BAD_SHAPE;
    abc[0] = x[0] / sh;
    abc[1] = x[1] / sg;
    abc[2] = x[2] + mt - abc[0] * mh - abc[1] * mg;
    if (accuracy) {
        double err = 0.0;
        for (int i = 0; i < n; ++i)
            err += std::fabs(abc[0] * h[i] + abc[1] * g[i] + abc[2] - tau[i]) / tau[i];
        *accuracy = 1.0 - err / n;
    }
    return HETIS_OK;
}

// Least squares with (a, b) held at zero where `free_a` / `free_b` is false.  Returns the sum of
// squared residuals, or a negative value when the free parameters are not determined.
static double fit_subset(const double *h, const double *g, const double *tau, int n, bool free_a,
                         bool free_b, double *abc)
{
    if (free_a && free_b) {
        if (hetis_profiler_fit(h, g, tau, n, abc, nullptr) != HETIS_OK) return -1.0;
    } else {
        abc[0] = abc[1] = 0.0;
        double mt = 0.0;
        for (int i = 0; i < n; ++i) mt += tau[i];
        mt /= n;
        abc[2] = mt;
        if (free_a || free_b) {                      // one slope: simple regression
            const double *x = free_a ? h : g;
            double mx = 0.0;
            for (int i = 0; i < n; ++i) mx += x[i];
            mx /= n;
            double sxx = 0.0, sxy = 0.0;
            for (int i = 0; i < n; ++i) {
                sxx += (x[i] - mx) * (x[i] - mx);
                sxy += (x[i] - mx) * (tau[i] - mt);
            }
            if (!(sxx > 0.0)) return -1.0;
            const double slope = sxy / sxx;
            abc[free_a ? 0 : 1] = slope;
            abc[2] = mt - slope * mx;
        }
    }
    double ss = 0.0;
    for (int i = 0; i < n; ++i) {
        const double e = abc[0] * h[i] + abc[1] * g[i] + abc[2] - tau[i];
        ss += e * e;
    }
    return ss;
}

int hetis_profiler_fit_nonneg(const double *h, const double *g, const double *tau, int32_t n,
                              double *abc, double *accuracy)
{
    double best[3];
    int rc = hetis_profiler_fit(h, g, tau, n, best, nullptr);     // also validates the samples
    if (rc != HETIS_OK) return rc;
    if (best[0] < 0.0 || best[1] < 0.0) {
        // two sign constraints: the constrained optimum is the best feasible one among the
        // least-squares solutions with some of the constrained parameters held at zero
        double best_ss = -1.0;
        const bool sets[3][2] = {{false, true}, {true, false}, {false, false}};
        for (const auto &set : sets) {
            double cand[3];
            const double ss = fit_subset(h, g, tau, n, set[0], set[1], cand);
            if (ss < 0.0 || cand[0] < 0.0 || cand[1] < 0.0) continue;
            if (best_ss < 0.0 || ss < best_ss) {
                best_ss = ss;
                for (int k = 0; k < 3; ++k) best[k] = cand[k];
            }
        }
        if (best_ss < 0.0) return HETIS_ERR_BAD_SHAPE;
    }
    for (int k = 0; k < 3; ++k) abc[k] = best[k];
    if (accuracy) {
        double err = 0.0;
        for (int i = 0; i < n; ++i)
            err += std::fabs(abc[0] * h[i] + abc[1] * g[i] + abc[2] - tau[i]) / tau[i];
        *accuracy = 1.0 - err / n;
    }
    return HETIS_OK;
}

int hetis_profiler_predict(const double *abc, const double *h, const double *g, int32_t n,
                           double *tau_out)
{
    if (n < 0) return HETIS_ERR_BAD_SHAPE;
    if (!abc || (n > 0 && (!h || !g || !tau_out))) return HETIS_ERR_NULL;
    for (int i = 0; i < n; ++i) tau_out[i] = abc[0] * h[i] + abc[1] * g[i] + abc[2];
    return HETIS_OK;
}

}  // extern "C"
