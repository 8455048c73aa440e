/*
 * hetis_profiler.h - the Profiler's model of Attention time (Section 5.1, Eq. (3) of the
 * Hetis paper), host side.
 *
 * The decode-phase Attention time of a device is modelled as a linear function of the
 * number of query heads among its requests, h, and the amount of cache those heads
 * attend over, g:
 *         tau = a * h + b * g + c                                      (Eq. (3))
 * with per-device parameters a, b, c obtained from an offline run over a grid of (h, g)
 * values (Section 7.4, "Modeling accuracy": eight values of each).  The measurements come
 * from timing hetis_attn_decode_pairs on synthetic inputs; this header holds the fit and
 * the prediction.  All pointers are HOST pointers; nothing here touches the GPU.
 *
 * Units are the caller's (the package measures tau in microseconds, h in query heads and
 * g in cached tokens x KV heads).
 */
#ifndef HETIS_PROFILER_H
#define HETIS_PROFILER_H

#include "hetis_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Ordinary least squares for (a, b, c) over n samples (h[i], g[i], tau[i]).
 *   abc       out, 3 doubles: a, b, c
 *   accuracy  out (may be NULL): 1 - mean_i |a h_i + b g_i + c - tau_i| / tau_i, the mean
 *             relative accuracy of the fitted model on its own samples
 * Returns HETIS_OK; HETIS_ERR_NULL; HETIS_ERR_BAD_SHAPE if n < 3, a value is not finite, a
 * tau is not positive, or the samples do not determine the three parameters (all h equal,
 * all g equal, or h and g affinely dependent).
 */
int hetis_profiler_fit(const double *h, const double *g, const double *tau, int32_t n,
                       double *abc, double *accuracy);

/*
 * The same fit under a >= 0 and b >= 0.  Eq. (7) uses a and b as the cost of one more head
 * and one more unit of cache on a device, so a fit whose slope came out slightly negative
 * (a kernel whose time does not grow with the head count, plus measurement noise) must not
 * reach the Dispatcher as it is.  When the unconstrained solution already has both slopes
 * non-negative it is returned unchanged.  Arguments, accuracy and errors as above.
 */
int hetis_profiler_fit_nonneg(const double *h, const double *g, const double *tau, int32_t n,
                              double *abc, double *accuracy);

/* tau_out[i] = a * h[i] + b * g[i] + c for i < n (n >= 0). */
int hetis_profiler_predict(const double *abc, const double *h, const double *g, int32_t n,
                           double *tau_out);

#ifdef __cplusplus
}
#endif
#endif /* HETIS_PROFILER_H */
