/*
 * hetis_dispatch.h - the Dispatcher's head-wise division of newly arrived requests
 * (Section 5.2 of the Hetis paper, Eq. (5)-(8)), host side.
 *
 * New requests j = 1..J with context lengths l_j each bring H query heads; x[j][i] of them go
 * to device i of the stage.  Device i already serves h_i query heads over g_i cache units and
 * has the linear time model of Section 5.1, so after dispatching its Attention time is
 *     f_i = A_i * (h_i + sum_j x[j][i]) + b_i * (g_i + (2/r) * sum_j l_j * x[j][i]) + C_i,
 * A_i = a_i, C_i = c_i on a Primary worker and A_i = a_i + (2 + 2/r) * gamma_i, C_i = c_i +
 * beta_i on an Attention worker (Eq. (3), (4); r = query heads per KV head).  The division
 * minimises max_i f_i subject to sum_i x[j][i] = H for every request and to every device's
 * cache capacity (Eq. (7)); heads move in whole groups of r (Section 5.2.1).
 *
 * Readings where the paper leaves a choice:
 *   - capacity is the device's TOTAL capacity in the units of g (one unit = the K or the V
 *     vector of one token of one KV head); the new heads may use what is left:
 *     (2/r) * sum_j l_j * x[j][i] <= capacity_i - g_i.
 *   - the linear programme is solved exactly (two-phase simplex), then rounded: per request
 *     the group counts x / r are floored and the missing groups go to the devices with the
 *     largest fractional parts (ties: lower device index); while a device exceeds its
 *     capacity, one group of the request with the longest context on it moves to the device
 *     that has room and ends up with the smallest f (ties: lower index).
 *
 * All pointers are HOST pointers; nothing here touches the GPU.
 */
#ifndef HETIS_DISPATCH_H
#define HETIS_DISPATCH_H

#include "hetis_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    double a, b, c;         /* Eq. (3): time per query head, per cache unit, constant */
    double gamma, beta;     /* Eq. (4): link time per head-vector, constant (Attention workers) */
    double h, g;            /* query heads and cache units already on the device */
    double capacity;        /* cache units the device can hold in total */
    int32_t is_primary;     /* 1: Primary worker (no transfer term), 0: Attention worker */
    int32_t reserved;       /* 0 */
} hetis_dispatch_device;

/*
 *   devices    [n_devices]             lengths  [n_requests] context lengths l_j (> 0)
 *   n_heads    H, a positive multiple of group (= r)
 *   x_frac     out, [n_requests][n_devices] optimal fractional heads, or NULL
 *   x_heads    out, [n_requests][n_devices] whole heads, multiples of group, rows sum to H
 *   z_lp       out, or NULL: optimal max_i f_i of the linear programme
 *   z_rounded  out, or NULL: max_i f_i of x_heads
 * Returns HETIS_OK; HETIS_ERR_NULL; HETIS_ERR_BAD_SHAPE (sizes, non-finite or negative
 * inputs, H not a multiple of r; more than 64 devices or 4096 requests); HETIS_ERR_INFEASIBLE
 * when the capacities cannot hold the requests.
 */
int hetis_dispatch_solve(const hetis_dispatch_device *devices, int32_t n_devices,
                         const double *lengths, int32_t n_requests, int32_t n_heads,
                         int32_t group, double *x_frac, int32_t *x_heads, double *z_lp,
                         double *z_rounded);

#ifdef __cplusplus
}
#endif
#endif /* HETIS_DISPATCH_H */
