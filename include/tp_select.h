/*
 * tp_select.h — C ABI of the TP subgroup selection (host code only; no GPU work).
 *
 * Section 6.1, "Selective Device Exclusion Within Affected TP Groups": G is the original TP
 * group, F_stop its fail-stop devices, G' = G \ F_stop.  Feasible TP degrees (Eq. 3):
 *     K = { k : k_min <= k <= |G'|, k a power of two }.
 * For each k in K the candidate S_k is the top-k devices of G' ranked by normalised throughput
 * p_i (relative to the device's healthy peak), and the chosen subgroup (Eq. 4) is
 *     S* = argmax over k in K of  k * min_{i in S_k} p_i .
 * Devices of G' outside S* stay online as node-local standby devices.
 * Ties between degrees go to the larger degree, ties between devices to the lower index.
 *
 * All pointers are HOST pointers owned by the caller.
 */
#ifndef TP_SELECT_H_
#define TP_SELECT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TP_SELECT_OK 0
#define TP_SELECT_INVALID_ARG (-1)   /* null pointer, group_size < 1 or > 64, k_min < 1,
                                        p_i negative or not finite */
#define TP_SELECT_NO_FEASIBLE_DEGREE 1 /* K is empty: degree 0, no members, G' all standby */

#define TP_SELECT_ROLE_FAIL_STOP 0
#define TP_SELECT_ROLE_MEMBER 1
#define TP_SELECT_ROLE_STANDBY 2

/* throughput: p_i for the group_size devices of G; fail_stop: group_size flags (non-zero =
 * the device is in F_stop; its p_i is ignored).  Writes the chosen degree, its estimated
 * aggregate throughput k * min p_i, and for every device its role (TP_SELECT_ROLE_*).
 * Returns TP_SELECT_OK, TP_SELECT_NO_FEASIBLE_DEGREE or TP_SELECT_INVALID_ARG. */
int tp_select_subgroup(const double* throughput, const uint8_t* fail_stop, int32_t group_size,
                       int32_t k_min, int32_t* degree, double* aggregate_throughput,
                       int32_t* role);

#ifdef __cplusplus
}
#endif
#endif /* TP_SELECT_H_ */
