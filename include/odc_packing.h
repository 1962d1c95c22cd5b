/*
 * odc_packing.h -- host-side load balancing that ODC enables (paper Section 4, Appendix C).
 *
 * With per-layer collectives every device must run the same number of microbatches, so
 * balancing happens per microbatch (LB-Micro).  ODC removes that constraint: the minibatch is
 * balanced over the devices by total compute cost alone and every device then packs its own
 * samples into as many microbatches as its memory needs (LB-Mini).  Both use Karmarkar-Karp
 * number partitioning (the largest differencing method), whose interface Appendix C gives:
 * karmarkar_karp(costs, k, equal_size), get_compute_costs, check_oom, minibatch_partition,
 * microbatch_partition.  The bodies the paper does not print are fixed as follows:
 *   cost(s)    = s * (s + 6 * hidden)      (Section 4: runtime O(s^2), memory O(s); hidden = 0
 *                                           is the pure quadratic model)
 *   check_oom  = a microbatch is infeasible when it holds more than one sample and its tokens
 *                exceed max_tokens (a single longer sample cannot be split and is accepted alone)
 *   ties       = larger spread first, then the partial solution created earlier; inside a
 *                partial solution subsets are ordered by sum (descending), then by smallest index.
 * Everything here is plain host code: pointers are HOST pointers, nothing touches the GPU.
 * All functions return ODC_OK or a negative ODC_ERR_* code (see odc.h).
 */
#ifndef ODC_PACKING_H
#define ODC_PACKING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* cost(s) = s * (s + 6 * hidden); returns -1 if s < 0, hidden < 0 or the product overflows. */
int64_t odc_compute_cost(int64_t seqlen, int64_t hidden);

/*
 * k-way Karmarkar-Karp partition of n non-negative costs.
 *   part_of [n] out: part index 0..k-1 of every item; parts are numbered by final subset sum,
 *           largest first (ties: smaller smallest-index first, empty parts last).
 *   equal_size != 0 requires n % k == 0 and gives every part n / k items.
 * Errors: ODC_ERR_INVALID_ARG (null pointer, n < 0, k < 1, negative cost, equal_size with
 * n % k != 0), ODC_ERR_OVERFLOW (sum of costs does not fit 63 bits), ODC_ERR_NOMEM.
 */
int odc_kk_partition(const int64_t *costs, int n, int k, int equal_size, int *part_of);

/*
 * One minibatch of n samples over `world` devices.
 *   mode 0 = LB-Mini: devices balanced by cost with unequal sample counts; each device raises
 *            its own microbatch count until every microbatch has at most max_tokens tokens.
 *   mode 1 = LB-Micro: equal sample counts (n % world must be 0) and one common microbatch
 *            count, raised until no device has an infeasible microbatch.
 *   mode 2 = LocalSort (the unpacked baseline of Section 5.1): the samples are dealt to the
 *            devices in the order given, n / world each (n % world must be 0); every device
 *            sorts its own by length, longest first, and runs one sample per microbatch.
 *            max_tokens is not used.
 *   device_of [n] out, micro_of [n] out: device and microbatch (index within the device) of
 *            every sample; micro_count [world] out: microbatches per device (empty ones are
 *            not counted in LB-Mini; LB-Micro counts the common k on every device).
 * A sample longer than max_tokens is accepted once it is alone in a microbatch.
 */
int odc_plan_minibatch(const int64_t *seqlens, int n, int world, int64_t max_tokens, int64_t hidden,
                       int mode, int *device_of, int *micro_of, int *micro_count);

/*
 * Runtime estimate of a plan in cost units (Eq. 1 and its ODC counterpart) and bubble rates
 * (Appendix F: idle time over total time).
 *   t_collective = sum over microbatch steps m of max over devices of cost(d, m)
 *   t_odc        = max over devices of sum over m of cost(d, m)
 *   busy [world] out (may be NULL): sum of cost(d, m) per device
 *   bubble_collective, bubble_odc: 1 - sum(busy) / (world * t)
 */
int odc_plan_runtime(const int64_t *seqlens, int n, int world, int64_t hidden, const int *device_of,
                     const int *micro_of, int64_t *t_collective, int64_t *t_odc, int64_t *busy,
                     double *bubble_collective, double *bubble_odc);

#ifdef __cplusplus
}
#endif
#endif /* ODC_PACKING_H */
