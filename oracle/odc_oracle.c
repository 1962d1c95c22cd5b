/*
 * CPU oracle for the On-Demand Communication (ODC) data-parallel hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the GPU path must compute.  It shares no code, header, table or helper with
 * the HIP library and must never be linked into or called from the product
 * path; only tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What it follows (paper: "Revisiting Parameter Server in LLM Post-Training"):
 *   - Section 3.1: parameters and gradients are partitioned evenly over all R
 *     devices; each device owns one shard (decentralised parameter server that
 *     keeps FSDP's memory layout, Section 3).
 *   - Section 3: gather replaces all-gather (a worker fetches every owner's
 *     parameter shard and so obtains the full layer); scatter-accumulate
 *     replaces reduce-scatter (a worker pushes slice r of its gradient to
 *     owner r, who adds it to its gradient shard).  Appendix B: the owner
 *     accumulates each contribution when it is received.
 *   - Section 2.1: the accumulated gradient is the sum over microbatches of
 *     w_m * g^(m); here w_m = 1.
 *   - Section 3.2: accumulated gradients are retrieved at the minibatch end
 *     (retrieve), so the accumulators are cleared before the next minibatch (reset).
 *
 * Readings where the paper is silent (kept identical in the design notes):
 *   - element types: bf16 parameters and gradient contributions (raw 16-bit
 *     patterns here), IEEE-754 binary32 accumulators;
 *   - R does not divide N: S = ceil(N / R), owner r holds flat indices
 *     [r*S, (r+1)*S), indices >= N are padding and are never read or written;
 *   - the order of contributions is fixed by the caller (worker ascending,
 *     then microbatch ascending); one call below applies ONE contribution;
 *   - the worker's own slice is treated like every other slice.
 *
 * Every routine takes a flat index range [j_begin, j_end) and touches only
 * elements inside it, so that a driver can split the element range over
 * threads without changing any element's sequence of operations.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC.  No flush-to-
 * zero: x86-64 SSE default keeps subnormals.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Section 3.1, even partition: elements per owner shard. */
int64_t odc_oracle_shard_elems(int64_t N, int64_t R)
{
    return (N + R - 1) / R;
}

/* Number of non-padding elements in owner r's shard. */
int64_t odc_oracle_valid_elems(int64_t N, int64_t R, int64_t r)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    int64_t v = N - r * S;
    if (v < 0) v = 0;
    if (v > S) v = S;
    return v;
}

/* bf16 -> binary32 is exact: the 16 bits become the high half of the word. */
static float widen_bf16(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static int64_t lo_clip(int64_t j_begin, int64_t base)
{
    int64_t i = j_begin - base;
    return i < 0 ? 0 : i;
}

static int64_t hi_clip(int64_t j_end, int64_t base, int64_t valid)
{
    int64_t i = j_end - base;
    return i > valid ? valid : i;
}

/*
 * Split a flat parameter into owner r's shard (the inverse of gather; used to
 * prepare inputs and for the round-trip invariant).  shard_out has S slots;
 * only the valid ones are written.
 */
void odc_oracle_make_shard(const uint16_t *flat, int64_t N, int64_t R, int64_t r,
                           uint16_t *shard_out)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    int64_t valid = odc_oracle_valid_elems(N, R, r);
    for (int64_t i = 0; i < valid; ++i)
        shard_out[i] = flat[r * S + i];
}

/*
 * Gather (Section 3; Appendix B "pulls data from all ranks"):
 *   full[r*S + i] = shard_r[i]   for every owner r and every valid i.
 * Bits are moved unchanged.  full[j] for j >= N is never written.
 */
void odc_oracle_gather(const uint16_t *const *shards, int64_t N, int64_t R,
                       uint16_t *full, int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i)
            full[r * S + i] = shards[r][i];
    }
}

/*
 * Reset (Section 3.2): valid accumulator elements become +0.0f.
 * Padding slots are never written.
 */
void odc_oracle_reset(float *const *acc, int64_t N, int64_t R,
                      int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i)
            acc[r][i] = 0.0f;
    }
}

/*
 * One scatter-accumulate contribution (Section 3; Appendix B; Section 2.1 with
 * w_m = 1): the worker's full-length gradient g is cut into R slices, slice r
 * goes to owner r, who performs
 *   acc_r[i] = fl32( acc_r[i] + widen(g[r*S + i]) )    for every valid i
 * with one binary32 addition, round-to-nearest-even.  Calling this once per
 * (worker, microbatch) in ascending order gives the ordered result.
 */
void odc_oracle_accumulate(const uint16_t *g, float *const *acc, int64_t N, int64_t R,
                           int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i)
            acc[r][i] = acc[r][i] + widen_bf16(g[r * S + i]);
    }
}

/*
 * Weighted contribution (Section 2.1: the accumulated gradient is the sum over microbatches
 * of w_m * g^(m), where w_m is 1 for a plain sum and a token- or sample-proportional weight
 * for an average).  The paper does not say how the product is rounded; the reading taken
 * is one fused multiply-add in binary32 per element,
 *   acc_r[i] = fma32(w, widen(g[r*S + i]), acc_r[i]),
 * i.e. a single rounding of the exact value w*g + acc.  fmaf() is the correctly rounded C99
 * routine.  With w = 1 this is the unweighted contribution bit for bit.
 */
void odc_oracle_accumulate_weighted(const uint16_t *g, float *const *acc, int64_t N, int64_t R,
                                    float w, int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i)
            acc[r][i] = fmaf(w, widen_bf16(g[r * S + i]), acc[r][i]);
    }
}

/* binary32 -> bf16, round-to-nearest-even; a NaN stays a (quiet) NaN. */
static uint16_t narrow_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/*
 * Retrieval at the minibatch end (Section 3.2: besides swapping the collectives for the two
 * primitives, an integration only has to read the accumulated gradients back once per
 * minibatch; after it each owner holds what reduce-scatter would have left on the device,
 * Section 2.2).  Owner r's valid accumulator elements are
 * read, multiplied by `scale` (1 for a plain sum, 1/tokens or 1/samples for an average) with
 * one binary32 multiplication, and written out either as binary32 or, rounded once more to
 * nearest-even, as bf16.  The accumulators are not changed; padding slots of the outputs are
 * never written.
 */
void odc_oracle_retrieve_f32(const float *const *acc, float *const *out, int64_t N, int64_t R,
                             float scale, int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i)
            out[r][i] = scale * acc[r][i];
    }
}

void odc_oracle_retrieve_bf16(const float *const *acc, uint16_t *const *out, int64_t N, int64_t R,
                              float scale, int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i) {
            float v = scale * acc[r][i];
            out[r][i] = narrow_to_bf16(v);
        }
    }
}

/*
 * Hybrid sharding (Section 6.1; Appendix E): parameters and gradients are sharded inside a
 * group of R devices only (a node), so each of the K groups ends a minibatch holding its own
 * accumulated gradient shards, and shard r of the minibatch gradient is the sum over the K
 * groups of their shard r (the step that crosses nodes once per minibatch, in place of the
 * per-layer cross-node traffic of full sharding).  The paper does not fix the order of that
 * sum; the reading taken is ascending group order, one binary32 addition per further group:
 *   out_r[i] = (((a_{0,r}[i] + a_{1,r}[i]) + a_{2,r}[i]) + ... + a_{K-1,r}[i])   for valid i.
 * group_acc is group-major: group k's shard of owner r is group_acc[k*R + r].  out_r may be
 * group 0's shard r (the sum then replaces it).  Padding slots are never read or written.
 */
void odc_oracle_reduce_groups(const float *const *group_acc, int64_t K, float *const *out,
                              int64_t N, int64_t R, int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i) {
            float s = group_acc[r][i];
            for (int64_t k = 1; k < K; ++k)
                s = s + group_acc[k * R + r][i];
            out[r][i] = s;
        }
    }
}

/*
 * Wide accumulators for the unordered mode.  When contributions are added in whatever order
 * they arrive (Appendix B: the owner accumulates on receipt, several clients push at once), a
 * binary32 accumulator can be off by up to (C - 1) * 2^-24 * sum|g| after C contributions, more
 * than the 1e-6 tolerance of the unordered mode once C > 17.  Keeping the running sum in binary64
 * removes the dependence on C and on the order: every addition of a widened bf16 value is
 * rounded at 2^-53, and the sum is rounded to binary32 once, at retrieval (Section 3.2), so the
 * retrieved gradient is within 2^-24 * (1 + C * 2^-29) of the exact sum relative to sum|g|.
 *   accumulate_wide:  acc64_r[i] = fl64(acc64_r[i] + widen(g[r*S + i]))      for valid i
 *   reset_wide:       acc64_r[i] = +0.0
 *   retrieve_wide:    out_r[i]   = cast(fl32(scale * fl32(acc64_r[i])))      (binary32 or bf16 out)
 * The reading taken for the retrieval: one rounding to binary32 first, then the same multiply
 * and cast as the binary32 retrieval, so that both retrievals treat a value alike.
 */
void odc_oracle_accumulate_wide(const uint16_t *g, double *const *acc, int64_t N, int64_t R,
                                int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i)
            acc[r][i] = acc[r][i] + (double)widen_bf16(g[r * S + i]);
    }
}

void odc_oracle_reset_wide(double *const *acc, int64_t N, int64_t R, int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i)
            acc[r][i] = 0.0;
    }
}

/* out_is_bf16 = 0: out holds binary32; 1: bf16 bit patterns. */
void odc_oracle_retrieve_wide(const double *const *acc, void *const *out, int64_t N, int64_t R,
                              float scale, int out_is_bf16, int64_t j_begin, int64_t j_end)
{
    int64_t S = odc_oracle_shard_elems(N, R);
    for (int64_t r = 0; r < R; ++r) {
        int64_t valid = odc_oracle_valid_elems(N, R, r);
        int64_t i0 = lo_clip(j_begin, r * S);
        int64_t i1 = hi_clip(j_end, r * S, valid);
        for (int64_t i = i0; i < i1; ++i) {
            float narrow = (float)acc[r][i];
            float v = scale * narrow;
            if (out_is_bf16) ((uint16_t *)out[r])[i] = narrow_to_bf16(v);
            else ((float *)out[r])[i] = v;
        }
    }
}

/*
 * Batched forms (the many-small-tensor workload): T flat parameters, each
 * partitioned on its own by the rule above.  Where tensor t sits inside an
 * owner's buffer (shard_off[t], in elements, the same for every owner) and
 * inside the full-length buffer (full_off[t]) is buffer placement chosen by
 * the caller, not part of the method, so both arrive as inputs.  Each tensor
 * is handled by the single-tensor routine, one after the other.
 * Returns 0, or -1 if the scratch pointer array cannot be allocated.
 */
int odc_oracle_gather_batched(const uint16_t *const *arenas, int64_t T, const int64_t *numel,
                              const int64_t *shard_off, const int64_t *full_off, int64_t R,
                              uint16_t *full)
{
    const uint16_t **sh = (const uint16_t **)malloc((size_t)R * sizeof *sh);
    if (!sh) return -1;
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t r = 0; r < R; ++r) sh[r] = arenas[r] + shard_off[t];
        odc_oracle_gather(sh, numel[t], R, full + full_off[t], 0, numel[t]);
    }
    free(sh);
    return 0;
}

int odc_oracle_reset_batched(float *const *acc_arenas, int64_t T, const int64_t *numel,
                             const int64_t *shard_off, int64_t R)
{
    float **ac = (float **)malloc((size_t)R * sizeof *ac);
    if (!ac) return -1;
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t r = 0; r < R; ++r) ac[r] = acc_arenas[r] + shard_off[t];
        odc_oracle_reset(ac, numel[t], R, 0, numel[t]);
    }
    free(ac);
    return 0;
}

int odc_oracle_accumulate_batched(const uint16_t *g_full, float *const *acc_arenas, int64_t T,
                                  const int64_t *numel, const int64_t *shard_off,
                                  const int64_t *full_off, int64_t R)
{
    float **ac = (float **)malloc((size_t)R * sizeof *ac);
    if (!ac) return -1;
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t r = 0; r < R; ++r) ac[r] = acc_arenas[r] + shard_off[t];
        odc_oracle_accumulate(g_full + full_off[t], ac, numel[t], R, 0, numel[t]);
    }
    free(ac);
    return 0;
}

int odc_oracle_accumulate_weighted_batched(const uint16_t *g_full, float *const *acc_arenas, int64_t T,
                                           const int64_t *numel, const int64_t *shard_off,
                                           const int64_t *full_off, int64_t R, float w)
{
    float **ac = (float **)malloc((size_t)R * sizeof *ac);
    if (!ac) return -1;
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t r = 0; r < R; ++r) ac[r] = acc_arenas[r] + shard_off[t];
        odc_oracle_accumulate_weighted(g_full + full_off[t], ac, numel[t], R, w, 0, numel[t]);
    }
    free(ac);
    return 0;
}

/* out_is_bf16 = 0: out arenas hold binary32; 1: bf16 bit patterns. */
int odc_oracle_retrieve_batched(const float *const *acc_arenas, void *const *out_arenas, int64_t T,
                                const int64_t *numel, const int64_t *shard_off, int64_t R,
                                float scale, int out_is_bf16)
{
    const float **ac = (const float **)malloc((size_t)R * sizeof *ac);
    void **ou = (void **)malloc((size_t)R * sizeof *ou);
    if (!ac || !ou) {
        free(ac);
        free(ou);
        return -1;
    }
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t r = 0; r < R; ++r) {
            ac[r] = acc_arenas[r] + shard_off[t];
            ou[r] = out_is_bf16 ? (void *)((uint16_t *)out_arenas[r] + shard_off[t])
                                : (void *)((float *)out_arenas[r] + shard_off[t]);
        }
        if (out_is_bf16)
            odc_oracle_retrieve_bf16(ac, (uint16_t *const *)ou, numel[t], R, scale, 0, numel[t]);
        else
            odc_oracle_retrieve_f32(ac, (float *const *)ou, numel[t], R, scale, 0, numel[t]);
    }
    free(ac);
    free(ou);
    return 0;
}

int odc_oracle_reduce_groups_batched(const float *const *group_arenas, int64_t K, float *const *out_arenas,
                                     int64_t T, const int64_t *numel, const int64_t *shard_off, int64_t R)
{
    const float **ga = (const float **)malloc((size_t)(K * R) * sizeof *ga);
    float **ou = (float **)malloc((size_t)R * sizeof *ou);
    if (!ga || !ou) {
        free(ga);
        free(ou);
        return -1;
    }
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t q = 0; q < K * R; ++q) ga[q] = group_arenas[q] + shard_off[t];
        for (int64_t r = 0; r < R; ++r) ou[r] = out_arenas[r] + shard_off[t];
        odc_oracle_reduce_groups(ga, K, ou, numel[t], R, 0, numel[t]);
    }
    free(ga);
    free(ou);
    return 0;
}
