/*
 * A plain C99 consumer of the C ABI (test infrastructure): no Python, no torch.  It builds a
 * layout, allocates every buffer with hipMalloc, runs gather, reset, three ordered
 * contributions and a retrieval on its own stream, and writes inputs and outputs to files in
 * the directory given as argv[1]; the test compares them with the CPU oracle.
 *
 * usage: c_abi_check <dir> <R> <numel_0> [numel_1 ...]
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "odc.h"

#define CHECK_HIP(call)                                                              \
    do {                                                                             \
        hipError_t e_ = (call);                                                      \
        if (e_ != hipSuccess) {                                                      \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));        \
            return 3;                                                                \
        }                                                                            \
    } while (0)

#define CHECK_ODC(call)                                                              \
    do {                                                                             \
        int rc_ = (call);                                                            \
        if (rc_ != ODC_OK) {                                                         \
            fprintf(stderr, "%s failed: %s\n", #call, odc_strerror(rc_));            \
            return 4;                                                                \
        }                                                                            \
    } while (0)

static uint32_t lcg(uint32_t *s) { return *s = *s * 1664525u + 1013904223u; }

/* bf16 bit pattern of a small value: sign, exponent 117..124, 7 mantissa bits (finite, normal) */
static uint16_t some_bf16(uint32_t *s)
{
    const uint32_t r = lcg(s) >> 8;
    return (uint16_t)(((r & 1u) << 15) | ((117u + ((r >> 1) & 7u)) << 7) | ((r >> 4) & 127u));
}

static int dump(const char *dir, const char *name, const void *p, size_t bytes)
{
    char path[1024];
    FILE *f;
    snprintf(path, sizeof path, "%s/%s", dir, name);
    f = fopen(path, "wb");
    if (!f || (bytes && fwrite(p, 1, bytes, f) != bytes)) return 1;
    return fclose(f);
}

int main(int argc, char **argv)
{
    if (argc < 4) {
        fprintf(stderr, "usage: %s dir R numel...\n", argv[0]);
        return 2;
    }
    const char *dir = argv[1];
    const int R = atoi(argv[2]);
    const int T = argc - 3;
    int64_t *numel = (int64_t *)malloc(sizeof(int64_t) * (size_t)T);
    for (int t = 0; t < T; ++t) numel[t] = atoll(argv[3 + t]);

    odc_layout_t *L = NULL;
    CHECK_ODC(odc_init_layout(R, T, numel, 0, &L));
    const size_t arena = (size_t)odc_rank_arena_elems(L), full_n = (size_t)odc_full_elems(L);
    printf("R=%d T=%d arena=%zu full=%zu\n", R, T, arena, full_n);

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    uint32_t seed = 12345u;

    /* parameter arenas: every slot random (padding included: it must never reach the output) */
    uint16_t *h_arenas = (uint16_t *)malloc(2 * arena * (size_t)R);
    for (size_t i = 0; i < arena * (size_t)R; ++i) h_arenas[i] = some_bf16(&seed);
    void **d_params = (void **)malloc(sizeof(void *) * (size_t)R);
    void **d_acc = (void **)malloc(sizeof(void *) * (size_t)R);
    void **d_out = (void **)malloc(sizeof(void *) * (size_t)R);
    float *h_acc = (float *)malloc(4 * arena * (size_t)R);
    for (size_t i = 0; i < arena * (size_t)R; ++i) h_acc[i] = -7.5f;   /* sentinel */
    for (int r = 0; r < R; ++r) {
        CHECK_HIP(hipMalloc(&d_params[r], 2 * arena));
        CHECK_HIP(hipMalloc(&d_acc[r], 4 * arena));
        CHECK_HIP(hipMalloc(&d_out[r], 4 * arena));
        CHECK_HIP(hipMemcpy(d_params[r], h_arenas + arena * (size_t)r, 2 * arena, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemcpy(d_acc[r], h_acc + arena * (size_t)r, 4 * arena, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemcpy(d_out[r], h_acc + arena * (size_t)r, 4 * arena, hipMemcpyHostToDevice));
    }
    uint16_t *h_full = (uint16_t *)malloc(2 * full_n);
    for (size_t i = 0; i < full_n; ++i) h_full[i] = 0xBEEF;
    void *d_full, *d_grad;
    CHECK_HIP(hipMalloc(&d_full, 2 * full_n));
    CHECK_HIP(hipMalloc(&d_grad, 2 * full_n));
    CHECK_HIP(hipMemcpy(d_full, h_full, 2 * full_n, hipMemcpyHostToDevice));
    if (dump(dir, "arenas.u16", h_arenas, 2 * arena * (size_t)R)) return 5;

    CHECK_ODC(odc_gather(L, (const void *const *)d_params, d_full, stream));
    CHECK_ODC(odc_reset_accum(L, d_acc, stream));
    uint16_t *h_grad = (uint16_t *)malloc(2 * full_n);
    for (int k = 0; k < 3; ++k) {
        char name[64];
        for (size_t i = 0; i < full_n; ++i) h_grad[i] = some_bf16(&seed);
        snprintf(name, sizeof name, "grad%d.u16", k);
        if (dump(dir, name, h_grad, 2 * full_n)) return 5;
        CHECK_HIP(hipStreamSynchronize(stream));   /* the previous contribution has read d_grad */
        CHECK_HIP(hipMemcpy(d_grad, h_grad, 2 * full_n, hipMemcpyHostToDevice));
        CHECK_ODC(odc_scatter_accumulate(L, d_grad, d_acc, k == 2 ? R - 1 : 0, k == 2 ? 0 : k, ODC_ORDERED, stream));
    }
    /* an out-of-order contribution is refused and enqueues nothing */
    if (odc_scatter_accumulate(L, d_grad, d_acc, 0, 0, ODC_ORDERED, stream) != ODC_ERR_ORDER) return 6;
    CHECK_ODC(odc_retrieve_grads(L, (const void *const *)d_acc, d_out, 0.25f, ODC_OUT_F32, stream));
    CHECK_HIP(hipStreamSynchronize(stream));

    CHECK_HIP(hipMemcpy(h_full, d_full, 2 * full_n, hipMemcpyDeviceToHost));
    if (dump(dir, "full.out", h_full, 2 * full_n)) return 5;
    for (int r = 0; r < R; ++r)
        CHECK_HIP(hipMemcpy(h_acc + arena * (size_t)r, d_acc[r], 4 * arena, hipMemcpyDeviceToHost));
    if (dump(dir, "acc.out", h_acc, 4 * arena * (size_t)R)) return 5;
    for (int r = 0; r < R; ++r)
        CHECK_HIP(hipMemcpy(h_acc + arena * (size_t)r, d_out[r], 4 * arena, hipMemcpyDeviceToHost));
    if (dump(dir, "retrieved.out", h_acc, 4 * arena * (size_t)R)) return 5;

    for (int r = 0; r < R; ++r) {
        CHECK_HIP(hipFree(d_params[r]));
        CHECK_HIP(hipFree(d_acc[r]));
        CHECK_HIP(hipFree(d_out[r]));
    }
    CHECK_HIP(hipFree(d_full));
    CHECK_HIP(hipFree(d_grad));
    CHECK_HIP(hipStreamDestroy(stream));
    odc_free_layout(L);
    free(numel); free(h_arenas); free(h_acc); free(h_full); free(h_grad); free(d_params); free(d_acc); free(d_out);
    printf("c_abi_check done\n");
    return 0;
}
