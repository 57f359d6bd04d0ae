/*
 * The library used from plain C through its boundary alone (no Python, no PyTorch): device memory from the
 * HIP runtime, one pass of plan -> dispatch -> combine, and checks that need no reference implementation:
 * every slot holds its token's row, and with weights 1/k the combined output is the input bit for bit.
 *
 * Build (done by __graft_entry__.build()):
 *   gcc -std=c99 examples/c_abi_usage.c -I include -I /opt/rocm/include -D__HIP_PLATFORM_AMD__ \
 *       -L paper_2512_22036_amd -lfusco -L /opt/rocm/lib -lamdhip64 -o examples/c_abi_usage
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "fusco.h"

#define CHECK_HIP(call)                                                                        \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess) {                                                                \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));                  \
            return 2;                                                                          \
        }                                                                                      \
    } while (0)
#define CHECK_FUSCO(call)                                                                      \
    do {                                                                                       \
        int rc_ = (call);                                                                      \
        if (rc_ != FUSCO_OK) {                                                                 \
            fprintf(stderr, "%s failed: %s\n", #call, fusco_status_string(rc_));               \
            return 3;                                                                          \
        }                                                                                      \
    } while (0)

int main(void)
{
    enum { N = 1000, K = 4, E = 32, D = 8, H = 192 };   /* H bf16 elements: 384-byte rows */
    const int P = N * K;
    const size_t row_bytes = (size_t)H * 2;
    int32_t *topk = malloc(sizeof(int32_t) * P);
    uint16_t *x = malloc(row_bytes * N), *out = malloc(row_bytes * N), *expert = malloc(row_bytes * P);
    float *w = malloc(sizeof(float) * P);
    int32_t *slot_token = malloc(sizeof(int32_t) * P), *exp_off = malloc(sizeof(int32_t) * (E + 1));
    uint32_t rng = 12345u;
    int t, j, i;
    if (!topk || !x || !out || !expert || !w || !slot_token || !exp_off) return 1;
    for (t = 0; t < N; ++t) {
        /* K distinct experts per token: a random start and a stride coprime to E */
        rng = rng * 1664525u + 1013904223u;
        for (j = 0; j < K; ++j) topk[t * K + j] = (int32_t)(((rng >> 8) + (uint32_t)j * 7u) % E);
        for (j = 0; j < K; ++j) w[t * K + j] = 1.0f / K;
        for (i = 0; i < H; ++i) {
            rng = rng * 1664525u + 1013904223u;
            x[(size_t)t * H + i] = (uint16_t)(0x3C00u + ((rng >> 12) & 0x07FFu));   /* bfloat16 values of ordinary size */
        }
    }

    const size_t layout_bytes = fusco_layout_bytes(N, K, E, D), scratch_bytes = fusco_scratch_bytes(N, K, E, D);
    void *d_layout, *d_scratch, *d_topk, *d_x, *d_expert, *d_w, *d_out;
    fusco_layout L;
    int32_t status = -1;
    CHECK_HIP(hipMalloc(&d_layout, layout_bytes));
    CHECK_HIP(hipMalloc(&d_scratch, scratch_bytes));
    CHECK_HIP(hipMalloc(&d_topk, sizeof(int32_t) * P));
    CHECK_HIP(hipMalloc(&d_x, row_bytes * N));
    CHECK_HIP(hipMalloc(&d_expert, row_bytes * P));
    CHECK_HIP(hipMalloc(&d_w, sizeof(float) * P));
    CHECK_HIP(hipMalloc(&d_out, row_bytes * N));
    CHECK_HIP(hipMemcpy(d_topk, topk, sizeof(int32_t) * P, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_x, x, row_bytes * N, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_w, w, sizeof(float) * P, hipMemcpyHostToDevice));

    CHECK_FUSCO(fusco_layout_bind(&L, N, K, E, D, d_layout, layout_bytes));
    CHECK_FUSCO(fusco_plan(&L, d_topk, d_scratch, scratch_bytes, NULL));
    CHECK_FUSCO(fusco_dispatch(&L, d_x, row_bytes, NULL, 0, d_expert, NULL, NULL, NULL, 0, NULL));
    CHECK_FUSCO(fusco_combine(&L, d_expert, FUSCO_BF16, d_w, d_out, FUSCO_BF16, H, 0, NULL));
    CHECK_HIP(hipDeviceSynchronize());

    CHECK_HIP(hipMemcpy(&status, L.status, sizeof(status), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(slot_token, L.slot_token, sizeof(int32_t) * P, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(exp_off, L.exp_off, sizeof(int32_t) * (E + 1), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(expert, d_expert, row_bytes * P, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(out, d_out, row_bytes * N, hipMemcpyDeviceToHost));

    if (status != 0 || exp_off[0] != 0 || exp_off[E] != P) {
        fprintf(stderr, "bad plan: status %d, exp_off[0] %d, exp_off[E] %d\n", status, exp_off[0], exp_off[E]);
        return 4;
    }
    for (i = 0; i < P; ++i) {
        if (slot_token[i] < 0 || slot_token[i] >= N ||
            memcmp(expert + (size_t)i * H, x + (size_t)slot_token[i] * H, row_bytes) != 0) {
            fprintf(stderr, "slot %d does not hold the row of its token\n", i);
            return 5;
        }
        if (i > 0 && slot_token[i] <= slot_token[i - 1]) {
            /* token order may only restart where a new expert segment begins */
            int e, boundary = 0;
            for (e = 0; e <= E; ++e) boundary |= exp_off[e] == i;
            if (!boundary) {
                fprintf(stderr, "rows of one expert are not in ascending token order at slot %d\n", i);
                return 6;
            }
        }
    }
    if (memcmp(out, x, row_bytes * N) != 0) {
        fprintf(stderr, "combine with weights 1/k did not return the input\n");
        return 7;
    }
    printf("c_abi_usage ok: version %d, %d tokens, %d pairs\n", fusco_version(), N, P);
    hipFree(d_layout); hipFree(d_scratch); hipFree(d_topk); hipFree(d_x); hipFree(d_expert); hipFree(d_w); hipFree(d_out);
    free(topk); free(x); free(out); free(expert); free(w); free(slot_token); free(exp_off);
    return 0;
}
