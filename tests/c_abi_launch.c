/* A plain C program that drives both hot-path entry points of libpk.so on a GPU through include/pk.h and the HIP
 * runtime's C interface alone: device buffers from hipMalloc, no Python, no torch.  Operands hold -1, 0 and 1 so that
 * every product sum is a small integer, exact in fp32: the expected bits are computed here with integer loops, rounded
 * to bf16 (nearest even) and compared bit for bit.  pk_c_abi_launch() returns 0 on success; built as a shared object it
 * is called from the test process, with PK_C_ABI_LAUNCH_MAIN defined it is a program of its own. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "pk.h"

#define CHECK_HIP(x)                                                                  \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_)); \
            return 100;                                                               \
        }                                                                             \
    } while (0)
#define CHECK_PK(x)                                                                          \
    do {                                                                                     \
        pk_status s_ = (x);                                                                  \
        if (s_ != PK_OK) {                                                                   \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, pk_status_str((int)s_));      \
            return 101;                                                                      \
        }                                                                                    \
    } while (0)

static uint32_t lcg_state = 12345u;
static int tri(void) { /* -1, 0 or 1 */
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (int)((lcg_state >> 16) % 3u) - 1;
}
static uint16_t bf16_of_small_int(int v) { /* round to nearest even; v is exact in fp32 */
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

static int run_ag_gemm(void) {
    enum { P = 2, RANK = 1, M = 512, N = 1024, K = 256, NL = N / P };
    static int8_t a[M * K], b[K * NL];
    static uint16_t ha[M * K], hb[K * NL], hc[M * NL];
    uint32_t hflags[P] = {7u, 7u}, hstatus[PK_STATUS_WORDS];
    void *dA, *dB, *dC, *dflags, *dstatus;
    for (int i = 0; i < M * K; ++i) ha[i] = bf16_of_small_int(a[i] = (int8_t)tri());
    for (int i = 0; i < K * NL; ++i) hb[i] = bf16_of_small_int(b[i] = (int8_t)tri());
    CHECK_HIP(hipMalloc(&dA, sizeof ha));
    CHECK_HIP(hipMalloc(&dB, sizeof hb));
    CHECK_HIP(hipMalloc(&dC, sizeof hc));
    CHECK_HIP(hipMalloc(&dflags, sizeof hflags));
    CHECK_HIP(hipMalloc(&dstatus, sizeof hstatus));
    CHECK_HIP(hipMemcpy(dA, ha, sizeof ha, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dB, hb, sizeof hb, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dflags, hflags, sizeof hflags, hipMemcpyHostToDevice)); /* every chunk has landed at epoch 7 */
    CHECK_HIP(hipMemset(dC, 0xFF, sizeof hc));
    CHECK_HIP(hipMemset(dstatus, 0, sizeof hstatus));
    CHECK_PK(pk_ag_gemm(P, RANK, M, N, K, PK_BF16, dA, dB, NULL, NULL, (const uint32_t*)dflags, 7u, dC, 0, PK_ACT_NONE,
                        PK_B_ROW_MAJOR, NULL, 0, (uint32_t*)dstatus, 2000000, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(hc, dC, sizeof hc, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hstatus, dstatus, sizeof hstatus, hipMemcpyDeviceToHost));
    if (hstatus[0] != 0) {
        fprintf(stderr, "ag_gemm: device status %u\n", hstatus[0]);
        return 1;
    }
    for (int r = 0; r < M; ++r)
        for (int c = 0; c < NL; ++c) {
            int s = 0;
            for (int k = 0; k < K; ++k) s += a[r * K + k] * b[k * NL + c];
            if (hc[r * NL + c] != bf16_of_small_int(s)) {
                fprintf(stderr, "ag_gemm: C[%d][%d] = 0x%04x, expected 0x%04x (%d)\n", r, c, hc[r * NL + c], bf16_of_small_int(s), s);
                return 2;
            }
        }
    CHECK_HIP(hipFree(dA));
    CHECK_HIP(hipFree(dB));
    CHECK_HIP(hipFree(dC));
    CHECK_HIP(hipFree(dflags));
    CHECK_HIP(hipFree(dstatus));
    return 0;
}

static int run_gemm_rs(void) {
    enum { P = 2, RANK = 0, M = 512, N = 264, K = 512, KL = K / P, MP = M / P }; /* N = 264: a ragged column tile */
    static int8_t a[M * KL], b[KL * N];
    static uint16_t ha[M * KL], hb[KL * N], hout[MP * N];
    static float hpart[P * MP * N], hgo[P * MP * N];
    static int peer[MP * N];
    uint32_t hstatus[PK_STATUS_WORDS], *hflags;
    void *dA, *dB, *dpart, *dgo, *dfin, *dfout, *dout, *dstatus;
    pk_plan plan;
    size_t flag_bytes;
    CHECK_PK(pk_gemm_rs_plan(P, M, N, K, PK_BF16, &plan));
    flag_bytes = (size_t)P * (size_t)plan.flags_per_slot * sizeof(uint32_t);
    hflags = (uint32_t*)malloc(flag_bytes);
    if (!hflags) return 102;
    for (int i = 0; i < M * KL; ++i) ha[i] = bf16_of_small_int(a[i] = (int8_t)tri());
    for (int i = 0; i < KL * N; ++i) hb[i] = bf16_of_small_int(b[i] = (int8_t)tri());
    memset(hpart, 0, sizeof hpart);
    for (int i = 0; i < MP * N; ++i) hpart[(1 - RANK) * MP * N + i] = (float)(peer[i] = 3 * tri()); /* the peer's slot, landed */
    for (size_t i = 0; i < flag_bytes / 4; ++i)                                                     /* at epoch 3 */
        hflags[i] = (int)(i / (size_t)plan.flags_per_slot) == RANK ? 0u : 3u;                       /* own slot: the call signals it */
    CHECK_HIP(hipMalloc(&dA, sizeof ha));
    CHECK_HIP(hipMalloc(&dB, sizeof hb));
    CHECK_HIP(hipMalloc(&dpart, sizeof hpart));
    CHECK_HIP(hipMalloc(&dgo, sizeof hgo));
    CHECK_HIP(hipMalloc(&dfin, flag_bytes));
    CHECK_HIP(hipMalloc(&dfout, flag_bytes));
    CHECK_HIP(hipMalloc(&dout, sizeof hout));
    CHECK_HIP(hipMalloc(&dstatus, sizeof hstatus));
    CHECK_HIP(hipMemcpy(dA, ha, sizeof ha, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dB, hb, sizeof hb, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dpart, hpart, sizeof hpart, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dfin, hflags, flag_bytes, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(dfout, 0, flag_bytes));
    CHECK_HIP(hipMemset(dgo, 0, sizeof hgo));
    CHECK_HIP(hipMemset(dout, 0xFF, sizeof hout));
    CHECK_HIP(hipMemset(dstatus, 0, sizeof hstatus));
    CHECK_PK(pk_gemm_rs(P, RANK, M, N, K, PK_BF16, dA, dB, NULL, NULL, dpart, dgo, (uint32_t*)dfin, (uint32_t*)dfout, 3u, dout,
                        PK_PHASE_ALL, 0, PK_PARTIAL_F32, PK_B_ROW_MAJOR, NULL, 0, (uint32_t*)dstatus, 2000000, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(hout, dout, sizeof hout, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hgo, dgo, sizeof hgo, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hflags, dfout, flag_bytes, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hstatus, dstatus, sizeof hstatus, hipMemcpyDeviceToHost));
    if (hstatus[0] != 0) {
        fprintf(stderr, "gemm_rs: device status %u\n", hstatus[0]);
        return 3;
    }
    for (int r = 0; r < M; ++r)
        for (int c = 0; c < N; ++c) {
            int s = 0, q = r / MP, rr = r % MP;
            for (int k = 0; k < KL; ++k) s += a[r * KL + k] * b[k * N + c];
            if (q == RANK) { /* own block: reduced with the peer's slot */
                uint16_t want = bf16_of_small_int(s + peer[rr * N + c]);
                if (hout[rr * N + c] != want) {
                    fprintf(stderr, "gemm_rs: out[%d][%d] = 0x%04x, expected 0x%04x\n", rr, c, hout[rr * N + c], want);
                    return 4;
                }
            } else if (hgo[(q * MP + rr) * N + c] != (float)s) { /* the peer's block: raw fp32 sums in its outgoing slot */
                fprintf(stderr, "gemm_rs: outgoing[%d][%d][%d] = %g, expected %d\n", q, rr, c, hgo[(q * MP + rr) * N + c], s);
                return 5;
            }
        }
    { /* every tile of the outgoing slot was signalled at the epoch */
        int tiles = ((MP + plan.tile_m - 1) / plan.tile_m) * ((N + plan.tile_n - 1) / plan.tile_n), seen = 0;
        for (int i = 0; i < plan.flags_per_slot; ++i) seen += hflags[(1 - RANK) * plan.flags_per_slot + i] == 3u;
        if (seen < tiles) {
            fprintf(stderr, "gemm_rs: %d of %d outgoing tiles signalled\n", seen, tiles);
            return 6;
        }
    }
    free(hflags);
    CHECK_HIP(hipFree(dA));
    CHECK_HIP(hipFree(dB));
    CHECK_HIP(hipFree(dpart));
    CHECK_HIP(hipFree(dgo));
    CHECK_HIP(hipFree(dfin));
    CHECK_HIP(hipFree(dfout));
    CHECK_HIP(hipFree(dout));
    CHECK_HIP(hipFree(dstatus));
    return 0;
}

int pk_c_abi_launch(void) {
    int n = 0, rc;
    CHECK_HIP(hipGetDeviceCount(&n));
    if (n < 1) {
        fprintf(stderr, "no GPU\n");
        return 77;
    }
    CHECK_HIP(hipSetDevice(0));
    printf("c launch: pk_ag_gemm\n");
    fflush(stdout);
    if ((rc = run_ag_gemm()) != 0) return rc;
    printf("c launch: pk_gemm_rs\n");
    fflush(stdout);
    if ((rc = run_gemm_rs()) != 0) return rc;
    printf("c launch ok\n");
    fflush(stdout);
    return 0;
}

#ifdef PK_C_ABI_LAUNCH_MAIN
int main(void) { return pk_c_abi_launch(); }
#endif
