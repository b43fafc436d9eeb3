// The MFMA GEMM kernel behind pk_gemm_rs and pk_ag_gemm (gfx950 only).
//
// One workgroup of 4 waves (2 x 2) computes one BM x BN tile of the local product; each wave owns a
// (BM/2) x (BN/2) sub-tile as (BM/64) x (BN/64) accumulators of the 32x32 MFMA.  Per k-tile of 128 bytes
// of A-row (64 bf16 or 128 fp8):
//   * the A tile (BM x 128 B) and B tile (128*BN B) are copied global -> LDS with 16-byte direct-to-LDS
//     loads (no VGPR staging) into the buffer not being computed on (two stages);
//   * A fragments are read with ds_read_b128, B fragments with the transposing ds_read_b64_tr_b16 /
//     _tr_b8 (B is row-major K x N, the MFMA wants k-contiguous lanes);
//   * both LDS tiles are XOR-swizzled at 16-byte-chunk granularity; a direct-to-LDS load writes lane l's
//     16 bytes at base + 16*l, so the swizzle is applied by choosing which global chunk each lane fetches.
// The operands are passed to the MFMA swapped (B fragment first), which leaves each lane with four
// consecutive columns of one row, i.e. a 16-byte fp32 (8-byte bf16) store per accumulator quad.
//
// Roles of the paper's program template (section 3.2.3, appendix D): the direct-to-LDS loads are the
// loader, the MFMA loop the consumer, the epilogue the storer; the epilogue of the reduce-scatter mode
// also does the per-tile `signal` (section 3.1.3, intra-SM overlap: the transfer is issued from the
// compute workgroup itself).  In all-gather mode the workgroup does the `wait` on its chunk's flag
// before its first load (section 3.1.3, inter-SM overlap seen from the compute side).
#pragma once
#include "pk_device.h"

namespace pk {

enum { EPI_RS = 0, EPI_AG = 1 };

struct GemmArgs {
    const char* A;            // local first operand, row-major
    const char* B;            // local second operand, row-major
    int64_t lda, ldb;         // bytes per row
    int32_t n;                // columns of the local product
    int32_t ktiles;           // local k / (elements per 128-byte k-tile)
    // tile space: (P * tiles_m_shard) x tiles_n; a tile never crosses a multiple of rows_per_shard
    int32_t rows_per_shard;   // M/P
    int32_t tiles_m_shard;    // ceil(rows_per_shard / BM)
    int32_t tiles_n;
    // schedule: n_groups groups of grp_tile_rows tile rows, visited group0, group0+1, ... (mod n_groups);
    // inside a group each XCD (workgroup id mod 8) takes a contiguous run of tiles
    int32_t grp_tile_rows;
    int32_t n_groups;
    int32_t group0;
    int32_t wg_per_group;     // 8 * ceil(grp_tile_rows * tiles_n / 8)
    int32_t rank;
    // reduce-scatter epilogue
    float* partials;          // [P][rows_per_shard][n]
    float* outgoing;          // [P][rows_per_shard][n]
    uint32_t* flags_in;       // [P][flags_per_slot]
    uint32_t* flags_out;      // [P][flags_per_slot]
    int64_t slot_elems;       // rows_per_shard * n
    int64_t flags_per_slot;   // tiles_m_shard * tiles_n
    // all-gather epilogue
    uint16_t* C;              // (P*rows_per_shard) x n bf16
    const uint32_t* chunk_flags;
    const float* scale_a;     // fp8 only
    const float* scale_b;
    uint32_t epoch;
    uint32_t* status;
    uint64_t timeout_ticks;
};

template <int BM, int BN>
constexpr int gemm_lds_bytes() { return 2 * (BM * 128 + BN * 128); }

template <int BM, int BN, bool FP8, int EPI>
__global__ __launch_bounds__(256, 1) void gemm_kernel(const GemmArgs g) {
    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    PK_LDS char* lds = (PK_LDS char*)smem_generic;

    constexpr int TM = BM / 64, TN = BN / 64;           // 32x32 accumulators per wave: TM x TN
    constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
    constexpr int ELEM = FP8 ? 1 : 2;
    constexpr int B_ROWS = FP8 ? 128 : 64;               // k-rows in a B tile
    constexpr int B_ROW_BYTES = BN * ELEM;
    constexpr int CPR = B_ROW_BYTES / 16;                // 16-byte chunks per B tile row
    constexpr int RPI = 64 / CPR;                        // B rows covered by one wave-wide load
    constexpr int NA = BM / 32, NB = BN / 32;            // wave-wide loads per thread per k-tile
    constexpr int KS = FP8 ? 2 : 4;                      // MFMA k-steps per k-tile
    constexpr int BAND = 4;                              // tile rows swept column-major inside a group
    static_assert(CPR >= 8 && RPI >= 1, "tile too narrow");

    const int tid = threadIdx.x;
    const int l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;
    const int h = l >> 5;

    // ---- which tile (paper listing: interpret_task) ----
    const int gi = blockIdx.x / g.wg_per_group;
    const int u = blockIdx.x - gi * g.wg_per_group;
    const int G = g.grp_tile_rows * g.tiles_n;
    const int t = (u & 7) * (g.wg_per_group >> 3) + (u >> 3);
    if (t >= G) return;
    const int band = t / (BAND * g.tiles_n);
    const int rem = t - band * BAND * g.tiles_n;
    const int rows_in_band = min(BAND, g.grp_tile_rows - band * BAND);
    const int tc = rem / rows_in_band;
    const int tr = band * BAND + (rem - tc * rows_in_band);
    int grp = g.group0 + gi;
    if (grp >= g.n_groups) grp -= g.n_groups;
    const int tile_row = grp * g.grp_tile_rows + tr;
    const int q = tile_row / g.tiles_m_shard;            // destination rank (RS) / source chunk (AG)
    const int tmi = tile_row - q * g.tiles_m_shard;
    const int row0 = q * g.rows_per_shard + tmi * BM;
    const int row_end = (q + 1) * g.rows_per_shard;
    const int col0 = tc * BN;

    // ---- all-gather: wait until the chunk this tile reads has landed ----
    if constexpr (EPI == EPI_AG) {
        if (q != g.rank) {
            int late = 0;
            if (tid == 0) {
                late = flag_wait(g.chunk_flags + q, g.epoch, g.timeout_ticks) ? 0 : 1;
                if (late) report_timeout(g.status, (uint32_t)q, 1u);
            }
            if (__syncthreads_or(late)) return;
            acquire_agent();
        }
    }

    // ---- per-lane global source addresses of the direct-to-LDS loads ----
    const char* a_ptr[NA];
    {
        const int r_in = l >> 3, cp = l & 7;
        const int gchunk = cp ^ (r_in ^ (w & 1));        // swizzle fA(r) = (r & 7) ^ ((r >> 3) & 1)
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            const int r = 32 * j + 8 * w + r_in;
            const int grow = min(row0 + r, row_end - 1);
            a_ptr[j] = g.A + (int64_t)grow * g.lda + gchunk * 16;
        }
    }
    const char* b_ptr[NB];
    {
        const int kr_in = l / CPR, cp = l % CPR;
        const int n_bytes = g.n * ELEM;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int kr = (j * 4 + w) * RPI + kr_in;
            const int sw = FP8 ? 2 * ((kr & 7) % (CPR / 2))
                               : 4 * (((kr & 3) | ((kr >> 1) & 4)) % (CPR / 4));
            int colbyte = col0 * ELEM + (cp ^ sw) * 16;
            if (colbyte >= n_bytes) colbyte = n_bytes - 16;   // edge tile: fetch valid memory, never stored
            b_ptr[j] = g.B + (int64_t)kr * g.ldb + colbyte;
        }
    }
    const int64_t b_step = (int64_t)B_ROWS * g.ldb;

    auto issue_loads = [&](int stage) {
        PK_LDS char* sa = lds + stage * STAGE + w * 1024;
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            __builtin_amdgcn_global_load_lds((PK_GLOBAL const void*)a_ptr[j], (PK_LDS void*)(sa + j * 4096), 16, 0, 0);
            a_ptr[j] += 128;
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            __builtin_amdgcn_global_load_lds((PK_GLOBAL const void*)b_ptr[j], (PK_LDS void*)(sa + A_BYTES + j * 4096), 16, 0, 0);
            b_ptr[j] += b_step;
        }
    };

    // ---- per-lane LDS fragment addresses ----
    const int fa = (l & 7) ^ ((l >> 3) & 1);
    const uint32_t a_row_off = (uint32_t)(wm * (BM / 2) + (l & 31)) * 128;
    const int s16 = l & 15, nhalf = (l >> 4) & 1;
    uint32_t b_off[TN];
    if constexpr (!FP8) {
        const int krow_base = 8 * h + (s16 >> 2);
        const int gsw = ((s16 >> 2) | (h << 2)) % (CPR / 4);
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) {
            const int c = wn * (BN / 16) + tj * 4 + 2 * nhalf + ((s16 & 3) >> 1);
            b_off[tj] = (uint32_t)(A_BYTES + krow_base * B_ROW_BYTES + (c ^ (4 * gsw)) * 16 + (s16 & 1) * 8);
        }
    } else {
        const int krow_base = 32 * h + (s16 >> 1);
        const int gsw = ((s16 >> 1) & 7) % (CPR / 2);
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) {
            const int c = wn * (BN / 32) + tj * 2 + nhalf;
            b_off[tj] = (uint32_t)(A_BYTES + krow_base * B_ROW_BYTES + (c ^ (2 * gsw)) * 16 + (s16 & 1) * 8);
        }
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // ---- main loop: two LDS stages, one barrier per k-tile ----
    issue_loads(0);
    __builtin_amdgcn_s_waitcnt(PK_WAIT_VMCNT0);
    __syncthreads();

    for (int kt = 0; kt < g.ktiles; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < g.ktiles) issue_loads(cur ^ 1);
        PK_LDS char* st = lds + cur * STAGE;

#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            if constexpr (!FP8) {
                bf16x8 af[TM], bfr[TN];
                const uint32_t ao = a_row_off + (uint32_t)((((h ^ fa) ^ (2 * kk)) & 7) * 16);
#pragma unroll
                for (int ti = 0; ti < TM; ++ti)
                    af[ti] = *(PK_LDS bf16x8*)(st + ao + ti * 4096);
#pragma unroll
                for (int tj = 0; tj < TN; ++tj) {
                    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (PK_LDS s16x4*)(st + b_off[tj] + (16 * kk) * B_ROW_BYTES));
                    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (PK_LDS s16x4*)(st + b_off[tj] + (16 * kk + 4) * B_ROW_BYTES));
                    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    bfr[tj] = __builtin_bit_cast(bf16x8, both);
                }
#pragma unroll
                for (int ti = 0; ti < TM; ++ti)
#pragma unroll
                    for (int tj = 0; tj < TN; ++tj)
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[tj], af[ti], acc[ti][tj], 0, 0, 0);
            } else {
                i32x8 af[TM], bfr[TN];
                const uint32_t ao0 = a_row_off + (uint32_t)(((((2 * h) ^ fa) ^ (4 * kk)) & 7) * 16);
                const uint32_t ao1 = a_row_off + (uint32_t)(((((2 * h + 1) ^ fa) ^ (4 * kk)) & 7) * 16);
#pragma unroll
                for (int ti = 0; ti < TM; ++ti) {
                    i32x4 x0 = *(PK_LDS i32x4*)(st + ao0 + ti * 4096);
                    i32x4 x1 = *(PK_LDS i32x4*)(st + ao1 + ti * 4096);
                    af[ti] = __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int tj = 0; tj < TN; ++tj) {
                    i32x2 p[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        p[r] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                            (PK_LDS i32x2*)(st + b_off[tj] + (64 * kk + 8 * r) * B_ROW_BYTES));
                    i32x4 q0 = __builtin_shufflevector(p[0], p[1], 0, 1, 2, 3);
                    i32x4 q1 = __builtin_shufflevector(p[2], p[3], 0, 1, 2, 3);
                    bfr[tj] = __builtin_shufflevector(q0, q1, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int ti = 0; ti < TM; ++ti)
#pragma unroll
                    for (int tj = 0; tj < TN; ++tj)
                        acc[ti][tj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                            bfr[tj], af[ti], acc[ti][tj], 0, 0, 0, 0, 0, 0);
            }
        }
        __builtin_amdgcn_s_waitcnt(PK_WAIT_VMCNT0);
        __syncthreads();
    }

    // ---- epilogue (the storer): lane holds rows (l & 31), columns 8*b + 4*h + {0..3} of each 32x32 block ----
    float scale = 1.f;
    if constexpr (FP8) scale = g.scale_a[0] * g.scale_b[0];
    const int row_l = row0 + wm * (BM / 2) + (l & 31);
    const int col_l = col0 + wn * (BN / 2) + 4 * h;

    if constexpr (EPI == EPI_RS) {
        float* dst = (q == g.rank) ? g.partials + (int64_t)g.rank * g.slot_elems
                                   : g.outgoing + (int64_t)q * g.slot_elems;
        const int shard_row0 = q * g.rows_per_shard;
#pragma unroll
        for (int ti = 0; ti < TM; ++ti) {
            const int row = row_l + ti * 32;
            if (row < row_end) {
                float* drow = dst + (int64_t)(row - shard_row0) * g.n;
#pragma unroll
                for (int tj = 0; tj < TN; ++tj)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int col = col_l + tj * 32 + 8 * b;
                        if (col < g.n) {
                            f32x4 v = {acc[ti][tj][4 * b] * scale, acc[ti][tj][4 * b + 1] * scale,
                                       acc[ti][tj][4 * b + 2] * scale, acc[ti][tj][4 * b + 3] * scale};
                            *(f32x4*)(drow + col) = v;
                        }
                    }
            }
        }
        // signal: every wave's stores are released at device scope before the flag is published
        release_agent();
        __syncthreads();
        if (tid == 0) {
            uint32_t* flags = (q == g.rank) ? g.flags_in + (int64_t)g.rank * g.flags_per_slot
                                            : g.flags_out + (int64_t)q * g.flags_per_slot;
            flag_signal(flags + (int64_t)tmi * g.tiles_n + tc, g.epoch);
        }
    } else {
#pragma unroll
        for (int ti = 0; ti < TM; ++ti) {
            const int row = row_l + ti * 32;
            if (row < row_end) {
                uint16_t* drow = g.C + (int64_t)row * g.n;
#pragma unroll
                for (int tj = 0; tj < TN; ++tj)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int col = col_l + tj * 32 + 8 * b;
                        if (col < g.n) {
                            bf16x4 v = {(__bf16)(acc[ti][tj][4 * b] * scale), (__bf16)(acc[ti][tj][4 * b + 1] * scale),
                                        (__bf16)(acc[ti][tj][4 * b + 2] * scale), (__bf16)(acc[ti][tj][4 * b + 3] * scale)};
                            *(bf16x4*)(drow + col) = v;
                        }
                    }
            }
        }
    }
}

}  // namespace pk
