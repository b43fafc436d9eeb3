// The MFMA GEMM kernel behind pk_gemm_rs and pk_ag_gemm (gfx950 only).
//
// A persistent workgroup of WM x WN waves walks over BM x BN tiles of the local product; each wave owns a
// (BM/WM) x (BN/WN) sub-tile as 32x32 MFMA accumulators.  The reduction runs in k-tiles of KB bytes of
// A-row (KB = 64 or 128: 32 or 64 bf16, 64 or 128 fp8):
//   * the A tile (BM x KB bytes) and B tile (KB*BN bytes) are copied global -> LDS with 16-byte
//     direct-to-LDS loads (no VGPR staging) into a ring of NS LDS stages, NS-1 k-tiles ahead of their use,
//     so that the loads of a k-tile have NS-1 k-tiles of time to land and are issued a few per k-tile;
//   * A fragments are read with ds_read_b128, B fragments with the transposing ds_read_b64_tr_b16 /
//     _tr_b8 (B is row-major K x N, the MFMA wants k-contiguous lanes);
//   * the A tile is XOR-swizzled at 16-byte-chunk granularity; the bf16 B tile is laid out as 64-column
//     panels (the fp8 B tile as swizzled rows); a direct-to-LDS load writes lane l's 16 bytes at
//     base + 16*l, so a layout is applied by choosing which global chunk each lane fetches;
//   * the loop is software-pipelined: the fragments of k-step s+1 are read while the MFMAs of step s issue,
//     and the single barrier of a k-tile sits before its last k-step, so the loads of a later k-tile and
//     the first fragments of the next k-tile are issued under that step's MFMAs.
// The operands are passed to the MFMA swapped (B fragment first), which leaves each lane with four
// consecutive columns of one row; the epilogue transposes through a 32 KB LDS staging area so that global
// stores are 16 bytes per lane over whole row segments of the wave's sub-tile.  The epilogue of tile t runs
// after the first loads of tile t+1 have been issued.
//
// Roles of the paper's program template (section 3.2.3, appendix D): the direct-to-LDS loads are the
// loader, the MFMA loop the consumer, the epilogue the storer; the epilogue of the reduce-scatter mode
// also does the per-tile `signal` (section 3.1.3, intra-SM overlap: the transfer is issued from the
// compute workgroup itself).  In all-gather mode the workgroup does the `wait` on its chunk's flag
// before its first load (section 3.1.3, inter-SM overlap seen from the compute side).
#pragma once
#include <type_traits>

#include "pk_device.h"

namespace pk {

// reduce-scatter with fp32 slots; all-gather of row chunks; reduce-scatter with bf16 slots; all-gather of column (K) chunks
enum { EPI_RS = 0, EPI_AG = 1, EPI_RS16 = 2, EPI_AGK = 3 };

struct GemmArgs {
    const char* A;            // local first operand, row-major
    const char* B;            // local second operand, row-major
    int64_t lda, ldb;         // bytes per row
    int32_t n;                // columns of the local product
    int32_t ktiles;           // local k in k-tiles of KB bytes of A-row
    // tile space: (P * tiles_m_shard) x tiles_n; a tile never crosses a multiple of rows_per_shard
    int32_t rows_per_shard;   // M/P
    int32_t tiles_m_shard;    // ceil(rows_per_shard / BM)
    int32_t tiles_n;
    // schedule: n_groups groups of grp_tile_rows tile rows, visited group0, group0+1, ... (mod n_groups);
    // inside a group each XCD (workgroup id mod 8) takes a contiguous run of tiles
    int32_t grp_tile_rows;
    int32_t n_groups;
    int32_t group0;
    int32_t wg_per_group;     // 8 * ceil(grp_tile_rows * tiles_n / 8): tile slots of one group
    int32_t band;             // tile rows swept column-major inside a group (1 = plain row-major)
    // scatter along the last dimension (reduce-scatter modes only; 0 = scatter along rows): destination rank from the
    // tile column, tiles_n = P * tiles_n_shard, rows_per_shard = all rows, one row shard
    int32_t cols_per_shard;   // N/P
    int32_t tiles_n_shard;    // ceil(cols_per_shard / BN)
    int32_t rank;
    // reduce-scatter epilogue
    void* partials;           // [P][rows_per_shard][n], fp32 (EPI_RS) or bf16 (EPI_RS16)
    void* outgoing;           // [P][rows_per_shard][n]
    uint32_t* flags_in;       // [P][flags_per_slot]
    uint32_t* flags_out;      // [P][flags_per_slot]
    int64_t slot_elems;       // rows_per_shard * n
    int64_t flags_per_slot;   // tiles_m_shard * tiles_n
    // all-gather epilogue
    uint16_t* C;              // (P*rows_per_shard) x n bf16
    const uint32_t* chunk_flags;
    int32_t k_chunks;         // EPI_AGK: A arrives in this many column blocks of K/k_chunks (chunk q from rank q)
    int32_t act;              // pk_activation applied to the accumulator before the bf16 rounding (all-gather mode)
    const float* scale_a;     // fp8 only
    const float* scale_b;
    uint32_t epoch;
    uint32_t* status;
    uint64_t timeout_ticks;
    // stream-K tail: the first sk_dp_slots tile slots are computed whole, one per workgroup and round; the k range of the
    // remaining ones is shared out evenly (sk_dp_slots = all slots: no such tail)
    int32_t sk_dp_slots;
    // A launch may cover a range of the problem's tile rows only: its groups span n_groups * grp_tile_rows rows that start
    // at tile row row_rot and wrap around at all_tile_rows (0 = the groups cover every row, no rotation).
    int32_t row_rot, all_tile_rows;
    char* ws_tiles;           // [gridDim.x] raw accumulator tiles of BM * BN fp32 (a workgroup's piece that does not start a tile)
    uint32_t* ws_flags;       // [gridDim.x] ready flags of those pieces (ws_epoch)
    uint32_t ws_epoch;
};

// kinds of work unit: a whole tile; the piece of a tile's k range that starts it (its owner adds the other pieces and
// runs the epilogue); any other piece (accumulators handed to the owner through ws_tiles)
enum { UNIT_FULL = 0, UNIT_HEAD = 1, UNIT_PART = 2 };

constexpr int kEpiStageBytes = 32 * 1024;   // LDS staging of the epilogue, shared out evenly to the waves

template <int BM, int BN, int KB, int NS>
constexpr int gemm_lds_bytes() { return NS * (BM + BN) * KB + kEpiStageBytes; }

// s_waitcnt immediate for vmcnt(N) lgkmcnt(0) (gfx9 encoding, expcnt left alone)
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4); }

// BT: the second operand is stored k-contiguous (N x K row-major, the transpose of the K x N matrix): its tile then has
// the layout of the A tile and its fragments come in with the same 16-byte reads, no transposing reads.
// SK: built with the stream-K tail (its code paths cost registers, so launches that share out no tile use SK = false).
template <int BM, int BN, int WM, int WN, int KB, int NS, bool FP8, int EPI, bool BT = false, bool SK = false>
__global__ __launch_bounds__(64 * WM * WN, 1) void gemm_kernel(const GemmArgs g) {
    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    PK_LDS char* lds = (PK_LDS char*)smem_generic;

    constexpr bool IS_RS = EPI == EPI_RS || EPI == EPI_RS16;
    constexpr int NW = WM * WN;                          // waves per workgroup
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;  // 32x32 accumulators per wave: TM x TN
    constexpr int A_BYTES = BM * KB, B_BYTES = BN * KB, STAGE = A_BYTES + B_BYTES;
    constexpr int ELEM = FP8 ? 1 : 2;
    constexpr int CPA = KB / 16;                         // 16-byte chunks per A tile row (8 or 4)
    constexpr int B_ROWS = KB / ELEM;                    // k-rows in a B tile
    constexpr int B_ROW_BYTES = BN * ELEM;
    constexpr int CPR = B_ROW_BYTES / 16;                // 16-byte chunks per B tile row
    constexpr int RPI = 64 / CPR;                        // B rows covered by one wave-wide load
    constexpr int NA = A_BYTES / 1024 / NW, NB = B_BYTES / 1024 / NW;   // wave-wide loads per wave per k-tile
    constexpr int NL = NA + NB;
    constexpr int KS = FP8 ? KB / 64 : KB / 32;          // MFMA k-steps per k-tile
    constexpr int EPI_OFF = NS * STAGE;                  // LDS offset of the epilogue staging area
    static_assert(KB == 64 || KB == 128, "k-tile is 64 or 128 bytes of A row");
    static_assert(KS >= 1, "a k-tile holds at least one MFMA k-step");
    static_assert(CPR >= 8 && RPI >= 1, "tile too narrow");
    static_assert(NW % 2 == 0 && NA >= 1 && NB >= 1, "wave grid does not fit the tile");
    static_assert((NS - 2) * NL <= 63, "too many loads in flight for the counter");
    typedef typename std::conditional<FP8, i32x8, bf16x8>::type frag_t;

    const int tid = threadIdx.x;
    const int l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w / WN, wn = w % WN;
    const int h = l >> 5;

    // A-tile swizzle: LDS chunk position = k-chunk ^ fA(row).
    //   128-byte rows: fA(r) = (r & 7) ^ ((r >> 3) & 1);  64-byte rows: fA(r) = ((r >> 1) & 3) ^ ((r >> 3) & 1)
    auto fA = [](int r) { return KB == 128 ? ((r & 7) ^ ((r >> 3) & 1)) : (((r >> 1) & 3) ^ ((r >> 3) & 1)); };

    // ---- per-lane LDS fragment addresses (relative to a stage) ----
    const int fa = fA(l & 31);                           // rows of a fragment differ from (l & 31) by multiples of 32
    const uint32_t a_row_off = (uint32_t)(wm * (BM / WM) + (l & 31)) * KB;
    const int s16 = l & 15, nhalf = (l >> 4) & 1;
    uint32_t b_off[TN];
    const uint32_t bt_row_off = (uint32_t)(A_BYTES + (wn * (BN / WN) + (l & 31)) * KB);   // BT: B tile = BN rows of KB bytes
    if constexpr (BT) {
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) b_off[tj] = bt_row_off + (uint32_t)(tj * 32 * KB);
    } else if constexpr (!FP8) {
        // bf16 B tile: panels of 64 columns (128 bytes per k-row, k-rows consecutive);
        // inside a row the two 32-byte pieces of each 64-byte half trade places on k-rows with bit 1 set
        static_assert((BN / WN) % 64 == 0, "a wave column covers whole 64-column panels");
        const int krow_base = 8 * h + (s16 >> 2);
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) {
            const int panel = wn * (BN / WN / 64) + (tj >> 1);
            const int piece = (2 * (tj & 1) + nhalf) ^ ((s16 >> 3) & 1);
            b_off[tj] = (uint32_t)(A_BYTES + panel * (B_ROWS * 128) + krow_base * 128 + piece * 32 + (s16 & 3) * 8);
        }
    } else {
        const int krow_base = 32 * h + (s16 >> 1);
        const int gsw = ((s16 >> 1) & 7) % (CPR / 2);
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) {
            const int c = wn * (BN / WN / 16) + tj * 2 + nhalf;
            b_off[tj] = (uint32_t)(A_BYTES + krow_base * B_ROW_BYTES + (c ^ (2 * gsw)) * 16 + (s16 & 1) * 8);
        }
    }

    // Fragment reads of k-step kk of the k-tile held in LDS stage `st`, as NU = TN + TM units in the order the
    // MFMAs need them: B fragments first, then A fragments.
    constexpr int NU = TN + TM;
    auto read_unit = [&](PK_LDS char* st, int kk, int u, frag_t (&af)[TM], frag_t (&bfr)[TN]) {
        if constexpr (BT) {
            // both operands: rows of KB bytes, 16-byte chunks XOR-swizzled by row; rows of a fragment differ by multiples of 32
            const uint32_t base = u < TN ? b_off[u] : a_row_off + (uint32_t)((u - TN) * 32 * KB);
            if constexpr (!FP8) {
                const bf16x8 v = *(PK_LDS bf16x8*)(st + base + (uint32_t)((((2 * kk + h) ^ fa) & (CPA - 1)) * 16));
                if (u < TN) bfr[u] = v;
                else af[u - TN] = v;
            } else {
                i32x4 x0 = *(PK_LDS i32x4*)(st + base + (uint32_t)((((4 * kk + 2 * h) ^ fa) & (CPA - 1)) * 16));
                i32x4 x1 = *(PK_LDS i32x4*)(st + base + (uint32_t)((((4 * kk + 2 * h + 1) ^ fa) & (CPA - 1)) * 16));
                const i32x8 v = __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7);
                if (u < TN) bfr[u] = v;
                else af[u - TN] = v;
            }
        } else if constexpr (!FP8) {
            if (u < TN) {
                const int tj = u;
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (PK_LDS s16x4*)(st + b_off[tj] + (16 * kk) * 128));
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (PK_LDS s16x4*)(st + b_off[tj] + (16 * kk + 4) * 128));
                s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                bfr[tj] = __builtin_bit_cast(bf16x8, both);
            } else {
                const int ti = u - TN;
                const uint32_t ao = a_row_off + (uint32_t)((((2 * kk + h) ^ fa) & (CPA - 1)) * 16);
                af[ti] = *(PK_LDS bf16x8*)(st + ao + ti * 32 * KB);
            }
        } else {
            if (u < TN) {
                const int tj = u;
                i32x2 p[4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    p[r] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                        (PK_LDS i32x2*)(st + b_off[tj] + (64 * kk + 8 * r) * B_ROW_BYTES));
                i32x4 q0 = __builtin_shufflevector(p[0], p[1], 0, 1, 2, 3);
                i32x4 q1 = __builtin_shufflevector(p[2], p[3], 0, 1, 2, 3);
                bfr[tj] = __builtin_shufflevector(q0, q1, 0, 1, 2, 3, 4, 5, 6, 7);
            } else {
                const int ti = u - TN;
                const uint32_t ao0 = a_row_off + (uint32_t)((((4 * kk + 2 * h) ^ fa) & (CPA - 1)) * 16);
                const uint32_t ao1 = a_row_off + (uint32_t)((((4 * kk + 2 * h + 1) ^ fa) & (CPA - 1)) * 16);
                i32x4 x0 = *(PK_LDS i32x4*)(st + ao0 + ti * 32 * KB);
                i32x4 x1 = *(PK_LDS i32x4*)(st + ao1 + ti * 32 * KB);
                af[ti] = __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        }
    };
    auto load_frags = [&](PK_LDS char* st, int kk, frag_t (&af)[TM], frag_t (&bfr)[TN]) {
#pragma unroll
        for (int u = 0; u < NU; ++u) read_unit(st, kk, u, af, bfr);
    };

    f32x16 acc[TM][TN];
    auto mfma_one = [&](int ti, int tj, const frag_t (&af)[TM], const frag_t (&bfr)[TN]) {
        if constexpr (!FP8)
            acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[tj], af[ti], acc[ti][tj], 0, 0, 0);
        else
            acc[ti][tj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bfr[tj], af[ti], acc[ti][tj], 0, 0, 0, 0, 0, 0);
    };

    // tile bookkeeping carried from one iteration to the next (the epilogue of a tile runs one iteration late)
    int p_q = -1, p_flag = 0, p_row0 = 0, p_row_end = 0, p_col0 = 0, p_col_end = 0;
    int p_kind = UNIT_FULL, p_part_lo = 0, p_tile_end = 0;
    bool p_dead = false;                                 // the previous tile was given up (a wait timed out): no signal
    const int slots_total = g.wg_per_group * g.n_groups;
    const int G = g.grp_tile_rows * g.tiles_n;
    float scale = 1.f;
    if constexpr (FP8) scale = g.scale_a[0] * g.scale_b[0];
    // the non-linearity between the two GEMMs of the MLP (paper section 4.1), fused into the all-gather epilogue
    auto activate = [&](float x) -> float {
        switch (g.act) {
            case PK_ACT_RELU: return fmaxf(x, 0.f);
            case PK_ACT_GELU_TANH: return 0.5f * x * (1.f + tanhf(0.7978845608028654f * (x + 0.044715f * x * x * x)));
            case PK_ACT_SILU: return x / (1.f + expf(-x));
            default: return x;
        }
    };

    auto signal_prev = [&]() {   // paper appendix C `signal` for the tile whose stores have completed
        if (SK && p_kind == UNIT_PART) {
            if (tid == 0) flag_publish(g.ws_flags + blockIdx.x, g.ws_epoch);
        } else if constexpr (IS_RS) {
            if (tid == 0 && !p_dead) {
                uint32_t* flags = (p_q == g.rank) ? g.flags_in + (int64_t)g.rank * g.flags_per_slot
                                                  : g.flags_out + (int64_t)p_q * g.flags_per_slot;
                flag_publish(flags + p_flag, g.epoch);
            }
        }
    };

    // chunks of A known to have landed (the own one, and those this workgroup has waited for): EPI_AG, EPI_AGK
    // workgroup 0 reports how long it ran, in ticks of the 100 MHz wall clock and in core-clock cycles, and how many of
    // those cycles its main loops took: status[4..7] (the ratio of the first two is the clock the chip held)
    const uint64_t t_wall0 = wall_clock64(), t_core0 = clock64();
    uint64_t t_loops = 0;
    uint32_t n_tiles_done = 0;
    uint64_t seen_chunks = 1ull << (g.rank & 63);
    const uint64_t all_chunks = g.k_chunks >= 64 ? ~0ull : (1ull << g.k_chunks) - 1;
    int v = blockIdx.x;
    // EPI_AG: a slot whose chunk has not landed when it is first visited is put aside (bit i = this workgroup's i-th slot)
    // and taken up again, now waiting, once the workgroup has gone through its other slots: tiles of chunks that are
    // already there never queue behind a late one.  Slots beyond the 64th wait on the spot.
    uint64_t deferred = 0;
    int visit = 0;
    // Stream-K tail (the tile slots from sk_dp_slots on): slot sk_dp_slots + 8*i + x belongs to XCD x = workgroup id
    // mod 8, whose W workgroups share the R * KT k-tiles of its R slots evenly, workgroup j of the XCD taking
    // [sk_bnd(j), sk_bnd(j+1)).  A range is cut at tile boundaries into pieces; cuts closer than SK_MINP k-tiles to a
    // tile boundary are moved onto it.  A workgroup has at most one piece that does not start a tile, its first.
    constexpr int SK_Q = (KS % 2) ? 2 : 1, SK_MINP = 2 * NS;
    const int KT = g.ktiles;
    const int sk_x = blockIdx.x & 7, sk_j = blockIdx.x >> 3, sk_W = gridDim.x >> 3;
    const int sk_R = SK ? (slots_total - g.sk_dp_slots) >> 3 : 0;
    auto sk_bnd = [&](int j) -> int {
        int b = (int)((int64_t)sk_R * KT * j / sk_W);
        b -= b % SK_Q;
        const int r = b % KT;
        if (r < SK_MINP) b -= r;
        else if (KT - r < SK_MINP) b += KT - r;
        return b;
    };
    int sk_c = 0, sk_e = 0;
    if (sk_R > 0) {
        sk_c = sk_bnd(sk_j);
        sk_e = sk_bnd(sk_j + 1);
    }
    for (;;) {
        // ---- which tile (paper listing: interpret_task) ----
        int q = 0, tmi = 0, tc = 0, row0 = 0, row_end = 0, col0 = 0, col_end = 0, flag = 0;
        int kind = UNIT_FULL, kt0 = 0, nkt = KT, part_lo = 0, tile_end = 0;
        bool have = false;
        for (;;) {
            int slot, slot_index = 64;
            bool may_defer = false;
            if (v < g.sk_dp_slots) {
                slot = v;
                slot_index = visit;
                v += gridDim.x;
                ++visit;
                may_defer = (EPI == EPI_AG) && slot_index < 64;
            } else if ((EPI == EPI_AG) && deferred != 0) {
                slot_index = __builtin_ctzll(deferred);
                deferred &= deferred - 1;
                slot = (int)blockIdx.x + slot_index * (int)gridDim.x;
            } else if (SK && sk_c < sk_e) {
                const int i = sk_c / KT;
                tile_end = (i + 1) * KT;
                const int e = min(sk_e, tile_end);
                slot = g.sk_dp_slots + 8 * i + sk_x;
                kt0 = sk_c - i * KT;
                nkt = e - sk_c;
                kind = kt0 != 0 ? UNIT_PART : (nkt == KT ? UNIT_FULL : UNIT_HEAD);
                part_lo = sk_j + 1;          // the workgroups of this XCD that may hold the other pieces of a tile started here
                sk_c = e;
            } else {
                break;
            }
            const int gi = slot / g.wg_per_group;
            const int u = slot - gi * g.wg_per_group;
            const int t = (u & 7) * (g.wg_per_group >> 3) + (u >> 3);
            if (t >= G) continue;
            const int BAND = g.band > 0 ? g.band : 1;
            const int band = t / (BAND * g.tiles_n);
            const int rem = t - band * BAND * g.tiles_n;
            const int rows_in_band = min(BAND, g.grp_tile_rows - band * BAND);
            tc = rem / rows_in_band;
            const int tr = band * BAND + (rem - tc * rows_in_band);
            int grp = g.group0 + gi;
            if (grp >= g.n_groups) grp -= g.n_groups;
            int tile_row = grp * g.grp_tile_rows + tr;
            if (g.all_tile_rows > 0) {
                tile_row += g.row_rot;
                if (tile_row >= g.all_tile_rows) tile_row -= g.all_tile_rows;
            }
            q = tile_row / g.tiles_m_shard;              // destination rank (RS) / source chunk (AG)
            tmi = tile_row - q * g.tiles_m_shard;
            row0 = q * g.rows_per_shard + tmi * BM;
            row_end = (q + 1) * g.rows_per_shard;
            col0 = tc * BN;
            col_end = g.n;
            flag = tmi * g.tiles_n + tc;
            if constexpr (IS_RS) {
                if (g.cols_per_shard > 0) {              // destination rank from the tile column (q was 0: one row shard)
                    q = tc / g.tiles_n_shard;
                    const int tci = tc - q * g.tiles_n_shard;
                    col0 = q * g.cols_per_shard + tci * BN;
                    col_end = (q + 1) * g.cols_per_shard;
                    flag = tmi * g.tiles_n_shard + tci;
                }
            }
            have = true;

            // all-gather: the chunk this tile reads must have landed (paper appendix C `wait`)
            if constexpr (EPI == EPI_AG) {
                if (!((seen_chunks >> (q & 63)) & 1)) {
                    // lane 0 polls; the verdict (0 landed, 1 timed out, 2 not yet: put the slot aside) goes through a
                    // word of the (idle) epilogue staging area, since the kernel leaves no LDS for a static variable
                    PK_LDS int* verdict = (PK_LDS int*)(lds + EPI_OFF);
                    if (tid == 0) {
                        int vd = 0;
                        if (!flag_ready(g.chunk_flags + q, g.epoch)) {
                            if (may_defer) {
                                vd = 2;
                            } else if (!flag_wait(g.chunk_flags + q, g.epoch, g.timeout_ticks)) {
                                report_timeout(g.status, (uint32_t)q, 1u);
                                vd = 1;
                            }
                        }
                        *verdict = vd;
                    }
                    __syncthreads();
                    const int vd_all = *verdict;
                    __syncthreads();
                    if (vd_all == 2) {
                        deferred |= 1ull << slot_index;
                        have = false;
                        continue;
                    }
                    if (vd_all == 1) {
                        have = false;                       // drain: this tile's and the later tiles' rows stay untouched
                        v = slots_total;
                        deferred = 0;
                        sk_c = sk_e;
                        break;
                    }
                    acquire_agent();
                    if (q < 64) seen_chunks |= 1ull << q;
                }
            }
            break;
        }
        uint32_t a_voff[NA], b_voff[NB];           // per-lane byte offsets from the k-tile base pointers
        const char* a_base = g.A;                    // wave-uniform, advanced by one k-tile per issue
        const char* b_base = g.B;
        const int64_t b_step = BT ? (int64_t)KB : (int64_t)B_ROWS * g.ldb;   // bytes from one k-tile of B to the next
        // k-tiles handled between two pipeline fills: all of them, or one column chunk of A at a time (EPI_AGK, own
        // chunk); once this workgroup has seen every chunk, its later tiles run the whole k range in one go
        const bool by_chunk = (EPI == EPI_AGK) && seen_chunks != all_chunks;
        const int seg_ktiles = by_chunk ? g.ktiles / g.k_chunks : nkt;
        if (by_chunk) {
            a_base += (int64_t)g.rank * seg_ktiles * KB;
            b_base += (int64_t)g.rank * seg_ktiles * b_step;
        } else {
            a_base += (int64_t)kt0 * KB;             // a piece of a stream-K tile starts at k-tile kt0
            b_base += (int64_t)kt0 * b_step;
        }
        if (have) {
            // per-lane global source addresses of the direct-to-LDS loads.  Wave-wide load j of wave w fills
            // the 1 KB LDS block j*NW + w of the A (or B) tile.
            {
                const int r_in = l / CPA, cp = l % CPA;
#pragma unroll
                for (int j = 0; j < NA; ++j) {
                    const int r = (64 / CPA) * (j * NW + w) + r_in;
                    const int grow = min(row0 + r, row_end - 1);
                    a_voff[j] = (uint32_t)((int64_t)grow * g.lda + (cp ^ fA(r)) * 16);
                }
            }
            if constexpr (BT) {
                // as the A tile: 1 KB block = 64 / CPA rows (columns of the product) of KB bytes
                const int r_in = l / CPA, cp = l % CPA;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int r = (64 / CPA) * (j * NW + w) + r_in;
                    const int gcol = min(col0 + r, g.n - 1);        // edge tile: valid memory, never stored
                    b_voff[j] = (uint32_t)((int64_t)gcol * g.ldb + (cp ^ fA(r)) * 16);
                }
            } else if constexpr (!FP8) {
                // 1 KB block bi of the B tile = 8 k-rows of one 64-column panel
                const int kr_in = l >> 3, cp = l & 7;
                const int n_bytes = g.n * 2;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int bi = j * NW + w;
                    const int panel = bi / (B_ROWS / 8);
                    const int kr = (bi % (B_ROWS / 8)) * 8 + kr_in;
                    int colbyte = (col0 + panel * 64) * 2 + (cp ^ (2 * ((kr >> 1) & 1))) * 16;
                    if (colbyte >= n_bytes) colbyte = n_bytes - 16;   // edge tile: valid memory, never stored
                    b_voff[j] = (uint32_t)((int64_t)kr * g.ldb + colbyte);
                }
            } else {
                const int kr_in = l / CPR, cp = l % CPR;
                const int n_bytes = g.n;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int kr = (j * NW + w) * RPI + kr_in;
                    const int sw = 2 * ((kr & 7) % (CPR / 2));
                    int colbyte = col0 + (cp ^ sw) * 16;
                    if (colbyte >= n_bytes) colbyte = n_bytes - 16;   // edge tile: valid memory, never stored
                    b_voff[j] = (uint32_t)((int64_t)kr * g.ldb + colbyte);
                }
            }
        }
        // load number i (0 .. NL-1) of this wave for the next k-tile to fetch, into LDS stage `stage`
        const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
        auto issue_load = [&](int stage, int i) {
            const uint32_t sa = lds_base + stage * STAGE + w * 1024;
            if (i < NA) dma_load16(a_base, a_voff[i], sa + i * NW * 1024);
            else dma_load16(b_base, b_voff[i - NA], sa + A_BYTES + (i - NA) * NW * 1024);
            if (i == NL - 1) {
                a_base += KB;
                b_base += b_step;
            }
        };
        auto issue_loads = [&](int stage) {
#pragma unroll
            for (int i = 0; i < NL; ++i) issue_load(stage, i);
        };
        // the LDS stages are free here: every wave passed the last barrier of the previous tile's loop
        // after its final fragment reads were issued and waited for
        if (have) {
#pragma unroll
            for (int s = 0; s < NS; ++s)
                if (s < seg_ktiles) issue_loads(s);
        }

        // ---- epilogue of the previous tile (the storer), under the latency of the loads just issued ----
        bool skip_epilogue = false;
        if (SK && p_q >= 0 && p_kind == UNIT_PART) {
            // hand the raw accumulators to the owner of the tile: register image, 16 bytes per lane, written through
            char* wsb = g.ws_tiles + (int64_t)blockIdx.x * (BM * BN * 4) + (w * (TM * TN * 4)) * 1024 + l * 16;
#pragma unroll
            for (int ti = 0; ti < TM; ++ti)
#pragma unroll
                for (int tj = 0; tj < TN; ++tj)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        f32x4 val = {acc[ti][tj][4 * b], acc[ti][tj][4 * b + 1], acc[ti][tj][4 * b + 2], acc[ti][tj][4 * b + 3]};
                        store16_writethrough(wsb + ((ti * TN + tj) * 4 + b) * 1024, __builtin_bit_cast(i32x4, val));
                    }
            skip_epilogue = true;
        }
        if (SK && p_q >= 0 && p_kind == UNIT_HEAD) {
            // add the other pieces of this tile: those of the following workgroups of this XCD whose ranges start inside it
            for (int jp = p_part_lo; jp < sk_W; ++jp) {
                const int s0 = sk_bnd(jp);
                if (s0 >= p_tile_end) break;
                if (sk_bnd(jp + 1) == s0) continue;              // that workgroup has no work
                const int owner = jp * 8 + sk_x;
                PK_LDS int* verdict = (PK_LDS int*)(lds + EPI_OFF);
                if (tid == 0) {
                    const int late = flag_wait(g.ws_flags + owner, g.ws_epoch, g.timeout_ticks) ? 0 : 1;
                    if (late) report_timeout(g.status, (uint32_t)owner, 4u);
                    *verdict = late;
                }
                __syncthreads();
                const int late_all = *verdict;
                __syncthreads();
                if (late_all) {
                    skip_epilogue = true;                           // the tile stays unwritten and unsignalled
                    p_dead = true;
                    break;
                }
                // the piece was written through by another compute unit: read it past this XCD's L2
                const auto rsrc = __builtin_amdgcn_make_buffer_rsrc(g.ws_tiles + (int64_t)owner * (BM * BN * 4), 0, BM * BN * 4,
                                                                    0x00020000);
                const uint32_t off0 = (uint32_t)((w * (TM * TN * 4)) * 1024 + l * 16);
#pragma unroll
                for (int ti = 0; ti < TM; ++ti) {
                    f32x4 pv[TN][4];
#pragma unroll
                    for (int tj = 0; tj < TN; ++tj)
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            pv[tj][b] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                rsrc, off0 + (uint32_t)(((ti * TN + tj) * 4 + b) * 1024), 0, 1 | 2 | 16));
#pragma unroll
                    for (int tj = 0; tj < TN; ++tj)
#pragma unroll
                        for (int b = 0; b < 4; ++b)
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[ti][tj][4 * b + e] += pv[tj][b][e];
                }
            }
        }
        if (p_q >= 0 && !skip_epilogue) {
            // lane holds, for each 32x32 block, rows (l & 31) and columns 8*b + 4*h + {0..3}.  Per pass a slab of
            // ROWS_PASS rows x (BN/WN) columns goes through the wave's private staging area, then out as whole
            // row segments, 16 bytes per lane.
            PK_LDS char* stg = lds + EPI_OFF + w * (kEpiStageBytes / NW);
            constexpr int WCOLS = BN / WN;                   // columns of the wave's sub-tile
            constexpr int OUT_ELEM = (EPI == EPI_RS) ? 4 : 2;
            constexpr int ROW_BYTES = WCOLS * OUT_ELEM;
            constexpr int ROWS_PASS = (kEpiStageBytes / NW) / ROW_BYTES >= 32 ? 32 : (kEpiStageBytes / NW) / ROW_BYTES;
            static_assert(ROWS_PASS == 32 || ROWS_PASS == 16 || ROWS_PASS == 8, "staging area too small");
            constexpr int CH = ROW_BYTES / 16;               // 16-byte chunks per staged row
            constexpr int LANES_ROW = CH;                    // lanes that cover one row on the way out
            constexpr int ROWS_INSTR = 64 / LANES_ROW;       // rows written by one wave-wide store
            const int col_w0 = p_col0 + wn * WCOLS;
            char* dst_base;
            int64_t dst_pitch;
            int dst_row0;                                    // global row -> row inside the destination
            int dst_col0 = 0;                                // global column -> column inside the destination
            if constexpr (IS_RS) {
                dst_base = (p_q == g.rank) ? (char*)g.partials + (int64_t)g.rank * g.slot_elems * OUT_ELEM
                                           : (char*)g.outgoing + (int64_t)p_q * g.slot_elems * OUT_ELEM;
                if (g.cols_per_shard > 0) {
                    dst_pitch = (int64_t)g.cols_per_shard * OUT_ELEM;
                    dst_row0 = 0;
                    dst_col0 = p_q * g.cols_per_shard;
                } else {
                    dst_pitch = (int64_t)g.n * OUT_ELEM;
                    dst_row0 = p_q * g.rows_per_shard;
                }
            } else {
                dst_base = (char*)g.C;
                dst_pitch = (int64_t)g.n * 2;
                dst_row0 = 0;
            }
#pragma unroll
            for (int ti = 0; ti < TM; ++ti) {
#pragma unroll
                for (int half = 0; half < 32 / ROWS_PASS; ++half) {
                    // write: lanes whose row falls in this pass store their quads; chunk position swizzled by row
                    const int rl = l & 31;
                    if (ROWS_PASS == 32 || (rl / ROWS_PASS) == half) {
                        const int rs = rl % ROWS_PASS;
#pragma unroll
                        for (int tj = 0; tj < TN; ++tj)
#pragma unroll
                            for (int b = 0; b < 4; ++b) {
                                const int colw = tj * 32 + 8 * b + 4 * h;     // column inside the wave sub-tile
                                if constexpr (EPI == EPI_RS) {
                                    const int ch = colw >> 2;                  // 16-byte chunk (4 floats)
                                    f32x4 val = {acc[ti][tj][4 * b] * scale, acc[ti][tj][4 * b + 1] * scale,
                                                 acc[ti][tj][4 * b + 2] * scale, acc[ti][tj][4 * b + 3] * scale};
                                    *(PK_LDS f32x4*)(stg + rs * ROW_BYTES + ((ch ^ (rs & (CH - 1))) * 16)) = val;
                                } else {
                                    const int ch = colw >> 3;                  // 16-byte chunk (8 bf16)
                                    float x0 = acc[ti][tj][4 * b] * scale, x1 = acc[ti][tj][4 * b + 1] * scale,
                                          x2 = acc[ti][tj][4 * b + 2] * scale, x3 = acc[ti][tj][4 * b + 3] * scale;
                                    if constexpr (!IS_RS) if (g.act != PK_ACT_NONE) {
                                        x0 = activate(x0);
                                        x1 = activate(x1);
                                        x2 = activate(x2);
                                        x3 = activate(x3);
                                    }
                                    bf16x4 val = {(__bf16)x0, (__bf16)x1, (__bf16)x2, (__bf16)x3};
                                    *(PK_LDS bf16x4*)(stg + rs * ROW_BYTES + ((ch ^ (rs & (CH - 1))) * 16) + (h * 8)) = val;
                                }
                            }
                    }
                    // read back row-wise and store: lane -> (row = i*ROWS_INSTR + l / LANES_ROW, chunk = l % LANES_ROW)
#pragma unroll
                    for (int i = 0; i < ROWS_PASS / ROWS_INSTR; ++i) {
                        const int rs = i * ROWS_INSTR + l / LANES_ROW;
                        const int ch = l % LANES_ROW;
                        i32x4 val = *(PK_LDS i32x4*)(stg + rs * ROW_BYTES + ((ch ^ (rs & (CH - 1))) * 16));
                        const int row = p_row0 + wm * (BM / WM) + ti * 32 + half * ROWS_PASS + rs;
                        const int col = col_w0 + ch * (16 / OUT_ELEM);
                        if (row < p_row_end && col < p_col_end) {
                            char* dp = dst_base + (int64_t)(row - dst_row0) * dst_pitch + (int64_t)(col - dst_col0) * OUT_ELEM;
                            // reduce-scatter tiles are consumed by another kernel through a flag: write through
                            if constexpr (IS_RS) store16_writethrough(dp, val);
                            else __builtin_nontemporal_store(val, (i32x4*)dp);
                        }
                    }
                }
            }
        }
        if (!have) break;

#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        // the first k-tiles have landed; the previous tile's stores (same counter) are complete as well
        __builtin_amdgcn_s_waitcnt(PK_WAIT_VMCNT0);
        __syncthreads();
        if (p_q >= 0) signal_prev();

        // ---- main loop ----
        frag_t af0[TM], bf0[TN], af1[TM], bf1[TN];
        // One k-tile: KS-1 pipelined k-steps, the barrier, then the last k-step, under which the loads of
        // k-tile kt+NS (LOADS) and the first fragments of k-tile kt+1 (NEXT) are issued.  At the barrier every
        // wave has finished reading k-tile kt's stage, so it can be refilled, and k-tile kt+1 has landed: in the
        // steady state only the loads of the NS-2 k-tiles after it may still be in flight.
        // One k-step: the NM MFMAs on fragment set (ca, cb), with, pinned between them in this order, the reads
        // of the next step's fragments into (na, nb) behind the first half of the MFMAs (they then have the
        // second half of the step to arrive) and the direct-to-LDS loads of a later k-tile behind the second half.
        auto kstep = [&](const frag_t (&ca)[TM], const frag_t (&cb)[TN], frag_t (&na)[TM], frag_t (&nb)[TN],
                         PK_LDS char* rd_stage, int rd_kk, auto reads_c, int ld_stage, auto loads_c) {
            constexpr bool READS = decltype(reads_c)::value, LOADS = decltype(loads_c)::value;
            constexpr int NM = TM * TN, H = NM / 2;
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                mfma_one(i / TN, i % TN, ca, cb);
                if constexpr (READS && FP8) {
                    // 8-bit fragments are 8 registers each: two full sets next to the accumulators do not fit.  The MFMAs run
                    // row by row (ti-major), so the A fragment of row ti is dead after MFMA ti*TN + TN-1, and the next step's
                    // A fragment of that row is read right behind it, into the same registers; only the B fragments are double.
                    if (i == 0) {
#pragma unroll
                        for (int u = 0; u < TN; ++u) read_unit(rd_stage, rd_kk, u, na, nb);
                    }
                    if (i % TN == TN - 1) read_unit(rd_stage, rd_kk, TN + i / TN, na, nb);
                } else if constexpr (READS) {
                    if (i < H) {
#pragma unroll
                        for (int u = (NU * i) / H; u < (NU * (i + 1)) / H; ++u) read_unit(rd_stage, rd_kk, u, na, nb);
                    }
                }
                if constexpr (LOADS) {
                    if (i >= NM - H) {
#pragma unroll
                        for (int x = (NL * (i - (NM - H))) / H; x < (NL * (i - (NM - H) + 1)) / H; ++x)
                            issue_load(ld_stage, x);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        auto ktile = [&](int kt, auto loads_c, auto next_c, auto par_c) {
            constexpr bool LOADS = decltype(loads_c)::value;
            constexpr int P0 = decltype(par_c)::value;   // fragment set that holds this k-tile's first fragments
            const int sidx = kt % NS;
            PK_LDS char* st = lds + sidx * STAGE;
            PK_LDS char* nx = lds + (sidx + 1 == NS ? 0 : sidx + 1) * STAGE;
            // fragment set `par` is consumed, the other one refilled
            auto step = [&](auto par, PK_LDS char* rd_stage, int rd_kk, auto reads_c, int ld_stage, auto lds_c) {
                if constexpr (decltype(par)::value) kstep(af1, bf1, af0, bf0, rd_stage, rd_kk, reads_c, ld_stage, lds_c);
                else kstep(af0, bf0, af1, bf1, rd_stage, rd_kk, reads_c, ld_stage, lds_c);
            };
            if constexpr (KS >= 2) step(std::integral_constant<int, P0>{}, st, 1, std::true_type{}, 0, std::false_type{});
            if constexpr (KS >= 3) step(std::integral_constant<int, P0 ^ 1>{}, st, 2, std::true_type{}, 0, std::false_type{});
            if constexpr (KS >= 4) step(std::integral_constant<int, P0>{}, st, 3, std::true_type{}, 0, std::false_type{});
            static_assert(KS <= 4, "at most four k-steps per k-tile");
            if constexpr (LOADS) __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NS - 2) * NL));
            else __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
            __syncthreads();
            step(std::integral_constant<int, (P0 + KS - 1) & 1>{}, nx, 0, next_c, sidx, loads_c);
        };
        // the k-tiles of one pipeline fill: the first NS are in flight or landed, stage 0 holds the first
        auto run_ktiles = [&](int nkt) {
            using T = std::true_type;
            using F = std::false_type;
            using E = std::integral_constant<int, 0>;    // k-tile starts on fragment set 0
            using O = std::integral_constant<int, 1>;    // ... on set 1
            load_frags(lds, 0, af0, bf0);
            int kt = 0;
            if constexpr (KS % 2 == 0) {
                for (; kt + NS < nkt; ++kt) ktile(kt, T{}, T{}, E{});
                for (; kt + 1 < nkt; ++kt) ktile(kt, F{}, T{}, E{});
                ktile(kt, F{}, F{}, E{});
            } else {
                // odd k-steps per k-tile: the starting set alternates, so k-tiles go in pairs (nkt and NS are even: the
                // host admits only k ranges of whole 128-byte units)
                static_assert(KS % 2 == 0 || NS % 2 == 0, "pairs of k-tiles need an even ring");
                for (; kt + NS < nkt; kt += 2) {
                    ktile(kt, T{}, T{}, E{});
                    ktile(kt + 1, T{}, T{}, O{});
                }
                for (; kt + 2 < nkt; kt += 2) {
                    ktile(kt, F{}, T{}, E{});
                    ktile(kt + 1, F{}, T{}, O{});
                }
                ktile(kt, F{}, T{}, E{});
                ktile(kt + 1, F{}, F{}, O{});
            }
        };
        const uint64_t t_loop0 = clock64();
        run_ktiles(seg_ktiles);
        if (by_chunk) {
            // the other column chunks of A, in ring order from the own one; the first tile that touches a chunk waits for
            // its flag (paper appendix C `wait`), later tiles of this workgroup know it has landed
            for (int sgm = 1; sgm < g.k_chunks; ++sgm) {
                int c = g.rank + sgm;
                if (c >= g.k_chunks) c -= g.k_chunks;
                if (!((seen_chunks >> c) & 1)) {
                    PK_LDS int* verdict = (PK_LDS int*)(lds + EPI_OFF);
                    if (tid == 0) {
                        const int late = flag_wait(g.chunk_flags + c, g.epoch, g.timeout_ticks) ? 0 : 1;
                        if (late) report_timeout(g.status, (uint32_t)c, 1u);
                        *verdict = late;
                    }
                    __syncthreads();
                    const int late_all = *verdict;
                    __syncthreads();
                    if (late_all) return;                 // drain: this tile and the rest of this workgroup's stay untouched
                    acquire_agent();
                    seen_chunks |= 1ull << c;
                }
                a_base = g.A + (int64_t)c * seg_ktiles * KB;
                b_base = g.B + (int64_t)c * seg_ktiles * b_step;
#pragma unroll
                for (int s = 0; s < NS; ++s)
                    if (s < seg_ktiles) issue_loads(s);
                __builtin_amdgcn_s_waitcnt(PK_WAIT_VMCNT0);
                __syncthreads();
                run_ktiles(seg_ktiles);
            }
        }

        t_loops += clock64() - t_loop0;
        ++n_tiles_done;
        p_dead = false;
        p_kind = kind;
        p_part_lo = part_lo;
        p_tile_end = tile_end;
        p_q = q;
        p_flag = flag;
        p_row0 = row0;
        p_row_end = row_end;
        p_col0 = col0;
        p_col_end = col_end;
    }

    // the last tile's stores: every wave waits for its write-through stores, then the flag is published
    if (p_q >= 0 && (IS_RS || (SK && p_kind == UNIT_PART))) {
        __builtin_amdgcn_s_waitcnt(PK_WAIT_VMCNT0);
        __syncthreads();
        signal_prev();
    }
    if (blockIdx.x == 0 && tid == 0) {
        g.status[4] = (uint32_t)(wall_clock64() - t_wall0);
        g.status[5] = (uint32_t)(clock64() - t_core0);
        g.status[6] = (uint32_t)t_loops;
        g.status[7] = n_tiles_done;
    }
}

}  // namespace pk
