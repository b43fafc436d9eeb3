// libpk: kernels other than the GEMM, and the C-ABI entry points (see include/pk.h).
#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>

#include "pk_device.h"
#include "pk_gemm.h"

namespace pk {

// ------------------------------------------------------------------------------------------------
// Fused reduce of the P partial slots of this rank's shard (paper appendix C `reduce`: load the same
// tile from every device, reduce, store to local memory; section 3.1.3: the owner accumulates the
// tiles that the P ranks produced).  Pure streaming: per 8 output elements a thread issues 2 x P
// independent 16-byte loads, adds in slot order 0..P-1 in fp32, rounds to bf16 and stores 16 bytes.
// One workgroup handles `rows_sub` rows of one flag tile after waiting for that tile's P flags.
// ------------------------------------------------------------------------------------------------
struct ReduceArgs {
    const void* partials;     // [P][rows][n] fp32, or bf16 when the kernel is instantiated with S16
    uint16_t* out;            // rows x n bf16
    const uint32_t* flags_in; // [P][flags_per_slot]
    int32_t P, rows, n;
    int32_t tile_m, tile_n, tiles_n, sub, rows_sub;
    int64_t slot_elems, flags_per_slot;
    uint32_t epoch;
    uint32_t* status;
    uint64_t timeout_ticks;
    // all-reduce mode (bcast_out != nullptr or ar_flags_in != nullptr): the reduced block also goes to every
    // other rank's slot of bcast_out, and each 8-row block is announced per destination
    uint16_t* bcast_out;      // [P][rows][n] bf16
    uint32_t* ar_flags_in;    // [P][ar_flags_per_slot]; only slot `rank` is written
    uint32_t* ar_flags_out;   // [P][ar_flags_per_slot]
    int64_t ar_flags_per_slot;
    int32_t rank;
};

// cache policy of the partial-slot loads: system-coherent (sc0 sc1) and streaming (nt).  The slots are written
// by other workgroups / kernels (write-through) and announced through flags; loading them past this XCD's L2
// makes an acquire fence (a whole-L2 invalidate per workgroup) unnecessary.
constexpr int kCoherentStream = 1 | 2 | 16;

// PT > 0: compile-time P; PT == 0: runtime P.  S16: the slots hold bf16.  AR: all-reduce mode (the reduced rows are also
// pushed to the other ranks and announced).  NARROW: 4 output elements per thread and pass instead of 8 (one 16-byte load
// per slot in flight: under 48 registers), for launches that must fit beside a GEMM workgroup that leaves few registers.
template <int PT, bool S16, bool AR, bool NARROW = false>
__global__ __launch_bounds__(256) void reduce_kernel(const ReduceArgs r) {
    const int tid = threadIdx.x;
    const int P = PT > 0 ? PT : r.P;
    const int tile = blockIdx.x / r.sub;
    const int sb = blockIdx.x - tile * r.sub;
    const int tmi = tile / r.tiles_n, tc = tile - tmi * r.tiles_n;

    // wait (paper appendix C): one lane per source rank polls that rank's flag for this tile
    int late = 0;
    if constexpr (AR) {
        if (tid < P) {
            if (!flag_wait(r.flags_in + (int64_t)tid * r.flags_per_slot + tile, r.epoch, r.timeout_ticks)) {
                report_timeout(r.status, (uint32_t)tile, 2u);
                late = 1;
            }
        }
        if (__syncthreads_or(late)) return;      // the whole workgroup leaves together: it meets at a barrier below
    } else {
        // every wave polls for itself and decides with a ballot: this instantiation uses no LDS, not even the word a
        // workgroup-wide vote takes, so that its workgroups fit on a compute unit whose LDS a GEMM workgroup holds whole
        for (int p = tid & 63; p < P; p += 64) {
            if (!flag_wait(r.flags_in + (int64_t)p * r.flags_per_slot + tile, r.epoch, r.timeout_ticks)) {
                if (tid < 64) report_timeout(r.status, (uint32_t)tile, 2u);
                late = 1;
            }
        }
        if (__ballot(late) != 0) return;
    }

    constexpr int SLOT_ELEM = S16 ? 2 : 4;
    // one buffer descriptor per slot (a slot stays below 4 GiB, all P together need not)
    const uint32_t slot_bytes = (uint32_t)(r.slot_elems * SLOT_ELEM);
    auto slot = [&](int p) {
        return __builtin_amdgcn_make_buffer_rsrc((char*)r.partials + (int64_t)p * r.slot_elems * SLOT_ELEM, 0, (int)slot_bytes,
                                                 0x00020000);
    };
    const int row_start = tmi * r.tile_m + sb * r.rows_sub;
    const int row_stop = min(min(row_start + r.rows_sub, (tmi + 1) * r.tile_m), r.rows);
    const int col0 = tc * r.tile_n;
    const int cpr = min(r.tile_n, r.n - col0) >> 3;          // 8-element chunks per row of this tile
    const int total = (row_stop - row_start) * cpr;
    // bf16 -> fp32 of the 8 values of one 16-byte load, added to (s0, s1)
    auto add16 = [](f32x4& s0, f32x4& s1, i32x4 v) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t w = (uint32_t)v[e];
            const float lo = __builtin_bit_cast(float, w << 16), hi = __builtin_bit_cast(float, w & 0xFFFF0000u);
            if (e < 2) {
                s0[2 * e] += lo;
                s0[2 * e + 1] += hi;
            } else {
                s1[2 * e - 4] += lo;
                s1[2 * e - 3] += hi;
            }
        }
    };
    if constexpr (NARROW) {
        static_assert(!NARROW || (!S16 && !AR && PT > 0), "the narrow form is built for fp32 slots, compile-time P, no all-reduce");
        const int cpr4 = cpr * 2;
        for (int idx = tid; idx < total * 2; idx += 256) {
            const int rr = idx / cpr4, cc = idx - rr * cpr4;
            const int64_t off = (int64_t)(row_start + rr) * r.n + col0 + cc * 4;
            const uint32_t boff = (uint32_t)(off * 4);
            f32x4 v[PT > 0 ? PT : 1];
#pragma unroll
            for (int p = 0; p < PT; ++p)
                v[p] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(slot(p), boff, 0, kCoherentStream));
            f32x4 sum = v[0];
#pragma unroll
            for (int p = 1; p < PT; ++p) sum += v[p];
            bf16x4 o = {(__bf16)sum[0], (__bf16)sum[1], (__bf16)sum[2], (__bf16)sum[3]};
            __builtin_nontemporal_store(o, (bf16x4*)(r.out + off));
        }
        return;
    }
    for (int idx = tid; idx < total; idx += 256) {
        const int rr = idx / cpr, cc = idx - rr * cpr;
        const int64_t off = (int64_t)(row_start + rr) * r.n + col0 + cc * 8;
        const uint32_t boff = (uint32_t)(off * SLOT_ELEM);
        f32x4 s0, s1;
        if constexpr (S16) {
            s0 = f32x4{0.f, 0.f, 0.f, 0.f};
            s1 = s0;
            if constexpr (PT > 0) {
                i32x4 v[PT];
#pragma unroll
                for (int p = 0; p < PT; ++p) v[p] = __builtin_amdgcn_raw_buffer_load_b128(slot(p), boff, 0, kCoherentStream);
#pragma unroll
                for (int p = 0; p < PT; ++p) add16(s0, s1, v[p]);
            } else {
                for (int p = 0; p < P; ++p) add16(s0, s1, __builtin_amdgcn_raw_buffer_load_b128(slot(p), boff, 0, kCoherentStream));
            }
        } else if constexpr (PT > 0) {
            f32x4 v0[PT], v1[PT];
#pragma unroll
            for (int p = 0; p < PT; ++p) {
                v0[p] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(slot(p), boff, 0, kCoherentStream));
                v1[p] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(slot(p), boff + 16, 0, kCoherentStream));
            }
            s0 = v0[0];
            s1 = v1[0];
#pragma unroll
            for (int p = 1; p < PT; ++p) {
                s0 += v0[p];
                s1 += v1[p];
            }
        } else {
            s0 = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(slot(0), boff, 0, kCoherentStream));
            s1 = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(slot(0), boff + 16, 0, kCoherentStream));
            for (int p = 1; p < P; ++p) {
                s0 += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(slot(p), boff, 0, kCoherentStream));
                s1 += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(slot(p), boff + 16, 0, kCoherentStream));
            }
        }
        bf16x8 o = {(__bf16)s0[0], (__bf16)s0[1], (__bf16)s0[2], (__bf16)s0[3],
                    (__bf16)s1[0], (__bf16)s1[1], (__bf16)s1[2], (__bf16)s1[3]};
        if constexpr (AR) {
            // all-reduce: consumers find these rows through flags, so write through
            const i32x4 ov = __builtin_bit_cast(i32x4, o);
            store16_writethrough(r.out + off, ov);
            for (int q = 0; q < P; ++q)
                if (q != r.rank) store16_writethrough(r.bcast_out + (int64_t)q * r.slot_elems + off, ov);
        } else {
            __builtin_nontemporal_store(o, (bf16x8*)(r.out + off));
        }
    }
    if (AR && row_start < r.rows) {
        // `signal` per destination for this 8-row block: every wave waits for its stores, then one lane per rank
        __builtin_amdgcn_s_waitcnt(PK_WAIT_VMCNT0);
        __syncthreads();
        if (tid < P) {
            const int64_t b = (int64_t)(row_start / PK_AR_ROWS) * r.tiles_n + tc;
            uint32_t* f = (tid == r.rank ? r.ar_flags_in : r.ar_flags_out) + (int64_t)tid * r.ar_flags_per_slot + b;
            flag_publish(f, r.epoch);
        }
    }
}

// Completion of the all-reduce on this rank: one thread per flag of ar_flags_in waits (bounded) for the epoch.
__global__ __launch_bounds__(256) void ar_wait_kernel(const uint32_t* flags, int64_t n_flags, uint32_t epoch,
                                                      uint32_t* status, uint64_t timeout_ticks) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n_flags && !flag_wait(flags + i, epoch, timeout_ticks)) report_timeout(status, (uint32_t)i, 3u);
}

// ------------------------------------------------------------------------------------------------
// Peer emulation (not part of the method): what other ranks' communicator workers would push here.
// ------------------------------------------------------------------------------------------------
struct EmuOrder {
    int32_t n;
    int32_t q[PK_EMU_MAX_ORDER];
};

__device__ __forceinline__ void idle_us(uint32_t us) {
    if (us == 0) return;
    const uint64_t t0 = wall_clock64();
    const uint64_t ticks = (uint64_t)us * kWallClockTicksPerUs;
    while (wall_clock64() - t0 < ticks) __builtin_amdgcn_s_sleep(16);
}

// Both emulators publish like the GEMM epilogue does: write-through stores, every wave waits for its own stores,
// workgroup barrier, then a relaxed device-scope flag store (no L2 write-back fence per workgroup).
__global__ __launch_bounds__(256) void emu_chunks_kernel(const char* staging, char* A_gathered, int64_t chunk_bytes,
                                                         uint32_t* chunk_flags, uint32_t epoch, EmuOrder ord,
                                                         uint32_t gap_us, uint32_t* counters) {
    const int64_t n16 = chunk_bytes >> 4;
    for (int i = 0; i < ord.n; ++i) {
        const int q = ord.q[i];
        const i32x4* src = (const i32x4*)(staging + (int64_t)q * chunk_bytes);
        i32x4* dst = (i32x4*)(A_gathered + (int64_t)q * chunk_bytes);
        // 8 independent 16-byte loads in flight per thread: few workgroups must still move a chunk quickly
        const int64_t stride = (int64_t)gridDim.x * 256;
        int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
        for (; idx + 7 * stride < n16; idx += 8 * stride) {
            i32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + idx + u * stride);
#pragma unroll
            for (int u = 0; u < 8; ++u) store16_writethrough(dst + idx + u * stride, v[u]);
        }
        for (; idx < n16; idx += stride) store16_writethrough(dst + idx, __builtin_nontemporal_load(src + idx));
        __builtin_amdgcn_s_waitcnt(PK_WAIT_VMCNT0);
        __syncthreads();
        if (threadIdx.x == 0) {
            // the last workgroup to finish its part of the chunk publishes the flag
            uint32_t old = __hip_atomic_fetch_add(counters + i, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (old == gridDim.x - 1) flag_publish(chunk_flags + q, epoch);
        }
        idle_us(gap_us);
    }
}

__global__ __launch_bounds__(256) void emu_partials_kernel(const float* staging, float* partials, uint32_t* flags_in,
                                                           uint32_t epoch, EmuOrder ord, uint32_t gap_us,
                                                           int rows, int n, int tile_m, int tile_n,
                                                           int tiles_m, int tiles_n) {
    const int64_t slot_elems = (int64_t)rows * n;
    const int64_t fps = (int64_t)tiles_m * tiles_n;
    for (int i = 0; i < ord.n; ++i) {
        const int q = ord.q[i];
        for (int tile = blockIdx.x; tile < tiles_m * tiles_n; tile += gridDim.x) {
            const int tmi = tile / tiles_n, tc = tile - tmi * tiles_n;
            const int r0 = tmi * tile_m, r1 = min(r0 + tile_m, rows);
            const int c0 = tc * tile_n, w4 = min(tile_n, n - c0) >> 2;
            const int total = (r1 - r0) * w4;
            for (int idx = threadIdx.x; idx < total; idx += 256) {
                const int rr = idx / w4, cc = idx - rr * w4;
                const int64_t off = (int64_t)q * slot_elems + (int64_t)(r0 + rr) * n + c0 + cc * 4;
                store16_writethrough(partials + off, __builtin_nontemporal_load((const i32x4*)(staging + off)));
            }
            __builtin_amdgcn_s_waitcnt(PK_WAIT_VMCNT0);
            __syncthreads();
            if (threadIdx.x == 0) flag_publish(flags_in + (int64_t)q * fps + tile, epoch);
        }
        idle_us(gap_us);
    }
}

// ------------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------------
struct TileCfg {
    int bm, bn;
};

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// 256 x 256 tiles when they still give every CU a tile, else 128 x 128.
static TileCfg pick_tile(int P, int64_t rows_per_shard, int64_t n) {
    const int64_t big = (int64_t)P * ceil_div(rows_per_shard, 256) * ceil_div(n, 256);
    if (rows_per_shard >= 256 && n >= 256 && big >= 256) return {256, 256};
    return {128, 128};
}

// Shape of an XCD's run of tiles inside a scheduling group.  The run (`run` consecutive tiles in the group's
// linear order) should be a compact block so that the tiles an XCD works on at the same time share A and B
// panels in its L2: up to 32 tiles are resident per XCD, ideally 4 rows x 8 columns.  When a run is no longer
// than a tile row (all-gather: one chunk's tiles are split 8 ways), plain row-major keeps each XCD on one A
// panel and on the same B column strip in every chunk.
static int pick_band(int grp_tile_rows, int tiles_n, int run) {
    if (run <= tiles_n) return 1;
    return grp_tile_rows < 4 ? grp_tile_rows : 4;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// rs: GEMM + reduce-scatter (K sharded) as opposed to all-gather + GEMM (N sharded); rs_cols: the reduce-scatter is along
// the last dimension (then M need not divide by P, N must); ag_k: the all-gather is along the last dimension of A (K)
static pk_status check_dims(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, bool rs,
                            int64_t* lm, int64_t* ln, int64_t* lk, bool rs_cols = false, bool ag_k = false) {
    if (dt != PK_BF16 && dt != PK_FP8_E4M3) return PK_ERR_DTYPE;
    if (P < 1 || P > PK_EMU_MAX_ORDER || M < 1 || N < 1 || K < 1) return PK_ERR_SHAPE;
    if (M % P && !rs_cols && !ag_k) return PK_ERR_SHAPE;
    if (rs ? (K % P) : (N % P)) return PK_ERR_SHAPE;
    if (rs_cols && (N % P || (N / P) % (dt == PK_FP8_E4M3 ? 16 : 8))) return PK_ERR_SHAPE;
    const int64_t m = M, n = rs ? N : N / P, k = rs ? K / P : K;
    const int kt = dt == PK_FP8_E4M3 ? 128 : 64, nv = dt == PK_FP8_E4M3 ? 16 : 8;
    if (k % kt || n % nv) return PK_ERR_SHAPE;
    if (ag_k && (K % P || (K / P) % kt)) return PK_ERR_SHAPE;   // A arrives in column chunks of whole k-tiles
    if (m > (1 << 30) || n > (1 << 30) || k > (1 << 30)) return PK_ERR_SHAPE;
    // the kernels address each operand, and each partial slot (M*N/P elements, at most 4 bytes each), with 32-bit byte
    // offsets from its base
    if (m * k * 2 >= ((int64_t)1 << 32) || k * n * 2 >= ((int64_t)1 << 32)) return PK_ERR_SHAPE;
    if (rs && m * n / P * 4 >= ((int64_t)1 << 32)) return PK_ERR_SHAPE;
    *lm = m;
    *ln = n;
    *lk = k;
    return PK_OK;
}

// compute units of the current device (cached per device ordinal)
static int num_cus() {
    static std::atomic<int> cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cache[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        int v = 0;
        n = (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) ? v : 256;
        cache[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

constexpr size_t kWsFlagBytes = 4096;   // the first bytes of a workspace hold one ready flag per workgroup

static pk_status make_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, bool rs, pk_plan* plan) {
    if (!plan) return PK_ERR_NULL;
    int64_t m, n, k;
    pk_status st = check_dims(P, M, N, K, dt, rs, &m, &n, &k);
    if (st != PK_OK) return st;
    const TileCfg tc = pick_tile(P, M / P, n);
    plan->tile_m = tc.bm;
    plan->tile_n = tc.bn;
    plan->tiles_m = (int32_t)ceil_div(M / P, tc.bm);
    plan->tiles_n = (int32_t)ceil_div(n, tc.bn);
    plan->flags_per_slot = (int64_t)plan->tiles_m * plan->tiles_n;
    plan->local_m = m;
    plan->local_n = n;
    plan->local_k = k;
    plan->ar_flags_per_slot = 0;
    plan->workspace_bytes = (int64_t)kWsFlagBytes + (int64_t)num_cus() * tc.bm * tc.bn * 4;
    return PK_OK;
}

// Last-dimension scatter: the shard is M x N/P, flags cover tiles of that shard.
static pk_status make_plan_cols(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan) {
    if (!plan) return PK_ERR_NULL;
    int64_t m, n, k;
    pk_status st = check_dims(P, M, N, K, dt, true, &m, &n, &k, true);
    if (st != PK_OK) return st;
    const int64_t ns = N / P;
    const int64_t big = ceil_div(M, 256) * P * ceil_div(ns, 256);
    const TileCfg tc = (M >= 256 && ns >= 256 && big >= 256) ? TileCfg{256, 256} : TileCfg{128, 128};
    plan->tile_m = tc.bm;
    plan->tile_n = tc.bn;
    plan->tiles_m = (int32_t)ceil_div(M, tc.bm);
    plan->tiles_n = (int32_t)ceil_div(ns, tc.bn);
    plan->flags_per_slot = (int64_t)plan->tiles_m * plan->tiles_n;
    plan->local_m = M;
    plan->local_n = N;
    plan->local_k = k;
    plan->ar_flags_per_slot = 0;
    plan->workspace_bytes = 0;
    return PK_OK;
}

// Persistent launch: one workgroup per CU (a multiple of 8 so that workgroup id mod 8 stays the XCD), or fewer
// when there are fewer tile slots.
// one launch of one instantiation; the dynamic LDS size of an instantiation is raised once per device
template <int BM, int BN, int WM, int WN, int KB, int NS, bool FP8, int EPI, bool BT, bool SK>
static pk_status launch_kernel(const GemmArgs& a, int grid, hipStream_t stream) {
    static std::atomic<uint64_t> configured{0};              // bit d = done on device d
    auto kern = gemm_kernel<BM, BN, WM, WN, KB, NS, FP8, EPI, BT, SK>;
    constexpr int lds = gemm_lds_bytes<BM, BN, KB, NS>();
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PK_ERR_HIP;
    const uint64_t bit = 1ull << (dev & 63);
    if (!(configured.load(std::memory_order_acquire) & bit)) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return PK_ERR_HIP;
        configured.fetch_or(bit, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * WM * WN), lds, stream, a);
    return hipGetLastError() == hipSuccess ? PK_OK : PK_ERR_HIP;
}

// workgroups of a launch that shares out no tile: one per compute unit left to the GEMM (a multiple of 8, so that
// workgroup id mod 8 stays the XCD), or the fewest that finish in the same number of rounds (448 slots on 256 CUs: 2
// rounds of 224)
static int schedule_grid(int slots, int comm_cus) {
    int grid = (num_cus() - comm_cus) / 8 * 8;
    if (grid < 8) grid = 8;
    const int rounds = (slots + grid - 1) / grid;
    const int even = ((slots + rounds - 1) / rounds + 7) / 8 * 8;
    return even < grid ? even : grid;
}

template <int BM, int BN, int WM, int WN, int KB, int NS, bool FP8, int EPI, bool BT = false>
static pk_status launch_gemm(GemmArgs a, int slots, int comm_cus, void* ws, size_t ws_bytes, hipStream_t stream) {
    a.ktiles = a.ktiles * 128 / KB;          // callers count k-tiles of 128 bytes
    constexpr bool HAS_SK = !BT && (EPI == EPI_RS || EPI == EPI_AG);   // the stream-K tail is built for these
    int grid = (num_cus() - comm_cus) / 8 * 8;
    if (grid < 8) grid = 8;
    a.sk_dp_slots = slots;
    const int rem = slots % grid;
    if (ws && HAS_SK && slots > grid && rem != 0 && a.ktiles >= 8 * NS && grid <= (int)(kWsFlagBytes / 4)) {
        // With a workspace every compute unit works to the end: whole rounds of tiles, then the k range of the left-over
        // tiles shared out evenly (448 slots on 256 CUs: 256 whole tiles, then 192 tiles as 256 pieces of 3/4 tile).
        if (ws_bytes < kWsFlagBytes + (size_t)grid * BM * BN * 4) return PK_ERR_ARG;
        a.sk_dp_slots = slots - rem;
        a.ws_flags = (uint32_t*)ws;
        a.ws_tiles = (char*)ws + kWsFlagBytes;
        if (a.ws_epoch == 0) a.ws_epoch = a.epoch;     // a caller's workspace follows the caller's epochs
    } else {
        grid = schedule_grid(slots, comm_cus);
    }
    if constexpr (HAS_SK) {
        if (a.sk_dp_slots != slots) return launch_kernel<BM, BN, WM, WN, KB, NS, FP8, EPI, BT, true>(a, grid, stream);
    }
    return launch_kernel<BM, BN, WM, WN, KB, NS, FP8, EPI, BT, false>(a, grid, stream);
}

template <int EPI>
static pk_status dispatch_gemm(const GemmArgs& a, int slots, int comm_cus, const TileCfg& tc, bool fp8,
                               void* ws, size_t ws_bytes, hipStream_t stream, bool bt = false) {
    if (bt) {
        // second operand stored k-contiguous: built for the two base epilogues only
        if constexpr (EPI == EPI_RS || EPI == EPI_AG) {
            // 128-byte k-tiles in a ring of 2 stages: a k-contiguous operand is fetched as one piece per row and k-tile, and
            // 64-byte pieces use half of every 128-byte line they touch (measured: 7% slower than the row-major path)
            if (tc.bm == 256)
                return fp8 ? launch_gemm<256, 256, 2, 4, 128, 2, true, EPI, true>(a, slots, comm_cus, ws, ws_bytes, stream)
                           : launch_gemm<256, 256, 2, 4, 128, 2, false, EPI, true>(a, slots, comm_cus, ws, ws_bytes, stream);
            return fp8 ? launch_gemm<128, 128, 2, 2, 128, 2, true, EPI, true>(a, slots, comm_cus, ws, ws_bytes, stream)
                       : launch_gemm<128, 128, 2, 2, 128, 2, false, EPI, true>(a, slots, comm_cus, ws, ws_bytes, stream);
        } else {
            return PK_ERR_ARG;
        }
    }
    if (tc.bm == 256) {
        // 8 waves, 64-byte k-tiles (32 bf16 or 64 fp8 of k) in a ring of 4 LDS stages
        return fp8 ? launch_gemm<256, 256, 2, 4, 64, 4, true, EPI>(a, slots, comm_cus, ws, ws_bytes, stream)
                   : launch_gemm<256, 256, 2, 4, 64, 4, false, EPI>(a, slots, comm_cus, ws, ws_bytes, stream);
    }
    return fp8 ? launch_gemm<128, 128, 2, 2, 128, 2, true, EPI>(a, slots, comm_cus, ws, ws_bytes, stream)
               : launch_gemm<128, 128, 2, 2, 128, 2, false, EPI>(a, slots, comm_cus, ws, ws_bytes, stream);
}

// ------------------------------------------------------------------------------------------------
// Scratch memory of the library itself, for pk_ag_gemm_static (callers that cannot allocate): the workspace of the
// stream-K tail.  Each device that loads the library holds its own copy of the array at its own address.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PK_STATIC_WS_BYTES];

// address of this device's copy of `scratch` (looked up once per device; the array's name itself is no device address)
static pk_status scratch_of_device(void** out) {
    static std::atomic<void*> cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PK_ERR_HIP;
    void* p = cache[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PK_ERR_HIP;
        cache[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return PK_OK;
}

__global__ __launch_bounds__(1024) void fill_zero_kernel(uint32_t* p, int n) {
    for (int i = threadIdx.x; i < n; i += 1024) p[i] = 0u;
}

static uint64_t timeout_ticks(uint64_t timeout_us) {
    if (timeout_us == 0) timeout_us = 2000000;
    return timeout_us * kWallClockTicksPerUs;
}

// ------------------------------------------------------------------------------------------------
// Measurement aid (not part of the method): register-only MFMA loop.  Each wave runs `iters` rounds of 16
// independent 32x32x16 bf16 MFMAs on operands held in registers, either all 1.0 or random sign + mantissa.
// The sustained rate with random operands is the ceiling a GEMM on random data can reach: the chip lowers its
// clock under data-dependent power.  One lane also reports wall-clock ticks and core-clock cycles.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int random_operands, uint64_t* report) {
    const uint64_t w0 = wall_clock64(), c0 = clock64();
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    bf16x8 a[4], b[4];
    uint32_t x = 1u + threadIdx.x * 2654435761u + blockIdx.x * 40503u;
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        s16x8 ra, rb;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x = x * 1664525u + 1013904223u;
            const uint32_t m1 = x >> 16;
            x = x * 1664525u + 1013904223u;
            const uint32_t m2 = x >> 16;
            ra[j] = random_operands ? (short)((m1 & 0x807F) | 0x3C00) : (short)0x3F80;
            rb[j] = random_operands ? (short)((m2 & 0x807F) | 0x3C00) : (short)0x3F80;
        }
        a[f] = __builtin_bit_cast(bf16x8, ra);
        b[f] = __builtin_bit_cast(bf16x8, rb);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[i >> 2], acc[i], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += acc[i][0];
    if (threadIdx.x == 0 && blockIdx.x == 7) {
        report[0] = wall_clock64() - w0;
        report[1] = clock64() - c0;
    }
    if (sum == 12345.678f) report[2] = 1;   // keeps the loop alive
}

}  // namespace pk


using namespace pk;

// A second stream per device, with the two events that fork it from and join it to the caller's stream: the reduce
// phase of pk_gemm_rs runs on it beside the rest of the GEMM (PK_PHASE_OVERLAP).  Created at the first such call on a
// device and kept until the process ends; default priority.  `lock` serialises the callers' fork/join sequences.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool ready = false;
};
static std::mutex side_lock;
static SideStream side_streams[64];

static pk_status side_stream_of_device(SideStream** out) {   // call with side_lock held
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PK_ERR_HIP;
    SideStream& h = side_streams[dev];
    if (!h.ready) {
        if (hipStreamCreateWithFlags(&h.stream, hipStreamNonBlocking) != hipSuccess) return PK_ERR_HIP;
        if (hipEventCreateWithFlags(&h.fork, hipEventDisableTiming) != hipSuccess) return PK_ERR_HIP;
        if (hipEventCreateWithFlags(&h.join, hipEventDisableTiming) != hipSuccess) return PK_ERR_HIP;
        h.ready = true;
    }
    *out = &h;
    return PK_OK;
}

struct AllReduceOut {
    uint16_t* bcast_out;
    uint32_t* ar_flags_in;
    uint32_t* ar_flags_out;
    int64_t ar_flags_per_slot;
};

// GEMM + reduce-scatter; with `ar` the reduce phase also hands the reduced rows to every rank (all-reduce)
static pk_status gemm_rs_impl(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                              const void* A_local, const void* B_local, const float* scale_a, const float* scale_b,
                              void* partials, void* outgoing, uint32_t* flags_in, uint32_t* flags_out,
                              uint32_t epoch, void* out_shard, const AllReduceOut* ar, uint32_t phases, int comm_cus,
                              int partial_dt, bool cols, void* ws, size_t ws_bytes, uint32_t* status, uint64_t timeout_us,
                              void* stream, int b_layout = PK_B_ROW_MAJOR) {
    pk_plan pl;
    pk_status st = cols ? make_plan_cols(P, M, N, K, dt, &pl) : make_plan(P, M, N, K, dt, true, &pl);
    if (st != PK_OK) return st;
    if (rank < 0 || rank >= P) return PK_ERR_RANK;
    if (comm_cus < 0 || comm_cus > 4096) return PK_ERR_ARG;
    if (partial_dt != PK_PARTIAL_F32 && partial_dt != PK_PARTIAL_BF16) return PK_ERR_DTYPE;
    if (b_layout != PK_B_ROW_MAJOR && b_layout != PK_B_K_CONTIGUOUS) return PK_ERR_ARG;
    const bool bf16_slots = partial_dt == PK_PARTIAL_BF16;
    const bool bt = b_layout == PK_B_K_CONTIGUOUS;
    if (bt && bf16_slots) return PK_ERR_ARG;
    const bool fp8 = dt == PK_FP8_E4M3;
    const bool do_gemm = phases & PK_PHASE_GEMM, do_reduce = phases & PK_PHASE_REDUCE;
    if (!partials || !flags_in || !status) return PK_ERR_NULL;
    if (do_gemm && (!A_local || !B_local)) return PK_ERR_NULL;
    if (do_gemm && P > 1 && (!outgoing || !flags_out)) return PK_ERR_NULL;
    if (do_reduce && !out_shard) return PK_ERR_NULL;
    if (do_gemm && fp8 && (!scale_a || !scale_b)) return PK_ERR_DTYPE;
    if (!aligned16(A_local) || !aligned16(B_local) || !aligned16(partials) || !aligned16(outgoing) ||
        !aligned16(out_shard))
        return PK_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    const TileCfg tc = {pl.tile_m, pl.tile_n};
    // Overlapped reduce: the GEMM is launched in two parts, the tile rows of this rank's own block (plus as many of the
    // next ranks' as fill whole rounds) and the rest; the reduce runs on the library's second stream beside the second
    // part: its workgroups use no LDS and few enough registers to sit next to a GEMM workgroup.  It waits for nothing
    // the second part produces, so whichever of the two the hardware places first, both finish.
    bool overlap = (phases & PK_PHASE_OVERLAP) && do_gemm && do_reduce && !ar && !cols && P > 1;
    int first_rows = 0;                      // tile rows of the first part (0: one launch for everything)
    // Registers per lane that the 256x256 GEMM kernels leave beside their two waves per SIMD: bf16 96, bf16 with the second
    // operand k-contiguous 48, fp8 48 (32 with bf16 slots, 16 with the second operand k-contiguous: too few).  Next to the
    // ones that leave 48 the narrow reduce kernel runs, built for fp32 slots and P of 2, 4 or 8; otherwise no overlap there.
    const bool narrow_reduce = pl.tile_m == 256 && (fp8 || bt);
    if (narrow_reduce && (bf16_slots || (fp8 && bt) || (P != 2 && P != 4 && P != 8))) overlap = false;
    if (overlap) {
        // a stream that is being captured into a graph takes the second stream along only if that one exists already
        // (it is created by the first eager call with the flag): no stream is created in the middle of a capture
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(s, &cap) != hipSuccess) return PK_ERR_HIP;
        if (cap != hipStreamCaptureStatusNone) {
            std::lock_guard<std::mutex> guard(side_lock);
            int dev = 0;
            if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PK_ERR_HIP;
            if (!side_streams[dev].ready) overlap = false;
        }
    }
    // one shard (slot): rows x cols.  Scatter along rows: M/P x N; along the last dimension: M x N/P
    const int64_t rows = cols ? M : M / P;
    const int64_t slot_cols = cols ? N / P : N;

    GemmArgs a = {};
    const int all_rows = cols ? pl.tiles_m : P * pl.tiles_m;     // tile rows of the whole local product
    const int tiles_n_all = cols ? P * pl.tiles_n : pl.tiles_n;
    // one launch over `n_rows` tile rows that start at tile row `row0` (wrapping around at all_rows)
    auto gemm = [&](int row0, int n_rows) {
        a.grp_tile_rows = n_rows;
        a.row_rot = row0;
        a.all_tile_rows = (row0 == 0 && n_rows == all_rows) ? 0 : all_rows;
        const int64_t G = (int64_t)n_rows * a.tiles_n;
        a.wg_per_group = (int32_t)(8 * ceil_div(G, 8));
        a.band = pick_band(n_rows, a.tiles_n, a.wg_per_group / 8);
        return bf16_slots ? dispatch_gemm<EPI_RS16>(a, a.wg_per_group, comm_cus, tc, fp8, ws, ws_bytes, s)
                          : dispatch_gemm<EPI_RS>(a, a.wg_per_group, comm_cus, tc, fp8, ws, ws_bytes, s, bt);
    };
    if (do_gemm) {
        const int elem = fp8 ? 1 : 2;
        a.A = (const char*)A_local;
        a.B = (const char*)B_local;
        a.lda = pl.local_k * elem;
        a.ldb = (bt ? pl.local_k : pl.local_n) * elem;
        a.n = (int32_t)pl.local_n;
        a.ktiles = (int32_t)(pl.local_k / (fp8 ? 128 : 64));
        a.rows_per_shard = (int32_t)rows;
        a.tiles_m_shard = pl.tiles_m;
        a.tiles_n = tiles_n_all;
        a.cols_per_shard = cols ? (int32_t)slot_cols : 0;
        a.tiles_n_shard = cols ? pl.tiles_n : 0;
        a.n_groups = 1;
        a.group0 = 0;
        if (overlap) {
            // The first part: the own block's rows rounded up to whole bands of 4, then as many more bands (up to 7) as
            // waste the least of its last round.  No second part left: one launch, reduce afterwards.
            int grid = (num_cus() - comm_cus) / 8 * 8;
            if (grid < 8) grid = 8;
            const int band = 4;
            int best = 0;
            double best_waste = 2.0;
            for (int k = 0; k < 8; ++k) {
                const int r1 = (int)ceil_div(pl.tiles_m, band) * band + k * band;
                if (r1 >= all_rows) break;
                const int64_t t1 = (int64_t)r1 * tiles_n_all;
                const double waste = (double)(ceil_div(t1, grid) * grid - t1) / grid + 0.02 * k;
                if (waste < best_waste) {
                    best_waste = waste;
                    best = r1;
                }
            }
            first_rows = best;
            if (first_rows == 0) overlap = false;
        }
        a.rank = rank;
        a.partials = partials;
        a.outgoing = outgoing;
        a.flags_in = flags_in;
        a.flags_out = flags_out;
        a.slot_elems = rows * slot_cols;
        a.flags_per_slot = pl.flags_per_slot;
        a.scale_a = scale_a;
        a.scale_b = scale_b;
        a.epoch = epoch;
        a.status = status;
        a.timeout_ticks = timeout_ticks(timeout_us);
        st = overlap ? gemm(rank * pl.tiles_m, first_rows) : gemm(0, all_rows);
        if (st != PK_OK) return st;
    }
    std::unique_lock<std::mutex> side_guard(side_lock, std::defer_lock);
    SideStream* side = nullptr;
    hipStream_t reduce_stream = s;
    if (overlap) {
        side_guard.lock();
        st = side_stream_of_device(&side);
        if (st != PK_OK) return st;
        if (hipEventRecord(side->fork, s) != hipSuccess || hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess)
            return PK_ERR_HIP;
        reduce_stream = side->stream;
        // the rest of the GEMM is enqueued before the reduce, so that it is first in line for the compute units
        st = gemm((rank * pl.tiles_m + first_rows) % all_rows, all_rows - first_rows);
        if (st != PK_OK) return st;
    }
    if (do_reduce) {
        ReduceArgs r = {};
        r.partials = partials;
        r.out = (uint16_t*)out_shard;
        r.flags_in = flags_in;
        r.P = P;
        r.rows = (int32_t)rows;
        r.n = (int32_t)slot_cols;
        r.tile_m = pl.tile_m;
        r.tile_n = pl.tile_n;
        r.tiles_n = pl.tiles_n;
        r.rows_sub = 8;                       // 8 rows x tile_n columns x P slots per work item
        r.sub = pl.tile_m / r.rows_sub;
        r.slot_elems = rows * slot_cols;
        r.flags_per_slot = pl.flags_per_slot;
        r.epoch = epoch;
        r.status = status;
        r.timeout_ticks = timeout_ticks(timeout_us);
        r.rank = rank;
        if (ar) {
            r.bcast_out = ar->bcast_out;
            r.ar_flags_in = ar->ar_flags_in;
            r.ar_flags_out = ar->ar_flags_out;
            r.ar_flags_per_slot = ar->ar_flags_per_slot;
        }
        const int grid = (int)(pl.flags_per_slot * r.sub);   // one workgroup per work item
        hipStream_t s = reduce_stream;
        auto launch = [&](auto s16, auto armode) {
            constexpr bool S16 = decltype(s16)::value, AR = decltype(armode)::value;
            switch (P) {
                case 1: hipLaunchKernelGGL((reduce_kernel<1, S16, AR>), dim3(grid), dim3(256), 0, s, r); break;
                case 2: hipLaunchKernelGGL((reduce_kernel<2, S16, AR>), dim3(grid), dim3(256), 0, s, r); break;
                case 4: hipLaunchKernelGGL((reduce_kernel<4, S16, AR>), dim3(grid), dim3(256), 0, s, r); break;
                case 8: hipLaunchKernelGGL((reduce_kernel<8, S16, AR>), dim3(grid), dim3(256), 0, s, r); break;
                default: hipLaunchKernelGGL((reduce_kernel<0, S16, AR>), dim3(grid), dim3(256), 0, s, r); break;
            }
        };
        const bool ar_mode = r.ar_flags_in != nullptr;
        if (overlap && narrow_reduce) {
            switch (P) {
                case 2: hipLaunchKernelGGL((reduce_kernel<2, false, false, true>), dim3(grid), dim3(256), 0, s, r); break;
                case 4: hipLaunchKernelGGL((reduce_kernel<4, false, false, true>), dim3(grid), dim3(256), 0, s, r); break;
                default: hipLaunchKernelGGL((reduce_kernel<8, false, false, true>), dim3(grid), dim3(256), 0, s, r); break;
            }
        } else if (bf16_slots) ar_mode ? launch(std::true_type{}, std::true_type{}) : launch(std::true_type{}, std::false_type{});
        else ar_mode ? launch(std::false_type{}, std::true_type{}) : launch(std::false_type{}, std::false_type{});
        if (hipGetLastError() != hipSuccess) return PK_ERR_HIP;
    }
    if (overlap) {
        if (hipEventRecord(side->join, side->stream) != hipSuccess || hipStreamWaitEvent(s, side->join, 0) != hipSuccess)
            return PK_ERR_HIP;
    }
    return PK_OK;
}

static pk_status make_plan_ag_k(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan) {
    if (!plan) return PK_ERR_NULL;
    int64_t m, n, k;
    pk_status st = check_dims(P, M, N, K, dt, false, &m, &n, &k, false, true);
    if (st != PK_OK) return st;
    const TileCfg tc = pick_tile(1, M, n);
    plan->tile_m = tc.bm;
    plan->tile_n = tc.bn;
    plan->tiles_m = (int32_t)ceil_div(M, tc.bm);
    plan->tiles_n = (int32_t)ceil_div(n, tc.bn);
    plan->flags_per_slot = (int64_t)plan->tiles_m * plan->tiles_n;
    plan->local_m = m;
    plan->local_n = n;
    plan->local_k = k;
    plan->ar_flags_per_slot = 0;
    plan->workspace_bytes = 0;
    return PK_OK;
}

static pk_status ag_gemm_impl(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                              const void* A_gathered, const void* B_local, const float* scale_a, const float* scale_b,
                              const uint32_t* chunk_flags, uint32_t epoch, void* C_local, int comm_cus, int activation,
                              bool k_chunks, void* ws, size_t ws_bytes, bool ws_is_static, uint32_t* status, uint64_t timeout_us,
                              void* stream, int b_layout = PK_B_ROW_MAJOR) {
    pk_plan pl;
    pk_status st = k_chunks ? make_plan_ag_k(P, M, N, K, dt, &pl) : make_plan(P, M, N, K, dt, false, &pl);
    if (st != PK_OK) return st;
    if (rank < 0 || rank >= P) return PK_ERR_RANK;
    if (comm_cus < 0 || comm_cus > 4096) return PK_ERR_ARG;
    if (activation < PK_ACT_NONE || activation > PK_ACT_SILU) return PK_ERR_ARG;
    if (b_layout != PK_B_ROW_MAJOR && b_layout != PK_B_K_CONTIGUOUS) return PK_ERR_ARG;
    const bool bt = b_layout == PK_B_K_CONTIGUOUS;
    if (bt && k_chunks) return PK_ERR_ARG;
    const bool fp8 = dt == PK_FP8_E4M3;
    if (!A_gathered || !B_local || !C_local || !status) return PK_ERR_NULL;
    if (P > 1 && !chunk_flags) return PK_ERR_NULL;
    if (fp8 && (!scale_a || !scale_b)) return PK_ERR_DTYPE;
    if (!aligned16(A_gathered) || !aligned16(B_local) || !aligned16(C_local)) return PK_ERR_ALIGN;
    const TileCfg tc = {pl.tile_m, pl.tile_n};
    const int elem = fp8 ? 1 : 2;
    GemmArgs a = {};
    a.A = (const char*)A_gathered;
    a.B = (const char*)B_local;
    a.lda = pl.local_k * elem;
    a.ldb = (bt ? pl.local_k : pl.local_n) * elem;
    a.n = (int32_t)pl.local_n;
    a.ktiles = (int32_t)(pl.local_k / (fp8 ? 128 : 64));
    // row chunks: one scheduling group per chunk, visited from the own one; column chunks: every tile needs every chunk
    a.rows_per_shard = (int32_t)(k_chunks ? M : M / P);
    a.tiles_m_shard = pl.tiles_m;
    a.tiles_n = pl.tiles_n;
    a.grp_tile_rows = pl.tiles_m;
    a.n_groups = k_chunks ? 1 : P;
    a.group0 = k_chunks ? 0 : rank;
    a.k_chunks = k_chunks ? P : 0;
    a.act = activation;
    const int64_t G = (int64_t)a.grp_tile_rows * a.tiles_n;
    a.wg_per_group = (int32_t)(8 * ceil_div(G, 8));
    a.band = pick_band(a.grp_tile_rows, a.tiles_n, a.wg_per_group / 8);
    a.rank = rank;
    a.C = (uint16_t*)C_local;
    a.chunk_flags = chunk_flags;
    a.scale_a = scale_a;
    a.scale_b = scale_b;
    a.epoch = epoch;
    a.status = status;
    a.timeout_ticks = timeout_ticks(timeout_us);
    if (ws_is_static) {
        // the library's own scratch keeps the last call's flags, whatever its epoch was: clear them (with a kernel, so
        // that the call can be captured into a graph) and use an epoch of its own
        hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, (uint32_t*)ws, (int)(kWsFlagBytes / 4));
        if (hipGetLastError() != hipSuccess) return PK_ERR_HIP;
        a.ws_epoch = 1;
    }
    return k_chunks ? dispatch_gemm<EPI_AGK>(a, a.wg_per_group, comm_cus, tc, fp8, nullptr, 0, (hipStream_t)stream)
                    : dispatch_gemm<EPI_AG>(a, a.wg_per_group * P, comm_cus, tc, fp8, ws, ws_bytes, (hipStream_t)stream, bt);
}

static pk_status make_order(const int* order, int n_order, int P, EmuOrder* o) {
    if (n_order < 0 || n_order > PK_EMU_MAX_ORDER) return PK_ERR_ARG;
    if (n_order > 0 && !order) return PK_ERR_NULL;
    o->n = n_order;
    for (int i = 0; i < n_order; ++i) {
        if (order[i] < 0 || order[i] >= P) return PK_ERR_ARG;
        for (int j = 0; j < i; ++j)
            if (order[j] == order[i]) return PK_ERR_ARG;
        o->q[i] = order[i];
    }
    return PK_OK;
}

extern "C" {

int pk_version(void) { return 1; }

const char* pk_status_str(int s) {
    switch (s) {
        case PK_OK: return "ok";
        case PK_ERR_NULL: return "null pointer";
        case PK_ERR_SHAPE: return "unsupported shape";
        case PK_ERR_DTYPE: return "bad dtype or missing scales";
        case PK_ERR_ALIGN: return "pointer not 16-byte aligned";
        case PK_ERR_RANK: return "rank out of range";
        case PK_ERR_ARG: return "invalid argument";
        case PK_ERR_HIP: return "HIP launch failed";
        case PK_ERR_TIMEOUT: return "timed out waiting for a ready flag";
        default: return "unknown status";
    }
}

pk_status pk_gemm_rs_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan) {
    return make_plan(P, M, N, K, dt, true, plan);
}

pk_status pk_ag_gemm_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan) {
    return make_plan(P, M, N, K, dt, false, plan);
}

pk_status pk_gemm_rs(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                     const void* A_local, const void* B_local, const float* scale_a, const float* scale_b,
                     void* partials, void* outgoing, uint32_t* flags_in, uint32_t* flags_out, uint32_t epoch,
                     void* out_shard, uint32_t phases, int comm_cus, int partial_dt, int b_layout, void* workspace,
                     size_t workspace_bytes, uint32_t* status, uint64_t timeout_us, void* stream) {
    if ((phases & PK_PHASE_ALL) == 0 || (phases & ~(PK_PHASE_ALL | PK_PHASE_OVERLAP))) return PK_ERR_ARG;
    if ((phases & PK_PHASE_OVERLAP) && (phases & PK_PHASE_ALL) != PK_PHASE_ALL) return PK_ERR_ARG;
    if (!aligned16(workspace)) return PK_ERR_ALIGN;
    return gemm_rs_impl(P, rank, M, N, K, dt, A_local, B_local, scale_a, scale_b, partials, outgoing, flags_in,
                        flags_out, epoch, out_shard, nullptr, phases, comm_cus, partial_dt, false, workspace, workspace_bytes,
                        status, timeout_us, stream, b_layout);
}

pk_status pk_gemm_rs_cols_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan) {
    return make_plan_cols(P, M, N, K, dt, plan);
}

pk_status pk_gemm_rs_cols(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                          const void* A_local, const void* B_local, const float* scale_a, const float* scale_b,
                          void* partials, void* outgoing, uint32_t* flags_in, uint32_t* flags_out, uint32_t epoch,
                          void* out_shard, uint32_t phases, int comm_cus, int partial_dt, uint32_t* status,
                          uint64_t timeout_us, void* stream) {
    if (phases == 0 || (phases & ~PK_PHASE_ALL)) return PK_ERR_ARG;
    return gemm_rs_impl(P, rank, M, N, K, dt, A_local, B_local, scale_a, scale_b, partials, outgoing, flags_in,
                        flags_out, epoch, out_shard, nullptr, phases, comm_cus, partial_dt, true, nullptr, 0, status, timeout_us,
                        stream);
}

pk_status pk_gemm_ar_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan) {
    pk_status st = make_plan(P, M, N, K, dt, true, plan);
    if (st != PK_OK) return st;
    plan->ar_flags_per_slot = ceil_div(M / P, PK_AR_ROWS) * plan->tiles_n;
    return PK_OK;
}

pk_status pk_gemm_ar(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                     const void* A_local, const void* B_local, const float* scale_a, const float* scale_b,
                     void* partials, void* outgoing, uint32_t* flags_in, uint32_t* flags_out,
                     void* out_full, void* bcast_out, uint32_t* ar_flags_in, uint32_t* ar_flags_out,
                     uint32_t epoch, uint32_t phases, int comm_cus, int partial_dt, uint32_t* status,
                     uint64_t timeout_us, void* stream) {
    if (phases == 0 || (phases & ~(PK_PHASE_ALL | PK_PHASE_WAIT))) return PK_ERR_ARG;
    if (!out_full || !ar_flags_in || !status) return PK_ERR_NULL;
    if (P > 1 && (!bcast_out || !ar_flags_out)) return PK_ERR_NULL;
    if (!aligned16(out_full) || !aligned16(bcast_out)) return PK_ERR_ALIGN;
    pk_plan pl;
    pk_status st = pk_gemm_ar_plan(P, M, N, K, dt, &pl);
    if (st != PK_OK) return st;
    if (rank < 0 || rank >= P) return PK_ERR_RANK;
    AllReduceOut ar = {(uint16_t*)bcast_out, ar_flags_in, ar_flags_out, pl.ar_flags_per_slot};
    if (phases & PK_PHASE_ALL) {
        // the reduce phase writes rows R_rank of out_full
        uint16_t* own_rows = (uint16_t*)out_full + (int64_t)rank * (M / P) * N;
        st = gemm_rs_impl(P, rank, M, N, K, dt, A_local, B_local, scale_a, scale_b, partials, outgoing, flags_in,
                          flags_out, epoch, own_rows, &ar, phases & PK_PHASE_ALL, comm_cus, partial_dt, false, nullptr, 0, status,
                          timeout_us, stream);
        if (st != PK_OK) return st;
    }
    if (phases & PK_PHASE_WAIT) {
        const int64_t n_flags = (int64_t)P * pl.ar_flags_per_slot;
        hipLaunchKernelGGL(ar_wait_kernel, dim3((unsigned)ceil_div(n_flags, 256)), dim3(256), 0, (hipStream_t)stream,
                           (const uint32_t*)ar_flags_in, n_flags, epoch, status, timeout_ticks(timeout_us));
        if (hipGetLastError() != hipSuccess) return PK_ERR_HIP;
    }
    return PK_OK;
}

pk_status pk_ag_gemm(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                     const void* A_gathered, const void* B_local, const float* scale_a, const float* scale_b,
                     const uint32_t* chunk_flags, uint32_t epoch, void* C_local, int comm_cus, int activation,
                     int b_layout, void* workspace, size_t workspace_bytes, uint32_t* status, uint64_t timeout_us,
                     void* stream) {
    if (!aligned16(workspace)) return PK_ERR_ALIGN;
    return ag_gemm_impl(P, rank, M, N, K, dt, A_gathered, B_local, scale_a, scale_b, chunk_flags, epoch, C_local, comm_cus,
                        activation, false, workspace, workspace_bytes, false, status, timeout_us, stream, b_layout);
}

pk_status pk_ag_gemm_static(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                            const void* A_gathered, const void* B_local, const float* scale_a, const float* scale_b,
                            const uint32_t* chunk_flags, uint32_t epoch, void* C_local, int comm_cus, int activation,
                            uint32_t* status, uint64_t timeout_us, void* stream) {
    // the tiles of one launch must fit the scratch array: one fp32 tile per workgroup, one workgroup per compute unit
    pk_plan pl;
    pk_status st = make_plan(P, M, N, K, dt, false, &pl);
    if (st != PK_OK) return st;
    if ((size_t)pl.workspace_bytes > (size_t)PK_STATIC_WS_BYTES) return PK_ERR_ARG;
    void* ws = nullptr;
    st = scratch_of_device(&ws);
    if (st != PK_OK) return st;
    return ag_gemm_impl(P, rank, M, N, K, dt, A_gathered, B_local, scale_a, scale_b, chunk_flags, epoch, C_local, comm_cus,
                        activation, false, ws, (size_t)PK_STATIC_WS_BYTES, true, status, timeout_us, stream);
}

pk_status pk_ag_gemm_k_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan) {
    return make_plan_ag_k(P, M, N, K, dt, plan);
}

pk_status pk_ag_gemm_k(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                       const void* A_gathered, const void* B_local, const float* scale_a, const float* scale_b,
                       const uint32_t* chunk_flags, uint32_t epoch, void* C_local, int comm_cus, int activation,
                       uint32_t* status, uint64_t timeout_us, void* stream) {
    return ag_gemm_impl(P, rank, M, N, K, dt, A_gathered, B_local, scale_a, scale_b, chunk_flags, epoch, C_local, comm_cus,
                        activation, true, nullptr, 0, false, status, timeout_us, stream);
}

pk_status pk_emu_deliver_kchunks_dma(int P, int64_t M, int64_t K, int elem_bytes, const void* staging, void* A_gathered,
                                     uint32_t* chunk_flags, uint32_t epoch, const int* order, int n_order, void* stream) {
    if (P < 1 || P > PK_EMU_MAX_ORDER || M < 1 || K < 1 || K % P) return PK_ERR_SHAPE;
    if (elem_bytes != 1 && elem_bytes != 2) return PK_ERR_DTYPE;
    if (!staging || !A_gathered || !chunk_flags) return PK_ERR_NULL;
    const size_t pitch = (size_t)K * elem_bytes, width = (size_t)(K / P) * elem_bytes;
    EmuOrder o;
    pk_status st = make_order(order, n_order, P, &o);
    if (st != PK_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    for (int i = 0; i < o.n; ++i) {
        const size_t off = (size_t)o.q[i] * width;
        // M pieces of K/P elements, one per row: the strided layout of a gather along the last dimension
        if (hipMemcpy2DAsync((char*)A_gathered + off, pitch, (const char*)staging + off, pitch, width, (size_t)M,
                             hipMemcpyDeviceToDevice, s) != hipSuccess)
            return PK_ERR_HIP;
        if (hipStreamWriteValue32(s, chunk_flags + o.q[i], epoch, 0) != hipSuccess) return PK_ERR_HIP;
    }
    return PK_OK;
}

pk_status pk_emu_deliver_chunks(int P, int64_t M, int64_t K, int elem_bytes, const void* staging, void* A_gathered,
                                uint32_t* chunk_flags, uint32_t epoch, const int* order, int n_order,
                                uint32_t gap_us, int n_wg, uint32_t* counters, void* stream) {
    if (P < 1 || P > PK_EMU_MAX_ORDER || M < 1 || K < 1 || M % P) return PK_ERR_SHAPE;
    if (elem_bytes != 1 && elem_bytes != 2) return PK_ERR_DTYPE;
    if (n_wg < 0 || n_wg > 4096) return PK_ERR_ARG;
    if (!staging || !A_gathered || !chunk_flags || !counters) return PK_ERR_NULL;
    const int64_t chunk_bytes = (M / P) * K * elem_bytes;
    if (chunk_bytes % 16) return PK_ERR_SHAPE;
    if (!aligned16(staging) || !aligned16(A_gathered)) return PK_ERR_ALIGN;
    EmuOrder o;
    pk_status st = make_order(order, n_order, P, &o);
    if (st != PK_OK) return st;
    if (n_order == 0) return PK_OK;
    hipLaunchKernelGGL(emu_chunks_kernel, dim3(n_wg ? n_wg : 32), dim3(256), 0, (hipStream_t)stream, (const char*)staging,
                       (char*)A_gathered, chunk_bytes, chunk_flags, epoch, o, gap_us, counters);
    return hipGetLastError() == hipSuccess ? PK_OK : PK_ERR_HIP;
}

pk_status pk_emu_deliver_chunks_dma(int P, int64_t M, int64_t K, int elem_bytes, const void* staging, void* A_gathered,
                                    uint32_t* chunk_flags, uint32_t epoch, const int* order, int n_order, void* stream) {
    if (P < 1 || P > PK_EMU_MAX_ORDER || M < 1 || K < 1 || M % P) return PK_ERR_SHAPE;
    if (elem_bytes != 1 && elem_bytes != 2) return PK_ERR_DTYPE;
    if (!staging || !A_gathered || !chunk_flags) return PK_ERR_NULL;
    const int64_t chunk_bytes = (M / P) * K * elem_bytes;
    EmuOrder o;
    pk_status st = make_order(order, n_order, P, &o);
    if (st != PK_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    for (int i = 0; i < o.n; ++i) {
        const int64_t off = (int64_t)o.q[i] * chunk_bytes;
        // stream order puts the flag write behind the completed copy
        if (hipMemcpyAsync((char*)A_gathered + off, (const char*)staging + off, (size_t)chunk_bytes, hipMemcpyDeviceToDevice,
                           s) != hipSuccess)
            return PK_ERR_HIP;
        if (hipStreamWriteValue32(s, chunk_flags + o.q[i], epoch, 0) != hipSuccess) return PK_ERR_HIP;
    }
    return PK_OK;
}

pk_status pk_emu_deliver_partials(int P, int64_t M, int64_t N, int tile_m, int tile_n, const float* staging,
                                  float* partials, uint32_t* flags_in, uint32_t epoch, const int* order, int n_order,
                                  uint32_t gap_us, int n_wg, void* stream) {
    if (P < 1 || P > PK_EMU_MAX_ORDER || M < 1 || N < 1 || M % P || N % 4) return PK_ERR_SHAPE;
    if (tile_m < 1 || tile_n < 4 || tile_n % 4 || n_wg < 0 || n_wg > 4096) return PK_ERR_ARG;
    if (!staging || !partials || !flags_in) return PK_ERR_NULL;
    if (!aligned16(staging) || !aligned16(partials)) return PK_ERR_ALIGN;
    EmuOrder o;
    pk_status st = make_order(order, n_order, P, &o);
    if (st != PK_OK) return st;
    if (n_order == 0) return PK_OK;
    const int rows = (int)(M / P);
    const int tiles_m = (int)ceil_div(rows, tile_m), tiles_n = (int)ceil_div(N, tile_n);
    hipLaunchKernelGGL(emu_partials_kernel, dim3(n_wg ? n_wg : 32), dim3(256), 0, (hipStream_t)stream, staging, partials, flags_in,
                       epoch, o, gap_us, rows, (int)N, tile_m, tile_n, tiles_m, tiles_n);
    return hipGetLastError() == hipSuccess ? PK_OK : PK_ERR_HIP;
}

pk_status pk_probe_mfma(int iters, int random_operands, uint64_t* report, double* flops_out, void* stream) {
    if (!report) return PK_ERR_NULL;
    if (iters < 1 || iters > (1 << 22)) return PK_ERR_ARG;
    const int n_wg = 2 * num_cus();
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(n_wg), dim3(256), 0, (hipStream_t)stream, iters, random_operands ? 1 : 0, report);
    if (hipGetLastError() != hipSuccess) return PK_ERR_HIP;
    if (flops_out) *flops_out = (double)n_wg * 4.0 * (double)iters * 16.0 * 32768.0;
    return PK_OK;
}

pk_status pk_partition_create(int comm_cus, void** compute_stream, void** comm_stream) {
    if (!compute_stream || !comm_stream) return PK_ERR_NULL;
    const int ncu = num_cus();
    if (comm_cus < 8 || comm_cus % 8 || comm_cus > ncu - 8 || ncu > 1024) return PK_ERR_ARG;
    // Bit i of the mask is compute unit i/8 of XCD i%8 (checked on the device: a mask of the first 8*k bits
    // enables k compute units on each of the 8 XCDs), so both partitions span all XCDs and their L2s.
    uint32_t comm[32] = {0}, comp[32] = {0};
    const int words = (ncu + 31) / 32;
    for (int i = 0; i < ncu; ++i) (i < comm_cus ? comm : comp)[i >> 5] |= 1u << (i & 31);
    hipStream_t sc = nullptr, sm = nullptr;
    if (hipExtStreamCreateWithCUMask(&sc, words, comp) != hipSuccess) return PK_ERR_HIP;
    if (hipExtStreamCreateWithCUMask(&sm, words, comm) != hipSuccess) {
        (void)hipStreamDestroy(sc);
        return PK_ERR_HIP;
    }
    *compute_stream = sc;
    *comm_stream = sm;
    return PK_OK;
}

pk_status pk_partition_destroy(void* compute_stream, void* comm_stream) {
    pk_status st = PK_OK;
    if (compute_stream && hipStreamDestroy((hipStream_t)compute_stream) != hipSuccess) st = PK_ERR_HIP;
    if (comm_stream && hipStreamDestroy((hipStream_t)comm_stream) != hipSuccess) st = PK_ERR_HIP;
    return st;
}

}  // extern "C"
