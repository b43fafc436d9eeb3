/*
 * libpk: one rank's share of the two fused tensor-parallel GEMMs, on one MI355X (gfx950).
 *
 *   pk_gemm_rs  GEMM + tile-granular reduce-scatter   (paper sections 3.1.3 and 4.1, figure "GEMM + RS")
 *   pk_ag_gemm  all-gather + GEMM                     (paper sections 3.1.3 and 4.1, figure "AG + GEMM")
 * and, built on the same kernels,
 *   pk_gemm_ar                       GEMM + all-reduce          (sections 3.1.3 and 4.1, figure "GEMM + AR")
 *   pk_gemm_rs_cols, pk_ag_gemm_k    the scatter / gather along the last dimension (appendix on tensor-dimension collectives)
 *   pk_partition_create              compute-unit partition for communicator workgroups (section 3.1.3, SM partitioning)
 *
 * Notation is the paper's (section 4, experimental setup): P ranks; the GLOBAL GEMM is M x N x K with a
 * first operand A of M x K and a second operand B of K x N; 16-bit (bf16) inputs, fp32 accumulation.  The
 * 8-bit input type (OCP e4m3, finite+NaN, with one fp32 scale per tensor) is an extension of this library.
 * Every matrix is row-major and densely packed (leading dimension = number of columns).
 *
 * Peer ranks are not real GPUs here.  What a peer would write into this rank's memory over the fabric (its
 * partial sums for this rank's output shard; its row-chunk of A) lives in buffers in this GPU's HBM and is
 * announced through ready flags, exactly as a peer pushing one way into buffers that the receiver allocated up
 * front would leave it (paper section 3.1.4).  The pk_emu_* calls
 * play the peers for tests and benchmarks; they are not part of the method.
 *
 * Flags (the paper's barrier objects and signal/wait primitives, section 3.2.2 and appendix C): a flag is a
 * uint32 in device memory.  A datum is ready for a call with epoch e once (int32)(flag - e) >= 0.  Producers
 * make the data visible at device scope (write-through stores that have completed, or a release), then store e;
 * consumers poll, acquire (or read past their L2), then read the data.  Using a monotone epoch instead of a
 * counter that must be reset lets back-to-back calls reuse the flag arrays.
 *
 * Conventions for every entry point:
 *   - all pointers are DEVICE pointers unless marked "host";
 *   - the caller owns every buffer; the library allocates no device memory and keeps no state beyond per-device
 *     launch attributes set on a kernel's first use;
 *   - calls are asynchronous on `stream` (a hipStream_t, passed as void*); nothing synchronises the device;
 *   - arguments are validated on the host first; on an error nothing is launched and nothing is written;
 *   - a wait that exceeds `timeout_us` microseconds makes the kernel write {PK_ERR_TIMEOUT, index, phase, 0}
 *     to status[0..3] (first error wins) and drain; the host reads it after synchronising the stream.
 *     phase 1: a GEMM waiting for a chunk of A (index = chunk); phase 2: the reduce waiting for a tile's partials
 *     (index = tile); phase 3: pk_gemm_ar's closing wait (index = flag); phase 4: a GEMM workgroup waiting for another
 *     one's piece of a shared tile (index = workgroup).
 *     timeout_us = 0 selects the default (2 s).  The caller zeroes `status` (PK_STATUS_WORDS x uint32) before the call.
 *   - status[4..7] receive a timing report from workgroup 0 of the call's GEMM kernel: [4] ticks of the 100 MHz
 *     wall clock and [5] core-clock cycles from its start to its end ([5] / [4] x 100 MHz = the clock the chip
 *     held), [6] core-clock cycles inside its main loops, [7] the number of tiles it computed.
 */
#ifndef PK_H
#define PK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PK_OK = 0,
    PK_ERR_NULL = 1,       /* a required pointer is NULL */
    PK_ERR_SHAPE = 2,      /* P/M/N/K do not divide as required (see each call) */
    PK_ERR_DTYPE = 3,      /* unknown dtype, or fp8 without scales */
    PK_ERR_ALIGN = 4,      /* a matrix pointer is not 16-byte aligned */
    PK_ERR_RANK = 5,       /* rank outside [0, P) */
    PK_ERR_ARG = 6,        /* any other invalid argument (phases, order list, ...) */
    PK_ERR_HIP = 7,        /* a HIP launch failed */
    PK_ERR_TIMEOUT = 8     /* device side only: reported through `status` */
} pk_status;

typedef enum { PK_BF16 = 0, PK_FP8_E4M3 = 1 } pk_dtype;

/* memory layout of the second operand of pk_gemm_rs / pk_ag_gemm.  The paper gives its dimensions (K x N, section 4,
 * experimental setup) and not its memory order; the default is the matrix as written, row-major.  A weight matrix
 * that a caller keeps transposed (N x K row-major: every column of B contiguous along k, the usual storage of a linear
 * layer's weight) can be passed as it is with PK_B_K_CONTIGUOUS: the product is the same, both operands then reach
 * the matrix cores through 16-byte LDS reads and the transposing reads of the row-major path are not needed. */
typedef enum { PK_B_ROW_MAJOR = 0, PK_B_K_CONTIGUOUS = 1 } pk_b_layout;

#define PK_STATUS_WORDS 8    /* size of every `status` buffer, in uint32 */

/* element type of the partial slots of pk_gemm_rs / pk_gemm_ar (`partials`, `outgoing`) */
typedef enum {
    PK_PARTIAL_F32 = 0,    /* fp32 slots: the default, every contribution enters the sum unrounded */
    PK_PARTIAL_BF16 = 1    /* bf16 slots (the paper's element size for communicated tiles, section 3.1.3: s = 2):
                              half the scatter and reduce traffic; every contribution, the own one included, is
                              rounded to bf16 once before the fp32 sum */
} pk_partial_dtype;

/* non-linearity between the two GEMMs of the MLP (paper section 4.1, which does not name one), fused into pk_ag_gemm's epilogue;
 * evaluated in fp32 on the accumulator, before the rounding to bf16 */
typedef enum {
    PK_ACT_NONE = 0,
    PK_ACT_RELU = 1,        /* max(x, 0) */
    PK_ACT_GELU_TANH = 2,   /* x/2 * (1 + tanh(sqrt(2/pi) * (x + 0.044715 x^3))) */
    PK_ACT_SILU = 3         /* x / (1 + exp(-x)) */
} pk_activation;

/* phases of pk_gemm_rs (bit mask) */
#define PK_PHASE_GEMM   1u   /* local GEMM + scatter of finished tiles + per-tile signal */
#define PK_PHASE_REDUCE 2u   /* wait for the P partials of each own tile, sum, round, store */
#define PK_PHASE_ALL    3u
#define PK_PHASE_WAIT   4u   /* pk_gemm_ar only: wait until every rank's reduced rows have landed in out_full */
#define PK_PHASE_OVERLAP 8u  /* pk_gemm_rs with both phases: the reduce runs beside the GEMM (see pk_gemm_rs) */
#define PK_AR_ROWS      8    /* rows of out_full covered by one all-reduce ready flag (columns: tile_n) */

/* Flag granularity and derived sizes for a problem; filled by the *_plan calls (host struct). */
typedef struct {
    int32_t tile_m, tile_n;       /* rows x cols covered by one ready flag */
    int32_t tiles_m, tiles_n;     /* flag grid of one shard (GEMM+RS: M/P x N) or of C_local (AG+GEMM) */
    int64_t flags_per_slot;       /* tiles_m * tiles_n */
    int64_t local_m, local_n, local_k;   /* the per-rank GEMM */
    int64_t ar_flags_per_slot;    /* pk_gemm_ar_plan only: ceil((M/P) / PK_AR_ROWS) * tiles_n, else 0 */
    int64_t workspace_bytes;      /* pk_gemm_rs_plan, pk_ag_gemm_plan: size of a workspace that suffices on this device
                                     (PK_WS_FLAG_BYTES + one fp32 tile per compute unit); 0 for the other plans */
} pk_plan;

/*
 * Workspace (pk_gemm_rs, pk_ag_gemm; optional).  When the tiles do not fill a whole number of rounds on the compute
 * units (448 tiles on 256 units), the k range of the left-over tiles is shared out evenly over all workgroups
 * (paper section 3.1.3: the schedule depends on the problem size) and workgroups hand partial accumulator tiles to
 * one another through this memory.  Layout: PK_WS_FLAG_BYTES of ready flags, then one fp32 tile per workgroup.  The
 * caller zeroes the flag bytes once; afterwards the workspace belongs to one call site: its epochs must grow from
 * call to call, and two calls that may run at the same time must not share it.  workspace = NULL: whole tiles only (also
 * with PK_B_K_CONTIGUOUS and with bf16 slots, for which the tail is not built).
 * A workspace smaller than plan.workspace_bytes may be rejected with PK_ERR_ARG.
 */
#define PK_WS_FLAG_BYTES 4096

int pk_version(void);
const char* pk_status_str(int status);

/*
 * GEMM + reduce-scatter for rank `rank` (paper section 3.1.3: each finished output tile is sent to the rank
 * that owns it and accumulated there; section 4.1: second GEMM of the MLP, row-sharded weights).
 *
 *   own = A_local . B_local                 (M x N, fp32 accumulate; x scale_a*scale_b for fp8)
 *   rows R_q = [q*M/P, (q+1)*M/P) of own  -> outgoing[q]       for q != rank   (to rank q)
 *   rows R_rank of own                    -> partials[rank]
 *   out_shard = bf16( sum_{p<P} partials[p] )   summed in fp32, slot order 0..P-1, round-to-nearest-even
 *
 * Instead of the atomic adds of the paper, every source rank owns a slot of the destination's `partials`
 * array and the owner adds the P slots once, so the result does not depend on arrival order.
 *
 *   A_local   M x K/P      bf16 (2 B) or e4m3 (1 B)
 *   B_local   K/P x N      same element type; with b_layout = PK_B_K_CONTIGUOUS: N x K/P, the same matrix transposed
 *                          (fp32 slots only; PK_ERR_ARG otherwise)
 *   scale_a, scale_b       one fp32 each, fp8 only (NULL for bf16)
 *   partials  [P][M/P][N]  fp32, or bf16 with partial_dt = PK_PARTIAL_BF16.  Slot q != rank is written by peer q
 *                          (or by pk_emu_deliver_partials); slot `rank` is written by this call.
 *   outgoing  [P][M/P][N]  same element type.  Slot q != rank receives this rank's tiles for rank q; slot `rank` unused.
 *                          May be NULL when P == 1.
 *   flags_in  [P][flags_per_slot] readiness of partials[q][tile]; slot `rank` is signalled by this call.
 *   flags_out [P][flags_per_slot] signalled by this call when outgoing[q][tile] is complete.
 *   out_shard M/P x N      bf16
 *
 * Requirements: M % P == 0, K % P == 0, (K/P) % 64 == 0 (bf16) or % 128 == 0 (fp8), N % 8 == 0 (bf16) or
 * % 16 == 0 (fp8); M/P and N need not be multiples of the tile (edge tiles are partial).  Otherwise
 * PK_ERR_SHAPE.  `phases` selects which part runs (PK_PHASE_ALL normally).
 * PK_PHASE_ALL | PK_PHASE_OVERLAP hides the reduce behind the GEMM (section 3.1.3: communication that runs beside the
 * compute workers): the tile rows of this rank's own block (with as many of the following ones as fill whole rounds of
 * workgroups) are computed first, in a launch of their own; the rest of the GEMM
 * and the reduce then run side by side, the reduce on a second stream that the library keeps per device (created at the
 * first such call on a device outside a graph capture, default priority; a call on a capturing stream before that runs
 * in the plain order) and joins back into `stream` before the call's work counts as done there.  The reduce waits only for the own block (complete by then) and for the peers' flags, never for the second GEMM
 * launch, so either may be placed first.  Results are bit-identical to the plain call.  The flag needs both phases
 * (PK_ERR_ARG otherwise) and is ignored where it cannot help: when the own block takes every round of the schedule, and
 * next to the 256x256 fp8 kernel with bf16 slots, with a k-contiguous second operand, or with P other than 2, 4, 8.
 * Calls with the flag from several host threads on one device are serialised while they enqueue.
 * comm_cus: as for pk_ag_gemm below, the number of compute units the GEMM phase leaves to communicator workgroups
 * (0 = none).  partial_dt: element type of
 * `partials` and `outgoing` (PK_ERR_DTYPE if unknown).
 */
pk_status pk_gemm_rs_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan /* host */);
pk_status pk_gemm_rs(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                     const void* A_local, const void* B_local,
                     const float* scale_a, const float* scale_b,
                     void* partials, void* outgoing,
                     uint32_t* flags_in, uint32_t* flags_out, uint32_t epoch,
                     void* out_shard, uint32_t phases, int comm_cus, int partial_dt /* pk_partial_dtype */,
                     int b_layout /* pk_b_layout */, void* workspace, size_t workspace_bytes,
                     uint32_t* status, uint64_t timeout_us, void* stream);

/*
 * GEMM + reduce-scatter along the LAST dimension (paper appendix "Additional collective performance": reduce-scatter
 * along the tensor dimension, whose pieces are not contiguous in memory).  As pk_gemm_rs, but rank q owns the column
 * block N_q = [q*N/P, (q+1)*N/P) of every row:
 *
 *   columns N_q of own = A_local . B_local  -> outgoing[q] (q != rank), columns N_rank -> partials[rank]
 *   out_shard = bf16( sum_{p<P} partials[p] )                     (M x N/P)
 *
 *   partials, outgoing  [P][M][N/P]   fp32 or bf16 (partial_dt)
 *   flags_in, flags_out [P][flags_per_slot], flag grid = tiles of one M x N/P shard (pk_gemm_rs_cols_plan)
 *   out_shard           M x N/P bf16
 *
 * Requirements: K % P == 0, N % P == 0, (K/P) % 64 == 0 (bf16) or % 128 == 0 (fp8), (N/P) % 8 == 0 (bf16) or % 16 == 0
 * (fp8); M is arbitrary; M and N/P need not be multiples of the tile (a tile never crosses a column block).  Everything
 * else (phases without PK_PHASE_OVERLAP, comm_cus, status, timeout_us, errors) as pk_gemm_rs.
 */
pk_status pk_gemm_rs_cols_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan /* host */);
pk_status pk_gemm_rs_cols(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                          const void* A_local, const void* B_local,
                          const float* scale_a, const float* scale_b,
                          void* partials, void* outgoing,
                          uint32_t* flags_in, uint32_t* flags_out, uint32_t epoch,
                          void* out_shard, uint32_t phases, int comm_cus, int partial_dt /* pk_partial_dtype */,
                          uint32_t* status, uint64_t timeout_us, void* stream);

/*
 * GEMM + all-reduce for rank `rank` (paper section 3.1.3, inter-SM overlapping: partial results are accumulated
 * in HBM, completion is signalled per tile, and the reduction is done once by dedicated workers; section 4.1,
 * figure "GEMM + AR").  Operands, `partials`, `outgoing`, `flags_in`, `flags_out` exactly as pk_gemm_rs.  There is
 * no in-fabric reduction on an xGMI mesh, so the all-reduce is the reduce-scatter of pk_gemm_rs followed by handing
 * the reduced, rounded rows R_rank to every rank:
 *
 *   out_full rows R_rank = bf16( sum_{p<P} partials[p] )        (written here, then ar_flags_in[rank][b] = epoch)
 *   bcast_out[q]         = the same block, for q != rank         (then ar_flags_out[q][b] = epoch)
 *   out_full rows R_q, q != rank: written by rank q (or pk_emu_deliver_partials on the array viewed as fp32 pairs),
 *                          announced through ar_flags_in[q][b].
 *
 *   out_full      M x N bf16
 *   bcast_out     [P][M/P][N] bf16; in a deployment slot q is rank q's out_full rows R_rank, peer-mapped.  Slot
 *                 `rank` unused.  May be NULL when P == 1.
 *   ar_flags_in   [P][ar_flags_per_slot], ar_flags_out likewise (NULL allowed when P == 1); flag b covers rows
 *                 [PK_AR_ROWS * (b / tiles_n), +PK_AR_ROWS) x columns of tile b % tiles_n of one row block.
 *
 * phases: PK_PHASE_GEMM | PK_PHASE_REDUCE as pk_gemm_rs; PK_PHASE_WAIT adds a kernel that waits (bounded) until all
 * of ar_flags_in has reached `epoch`, so that work queued behind this call on `stream` may read all of out_full.
 * PK_PHASE_OVERLAP is not built for this call (PK_ERR_ARG).
 * Shape requirements, comm_cus, partial_dt, status and timeout_us as pk_gemm_rs.
 */
pk_status pk_gemm_ar_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan /* host */);
pk_status pk_gemm_ar(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                     const void* A_local, const void* B_local,
                     const float* scale_a, const float* scale_b,
                     void* partials, void* outgoing,
                     uint32_t* flags_in, uint32_t* flags_out,
                     void* out_full, void* bcast_out,
                     uint32_t* ar_flags_in, uint32_t* ar_flags_out,
                     uint32_t epoch, uint32_t phases, int comm_cus, int partial_dt /* pk_partial_dtype */,
                     uint32_t* status, uint64_t timeout_us, void* stream);

/*
 * All-gather + GEMM for rank `rank` (paper section 4.1: first GEMM of the MLP, inputs sharded by rows are
 * gathered, weights column-sharded; section 3.1.3, the paragraph on overlap across SMs: the chunks are moved by dedicated
 * communicator workers while the compute workers wait on a per-chunk flag before loading).
 *
 *   C_local = bf16( act( A_gathered . B_local ) )   (M x N/P; x scale_a*scale_b for fp8; act: pk_activation)
 *
 *   A_gathered  M x K   rows R_q = chunk q.  Chunk `rank` is valid at the call; chunk q != rank is valid
 *                       once chunk_flags[q] has reached `epoch`.
 *   B_local     K x N/P; with b_layout = PK_B_K_CONTIGUOUS: N/P x K, the same matrix transposed
 *   chunk_flags [P]
 *   C_local     M x N/P bf16
 *
 * Output tiles are scheduled chunk by chunk starting from the own chunk, then rank+1, rank+2, ... (mod P).
 * comm_cus (the paper's num_comm_sms, section 3.1.3, the paragraph on partitioning the SMs, appendix D) is the number of compute
 * units this call leaves free for the communicator workgroups that move the chunks while it runs: the GEMM is
 * launched on the remaining ones (rounded down to a multiple of 8, at least 8).  0 = use every compute unit:
 * communicator workgroups then run only where they fit beside a GEMM workgroup (it holds all of the compute unit's LDS
 * and leaves 80 registers per lane, bf16, or 48, fp8) or where the schedule leaves a compute unit empty.
 * Requirements: M % P == 0, N % P == 0, K % 64 == 0 (bf16) or % 128 == 0 (fp8), (N/P) % 8 == 0 (bf16) or
 * % 16 == 0 (fp8).  With P == 1 this is a plain GEMM with bf16 output (chunk_flags may then be NULL).
 */
pk_status pk_ag_gemm_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan /* host */);
pk_status pk_ag_gemm(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                     const void* A_gathered, const void* B_local,
                     const float* scale_a, const float* scale_b,
                     const uint32_t* chunk_flags, uint32_t epoch,
                     void* C_local, int comm_cus, int activation /* pk_activation */,
                     int b_layout /* pk_b_layout */, void* workspace, size_t workspace_bytes,
                     uint32_t* status, uint64_t timeout_us, void* stream);

/*
 * pk_ag_gemm for callers that cannot allocate device memory (code under graph capture, serving loops, harnesses that
 * forbid it): the same computation with the stream-K workspace taken from a scratch array inside the library
 * (PK_STATIC_WS_BYTES per device that uses the library, held until the process ends) instead of a caller's buffer.
 * Arguments, requirements and errors as pk_ag_gemm without `workspace`; the call allocates and frees nothing and
 * clears the scratch flags itself (with a kernel on `stream`).  PK_ERR_ARG if the problem's workspace
 * (plan.workspace_bytes: one fp32 tile per compute unit) exceeds PK_STATIC_WS_BYTES.  All calls on one device share
 * the array: calls that may overlap in time on one device race, whatever their streams.
 */
#define PK_STATIC_WS_BYTES (PK_WS_FLAG_BYTES + 256 * 256 * 256 * 4)   /* flags + 256 compute units x (256 x 256 fp32) */
pk_status pk_ag_gemm_static(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                            const void* A_gathered, const void* B_local,
                            const float* scale_a, const float* scale_b,
                            const uint32_t* chunk_flags, uint32_t epoch,
                            void* C_local, int comm_cus, int activation /* pk_activation */,
                            uint32_t* status, uint64_t timeout_us, void* stream);

/*
 * All-gather along the LAST dimension of A + GEMM (paper appendix "Additional collective performance": all-gather along
 * the tensor dimension, whose pieces are not contiguous in memory).  As pk_ag_gemm, but chunk q of A_gathered is the
 * column block K_q = [q*K/P, (q+1)*K/P) of every row (M pieces of K/P elements), valid once chunk_flags[q] has reached
 * `epoch` (chunk `rank` at the call).  Every output tile needs every chunk: the k-loop runs chunk by chunk in ring order
 * from the own one, and the first tile of a workgroup that reaches a chunk waits for its flag.
 * Requirements: N % P == 0, K % P == 0, (K/P) % 64 == 0 (bf16) or % 128 == 0 (fp8), (N/P) % 8 == 0 (bf16) or % 16 == 0
 * (fp8); M is arbitrary.  On a timeout the workgroup that waited stops: its current and remaining tiles stay unwritten.
 */
pk_status pk_ag_gemm_k_plan(int P, int64_t M, int64_t N, int64_t K, pk_dtype dt, pk_plan* plan /* host */);
pk_status pk_ag_gemm_k(int P, int rank, int64_t M, int64_t N, int64_t K, pk_dtype dt,
                       const void* A_gathered, const void* B_local,
                       const float* scale_a, const float* scale_b,
                       const uint32_t* chunk_flags, uint32_t epoch,
                       void* C_local, int comm_cus, int activation /* pk_activation */,
                       uint32_t* status, uint64_t timeout_us, void* stream);

/*
 * Peer emulation (tests and benchmarks only; stands in for what other ranks would push over the fabric).
 *
 * pk_emu_deliver_chunks: for i = 0..n_order-1, copy chunk q = order[i] (M/P x K elements of `elem_bytes`
 * bytes) from staging[q] = staging + q*chunk_bytes into rows R_q of A_gathered, release, set
 * chunk_flags[q] = epoch, then idle `gap_us` microseconds before the next chunk.
 *
 * pk_emu_deliver_partials: for i = 0..n_order-1, q = order[i]: copy every flag tile of staging slot q
 * ([P][M/P][N] fp32, same layout as `partials`) into partials[q], tile by tile, release and set
 * flags_in[q][tile] = epoch after each tile; idle `gap_us` between slots.
 *
 * `order` is a HOST array of at most PK_EMU_MAX_ORDER distinct ranks (the caller excludes its own rank).
 * n_wg is the number of communicator workgroups (one per compute unit; it sets the delivery bandwidth), 0 = 32.
 * `counters` is device scratch of at least PK_EMU_MAX_ORDER uint32, zeroed by the caller before each call.
 * Launch these on a second stream BEFORE the consuming call so that their workgroups are resident.
 */
#define PK_EMU_MAX_ORDER 64
pk_status pk_emu_deliver_chunks(int P, int64_t M, int64_t K, int elem_bytes,
                                const void* staging, void* A_gathered,
                                uint32_t* chunk_flags, uint32_t epoch,
                                const int* order /* host */, int n_order, uint32_t gap_us, int n_wg,
                                uint32_t* counters, void* stream);
/* The same delivery of chunks without communicator workgroups (paper section 3.1.2, host-initiated copy engine
 * transfers): one device-to-device copy per chunk on `stream`, each followed by a stream memory operation that writes the
 * chunk's flag.  No compute unit is taken from the consumer; granularity is a whole chunk. */
pk_status pk_emu_deliver_chunks_dma(int P, int64_t M, int64_t K, int elem_bytes,
                                    const void* staging, void* A_gathered,
                                    uint32_t* chunk_flags, uint32_t epoch,
                                    const int* order /* host */, int n_order, void* stream);
/* Column chunks for pk_ag_gemm_k, moved the same way: one strided (2-D) device-to-device copy per chunk, M pieces of
 * K/P elements, then the chunk's flag by a stream memory operation. */
pk_status pk_emu_deliver_kchunks_dma(int P, int64_t M, int64_t K, int elem_bytes,
                                     const void* staging, void* A_gathered,
                                     uint32_t* chunk_flags, uint32_t epoch,
                                     const int* order /* host */, int n_order, void* stream);
pk_status pk_emu_deliver_partials(int P, int64_t M, int64_t N, int tile_m, int tile_n,
                                  const float* staging, float* partials,
                                  uint32_t* flags_in, uint32_t epoch,
                                  const int* order /* host */, int n_order, uint32_t gap_us, int n_wg,
                                  void* stream);

/*
 * Measurement aid, not part of the method: a register-only loop of 32x32x16 bf16 MFMAs (2 workgroups of 4 waves
 * per compute unit, `iters` rounds of 16 MFMAs per wave) on operands that are all 1.0 (random_operands = 0) or
 * random sign + mantissa (1).  Timed by the caller with events around the call, it gives the MFMA rate the chip
 * sustains at the clock it holds under that data; `*flops_out` (host, may be NULL) receives the flop count of the
 * launch.  `report` is device memory of 4 uint64: [0] wall-clock ticks (100 MHz) and [1] core-clock cycles that one
 * workgroup ran, [2..3] reserved.  Asynchronous on `stream`; PK_ERR_NULL / PK_ERR_ARG (iters outside [1, 2^22]).
 */
pk_status pk_probe_mfma(int iters, int random_operands, uint64_t* report, double* flops_out /* host */, void* stream);

/*
 * Compute-unit partition (paper section 3.1.3, overlap across SMs and its SM-partition study; appendix D
 * num_comm_sms): creates two streams whose kernels run on disjoint sets of compute units, `comm_cus` of them
 * (a multiple of 8 in [8, #CU - 8], spread evenly over the 8 XCDs) for the communicator side and the rest for
 * the compute side.  Launch the communicator (here: pk_emu_deliver_*) on *comm_stream and pk_gemm_rs /
 * pk_ag_gemm with the same comm_cus on *compute_stream: the persistent GEMM then fills exactly its partition and
 * neither side waits for, or shares a compute unit with, the other.  Both handles are hipStream_t, owned by the
 * caller until pk_partition_destroy (which does not synchronise: drain them first).  Host call; PK_ERR_NULL,
 * PK_ERR_ARG (comm_cus), PK_ERR_HIP.
 */
pk_status pk_partition_create(int comm_cus, void** compute_stream /* host out */, void** comm_stream /* host out */);
pk_status pk_partition_destroy(void* compute_stream, void* comm_stream);

#ifdef __cplusplus
}
#endif
#endif /* PK_H */
