/*
 * tf.h -- C boundary of libtf_gfx950.so
 *
 * A family of hand-written gfx950 (MI355X) kernels for the tile kernel
 *
 *      Y = GELU_erf(A . B + bias)          A[M,K], B[K,N], bias[N], Y[M,N], bf16, fp32 accumulate
 *
 * (further epilogues: tf_epilogue) and the profiling-guided variant loop of the paper (Sec. 3.3,
 * Algorithm 1) over that family; behind the same calls, the operations of the paper's three case
 * studies (Sec. 5; tf_op).  The paper's objects map as follows:
 *   hardware profile H ............ tf_hw            (tf_hw_query)
 *   kernel K, candidates K' ....... tf_variant_desc  (tf_variant_enumerate; id 0 is the baseline kernel)
 *   BuildRun(K') .................. tf_variant_run   (a non-OK status is the paper's "res = fail")
 *   Profile(K') -> R' ............. tf_variant_profile (Sec. 3.4 "Profiling": warm-up + timed iterations
 *                                   bracketed by events and a synchronisation)
 *   Arbiter, RefineHint, Proposal . tf_arbiter, tf_refine_hint, tf_proposal (host only, no GPU needed)
 *   the whole loop ................ tf_tune
 *
 * Conventions
 *   - C linkage, no exceptions cross the boundary; functions return a tf_status
 *     (0 = ok, negative = error; nothing is launched on error) unless stated otherwise.
 *     tf_last_error() gives a thread-local message for the last failure.
 *   - "device pointer" = address in the memory of the GPU the problem was created for; the
 *     caller owns every buffer and the stream.  "host pointer" = ordinary process memory.
 *   - bf16 tensors are raw uint16_t bit patterns, row-major, leading dimensions in elements.
 *   - A kernel launch is asynchronous on the given stream; tf_variant_profile and tf_tune
 *     synchronise that stream before they return.
 *   - There is no CPU fallback: without a GPU every launching call fails with TF_E_LAUNCH.
 *   - A tf_problem is not thread safe (it owns a lazily allocated workspace and per-kernel set-up
 *     flags): one thread at a time per problem; different problems are independent. Launches of one
 *     problem that use its own split-K workspace must be ordered on one stream (they share it).
 *   - After one eager call of a variant, tf_variant_run records nothing but kernel launches, so it
 *     may be captured into a HIP graph.
 */
#ifndef TF_H_
#define TF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TF_OK = 0,
  TF_E_INVALID = -1,      /* bad argument (null pointer, negative size, unknown id ...) */
  TF_E_UNSUPPORTED = -2,  /* the variant cannot run this problem (shape, alignment, LDS, workspace) */
  TF_E_LAUNCH = -3,       /* HIP reported an error (no device, launch failure ...) */
  TF_E_NOMEM = -4,        /* host or device allocation failed */
  TF_E_RANGE = -5,        /* output capacity too small */
  TF_E_PROFILER = -6      /* counter file missing or not parseable */
} tf_status;

typedef enum {
  TF_EPI_BIAS_GELU_ERF = 0, /* Y (bf16) = round_nearest_even(GELU_erf(A.B + bias))                  */
  TF_EPI_NONE_F32 = 1,      /* Y (float) = A.B + bias, the fp32 pre-activation; used by exactness tests */
  TF_EPI_BIAS = 2,          /* Y (bf16) = round_nearest_even(A.B + bias): bias only, no activation         */
  TF_EPI_BIAS_GELU_TANH = 3 /* Y (bf16) = round_nearest_even(GELU_tanh(A.B + bias)),
                               GELU_tanh(z) = z/2 (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3)))               */
} tf_epilogue;

typedef enum {
  TF_KIND_NAIVE = 0,        /* one thread per output element, scalar FMA loop: the baseline kernel K */
  TF_KIND_MFMA_DIRECT = 1,  /* one wave per 32x32 tile, MFMA operands loaded straight from memory     */
  TF_KIND_MFMA_LDS = 2,     /* LDS-staged, multi-buffered, swizzled MFMA tile kernel                  */
  TF_KIND_MFMA_STREAM = 3,  /* skinny problems (M <= 32): B streamed once from memory into MFMA operand
                               registers, no LDS staging; the waves of a work-group split K            */
  TF_KIND_VECMAT_NAIVE = 4, /* TF_OP_BATCHED_VECMAT baseline: one thread per output, scalar loop over k */
  TF_KIND_VECMAT_STREAM = 5, /* TF_OP_BATCHED_VECMAT: a wave per group of rows, k-contiguous 16-byte loads,
                               lane-exchange reduction. Descriptor fields: bm = rows per wave, bk = 512,
                               stages = k chunks in flight per row, waves_k = waves per work-group,
                               group_m = work-groups per compute unit the grid is cut to (0 = one wave
                               per row group)                                                          */
  TF_KIND_BGEMM_TN_NAIVE = 6,/* TF_OP_BATCHED_GEMM_TN baseline: one thread per output element (its tile kernels
                               are TF_KIND_MFMA_LDS, see trans_a)                                       */
  TF_KIND_SIN = 7            /* TF_OP_ELEMENTWISE_SIN: one arithmetic, many launch shapes. Descriptor fields: threads,
                               bn = elements per work-group and pass (the paper's BLOCK_SIZE; variant 0 has 4),
                               bk = consecutive elements per thread, stages = passes per work-group,
                               group_m = work-groups per compute unit of a grid-stride launch (0 = one
                               work-group per block of elements)                                        */
} tf_kind;

/* Bottleneck classes produced by tf_refine_hint (Sec. 3.3 "Targeted-Refinement-Hint":
 * profiler deltas become a direction for the next proposal). */
typedef enum {
  TF_BN_UNKNOWN = 0,
  TF_BN_UNDERFILLED = 1,   /* fewer work-groups than compute units, or a badly quantised last wave  */
  TF_BN_HBM = 2,           /* memory traffic near the HBM roof on a shape below the ridge point      */
  TF_BN_MFMA = 3,          /* matrix pipes busy: nothing left but quantisation                       */
  TF_BN_LDS_CONFLICT = 4,  /* LDS bank conflicts above the threshold                                  */
  TF_BN_OCCUPANCY = 5,     /* resident waves limited by registers / LDS                               */
  TF_BN_LATENCY = 6        /* nothing saturated: stalls on staging, needs deeper buffering            */
} tf_bottleneck;

typedef enum { TF_DEC_CONTINUE = 0, TF_DEC_ACCEPT = 1, TF_DEC_FINISH = 2 } tf_decision;

/* The operation. */
typedef enum {
  TF_OP_GEMM_EPILOGUE = 0,  /* Y = epilogue(A.B + bias): A [M][lda], B [K][ldb] (or [N][ldb], see trans_b), bias [N], Y [M][ldy] */
  TF_OP_BATCHED_VECMAT = 1, /* Case Study 2 of the paper (Sec. 5): C[m][n] = sum_k A[m][k] B[m][n][k].
                               A [M][lda] bf16 (lda >= K); B [M][N][ldb] bf16, k contiguous (ldb >= K),
                               matrix m starting N * ldb elements after matrix m - 1; Y = C as fp32
                               [M][ldy] (epi must be TF_EPI_NONE_F32); bias is not read (may be NULL) */
  TF_OP_BATCHED_GEMM_TN = 2,/* Case Study 3 of the paper (Sec. 5), dB = dO^T A per chunk:
                               C[b][m][n] = sum_k A[b][k][m] B[b][k][n], b < batch.
                               A [batch][K][lda] bf16 with m contiguous (lda >= M), B [batch][K][ldb] bf16
                               (ldb >= N), Y = C as fp32 [batch][M][ldy] (epi must be TF_EPI_NONE_F32);
                               consecutive items are stride_a / stride_b / stride_y elements apart;
                               bias is not read (may be NULL) */
  TF_OP_ELEMENTWISE_SIN = 3 /* Case Study 1 of the paper (Sec. 5): Y[i] = sin(A[i]), i < N, A and Y fp32 (binary32)
                               arrays of N elements (M = 1, K = 0; epi must be TF_EPI_NONE_F32); B and bias
                               are not read (may be NULL)                                               */
} tf_op;

/* The problem: shapes and strides of one call of the tile kernel. */
typedef struct {
  int32_t M, N, K;
  int64_t lda, ldb, ldy;   /* leading dimensions in elements; lda >= K, ldb >= N (TF_OP_BATCHED_VECMAT: >= K), ldy >= N */
  int32_t epi;             /* tf_epilogue */
  int32_t device;          /* HIP device ordinal */
  int32_t op;              /* tf_op */
  int32_t batch;           /* TF_OP_BATCHED_GEMM_TN: number of items (>= 0); otherwise ignored */
  int64_t stride_a, stride_b, stride_y;   /* TF_OP_BATCHED_GEMM_TN: elements between consecutive items
                                             (>= K * lda, K * ldb, M * ldy); otherwise ignored */
  int32_t trans_b;         /* TF_OP_GEMM_EPILOGUE: 1 = B is given as [N][ldb] with k contiguous (ldb >= K), a weight
                              matrix stored output-major; 0 = B is [K][ldb] (ldb >= N). Otherwise ignored */
} tf_problem_desc;

/* One member of the kernel family: the paper's "tiling/block shapes, num_warps, vectorization
 * width, memory layout, prefetching, loop splitting" axes (Sec. 3.3, Initialization-and-Proposal). */
typedef struct {
  int32_t id;              /* index for tf_variant_run; 0 is always the naive baseline */
  int32_t kind;            /* tf_kind */
  int32_t bm, bn, bk;      /* macro tile M, N, K (tile kernels: bk = 32, 64 or 128); TF_KIND_SIN: bn = elements per work-group and pass of its grid stride (the
                              case's BLOCK_SIZE), bk = consecutive elements per lane and access, stages = accesses
                              per lane and pass, group_m = work-groups per CU of a grid-stride launch (0: one
                              work-group per bn elements) */
  int32_t waves_m, waves_n;/* wave grid inside the work-group (64-lane waves) */
  int32_t waves_k;         /* wave groups along k: each takes 1/waves_k of every K step of the same tile, the groups
                              add their accumulators through LDS before the epilogue (1 = none) */
  int32_t stages;          /* LDS buffers in the ring */
  int32_t split_k;         /* K slices, summed in fp32 in slice order (1 = no split) */
  int32_t fused_reduce;    /* split_k > 1: 2 = as 1, with the partial tiles exchanged through the L2 of the one XCD
                              that all slices of a tile run on (offered when the tile count is a multiple of 8 and
                              the rows of the partial sums are whole 128-byte lines, N a multiple of 32; launched
                              only on a device whose work-group placement has been probed, see tf_variant_run);
                              1 = the last slice to arrive reduces inside the GEMM kernel (one launch,
                              arrival counters); 0 = a second kernel sums the slices and applies the epilogue */
  int32_t direct_to_lds;   /* 1: global_load_lds staging; 0: via registers (allows a ragged K tail) */
  int32_t a_bypass_lds;    /* 1: A fragments are loaded from memory straight into MFMA operand registers, only B is
                              staged in LDS (one wave column per work-group) */
  int32_t trans_a;         /* TF_OP_BATCHED_GEMM_TN, tile kernels: 1 = the A tile is staged as it lies in memory
                              ([k][m]) and transposed by the LDS read; 0 = a separate pass first writes A^T
                              into the workspace and the tile kernel reads that                        */
  int32_t trans_b;         /* problems with B given as [N][K] (tf_problem_desc.trans_b): 1 = a tile kernel compiled for
                              that layout (the B tile is staged [n][k] and read like the A tile); 0 on a tile kernel
                              = a separate pass first writes B^T ([K][N]) into the workspace and an ordinary tile
                              kernel reads that (names ending in `pretransB`) - the kernel-or-host transposition
                              question of the paper's Case Study 3                                      */
  int32_t stream_k;        /* 1: stream-K scheduling. All but the last one to two rounds of tiles are computed whole,
                              one work-group each; the K steps of the remaining tiles are dealt out evenly to one
                              further work-group per CU, each taking up to three (tile, K range) pieces; a tile
                              has at most two contributors, who exchange fp32 partial tiles through the workspace
                              like two split-K slices (offered when the tile count is above the CU count and no
                              multiple of it; split_k stays 1) */
  int32_t k_rotate;        /* tile kernels without split-K: 1 = the work-groups of XCD x walk through K starting x/8 of the
                              way in and wrapping round, so that the eight XCDs fetch different slabs of A and B at
                              any moment (a different, equally valid, summation order) */
  int32_t persistent;      /* TF_OP_BATCHED_GEMM_TN tile kernels: 1 = one work-group per CU walks through many output
                              tiles and fetches the next tile's K steps while the current one multiplies and
                              writes out (whole tiles, at least stages - 1 K steps per tile); grid = work-groups */
  int32_t bn_tail;         /* tile kernels: > 0 = a launch with a lighter last round. Whole rounds of bm x bn tiles (one
                              per CU and round) cover the leading columns; one more round of exactly one work-group
                              per CU shares out the remaining columns of every row panel in tiles of which only
                              bn_tail columns are multiplied, so every CU gets the same number of tiles and nearly
                              the same work (offered when the rows make a whole number of CUs per row panel and the
                              remaining columns fit such a round; names with `tail`); 0 = all tiles alike */
  int32_t nontemporal;     /* TF_KIND_SIN: 1 = loads and stores marked non-temporal (each element is touched once) */
  int32_t xcd_swizzle;     /* 1: work-group ids renumbered so that neighbouring tiles share an XCD L2;
                              0 (names with _rr, problems with one row of tiles): tiles dealt round-robin over the
                              XCDs, slice by slice, so that every row of B is read through all eight L2s at once */
  int32_t group_m;         /* tile rows per group in the tile order */
  int32_t threads;         /* work-group size */
  int32_t lds_bytes;       /* LDS per work-group */
  int32_t grid;            /* work-groups launched for this problem */
  int64_t workspace_bytes; /* device workspace tf_variant_run needs (0 if none) */
  char name[64];
} tf_variant_desc;

/* The profiler report R of the paper for one variant on one problem. */
typedef struct {
  int32_t variant_id;
  int32_t status;                /* tf_status of the run; timing fields are valid only for TF_OK */
  int32_t warmup, iters, launches_per_iter;
  double t_min_us, t_med_us, t_mean_us, t_max_us;   /* per launch */
  double tflops, gbytes_per_s;   /* from the algorithmic flops 2MNK and bytes 2(MK + KN + MN + N) */
  double pct_mfma_peak, pct_hbm_peak;
  double arithmetic_intensity;   /* algorithmic flop per byte of the problem */
  int32_t grid, waves_per_simd;  /* launch size; resident waves per SIMD allowed by registers and LDS */
  int32_t vgprs, agprs, sgprs, spill_bytes, lds_bytes;
  double occupancy_pct;          /* waves_per_simd / 8 */
  double grid_fill;              /* grid / (compute units * resident work-groups per CU), tail included */
  int32_t have_counters;         /* 1 once tf_report_set_counters has filled (some of) the next six fields */
  double mfma_busy_pct, lds_bank_conflict_pct, hbm_read_gbs, hbm_write_gbs, l2_hit_pct;
  double achieved_occupancy_pct; /* resident waves per SIMD over the dispatch, as a share of max_waves_per_simd */
  int32_t bottleneck;            /* tf_bottleneck, filled by tf_refine_hint / tf_tune */
  int32_t parity_ok;             /* set by the caller's correctness gate; tf_tune takes it from its callback */
} tf_report;

/* Hardware profile H. */
typedef struct {
  char name[64];
  int32_t cus, simds_per_cu, wave_size, xcds;
  int32_t lds_bytes_per_cu, vgprs_per_simd_lane, max_waves_per_simd;
  int64_t l2_bytes, hbm_bytes;
  double clock_mhz, hbm_gbs_peak, bf16_tflops_peak;
} tf_hw;

/* Arbiter thresholds (the paper's Theta; it names the criteria, the values are this library's). */
typedef struct {
  double first_accept_speedup;  /* a candidate replaces the baseline only at >= this speedup (1.05) */
  double later_accept_gain;     /* ... and a previously accepted best at >= this (1.02)              */
  double robust_spread;         /* reject timings whose (median - min) / median exceeds this (0.10) */
  int32_t patience;             /* finish after this many consecutive rounds without an accept (4)  */
  int32_t max_rounds;           /* hard cap on optimisation rounds (8)                               */
  int64_t cold_bytes;           /* Profile stage of tf_tune: > 0 = time every candidate on rotating copies of
                                   A, B and Y that together exceed this many bytes, so that no launch finds
                                   its operands in cache (as a kernel profiler that flushes caches between
                                   replays would measure; default 512 MiB, twice the memory-side cache);
                                   0 = time back-to-back launches on the caller's buffers               */
} tf_theta;

typedef struct tf_problem tf_problem;   /* opaque; created and destroyed by the library */

/* Fills *out with the library defaults for Theta. */
void tf_theta_default(tf_theta* out);

/* H of device `device` (host pointer out). */
tf_status tf_hw_query(int32_t device, tf_hw* out);
/* Same structure without touching a GPU: the published MI355X figures. */
void tf_hw_nominal(tf_hw* out);
/* What device `device` sustains, measured now (host pointers out, either may be NULL): bf16 MFMA
 * TFLOP/s of a register-only 32x32x16 loop on data-like operands running for a few milliseconds
 * (the clock under MFMA load depends on the operand bits), and GB/s of a streaming read of 1 GiB
 * that the library allocates and frees. Synchronises hip_stream. Context for the roofline
 * fractions, which are quoted against the published peaks. */
tf_status tf_hw_measure(int32_t device, void* hip_stream, double* mfma_tflops, double* hbm_read_gbs);

/* The rate of a plain streaming read at a given size, for comparison with a memory-bound kernel of that size:
 * `launches` launches of a kernel that reads `bytes` bytes once (every wave 8 KB of its own, contiguous, as eight
 * 16-byte non-temporal loads per lane all in flight together: the fastest of the read patterns tried; column
 * strips or a grid-stride walk read up to a quarter slower), launch i from buffers[i % n_buffers] (a host
 * array of device pointers to caller-owned buffers of at least `bytes` bytes each, 16-byte aligned; rotate over
 * more than the memory-side cache holds to read from HBM every time). *gbs (host pointer) gets the average rate
 * per launch between two events on hip_stream, which is synchronised. */
tf_status tf_hw_read_rate(int32_t device, void* hip_stream, const void* const* buffers, int32_t n_buffers,
                          int64_t bytes, int32_t launches, double* gbs);

/* Validates desc (host pointer) and creates the problem. M, N, K >= 0. */
tf_status tf_problem_create(const tf_problem_desc* desc, tf_problem** out);
void tf_problem_destroy(tf_problem* p);

/* Lists the variants that can run this problem (shape, alignment and LDS limits checked).
 * out may be NULL to ask for the count. Returns the count (>= 1), or a negative tf_status;
 * TF_E_RANGE if cap is too small. Needs no GPU. */
int32_t tf_variant_enumerate(const tf_problem* p, tf_variant_desc* out, int32_t cap);

/* BuildRun: launches variant `variant_id` on `hip_stream` (a hipStream_t, may be NULL for the
 * default stream). A, B, bias, Y: device pointers (Y: bf16 or float per desc.epi).
 * workspace: device pointer of at least the variant's workspace_bytes, 256-byte aligned, or NULL to
 * let the library use a buffer it allocates once per problem and keeps until tf_problem_destroy.
 * Layout: [arrival counters and one status word | fp32 partial sums]. A caller's workspace has its
 * counter area zeroed by a fill kernel ahead of every launch (its contents between calls are the
 * caller's); the library's own buffer is zeroed once, the kernels leave the counters zero.
 * Calls that share a workspace must not overlap.
 * Variants with fused_reduce == 2 rely on work-groups whose ids are equal modulo 8 running on one
 * XCD. The first such launch on a device runs a small probe kernel and waits for it (a
 * synchronisation of the stream, once per device and process); if the probe does not confirm the
 * placement, these variants fail with TF_E_UNSUPPORTED on that device and nothing is launched.
 * Should a later launch still find the slices of a tile on different XCDs, the tile is written as
 * NaN and the status word of the workspace is set: tf_variant_profile, tf_tune and
 * tf_workspace_status then fail with TF_E_LAUNCH. */
tf_status tf_variant_run(tf_problem* p, int32_t variant_id, const void* A, const void* B,
                         const void* bias, void* Y, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/* Same launch for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the workspace is a buffer of
 * tf_static_scratch_bytes() bytes that is part of the library's device image, one copy per GPU,
 * held until the process ends. The call allocates nothing and frees nothing. Variants whose
 * workspace_bytes exceed the buffer fail with TF_E_UNSUPPORTED (nothing launched). The counter
 * area is zeroed by a fill kernel ahead of every launch (no memset node), the rest keeps the last
 * call's contents. Every call on a GPU shares that GPU's buffer: calls that overlap on one GPU
 * race, whatever their streams or problems. The first fused_reduce == 2 launch on a device still
 * runs the placement probe described above (it uses the same buffer). */
tf_status tf_variant_run_static(tf_problem* p, int32_t variant_id, const void* A, const void* B,
                                const void* bias, void* Y, void* hip_stream);
/* Size of that buffer in bytes. */
int64_t tf_static_scratch_bytes(void);

/* Synchronises hip_stream and reads the status word of `workspace` (device pointer; NULL = the
 * problem's own buffer): TF_OK, or TF_E_LAUNCH if a launch since the last zeroing of the counter
 * area found the slices of a tile on different XCDs (fused_reduce == 2). */
tf_status tf_workspace_status(tf_problem* p, const void* workspace, void* hip_stream);

/* The host-side decision of the placement probe: xcc_of_wg[i] (host pointer) is the XCD that
 * work-group i of a probe launch reported, n their number. Returns 1 if all work-groups with equal
 * i modulo 8 ran on one XCD (n >= 16), else 0. Needs no GPU. */
int32_t tf_xcc_placement_ok(const uint32_t* xcc_of_wg, int32_t n);

/* Profile: `warmup` untimed iterations, then `iters` timed ones; each iteration brackets
 * `launches_per_iter` back-to-back launches (0 = pick so that an iteration lasts >= ~1 ms)
 * between two events on the stream and synchronises. Fills *out (host pointer), including the
 * static resource figures. Synchronous. */
tf_status tf_variant_profile(tf_problem* p, int32_t variant_id, const void* A, const void* B,
                             const void* bias, void* Y, void* workspace, size_t workspace_bytes,
                             void* hip_stream, int32_t warmup, int32_t iters,
                             int32_t launches_per_iter, tf_report* out);

/* Reads a rocprofv3 counter CSV (`rocprofv3 --pmc ... --output-format csv`: columns Kernel_Name,
 * Counter_Name, Counter_Value; Dispatch_Id, Start_Timestamp, End_Timestamp if present) and fills
 * the counter fields of *r (Sec. 3.4 "Profiling": the report carries what the profiler measured)
 * from the rows whose kernel name contains `kernel_substr`, averaged over its dispatches:
 *   mfma_busy_pct          SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / xcds * cus * simds_per_cu)
 *                          (without GRBM_GUI_ACTIVE: / (SQ_BUSY_CU_CYCLES * simds_per_cu))
 *   achieved_occupancy_pct 4 SQ_WAVE_CYCLES / (GRBM_GUI_ACTIVE / xcds * cus * simds_per_cu * max_waves_per_simd)
 *   lds_bank_conflict_pct  SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE
 *   hbm_read_gbs           2 * FETCH_SIZE KiB / dispatch time;  hbm_write_gbs  WRITE_SIZE KiB / dispatch time
 *   l2_hit_pct             TCC_HIT_sum / (TCC_HIT_sum + TCC_MISS_sum)
 * A file holds the counters of one profiler pass; call once per file, fields a file does not cover keep
 * their values. Sets have_counters and re-classifies r->bottleneck. TF_E_PROFILER if the file cannot be
 * read, has no matching row or none of these counters. hw, csv_path, kernel_substr: host pointers. */
tf_status tf_report_set_counters(tf_report* r, const tf_hw* hw, const char* csv_path,
                                 const char* kernel_substr);

/* The part of a kernel's name in profiler output that identifies the compiled kernel behind variant v
 * (variants that differ only in launch parameters, such as K slices or the K order, share a kernel),
 * written to buf (host pointer, cap bytes, NUL-terminated): the kernel_substr for
 * tf_report_set_counters. Returns its length, 0 for kernels whose template arguments the
 * descriptor does not spell out (buf is then empty), TF_E_RANGE if cap is too small. Needs no GPU. */
int32_t tf_variant_kernel_name(const tf_variant_desc* v, char* buf, int32_t cap);

/* Hands the loop what a profiler measured (Sec. 3.4 "Profiling": the report that RefineHint reads
 * carries the profiler's figures): csv_paths[0..n) (host pointers, copied) are rocprofv3 counter
 * CSVs of earlier passes over this problem's kernels, one per counter set, e.g. of a command that
 * launches every variant the loop may visit. tf_tune then fills the counter fields of every
 * round's report from the rows of that round's kernel (tf_report_set_counters with
 * tf_variant_kernel_name) before RefineHint classifies it, so that the hint rests on matrix-pipe
 * busy, HBM and LDS-conflict figures instead of rates derived from the time; a kernel that no file
 * holds keeps have_counters = 0. Pass the matrix-pipe and the memory passes together: a figure no
 * file holds reads zero. n = 0 forgets the files. TF_E_INVALID if a file cannot be opened. */
tf_status tf_problem_set_counter_files(tf_problem* p, const char* const* csv_paths, int32_t n);

/* ---- the loop's host logic: pure functions, callable without a GPU ---------------------- */

/* Performance-Arbiter: decision for candidate report `cand` against best-so-far `best`.
 * best_is_baseline != 0 while nothing has been accepted yet; stall_rounds = consecutive
 * rounds without an accept before this one; round = 1-based index of this round. */
int32_t tf_arbiter(const tf_report* cand, const tf_report* best, const tf_theta* theta,
                   int32_t best_is_baseline, int32_t stall_rounds, int32_t round);

/* Targeted-Refinement-Hint (Sec. 3.3): classifies the bottleneck of `cand` (tf_bottleneck) from its
 * counters if it has any, else from its achieved rates. `prev` (may be NULL) is the report of the
 * round before, whose bottleneck field is the hint `cand` was proposed under (TF_BN_UNKNOWN: read
 * from prev's own figures): if cand is more than 2 % slower than prev and its figures call for that
 * same remedy again, the remedy has just failed and the hint turns round between "occupancy" and
 * "latency" (the alternation of the rounds of Case Study 3, Sec. 5). */
int32_t tf_refine_hint(const tf_report* prev, const tf_report* cand, const tf_hw* hw);

/* Proposal: id of the next candidate among family[0..n), none of which has tried[id] != 0,
 * given the current kernel `base_id` and its bottleneck class; -1 when the family is
 * exhausted. prob gives the shape. */
int32_t tf_proposal(const tf_problem_desc* prob, const tf_hw* hw, const tf_variant_desc* family,
                    int32_t n, const uint8_t* tried, int32_t base_id, int32_t bottleneck);

/* Proposal given the family's predicted times (predicted_us[i] for family[i]): among the
 * untried tile kernels that move in the direction the bottleneck asks for, relative to
 * family[base_id], the one with the smallest predicted time; if none qualifies (or the base is
 * not a tile kernel, or the class is TF_BN_UNKNOWN) the untried variant with the smallest
 * predicted time; -1 if every variant has been tried. Ties go to the lower id. */
int32_t tf_proposal_from(const tf_hw* hw, const tf_variant_desc* family, const double* predicted_us,
                         int32_t n, const uint8_t* tried, int32_t base_id, int32_t bottleneck);

/* Static cost model behind tf_proposal: predicted time in microseconds of variant v on the
 * problem, from tile shape, wave quantisation and the measured LDS / load-path rates. */
double tf_predict_us(const tf_problem_desc* prob, const tf_hw* hw, const tf_variant_desc* v);
/* Work-groups of v that fit on one compute unit (registers and LDS), 1..8. */
int32_t tf_resident_wgs(const tf_hw* hw, const tf_variant_desc* v);
/* v->grid / (rounds * cus * resident work-groups): 1.0 when the last round is full. */
double tf_grid_fill(const tf_hw* hw, const tf_variant_desc* v);

/* Algorithm 1 over pre-made reports: reports[i] is what Profile would return for family[i]
 * (reports[0] the baseline). Same outputs as tf_tune; needs no GPU. */
tf_status tf_tune_replay(const tf_problem_desc* prob, const tf_hw* hw, const tf_variant_desc* family,
                         const tf_report* reports, int32_t n, const tf_theta* theta,
                         int32_t* best_variant, tf_report* best, tf_report* round_log,
                         int32_t log_cap, int32_t* n_log);

/* Correctness gate used by tf_tune after each BuildRun (the paper verifies functional
 * equivalence of every candidate before its time counts). Returns non-zero if Y is accepted. */
typedef int32_t (*tf_parity_fn)(void* user, int32_t variant_id);

/* The comparison of tf_tune's built-in gate, on host arrays (all host pointers; needs no GPU).
 * Y: the candidate's output, rows x N with leading dimension ldy, bf16 bit patterns or float per
 * epi. zref: fp32 pre-activation of the baseline kernel, dense rows x N (for the operations
 * without bias: its output). norm_a[m], norm_b[m * norm_b_row_stride + n]: Euclidean norms of
 * the two vectors whose dot product element (m, n) is; their product bounds sum |a b|.
 * An element passes if
 *   |y - act(zref)| <= 2^-8 |act(zref)| + 1.13 (3 g norm_a norm_b + 2^-22 |zref|) + 2e-6 (1 + |zref|)
 * for a bf16 epilogue (act = the epilogue's activation evaluated with the math library), and
 *   |y - zref| <= 3 g norm_a norm_b + 2^-22 |zref| + 1e-30
 * for fp32 output, with g = (K + 1) 2^-24 / (1 - (K + 1) 2^-24): one bf16 rounding, the
 * summation error of two fp32 evaluations in any order, the activation's slope. A NaN never
 * passes. Returns the number of elements that fail, or a negative tf_status. */
int64_t tf_gate_count_bad(const void* Y, int64_t ldy, const float* zref, const float* norm_a,
                          const float* norm_b, int64_t norm_b_row_stride, int32_t rows, int32_t N,
                          int32_t K, int32_t epi);

/* Algorithm 1. Profiles the baseline (variant 0), then runs at most theta->max_rounds rounds of
 * Proposal -> BuildRun -> parity gate -> Profile -> Arbiter -> RefineHint. round_log (host
 * pointer, capacity log_cap >= 1 + max_rounds) receives the baseline report followed by one
 * report per round; *n_log their number. *best_variant / *best get K* and R*. Y is filled with
 * NaN before every candidate's BuildRun, so an element a candidate does not write fails the gate.
 * parity may be NULL: the library then compares every candidate with the baseline kernel's fp32
 * pre-activation by the rule of tf_gate_count_bad (on the device). Profile here is Sec. 3.4's
 * 3 warm-up + 5 timed iterations, each timed iteration a batch of launches of about 3 ms, after
 * further untimed launches until 60 ms have been spent on the candidate (the clock needs that
 * long to settle after a change of load), on rotating copies of the operands (theta->cold_bytes). */
tf_status tf_tune(tf_problem* p, const void* A, const void* B, const void* bias, void* Y,
                  void* workspace, size_t workspace_bytes, void* hip_stream,
                  const tf_theta* theta, tf_parity_fn parity, void* parity_user,
                  int32_t* best_variant, tf_report* best, tf_report* round_log, int32_t log_cap,
                  int32_t* n_log);

const char* tf_last_error(void);
const char* tf_version(void);
/* sizeof of tf_problem_desc, tf_variant_desc, tf_report, tf_hw, tf_theta as this library was built, in that
 * order (host pointer out): a binding checks them against its own mirrors before it calls anything else. */
void tf_struct_sizes(int32_t out[5]);

#ifdef __cplusplus
}
#endif
#endif /* TF_H_ */
