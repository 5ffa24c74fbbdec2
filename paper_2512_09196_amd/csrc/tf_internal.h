// Internal declarations shared by the translation units of libtf_gfx950.so.
// Not part of the public boundary (that is include/tf.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "tf.h"

namespace tf {

// Arguments of every GEMM kernel of the family. All pointers are device pointers.
struct GemmParams {
  const uint16_t* A;      // [M, lda] bf16 bits, row-major
  const uint16_t* B;      // [K, ldb] bf16 bits, row-major
  const uint16_t* bias;   // [N] bf16 bits
  void* Y;                // [M, ldy]: bf16 bits (TF_EPI_BIAS_GELU_ERF) or float (TF_EPI_NONE_F32)
  float* ws;              // split-K partial sums [split_k][M][N] (unused when split_k == 1)
  unsigned* counters;     // one 8-byte arrival counter per output tile, zero between launches
  unsigned* status;       // status word of the workspace (behind the counters): bit 0 = an L2-local reduction found its slices on different XCDs
  int M, N, K;
  long lda, ldb, ldy;     // in elements
  long stride_a, stride_b, stride_y;   // batched problems (grid.y = batch items): elements between consecutive items
  int tiles_m, tiles_n;
  int split_k;            // number of K slices
  int fused_reduce;       // split-K: 1 = the last slice to arrive reduces inside the GEMM kernel; 0 = a second kernel does
  int ktiles_per_split;   // K tiles (of BK) per slice; the last slice may be shorter
  int epi;                // tf_epilogue
  int group_m;            // tile rows per L2 group in the tile order (>= 1)
  int xcd_swizzle;        // 1: remap work-group ids so that neighbouring tiles share an XCD
  int slice_major;        // split-K tile order: 1 = slice by slice (two-kernel reduction), 0 = the slices of a tile side by side
  int batch;              // batched problems: number of items (the persistent kernel deals them out itself)
  int stream_k;           // 1: work-groups from sk_first_wg on share the K steps of the last sk_tiles tiles evenly
  int sk_first_wg, sk_tiles, sk_wgs;   // (stream_k) first such work-group = number of tiles computed whole; tiles and work-groups of the shared part
  int k_rotate;           // 1: the K tiles of a work-group start a (blockIdx mod 8) / 8 of the way in and wrap round
  int k_interleave;       // 1 (split-K, direct staging): slice s takes the K tiles s, s + split_k, ... instead of a contiguous range
  int batch_xcd;          // batched problems: 1 = all tiles of a batch item on one XCD (batch a multiple of 8)
  int ws_vec16;           // 1: the split-K workspace starts on a 16-byte boundary (its rows of N floats then do too)
  int y_vec16;            // 1: every row of Y (of every batch item) starts on a 16-byte boundary
  int trans_b;            // 1: B is [N][ldb] with k contiguous (the unstaged kernels read it that way; tile kernels are compiled for one layout)
  // mixed grid (tf_gemm_mixed_kernel): the first mix_main_wgs work-groups compute BN-wide tiles (tiles_m x tiles_n of them),
  // then tiles_m x mix_tiles work-groups share out the mix_blocks blocks of 32 columns that begin at column mix_n_origin
  int mix_main_wgs, mix_tiles, mix_blocks, mix_n_origin;
};

// One compiled kernel of the LDS-staged MFMA family.
struct LdsKernelInfo {
  int bm, bn, bk, waves_m, waves_n, waves_k, stages, direct_to_lds, a_bypass_lds;
  int trans_a;            // 1: A is [K][lda] with m contiguous (staged and read like the B tile)
  int trans_b;            // 1: B is [N][ldb] with k contiguous (staged and read like the A tile)
  int threads, lds_bytes;
  int fused_ok;           // 1: the kernel contains the in-kernel split-K reduction (fused_reduce 1 and 2)
  int stream_k;           // 1: instance with the loop over (tile, K range) segments compiled in (stream-K variants only)
  int persistent;         // 1: tf_bgemm_persist_kernel (one work-group per CU walks through many tiles; grid.x = work-groups)
  int bn_tail;            // > 0: tf_gemm_mixed_kernel, width of the tiles of its lighter last round
  const void* func;       // kernel symbol, for hipFuncGetAttributes / occupancy queries
  void (*launch)(const GemmParams&, dim3 grid, hipStream_t);
};
int lds_kernel_count();
const LdsKernelInfo* lds_kernel_table();

// One compiled kernel of the streaming family for skinny problems (B read once, no LDS staging).
// GemmParams: tiles_n = column blocks of block_n, ktiles_per_split = K blocks of 32 per slice.
struct StreamKernelInfo {
  int m_blocks;           // 16-row blocks of A it covers: M <= 16 m_blocks
  int waves, depth, threads, lds_bytes;   // depth: register sets per wave (depth - 1 K blocks in flight)
  int block_n;            // columns per work-group (128 or 64)
  const void* func;
  void (*launch)(const GemmParams&, dim3 grid, hipStream_t);
};
int stream_kernel_count();
const StreamKernelInfo* stream_kernel_table();

// One compiled kernel of the streaming family of the batched vector-matrix product.
// GemmParams: A [M][lda], B [M][N][ldb] (k contiguous), Y fp32 [M][ldy]; group_m unused.
struct VecmatKernelInfo {
  int rows;               // rows (m, n .. n + rows - 1) a wave works on at a time
  int unroll;             // 512-element k chunks in flight per row
  int waves, threads;
  const void* func;
  void (*launch)(const GemmParams&, dim3 grid, hipStream_t);
};
int vecmat_kernel_count();
const VecmatKernelInfo* vecmat_kernel_table();
void launch_vecmat_naive(const GemmParams&, hipStream_t);
const void* vecmat_naive_func();

// One compiled kernel of the element-wise sine: `block` = threads * vec * iters elements per work-group and pass.
struct SinKernelInfo {
  int threads, vec, iters, block, nontemporal;
  const void* func;
  void (*launch)(const float* x, float* y, size_t n, unsigned grid, hipStream_t);
};
int sin_kernel_count();
const SinKernelInfo* sin_kernel_table();
void launch_sin_block4(const float* x, float* y, size_t n, hipStream_t);     // the baseline: four elements per work-group
const void* sin_block4_func();

void launch_bgemm_tn_naive(const GemmParams&, int batch, hipStream_t);      // C[b] = A[b]^T B[b], one thread per element
const void* bgemm_tn_naive_func();
void launch_transpose(const uint16_t* A, uint16_t* At, int K, int M, long lda, long stride_a, long ldt, long stride_t,
                      int batch, hipStream_t);                              // At[b][m][k] = A[b][k][m]
void launch_naive(const GemmParams&, hipStream_t);
void launch_mfma_direct(const GemmParams&, hipStream_t);
const void* naive_func();
const void* mfma_direct_func();
void launch_fill_u32(unsigned* p, size_t n, unsigned v, hipStream_t);
void launch_fill_rows(void* y, size_t rows, size_t row_bytes, size_t ld_bytes, unsigned pattern, hipStream_t);   // row_bytes, ld_bytes multiples of 2; pattern repeated per 4 bytes (2-byte elements take its low half)
void launch_xcc_probe(unsigned* out, int wgs, hipStream_t);                // out[i] = XCD id work-group i ran on
// Euclidean norms of n_outer x n_inner vectors of `len` bf16 elements: vector (o, i) starts at X + o * outer_stride + i * inner_stride,
// its elements are elem_stride apart; out[o * n_inner + i]
void launch_norms(const uint16_t* X, long n_outer, long outer_stride, long n_inner, long inner_stride, long len, long elem_stride,
                  float* out, hipStream_t);
void launch_calib_mfma(float* sink, int wgs, int iters, hipStream_t);                       // 4 * iters MFMA 32x32x16 per wave, 4 waves per work-group
void launch_calib_read(const void* src, size_t bytes, unsigned* sink, int wgs, hipStream_t);  // reads every byte once
void launch_splitk_reduce(const GemmParams&, hipStream_t);   // sums ws slices in order, bias + epilogue -> Y
const void* splitk_reduce_func();

}  // namespace tf
