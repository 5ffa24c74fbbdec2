// Streaming bf16 MFMA GEMM for skinny problems (M <= 32) on gfx950: Y = epilogue(A B + bias)
// where the whole cost is reading B once from HBM.
//
// B never enters LDS and no barrier sits in the main loop. A work-group owns a block of
// 16 CW columns of Y (CW = 8 or 4 columns per lane) and one slice of K; its NW waves each
// take a contiguous run of 32-row K blocks of that slice and keep their own accumulators, which
// are added through LDS once at the end. Slices of K taken by different work-groups are summed
// in slice order either by the last of them to arrive (arrival counter per column block) or by
// a second kernel; both cost trips to memory after the stream has ended, but one work-group
// per column block over the whole of K leaves most of the chip idle (measured: a CU draws at
// most about 37 GB/s from HBM, and row pieces narrower than 256 bytes lower the rate further).
//
// One K block of one wave is B[k0 .. k0+32)[n0 .. n0 + 16 CW): lane (j = lane % 16,
// g = lane / 16) loads, for e = 0..7, the 2 CW bytes at row k0 + 8 g + e, columns
// n0 + CW j .. + CW: eight global loads per block, each covering four row segments of 32 CW
// bytes. The MFMA (v_mfma_f32_16x16x32_bf16) wants, per lane, eight consecutive k of ONE
// column; the loads deliver CW consecutive columns of one k. Because the lane already holds
// rows k0 + 8 g + 0..7 of its columns, a transposition inside the lane is enough: operand c
// (c = 0 .. CW-1) takes element c of each of the eight loaded vectors (four v_perm_b32), and
// stands for the columns n0 + CW j + c, j = 0..15. The permuted column order only shows in the
// addressing of the (small) output. The A operand, rows of A with eight consecutive k, is
// loaded from memory in MFMA layout directly; A is small and stays in L2.
//
// Accumulators: acc[i][c], lane (j, g), register r  <->  m = 16 i + 4 g + r,  n = n0 + CW j + c.
#include "tf_device.h"

namespace tf {

template <int TMB_, int NW_, int DEPTH_, int CW_ = 8>
struct StreamCfg {
  static constexpr int CW = CW_;              // columns per lane: the column block is 16 CW wide
  static constexpr int NBW = 16 * CW_;
  static_assert(CW == 8 || CW == 4, "16- or 8-byte loads");
  static constexpr int TMB = TMB_;            // 16-row blocks of A: M <= 16 TMB
  static constexpr int NW = NW_;              // waves per work-group, all on the same 128 columns
  static constexpr int DEPTH = DEPTH_;        // register sets per wave: DEPTH - 1 K blocks (8 KB each) in flight
  static_assert(DEPTH >= 2 && DEPTH <= 4, "two to four register sets");
  static constexpr int THREADS = NW * 64;
  static constexpr int FRAGS = TMB * CW;      // 16x16 accumulator blocks per wave
  static constexpr int LDS_BYTES = NW * FRAGS * 1024;
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");

};

template <class C>
__global__ void __launch_bounds__(C::THREADS) tf_gemm_stream_kernel(const GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, g = lane >> 4;
  // consecutive work-groups (which the hardware deals round-robin over the XCDs) take neighbouring
  // column blocks of the same K slice: together they read whole rows of B
  const int tn = blockIdx.x % p.tiles_n, ks = blockIdx.x / p.tiles_n;
  const int n0 = tn * C::NBW;

  // K blocks (of 32) of this work-group's slice, and this wave's run of them
  const int kb_total = p.K / 32;
  const int kb0 = ks * p.ktiles_per_split;
  int kb1 = kb0 + p.ktiles_per_split;
  if (kb1 > kb_total) kb1 = kb_total;
  const int span = kb1 > kb0 ? kb1 - kb0 : 0;
  const int per = (span + C::NW - 1) / C::NW;
  const int wb0 = kb0 + wave * per;
  int wb1 = wb0 + per;
  if (wb1 > kb1) wb1 = kb1;
  const int nb = wb1 - wb0;                    // <= 0: this wave contributes zeros

  int ncol = n0 + C::CW * j;
  const bool n_ok = ncol < p.N;               // N is a multiple of 8: a lane's group of columns is all in or all out
  if (!n_ok) ncol = 0;
  const size_t b_row = (size_t)p.ldb * 2;
  const char* bptr = (const char*)p.B + ((size_t)(32 * (size_t)(nb > 0 ? wb0 : 0) + 8 * g) * p.ldb + ncol) * 2;
  const char* aptr[C::TMB];
#pragma unroll
  for (int i = 0; i < C::TMB; ++i) {
    int m = 16 * i + j;
    if (m >= p.M) m = p.M - 1;                // rows past M repeat the last row; their results are never stored
    aptr[i] = (const char*)p.A + ((size_t)m * p.lda + 32 * (size_t)(nb > 0 ? wb0 : 0) + 8 * g) * 2;
  }

  f32x4 acc[C::TMB][C::CW];
#pragma unroll
  for (int i = 0; i < C::TMB; ++i)
#pragma unroll
    for (int c = 0; c < C::CW; ++c) acc[i][c] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

  typedef unsigned bvec __attribute__((ext_vector_type(C::CW / 2)));   // CW bf16 of one row
  struct Block { bvec b[8]; u32x4 a[C::TMB]; };
  auto dword = [](const bvec& v, int i) -> unsigned { return v[i]; };
  auto load = [&](Block& blk, int rel) {       // K block wb0 + rel of this wave
    const char* bp = bptr + (size_t)rel * 32 * b_row;
#pragma unroll
    for (int e = 0; e < 8; ++e) blk.b[e] = __builtin_nontemporal_load((const bvec*)(bp + e * b_row));   // read once by one wave
#pragma unroll
    for (int i = 0; i < C::TMB; ++i) blk.a[i] = *(const u32x4*)(aptr[i] + (size_t)rel * 64);
  };
  auto compute = [&](const Block& blk) {
#pragma unroll
    for (int c = 0; c < C::CW; ++c) {
      // element c of the eight loaded vectors: dword c / 2, low half for even c, high half for odd c
      const unsigned sel = (c & 1) ? 0x07060302u : 0x05040100u;
      u32x4 f;
#pragma unroll
      for (int q = 0; q < 4; ++q) f[q] = __builtin_amdgcn_perm(dword(blk.b[2 * q + 1], c >> 1), dword(blk.b[2 * q], c >> 1), sel);
      const bf16x8 bf = __builtin_bit_cast(bf16x8, f);
#pragma unroll
      for (int i = 0; i < C::TMB; ++i)
        acc[i][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, blk.a[i]), bf, acc[i][c], 0, 0, 0);
    }
  };

  // DEPTH register sets rotate: while one block is multiplied, the loads of the next DEPTH - 1 are
  // in flight. A load that would run past the wave's last block fetches the last block again, so
  // the loop body has no branch and the compiler's load counters stay exact. The scheduling
  // barriers keep every batch of loads ahead of the MFMAs that cover its latency.
  if (nb > 0) {
    constexpr int D = C::DEPTH;
    Block set[D];
#pragma unroll
    for (int d = 0; d < D - 1; ++d) load(set[d], d < nb ? d : nb - 1);
    int b = 0;
    for (; b + D <= nb; b += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const int nxt = b + d + D - 1;
        load(set[(d + D - 1) % D], nxt < nb ? nxt : nb - 1);
        __builtin_amdgcn_sched_barrier(0);
        compute(set[d]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // fewer than D blocks are left, all of them already loaded: sets 0 .. nb - b - 1
#pragma unroll
    for (int d = 0; d < D - 1; ++d)
      if (b + d < nb) compute(set[d]);
  }

  // ---- sum over the waves, through LDS, in wave order (ascending k)
#pragma unroll
  for (int i = 0; i < C::TMB; ++i)
#pragma unroll
    for (int c = 0; c < C::CW; ++c)
      *(f32x4*)(smem + ((wave * C::FRAGS + i * C::CW + c) * 64 + lane) * 16) = acc[i][c];
  __syncthreads();

  // wave w owns the accumulator blocks w, w + NW, ...: block f = CW i + c covers rows 16 i + 4 g + r
  // and columns n0 + CW j + c
  constexpr int OWN = (C::FRAGS + C::NW - 1) / C::NW;
  const int m_lane = 4 * g, n_lane = n0 + C::CW * j;
  const size_t slice = (size_t)p.M * p.N;
  f32x4 sum[OWN];
#pragma unroll
  for (int o = 0; o < OWN; ++o) {
    const int f = wave + o * C::NW;
    sum[o] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (f < C::FRAGS) {
#pragma unroll
      for (int w = 0; w < C::NW; ++w) sum[o] += *(const f32x4*)(smem + ((w * C::FRAGS + f) * 64 + lane) * 16);
    }
  }

  bool poisoned = false;
  if (p.split_k > 1) {
    // publish this slice's partial sums
    float* wsk = p.ws + (size_t)ks * slice;
#pragma unroll
    for (int o = 0; o < OWN; ++o) {
      const int f = wave + o * C::NW;
      if (f >= C::FRAGS || !n_ok) continue;
      const int n = n_lane + (f % C::CW);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = 16 * (f / C::CW) + m_lane + r;
        if (m >= p.M) continue;
        float* dst = wsk + (size_t)m * p.N + n;
        if (p.fused_reduce == 1) __hip_atomic_store(dst, sum[o][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // through this XCD's L2
        else *dst = sum[o][r];     // summed by the reduce kernel, or (fused_reduce 2) left in the L2 all slices share
      }
    }
    if (!p.fused_reduce) return;
    // The last slice of this column block to arrive sums all slices, in slice order. Every store
    // above has been acknowledged before its wave reaches the barrier, so the ticket taken after
    // the barrier is ordered behind the whole work-group's partial sums.
    // fused_reduce 2: the host has made sure that the slices of a column block are work-groups
    // with the same id modulo 8, i.e. on one XCD, whose L2 holds the plain stores above; every
    // slice reports the XCD it really ran on in its ticket (7-bit field per XCD above the arrival
    // count), and a column block whose slices did not share one is poisoned with NaN.
    const bool local = p.fused_reduce == 2;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    __shared__ unsigned long long ticket;
    unsigned long long* ctr = (unsigned long long*)p.counters + tn;
    const unsigned xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 7u;      // HW_REG_XCC_ID
    const unsigned long long mine = 1ull + (1ull << (8 + 7 * xcc));
    // (L2-local mode: the ticket is taken in this XCD's L2 too, with an atomic of narrower scope)
    if (threadIdx.x == 0)
      ticket = (local ? __hip_atomic_fetch_add(ctr, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : atomicAdd(ctr, mine)) + mine;
    __syncthreads();
    const unsigned long long tk = ticket;
    if ((unsigned)(tk & 255u) != (unsigned)p.split_k) return;
    if (threadIdx.x == 0) *ctr = 0ull;          // ready for the next launch
    poisoned = local && (unsigned)((tk >> (8 + 7 * xcc)) & 127u) != (unsigned)p.split_k;
    if (poisoned && threadIdx.x == 0) atomicOr(p.status, 1u);   // reported by the next synchronous call of the library
#pragma unroll
    for (int o = 0; o < OWN; ++o) {
      const int f = wave + o * C::NW;
      sum[o] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      if (f >= C::FRAGS || !n_ok) continue;
      const int n = n_lane + (f % C::CW);
      for (int sidx = 0; sidx < p.split_k; ++sidx) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int m = 16 * (f / C::CW) + m_lane + r;
          if (m >= p.M) continue;
          const float* src = p.ws + (size_t)sidx * slice + (size_t)m * p.N + n;
          // device-scope loads: from memory, never from a line this XCD's L2 kept from an earlier launch
          sum[o][r] += local ? *src : __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
  }

  // ---- epilogue: + bias, GELU, round to bf16 (or raw fp32 pre-activation)
#pragma unroll
  for (int o = 0; o < OWN; ++o) {
    const int f = wave + o * C::NW;
    if (f >= C::FRAGS || !n_ok) continue;
    if (poisoned) sum[o] = f32x4{__builtin_nanf(""), __builtin_nanf(""), __builtin_nanf(""), __builtin_nanf("")};
    const int n = n_lane + (f % C::CW);
    const float bias = bf16_bits_to_f32(p.bias[n]);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int m = 16 * (f / C::CW) + m_lane + r;
      if (m >= p.M) continue;
      const float z = sum[o][r] + bias;
      if (p.epi == TF_EPI_NONE_F32) ((float*)p.Y)[(size_t)m * p.ldy + n] = z;
      else ((uint16_t*)p.Y)[(size_t)m * p.ldy + n] = f32_to_bf16_bits(activate(z, p.epi));
    }
  }
}

template <class C>
static void launch_stream(const GemmParams& p, dim3 grid, hipStream_t stream) {
  hipLaunchKernelGGL(tf_gemm_stream_kernel<C>, grid, dim3(C::THREADS), C::LDS_BYTES, stream, p);
}

template <class C>
static StreamKernelInfo make_stream_info() {
  StreamKernelInfo k;
  k.m_blocks = C::TMB; k.waves = C::NW; k.depth = C::DEPTH; k.block_n = C::NBW; k.threads = C::THREADS; k.lds_bytes = C::LDS_BYTES;
  k.func = (const void*)tf_gemm_stream_kernel<C>;
  k.launch = launch_stream<C>;
  return k;
}

static StreamKernelInfo g_stream_table[] = {
    make_stream_info<StreamCfg<1, 4, 2>>(), make_stream_info<StreamCfg<1, 8, 2>>(),
    make_stream_info<StreamCfg<1, 8, 4>>(),
    make_stream_info<StreamCfg<2, 4, 2>>(), make_stream_info<StreamCfg<2, 8, 2>>(),
    // narrower column blocks with sixteen waves, for problems with few columns
    make_stream_info<StreamCfg<1, 16, 3, 4>>(), make_stream_info<StreamCfg<2, 16, 2, 4>>(),
};

int stream_kernel_count() { return (int)(sizeof(g_stream_table) / sizeof(g_stream_table[0])); }
const StreamKernelInfo* stream_kernel_table() { return g_stream_table; }

}  // namespace tf
