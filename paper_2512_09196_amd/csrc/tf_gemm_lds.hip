// LDS-staged bf16 MFMA GEMM with fused bias + GELU(erf) epilogue for gfx950.
//
// One work-group computes one BM x BN tile of Y (or one K slice of it). Per K step of
// BK (32, 64 or 128) it stages an A tile [BM][BK] and a B tile [BK][BN] in LDS, multi-buffered,
// and each of the WM x WN waves accumulates a (BM/WM) x (BN/WN) sub-tile with
// v_mfma_f32_32x32x16_bf16 in fp32.
//
// LDS layouts (chosen from measured bank behaviour: 64 banks x 4 B, b128 reads are
// conflict free when 16 consecutive lanes cover 16 distinct 16-byte slots of a 256-byte line):
//   A tile: row-major, 2 BK bytes per row, BK / 8 16-byte chunks per row; chunk c of row r is
//           stored in slot c ^ f(r), f(r) = (r / rows per 256-byte line) mod chunks per row
//           (BK = 64: c ^ ((r >> 1) & 7)). MFMA A operands are ds_read_b128.
//   B tile: row-major as in memory ([k][n], n contiguous), BN*2 bytes per row, split in
//           64-byte pieces; piece j of row k is stored in slot j ^ f(k) so that four
//           consecutive k rows fall in four different bank groups. MFMA B operands, which
//           need 8 consecutive k per lane, are read with the transposing
//           ds_read_b64_tr_b16 (two per operand), so B is never transposed by ALU code.
// Both tiles are written either by global_load_lds_dwordx4 (memory -> LDS without passing
// through registers; the lane -> slot map is fixed by hardware, the swizzle is applied to
// the global address instead) or by 16-byte global loads into registers followed by
// ds_write_b128, which allows zero fill of a ragged K tail.
#include "tf_device.h"

namespace tf {

template <int BM_, int BN_, int BK_, int WM_, int WN_, int STAGES_, bool DIRECT_, bool ABYPASS_ = false, int WK_ = 1, bool TRANSA_ = false,
          bool TRANSB_ = false, int BN_ACT_ = BN_>
struct LdsCfg {
  // BN_ACT < BN: a narrower tile that shares everything else with the BN-wide one. The B tile is staged BN wide as
  // always (same ring, same transfers), but only the first BN_ACT columns are multiplied and written out: the
  // tiles of a last, deliberately lighter round of a launch (see tf_gemm_mixed_kernel).
  static constexpr int BN_ACT = BN_ACT_;
  static_assert(BN_ACT_ <= BN_ && BN_ACT_ % (32 * WN_) == 0, "active width: whole 32-column blocks per wave column");
  // TRANSA: A is given transposed, [K][lda] with m contiguous (the dO^T A product of the paper's
  // Case Study 3). Its tile is then staged exactly like the B tile, [64][BM] row-major with the
  // same 64-byte piece swizzle, and its MFMA operands come from the transposing LDS read too:
  // the loads from memory stay fully coalesced and nothing is transposed by ALU code or by a
  // separate pass.
  static constexpr bool TRANSA = TRANSA_;
  static constexpr int A_ROW_BYTES = BM_ * 2, A_PIECES = A_ROW_BYTES / 64, A_ROWS_PER_INSTR = 1024 / A_ROW_BYTES;
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, STAGES = STAGES_;
  static_assert(BK == 32 || BK == 64 || BK == 128, "K tile of 32, 64 or 128");
  // TRANSB: B is given as [N][ldb] with k contiguous (weights stored output-major). Its tile is then staged
  // exactly like the A tile, [BN][BK] with the same chunk swizzle, and its MFMA operands are ds_read_b128.
  static constexpr bool TRANSB = TRANSB_;
  // A tile rows (and B tile rows under TRANSB): BK / 8 chunks of 16 bytes; slot = chunk ^ row_swz(row)
  static constexpr int K_ROW_BYTES = BK * 2, K_CHUNKS = BK / 8, K_ROWS_PER_LINE = 16 / K_CHUNKS, K_ROWS_PER_INSTR = 64 / K_CHUNKS;
  static constexpr int KSTEPS = BK / 16;                   // 16-wide MFMA steps per K tile
  // WK: wave groups along k. With WK = 2 a second set of WM x WN waves works on the same
  // BM x BN tile but takes the other half of every 64-wide K step; the two sets add their
  // accumulators through LDS after the main loop. Eight waves then keep the LDS busier than
  // four can (a wave issues one LDS instruction every twenty-odd cycles) without the extra
  // fragment reads that a finer split of the tile along m or n costs.
  static constexpr int WK = WK_, KS = KSTEPS / WK_;        // k16-steps per wave per K step
  static_assert(KS >= 2 && KS % 2 == 0, "the pipeline alternates two fragment sets per k16-step");
  static constexpr bool DIRECT = DIRECT_;
  // ABYPASS: the A operand never enters LDS. Each wave loads its own A fragments from memory
  // straight into registers (WN must be 1, so no two waves need the same A rows) and only B is
  // staged. This halves the LDS write traffic, which is what bounds the two-operand scheme.
  static constexpr bool ABYPASS = ABYPASS_;
  static constexpr int NWAVES = WM * WN * WK, THREADS = NWAVES * 64;
  static constexpr int WTM = BM / WM, WTN = BN_ACT / WN;   // wave tile
  static constexpr int TM = WTM / 32, TN = WTN / 32;       // 32x32 MFMA blocks per wave
  static constexpr int A_BYTES = ABYPASS ? 0 : BM * BK * 2, B_BYTES = BK * BN * 2;
  static_assert(!ABYPASS || (WN == 1 && DIRECT && STAGES == 2 && WK_ == 1 && BK == 64 && !TRANSB_), "A bypass: one wave column, direct B staging, two buffers, K tile of 64");
  static_assert(DIRECT || BK == 64, "register staging: K tile of 64");
  static_assert(!TRANSB_ || !TRANSA_, "one transposed operand at a time");
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int RING_BYTES = STAGES * STAGE_BYTES;
  // behind the ring: this tile's BN bias values, fetched at kernel start so that the epilogue
  // does not begin with a trip to memory
  static constexpr int BIAS_OFF = RING_BYTES, BIAS_BYTES = 512;
  static constexpr int LDS_BYTES = RING_BYTES + BIAS_BYTES;
  static constexpr int A_INSTR = A_BYTES / 1024;           // wave-wide 1 KB transfers per tile
  static constexpr int B_INSTR = B_BYTES / 1024;
  static constexpr int A_PER_WAVE = A_INSTR / NWAVES, B_PER_WAVE = B_INSTR / NWAVES;
  static constexpr int B_ROW_BYTES = TRANSB ? K_ROW_BYTES : BN * 2;
  static constexpr int B_ROWS_PER_INSTR = 1024 / B_ROW_BYTES;
  static constexpr int B_SLOTS_PER_ROW = B_ROW_BYTES / 16;  // 16-byte slots per B row
  static constexpr int B_PIECES = B_ROW_BYTES / 64;         // 64-byte pieces per B row
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 blocks");
  static_assert(A_INSTR % NWAVES == 0 && B_INSTR % NWAVES == 0, "tile loads must divide over the waves");
  static_assert(BN == 32 || BN == 64 || BN == 128 || BN == 256, "B row must be 64, 128, 256 or 512 bytes");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
  static_assert(WK == 1 || (WK == 2 && TM % 2 == 0 && DIRECT && !ABYPASS), "k groups: two, each keeps half of the row blocks");
  static_assert(!TRANSA || (DIRECT && !ABYPASS && (BM == 32 || BM == 64 || BM == 128 || BM == 256)), "transposed A: direct staging, A row of 64 to 512 bytes");
  static_assert(WK == 1 || RING_BYTES >= NWAVES * (TM / 2) * TN * 4096, "the accumulator exchange reuses the tile buffers");
  static constexpr int TM_OUT = TM / WK;                   // row blocks a wave writes out
  // The in-kernel split-K reduction is only compiled for wave tiles of at most 64 accumulator
  // registers: behind bigger ones its code makes the compiler spill, and the scratch memory
  // that reserves per wave slows every launch of the kernel, split or not.
  static constexpr bool FUSED_OK = TM * TN <= 4;
  static constexpr bool SEGMENTS = false;                  // see StreamKCfg
  // Output staging (see epilogue_staged): each pass moves 32 rows per wave row (and k group) through the tile
  // ring, rows padded by 16 bytes; used for an output type when one pass fits into the ring.
  static constexpr int ST_ROWS = 32 * WM * WK_;
  // (not behind wave tiles of 256 accumulator registers: the extra code makes the compiler spill there)
  // the persistent kernel's fp32 staging area lies behind the ring
  static constexpr int PERSIST_LDS_BYTES = RING_BYTES + ST_ROWS * (BN * 4 + 16);
  static constexpr bool stage_ok(int esz) { return TM * TN <= 8 && ST_ROWS * (BN_ACT * esz + 16) <= RING_BYTES; }
  // 32-row tiles serve problems of few rows, where every B element is read by one work-group only: its
  // loads are marked non-temporal
  static constexpr bool B_NT = BM <= 32;
  // slot permutation of the 16-byte chunks of a k-contiguous tile row (see the file header)
  __device__ __forceinline__ static constexpr int row_swz(int r) { return (r / K_ROWS_PER_LINE) & (K_CHUNKS - 1); }
};

// Slot permutation of the 64-byte pieces of B row k (see header).
template <int PIECES>
__device__ __forceinline__ int b_swz(int k) {
  if (PIECES >= 4) return k & 3;
  if (PIECES == 2) return (k >> 1) & 1;
  return 0;
}

template <class C>
struct TileLoader {
  // Per-lane, per-transfer source offsets (in elements, relative to the tile's first k) and
  // validity. Computed once; the K step only moves the base pointers.
  // (byte offsets from the tile's first k; 32 bits: the host rejects tensors of 4 GiB or more)
  static constexpr int NA = C::A_PER_WAVE > 0 ? C::A_PER_WAVE : 1;   // (no zero-length arrays)
  unsigned a_src[NA];
  unsigned b_src[C::B_PER_WAVE];
  int a_k[NA];                   // k offset (elements) of the lane's chunk inside the tile
  int b_k[C::B_PER_WAVE];        // k row of the lane inside the tile
  bool b_ok[C::B_PER_WAVE];      // column chunk inside N
  bool a_ok[NA];                 // row inside M

  __device__ __forceinline__ void init(const GemmParams& p, int m0, int n0, int wave, int lane) {
#pragma unroll
    for (int q = 0; q < C::A_PER_WAVE; ++q) {
      const int ia = wave + C::NWAVES * q;
      if constexpr (C::TRANSA) {
        // rows of the tile are k, columns m: the scheme of the B tile with m in place of n
        constexpr int LPR = 64 / C::A_ROWS_PER_INSTR;
        const int krow = C::A_ROWS_PER_INSTR * ia + lane / LPR;
        const int s16 = lane % LPR;
        const int piece = (s16 >> 2) ^ b_swz<C::A_PIECES>(krow);
        int m = m0 + 32 * piece + 8 * (s16 & 3);
        a_ok[q] = m < p.M;
        if (m >= p.M) m = 0;
        a_src[q] = ((unsigned)krow * (unsigned)p.lda + (unsigned)m) * 2u;
        a_k[q] = krow;
      } else {
        const int row = C::K_ROWS_PER_INSTR * ia + lane / C::K_CHUNKS;
        const int slot = lane % C::K_CHUNKS;
        const int c = slot ^ C::row_swz(row);
        int m = m0 + row;
        a_ok[q] = m < p.M;
        if (m >= p.M) m = p.M - 1;
        a_src[q] = ((unsigned)m * (unsigned)p.lda + 8u * c) * 2u;
        a_k[q] = 8 * c;
      }
    }
#pragma unroll
    for (int q = 0; q < C::B_PER_WAVE; ++q) {
      const int ib = wave + C::NWAVES * q;
      if constexpr (C::TRANSB) {
        // rows of the tile are n, columns k: the scheme of the A tile with n in place of m
        const int row = C::K_ROWS_PER_INSTR * ib + lane / C::K_CHUNKS;
        const int slot = lane % C::K_CHUNKS;
        const int c = slot ^ C::row_swz(row);
        int n = n0 + row;
        b_ok[q] = n < p.N;
        if (n >= p.N) n = p.N - 1;
        b_src[q] = ((unsigned)n * (unsigned)p.ldb + 8u * c) * 2u;
        b_k[q] = 8 * c;
      } else {
        constexpr int LPR = 64 / C::B_ROWS_PER_INSTR;          // lanes per row
        const int krow = C::B_ROWS_PER_INSTR * ib + lane / LPR;
        const int s16 = lane % LPR;
        const int piece = (s16 >> 2) ^ b_swz<C::B_PIECES>(krow);
        int n = n0 + 32 * piece + 8 * (s16 & 3);
        b_ok[q] = n < p.N;
        if (n >= p.N) n = 0;
        b_src[q] = ((unsigned)krow * (unsigned)p.ldb + (unsigned)n) * 2u;
        b_k[q] = krow;
      }
    }
  }

  // memory -> LDS without registers. Requires every k of the tile to be < K.
  // Written as inline assembly: M0 carries the wave-uniform LDS destination, each lane lands
  // at M0 + 16 * lane, the source is an SGPR base plus this lane's 32-bit byte offset. The
  // transfers are counted by vmcnt; the kernel waits for them explicitly before the barrier
  // that publishes a tile, so the compiler needs no knowledge of them (given the builtin, it
  // would make every later LDS read wait for all transfers in flight, including the tiles
  // prefetched for later steps). Nothing else in these kernels uses M0.
  template <bool NT = false>
  __device__ __forceinline__ static void gload_lds16(unsigned lds_addr, unsigned voff, const void* base) {
    // the base is the same for every lane; say so, or it may be handed over in vector registers
    const unsigned long long b = (unsigned long long)base;
    // (the builtin returns a signed int: go through unsigned, or the low half sign-extends)
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(b >> 32));
    const unsigned long long sb = (unsigned long long)lo | ((unsigned long long)hi << 32);
    const void* sbase = (const void*)sb;
    if constexpr (NT)      // non-temporal: data that no other work-group reads again need not stay in the caches
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                   :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
    else
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
  }
  // same, four bytes per lane (lane l lands at M0 + 4 l; lanes switched off transfer nothing)
  __device__ __forceinline__ static void gload_lds4(unsigned lds_addr, unsigned voff, const void* base) {
    const unsigned long long b = (unsigned long long)base;
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(b >> 32));
    const unsigned long long sb = (unsigned long long)lo | ((unsigned long long)hi << 32);
    const void* sbase = (const void*)sb;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
  }
  __device__ __forceinline__ void issue_direct(const uint16_t* Ak, const uint16_t* Bk, unsigned stage_lds, int wave) const {
#pragma unroll
    for (int q = 0; q < C::A_PER_WAVE; ++q) {
      const int ia = wave + C::NWAVES * q;
      gload_lds16(__builtin_amdgcn_readfirstlane(stage_lds + ia * 1024), a_src[q], Ak);
    }
#pragma unroll
    for (int q = 0; q < C::B_PER_WAVE; ++q) {
      const int ib = wave + C::NWAVES * q;
      gload_lds16<C::B_NT>(__builtin_amdgcn_readfirstlane(stage_lds + C::A_BYTES + ib * 1024), b_src[q], Bk);
    }
  }

  __device__ __forceinline__ void issue_a_one(int q, const uint16_t* Ak, unsigned stage_lds, int wave) const {
    const int ia = wave + C::NWAVES * q;
    gload_lds16(__builtin_amdgcn_readfirstlane(stage_lds + ia * 1024), a_src[q < NA ? q : 0], Ak);
  }
  __device__ __forceinline__ void issue_b_one(int q, const uint16_t* Bk, unsigned stage_lds, int wave) const {
    const int ib = wave + C::NWAVES * q;
    gload_lds16<C::B_NT>(__builtin_amdgcn_readfirstlane(stage_lds + C::A_BYTES + ib * 1024), b_src[q], Bk);
  }
  __device__ __forceinline__ void issue_a_all(const uint16_t* Ak, unsigned stage_lds, int wave) const {
#pragma unroll
    for (int q = 0; q < C::A_PER_WAVE; ++q) issue_a_one(q, Ak, stage_lds, wave);
  }
  __device__ __forceinline__ void issue_b_direct(const uint16_t* Bk, unsigned stage_lds, int wave) const {
#pragma unroll
    for (int q = 0; q < C::B_PER_WAVE; ++q) {
      const int ib = wave + C::NWAVES * q;
      gload_lds16<C::B_NT>(__builtin_amdgcn_readfirstlane(stage_lds + C::A_BYTES + ib * 1024), b_src[q], Bk);
    }
  }

  // memory -> registers, zero where k >= K (ragged tail) or outside M / N.
  __device__ __forceinline__ void load_regs(const uint16_t* Ak, const uint16_t* Bk, int k0, int K,
                                            u32x4 (&ra)[NA], u32x4 (&rb)[C::B_PER_WAVE]) const {
#pragma unroll
    for (int q = 0; q < C::A_PER_WAVE; ++q) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (a_ok[q] && k0 + a_k[q] < K) v = *(const u32x4*)((const char*)Ak + a_src[q]);
      ra[q] = v;
    }
#pragma unroll
    for (int q = 0; q < C::B_PER_WAVE; ++q) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (b_ok[q] && k0 + b_k[q] < K) v = *(const u32x4*)((const char*)Bk + b_src[q]);
      rb[q] = v;
    }
  }
  __device__ __forceinline__ void store_regs(char* stage, int wave, int lane,
                                             const u32x4 (&ra)[NA], const u32x4 (&rb)[C::B_PER_WAVE]) const {
#pragma unroll
    for (int q = 0; q < C::A_PER_WAVE; ++q) {
      const int ia = wave + C::NWAVES * q;
      *(u32x4*)(stage + ia * 1024 + lane * 16) = ra[q];
    }
#pragma unroll
    for (int q = 0; q < C::B_PER_WAVE; ++q) {
      const int ib = wave + C::NWAVES * q;
      *(u32x4*)(stage + C::A_BYTES + ib * 1024 + lane * 16) = rb[q];
    }
  }
};

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding:
// vmcnt = bits [3:0] and [15:14], expcnt [6:4] and lgkmcnt [11:8] left at "no wait").
// Work-group barrier for the direct-to-LDS pipeline: this wave's LDS reads have returned
// (lgkmcnt 0), then s_barrier. Unlike __syncthreads() it does not wait for vector-memory
// operations, so tiles prefetched for later steps stay in flight across it; the caller waits
// for the tile it is about to publish with wait_vmcnt<> first. The asm memory clobber keeps
// the compiler from moving LDS accesses across it.
__device__ __forceinline__ void barrier_lds() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Four fp32 stored with device ("agent") scope: written through the L2 of this XCD, so a
// work-group on another XCD (another L2) reads the new value from memory. Split-K uses it for
// the partial sums instead of a device-wide fence, which would write back and invalidate the
// whole L2 twice per work-group.
// (One 16-byte store with the device-scope bit, as the compiler emits for a relaxed device-scope atomic store
// of one dword; the atomic builtins themselves stop at 8 bytes. ptr is 16-byte aligned.)
__device__ __forceinline__ void store_through_f32x4(float* ptr, const f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" :: "v"(ptr), "v"(v) : "memory");
}
// The matching load: 16 bytes past this XCD's L2. Only issues it; the data is there after wait_through().
__device__ __forceinline__ void load_through_f32x4(f32x4& dst, const float* ptr) {
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=&v"(dst) : "v"(ptr) : "memory");
}
// Waits for every load above; the values pass through it, so that no use of them can be moved ahead of the wait.
__device__ __forceinline__ void wait_through(f32x4& a, f32x4& b, f32x4& c, f32x4& d) {
  asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) :: "memory");
}

// Split-K: one slice's partial tile -> workspace (fp32, [slice][M][N]).
template <class C, bool FULL, bool THROUGH>
__device__ __forceinline__ void store_partial(const f32x16 (&acc)[C::TM][C::TN], float* wsk, const GemmParams& p,
                                              int wm0, int wn0) {
#pragma unroll
  for (int i = 0; i < C::TM_OUT; ++i) {
    const int m = wm0 + 32 * i;
#pragma unroll
    for (int t = 0; t < C::TN; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = wn0 + 32 * t + 8 * q;
        if (FULL || (m < p.M && n < p.N)) {
          const f32x4 v = {acc[i][t][4 * q], acc[i][t][4 * q + 1], acc[i][t][4 * q + 2], acc[i][t][4 * q + 3]};
          if (THROUGH) store_through_f32x4(wsk + (size_t)m * p.N + n, v);
          else *(f32x4*)(wsk + (size_t)m * p.N + n) = v;
        }
      }
  }
}

// Split-K: sum of all slices, always in slice order 0, 1, ... so the result does not depend on
// which slice arrived last.
// THROUGH: device-scope loads (the slices may have been written through other XCDs' L2s);
// otherwise plain 16-byte loads, for slices known to sit in this XCD's L2.
template <class C, bool FULL, bool THROUGH>
__device__ __forceinline__ void sum_partials(f32x16 (&acc)[C::TM][C::TN], const GemmParams& p, int wm0, int wn0) {
  const size_t slice = (size_t)p.M * p.N;
  // 16-byte loads (device scope, or plain ones for slices that sit in this XCD's L2), whole slices in flight at a
  // time: a loop over the slices per element is one long chain of dependent trips to memory, and everything behind
  // the K loop of a memory-bound problem is time in which nothing is streamed. The accumulator registers are free
  // by now: their contents have been published. Pieces outside M or N (ragged tiles) count as zero.
  constexpr int NV = C::TM_OUT * C::TN * 4;
  static_assert(NV % 4 == 0 && NV <= 16, "register budget of the exchange");
  f32x4 sum[NV];
  bool ok[NV];
#pragma unroll
  for (int x = 0; x < NV; ++x) {
    const int i = x / (C::TN * 4), t = (x / 4) % C::TN, q = x % 4;
    sum[x] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    ok[x] = FULL || (wm0 + 32 * i < p.M && wn0 + 32 * t + 8 * q < p.N);
  }
  // G slices are loaded together (as many as sixteen 16-byte vectors per lane allow: small tiles with two or four
  // slices make one trip to memory in all), then added in slice order
  constexpr int G = NV <= 4 ? 4 : (NV <= 8 ? 2 : 1);
  for (int s0 = 0; s0 < p.split_k; s0 += G) {
    f32x4 v[G][NV];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      // (a slice past the last one reads the last one again and is not added)
      const int sidx = s0 + g < p.split_k ? s0 + g : p.split_k - 1;
      const float* base = p.ws + (size_t)sidx * slice;
#pragma unroll
      for (int x = 0; x < NV; ++x) {
        const int i = x / (C::TN * 4), t = (x / 4) % C::TN, q = x % 4;
        // (a piece outside the matrix reads the slice's first 16 bytes instead: no branch round the load, whose
        // result only counts after the wait below)
        const float* src = ok[x] ? base + (size_t)(wm0 + 32 * i) * p.N + (wn0 + 32 * t + 8 * q) : base;
        if constexpr (THROUGH) load_through_f32x4(v[g][x], src);
        else v[g][x] = *(const f32x4*)src;
      }
    }
    if constexpr (THROUGH) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int x = 0; x < NV; x += 4) wait_through(v[g][x], v[g][x + 1], v[g][x + 2], v[g][x + 3]);
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int x = 0; x < NV; ++x)
        if (ok[x] && s0 + g < p.split_k) sum[x] += v[g][x];
  }
#pragma unroll
  for (int x = 0; x < NV; ++x) {
    const int i = x / (C::TN * 4), t = (x / 4) % C::TN, q = x % 4;
    acc[i][t][4 * q] = sum[x][0]; acc[i][t][4 * q + 1] = sum[x][1];
    acc[i][t][4 * q + 2] = sum[x][2]; acc[i][t][4 * q + 3] = sum[x][3];
  }
}

template <int E> struct EpiTag { static constexpr int value = E; };

// bias_lds: this lane's first four bias values in LDS (columns wn0 .. wn0 + 3 of the tile's copy)
template <class C, bool FULL, int EPI>
__device__ __forceinline__ void epilogue(const f32x16 (&acc)[C::TM][C::TN], const GemmParams& p, int wm0, int wn0,
                                         const char* bias_lds, int n_end) {
#pragma unroll
  for (int t = 0; t < C::TN; ++t) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int n = wn0 + 32 * t + 8 * q;
      const bool n_ok = FULL || n < n_end;
      const u32x2 braw = *(const u32x2*)(bias_lds + (32 * t + 8 * q) * 2);   // (columns past N hold values nobody stores)
      const float b0 = __builtin_bit_cast(float, braw[0] << 16), b1 = __builtin_bit_cast(float, braw[0] & 0xffff0000u);
      const float b2 = __builtin_bit_cast(float, braw[1] << 16), b3 = __builtin_bit_cast(float, braw[1] & 0xffff0000u);
#pragma unroll
      for (int i = 0; i < C::TM_OUT; ++i) {
        const int m = wm0 + 32 * i;
        if (FULL || (n_ok && m < p.M)) {
          const float z0 = acc[i][t][4 * q] + b0, z1 = acc[i][t][4 * q + 1] + b1;
          const float z2 = acc[i][t][4 * q + 2] + b2, z3 = acc[i][t][4 * q + 3] + b3;
          if (EPI == TF_EPI_NONE_F32) {
            const f32x4 v = {z0, z1, z2, z3};
            *(f32x4*)((float*)p.Y + (size_t)m * p.ldy + n) = v;
          } else {
            u32x2 o;
            o[0] = pack_bf16x2(activate<EPI>(z0), activate<EPI>(z1));
            o[1] = pack_bf16x2(activate<EPI>(z2), activate<EPI>(z3));
            *(u32x2*)((uint16_t*)p.Y + (size_t)m * p.ldy + n) = o;
          }
        }
      }
    }
  }
}

// The same epilogue for whole tiles with 16-byte aligned output rows, with the stores coalesced through LDS.
// Written straight from the accumulators, a store instruction touches 32 rows with 16 or 32 bytes each, and
// the memory side handles every such piece as a request of its own: that, not the byte count, bounds the
// write-back. Here the work-group lays 32 rows per wave row out in LDS (the tile ring is free by now),
// and reads them back so that consecutive lanes hold consecutive 16-byte pieces of a row: a store
// instruction then writes whole rows of the tile, 64 x 16 bytes contiguous per BN * esz bytes.
// The lines go out complete, so the stores are marked non-temporal: nothing is left in the L2 for the
// write-back at the end of the kernel. PARTIAL: the raw accumulators (no bias) go to `dst`, a split-K slice of
// the workspace with rows of `ld` floats, instead of Y.
// Every wave of the work-group must call it (barriers inside).
template <class C, int EPI, bool PARTIAL = false>
__device__ __forceinline__ void epilogue_staged(const f32x16 (&acc)[C::TM][C::TN], const GemmParams& p, char* smem, int m0,
                                                int n0, int tid, int wave_m, int wave_n, int wave_k, int lane_m, int lane_g,
                                                char* dst, size_t ld, int ncols = C::BN_ACT) {
  // ncols: columns of the tile that exist / belong to it (a multiple of 8); pieces past them are not stored
  static_assert(!PARTIAL || EPI == TF_EPI_NONE_F32, "partial sums are fp32");
  constexpr int ESZ = EPI == TF_EPI_NONE_F32 ? 4 : 2;
  constexpr int ROWB = C::BN_ACT * ESZ + 16;             // staged row, padded: the 32 rows a store hits spread over the banks
  constexpr int CPR = C::BN_ACT * ESZ / 16;              // 16-byte pieces per row
  constexpr int PER_THREAD = C::ST_ROWS * CPR / C::THREADS;
  static_assert(C::ST_ROWS * CPR % C::THREADS == 0, "pieces divide over the threads");
  const char* bias_lds = smem + C::BIAS_OFF + (wave_n * C::WTN + 4 * lane_g) * 2;
  char* wr = smem + ((wave_m * C::WK + wave_k) * 32 + lane_m) * ROWB + (wave_n * C::WTN + 4 * lane_g) * ESZ;
  wait_vmcnt<0>();          // no transfer into the ring is in flight any more (the clamped tail prefetches)
  barrier_lds();            // and nobody reads tile fragments any more
#pragma unroll
  for (int i = 0; i < C::TM_OUT; ++i) {
    if (i) barrier_lds();   // the previous pass has been read back
#pragma unroll
    for (int t = 0; t < C::TN; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float z0 = acc[i][t][4 * q], z1 = acc[i][t][4 * q + 1], z2 = acc[i][t][4 * q + 2], z3 = acc[i][t][4 * q + 3];
        if (!PARTIAL) {
          const u32x2 braw = *(const u32x2*)(bias_lds + (32 * t + 8 * q) * 2);
          z0 += __builtin_bit_cast(float, braw[0] << 16);
          z1 += __builtin_bit_cast(float, braw[0] & 0xffff0000u);
          z2 += __builtin_bit_cast(float, braw[1] << 16);
          z3 += __builtin_bit_cast(float, braw[1] & 0xffff0000u);
        }
        if (EPI == TF_EPI_NONE_F32) {
          const f32x4 v = {z0, z1, z2, z3};
          *(f32x4*)(wr + (32 * t + 8 * q) * 4) = v;
        } else {
          u32x2 o;
          o[0] = pack_bf16x2(activate<EPI>(z0), activate<EPI>(z1));
          o[1] = pack_bf16x2(activate<EPI>(z2), activate<EPI>(z3));
          *(u32x2*)(wr + (32 * t + 8 * q) * 2) = o;
        }
      }
    barrier_lds();
#pragma unroll
    for (int j = 0; j < PER_THREAD; ++j) {
      const int c = tid + C::THREADS * j;
      const int rs = c / CPR, cc = c % CPR;
      const int g = rs >> 5;                               // wave row and k group the staged row came from
      const int m = m0 + (g / C::WK) * C::WTM + (g % C::WK) * 32 * (C::TM / 2) + 32 * i + (rs & 31);
      const u32x4 v = *(const u32x4*)(smem + rs * ROWB + cc * 16);
      if (cc * 16 < ncols * ESZ) {
        // the output is not read again by this launch: non-temporal; a partial tile is read back at once by the
        // reduction: ordinary stores, so that it may stay in the caches on the way
        if constexpr (PARTIAL) *(u32x4*)(dst + ((size_t)m * ld + n0) * ESZ + cc * 16) = v;
        else __builtin_nontemporal_store(v, (u32x4*)(dst + ((size_t)m * ld + n0) * ESZ + cc * 16));
      }
    }
  }
}

template <class C>
__device__ __forceinline__ void gemm_tile_body(const GemmParams& p_in) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // batched problems: blockIdx.y is the batch item, whose operands are a stride away
  GemmParams p = p_in;
  int tile_id = blockIdx.x;
  if (gridDim.y > 1) {
    int item = blockIdx.y;
    if (p.batch_xcd) {
      // Work-groups go to the eight XCDs in turn, in launch order (x fastest). Renumber them so that all tiles
      // of a batch item run on one XCD, whose L2 then fetches the item's operands once, not once per XCD:
      // XCD x takes items x, x + 8, ... (the host sets the flag only for a batch that is a multiple of 8).
      const unsigned launch_id = blockIdx.y * gridDim.x + blockIdx.x;
      const unsigned local = launch_id >> 3;
      item = (int)((launch_id & 7u) + 8u * (local / gridDim.x));
      tile_id = (int)(local % gridDim.x);
    }
    p.A += (size_t)item * p.stride_a;
    p.B += (size_t)item * p.stride_b;
    p.Y = (char*)p.Y + (size_t)item * p.stride_y * (p.epi == TF_EPI_NONE_F32 ? 4 : 2);
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_k = wave / (C::WM * C::WN), wave_mn = wave % (C::WM * C::WN);
  const int wave_m = wave_mn / C::WN, wave_n = wave_mn % C::WN;

  // A work-group computes one segment = one tile over one range of K tiles - except the stream-K work-groups,
  // which take an equal share of the K steps of the last tiles each, a share that may span up to three tiles
  // (the end of one, a whole one, the beginning of the next). The host arranges that a tile has at most two
  // contributors: they exchange partial tiles like two split-K slices (slice 0 = the part that begins the
  // tile), and since a sum of two terms does not depend on their order the result is the same whoever
  // arrives last.
  const int ktiles_total = (p.K + C::BK - 1) / C::BK;
  // (Compiled only into the stream-K instances, StreamKCfg<>; in every other kernel the loop below is one pass
  // and costs nothing: wrapped around the ordinary kernels it cost them 1-2 % through register pressure.)
  constexpr bool SEGMENTS = C::SEGMENTS;
  static_assert(!SEGMENTS || C::FUSED_OK, "stream-K needs the in-kernel reduction");
  int sk_cur = 0, sk_end = 0;
  const bool stream_k = SEGMENTS && p.stream_k;
  const bool stream_wg = stream_k && tile_id >= p.sk_first_wg;
  if (stream_wg) {
    // (the shares of the work-groups of one XCD lie side by side: they work on neighbouring tiles)
    const long g = xcd_run(tile_id - p.sk_first_wg, p.sk_wgs), total_steps = (long)p.sk_tiles * ktiles_total;
    sk_cur = (int)(g * total_steps / p.sk_wgs);
    sk_end = (int)((g + 1) * total_steps / p.sk_wgs);
  }
  bool more = true;
  for (int seg = 0; more; ++seg) {
  if (seg) {                       // the ring, the bias copy and the staging area are about to be reused
    wait_vmcnt<0>();
    __syncthreads();
  }
  TileCoord tc;
  int kt_begin, kt_end;
  bool split = p.split_k > 1;      // this segment is one of several contributions to its tile
  int n0_mixed = -1, n_end = p.N;  // (mixed grid) origin of a tile of the narrow round; first column that is not the tile's
  if (p.mix_main_wgs > 0) {
    // A launch of whole rounds of BN-wide tiles over the first columns, then one round of narrower tiles that
    // share out the remaining columns of every row panel evenly (see tf_gemm_mixed_kernel). No K slices.
    if constexpr (C::BN_ACT == C::BN) {
      tc = tile_at(p, xcd_run(tile_id, p.mix_main_wgs));          // p.tiles_n = tile columns of the wide part
    } else {
      const int t = xcd_run(tile_id - p.mix_main_wgs, p.tiles_m * p.mix_tiles);
      tc.tm = t / p.mix_tiles; tc.tn = 0; tc.ks = 0;
      const int j = t - tc.tm * p.mix_tiles;
      // tile j of the row panel starts at block floor(j R / T) of the remaining R blocks of 32 columns and owns the
      // blocks up to the start of tile j + 1 (at most BN_ACT / 32 of them; the host checked)
      const int b0 = (int)((long)j * p.mix_blocks / p.mix_tiles), b1 = (int)((long)(j + 1) * p.mix_blocks / p.mix_tiles);
      n0_mixed = p.mix_n_origin + 32 * b0;
      const int lim = p.mix_n_origin + 32 * b1;
      n_end = lim < p.N ? lim : p.N;
    }
    kt_begin = 0; kt_end = ktiles_total; split = false; more = false;
  } else if (!stream_k) {
    tc = map_tile(p, tile_id);
    kt_begin = tc.ks * p.ktiles_per_split;
    kt_end = kt_begin + p.ktiles_per_split;
    if (kt_end > ktiles_total) kt_end = ktiles_total;
    more = false;
  } else if (!stream_wg) {
    tc = tile_at(p, p.xcd_swizzle ? xcd_run(tile_id, p.sk_first_wg) : tile_id);
    kt_begin = 0; kt_end = ktiles_total; split = false; more = false;
  } else {
    if (sk_cur >= sk_end) break;   // (an empty share: more work-groups than steps)
    const int t = sk_cur / ktiles_total;
    kt_begin = sk_cur - t * ktiles_total;
    kt_end = kt_begin + (sk_end - sk_cur);
    if (kt_end > ktiles_total) kt_end = ktiles_total;
    tc = tile_at(p, p.sk_first_wg + t);
    split = !(kt_begin == 0 && kt_end == ktiles_total);
    tc.ks = kt_begin == 0 ? 0 : 1;
    sk_cur += kt_end - kt_begin;
    more = sk_cur < sk_end;
  }
  const int m0 = tc.tm * C::BM, n0 = n0_mixed >= 0 ? n0_mixed : tc.tn * C::BN;
  // K tiles dealt to the slices in turn (slice s takes the tiles s, s + S, s + 2 S, ...) instead of a contiguous range
  // each: at any moment all work-groups then read inside one narrow band of rows of B, which a streaming read of
  // column strips rewards (134 MB: 21.2 us against 23.2 us with two halves of K; host: direct staging only)
  const bool k_deal = C::DIRECT && p.k_interleave && split && !stream_k;
  const int nkt = k_deal ? (ktiles_total - tc.ks + p.split_k - 1) / p.split_k
                         : kt_end - kt_begin;   // may be <= 0 for a trailing empty slice: contributes zeros

  // ---- LDS read offsets of this lane (bytes inside a stage)
  int a_off[C::KS];
  {
    const int r = wave_m * C::WTM + (lane & 31);
    const int g = lane >> 5;
    const int sw = C::row_swz(r);          // (the same for the rows 32, 64, ... further down)
#pragma unroll
    for (int kk = 0; kk < C::KS; ++kk) a_off[kk] = r * C::K_ROW_BYTES + (((2 * (wave_k * C::KS + kk) + g) ^ sw) << 4);
  }
  // B given as [N][K]: its tile is read like the A tile. Its offsets are derived per read from two values (the
  // chunk index 2 k + g only differs from g above bit 0, so the swizzled slot of step k is (g ^ sw) ^ 2 k):
  // a table per k16-step as for A costs registers the big tiles do not have.
  int bt_row = 0, bt_c0 = 0;
  if constexpr (C::TRANSB) {
    const int r = wave_n * C::WTN + (lane & 31);
    bt_row = C::A_BYTES + r * C::K_ROW_BYTES;
    bt_c0 = ((lane >> 5) ^ C::row_swz(r)) << 4;
  }
  int a_toff[C::TRANSA ? C::TM : 1];     // transposed A: offsets for the transposing read, as for B
  if constexpr (C::TRANSA) {
    const int b = lane >> 4, s = lane & 15;
    const int krow = 8 * (b >> 1) + (s >> 2);
    const int within = (16 * (b & 1) + 4 * (s & 3)) * 2;
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
      const int j = (wave_m * C::WTM) / 32 + i;
      const int piece = j ^ b_swz<C::A_PIECES>(krow);
      a_toff[i] = (krow + wave_k * C::KS * 16) * C::A_ROW_BYTES + piece * 64 + within;
    }
  }
  // one A operand of k16-step kk (relative to the wave's first step), row block i
  auto read_a = [&](const char* stage, int kk, int i) -> bf16x8 {
    if constexpr (C::TRANSA) {
      const char* ap = stage + a_toff[i] + (16 * kk) * C::A_ROW_BYTES;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(ap));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(ap + 4 * C::A_ROW_BYTES));
      const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, v);
    } else {
      return *(const bf16x8*)(stage + a_off[kk] + i * 32 * C::K_ROW_BYTES);
    }
  };
  int b_off[C::TN];
  {
    const int b = lane >> 4, s = lane & 15;
    const int krow = 8 * (b >> 1) + (s >> 2);                 // + 16 kk + 4 h
    const int within = (16 * (b & 1) + 4 * (s & 3)) * 2;      // bytes inside the 64-byte piece
#pragma unroll
    for (int t = 0; t < C::TN; ++t) {
      const int j = (wave_n * C::WTN) / 32 + t;
      const int piece = j ^ b_swz<C::B_PIECES>(krow);
      b_off[t] = C::A_BYTES + (krow + wave_k * C::KS * 16) * C::B_ROW_BYTES + piece * 64 + within;
    }
  }
  // one B operand of k16-step kk (relative to the wave's first step), column block t
  auto read_b1 = [&](const char* stage, int kk, int t) -> bf16x8 {
    if constexpr (C::TRANSB) {
      return *(const bf16x8*)(stage + bt_row + (bt_c0 ^ ((wave_k * C::KS + kk) << 5)) + t * 32 * C::K_ROW_BYTES);
    } else {
      const char* bp = stage + b_off[t] + (16 * kk) * C::B_ROW_BYTES;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(bp));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(bp + 4 * C::B_ROW_BYTES));
      const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, v);
    }
  };

  f32x16 acc[C::TM][C::TN];
#pragma unroll
  for (int i = 0; i < C::TM; ++i)
#pragma unroll
    for (int t = 0; t < C::TN; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][t][r] = 0.0f;

  TileLoader<C> ld;
  ld.init(p, m0, n0, wave, lane);
  // bias of this tile -> LDS (two values per lane), ahead of the first tile: it is in place when
  // the first hand-over barrier has been passed
  if (wave == 0) {
#pragma unroll
    for (int r = 0; r < (C::BN + 127) / 128; ++r) {
      const int c = 128 * r + 2 * lane;                 // column inside the tile
      if (c < C::BN) {
        const int n = n0 + c;
        if (p.bias == nullptr) {
          *(unsigned*)(smem + C::BIAS_OFF + c * 2) = 0u;      // no bias: the epilogue adds zeros
        } else if constexpr (C::DIRECT) {
          TileLoader<C>::gload_lds4(__builtin_amdgcn_readfirstlane((unsigned)(size_t)smem + C::BIAS_OFF + 256 * r),
                                    n < p.N ? (unsigned)n * 2u : 0u, p.bias);
        } else {
          unsigned v = 0u;
          if (n < p.N) v = *(const unsigned*)(p.bias + n);
          *(unsigned*)(smem + C::BIAS_OFF + c * 2) = v;
        }
      }
    }
  }
  const long a_tile = C::TRANSA ? (long)C::BK * p.lda : (long)C::BK;     // one K tile further in A
  const long b_tile = C::TRANSB ? (long)C::BK : (long)C::BK * p.ldb;      // one K tile further in B
  const int first_kt = k_deal ? tc.ks : kt_begin;
  const long a_step = k_deal ? a_tile * p.split_k : a_tile;              // this work-group's next K tile
  const long b_step = k_deal ? b_tile * p.split_k : b_tile;
  const uint16_t* Ak = p.A + (long)first_kt * a_tile;
  const uint16_t* Bk = p.B + (long)first_kt * b_tile;

  // ---- main loop, software pipelined by hand (one wave per SIMD has nobody to hide behind):
  //  * fragments are double buffered in registers: the LDS reads of k16-step kk+1 are issued
  //    before the MFMAs of step kk;
  //  * the loop is rotated: the barrier that hands over the next tile, the global loads of the
  //    tile after it and the first fragment reads of the next tile are all issued BEFORE the
  //    last 16-wide step of the current tile, whose MFMAs cover their latency.
  bf16x8 af[2][C::TM], bfr[2][C::TN];
  auto read_frags = [&](const char* stage, int kk, int set) {
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
      af[set][i] = read_a(stage, kk, i);
#pragma unroll
    for (int t = 0; t < C::TN; ++t) bfr[set][t] = read_b1(stage, kk, t);
  };
  auto mfma_step = [&](int set) {
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int t = 0; t < C::TN; ++t)
        acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][t], af[set][i], acc[i][t], 0, 0, 0);
  };
  // scheduling hint for one pipelined step: alternate one MFMA with one LDS read until the
  // reads are all issued, so that the matrix pipe never waits for the whole batch of reads
  constexpr int N_DS = C::TM + (C::TRANSB ? 1 : 2) * C::TN, N_MFMA = C::TM * C::TN;
  auto interleave_hint = [&]() {
#pragma unroll
    for (int x = 0; x < (N_DS < N_MFMA ? N_DS : N_MFMA); ++x) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one DS read
    }
  };

  // The last tile is peeled off the loop, so the loop body has no branch inside and is
  // scheduled as one block. Prefetches that would run past the last tile re-fetch the last
  // tile instead (into a buffer nobody reads any more): the number of transfers in flight is
  // then the same in every iteration and the vmcnt waits are constants.
  const int last = nkt - 1;
  // Order of the K tiles (a sum: any order is right). Without split-K the work-groups of XCD x start an
  // eighth of the way further into K than those of XCD x - 1 and wrap round: at any moment the eight XCDs
  // then fetch eight different slabs of A and B, and seven times out of eight a line has already been
  // brought into the memory-side cache by another XCD instead of all eight waiting for it together.
  // (All work-groups of an XCD keep the same order, so they still share panels in its L2.)
  const int k_rot = (p.k_rotate && nkt > 0) ? (int)(((blockIdx.x & 7u) * (unsigned)nkt) >> 3) : 0;
  auto k_order = [&](int t) { const int u = t + k_rot; return u >= nkt ? u - nkt : u; };
  if constexpr (C::ABYPASS) {
    // A straight from memory into MFMA operand registers: lane l of a wave needs, for row block
    // i and k16-step kk, the 16 bytes at row 32 i + (l & 31), k = 16 kk + 8 (l >> 5): one
    // global_load_dwordx4. Two register sets alternate per tile (the loop is unrolled by two so
    // both are addressed statically); the loads of tile kt+1 are issued at the top of tile kt.
    // These loads are ordinary loads the compiler tracks; the B transfers are not, so every
    // hand-over waits for vmcnt 0, which by then only covers loads issued a tile earlier.
    const unsigned lds0 = (unsigned)(size_t)smem;
    unsigned a_goff[C::TM];
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
      int m = m0 + wave_m * C::WTM + 32 * i + (lane & 31);
      if (m >= p.M) m = p.M - 1;
      a_goff[i] = ((unsigned)m * (unsigned)p.lda + 8u * (lane >> 5)) * 2u;
    }
    auto tile_a = [&](int t) { return Ak + (long)k_order(t < last ? t : last) * a_step; };
    auto tile_b = [&](int t) { return Bk + (long)k_order(t < last ? t : last) * b_step; };
    auto load_a = [&](u32x4 (&dst)[C::TM][4], const uint16_t* base) {
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) dst[i][kk] = *(const u32x4*)((const char*)base + a_goff[i] + kk * 32);
    };
    auto read_b = [&](const char* stage, int kk, int set) {
#pragma unroll
      for (int t = 0; t < C::TN; ++t) {
        const char* bp = stage + b_off[t] + (16 * kk) * C::B_ROW_BYTES;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(bp));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(bp + 4 * C::B_ROW_BYTES));
        const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        bfr[set][t] = __builtin_bit_cast(bf16x8, v);
      }
    };
    auto mfma_a = [&](const u32x4 (&as)[C::TM][4], int kk, int set) {
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int t = 0; t < C::TN; ++t)
          acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][t], __builtin_bit_cast(bf16x8, as[i][kk]), acc[i][t], 0, 0, 0);
    };
    auto hint_b = [&]() {
#pragma unroll
      for (int x = 0; x < (2 * C::TN < C::TM * C::TN ? 2 * C::TN : C::TM * C::TN); ++x) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    };
    // one non-final tile t computed from register set `cur`, while `nxt` receives tile t+1
    auto half = [&](const u32x4 (&cur)[C::TM][4], u32x4 (&nxt)[C::TM][4], int t) {
      const char* sb = smem + (t & 1) * C::STAGE_BYTES;
      load_a(nxt, tile_a(t + 1));
      __builtin_amdgcn_sched_barrier(0);   // keep the loads up here: a whole tile of MFMAs covers their latency
#pragma unroll
      for (int kk = 0; kk < 3; ++kk) {
        read_b(sb, kk + 1, (kk + 1) & 1);
        mfma_a(cur, kk, kk & 1);
        hint_b();
      }
      wait_vmcnt<0>();      // B tile t+1 (issued one tile ago) and A tile t+1 have arrived
      barrier_lds();        // ... for every wave; every wave is done reading B tile t
      ld.issue_b_direct(tile_b(t + 2), lds0 + (t & 1) * C::STAGE_BYTES, wave);
      read_b(smem + ((t + 1) & 1) * C::STAGE_BYTES, 0, 0);
      mfma_a(cur, 3, 1);
      hint_b();
    };
    auto final_tile = [&](const u32x4 (&cur)[C::TM][4], int t) {
      const char* sb = smem + (t & 1) * C::STAGE_BYTES;
#pragma unroll
      for (int kk = 0; kk < 3; ++kk) {
        read_b(sb, kk + 1, (kk + 1) & 1);
        mfma_a(cur, kk, kk & 1);
        hint_b();
      }
      mfma_a(cur, 3, 1);
    };
    if (nkt > 0) {
      u32x4 A0[C::TM][4], A1[C::TM][4];
      ld.issue_b_direct(tile_b(0), lds0, wave);
      load_a(A0, tile_a(0));
      wait_vmcnt<0>();
      barrier_lds();
      ld.issue_b_direct(tile_b(1), lds0 + C::STAGE_BYTES, wave);
      read_b(smem, 0, 0);
      int kt = 0;
      for (; kt + 2 <= last; kt += 2) {
        half(A0, A1, kt);
        half(A1, A0, kt + 1);
      }
      if (kt < last) {
        half(A0, A1, kt);
        final_tile(A1, last);
      } else {
        final_tile(A0, last);
      }
      wait_vmcnt<0>();
    }
  } else if constexpr (C::DIRECT && C::TM * C::TN * C::KS <= 8) {
    // Small wave tiles (skinny problems): a k16-step has only one or two MFMAs, far too few to
    // cover an LDS read, so the step-by-step pipeline above would stall four times per tile.
    // Here all fragments of a tile are read at once, into one of two register sets, while the
    // MFMAs of the previous tile run; one wait + barrier per tile. Unrolled by two so that both
    // sets are addressed statically.
    constexpr int D = C::STAGES - 1;
    constexpr int PER_TILE = C::A_PER_WAVE + C::B_PER_WAVE;
    static_assert((D - 1) * PER_TILE < 64, "vmcnt range");
    const unsigned lds0 = (unsigned)(size_t)smem;
    auto tile_a = [&](int t) { return Ak + (long)k_order(t < last ? t : last) * a_step; };
    auto tile_b = [&](int t) { return Bk + (long)k_order(t < last ? t : last) * b_step; };
    bf16x8 fa[2][C::KS][C::TM], fb[2][C::KS][C::TN];
    auto read_tile = [&](const char* stage, bf16x8 (&a)[C::KS][C::TM], bf16x8 (&b)[C::KS][C::TN]) {
#pragma unroll
      for (int kk = 0; kk < C::KS; ++kk) {
#pragma unroll
        for (int i = 0; i < C::TM; ++i) a[kk][i] = read_a(stage, kk, i);
#pragma unroll
        for (int t = 0; t < C::TN; ++t) b[kk][t] = read_b1(stage, kk, t);
      }
    };
    auto mfma_tile = [&](const bf16x8 (&a)[C::KS][C::TM], const bf16x8 (&b)[C::KS][C::TN]) {
#pragma unroll
      for (int kk = 0; kk < C::KS; ++kk)
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
#pragma unroll
          for (int t = 0; t < C::TN; ++t)
            acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[kk][t], a[kk][i], acc[i][t], 0, 0, 0);
    };
    if (nkt > 0) {
#pragma unroll
      for (int s = 0; s < D; ++s) ld.issue_direct(tile_a(s), tile_b(s), lds0 + s * C::STAGE_BYTES, wave);
      wait_vmcnt<(D - 1) * PER_TILE>();
      barrier_lds();
      ld.issue_direct(tile_a(D), tile_b(D), lds0 + D * C::STAGE_BYTES, wave);
      read_tile(smem, fa[0], fb[0]);
      int stage = 0;
      // one non-final tile t: its fragments are in (ca, cb); (na, nb) receive tile t+1
      auto step = [&](int t, const bf16x8 (&ca)[C::KS][C::TM], const bf16x8 (&cb)[C::KS][C::TN],
                      bf16x8 (&na)[C::KS][C::TM], bf16x8 (&nb)[C::KS][C::TN]) {
        int nstage = stage + 1;
        if (nstage == C::STAGES) nstage = 0;
        wait_vmcnt<(D - 1) * PER_TILE>();    // tile t+1 has landed
        barrier_lds();                       // ... for every wave; every wave holds tile t in registers
        ld.issue_direct(tile_a(t + 1 + D), tile_b(t + 1 + D), lds0 + stage * C::STAGE_BYTES, wave);
        read_tile(smem + nstage * C::STAGE_BYTES, na, nb);
        mfma_tile(ca, cb);
        stage = nstage;
      };
      int kt = 0;
      for (; kt + 2 <= last; kt += 2) {
        step(kt, fa[0], fb[0], fa[1], fb[1]);
        step(kt + 1, fa[1], fb[1], fa[0], fb[0]);
      }
      if (kt < last) {
        step(kt, fa[0], fb[0], fa[1], fb[1]);
        mfma_tile(fa[1], fb[1]);
      } else {
        mfma_tile(fa[0], fb[0]);
      }
      wait_vmcnt<0>();
    }
  } else if constexpr (C::DIRECT) {
    constexpr int D = C::STAGES - 1;                            // tiles in flight ahead of the one computed
    constexpr int PER_TILE = C::A_PER_WAVE + C::B_PER_WAVE;   // transfers per wave per tile
    static_assert((D - 1) * PER_TILE < 64, "vmcnt range");
    const unsigned lds0 = (unsigned)(size_t)smem;
    auto tile_a = [&](int t) { return Ak + (long)k_order(t < last ? t : last) * a_step; };
    auto tile_b = [&](int t) { return Bk + (long)k_order(t < last ? t : last) * b_step; };
    // A wave issues in order: a burst of transfers right after the barrier would hold back the
    // MFMAs behind it for as long as the load unit takes to accept the burst (the four waves of a
    // CU share one, at about 16 cycles per transfer). So the transfers of a tile are dealt out
    // one at a time between the fragment reads of two k16-steps: its A part during the last step
    // of the tile whose buffer it takes over, its B part during the first step of the next tile.
    // which: 1 = A part, 2 = B part; the fragment reads and the transfers keep this order, the
    // MFMAs are spread between them by the scheduling hint.
    auto read_frags_issue = [&](const char* stage, int kk, int set, int which, const uint16_t* src, unsigned dst_lds) {
      constexpr int NR = C::TM + C::TN;                   // fragment reads (A: one b128, B: a tr pair)
      const int nx = which == 1 ? C::A_PER_WAVE : C::B_PER_WAVE;
#pragma unroll
      for (int x = 0; x < (NR > 8 ? NR : 8); ++x) {
        if (x < C::TM) af[set][x] = read_a(stage, kk, x);
        else if (x < NR) bfr[set][x - C::TM] = read_b1(stage, kk, x - C::TM);
        if (x < nx) {
          if (which == 1) ld.issue_a_one(x, src, dst_lds, wave);
          else ld.issue_b_one(x, src, dst_lds, wave);
        }
      }
    };
    static_assert(C::A_PER_WAVE <= 8 && C::B_PER_WAVE <= 8, "transfers of one part fit between the reads of one step");
    if (nkt > 0) {
#pragma unroll
      for (int s = 0; s < D; ++s) ld.issue_direct(tile_a(s), tile_b(s), lds0 + s * C::STAGE_BYTES, wave);
      wait_vmcnt<(D - 1) * PER_TILE>();      // tile 0 has landed, D-1 younger tiles may still fly
      barrier_lds();
      // tile D: A part now, B part during the first step of tile 0 (as in the steady state)
      ld.issue_a_all(tile_a(D), lds0 + D * C::STAGE_BYTES, wave);
      read_frags(smem, 0, 0);
      int stage = 0;
      for (int kt = 0; kt < last; ++kt) {
        const char* cur = smem + stage * C::STAGE_BYTES;
        int nstage = stage + 1;
        if (nstage == C::STAGES) nstage = 0;
        int pstage = stage + D;               // buffer of tile kt + D (freed by the barrier before this tile)
        if (pstage >= C::STAGES) pstage -= C::STAGES;
        read_frags_issue(cur, 1, 1, 2, tile_b(kt + D), lds0 + pstage * C::STAGE_BYTES);
        mfma_step(0);
        interleave_hint();
#pragma unroll
        for (int kk = 1; kk < C::KS - 1; ++kk) {
          read_frags(cur, kk + 1, (kk + 1) & 1);
          mfma_step(kk & 1);
          interleave_hint();
        }
        wait_vmcnt<(D - 1) * PER_TILE>();    // tile kt+1 has landed
        barrier_lds();                       // ... for every wave, and every wave is done reading tile kt
        read_frags_issue(smem + nstage * C::STAGE_BYTES, 0, 0, 1, tile_a(kt + 1 + D), lds0 + stage * C::STAGE_BYTES);
        mfma_step(1);                        // the last k16-step of tile kt covers the latencies above
        interleave_hint();
        stage = nstage;
      }
      {
        const char* cur = smem + stage * C::STAGE_BYTES;
        int pstage = stage + D;
        if (pstage >= C::STAGES) pstage -= C::STAGES;
        // (the B part that completes the redundant A part issued at the last hand-over)
        read_frags_issue(cur, 1, 1, 2, tile_b(last + D), lds0 + pstage * C::STAGE_BYTES);
        mfma_step(0);
        interleave_hint();
#pragma unroll
        for (int kk = 1; kk < C::KS - 1; ++kk) {
          read_frags(cur, kk + 1, (kk + 1) & 1);
          mfma_step(kk & 1);
          interleave_hint();
        }
        mfma_step(1);
      }
      wait_vmcnt<0>();                       // the redundant prefetches must not outlive their LDS
    }
  } else {
    // Register-staged double buffering: the global loads of tile kt+1 fly during tile kt and are
    // written to the other LDS buffer before the hand-over barrier.
    static_assert(C::DIRECT || C::STAGES == 2, "register staging uses two buffers");
    u32x4 ra[TileLoader<C>::NA], rb[C::B_PER_WAVE];
    const int kbase = kt_begin * C::BK;
    auto load_tile = [&](int t) {
      const int tt = t < last ? t : last;
      ld.load_regs(Ak + (long)tt * a_step, Bk + (long)tt * b_step, kbase + tt * C::BK, p.K, ra, rb);
    };
    if (nkt > 0) {
      load_tile(0);
      ld.store_regs(smem, wave, lane, ra, rb);
      __syncthreads();
      load_tile(1);
      read_frags(smem, 0, 0);
      for (int kt = 0; kt < last; ++kt) {
        const char* cur = smem + (kt & 1) * C::STAGE_BYTES;
        char* nxt = smem + ((kt + 1) & 1) * C::STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < C::KS - 1; ++kk) {
          read_frags(cur, kk + 1, (kk + 1) & 1);
          mfma_step(kk & 1);
          interleave_hint();
        }
        ld.store_regs(nxt, wave, lane, ra, rb);   // buffer last read in iteration kt-1, released by its barrier
        __syncthreads();
        load_tile(kt + 2);
        read_frags(nxt, 0, 0);
        mfma_step(1);
      }
      {
        const char* cur = smem + (last & 1) * C::STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < C::KS - 1; ++kk) {
          read_frags(cur, kk + 1, (kk + 1) & 1);
          mfma_step(kk & 1);
          interleave_hint();
        }
        mfma_step(1);
      }
    }
  }

  // ---- accumulator layout. The MFMA is issued with the B fragment as its first operand and
  // the A fragment as its second, so each 32x32 block is held transposed: lane l, register r
  // holds  m = block_m + (l & 31),  n = block_n + 8 (r / 4) + 4 (l / 32) + (r % 4).
  // A lane therefore owns runs of four consecutive n, which pack into one 8-byte (bf16) or
  // 16-byte (fp32) store without any cross-lane exchange.
  const int lane_m = lane & 31, lane_g = lane >> 5;
  if constexpr (C::WK == 2) {
    // The two k groups hold partial sums of the same wave tile. Group 0 keeps its first TM/2 row
    // blocks and hands the others to its partner wave of group 1, which does the reverse;
    // afterwards acc[0 .. TM/2) of every wave holds complete sums of the rows it writes out.
    constexpr int H = C::TM / 2;
    wait_vmcnt<0>();
    barrier_lds();                          // nobody reads tiles any more, no transfer is in flight
    char* mine = smem + wave * (H * C::TN * 4096);
    const char* theirs = smem + ((wave_mn + (1 - wave_k) * C::WM * C::WN)) * (H * C::TN * 4096);
#pragma unroll
    for (int i = 0; i < H; ++i)
#pragma unroll
      for (int t = 0; t < C::TN; ++t) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = wave_k ? acc[i][t][4 * q + e] : acc[i + H][t][4 * q + e];
          *(f32x4*)(mine + (((i * C::TN + t) * 4 + q) * 64 + lane) * 16) = v;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][t][r] = wave_k ? acc[i + H][t][r] : acc[i][t][r];
      }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < H; ++i)
#pragma unroll
      for (int t = 0; t < C::TN; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 v = *(const f32x4*)(theirs + (((i * C::TN + t) * 4 + q) * 64 + lane) * 16);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][t][4 * q + e] += v[e];
        }
  }
  const int wm0 = m0 + wave_m * C::WTM + lane_m + (C::WK == 2 ? wave_k * 32 * (C::TM / 2) : 0);   // + 32 i
  const int wn0 = n0 + wave_n * C::WTN + 4 * lane_g;          // + 32 t + 8 q
  const int ncols = n_end - n0 < C::BN_ACT ? n_end - n0 : C::BN_ACT;     // columns this tile writes (a multiple of 8)
  const bool rows_full = m0 + C::BM <= p.M;
  const bool full = rows_full && ncols == C::BN_ACT;

  if (split) {
    // publish the partial tile; the last slice to arrive sums all slices in slice order
    const size_t slice = (size_t)p.M * p.N;
    float* wsk = p.ws + (size_t)tc.ks * slice;
    if (!C::FUSED_OK || !p.fused_reduce) {
      // two-kernel split-K: plain stores; a reduce kernel launched behind this one sums the
      // slices in slice order and applies the epilogue (the kernel boundary orders the two)
      if (C::stage_ok(4) && full && p.ws_vec16) {
        if constexpr (C::stage_ok(4))
          epilogue_staged<C, TF_EPI_NONE_F32, true>(acc, p, smem, m0, n0, tid, wave_m, wave_n, wave_k, lane_m, lane_g, (char*)wsk, (size_t)p.N);
      } else if (full) store_partial<C, true, false>(acc, wsk, p, wm0, wn0);
      else store_partial<C, false, false>(acc, wsk, p, wm0, wn0);
      continue;
    }
    if constexpr (C::FUSED_OK) {
    // Two ways to hand the partial tiles to the last slice:
    //  fused_reduce 1: device-scope (write-through) stores and loads, valid wherever the slices run;
    //  fused_reduce 2: plain stores and loads. The host offers it only when the tile order puts
    //    all slices of a tile on one XCD (work-group i runs on XCD i mod 8), whose L2 then holds
    //    the partial tiles: a store acknowledged by the L2 (vmcnt) is what any CU of the same XCD
    //    reads afterwards, and no CU has read these addresses earlier in the launch. Every slice
    //    reports the XCD it really ran on with its ticket; if they differ, the tile is poisoned
    //    with NaN rather than summed from memory that may be stale, and the status word of the
    //    workspace is set (the host probes the placement once per device before it launches this mode).
    const bool local = p.fused_reduce == 2;
    if (local) {
      if (full) store_partial<C, true, false>(acc, wsk, p, wm0, wn0);
      else store_partial<C, false, false>(acc, wsk, p, wm0, wn0);
    } else {
      if (full) store_partial<C, true, true>(acc, wsk, p, wm0, wn0);
      else store_partial<C, false, true>(acc, wsk, p, wm0, wn0);
    }
    // every store of this wave has been acknowledged before the wave reaches the barrier, so
    // the ticket taken after it is ordered behind the whole work-group's partials
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    // ticket word: arrivals in bits 0..7, arrivals per XCD in 7-bit fields above
    __shared__ unsigned long long ticket;
    unsigned long long* ctr = (unsigned long long*)p.counters + (tc.tm * p.tiles_n + tc.tn);
    const unsigned xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 7u;      // HW_REG_XCC_ID, bits 0..3
    const unsigned long long mine = 1ull + (1ull << (8 + 7 * xcc));
    // (the L2-local mode takes its ticket in this XCD's L2 as well: an atomic of narrower scope is carried out there,
    // one of device scope past it, at several times the latency; all slices of the tile sit on this XCD)
    if (tid == 0)
      ticket = (local ? __hip_atomic_fetch_add(ctr, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : atomicAdd(ctr, mine)) + mine;
    __syncthreads();
    const unsigned long long tk = ticket;
    if ((unsigned)(tk & 255u) != (unsigned)p.split_k) continue;
    if (tid == 0) *ctr = 0ull;        // ready for the next launch
    if (local) {
      if (full) sum_partials<C, true, false>(acc, p, wm0, wn0);
      else sum_partials<C, false, false>(acc, p, wm0, wn0);
      if ((unsigned)((tk >> (8 + 7 * xcc)) & 127u) != (unsigned)p.split_k) {
        if (tid == 0) atomicOr(p.status, 1u);   // reported by the next synchronous call of the library
        const float nan = __builtin_nanf("");
#pragma unroll
        for (int i = 0; i < C::TM_OUT; ++i)
#pragma unroll
          for (int t = 0; t < C::TN; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][t][r] = nan;
      }
    } else {
      if (full) sum_partials<C, true, true>(acc, p, wm0, wn0);
      else sum_partials<C, false, true>(acc, p, wm0, wn0);
    }
    }
  }

  // ---- epilogue: + bias, GELU, round to bf16 (or raw fp32 pre-activation)
  if (nkt <= 0) {            // no K step, so no hand-over has published the bias copy yet
    wait_vmcnt<0>();
    __syncthreads();
  }
  const char* bias_lds = smem + C::BIAS_OFF + (wave_n * C::WTN + 4 * lane_g) * 2;
  // whole rows of the tile go out coalesced through LDS, also when the tile's last columns do not exist or belong
  // to its neighbour (their pieces are skipped)
  const bool staged = rows_full && ncols > 0 && p.y_vec16;      // the same for every wave of the work-group
  auto finish = [&](auto tag) {
    constexpr int EPI = decltype(tag)::value;
    constexpr int ESZ = EPI == TF_EPI_NONE_F32 ? 4 : 2;
    if (C::stage_ok(ESZ) && staged) {
      if constexpr (C::stage_ok(ESZ))
        epilogue_staged<C, EPI>(acc, p, smem, m0, n0, tid, wave_m, wave_n, wave_k, lane_m, lane_g, (char*)p.Y, (size_t)p.ldy, ncols);
    } else if (full) epilogue<C, true, EPI>(acc, p, wm0, wn0, bias_lds, n_end);
    else epilogue<C, false, EPI>(acc, p, wm0, wn0, bias_lds, n_end);
  };
  if (p.epi == TF_EPI_BIAS_GELU_ERF) finish(EpiTag<TF_EPI_BIAS_GELU_ERF>{});
  else if (p.epi == TF_EPI_NONE_F32) finish(EpiTag<TF_EPI_NONE_F32>{});
  else if (p.epi == TF_EPI_BIAS) finish(EpiTag<TF_EPI_BIAS>{});
  else finish(EpiTag<TF_EPI_BIAS_GELU_TANH>{});
  }   // segments
}

template <class C>
__global__ void __launch_bounds__(C::THREADS) tf_gemm_lds_kernel(const GemmParams p) {
  gemm_tile_body<C>(p);
}

// A launch with a lighter last round. Equal tiles leave the chip badly filled whenever the tile count is a little
// above a multiple of the CU count (688 tiles on 256 CUs: the third round runs on 176 of them). Here the first
// work-groups (whole rounds) compute BN-wide tiles over the leading columns, and one more round of exactly one
// work-group per CU shares out the remaining columns of every row panel in narrower tiles (CN: the same staging,
// fewer columns multiplied): every CU gets the same number of tiles and nearly the same work. Work-groups are
// handed to the CUs in id order, so the narrow round comes last.
template <class CM, class CN>
__global__ void __launch_bounds__(CM::THREADS) tf_gemm_mixed_kernel(const GemmParams p) {
  static_assert(CM::THREADS == CN::THREADS && CM::LDS_BYTES == CN::LDS_BYTES && CM::BM == CN::BM && CM::BN == CN::BN &&
                CM::BK == CN::BK && CN::BN_ACT < CN::BN, "the two tile shapes share the work-group shape and the staging");
  if ((int)blockIdx.x < p.mix_main_wgs) gemm_tile_body<CM>(p);
  else gemm_tile_body<CN>(p);
}

// Persistent kernel for the batched transposed-operand product with few K steps per tile
// (C[b] = A[b]^T B[b], whole tiles only). With four K steps a work-group spends most of its life waiting for
// its first tiles and for the end of its stores; here one work-group per CU walks through many output tiles
// and the ring never drains: the transfers of the next tile's K steps are issued while the current tile still
// multiplies and writes out. The output goes through a staging area of its own behind the ring, so the ring
// stays free for those transfers.
//   * work-group w runs on XCD w mod 8; XCD x takes the batch items x, x + 8, ..., so an item's operands are
//     fetched into one L2; the work-groups of an XCD deal that XCD's tiles out among themselves in turn.
//   * one "flat step" = one K step of one tile. At flat step f the transfers of step f + D (D = STAGES - 1)
//     are issued into the buffer that step f - 1 has just left. Past the end the last step is fetched again
//     (into a buffer nobody reads), which keeps the number of transfers in flight, and so the vmcnt waits,
//     constant.
//   * vector-memory operations of a wave complete in issue order, stores included, so a transfer issued
//     behind a tile's stores would only count as landed once those stores (a trip to memory) are done. The
//     waves therefore split the memory work: the first half of the waves issue all transfers into the ring,
//     the second half all stores of the output; every wave multiplies.
//   * tried and dropped: setting the finished tile's accumulators aside and writing them out pass by pass
//     during the next tile's first K steps (T2: 48 us against 42 us, also with the waves split as above: the
//     second barrier in the middle of a step costs more than the overlap gains), and a fourth buffer with
//     half-size output passes (43 us against 39 us).
template <class C>
__global__ void __launch_bounds__(C::THREADS) tf_bgemm_persist_kernel(const GemmParams p) {
  static_assert(C::TRANSA && !C::TRANSB && C::DIRECT && C::WK == 1 && !C::ABYPASS && C::STAGES >= 3, "transposed staging, direct, three buffers or more");
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int D = C::STAGES - 1;
  // the loading half of the waves moves the tiles exactly as a work-group of half as many wave columns would
  static_assert(C::WN % 2 == 0, "an even number of wave columns");
  using CL = LdsCfg<C::BM, C::BN, C::BK, C::WM, C::WN / 2, C::STAGES, true, false, 1, true>;
  constexpr int LW = CL::NWAVES, STORE_THREADS = C::THREADS - LW * 64;
  static_assert(CL::STAGE_BYTES == C::STAGE_BYTES && CL::A_BYTES == C::A_BYTES, "same ring layout");
  constexpr int PER_TILE = CL::A_PER_WAVE + CL::B_PER_WAVE;
  constexpr int ROWB = C::BN * 4 + 16, CPR = C::BN * 4 / 16;
  constexpr int PER_THREAD = C::ST_ROWS * CPR / STORE_THREADS;
  static_assert(C::ST_ROWS * CPR % STORE_THREADS == 0, "pieces divide over the storing threads");
  static_assert((D - 1) * PER_TILE < 64, "vmcnt range");
  static_assert(C::PERSIST_LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
  char* const staging = smem + C::RING_BYTES;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / C::WN, wave_n = wave % C::WN;
  const int lane_m = lane & 31, lane_g = lane >> 5;

  // ---- this work-group's tiles
  const int tiles = p.tiles_m * p.tiles_n;                       // per batch item
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3, per_xcd = gridDim.x >> 3;
  const int items_x = (p.batch - xcd + 7) / 8;                   // items x, x + 8, ... < batch
  const int n_flat = items_x * tiles;
  const int my_tiles = local < n_flat ? (n_flat - local + per_xcd - 1) / per_xcd : 0;
  const int nkt = p.K / C::BK;
  const int total = my_tiles * nkt;
  if (total <= 0) return;
  struct Where { const uint16_t* a; const uint16_t* b; char* y; int m0, n0; };
  auto where = [&](int k) -> Where {                               // k-th tile of this work-group
    const int j = local + k * per_xcd;
    const int item = xcd + 8 * (j / tiles), tile = j % tiles;
    Where w;
    w.m0 = (tile % p.tiles_m) * C::BM; w.n0 = (tile / p.tiles_m) * C::BN;
    w.a = p.A + (size_t)item * p.stride_a + w.m0;                  // A[b] is [K][lda], m contiguous
    w.b = p.B + (size_t)item * p.stride_b + w.n0;
    w.y = (char*)p.Y + (size_t)item * p.stride_y * 4;
    return w;
  };

  // ---- LDS read offsets of this lane (bytes inside a stage), as in tf_gemm_lds_kernel
  int a_toff[C::TM], b_off[C::TN];
  {
    const int b = lane >> 4, s = lane & 15;
    const int krow = 8 * (b >> 1) + (s >> 2);
    const int within = (16 * (b & 1) + 4 * (s & 3)) * 2;
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
      const int j = (wave_m * C::WTM) / 32 + i;
      a_toff[i] = krow * C::A_ROW_BYTES + (j ^ b_swz<C::A_PIECES>(krow)) * 64 + within;
    }
#pragma unroll
    for (int t = 0; t < C::TN; ++t) {
      const int j = (wave_n * C::WTN) / 32 + t;
      b_off[t] = C::A_BYTES + krow * C::B_ROW_BYTES + (j ^ b_swz<C::B_PIECES>(krow)) * 64 + within;
    }
  }
  auto read_tr = [&](const char* ptr, int row_bytes) -> bf16x8 {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(ptr));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(ptr + 4 * row_bytes));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[C::TM][C::TN];
#pragma unroll
  for (int i = 0; i < C::TM; ++i)
#pragma unroll
    for (int t = 0; t < C::TN; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][t][r] = 0.0f;

  const bool loader = wave < LW;                 // wave-uniform
  TileLoader<CL> ld;
  ld.init(p, 0, 0, loader ? wave : 0, lane);     // offsets relative to the tile's corner: whole tiles only
  const unsigned lds0 = (unsigned)(size_t)smem;
  const size_t a_step = (size_t)C::BK * p.lda, b_step = (size_t)C::BK * p.ldb;

  // the loader runs D flat steps ahead of the multiplier
  int l_tile = 0, l_kt = 0, l_stage = 0;
  Where lw = where(0);
  auto issue_next = [&]() {
    if (loader) ld.issue_direct(lw.a + (size_t)l_kt * a_step, lw.b + (size_t)l_kt * b_step, lds0 + l_stage * C::STAGE_BYTES, wave);
    if (++l_stage == C::STAGES) l_stage = 0;
    if (l_tile * nkt + l_kt + 1 < total) {       // else: stay on the last step (fetched again, never read)
      if (++l_kt == nkt) { l_kt = 0; ++l_tile; lw = where(l_tile); }
    }
  };
#pragma unroll
  for (int s = 0; s < D; ++s) issue_next();

  int c_tile = 0, c_kt = 0, c_stage = 0;
  Where cw = where(0);
  for (int f = 0; f < total; ++f) {
    if (loader) wait_vmcnt<(D - 1) * PER_TILE>();   // this wave's transfers of step f have landed (it issues nothing else)
    barrier_lds();                 // step f has landed for every wave; every wave has left the buffer of step f - 1
    issue_next();                  // step f + D into that buffer
    const char* cur = smem + c_stage * C::STAGE_BYTES;
#pragma unroll
    for (int kk = 0; kk < C::KSTEPS; ++kk) {
      bf16x8 af[C::TM], bfr[C::TN];
#pragma unroll
      for (int i = 0; i < C::TM; ++i) af[i] = read_tr(cur + a_toff[i] + (16 * kk) * C::A_ROW_BYTES, C::A_ROW_BYTES);
#pragma unroll
      for (int t = 0; t < C::TN; ++t) bfr[t] = read_tr(cur + b_off[t] + (16 * kk) * C::B_ROW_BYTES, C::B_ROW_BYTES);
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int t = 0; t < C::TN; ++t)
          acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[t], af[i], acc[i][t], 0, 0, 0);
    }
    if (++c_stage == C::STAGES) c_stage = 0;
    if (++c_kt == nkt) {
      // ---- the tile is complete: out through the staging area, 32 rows per wave row at a time
      char* wr = staging + (wave_m * 32 + lane_m) * ROWB + (wave_n * C::WTN + 4 * lane_g) * 4;
#pragma unroll
      for (int i = 0; i < C::TM; ++i) {
        if (i) barrier_lds();      // the previous pass has been read back
#pragma unroll
        for (int t = 0; t < C::TN; ++t)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f32x4 v = {acc[i][t][4 * q], acc[i][t][4 * q + 1], acc[i][t][4 * q + 2], acc[i][t][4 * q + 3]};
            *(f32x4*)(wr + (32 * t + 8 * q) * 4) = v;
          }
        barrier_lds();
        if (!loader) {
#pragma unroll
          for (int j = 0; j < PER_THREAD; ++j) {
            const int c = (tid - LW * 64) + STORE_THREADS * j;
            const int rs = c / CPR, cc = c % CPR;
            const int m = cw.m0 + (rs >> 5) * C::WTM + 32 * i + (rs & 31);
            const u32x4 v = *(const u32x4*)(staging + rs * ROWB + cc * 16);
            __builtin_nontemporal_store(v, (u32x4*)(cw.y + ((size_t)m * p.ldy + cw.n0) * 4 + cc * 16));
          }
        }
      }
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int t = 0; t < C::TN; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][t][r] = 0.0f;
      c_kt = 0; ++c_tile;
      if (c_tile < my_tiles) cw = where(c_tile);
    }
  }
  wait_vmcnt<0>();                 // no transfer may still be on its way into this work-group's LDS when it ends
}

template <class C>
static void launch_persist(const GemmParams& p, dim3 grid, hipStream_t stream) {
  hipLaunchKernelGGL(tf_bgemm_persist_kernel<C>, grid, dim3(C::THREADS), C::PERSIST_LDS_BYTES, stream, p);
}

template <class C>
static LdsKernelInfo make_persist_info();

template <class C>
static void launch_lds(const GemmParams& p, dim3 grid, hipStream_t stream) {
  hipLaunchKernelGGL(tf_gemm_lds_kernel<C>, grid, dim3(C::THREADS), C::LDS_BYTES, stream, p);
}
template <class CM, class CN>
static void launch_mixed(const GemmParams& p, dim3 grid, hipStream_t stream) {
  hipLaunchKernelGGL((tf_gemm_mixed_kernel<CM, CN>), grid, dim3(CM::THREADS), CM::LDS_BYTES, stream, p);
}

// The same kernel with the loop over segments compiled in: work-groups may take several (tile, K range) pieces.
template <class Base>
struct StreamKCfg : Base { static constexpr bool SEGMENTS = true; };

template <class C>
static LdsKernelInfo make_info() {
  LdsKernelInfo k;
  k.bm = C::BM; k.bn = C::BN; k.bk = C::BK; k.waves_m = C::WM; k.waves_n = C::WN; k.waves_k = C::WK;
  k.stages = C::STAGES; k.direct_to_lds = C::DIRECT ? 1 : 0; k.a_bypass_lds = C::ABYPASS ? 1 : 0; k.trans_a = C::TRANSA ? 1 : 0;
  k.trans_b = C::TRANSB ? 1 : 0;
  k.threads = C::THREADS; k.lds_bytes = C::LDS_BYTES; k.fused_ok = C::FUSED_OK ? 1 : 0;
  k.persistent = 0; k.stream_k = C::SEGMENTS ? 1 : 0; k.bn_tail = 0;
  k.func = (const void*)tf_gemm_lds_kernel<C>;
  k.launch = launch_lds<C>;
  return k;
}

template <class CM, class CN>
static LdsKernelInfo make_mixed_info() {
  LdsKernelInfo k = make_info<CM>();
  k.bn_tail = CN::BN_ACT;
  k.func = (const void*)tf_gemm_mixed_kernel<CM, CN>;
  k.launch = launch_mixed<CM, CN>;
  return k;
}

template <class C>
static LdsKernelInfo make_persist_info() {
  LdsKernelInfo k = make_info<C>();
  k.persistent = 1;
  k.lds_bytes = C::PERSIST_LDS_BYTES;
  k.func = (const void*)tf_bgemm_persist_kernel<C>;
  k.launch = launch_persist<C>;
  return k;
}

//                         BM   BN   BK  WM WN ST  direct
using K256x128_d2 = LdsCfg<256, 128, 64, 2, 2, 2, true>;
using K128x256_d2 = LdsCfg<128, 256, 64, 2, 2, 2, true>;
using K128x128_d2 = LdsCfg<128, 128, 64, 2, 2, 2, true>;
using K128x128_d3 = LdsCfg<128, 128, 64, 2, 2, 3, true>;
using K128x128_r2 = LdsCfg<128, 128, 64, 2, 2, 2, false>;
using K64x64_r2   = LdsCfg< 64,  64, 64, 2, 2, 2, false>;
using K64x64_d3   = LdsCfg< 64,  64, 64, 2, 2, 3, true>;
using K32x128_d3  = LdsCfg< 32, 128, 64, 1, 4, 3, true>;
using K32x64_d4   = LdsCfg< 32,  64, 64, 1, 2, 4, true>;
using K32x128_r2  = LdsCfg< 32, 128, 64, 1, 4, 2, false>;
using K32x128_d6  = LdsCfg< 32, 128, 64, 1, 4, 6, true>;
using K32x64_d8   = LdsCfg< 32,  64, 64, 1, 2, 8, true>;
using K32x256_d4  = LdsCfg< 32, 256, 64, 1, 4, 4, true>;
using K32x32_d4   = LdsCfg< 32,  32, 64, 1, 1, 4, true>;
using K32x32_d8   = LdsCfg< 32,  32, 64, 1, 1, 8, true>;
using K128x128_w8a = LdsCfg<128, 128, 64, 2, 4, 3, true>;   // eight waves: two per SIMD cover each other's overheads
using K128x128_w8b = LdsCfg<128, 128, 64, 4, 2, 3, true>;
using K128x128_w8c = LdsCfg<128, 128, 64, 2, 4, 4, true>;
using K128x256_ab = LdsCfg<128, 256, 64, 4, 1, 2, true, true>;
using K128x128_k2a = LdsCfg<128, 128, 64, 2, 2, 3, true, false, 2>;   // two k groups of 2x2 waves
using K128x128_k2b = LdsCfg<128, 128, 64, 2, 2, 4, true, false, 2>;
// first operand transposed in memory ([K][M])
using T128x128_w8  = LdsCfg<128, 128, 64, 2, 4, 3, true, false, 1, true>;
using T128x128_d3  = LdsCfg<128, 128, 64, 2, 2, 3, true, false, 1, true>;
using T128x128_d2  = LdsCfg<128, 128, 64, 2, 2, 2, true, false, 1, true>;
using T256x256_w8  = LdsCfg<256, 256, 64, 4, 2, 2, true, false, 1, true>;
using T256x128_d2  = LdsCfg<256, 128, 64, 2, 2, 2, true, false, 1, true>;
using T64x64_d3    = LdsCfg< 64,  64, 64, 2, 2, 3, true, false, 1, true>;
// two buffers only: short K (a chunk) means few K steps per tile, and several work-groups per CU
// cover each other's start-up better than a deeper ring in one
using T128x128_w8s2 = LdsCfg<128, 128, 64, 2, 4, 2, true, false, 1, true>;
using T128x64_d2   = LdsCfg<128,  64, 64, 2, 2, 2, true, false, 1, true>;
using T64x128_d2   = LdsCfg< 64, 128, 64, 2, 2, 2, true, false, 1, true>;
using T64x64_d2    = LdsCfg< 64,  64, 64, 2, 2, 2, true, false, 1, true>;
using K256x256_w8a = LdsCfg<256, 256, 64, 2, 4, 2, true>;   // eight waves on the big tile: 128x64 or 64x128 per wave
using K256x256_w8b = LdsCfg<256, 256, 64, 4, 2, 2, true>;
// other K tiles. 128 wide: half as many hand-over barriers per K and 256-byte row pieces from memory, two buffers of
// 64 KB; 32 wide: four buffers of 32 KB behind the big tile, three K tiles in flight instead of one
using K128x128x128_w8a = LdsCfg<128, 128, 128, 2, 4, 2, true>;
using K128x128x128_w8b = LdsCfg<128, 128, 128, 4, 2, 2, true>;
using K128x128x128_k2  = LdsCfg<128, 128, 128, 2, 2, 2, true, false, 2>;
using K256x256x32_w8a  = LdsCfg<256, 256,  32, 2, 4, 4, true>;
using K256x256x32_w8b  = LdsCfg<256, 256,  32, 4, 2, 4, true>;
using K64x64x128_d3    = LdsCfg< 64,  64, 128, 2, 2, 3, true>;
using K32x64x128_d4    = LdsCfg< 32,  64, 128, 1, 2, 4, true>;
// eight waves of 64 x 64 on the rectangular tiles, three buffers of 48 KB
using K256x128_w8 = LdsCfg<256, 128, 64, 4, 2, 3, true>;
using K128x256_w8 = LdsCfg<128, 256, 64, 2, 4, 3, true>;
// second operand given as [N][K], k contiguous: staged and read like the A tile
using N256x256_w8a = LdsCfg<256, 256, 64, 2, 4, 2, true, false, 1, false, true>;
using N256x256_w8b = LdsCfg<256, 256, 64, 4, 2, 2, true, false, 1, false, true>;
using N128x128_w8a = LdsCfg<128, 128, 64, 2, 4, 3, true, false, 1, false, true>;
using N128x128_w8b = LdsCfg<128, 128, 64, 4, 2, 3, true, false, 1, false, true>;
using N128x128_d2  = LdsCfg<128, 128, 64, 2, 2, 2, true, false, 1, false, true>;
using N128x128x128 = LdsCfg<128, 128, 128, 2, 4, 2, true, false, 1, false, true>;
using N64x64_d3    = LdsCfg< 64,  64, 64, 2, 2, 3, true, false, 1, false, true>;
using N32x64_d4    = LdsCfg< 32,  64, 64, 1, 2, 4, true, false, 1, false, true>;
using N32x128_d3   = LdsCfg< 32, 128, 64, 1, 4, 3, true, false, 1, false, true>;
using N32x32_d4    = LdsCfg< 32,  32, 64, 1, 1, 4, true, false, 1, false, true>;
using N256x128_w8 = LdsCfg<256, 128, 64, 4, 2, 3, true, false, 1, false, true>;
// staged through registers: a ragged K tail is filled with zeros (K no multiple of the K tile)
using N128x128_r2 = LdsCfg<128, 128, 64, 2, 2, 2, false, false, 1, false, true>;
using N64x64_r2   = LdsCfg< 64,  64, 64, 2, 2, 2, false, false, 1, false, true>;
using N32x128_r2  = LdsCfg< 32, 128, 64, 1, 4, 2, false, false, 1, false, true>;
using N128x256_w8 = LdsCfg<128, 256, 64, 2, 4, 3, true, false, 1, false, true>;
// the big tile with only 192 of its 256 columns multiplied (4 x 2 waves of 64 x 96): the lighter last round
using K256x192_w8b = LdsCfg<256, 256, 64, 4, 2, 2, true, false, 1, false, false, 192>;
using N256x192_w8b = LdsCfg<256, 256, 64, 4, 2, 2, true, false, 1, false, true, 192>;     // the same with B staged as [n][k]

static LdsKernelInfo g_table[] = {
    make_info<K256x128_d2>(), make_info<K128x256_d2>(),
    make_info<K128x128_d2>(), make_info<K128x128_d3>(), make_info<K128x128_r2>(),
    make_info<K64x64_r2>(),   make_info<K64x64_d3>(),   make_info<K32x128_d3>(),
    make_info<K32x64_d4>(),   make_info<K32x128_r2>(),  make_info<K128x256_ab>(),
     make_info<K32x128_d6>(),  make_info<K32x64_d8>(),
    make_info<K32x256_d4>(),  make_info<K32x32_d4>(),   make_info<K32x32_d8>(),
    make_info<K128x128_w8a>(), make_info<K128x128_w8b>(), make_info<K128x128_w8c>(),
    make_info<K128x128_k2a>(), make_info<K128x128_k2b>(),
    make_info<T128x128_w8>(), make_info<T128x128_d3>(), make_info<T128x128_d2>(), make_info<T256x256_w8>(),
    make_info<T256x128_d2>(), make_info<T64x64_d3>(),
    make_info<T128x128_w8s2>(), make_info<T128x64_d2>(), make_info<T64x128_d2>(), make_info<T64x64_d2>(),
    make_info<K256x256_w8a>(), make_info<K256x256_w8b>(),
    make_persist_info<T128x128_w8>(), make_persist_info<T128x128_d3>(),
    make_info<StreamKCfg<K128x128_w8a>>(), make_info<StreamKCfg<K128x128_w8b>>(), make_info<StreamKCfg<K128x128_k2a>>(),
    make_info<K128x128x128_w8a>(), make_info<K128x128x128_w8b>(), make_info<K128x128x128_k2>(),
    make_info<K256x256x32_w8a>(), make_info<K256x256x32_w8b>(), make_info<K64x64x128_d3>(), make_info<K32x64x128_d4>(),
    make_info<K256x128_w8>(), make_info<K128x256_w8>(),
    make_info<N256x256_w8a>(), make_info<N256x256_w8b>(), make_info<N128x128_w8a>(), make_info<N128x128_w8b>(),
    make_info<N128x128_d2>(), make_info<N128x128x128>(), make_info<N64x64_d3>(), make_info<N32x64_d4>(),
    make_info<N32x128_d3>(), make_info<N32x32_d4>(), make_info<N256x128_w8>(), make_info<N128x256_w8>(),
    make_mixed_info<K256x256_w8a, K256x192_w8b>(), make_mixed_info<K256x256_w8b, K256x192_w8b>(),
    make_mixed_info<N256x256_w8a, N256x192_w8b>(), make_mixed_info<N256x256_w8b, N256x192_w8b>(),
    make_info<N128x128_r2>(), make_info<N64x64_r2>(), make_info<N32x128_r2>(),
};

int lds_kernel_count() { return (int)(sizeof(g_table) / sizeof(g_table[0])); }
const LdsKernelInfo* lds_kernel_table() { return g_table; }

}  // namespace tf
