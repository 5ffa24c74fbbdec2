// Host logic of the profiling-guided variant loop (paper Sec. 3.3, Algorithm 1).
// Pure functions of reports and descriptors: nothing here touches the GPU, so the loop can
// be tested on synthetic reports.
//
// The paper names the roles (Proposal, BuildRun, Profile, Arbiter, RefineHint), the
// Arbiter's criteria (speedup, robustness, resource limits, diminishing returns), two
// example hints (memory stalls -> tiling/staging, low occupancy -> register pressure), the
// 1.05x success bar (Sec. 4.2) and the cap of 8 rounds; it gives no threshold values and its
// Proposal / RefineHint are an LLM. Here both are rules over a finite kernel family.
#include <math.h>
#include <string.h>

#include "tf_loop.h"

extern "C" void tf_theta_default(tf_theta* t) {
  if (!t) return;
  t->first_accept_speedup = 1.05;  // the paper's success bar against the baseline kernel
  t->later_accept_gain = 1.02;     // a new best must beat the old best by more than timing noise
  t->robust_spread = 0.10;
  t->patience = 4;   // Case Study 3 runs four consecutive non-improving rounds before it stops
  t->max_rounds = 8;
  t->cold_bytes = 512ll << 20;
}

extern "C" void tf_hw_nominal(tf_hw* h) {
  if (!h) return;
  memset(h, 0, sizeof(*h));
  strncpy(h->name, "AMD Instinct MI355X (published figures)", sizeof(h->name) - 1);
  h->cus = 256; h->simds_per_cu = 4; h->wave_size = 64; h->xcds = 8;
  h->lds_bytes_per_cu = 160 * 1024; h->vgprs_per_simd_lane = 512; h->max_waves_per_simd = 8;
  h->l2_bytes = 4ll << 20; h->hbm_bytes = 288ll << 30;
  h->clock_mhz = 2400.0; h->hbm_gbs_peak = 8000.0;
  h->bf16_tflops_peak = 256 * 4096.0 * 2400.0e6 / 1e12;   // 2516.6
}

// ------------------------------------------------------------------ Arbiter
extern "C" int32_t tf_arbiter(const tf_report* cand, const tf_report* best, const tf_theta* th,
                              int32_t best_is_baseline, int32_t stall_rounds, int32_t round) {
  if (!cand || !best || !th) return TF_DEC_FINISH;
  const bool usable = cand->status == TF_OK && cand->parity_ok != 0 && cand->t_med_us > 0.0 &&
                      best->t_med_us > 0.0;
  if (usable) {
    const double spread = (cand->t_med_us - cand->t_min_us) / cand->t_med_us;
    const double need = best_is_baseline ? th->first_accept_speedup : th->later_accept_gain;
    if (spread <= th->robust_spread && best->t_med_us / cand->t_med_us >= need) return TF_DEC_ACCEPT;
  }
  if (stall_rounds + 1 >= th->patience) return TF_DEC_FINISH;   // diminishing returns
  if (round >= th->max_rounds) return TF_DEC_FINISH;
  return TF_DEC_CONTINUE;
}

// ------------------------------------------------------------------ RefineHint
static int classify(const tf_report* r, const tf_hw* hw) {
  const double ridge = hw->bf16_tflops_peak * 1e3 / hw->hbm_gbs_peak;   // flop per byte
  const double mfma = r->have_counters ? r->mfma_busy_pct : r->pct_mfma_peak;
  const double hbm = r->have_counters ? 100.0 * (r->hbm_read_gbs + r->hbm_write_gbs) / hw->hbm_gbs_peak
                                      : r->pct_hbm_peak;
  if (r->grid_fill < 0.75) return TF_BN_UNDERFILLED;
  if (r->arithmetic_intensity < ridge && hbm >= 60.0) return TF_BN_HBM;
  if (mfma >= 70.0) return TF_BN_MFMA;
  if (r->have_counters && r->lds_bank_conflict_pct > 5.0) return TF_BN_LDS_CONFLICT;
  if (r->occupancy_pct < 25.0 && mfma < 50.0 && hbm < 50.0) return TF_BN_OCCUPANCY;
  return TF_BN_LATENCY;
}

extern "C" int32_t tf_refine_hint(const tf_report* prev, const tf_report* cand, const tf_hw* hw) {
  if (!cand || !hw) return TF_BN_UNKNOWN;
  if (cand->status != TF_OK || cand->t_med_us <= 0.0) return TF_BN_UNKNOWN;
  int c = classify(cand, hw);
  // The delta against the previous report: the candidate was proposed under the hint the previous report
  // carries (its bottleneck field; a report without one is read by its own figures). When that step made
  // things slower and the candidate's figures call for the same remedy again, the remedy has just failed:
  // swap between the two "nothing is saturated" diagnoses so that the next proposal goes the other way.
  // This reproduces the hints behind the rounds of Case Study 3 (Sec. 5): coalescing / staging, then lower
  // register use, then deeper pipelining, then less shared memory per work-group, each after a slower round.
  if (prev && prev->status == TF_OK && prev->t_med_us > 0.0 && cand->t_med_us > 1.02 * prev->t_med_us) {
    const int followed = prev->bottleneck != TF_BN_UNKNOWN ? prev->bottleneck : classify(prev, hw);
    if (followed == c) {
      if (c == TF_BN_OCCUPANCY) c = TF_BN_LATENCY;
      else if (c == TF_BN_LATENCY) c = TF_BN_OCCUPANCY;
    }
  }
  return c;
}

// ------------------------------------------------------------------ static cost model
static inline long cdiv(long a, long b) { return (a + b - 1) / b; }

extern "C" int32_t tf_resident_wgs(const tf_hw* hw, const tf_variant_desc* v) {
  if (v->kind == TF_KIND_MFMA_STREAM) {
    // about 128 registers per lane: four waves per SIMD; LDS only holds the final exchange
    const int waves = v->waves_k > 0 ? v->waves_k : 1;
    int r = 4 * hw->simds_per_cu / waves;
    const int by_lds = v->lds_bytes > 0 ? hw->lds_bytes_per_cu / v->lds_bytes : 8;
    if (by_lds < r) r = by_lds;
    return r < 1 ? 1 : (r > 8 ? 8 : r);
  }
  if (v->kind != TF_KIND_MFMA_LDS) return 8;
  const int acc_regs = (v->bm / v->waves_m) * (v->bn / v->waves_n) / 64;
  const int regs = acc_regs + 96;                      // fragments, staging, addresses
  int wps = hw->vgprs_per_simd_lane / regs;
  if (wps < 1) wps = 1;
  if (wps > hw->max_waves_per_simd) wps = hw->max_waves_per_simd;
  const int wg_waves = v->waves_m * v->waves_n * (v->waves_k > 1 ? v->waves_k : 1);
  int by_regs = wps * hw->simds_per_cu / wg_waves;
  if (by_regs < 1) by_regs = 1;
  int by_lds = v->lds_bytes > 0 ? hw->lds_bytes_per_cu / v->lds_bytes : 8;
  if (by_lds < 1) by_lds = 1;
  int r = by_regs < by_lds ? by_regs : by_lds;
  return r > 8 ? 8 : r;
}

extern "C" double tf_grid_fill(const tf_hw* hw, const tf_variant_desc* v) {
  const long slots = (long)hw->cus * tf_resident_wgs(hw, v);
  if (v->grid <= 0) return 0.0;
  return (double)v->grid / (double)(cdiv(v->grid, slots) * slots);
}

extern "C" double tf_predict_us(const tf_problem_desc* pr, const tf_hw* hw, const tf_variant_desc* v) {
  const double flops = 2.0 * pr->M * (double)pr->N * pr->K;
  const double bytes = 2.0 * ((double)pr->M * pr->K + (double)pr->K * pr->N + (double)pr->M * pr->N + pr->N);
  const double hbm_us = bytes / (hw->hbm_gbs_peak * 1e3);
  if (v->kind == TF_KIND_SIN) {
    // 8 bytes per element through HBM; a work-group costs about 0.45 us of one of the CU's slots to start and
    // retire whatever it does (few elements per work-group: that is all there is), and one- or two-element
    // accesses per lane reach about half the rate of 16-byte ones
    const double floor_us = 8.0 * (double)pr->N / (0.75 * hw->hbm_gbs_peak * 1e3);
    const double wg_us = (double)v->grid * 0.45 / ((double)hw->cus * 8.0);
    const double width = v->bk >= 4 ? 1.0 : (v->bk == 2 ? 0.9 : 0.55);
    // many passes per work-group hold many registers and leave few waves per SIMD; a grid-stride launch of
    // few work-groups loses the hardware's own balancing of the tail
    const double shape = 1.0 + 0.02 * (v->stages - 1) + (v->group_m ? 0.03 : 0.0) - (v->nontemporal ? 0.01 : 0.0);
    return fmax(floor_us / width * shape, wg_us) + 3.0;
  }
  if (pr->op == TF_OP_BATCHED_GEMM_TN) {
    // C[b] = A[b]^T B[b]: the tile model on one item with the whole grid, an HBM floor that counts the
    // fp32 output, and the transposing pass where the variant has one
    const double items = pr->batch > 0 ? (double)pr->batch : 1.0;
    const double tbytes = items * (2.0 * (double)pr->K * ((double)pr->M + pr->N) + 4.0 * (double)pr->M * pr->N);
    const double floor_us = tbytes / (0.75 * hw->hbm_gbs_peak * 1e3);
    if (v->kind == TF_KIND_BGEMM_TN_NAIVE) return items * 2.0 * pr->M * (double)pr->N * pr->K / (0.004 * hw->bf16_tflops_peak * 1e6) + 3.0;
    tf_problem_desc one = *pr;
    one.op = TF_OP_GEMM_EPILOGUE;
    tf_variant_desc v1 = *v;
    v1.trans_a = 0;
    if (v->persistent) {
      // one work-group per CU walks through the tiles and never lets its ring drain: the tile model over all
      // tiles, without the start-up that every work-group of the plain kernels pays
      v1.persistent = 0;
      v1.grid = (int32_t)(((pr->M + v->bm - 1) / v->bm) * (long)((pr->N + v->bn - 1) / v->bn) * (long)items);
      return fmax(0.8 * tf_predict_us(&one, hw, &v1), floor_us + 4.0);
    }
    double us = fmax(tf_predict_us(&one, hw, &v1), floor_us + 4.0);
    // with few K steps per tile a work-group is a short read - multiply - write sequence; alone on its CU
    // it leaves memory idle while it multiplies and the matrix pipes idle while it writes (measured 1.4-1.6x)
    const long slots_one = (long)hw->cus * tf_resident_wgs(hw, v);
    long co = cdiv(v->grid, hw->cus);
    if (co > slots_one / hw->cus) co = slots_one / hw->cus;
    if (co < 2) us *= 1.5;
    if (!v->trans_a) us += 3.0 + items * 4.0 * (double)pr->K * pr->M / (0.6 * hw->hbm_gbs_peak * 1e3);
    return us;
  }
  if (v->kind == TF_KIND_VECMAT_NAIVE || v->kind == TF_KIND_VECMAT_STREAM) {
    // C[m][n] = sum_k A[m][k] B[m][n][k]: B is read once; everything else is small
    const double vbytes = 2.0 * ((double)pr->M * pr->K + (double)pr->M * pr->N * pr->K) + 4.0 * (double)pr->M * pr->N;
    const double floor_us = vbytes / (hw->hbm_gbs_peak * 1e3);
    if (v->kind == TF_KIND_VECMAT_NAIVE) return floor_us / 0.12 + 3.0;     // 64 lines per load instruction
    // bytes a CU keeps in flight: resident waves (at most 16 by registers) x rows x chunks x 1 KB; about
    // 48 KB are needed for the rate the chip sustains (0.72 of the peak)
    double waves_per_cu = (double)v->grid * v->waves_k / hw->cus;
    if (waves_per_cu > 16.0) waves_per_cu = 16.0;
    double feed = waves_per_cu * v->bm * v->stages * 1024.0 / 49152.0;
    if (feed > 1.0) feed = 1.0;
    // a wave that takes many row groups in turn pays the memory latency once per group
    const double groups = (double)pr->M * (double)((pr->N + v->bm - 1) / v->bm);
    const double per_wave = groups / ((double)v->grid * v->waves_k);
    const double serial_us = per_wave * 2.0 / (waves_per_cu > 4.0 ? waves_per_cu / 4.0 : 1.0);
    return fmax(floor_us / (0.72 * feed), serial_us) + 3.0;
  }
  if (v->kind == TF_KIND_NAIVE) return fmax(flops / (0.004 * hw->bf16_tflops_peak * 1e6), hbm_us) + 2.0;
  if (v->kind == TF_KIND_MFMA_DIRECT) return fmax(flops / (0.02 * hw->bf16_tflops_peak * 1e6), hbm_us) + 2.0;
  if (v->kind == TF_KIND_MFMA_STREAM) {
    // B is read once at the rate the chip sustains from HBM, if enough waves keep loads in flight
    // (about 96 KB per CU; a wave keeps stages - 1 blocks of 8 KB outstanding)
    const double waves = (double)v->grid * (v->waves_k > 0 ? v->waves_k : 1);
    double feed = waves * (v->stages > 1 ? v->stages - 1 : 1) * 8192.0 / (98304.0 * hw->cus);
    if (feed > 1.0) feed = 1.0;
    const long kblocks = cdiv(cdiv(pr->K, 32), (long)v->split_k * (v->waves_k > 0 ? v->waves_k : 1));
    const double startup = 1.0 + 4.0 / (double)(kblocks > 0 ? kblocks : 1);      // short runs never reach the steady state
    // a CU draws at most about 37 GB/s from HBM (less in row pieces under 256 bytes): few work-groups cannot use the chip
    const double active = v->grid < hw->cus ? (double)v->grid : (double)hw->cus;
    const double cap_gbs = active * 37.0 * (v->bn >= 128 ? 1.0 : 0.65);
    double rate = 0.72 * feed * hw->hbm_gbs_peak;
    if (rate > cap_gbs) rate = cap_gbs;
    double us = bytes / (rate * 1e3) + startup + 2.5;
    // slices: the last work-group to arrive sums them after one more trip to memory, or a second launch does
    if (v->split_k > 1) us += (v->fused_reduce == 2 ? 2.0 : (v->fused_reduce ? 5.5 : 4.5)) + 2.0 * v->split_k * 4.0 * pr->M * (double)pr->N / (hw->hbm_gbs_peak * 1e3);
    return us;
  }
  const int resident = tf_resident_wgs(hw, v);
  const long slots = (long)hw->cus * resident;
  const int bk = v->bk > 0 ? v->bk : 64;
  const double kr = bk / 64.0;                      // the figures below are per 64 of K: a tile of bk is kr of them
  const long ktiles = cdiv(cdiv(pr->K, bk), v->split_k);
  const int mn_waves = v->waves_m * v->waves_n, wg_waves = mn_waves * (v->waves_k > 1 ? v->waves_k : 1);
  // Cycles one CU spends on one K tile (64 wide) of one work-group. The form of each term is what the kernels
  // do; the constants are a least-squares fit (of log predicted / measured, variants within 1.5x of the best) to
  // this family's measured times on MI355X on eight shapes (2048^3, 4096 x 11008 x 4096, 16 x 8192^2,
  // 1024^2 x 16384, 3072^3, 1024 x 8192 x 4096, 256 x 8192^2, 4096 x 2048^2) and were then checked on eight others:
  //  * the clock under MFMA load with every CU busy is about 1650 MHz, whatever the nominal figure says (the board
  //    is power limited); with fewer work-groups than CUs it is higher, by about 0.38 of the idle share; all
  //    cycle counts below are at that clock;
  //  * an MFMA 32x32x16 costs 36.5 cycles of its pipe, not 32;
  //  * tiles enter LDS at about 167 B/clk, fragments leave it at about 203 B/clk; reads and writes take turns;
  //  * a CU receives A tiles (short row pieces) at 82 B/clk and B tiles (long ones) at 52 B/clk when all CUs
  //    ask at once; 0.38 of that time is not hidden behind the matrix pipes;
  //  * per K step a chain of barrier, transfer issue, first fragment reads and first MFMA is
  //    exposed: about 490 cycles with two buffers, 237 with three or more, and a second wave per
  //    SIMD hides nearly all of it; register staging adds 300, the A-bypass loads 400.
  const double mfma = kr * v->bm * (double)v->bn / 32.0 * 1.14;
  const double stage_bytes = kr * (v->a_bypass_lds ? v->bn : v->bm + v->bn) * 128.0;
  const double lds_w = stage_bytes / 167.0;
  long co_resident = cdiv(v->grid, hw->cus);       // work-groups really sharing a CU, not how many would fit
  if (co_resident > resident) co_resident = resident;
  const double cu_waves = (double)wg_waves * co_resident;
  const double a_rows = v->a_bypass_lds ? 0.0 : (double)(v->bm / v->waves_m);
  const double lds_r = kr * mn_waves * (a_rows + (v->bn / v->waves_n)) * 128.0 / 203.0;
  const double ta = kr * (v->bm * 128.0 / 82.0 + v->bn * 128.0 / 52.0);         // global -> CU
  double chain = v->stages >= 3 ? 237.0 : 490.0;
  if (cu_waves >= 8) chain *= v->waves_k > 1 ? 0.455 : 0.05;    // k groups: half the MFMAs per wave and step to hide it behind
  // a K tile of 32 pays the chain twice per 64 of K
  if (bk < 64) chain *= 64.0 / bk;
  if (!v->direct_to_lds) chain += 300.0;
  if (v->a_bypass_lds) chain += 400.0;
  // the tile transfers are never fully hidden behind the matrix pipes: they share the LDS port with the fragment
  // reads and the L2 with the other CUs, and most of their time shows (measured: the 256 x 128 and 128 x 256
  // tiles, whose other figures match the 256 x 256 tile's, need 12-15 % more time per flop; they move 1.5 times
  // the bytes per flop)
  double ktile = fmax(fmax(mfma, lds_w + lds_r), ta) + chain + 0.376 * ta;
  // the in-kernel reductions keep the slices of a tile side by side, so the work-groups of an XCD work on
  // different K ranges and share fewer operand panels in its L2 than in the slice-by-slice order of the
  // two-kernel reduction (measured: about a quarter more time per K step)
  // (big tiles; the skinny tiles' operands are read once anyway)
  const double big = fmin(1.0, v->bm * (double)v->bn / 16384.0);
  if (v->split_k > 1 && v->fused_reduce) ktile *= 1.0 + 0.166 * big;
  // per tile: pipeline fill (first tiles from memory), then bias + GELU + pack at about 11 VALU
  // issue slots per element, or the fp32 partial tile at 32 B/clk when a second kernel reduces
  const double fill = 2900.0 / (double)co_resident;
  // (the raw fp32 output has no activation to evaluate: 16-byte stores at about 64 B/clk)
  // VALU issue slots per output element of the epilogue: erf-GELU 11, tanh-GELU 7, plain conversions 2
  const double epi_valu = pr->epi == TF_EPI_BIAS_GELU_ERF ? 11.0 : pr->epi == TF_EPI_BIAS_GELU_TANH ? 7.0 : 2.0;
  double tile_end = v->bm * (double)v->bn * epi_valu / 64.0;
  if (v->waves_k > 1) tile_end += v->bm * (double)v->bn * 4.0 * (1.0 / 85.0 + 1.0 / 256.0) / 2.0 * v->waves_k;   // accumulator exchange
  double reduce_us = 0.0, fused_tail_us = 0.0;
  const double active = v->grid < hw->cus ? (double)v->grid / hw->cus : 1.0;
  const double mhz = (hw->clock_mhz < 1650.0 ? hw->clock_mhz : 1650.0) * (1.0 + 0.38 * (1.0 - active));
  if (v->split_k > 1) {
    if (v->fused_reduce == 2) {
      // partial tiles stay in the L2 the slices share: 16-byte stores and loads, one round of tickets
      // ... but the last slice of a tile still sums all slices and runs the epilogue alone, on one CU
      fused_tail_us = 2.0 + 3.0 * big + v->bm * (double)v->bn * 4.0 * (1.0 + 2.0 * v->split_k) / 64.0 / mhz;
    } else if (v->fused_reduce) {
      // partial tiles go out and come back through 16-byte device-scope accesses; the store acknowledgement,
      // the ticket and one load round trip per slice are dependent trips to memory on the last slice's path
      fused_tail_us = 4.0 + 2.5 * v->split_k + v->bm * (double)v->bn * 4.0 * (1.0 + v->split_k) / 32.0 / mhz;
    } else {
      tile_end = v->bm * (double)v->bn * 4.0 / 32.0;
      reduce_us = 4.5 + (v->split_k + 0.5) * 4.0 * pr->M * (double)pr->N / (0.686 * hw->hbm_gbs_peak * 1e3);
    }
  }
  // CUs take the next work-group as they finish one: whole rounds, then a last round that takes between half a
  // round's time (few work-groups left: they have the chip's memory system and power budget to themselves)
  // and all of it, plus a ragged end
  double rounds = (double)v->grid / (double)slots;
  if (rounds <= 1.0) {
    rounds = 1.0;
  } else {
    const double whole = floor(rounds + 1e-9), part = rounds - whole;
    rounds = whole + (part < 1e-9 ? 0.0 : 0.51 + 0.49 * part) + 0.09;
  }
  // a lighter last round: whole rounds of full tiles, then one of tiles that multiply bn_tail of their bn columns
  if (v->bn_tail > 0 && v->bn > 0) rounds = (double)v->grid / (double)slots - 1.0 + (double)v->bn_tail / v->bn + 0.05;
  if (v->stream_k) {
    // every CU gets the same number of K steps: the tile count over the CU count, no ragged last round. But the
    // shares start at arbitrary K offsets, so the work-groups of an XCD no longer walk through K together and
    // stop sharing operand panels in its L2 (measured: about 1.6x the time per K step), each piece refills
    // the pipeline, and each shared tile costs its contributors the store acknowledgement, the ticket and a
    // load round trip, one after the other
    rounds = 1.6 * (double)((pr->M + v->bm - 1) / v->bm) * (double)((pr->N + v->bn - 1) / v->bn) / (double)hw->cus;
    fused_tail_us = 12.0;
  }
  const double per_cu = rounds * (double)co_resident;            // work-groups one CU works through
  const double us = per_cu * (ktiles * ktile + fill + tile_end) / mhz;
  const double ws_us = v->split_k > 1 ? 2.0 * v->split_k * 4.0 * pr->M * (double)pr->N / (hw->hbm_gbs_peak * 1e3) : 0.0;
  // HBM floor: about three quarters of the peak rate when at least 32 KB per CU are in flight
  // (prefetched tiles of all co-resident work-groups), in proportion below that
  double inflight = (double)co_resident * (v->stages - 1) * stage_bytes / 32768.0;
  if (inflight > 1.0) inflight = 1.0;
  // launch, first tile from HBM and drain: about 3.6 us per launch
  // K order rotated by XCD: measured 2-4 % faster on 2048^3, between equal and 10 % faster on
  // 4096 x 11008 x 4096 depending on the kernel and the chip: proposed first, the plain order right behind
  // (the eight-wave 256 x 128 and 128 x 256 tiles were 0-8 % slower with it on five other shapes)
  const double rot = !v->k_rotate ? 1.0 : ((long)v->bm * v->bn == 32768 && wg_waves == 8) ? 1.02 : 0.98;
  // B given as [N][K] behind a separate transposing pass: one more launch that reads and writes all of B
  const double pretrans_us = (pr->op == TF_OP_GEMM_EPILOGUE && pr->trans_b && !v->trans_b)
                                 ? 3.0 + 4.0 * (double)pr->K * pr->N / (0.6 * hw->hbm_gbs_peak * 1e3) : 0.0;
  // tiles dealt round-robin over the XCDs (offered for one row of tiles): every row of B is then pulled through all
  // eight L2s at once, which streams about a tenth faster than a contiguous run of columns per XCD
  // (and a K tile of 128 streamed 8-10 % slower than one of 64 on 16 x 8192 x 8192: 28.8-29.3 against 26.6-27.1 us)
  const double spread = (v->xcd_swizzle ? 1.0 : 0.9) * (bk > 64 ? 1.08 : 1.0);
  return fmax(us * rot, (hbm_us + ws_us) / (0.75 * inflight) * spread) + 3.6 + reduce_us + fused_tail_us + pretrans_us;
}

// ------------------------------------------------------------------ Proposal
static bool matches_hint(int bn, const tf_hw* hw, const tf_variant_desc* b, const tf_variant_desc* v) {
  const double fill_b = tf_grid_fill(hw, b), fill_v = tf_grid_fill(hw, v);
  const long area_b = (long)b->bm * b->bn, area_v = (long)v->bm * v->bn;
  switch (bn) {
    case TF_BN_UNDERFILLED:   // more, smaller units of work
      return fill_v > fill_b + 1e-9;
    case TF_BN_HBM:           // more bytes in flight
      return v->stages > b->stages || v->split_k > b->split_k || (v->direct_to_lds && !b->direct_to_lds) ||
             v->grid > b->grid;
    case TF_BN_MFMA:          // only quantisation and LDS traffic per MFMA are left
      return area_v >= area_b && fill_v >= fill_b - 1e-9;
    case TF_BN_LDS_CONFLICT:  // other staging path or other tile shape
      return v->direct_to_lds != b->direct_to_lds || v->bn != b->bn;
    case TF_BN_OCCUPANCY:     // fewer registers / less LDS per work-group
      return area_v < area_b || (area_v == area_b && v->lds_bytes < b->lds_bytes);
    case TF_BN_LATENCY:       // deeper staging (more buffers, or a longer K tile: fewer hand-overs), or bigger tiles to amortise it
      return v->stages > b->stages || v->bk > b->bk || (v->direct_to_lds && !b->direct_to_lds) || area_v > area_b;
    default:
      return true;
  }
}

extern "C" int32_t tf_proposal_from(const tf_hw* hw, const tf_variant_desc* family, const double* predicted_us,
                                    int32_t n, const uint8_t* tried, int32_t base_id, int32_t bottleneck) {
  if (!hw || !family || !predicted_us || !tried || n <= 0) return -1;
  const tf_variant_desc* base = (base_id >= 0 && base_id < n) ? &family[base_id] : nullptr;
  const bool use_hint = base && base->kind == TF_KIND_MFMA_LDS && bottleneck != TF_BN_UNKNOWN;
  int best = -1, best_any = -1;
  for (int i = 0; i < n; ++i) {
    if (tried[i]) continue;
    if (best_any < 0 || predicted_us[i] < predicted_us[best_any]) best_any = i;
    if (use_hint && family[i].kind == TF_KIND_MFMA_LDS && matches_hint(bottleneck, hw, base, &family[i])) {
      if (best < 0 || predicted_us[i] < predicted_us[best]) best = i;
    }
  }
  return best >= 0 ? best : best_any;
}

extern "C" int32_t tf_proposal(const tf_problem_desc* prob, const tf_hw* hw, const tf_variant_desc* family,
                               int32_t n, const uint8_t* tried, int32_t base_id, int32_t bottleneck) {
  if (!prob || !hw || !family || !tried || n <= 0) return -1;
  double* pred = new double[n];
  for (int i = 0; i < n; ++i) pred[i] = tf_predict_us(prob, hw, &family[i]);
  const int r = tf_proposal_from(hw, family, pred, n, tried, base_id, bottleneck);
  delete[] pred;
  return r;
}

// ------------------------------------------------------------------ Algorithm 1
namespace tf {

tf_status run_loop(const tf_problem_desc* prob, const tf_hw* hw, const tf_variant_desc* family, int32_t n,
                   const tf_theta* theta, profile_fn profile, void* user, int32_t* best_variant, tf_report* best,
                   tf_report* round_log, int32_t log_cap, int32_t* n_log) {
  if (!prob || !hw || !family || n <= 0 || !theta || !profile || !best_variant || !best || !round_log || !n_log)
    return TF_E_INVALID;
  if (log_cap < 1 + theta->max_rounds) return TF_E_RANGE;
  uint8_t* tried = new uint8_t[n]();
  // K* <- K, R* <- R : the baseline kernel is variant 0
  tf_report R;
  tf_status st = profile(user, 0, &R);
  if (st != TF_OK || R.status != TF_OK) { delete[] tried; return st != TF_OK ? st : (tf_status)R.status; }
  R.bottleneck = tf_refine_hint(nullptr, &R, hw);
  tried[0] = 1;
  int nl = 0;
  round_log[nl++] = R;
  tf_report Rstar = R;
  int kstar = 0, kcur = 0, bottleneck = TF_BN_UNKNOWN;   // first proposal: the static one-shot pick
  int stall = 0;
  for (int round = 1; round <= theta->max_rounds; ++round) {
    const int cand = tf_proposal(prob, hw, family, n, tried, kcur, bottleneck);
    if (cand < 0) break;                          // family exhausted
    tried[cand] = 1;
    tf_report Rc;
    st = profile(user, cand, &Rc);                // BuildRun + parity gate + Profile
    if (st != TF_OK) { Rc.status = st; Rc.variant_id = cand; }
    Rc.bottleneck = tf_refine_hint(&R, &Rc, hw);
    round_log[nl++] = Rc;
    const int dec = tf_arbiter(&Rc, &Rstar, theta, kstar == 0, stall, round);
    if (dec == TF_DEC_ACCEPT) { kstar = cand; Rstar = Rc; stall = 0; }
    else ++stall;
    if (dec == TF_DEC_FINISH) break;
    // K <- RefineHint(K, R, R'): an accepted candidate becomes the kernel the next proposal
    // starts from; otherwise the next proposal starts again from K*. Either way the newest
    // valid diagnosis gives the direction.
    kcur = (dec == TF_DEC_ACCEPT) ? cand : kstar;
    bottleneck = (Rc.status == TF_OK && Rc.t_med_us > 0.0) ? Rc.bottleneck : Rstar.bottleneck;
    R = Rc;
  }
  *best_variant = kstar;
  *best = Rstar;
  *n_log = nl;
  delete[] tried;
  return TF_OK;
}

}  // namespace tf

// Algorithm 1 over pre-made reports (reports[i] is what Profile would return for variant i):
// the loop without a GPU, for tests and for replaying recorded profiles.
struct SimCtx { const tf_report* reports; int n; };
static tf_status sim_profile(void* user, int32_t id, tf_report* out) {
  const SimCtx* c = (const SimCtx*)user;
  if (id < 0 || id >= c->n) return TF_E_INVALID;
  *out = c->reports[id];
  out->variant_id = id;
  return TF_OK;
}

extern "C" tf_status tf_tune_replay(const tf_problem_desc* prob, const tf_hw* hw, const tf_variant_desc* family,
                                    const tf_report* reports, int32_t n, const tf_theta* theta,
                                    int32_t* best_variant, tf_report* best, tf_report* round_log,
                                    int32_t log_cap, int32_t* n_log) {
  if (!reports) return TF_E_INVALID;
  SimCtx c{reports, n};
  return tf::run_loop(prob, hw, family, n, theta, sim_profile, &c, best_variant, best, round_log, log_cap, n_log);
}
