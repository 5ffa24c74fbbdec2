"""Plain-Python oracle of the variant loop (paper Sec. 3.3, Algorithm 1).

TEST INFRASTRUCTURE ONLY; never imported by the product.  It restates the loop's control
structure and the rule tables that stand where the paper uses an LLM, step by step in the
paper's notation (K, K', K*, R, R', R*, dec), on plain dicts:

  Algorithm 1:  K* <- K; R* <- R; repeat { K' <- Proposal(H, K, R); res <- BuildRun(K');
                R' <- Profile(K'); dec <- Arbiter(R', R*); if dec = accept: K*, R* <- K', R';
                K <- RefineHint(K, R, R'); R <- R' } until dec = finish; return K*, R*.
  The remediation loop of the paper (an LLM repairs a kernel that failed to build) has no
  counterpart for pre-written kernels: a failed BuildRun is a report with status != 0, which
  the Arbiter cannot accept.
  The paper caps the number of rounds at 8 (end of Sec. 3.3) and calls a kernel successful at
  a speedup >= 1.05x over the baseline (Sec. 4.2).

Readings where the paper gives names but no values (Theta of the Arbiter; the hint table):
  accept   : the candidate ran, passed the correctness gate, its timing spread
             (median - min) / median is at most robust_spread, and
             t_med(R*) / t_med(R') >= first_accept_speedup while K* is still the baseline,
             >= later_accept_gain afterwards.
  finish   : not accepted and this is the patience-th consecutive round without an accept, or
             the round cap is reached.  (Case Study 3 stops after four non-improving rounds.)
  continue : otherwise.
  hint     : first match of
             grid_fill < 0.75 -> underfilled; intensity below the ridge and HBM >= 60 % -> hbm;
             MFMA >= 70 % -> mfma; LDS bank conflicts > 5 % (counters only) -> lds_conflict;
             occupancy < 25 % and MFMA < 50 % and HBM < 50 % -> occupancy; else latency.
             MFMA / HBM percentages come from counters when the report has them, else from the
             achieved algorithmic rates.  If the candidate is more than 2 % slower than the
             previous report and both get the same class, occupancy and latency swap.
  proposal : among untried tile kernels that move in the hinted direction relative to K, the
             smallest predicted time; else the smallest predicted time among all untried;
             ties to the lower id; none left -> the loop ends.
Pinned by tests against the paper's Case Study 3 table, the 1.05x bar, the round cap and the
loop invariants (K* never slower than the baseline, every accepted candidate passed parity).
"""
from __future__ import annotations

UNKNOWN, UNDERFILLED, HBM, MFMA, LDS_CONFLICT, OCCUPANCY, LATENCY = range(7)
CONTINUE, ACCEPT, FINISH = 0, 1, 2
NAIVE, MFMA_DIRECT, MFMA_LDS = 0, 1, 2

DEFAULT_THETA = dict(first_accept_speedup=1.05, later_accept_gain=1.02, robust_spread=0.10,
                     patience=4, max_rounds=8)


def arbiter(r_new, r_best, theta, best_is_baseline, stall_rounds, rnd):
    ran = r_new["status"] == 0 and r_new["parity_ok"] and r_new["t_med_us"] > 0 and r_best["t_med_us"] > 0
    if ran:
        spread = (r_new["t_med_us"] - r_new["t_min_us"]) / r_new["t_med_us"]
        need = theta["first_accept_speedup"] if best_is_baseline else theta["later_accept_gain"]
        if spread <= theta["robust_spread"] and r_best["t_med_us"] / r_new["t_med_us"] >= need:
            return ACCEPT
    if stall_rounds + 1 >= theta["patience"]:
        return FINISH
    if rnd >= theta["max_rounds"]:
        return FINISH
    return CONTINUE


def classify(r, hw):
    ridge = hw["bf16_tflops_peak"] * 1e3 / hw["hbm_gbs_peak"]
    if r["have_counters"]:
        mfma = r["mfma_busy_pct"]
        hbm = 100.0 * (r["hbm_read_gbs"] + r["hbm_write_gbs"]) / hw["hbm_gbs_peak"]
    else:
        mfma = r["pct_mfma_peak"]
        hbm = r["pct_hbm_peak"]
    if r["grid_fill"] < 0.75:
        return UNDERFILLED
    if r["arithmetic_intensity"] < ridge and hbm >= 60.0:
        return HBM
    if mfma >= 70.0:
        return MFMA
    if r["have_counters"] and r["lds_bank_conflict_pct"] > 5.0:
        return LDS_CONFLICT
    if r["occupancy_pct"] < 25.0 and mfma < 50.0 and hbm < 50.0:
        return OCCUPANCY
    return LATENCY


def refine_hint(r_prev, r_new, hw):
    if r_new["status"] != 0 or r_new["t_med_us"] <= 0:
        return UNKNOWN
    c = classify(r_new, hw)
    if (r_prev is not None and r_prev["status"] == 0 and r_prev["t_med_us"] > 0
            and r_new["t_med_us"] > 1.02 * r_prev["t_med_us"]):
        # the hint r_new was proposed under: the one the previous report carries
        followed = r_prev.get("bottleneck", UNKNOWN)
        if followed == UNKNOWN:
            followed = classify(r_prev, hw)
        if followed == c:
            if c == OCCUPANCY:
                c = LATENCY
            elif c == LATENCY:
                c = OCCUPANCY
    return c


def moves_in_direction(hint, base, v, fill_base, fill_v):
    area_b, area_v = base["bm"] * base["bn"], v["bm"] * v["bn"]
    if hint == UNDERFILLED:
        return fill_v > fill_base + 1e-9
    if hint == HBM:
        return (v["stages"] > base["stages"] or v["split_k"] > base["split_k"]
                or (v["direct_to_lds"] and not base["direct_to_lds"]) or v["grid"] > base["grid"])
    if hint == MFMA:
        return area_v >= area_b and fill_v >= fill_base - 1e-9
    if hint == LDS_CONFLICT:
        return v["direct_to_lds"] != base["direct_to_lds"] or v["bn"] != base["bn"]
    if hint == OCCUPANCY:
        return area_v < area_b or (area_v == area_b and v["lds_bytes"] < base["lds_bytes"])
    if hint == LATENCY:
        return (v["stages"] > base["stages"] or v["bk"] > base["bk"]
                or (v["direct_to_lds"] and not base["direct_to_lds"]) or area_v > area_b)
    return True


def proposal(family, predicted, fill, tried, base_id, hint):
    base = family[base_id] if 0 <= base_id < len(family) else None
    use_hint = base is not None and base["kind"] == MFMA_LDS and hint != UNKNOWN
    best = best_any = None
    for i, v in enumerate(family):
        if tried[i]:
            continue
        if best_any is None or predicted[i] < predicted[best_any]:
            best_any = i
        if use_hint and v["kind"] == MFMA_LDS and moves_in_direction(hint, base, v, fill[base_id], fill[i]):
            if best is None or predicted[i] < predicted[best]:
                best = i
    if best is not None:
        return best
    return -1 if best_any is None else best_any


def optimize(family, predicted, fill, profile, hw, theta=None):
    """Algorithm 1.  profile(i) -> report dict for variant i (BuildRun + gate + Profile).

    Returns (k_star, r_star, log) with log = [baseline report, one report per round], each
    report carrying its 'bottleneck' class and, for rounds, the 'decision'.
    """
    theta = dict(DEFAULT_THETA if theta is None else theta)
    tried = [False] * len(family)
    r = dict(profile(0))
    r["variant_id"] = 0
    r["bottleneck"] = refine_hint(None, r, hw)
    tried[0] = True
    log = [r]
    k_star, r_star = 0, r
    k, hint, stall = 0, UNKNOWN, 0
    for rnd in range(1, theta["max_rounds"] + 1):
        k_new = proposal(family, predicted, fill, tried, k, hint)
        if k_new < 0:
            break
        tried[k_new] = True
        r_new = dict(profile(k_new))
        r_new["variant_id"] = k_new
        r_new["bottleneck"] = refine_hint(r, r_new, hw)
        dec = arbiter(r_new, r_star, theta, k_star == 0, stall, rnd)
        r_new["decision"] = dec
        log.append(r_new)
        if dec == ACCEPT:
            k_star, r_star, stall = k_new, r_new, 0
        else:
            stall += 1
        if dec == FINISH:
            break
        k = k_new if dec == ACCEPT else k_star
        hint = r_new["bottleneck"] if (r_new["status"] == 0 and r_new["t_med_us"] > 0) else r_star["bottleneck"]
        r = r_new
    return k_star, r_star, log
