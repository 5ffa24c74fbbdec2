"""Pins for the loop oracle (oracle/loop_oracle.py) against what the paper fixes:
the five-round table of Case Study 3, the 1.05x success bar (Sec. 4.2), the cap of 8
rounds (Sec. 3.3) and the invariants of Algorithm 1."""
import os
import random

import pytest

from oracle import loop_oracle as lo

HW = dict(bf16_tflops_peak=2516.6, hbm_gbs_peak=8000.0)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "case_study3_rounds.txt")


def report(t_med, **kw):
    r = dict(status=0, parity_ok=1, t_med_us=t_med, t_min_us=t_med * 0.99, grid_fill=1.0,
             arithmetic_intensity=1000.0, pct_mfma_peak=40.0, pct_hbm_peak=10.0, occupancy_pct=50.0,
             have_counters=0, mfma_busy_pct=0.0, hbm_read_gbs=0.0, hbm_write_gbs=0.0,
             lds_bank_conflict_pct=0.0)
    r.update(kw)
    return r


def variant(kind=lo.MFMA_LDS, bm=128, bn=128, stages=2, split_k=1, direct=1, lds=65536, grid=256, bk=64):
    return dict(kind=kind, bm=bm, bn=bn, bk=bk, stages=stages, split_k=split_k, direct_to_lds=direct, lds_bytes=lds,
                grid=grid)


def load_case_study3():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        rows.append(dict(round=int(f[0]), total_ms=float(f[1]), speedup=float(f[2]), kernel_ms=float(f[3]),
                         mem=float(f[4]), sm=float(f[5]), occ=float(f[6])))
    return rows


def test_case_study3_table_is_consistent_with_its_own_speedups():
    rows = load_case_study3()
    assert [r["round"] for r in rows] == [1, 2, 3, 4, 5]
    base = rows[0]["total_ms"]
    for r in rows:
        assert round(base / r["total_ms"], 2) == pytest.approx(r["speedup"], abs=0.011)
    assert base / rows[4]["total_ms"] == pytest.approx(1.0028, abs=5e-4)   # the text's 1.0028x


def test_case_study3_replay_no_round_is_accepted_and_round5_ends_the_loop():
    rows = load_case_study3()
    reports = [report(r["total_ms"] * 1e3, pct_mfma_peak=r["sm"], pct_hbm_peak=r["mem"], occupancy_pct=r["occ"])
               for r in rows]
    family = [variant(kind=lo.NAIVE)] + [variant() for _ in rows[1:]]
    # proposals in table order: predicted time increasing with the round index
    k_star, r_star, log = lo.optimize(family, predicted=[0, 1, 2, 3, 4], fill=[1.0] * 5,
                                      profile=lambda i: reports[i], hw=HW)
    assert k_star == 0 and r_star["t_med_us"] == pytest.approx(9690.0)
    assert [r["variant_id"] for r in log] == [0, 1, 2, 3, 4]
    assert [r["decision"] for r in log[1:]] == [lo.CONTINUE, lo.CONTINUE, lo.CONTINUE, lo.FINISH]
    # round 5 is faster than the baseline but below the 1.05x bar: "no improvement"
    assert log[4]["t_med_us"] < log[0]["t_med_us"]


def test_success_bar_is_1_05():
    th = lo.DEFAULT_THETA
    best = report(100.0)
    assert lo.arbiter(report(100.0 / 1.0499), best, th, True, 0, 1) == lo.CONTINUE
    assert lo.arbiter(report(100.0 / 1.0501), best, th, True, 0, 1) == lo.ACCEPT
    # once something has been accepted a smaller, still measurable gain is enough
    assert lo.arbiter(report(100.0 / 1.03), best, th, False, 0, 2) == lo.ACCEPT
    assert lo.arbiter(report(100.0 / 1.01), best, th, False, 0, 2) == lo.CONTINUE


def test_arbiter_rejects_failed_unverified_and_noisy_candidates():
    th = lo.DEFAULT_THETA
    best = report(100.0)
    assert lo.arbiter(report(10.0, status=-2), best, th, True, 0, 1) == lo.CONTINUE
    assert lo.arbiter(report(10.0, parity_ok=0), best, th, True, 0, 1) == lo.CONTINUE
    assert lo.arbiter(report(10.0, t_min_us=5.0), best, th, True, 0, 1) == lo.CONTINUE   # spread 50 %
    assert lo.arbiter(report(10.0), best, th, True, 0, 1) == lo.ACCEPT


def test_round_cap_and_patience():
    th = lo.DEFAULT_THETA
    best = report(100.0)
    slow = report(200.0)
    assert lo.arbiter(slow, best, th, True, 2, 3) == lo.CONTINUE
    assert lo.arbiter(slow, best, th, True, 3, 4) == lo.FINISH       # fourth miss in a row
    assert lo.arbiter(slow, best, th, False, 0, 8) == lo.FINISH      # cap
    assert lo.arbiter(report(50.0), best, th, False, 0, 8) == lo.ACCEPT


def test_loop_never_exceeds_eight_rounds_and_never_returns_something_slower():
    rng = random.Random(5)
    for trial in range(200):
        n = rng.randint(2, 30)
        family = [variant(kind=lo.NAIVE)] + [variant(bm=rng.choice([64, 128, 256]), bn=rng.choice([64, 128, 256]),
                                                     stages=rng.choice([2, 3]), split_k=rng.choice([1, 2, 4]),
                                                     direct=rng.randint(0, 1)) for _ in range(n - 1)]
        reports = [report(rng.uniform(5, 500), status=rng.choice([0, 0, 0, -2]), parity_ok=rng.choice([1, 1, 0]),
                          grid_fill=rng.uniform(0.2, 1.0), pct_mfma_peak=rng.uniform(1, 90),
                          occupancy_pct=rng.choice([12.5, 25.0, 50.0])) for _ in range(n)]
        reports[0]["status"], reports[0]["parity_ok"] = 0, 1
        calls = []

        def prof(i):
            calls.append(i)
            return reports[i]
        k_star, r_star, log = lo.optimize(family, [rng.random() for _ in range(n)], [rng.random() for _ in range(n)],
                                          prof, HW)
        assert len(log) - 1 <= 8
        assert len(set(calls)) == len(calls)                       # no variant profiled twice
        assert r_star["t_med_us"] <= reports[0]["t_med_us"]
        assert r_star["status"] == 0 and r_star["parity_ok"]
        if k_star != 0:
            assert reports[0]["t_med_us"] / r_star["t_med_us"] >= 1.05
        accepted = [r for r in log[1:] if r["decision"] == lo.ACCEPT]
        assert all(r["parity_ok"] and r["status"] == 0 for r in accepted)
        ts = [reports[0]["t_med_us"]] + [r["t_med_us"] for r in accepted]
        assert all(a > b for a, b in zip(ts, ts[1:]))              # every accept is an improvement


def test_hint_table():
    assert lo.classify(report(10, grid_fill=0.25), HW) == lo.UNDERFILLED
    assert lo.classify(report(10, arithmetic_intensity=16.0, pct_hbm_peak=75.0), HW) == lo.HBM
    assert lo.classify(report(10, pct_mfma_peak=72.0), HW) == lo.MFMA
    assert lo.classify(report(10, have_counters=1, mfma_busy_pct=30.0, lds_bank_conflict_pct=9.0), HW) == lo.LDS_CONFLICT
    assert lo.classify(report(10, occupancy_pct=12.5), HW) == lo.OCCUPANCY
    assert lo.classify(report(10, occupancy_pct=50.0), HW) == lo.LATENCY
    # counters override the achieved-rate estimates
    assert lo.classify(report(10, pct_mfma_peak=10.0, have_counters=1, mfma_busy_pct=80.0), HW) == lo.MFMA
    # the delta: same diagnosis and slower than before -> the other "nothing saturated" class
    prev, cur = report(10, occupancy_pct=12.5), report(11, occupancy_pct=12.5)
    assert lo.refine_hint(prev, cur, HW) == lo.LATENCY
    assert lo.refine_hint(None, cur, HW) == lo.OCCUPANCY
    assert lo.refine_hint(prev, report(11, status=-3), HW) == lo.UNKNOWN


def test_proposal_directions():
    fam = [variant(kind=lo.NAIVE), variant(bm=128, bn=128, grid=64), variant(kind=lo.MFMA_LDS, bm=64, bn=64, grid=256),
           variant(bm=128, bn=128, split_k=4, grid=256), variant(bm=256, bn=256, grid=16), variant(bm=128, bn=128, stages=3, grid=64)]
    pred = [1000, 20, 30, 25, 50, 22]
    fill = [1.0, 0.25, 1.0, 1.0, 0.06, 0.25]
    tried = [True, True, False, False, False, False]
    assert lo.proposal(fam, pred, fill, tried, 1, lo.UNDERFILLED) == 3     # better fill, best predicted of those
    assert lo.proposal(fam, pred, fill, tried, 1, lo.LATENCY) == 5         # deeper staging
    assert lo.proposal(fam, pred, fill, tried, 1, lo.OCCUPANCY) == 2       # smaller tile
    assert lo.proposal(fam, pred, fill, tried, 1, lo.UNKNOWN) == 5         # plain best predicted
    assert lo.proposal(fam, pred, fill, tried, 0, lo.LATENCY) == 5         # hints need a tile kernel as base
    assert lo.proposal(fam, pred, fill, [True] * 6, 1, lo.LATENCY) == -1
    # MFMA-bound: only equal-or-bigger tiles with no worse fill qualify (3 and 5; not the 256x256
    # one whose fill drops); the better predicted of the two wins
    assert lo.proposal(fam, pred, fill, tried, 1, lo.MFMA) == 5
    assert lo.proposal(fam, pred, fill, [True, True, False, False, False, True], 1, lo.MFMA) == 3


# ---- pins that come from the paper alone (the oracle was written next to the library's loop, so agreement
# between the two proves little; these fix what both must do)
GOLDEN2 = os.path.join(os.path.dirname(__file__), "golden", "case_study2_profile.txt")


def load_case_study2():
    t = {}
    for line in open(GOLDEN2):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        t[f[0]] = (float(f[1]), float(f[2]))
    return t


def case_study2_reports():
    t = load_case_study2()
    # a memory-bound kernel: one flop per byte, far below the ridge point
    before = report(t["runtime_us"][0], arithmetic_intensity=1.0, pct_hbm_peak=t["memory_pct"][0],
                    pct_mfma_peak=t["compute_pct"][0], occupancy_pct=t["occupancy_pct"][0])
    after = report(t["runtime_us"][1], arithmetic_intensity=1.0, pct_hbm_peak=t["memory_pct"][1],
                   pct_mfma_peak=t["compute_pct"][1], occupancy_pct=50.0)
    return t, before, after


def test_case_study2_profile_is_read_as_the_paper_reads_it():
    t, before, after = case_study2_reports()
    # the table's own arithmetic: 849.50 / 488.96 is the 1.74x of the text
    assert round(t["runtime_us"][0] / t["runtime_us"][1], 2) == 1.74
    # before: nothing is saturated (52 % memory, 6 % compute) -- the remedy the paper applies is a restructured
    # data flow (tiling / staging), not more compute; after: over 90 % of the DRAM peak on a kernel below the
    # ridge is the memory roof; neither profile may be called compute-bound
    assert lo.classify(before, HW) == lo.LATENCY
    assert lo.classify(after, HW) == lo.HBM
    assert lo.MFMA not in (lo.classify(before, HW), lo.classify(after, HW))
    # the same percentages arriving through counters instead of achieved rates give the same reading
    ctr = dict(after, have_counters=1, mfma_busy_pct=t["compute_pct"][1], pct_hbm_peak=0.0, pct_mfma_peak=0.0,
               hbm_read_gbs=HW["hbm_gbs_peak"] * t["memory_pct"][1] / 100.0, hbm_write_gbs=0.0)
    assert lo.classify(ctr, HW) == lo.HBM
    # and the Arbiter takes the 1.74x step (it is far above the 1.05x success bar of Sec. 4.2)
    assert lo.arbiter(after, before, lo.DEFAULT_THETA, True, 0, 1) == lo.ACCEPT


def test_the_two_hints_the_paper_spells_out():
    # Sec. 3.3, Targeted-Refinement-Hint: "memory stalls => improve tiling or staging"
    base = variant(bm=128, bn=128, stages=2, lds=65536)
    stalled = report(100.0, pct_mfma_peak=30.0, pct_hbm_peak=20.0, occupancy_pct=50.0)      # waiting, nothing saturated
    hint = lo.refine_hint(None, stalled, HW)
    assert lo.moves_in_direction(hint, base, variant(bm=128, bn=128, stages=3, lds=98304), 1.0, 1.0)      # deeper staging
    assert lo.moves_in_direction(hint, base, variant(bm=256, bn=256, stages=2, lds=131072), 1.0, 1.0)     # bigger tiles
    assert not lo.moves_in_direction(hint, base, variant(bm=64, bn=64, stages=2, lds=16384), 1.0, 1.0)
    # "low occupancy => adjust register pressure": fewer accumulator registers / less LDS per work-group
    starved = report(100.0, pct_mfma_peak=30.0, pct_hbm_peak=20.0, occupancy_pct=12.5)
    hint = lo.refine_hint(None, starved, HW)
    assert hint != lo.refine_hint(None, stalled, HW)
    assert lo.moves_in_direction(hint, base, variant(bm=64, bn=64, stages=2, lds=16384), 1.0, 1.0)
    assert lo.moves_in_direction(hint, base, variant(bm=128, bn=128, stages=2, lds=32768), 1.0, 1.0)
    assert not lo.moves_in_direction(hint, base, variant(bm=256, bn=256, stages=2, lds=131072), 1.0, 1.0)


def case_study3_hint_sequence(refine, chain):
    """The hints RefineHint gives along the five rounds of Case Study 3, each report carrying the hint it received
    (`chain(report, hint)`), the profile figures taken from the paper's table (a kernel above the ridge: a matrix
    product)."""
    rows = load_case_study3()
    hints, prev = [], None
    for row in rows:
        r = report(row["total_ms"] * 1e3, pct_mfma_peak=row["sm"], pct_hbm_peak=row["mem"], occupancy_pct=row["occ"])
        h = refine(prev, r)
        hints.append(h)
        prev = chain(r, h)
    return hints


def test_case_study3_hints_follow_the_papers_rounds():
    # Sec. 5, Case Study 3, what each round did after the profile of the one before:
    #   round 2: a pre-transposed operand to get coalesced access      -> data movement / staging   (after round 1)
    #   round 3: smaller tiles and fewer stages to lower register use   -> occupancy                 (after round 2, 4 % slower)
    #   round 4: deep pipelining (four stages), full coalescing         -> staging again             (after round 3, slower still)
    #   round 5: configurations with little shared memory, so that several work-groups stay resident -> occupancy (after round 4, the slowest)
    # Every round after the first was slower than the one before it, and each time the paper's next move went the
    # other way between "stage / tile differently" and "make room for more resident work-groups".
    def chain(r, h):
        r = dict(r)
        r["bottleneck"] = h
        return r
    hints = case_study3_hint_sequence(lambda p, r: lo.refine_hint(p, r, HW), chain)
    assert hints[:4] == [lo.LATENCY, lo.OCCUPANCY, lo.LATENCY, lo.OCCUPANCY]
    # the moves the paper made lie in those directions: round 4 (four stages, about 140 KB of shared memory) from
    # round 3's configuration (64 x 128 tiles, two stages); round 5 (under 76 KB, three stages) from round 4's
    r3cfg = variant(bm=64, bn=128, stages=2, lds=32768)
    r4cfg = variant(bm=64, bn=128, stages=4, lds=140 * 1024)
    assert lo.moves_in_direction(hints[2], r3cfg, r4cfg, 1.0, 1.0)
    assert not lo.moves_in_direction(hints[3], r3cfg, r4cfg, 1.0, 1.0)
    r5cfg = variant(bm=64, bn=128, stages=3, lds=76 * 1024)
    assert lo.moves_in_direction(hints[3], r4cfg, r5cfg, 1.0, 1.0)
    assert not lo.moves_in_direction(hints[3], r5cfg, r4cfg, 1.0, 1.0)
    # round 3's smaller tiles from a larger configuration
    assert lo.moves_in_direction(hints[1], variant(bm=128, bn=128, stages=3, lds=98304), r3cfg, 1.0, 1.0)
    # round 5 is faster than round 4: no turn, the hint is what its own figures say
    rows = load_case_study3()
    r4 = report(rows[3]["total_ms"] * 1e3, pct_mfma_peak=rows[3]["sm"], pct_hbm_peak=rows[3]["mem"], occupancy_pct=rows[3]["occ"], bottleneck=hints[3])
    r5 = report(rows[4]["total_ms"] * 1e3, pct_mfma_peak=rows[4]["sm"], pct_hbm_peak=rows[4]["mem"], occupancy_pct=rows[4]["occ"])
    assert lo.refine_hint(r4, r5, HW) == lo.classify(r5, HW)
