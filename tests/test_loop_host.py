"""The library's host-side loop logic (tf_arbiter, tf_refine_hint, tf_proposal_from,
tf_tune_replay) against the plain-Python loop oracle on synthetic reports, plus sanity of
the static cost model. No GPU involved."""
import os
import random

import pytest

from oracle import loop_oracle as lo
from paper_2512_09196_amd import tf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "case_study3_rounds.txt")
REPORT_KEYS = ["status", "parity_ok", "t_med_us", "t_min_us", "grid_fill", "arithmetic_intensity", "pct_mfma_peak",
               "pct_hbm_peak", "occupancy_pct", "have_counters", "mfma_busy_pct", "hbm_read_gbs", "hbm_write_gbs",
               "lds_bank_conflict_pct", "bottleneck"]
VARIANT_KEYS = ["kind", "bm", "bn", "bk", "stages", "split_k", "direct_to_lds", "lds_bytes", "grid"]


def c_report(d):
    r = tf.Report()
    for k in REPORT_KEYS:
        setattr(r, k, d[k])
    return r


def c_variant(d, i):
    v = tf.VariantDesc()
    for k in VARIANT_KEYS:
        setattr(v, k, d[k])
    v.id = i
    v.waves_m = v.waves_n = 2
    v.waves_k = 1
    v.threads = 256
    return v


def hw_dict(h):
    return dict(bf16_tflops_peak=h.bf16_tflops_peak, hbm_gbs_peak=h.hbm_gbs_peak)


def rand_report(rng):
    t = rng.uniform(5, 500)
    return dict(status=rng.choice([0, 0, 0, 0, -2, -3]), parity_ok=rng.choice([1, 1, 1, 0]), t_med_us=t,
                t_min_us=t * rng.choice([0.99, 0.97, 0.8]), grid_fill=rng.uniform(0.1, 1.0),
                arithmetic_intensity=rng.choice([16.0, 85.0, 500.0, 1700.0]), pct_mfma_peak=rng.uniform(0, 95),
                pct_hbm_peak=rng.uniform(0, 95), occupancy_pct=rng.choice([12.5, 25.0, 37.5, 50.0]),
                have_counters=rng.randint(0, 1), mfma_busy_pct=rng.uniform(0, 100), hbm_read_gbs=rng.uniform(0, 6000),
                hbm_write_gbs=rng.uniform(0, 2000), lds_bank_conflict_pct=rng.uniform(0, 12),
                bottleneck=rng.choice([0, 0, 1, 2, 3, 4, 5, 5, 6, 6]))       # the hint the report received (0: none)


def rand_variant(rng, kind=None):
    bm, bn = rng.choice([32, 64, 128, 256]), rng.choice([64, 128, 256])
    st = rng.choice([2, 3, 4])
    return dict(kind=rng.choice([1, 2, 2, 2]) if kind is None else kind, bm=bm, bn=bn, bk=rng.choice([32, 64, 64, 128]), stages=st,
                split_k=rng.choice([1, 2, 4, 8]), direct_to_lds=rng.randint(0, 1), lds_bytes=st * (bm + bn) * 128,
                grid=rng.choice([16, 64, 128, 256, 688, 1024, 2752]))


def test_arbiter_and_hint_match_oracle_on_random_reports():
    rng = random.Random(11)
    hw = tf.hw_nominal()
    th_c = tf.theta_default()
    th = dict(first_accept_speedup=th_c.first_accept_speedup, later_accept_gain=th_c.later_accept_gain,
              robust_spread=th_c.robust_spread, patience=th_c.patience, max_rounds=th_c.max_rounds)
    assert th == lo.DEFAULT_THETA
    seen_dec, seen_cls = set(), set()
    for _ in range(3000):
        a, b, pv = rand_report(rng), rand_report(rng), rand_report(rng)
        b["status"], b["parity_ok"] = 0, 1
        base, stall, rnd = rng.randint(0, 1), rng.randint(0, 4), rng.randint(1, 8)
        want = lo.arbiter(a, b, th, bool(base), stall, rnd)
        got = tf.arbiter(c_report(a), c_report(b), th_c, bool(base), stall, rnd)
        assert got == want
        seen_dec.add(got)
        prev = None if rng.random() < 0.3 else pv
        want = lo.refine_hint(prev, a, hw_dict(hw))
        got = tf.refine_hint(c_report(prev) if prev else None, c_report(a), hw)
        assert got == want
        seen_cls.add(got)
    assert seen_dec == {0, 1, 2} and seen_cls == set(range(7))


def test_proposal_matches_oracle_on_random_families():
    rng = random.Random(12)
    hw = tf.hw_nominal()
    for _ in range(400):
        n = rng.randint(1, 25)
        fam = [rand_variant(rng, kind=0)] + [rand_variant(rng) for _ in range(n - 1)]
        cfam = [c_variant(d, i) for i, d in enumerate(fam)]
        pred = [rng.choice([10.0, 20.0, 30.0, rng.uniform(1, 100)]) for _ in range(n)]
        fill = [tf.grid_fill(hw, v) for v in cfam]
        tried = [rng.random() < 0.4 for _ in range(n)]
        for hint in range(7):
            base = rng.randrange(n)
            assert tf.proposal_from(hw, cfam, pred, tried, base, hint) == lo.proposal(fam, pred, fill, tried, base, hint)


def test_tune_replay_matches_oracle_loop():
    rng = random.Random(13)
    hw = tf.hw_nominal()
    th = tf.theta_default()
    desc = tf.ProblemDesc(2048, 2048, 2048, 2048, 2048, 2048, 0, 0)
    for _ in range(150):
        n = rng.randint(1, 30)
        fam = [rand_variant(rng, kind=0)] + [rand_variant(rng) for _ in range(n - 1)]
        reps = [rand_report(rng) for _ in range(n)]
        reps[0]["status"], reps[0]["parity_ok"] = 0, 1
        cfam = [c_variant(d, i) for i, d in enumerate(fam)]
        pred = [tf.predict_us(desc, hw, v) for v in cfam]
        fill = [tf.grid_fill(hw, v) for v in cfam]
        k_star, r_star, log = lo.optimize(fam, pred, fill, lambda i: reps[i], hw_dict(hw))
        bv, best, clog = tf.tune_replay(desc, hw, cfam, [c_report(r) for r in reps], th)
        assert bv == k_star
        assert best.t_med_us == r_star["t_med_us"]
        assert [r.variant_id for r in clog] == [r["variant_id"] for r in log]
        assert [r.bottleneck for r in clog] == [r["bottleneck"] for r in log]
        assert len(clog) <= 9


def test_case_study3_replay_through_the_library():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    hw, th = tf.hw_nominal(), tf.theta_default()
    desc = tf.ProblemDesc(1024, 1024, 1024, 1024, 1024, 1024, 0, 0)
    reps = []
    for f in rows:
        d = rand_report(random.Random(0))
        d.update(status=0, parity_ok=1, t_med_us=float(f[1]) * 1e3, t_min_us=float(f[1]) * 990.0, grid_fill=1.0,
                 have_counters=0, pct_mfma_peak=float(f[5]), pct_hbm_peak=float(f[4]), occupancy_pct=float(f[6]),
                 arithmetic_intensity=1000.0)
        reps.append(c_report(d))
    fam = [c_variant(dict(kind=0, bm=4, bn=64, bk=1, stages=0, split_k=1, direct_to_lds=0, lds_bytes=0, grid=4096), 0)]
    fam += [c_variant(dict(kind=2, bm=128, bn=128, bk=64, stages=2, split_k=1, direct_to_lds=1, lds_bytes=65536, grid=64), i)
            for i in range(1, 5)]
    bv, best, log = tf.tune_replay(desc, hw, fam, reps, th)
    assert bv == 0 and best.t_med_us == pytest.approx(9690.0)
    assert len(log) == 5     # baseline + four rounds: the fourth miss in a row ends the loop
    assert sorted(r.variant_id for r in log) == [0, 1, 2, 3, 4]


def test_cost_model_orders_the_obvious_cases():
    hw = tf.hw_nominal()
    with tf.Problem(4096, 11008, 4096) as p:
        vs = p.variants()
        pred = {v.name.decode(): tf.predict_us(p.desc, hw, v) for v in vs}
    assert pred["naive_1elem_per_thread"] > pred["mfma32_direct_1wave"] > min(pred.values())
    best = min(pred, key=pred.get)
    assert best.startswith("lds_256x256"), best          # big tiles win on the large compute-bound shape
    assert 146.0 < pred[best] < 400.0                     # never below the MFMA roof
    with tf.Problem(16, 8192, 8192) as p:
        vs = p.variants()
        pr = [tf.predict_us(p.desc, hw, v) for v in vs]
        best = vs[pr.index(min(pr))]
    # the skinny shape needs narrow tiles or K slices: at least one work-group per compute unit
    assert best.kind == tf.TF_KIND_MFMA_LDS and best.grid >= hw.cus
    assert min(pr) >= 16.8                                # never below the HBM roof
    # resident work-groups: 256x256 tiles use the whole register file and most of the LDS;
    # 64x64 tiles are limited by LDS only (three 16 KB stages -> 3, two -> 4 by registers)
    with tf.Problem(2048, 2048, 2048) as p:
        for v in p.variants():
            if v.kind == tf.TF_KIND_MFMA_LDS and v.bm == 256 and v.bn == 256:
                assert tf.resident_wgs(hw, v) == 1
            if v.kind == tf.TF_KIND_MFMA_LDS and v.bm == 64 and v.bn == 64 and v.bk == 64:
                assert tf.resident_wgs(hw, v) == (3 if v.stages == 3 else 4)
            f = tf.grid_fill(hw, v)
            assert 0.0 < f <= 1.0


def test_case_study2_and_the_papers_two_hints_through_the_library():
    """The same paper-fixed pins as in test_loop_oracle.py, applied to the library's own functions: the
    profile table of Case Study 2 (Sec. 5) and the two example hints of Sec. 3.3."""
    t = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "case_study2_profile.txt")):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            t[f[0]] = (float(f[1]), float(f[2]))
    hw, th = tf.hw_nominal(), tf.theta_default()

    def rep(t_us, mem, comp, occ, intensity=1.0):
        d = rand_report(random.Random(0))
        d.update(status=0, parity_ok=1, t_med_us=t_us, t_min_us=0.99 * t_us, grid_fill=1.0, have_counters=0,
                 pct_mfma_peak=comp, pct_hbm_peak=mem, occupancy_pct=occ, arithmetic_intensity=intensity,
                 lds_bank_conflict_pct=0.0)
        return c_report(d)
    before = rep(t["runtime_us"][0], t["memory_pct"][0], t["compute_pct"][0], t["occupancy_pct"][0])
    after = rep(t["runtime_us"][1], t["memory_pct"][1], t["compute_pct"][1], 50.0)
    assert tf.refine_hint(None, before, hw) == tf.TF_BN_LATENCY
    assert tf.refine_hint(None, after, hw) == tf.TF_BN_HBM
    assert tf.arbiter(after, before, th, True, 0, 1) == tf.TF_DEC_ACCEPT
    # "memory stalls => improve tiling or staging", "low occupancy => adjust register pressure":
    # the next proposal from a 128x128 two-buffer kernel
    fam = [c_variant(dict(kind=0, bm=4, bn=64, bk=1, stages=0, split_k=1, direct_to_lds=0, lds_bytes=0, grid=4096), 0),
           c_variant(dict(kind=2, bm=128, bn=128, bk=64, stages=2, split_k=1, direct_to_lds=1, lds_bytes=65536, grid=256), 1),
           c_variant(dict(kind=2, bm=128, bn=128, bk=64, stages=3, split_k=1, direct_to_lds=1, lds_bytes=98304, grid=256), 2),
           c_variant(dict(kind=2, bm=64, bn=64, bk=64, stages=2, split_k=1, direct_to_lds=1, lds_bytes=32768, grid=1024), 3)]
    pred = [1000.0, 10.0, 20.0, 20.0]
    tried = [True, True, False, False]
    stalled = rep(100.0, 20.0, 30.0, 50.0, intensity=1000.0)
    starved = rep(100.0, 20.0, 30.0, 12.5, intensity=1000.0)
    assert tf.proposal_from(hw, fam, pred, tried, 1, tf.refine_hint(None, stalled, hw)) == 2     # deeper staging
    assert tf.proposal_from(hw, fam, pred, tried, 1, tf.refine_hint(None, starved, hw)) == 3     # smaller tile, less LDS


def test_cost_model_on_shapes_it_was_not_fitted_on():
    """The static cost model behind Proposal against recorded launch times of the tile-kernel variants on eight
    shapes that took no part in fitting its constants: its first pick is within 10 % of the fastest variant on
    every shape and within 3 % on average, the best of its first five (what the loop measures before it may stop)
    within 2 % on every shape, and the predicted time of the variants that matter is off by less than 15 % at
    the median."""
    import json, os
    import numpy as np
    rec = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "measured_variant_times_validation_shapes.json")))
    hw = tf.hw_nominal()
    picks, firsts = [], []
    for shape, times in rec["shapes"].items():
        M, N, K = (int(x) for x in shape.split("x"))
        with tf.Problem(M, N, K) as p:
            vs = [v for v in p.variants() if v.kind in (tf.TF_KIND_MFMA_LDS, tf.TF_KIND_MFMA_STREAM)]
            pred = np.array([tf.predict_us(p.desc, hw, v) for v in vs])
        names = [v.name.decode() for v in vs]
        best = min(times.values())
        order = np.argsort(pred, kind="stable")
        first_five = [times.get(names[i]) for i in order[:5]]
        assert first_five[0] is not None, "%s: the first pick %s is not among the variants within 1.6x of the best" % (shape, names[order[0]])
        picks.append(first_five[0] / best)
        firsts.append(min(t for t in first_five if t is not None) / best)
        err = [abs(pred[i] / times[n] - 1.0) for i, n in enumerate(names) if n in times and times[n] <= 1.2 * best]
        assert np.median(err) < 0.15, (shape, float(np.median(err)))
    assert max(picks) <= 1.10 and float(np.mean(picks)) <= 1.03, picks
    assert max(firsts) <= 1.02, firsts


def test_case_study3_hint_sequence_through_the_library():
    """The same pin as in test_loop_oracle.py (the hints behind the rounds of the paper's Case Study 3: staging,
    occupancy, staging, occupancy), through tf_refine_hint with every report carrying the hint it received."""
    from test_loop_oracle import case_study3_hint_sequence
    hw = tf.hw_nominal()

    def chain(r, h):
        r = dict(r)
        r["bottleneck"] = h
        return r

    def refine(prev, r):
        r = dict(r)
        r.setdefault("bottleneck", 0)
        return tf.refine_hint(c_report(prev) if prev else None, c_report(r), hw)

    hints = case_study3_hint_sequence(refine, chain)
    assert hints[:4] == [tf.TF_BN_LATENCY, tf.TF_BN_OCCUPANCY, tf.TF_BN_LATENCY, tf.TF_BN_OCCUPANCY]
    assert (tf.TF_BN_LATENCY, tf.TF_BN_OCCUPANCY) == (lo.LATENCY, lo.OCCUPANCY)
