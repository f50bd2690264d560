"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each test names the passage of
Lowery & Langou it relies on.
"""
from __future__ import annotations

import heapq
import math
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import oracle as O
import prs_inputs
from schedule_validator import validate

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
COSTS = [(0, 1, 0), (0, 1, 1), (1, 1, 0), (1, 1, 1), (2, 1, 1), (4, 1, 0), (3, 2, 5)]


# --------------------------------------------------------------------------- segmentation
def test_segmentation_cases():
    # Section 2: equal sizes, the last one possibly smaller
    assert O.segmentation(10, 3) == (3, 4, 2)
    assert O.segmentation(10, 4) == (4, 3, 1)
    assert O.segmentation(10, 6) == (5, 2, 2)          # 6 segments asked, 5 needed
    assert O.segmentation(3, 8) == (3, 1, 1)           # never more segments than elements
    assert O.segmentation(12, 4) == (4, 3, 3)
    assert O.segmentation(1, 1) == (1, 1, 1)
    for m in range(1, 60):
        for qr in range(1, 70):
            q, sz, last = O.segmentation(m, qr)
            assert 1 <= last <= sz and (q - 1) * sz + last == m and q <= qr and q <= m
            assert list(O.equi_sizes(m, qr)) == [sz] * (q - 1) + [last]


# --------------------------------------------------------------------------- uni-greedy
def _multiset_uni(p, c, g):
    """Independent restatement of Algorithm 1 on values only: the two smallest
    ready times v1 <= v2 are replaced by v2+c (leaves) and v2+c+g (stays)."""
    x = [0] * p
    for ck, gk in zip(c, g):
        heap = list(x)
        heapq.heapify(heap)
        gone = []
        while len(heap) > 1:
            heapq.heappop(heap)
            v2 = heapq.heappop(heap)
            gone.append(v2 + ck)
            heapq.heappush(heap, (v2 + ck) + gk)
        x = gone + heap
    return max(x)


def test_uni_single_segment_is_binomial():
    # Section 5.2: with one segment uni-greedy "is exactly the binomial algorithm";
    # Table I: ceil(log2 p) (alpha + beta m + gamma m)
    for p in range(2, 71):
        for a, b, g in COSTS:
            for m in (1, 7):
                s = O.uni_greedy(p, [m], a, b, g)
                L = math.ceil(math.log2(p))
                assert s.T == L * (a + b * m + g * m)
                assert s.T == O.binomial_construct(p, m, a, b, g)
                assert s.T == O.closed_forms(O.UNI, p, 1, m, m, a, b, g)["binomial"]


def test_uni_first_segment_takes_log_rounds():
    # Section 5.2, last paragraph: the first segment needs ceil(log2 p) steps
    for p in (5, 16, 33, 100):
        s = O.uni_greedy(p, [1] * 4, 3, 1, 2)
        first = s.seg == 0
        done = (s.t[first] + 4 + 2)[s.dst[first] == 0].max()
        assert done == math.ceil(math.log2(p)) * 6


@pytest.mark.parametrize("p", [2, 3, 4, 5, 6])
def test_uni_matches_exhaustive_optimum(p):
    # Theorem 1: minimal among all algorithms that reduce the segments in order
    qmax = 4 if p <= 5 else 3
    for q in range(1, qmax + 1):
        for a in (0, 1, 2, 4):
            for g in (0, 1):
                best = O.exhaustive_uni(p, [1] * q, a, 1, g)
                assert best == O.uni_greedy(p, [1] * q, a, 1, g).T, (p, q, a, g)


def test_uni_matches_exhaustive_unequal_segments():
    # Theorem 1 holds "for any segmentation" (Section 2)
    for p, sizes, a, b, g in [(5, [3, 1, 2], 1, 1, 1), (4, [2, 5, 1, 1], 2, 1, 1), (5, [1, 4], 0, 1, 2),
                              (4, [6, 1, 3], 3, 2, 0), (3, [2, 2, 1, 4], 1, 3, 1)]:
        assert O.exhaustive_uni(p, sizes, a, b, g) == O.uni_greedy(p, sizes, a, b, g).T


def test_exhaustive_search_beats_a_worse_rule():
    # the search itself must be able to tell schedules apart: a chain is slower
    p, q, a, b, g = 6, 3, 1, 1, 1
    assert O.exhaustive_uni(p, [1] * q, a, b, g) < O.pipeline_construct(p, [1] * q, a, b, g)


def test_uni_root_holds_maximum_and_validates():
    # proof of Theorem 1: x_0 = max(X_{q+1}); machine model of Section 2
    rng = np.random.default_rng(5)
    for _ in range(60):
        p = int(rng.integers(2, 40)); q = int(rng.integers(1, 7))
        sizes = rng.integers(1, 6, size=q)
        a, b, g = int(rng.integers(0, 5)), int(rng.integers(1, 3)), int(rng.integers(0, 3))
        s = O.uni_greedy(p, sizes, a, b, g)
        assert s.T == s.x_final.max() == s.x_final[0]
        c = [a + b * int(z) for z in sizes]; gg = [g * int(z) for z in sizes]
        T, problems = validate("uni", p, c, gg, s.seg, s.src, s.dst, s.t)
        assert not problems, problems[:3]
        assert T == s.T == _multiset_uni(p, c, gg)
        assert np.all(np.diff(s.seg) >= 0) and np.all(s.src != 0)
        for k in range(q):                       # start times never decrease within a segment
            assert np.all(np.diff(s.t[s.seg == k]) >= 0)


def test_uni_fp64_matches_value_only_restatement():
    cfg = prs_inputs.uni_sweep(400)
    for i in range(0, 400, 7):
        p, m, qr = int(cfg.p[i]), int(cfg.m[i]), int(cfg.q_req[i])
        if p * p * qr > 3e7:
            continue
        sizes = O.equi_sizes(m, qr)
        a, b, g = float(cfg.alpha[i]), float(cfg.beta[i]), float(cfg.gamma[i])
        s = O.uni_greedy(p, sizes, a, b, g, "f64", want_schedule=False)
        c = [a + b * float(z) for z in sizes]; gg = [g * float(z) for z in sizes]
        assert s.T == _multiset_uni(p, c, gg)


def test_uni_value_only_form_equals_algorithm_1():
    """The heap form (ready times only) against Algorithm 1 with its two scans: the whole integer sweep, the
    segmentations of Table IV's rows (unequal sizes), fp64 costs with rounding ties; and, where the two scans
    would take too long, against what the paper fixes for any p: one segment is the binomial tree (Section 5.2,
    Table I), Theorem 1 and Table II."""
    cfg = prs_inputs.tiny_sweep()
    for i in range(len(cfg)):
        p, q, a, g = int(cfg.p[i]), int(cfg.q_req[i]), int(cfg.alpha[i]), int(cfg.gamma[i])
        assert O.uni_greedy_time(p, [1] * q, a, 1, g) == O.uni_greedy(p, [1] * q, a, 1, g, want_schedule=False).T
    for p, a, g, _, equi, opts in _table4_rows():
        if p > 200:
            continue
        for sizes in [equi] + opts[:2]:
            assert O.uni_greedy_time(p, list(sizes), a, 1, g) == O.uni_greedy(p, list(sizes), a, 1, g, want_schedule=False).T
    full = prs_inputs.uni_sweep(600)
    for i in range(0, 600, 5):
        p, m, qr = int(full.p[i]), int(full.m[i]), int(full.q_req[i])
        if p * p * qr > 2e7:
            continue
        sizes = O.equi_sizes(m, qr)
        a, b, g = float(full.alpha[i]), float(full.beta[i]), float(full.gamma[i])
        assert O.uni_greedy_time(p, sizes, a, b, g, "f64") == O.uni_greedy(p, sizes, a, b, g, "f64", want_schedule=False).T
    for al, be, ga in [(1.0, 0.0, 2.0 ** -52), (0.75, 2.0 ** -54, 2.0 ** -51)]:       # sums that collide in rounding
        for p in (5, 17, 64):
            sizes = O.equi_sizes(29, 9)
            assert O.uni_greedy_time(p, sizes, al, be, ga, "f64") == O.uni_greedy(p, sizes, al, be, ga, "f64", want_schedule=False).T
    for p in (1024, 4097, 40000, 65536):
        L = math.ceil(math.log2(p))
        assert O.uni_greedy_time(p, [1000], 7, 2, 3) == L * (7 + 2000 + 3000)
        T = O.uni_greedy_time(p, [5] * 12, 3, 1, 2)
        cf = O.closed_forms(O.UNI, p, 12, 60, 5, 3, 1, 2)
        assert L * 3 <= T <= min(cf["pipeline"], cf["binary"]) and T >= 2 * 60 * 1 and T >= (L + 11) * 3


def test_uni_no_slower_than_in_order_baselines_and_above_bounds():
    # pipeline and binary reduce segments in order, so Theorem 1 bounds uni-greedy by both
    # (Table I); Table II gives the lower bounds of any reduction.
    for p in (4, 5, 7, 8, 15, 16, 31, 64, 129):
        for q in (1, 2, 3, 5, 8, 13):
            for a, b, g in COSTS:
                s = O.uni_greedy(p, [1] * q, a, b, g, want_schedule=False)
                cf = O.closed_forms(O.UNI, p, q, q, 1, a, b, g)
                assert s.T <= O.pipeline_construct(p, [1] * q, a, b, g) <= cf["pipeline"]
                assert s.T <= cf["binary"]
                L = math.ceil(math.log2(p))
                assert s.T >= L * a and s.T >= 2 * q * b and s.T * p >= (p - 1) * q * g


def test_uni_p64_curve_facts():
    # Section 5.2, Figure 4: p = 64, alpha = 10, beta = 1, gamma = 0, every algorithm at its
    # best segment size: greedy = binomial for small m (the text says m < 64), gains up to about
    # 50 % over the best standard algorithm for mid-size m, pipeline catches up for large m.
    p, a, b, g = 64, 10, 1, 0

    def best(fn, m):
        # every segment count for small m, segment sizes 2^i (Section 7) beyond
        counts = range(1, m + 1) if m <= 64 else [m >> i for i in range(0, m.bit_length())]
        return min(fn(O.equi_sizes(m, k), O.segmentation(m, k)) for k in counts)

    ratios = {}
    for m in (4, 16, 32, 64, 256, 1024, 4096):
        tg = best(lambda sizes, sg: O.uni_greedy(p, sizes, a, b, g, want_schedule=False).T, m)
        tb = O.closed_forms(O.UNI, p, 1, m, m, a, b, g)["binomial"]
        tp = best(lambda sizes, sg: O.closed_forms(O.UNI, p, sg[0], m, sg[1], a, b, g)["pipeline"], m)
        ty = best(lambda sizes, sg: O.closed_forms(O.UNI, p, sg[0], m, sg[1], a, b, g)["binary"], m)
        ratios[m] = (tb / tg, tp / tg, ty / tg)
    assert ratios[4][0] == 1.0 and ratios[16][0] == 1.0          # one segment is best: binomial
    assert 1.0 < ratios[32][0] < ratios[64][0] < 1.35             # the curves part around m = 64
    mid = [min(ratios[m]) for m in (256, 1024)]
    assert all(1.35 <= r <= 1.6 for r in mid), mid
    assert ratios[4096][1] < ratios[1024][1] < ratios[256][1]       # pipeline approaches greedy
    assert all(min(r) >= 1.0 for r in ratios.values())               # never beaten (Theorem 1)


# --------------------------------------------------------------------------- Table IV
def _compositions(m):
    for bits in range(1 << (m - 1)):
        parts, cur = [], 1
        for i in range(m - 1):
            if bits >> i & 1:
                parts.append(cur); cur = 1
            else:
                cur += 1
        parts.append(cur)
        yield tuple(parts)


def _table4_rows():
    rows = []
    with open(os.path.join(GOLDEN, "table4_unequal_segmentation.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p, a, g, ratio, equi, opt = line.split()
            rows.append((int(p), int(a), int(g), ratio, tuple(map(int, equi.split(","))),
                         sorted(tuple(map(int, s.split(","))) for s in opt.split(";"))))
    return rows


def test_table4_unequal_segmentation_rows():
    """Section 8, Table IV: for each printed (p, alpha, gamma) the oracle must find exactly the
    printed set of optimal segmentations of m = 10, the printed best equi-segmentation and the
    printed ratio to four decimals.  The table's equi-segmentations are those obtained from a
    segment count (sizes ceil(10/k): 10, 5, 4, 3, 2, 1)."""
    comps = list(_compositions(10))
    assert len(comps) == 512                                  # "a total of 512 possible segmentations"
    equi = sorted({tuple(int(v) for v in O.equi_sizes(10, k)) for k in range(1, 11)})
    rows = _table4_rows()
    assert len(rows) == 61                                    # "61 out of 986 experiments"

    def check(row):
        p, a, g, ratio, equi_printed, opt_printed = row
        T = {c: O.uni_greedy(p, list(c), a, 1, g, want_schedule=False).T for c in comps}
        best = min(T.values())
        opt = sorted(c for c in comps if T[c] == best)
        be = min(T[c] for c in equi)
        ok = (opt == opt_printed and f"{be / best:.4f}" == ratio and T[equi_printed] == be
              and not any(c in equi for c in opt))
        return ok, be / best

    with ThreadPoolExecutor(8) as ex:
        res = list(ex.map(check, rows))
    bad = [rows[i][:3] for i, (ok, _) in enumerate(res) if not ok]
    assert not bad, bad
    gains = [r - 1.0 for _, r in res]
    assert f"{max(gains) * 100:.1f}" == "7.3"                 # "maximum improvement ... 7.3%"
    assert f"{sum(gains) / len(gains) * 100:.1f}" == "2.0"    # "average improvement was 2.0%"


def test_unequal_segmentation_summary_matches_table4_rows():
    """Section 8 / Table IV through oracle.unequal_segmentation (the per-problem summary the GPU entry point
    also returns): for printed rows the ratio, the best equi-segmentation, the number of optimal
    segmentations and the first of them in cut-pattern order are the printed ones and no kind of
    equi-segmentation is optimal; an experiment the table does not list has ratio 1."""
    comps = O.compositions(10)
    assert len(comps) == 512 and comps[0] == (10,) and comps[511] == (1,) * 10 and comps[1] == (1, 9)
    rows = [r for r in _table4_rows() if r[0] <= 48]
    assert len(rows) >= 12
    for p, a, g, ratio, equi_printed, opt_printed in rows:
        r = O.unequal_segmentation(p, 10, a, 1, g)
        assert f"{r['T_equi'] / r['T_best']:.4f}" == ratio
        assert r["n_best"] == len(opt_printed) and comps[r["cuts_best"]] in opt_printed
        assert r["cuts_best"] == min(comps.index(c) for c in opt_printed)
        assert r["T_all"][comps.index(equi_printed)] == r["T_equi"] and r["equi_optimal"] == 0
    listed = {(p, a, g) for p, a, g, *_ in _table4_rows()}
    for p, a, g in [(4, 5, 0), (6, 20, 1), (8, 100, 0), (16, 1000, 1)]:
        assert (p, a, g) not in listed
        r = O.unequal_segmentation(p, 10, a, 1, g)
        assert r["T_equi"] == r["T_best"] and r["equi_optimal"] == 3
    # one unit: a single segmentation, which is the equi one
    r = O.unequal_segmentation(5, 1, 2, 1, 1)
    assert (r["n_best"], r["cuts_best"], r["equi_optimal"]) == (1, 0, 3) and r["T_best"] == 3 * (2 + 1 + 1)


def test_pipeline_is_optimised_by_equal_segments():
    # Section 8: "For the pipeline algorithm, all experiments were optimized by equi-segmentation"
    comps = list(_compositions(10))
    equi = [c for c in comps if all(x == c[0] for x in c[:-1]) and c[-1] <= c[0]]
    for p in (4, 6, 16, 48):
        for a in (0, 1, 3, 10, 100):
            for g in (0, 1):
                T = {c: O.pipeline_construct(p, list(c), a, 1, g) for c in comps}
                assert min(T[c] for c in equi) == min(T.values())


# --------------------------------------------------------------------------- bi-greedy
def test_bi_worked_example_matches_reverse_optimal_broadcast():
    # Figure 8 (p = 16, 5 segments, tcomm = 2, tcomp = 1) "matches the optimal broadcast":
    # Table III gives (ceil(log2 16) + 5 - 1) * 3 = 24
    for mode in (O.MODE_LITERAL, O.MODE_EVENT, O.MODE_EVENT | O.MODE_PRUNE):
        s = O.bi_greedy(16, [1] * 5, 1, 1, 1, mode=mode)
        assert s.T == 24 and s.status == 0
    assert O.closed_forms(O.BI, 16, 5, 5, 1, 1, 1, 1)["revopt"] == 24


def test_bi_conjecture_and_validity_equal_segments():
    # Section 6.2: "for all p and q the bi-greedy algorithm has the same time complexity as a
    # reverse optimal broadcast": (ceil(log2 p) + q - 1)(alpha + beta s + gamma s)  (Table III)
    for p in range(2, 41):
        for q in range(1, 9):
            for a, b, g in COSTS:
                s = O.bi_greedy(p, [1] * q, a, b, g, mode=O.MODE_EVENT | O.MODE_PRUNE)
                c, gg = a + b, g
                assert s.status == 0
                assert s.T == (math.ceil(math.log2(p)) + q - 1) * (c + gg), (p, q, a, b, g)
                T, problems = validate("bi", p, [c] * q, [gg] * q, s.seg, s.src, s.dst, s.t)
                assert not problems, (p, q, a, b, g, problems[:3])
                assert T == s.T == s.root_done.max()
                assert np.all(np.diff(s.t) >= 0)


def test_bi_time_advance_and_pruning_do_not_change_results():
    # Algorithm 2 "assumes a discrete time step"; jumping to the next time a port frees, and
    # leaving the segment loop once no pair can form, must reproduce it pair for pair.
    cases = []
    cfg = prs_inputs.tiny_sweep()
    for i in range(0, len(cfg), 3):
        cases.append((int(cfg.p[i]), [1] * int(cfg.q_req[i]), int(cfg.alpha[i]), 1, int(cfg.gamma[i])))
    rng = np.random.default_rng(11)
    for _ in range(80):                                       # ragged and unequal sizes as well
        p = int(rng.integers(2, 30)); m = int(rng.integers(1, 40)); qr = int(rng.integers(1, 9))
        cases.append((p, O.equi_sizes(m, qr), int(rng.integers(0, 6)), int(rng.integers(1, 3)), int(rng.integers(0, 3))))
    for p, sizes, a, b, g in cases:
        ref = O.bi_greedy(p, sizes, a, b, g, mode=O.MODE_LITERAL)
        for mode in (O.MODE_EVENT, O.MODE_EVENT | O.MODE_PRUNE, O.MODE_LITERAL | O.MODE_PRUNE):
            s = O.bi_greedy(p, sizes, a, b, g, mode=mode)
            assert s.T == ref.T and s.status == ref.status == 0
            for f in ("src", "dst", "seg", "t", "root_done"):
                assert np.array_equal(getattr(s, f), getattr(ref, f)), (p, list(sizes), a, b, g, mode, f)


def test_bi_ragged_last_segment_is_valid_and_sandwiched():
    """Section 2 allows a smaller last segment and forbids communication to overlap computation.  Every such
    schedule passes the validator with all rules on, and its time lies between two round counts: the root
    takes the q segments in one after the other and the segment it takes in last still needs ceil(log2 p)
    rounds of its own size (the bound of Table III's broadcast-based row, turned round, with each segment's
    own round time): (q-1) r + L r_last <= T; and T <= (L+q-2) r + L r_last, the first q-1 segments run to
    completion as Table III says and the last one after them on its own (an observation on this oracle, not a
    statement of the paper)."""
    rng = np.random.default_rng(3)
    seen = 0
    for _ in range(260):
        p = int(rng.integers(2, 90)); m = int(rng.integers(2, 200)); qr = int(rng.integers(2, 24))
        a, b, g = int(rng.integers(0, 50)), int(rng.integers(1, 4)), int(rng.integers(0, 4))
        q, sz, last = O.segmentation(m, qr)
        if last == sz:
            continue
        seen += 1
        sizes = O.equi_sizes(m, qr)
        s = O.bi_greedy(p, sizes, a, b, g, mode=O.MODE_EVENT | O.MODE_PRUNE)
        c = [a + b * int(z) for z in sizes]; gg = [g * int(z) for z in sizes]
        T, problems = validate("bi", p, c, gg, s.seg, s.src, s.dst, s.t)
        assert not problems and T == s.T, (p, list(sizes), a, b, g, problems[:3])
        L = math.ceil(math.log2(p)); r = c[0] + gg[0]; rl = c[-1] + gg[-1]
        assert (q - 1) * r + L * rl <= s.T <= (L + q - 2) * r + L * rl, (p, list(sizes), a, b, g, s.T)
    assert seen >= 150


def test_bi_section2_exclusion_matters_only_for_a_smaller_last_segment():
    """The exclusion that keeps a combine out of a running send (Section 2) never fires with equal segments:
    Algorithm 2 alone gives the same pairs.  With a smaller last segment Algorithm 2 alone overlaps a send
    and a combine in many cases, the oracle in none."""
    for p in (2, 3, 7, 16, 33):
        for q in (1, 2, 5, 8):
            for a, b, g in COSTS:
                s = O.bi_greedy(p, [3] * q, a, b, g, mode=O.MODE_EVENT)
                w = O.bi_greedy(p, [3] * q, a, b, g, mode=O.MODE_EVENT | O.MODE_LISTING_ONLY)
                for f in ("src", "dst", "seg", "t"):
                    assert np.array_equal(getattr(s, f), getattr(w, f))
    rng = np.random.default_rng(8)
    overlapping = 0
    for _ in range(120):
        p = int(rng.integers(3, 40)); q = int(rng.integers(2, 9)); sz = int(rng.integers(2, 9)); last = int(rng.integers(1, sz))
        a, b, g = int(rng.integers(0, 20)), int(rng.integers(1, 3)), int(rng.integers(1, 3))
        sizes = [sz] * (q - 1) + [last]
        c = [a + b * z for z in sizes]; gg = [g * z for z in sizes]
        w = O.bi_greedy(p, sizes, a, b, g, mode=O.MODE_EVENT | O.MODE_LISTING_ONLY)
        _, problems = validate("bi", p, c, gg, w.seg, w.src, w.dst, w.t)
        assert all("communication overlaps computation" in x for x in problems)
        overlapping += bool(problems)
        s = O.bi_greedy(p, sizes, a, b, g, mode=O.MODE_EVENT)
        assert not validate("bi", p, c, gg, s.seg, s.src, s.dst, s.t)[1]
    assert overlapping >= 30


def test_bi_fp64_schedules_are_valid_whatever_the_rounding():
    """Seconds instead of integer units: event times that are equal on paper can differ in the last bit.  The
    comparisons of Algorithm 2 between two transfers of the same segment size are decided by their start
    times, so every schedule still passes the validator (equal and smaller last segment alike)."""
    cfg = prs_inputs.uni_sweep(5000)
    seen = ragged = 0
    for i in range(0, 5000):
        p, m, qr = int(cfg.p[i]), int(cfg.m[i]), int(cfg.q_req[i])
        q, sz, last = O.segmentation(m, qr)
        if (p - 1) * q > 2500 or q < 2:
            continue
        a, b, g = float(cfg.alpha[i]), float(cfg.beta[i]), float(cfg.gamma[i])
        sizes = O.equi_sizes(m, qr)
        s = O.bi_greedy(p, sizes, a, b, g, "f64", mode=O.MODE_EVENT | O.MODE_PRUNE)
        c = [a + b * float(z) for z in sizes]; gg = [g * float(z) for z in sizes]
        T, problems = validate("bi", p, c, gg, s.seg, s.src, s.dst, s.t)
        assert s.status == 0 and not problems and T == s.T, (i, p, q, sz, last, problems[:2])
        seen += 1; ragged += last != sz
    assert seen >= 1500 and ragged >= 800


def test_bi_fp64_equals_round_count_when_segments_are_equal():
    cfg = prs_inputs.uni_sweep(3000)
    seen = 0
    for i in range(3000):
        p, m, qr = int(cfg.p[i]), int(cfg.m[i]), int(cfg.q_req[i])
        q, sz, last = O.segmentation(m, qr)
        if last != sz or p * q > 20000:
            continue
        a, b, g = float(cfg.alpha[i]), float(cfg.beta[i]), float(cfg.gamma[i])
        s = O.bi_greedy(p, O.equi_sizes(m, qr), a, b, g, "f64", mode=O.MODE_EVENT | O.MODE_PRUNE, want_schedule=False)
        rounds = math.ceil(math.log2(p)) + q - 1
        assert s.status == 0 and s.T == pytest.approx(rounds * ((a + b * sz) + g * sz), rel=1e-12)
        seen += 1
    assert seen >= 20


# --------------------------------------------------------------------------- closed forms
def test_closed_forms_reproduce_the_tables_optimal_rows():
    # Tables I and III print, next to each time formula, the optimal segment size and the time at
    # that size.  Parameters are chosen so that s_opt is an integer dividing m; evaluating the time
    # formula there must give T_opt.
    def check(model, key, p, m, a, bg, k, two):
        # T(s) = k_mult * (K + m/s) (a + bg s): s_opt = sqrt(w m a / (K bg)), T_opt = mult (sqrt(K a) + sqrt(w m bg))^2
        s_opt = math.sqrt(two * m * a / (k * bg))
        assert s_opt == int(s_opt) and m % int(s_opt) == 0
        sz = int(s_opt)
        got = O.closed_forms(model, p, m // sz, m, sz, a, bg, 0)[key]
        return got

    # unidirectional pipeline: (p-1 + 2(q-1)) r, s_opt = sqrt(2 m a / ((p-3)(b+g)))
    assert check(O.UNI, "pipeline", 5, 16, 1, 1, 2, 2) == pytest.approx((math.sqrt(2 * 1) + math.sqrt(2 * 16 * 1)) ** 2) == 50
    # unidirectional binary: N = ceil(log2(p+1)); p = 31 -> N = 5, s_opt = sqrt(2 m a / ((N-3)(b+g)))
    assert check(O.UNI, "binary", 31, 16, 1, 1, 2, 2) == pytest.approx(2 * (math.sqrt(2 * 1) + math.sqrt(2 * 16)) ** 2) == 100
    # bidirectional pipeline: (p+q-2) r, s_opt = sqrt(m a / ((p-2)(b+g)))
    assert check(O.BI, "pipeline", 6, 16, 4, 1, 4, 1) == pytest.approx((math.sqrt(4 * 4) + math.sqrt(16)) ** 2) == 64
    # bidirectional binary: 2 (N+q-2) r follows from the printed s_opt = sqrt(m a / ((N-2)(b+g)))
    assert check(O.BI, "binary", 63, 16, 4, 1, 4, 1) == pytest.approx(2 * (math.sqrt(4 * 4) + math.sqrt(16)) ** 2) == 128
    # bi-greedy / optimal broadcast: (L+q-1) r, s_opt = sqrt(m a / ((L-1)(b+g)))
    assert check(O.BI, "revopt", 32, 16, 4, 1, 4, 1) == pytest.approx((math.sqrt(4 * 4) + math.sqrt(16)) ** 2) == 64


def test_closed_forms_values_and_gamma_split():
    cf = O.closed_forms(O.UNI, 10, 4, 12, 3, 2, 1, 1)
    r = 2 + 3 + 3
    assert cf == {"binomial": 4 * (2 + 12 + 12), "pipeline": (9 + 6) * r, "binary": (2 * 3 + 12) * r,
                  "revopt": (4 + 3) * r, "butterfly": 2 * 4 * 2 + 2 * 0.9 * 12 + 0.9 * 12,
                  "lower_bound": 4 * 2 + 2 * 12 + 0.9 * 12}
    cb = O.closed_forms(O.BI, 10, 4, 12, 3, 2, 1, 1)
    assert (cb["pipeline"], cb["binary"], cb["lower_bound"]) == ((10 + 4 - 2) * r, 2 * (4 + 4 - 2) * r, 4 * 2 + 12 + 0.9 * 12)
    # Table II: p = 2 needs the message across the wire once
    assert O.closed_forms(O.UNI, 2, 1, 5, 5, 1, 1, 0)["lower_bound"] == 1 + 5
    # uni and bi binary agree at q = 1 (one segment leaves nothing to overlap)
    for p in (7, 15, 20):
        assert O.closed_forms(O.UNI, p, 1, 9, 9, 3, 1, 2)["binary"] == O.closed_forms(O.BI, p, 1, 9, 9, 3, 1, 2)["binary"]


def test_constructions_match_closed_forms_where_exact():
    for p in range(2, 40):
        for a, b, g in COSTS:
            assert O.binomial_construct(p, 6, a, b, g) == O.closed_forms(O.UNI, p, 1, 6, 6, a, b, g)["binomial"]
            for q in (1, 2, 5):
                cons = O.pipeline_construct(p, [2] * q, a, b, g)
                form = O.closed_forms(O.UNI, p, q, 2 * q, 2, a, b, g)["pipeline"]
                # Table I counts two full rounds per further segment; with a combine cost the chain's
                # real period is 2 tcomm + tcomp, so the table is exact for gamma = 0 and an upper
                # bound otherwise (p = 2 has no forwarding processor)
                if g == 0 and p > 2:
                    assert cons == form
                else:
                    assert cons <= form
                if p > 2:
                    c, gg = a + 2 * b, 2 * g
                    assert cons == (p - 1) * (c + gg) + (q - 1) * (2 * c + gg)
    for k in range(1, 11):                                   # Table III: exact for powers of two
        p = 1 << k
        got = O.butterfly_steps(p, 1 << 20, 3e-6, 2e-9, 5e-10)
        assert got == pytest.approx(O.closed_forms(O.BI, p, 1, 1 << 20, 1 << 20, 3e-6, 2e-9, 5e-10, "f64")["butterfly"], rel=1e-13)


def test_binary_tree_built_in_steps_meets_the_tables():
    """Section 4's binary tree built step by step (two senders per receiver in turn, extra processors first)
    and timed with the cost model: Table I's (2(N-1) + 4(q-1)) r with one port and, with two ports,
    2(N+q-2) r -- the form Table III's own optimal-size rows follow from, not the printed 2(N+q-1) r.  Equal for
    p = 2^n - 1 (the case the section describes) whatever the combine cost, never above the table for any
    p > 3 or with a smaller last segment (the tables' note: upper bounds then)."""
    for a, b, g in COSTS:
        for q in (1, 2, 3, 7):
            for p in (7, 15, 31, 63, 127):
                for model in (O.UNI, O.BI):
                    cf = O.closed_forms(model, p, q, 3 * q, 3, a, b, g)["binary"]
                    assert O.binary_construct(model, p, [3] * q, a, b, g) == cf, (model, p, q, a, b, g)
            r = a + 3 * b + 3 * g
            assert O.binary_construct(O.BI, 31, [3] * q, a, b, g) == 2 * (5 + q - 2) * r
            if r > 0:
                assert O.binary_construct(O.BI, 31, [3] * q, a, b, g) < 2 * (5 + q - 1) * r        # not the printed form
            for p in (4, 5, 6, 9, 12, 20, 33, 100):
                for model in (O.UNI, O.BI):
                    cf = O.closed_forms(model, p, q, 3 * q, 3, a, b, g)["binary"]
                    assert O.binary_construct(model, p, [3] * q, a, b, g) <= cf
                    if q > 1:
                        assert O.binary_construct(model, p, [3] * (q - 1) + [1], a, b, g) <= cf
    # uni-greedy is never slower than this in-order tree either (Theorem 1)
    for p in (7, 20, 63):
        for q in (1, 4):
            assert O.uni_greedy(p, [3] * q, 2, 1, 1, want_schedule=False).T <= O.binary_construct(O.UNI, p, [3] * q, 2, 1, 1)
    # fp64: same value up to the rounding of a product against a running sum
    got = O.binary_construct(O.UNI, 63, [4096] * 9, 3e-6, 2e-9, 5e-10, "f64")
    assert got == pytest.approx(O.closed_forms(O.UNI, 63, 9, 9 * 4096, 4096, 3e-6, 2e-9, 5e-10, "f64")["binary"], rel=1e-13)


# --------------------------------------------------------------------------- replay
def test_replay_int32_equals_plain_sum_and_fp32_is_close():
    # Section 1: the pieces "need to be combined using an associative operation to form the
    # results on the root"; for integers any valid combine order gives the plain sum.
    p, q, per = 23, 5, 37
    off = np.arange(q + 1, dtype=np.int64) * per
    off[-1] -= 9                                              # ragged last segment
    n = int(off[-1])
    for model in ("uni", "bi"):
        fn = O.uni_greedy if model == "uni" else O.bi_greedy
        s = fn(p, [4] * (q - 1) + [3], 2, 1, 1)
        bi = prs_inputs.replay_buffers(p, n, "i32")
        assert np.array_equal(O.replay(p, off, s.src, s.dst, s.seg, bi), bi.sum(axis=0, dtype=np.int64).astype(np.int32))
        bf = prs_inputs.replay_buffers(p, n, "f32")
        got = O.replay(p, off, s.src, s.dst, s.seg, bf)
        ref = bf.astype(np.float64).sum(axis=0)
        assert np.max(np.abs(got - ref)) <= p * 2.0 ** -23 * np.abs(bf).sum(axis=0).max()
        # the association is the schedule's: a different valid order changes fp32 bits somewhere
        assert got.dtype == np.float32


def test_replay_follows_the_schedule_order():
    # three processors, one segment: 2 -> 1 then 1 -> 0 gives (b0 + (b1 + b2))
    buf = np.array([[1.0], [2.0 ** -24], [2.0 ** -24]], dtype=np.float32)
    off = np.array([0, 1], np.int64)
    chain = O.replay(3, off, [2, 1], [1, 0], [0, 0], buf)
    star = O.replay(3, off, [1, 2], [0, 0], [0, 0], buf)
    assert chain[0] == np.float32(1.0) + np.float32(2.0 ** -23)
    assert star[0] == np.float32(1.0)


def test_replay_other_element_types_and_maximum():
    """Replay with 64-bit elements and with the maximum as the combine: integers wrap and give the plain
    sum modulo 2^64; the fp64 association is the schedule's; the maximum of a column does not depend on the
    schedule, orders -0 below +0 and puts a NaN with a clear sign bit on top."""
    p, q = 11, 3
    off = np.array([0, 7, 14, 18], np.int64)
    s = O.uni_greedy(p, [7, 7, 4], 2, 1, 1)
    big = prs_inputs.replay_buffers(p, 18, "i64") + (np.int64(1) << 61)           # 11 x 2^61 passes 2^63
    want = np.zeros(18, np.uint64)
    for row in big:
        want = want + row.view(np.uint64)
    assert np.array_equal(O.replay(p, off, s.src, s.dst, s.seg, big).view(np.uint64), want)
    buf = np.array([[1.0], [2.0 ** -53], [2.0 ** -53]], dtype=np.float64)
    one = np.array([0, 1], np.int64)
    assert O.replay(3, one, [2, 1], [1, 0], [0, 0], buf)[0] == 1.0 + 2.0 ** -52    # b0 + (b1 + b2)
    assert O.replay(3, one, [1, 2], [0, 0], [0, 0], buf)[0] == 1.0                 # (b0 + b1) + b2
    for kind in ("i32", "i64", "f32", "f64"):
        b = prs_inputs.replay_buffers(p, 18, kind)
        assert np.array_equal(O.replay(p, off, s.src, s.dst, s.seg, b, "max"), b.max(axis=0))
    z = np.array([[-0.0, -1.0, -0.0], [0.0, np.nan, -0.0], [-0.0, 5.0, -0.0]], np.float32)
    r = O.replay(3, np.array([0, 3], np.int64), [2, 1], [1, 0], [0, 0], z, "max")
    assert not np.signbit(r[0]) and r[0] == 0 and np.isnan(r[1]) and np.signbit(r[2])
    assert np.array_equal(O.total_order_key(np.array([-np.inf, -1.0, -0.0, 0.0, 1.0, np.inf])).argsort(), np.arange(6))


def test_replay_of_baseline_trees_has_their_association():
    """Section 4's trees as schedules: the pipeline folds from the far end, b0 + (b1 + (b2 + ...)); the
    binomial tree adds neighbours, then neighbours of neighbours; integers give the plain sum for all."""
    import baseline_trees as B
    p, q = 8, 2
    off = np.array([0, 5, 9], np.int64)
    bf = prs_inputs.replay_buffers(p, 9, "f32")
    chain = bf[p - 1].copy()
    for i in range(p - 2, -1, -1):
        chain = bf[i] + chain
    assert np.array_equal(O.replay(p, off, *B.pipeline(p, q), bf), chain)
    pairwise = ((bf[0] + bf[1]) + (bf[2] + bf[3])) + ((bf[4] + bf[5]) + (bf[6] + bf[7]))
    assert np.array_equal(O.replay(p, off, *B.binomial(p, q), bf), pairwise)
    heap = (bf[0] + ((bf[2] + bf[6]) + bf[5])) + ((bf[1] + bf[4]) + (bf[3] + bf[7]))
    assert np.array_equal(O.replay(p, off, *B.binary(p, q), bf), heap)
    for tree in (B.pipeline, B.binomial, B.binary):
        for pp in (2, 3, 13):
            bi = prs_inputs.replay_buffers(pp, 9, "i32")
            assert np.array_equal(O.replay(pp, off, *tree(pp, q), bi), bi.sum(axis=0, dtype=np.int64).astype(np.int32))


def test_butterfly_can_only_win_for_small_beta_over_gamma():
    """Section 6.1: below a line in the (p, beta/gamma) plane some message size lets the butterfly beat bi-greedy,
    above it never; "for up to 1000 processors the ratio would have to be less than 5".  The closed form of the
    line (segment count as a real number) stays below 5 up to 1024 processors and grows with p from 16 on; trying
    message sizes and segment counts one by one lands within a tenth of it; the machine of Figure 6 (ratio 6)
    is above the line for 64 processors, a ratio of 1 is below it."""
    line = {p: O.butterfly_threshold_closed_form(p) for p in [4, 8, 16, 32, 64, 128, 256, 512, 1000, 1024]}
    assert all(0 < r < 5 for r in line.values()) and line[1024] > 4.5
    assert all(line[a] < line[b] for a, b in zip([16, 32, 64, 128, 256, 512], [32, 64, 128, 256, 512, 1000]))
    ms = [2 ** k for k in range(4, 23)]
    for p in (16, 64):
        lo, hi = 0.25, 16.0
        for _ in range(10):
            mid = math.sqrt(lo * hi)
            lo, hi = (mid, hi) if O.butterfly_wins_somewhere(p, 1000.0, mid, 1.0, ms, 512) else (lo, mid)
        assert abs(math.sqrt(lo * hi) / line[p] - 1) < 0.1, (p, lo, hi, line[p])
    assert not O.butterfly_wins_somewhere(64, 50000.0, 6.0, 1.0, [2 ** k for k in range(10, 28)], 512)
    assert O.butterfly_wins_somewhere(64, 50000.0, 1.0, 1.0, [2 ** k for k in range(10, 28)], 512)
    # alpha drops out of the condition
    assert O.butterfly_wins_somewhere(64, 10.0, 2.0, 1.0, ms, 512) and O.butterfly_wins_somewhere(64, 1e5, 2.0, 1.0, [2 ** k for k in range(4, 30)], 4096)


def test_butterfly_threshold_bisection_brackets_the_line():
    """The bisection the device entry point mirrors: its bracket holds the closed form of the line to within a
    tenth, stays below 5 for 1024 processors, and returns the caller's bracket when no step is taken."""
    assert O.butterfly_threshold_bisect(64, 1000.0, 512, 4, 22, 0.25, 16.0, 0) == (0.25, 16.0)
    for p in (16, 64):
        lo, hi = O.butterfly_threshold_bisect(p, 1000.0, 512, 4, 22, 0.25, 16.0, 9)
        assert hi - lo == (16.0 - 0.25) / 512 and hi < 5
        assert abs(0.5 * (lo + hi) / O.butterfly_threshold_closed_form(p) - 1) < 0.1
        ms = [2 ** k for k in range(4, 23)]
        assert O.butterfly_wins_somewhere(p, 1000.0, lo, 1.0, ms, 512) and not O.butterfly_wins_somewhere(p, 1000.0, hi, 1.0, ms, 512)


# --------------------------------------------------------------------------- best segmentation (Sections 5.2, 6.1)
def _table1_pipeline_uni(p, q, m, a, b, g):
    sz = -(-m // q)
    qe = -(-m // sz)
    return (p - 1 + 2 * (qe - 1)) * (a + b * sz + g * sz)            # Table I, unidirectional pipeline


def test_best_segmentation_is_the_minimum_over_the_candidates():
    """The search is pinned by brute force: Table I's pipeline time written out here and minimised over the same
    candidates gives the same time and count; the greedy optimum is what trying each count one by one gives;
    with a single candidate the search is the plain simulation; a larger candidate set never does worse."""
    rng = np.random.default_rng(11)
    n = 40
    p = rng.integers(2, 48, n).astype(np.int32)
    m = rng.integers(1, 400, n).astype(np.int64)
    al = rng.integers(0, 40, n).astype(np.int64); be = rng.integers(1, 4, n).astype(np.int64); ga = rng.integers(0, 4, n).astype(np.int64)
    host = prs_inputs.SweepConfigs(p, np.full(n, 7, np.int32), m, al, be, ga, "i64")      # q_req must not matter
    got = O.optimal_segmentation(host, O.UNI, 64)
    cands = [1, 2, 4, 8, 16, 32, 64]
    for i in range(n):
        vals = [_table1_pipeline_uni(int(p[i]), q, int(m[i]), int(al[i]), int(be[i]), int(ga[i])) for q in cands]
        assert got["T_pipeline"][i] == min(vals)
        assert got["q_pipeline"][i] == cands[vals.index(min(vals))]
        gv = [O.uni_greedy(int(p[i]), O.equi_sizes(int(m[i]), q), int(al[i]), int(be[i]), int(ga[i]), "i64", want_schedule=False).T
              for q in cands]
        assert got["T_greedy"][i] == min(gv) and got["q_greedy"][i] == cands[gv.index(min(gv))]
    one = O.optimal_segmentation(host, O.UNI, 1)
    host1 = prs_inputs.SweepConfigs(p, np.ones(n, np.int32), m, al, be, ga, "i64")
    assert np.array_equal(one["T_greedy"], O.simulate_batch(host1, O.UNI).T_greedy) and np.all(one["q_greedy"] == 1)
    more = O.optimal_segmentation(host, O.UNI, 256)
    for a in ("greedy", "pipeline", "binary", "revopt"):
        assert np.all(more["T_" + a] <= got["T_" + a])
    # Theorem 1 at every segmentation: the greedy optimum is not above any in-order algorithm's optimum
    assert np.all(got["T_greedy"] <= got["T_pipeline"]) and np.all(got["T_greedy"] <= got["T_binary"])


def test_best_segmentation_bidirectional_meets_table3_at_its_best_count():
    """Bi-greedy at equal segments meets the reversed optimal broadcast (Table III), so their optima over the
    candidates that divide m coincide."""
    n = 24
    p = np.arange(2, 2 + n).astype(np.int32)
    m = np.full(n, 64, np.int64)                                       # every power-of-two count divides m
    host = prs_inputs.SweepConfigs(p, np.ones(n, np.int32), m, np.full(n, 9, np.int64), np.full(n, 2, np.int64),
                                   np.full(n, 1, np.int64), "i64")
    got = O.optimal_segmentation(host, O.BI, 64)
    assert np.array_equal(got["T_greedy"], got["T_revopt"]) and np.array_equal(got["q_greedy"], got["q_revopt"])
