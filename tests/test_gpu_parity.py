"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Integer results, schedules and replay must match
bit for bit; fp64 times within 1e-12 relative."""
from __future__ import annotations

import math

import numpy as np
import pytest

import oracle as O
import prs_inputs

pytestmark = pytest.mark.gpu

REL = 1e-12


@pytest.fixture(scope="module")
def prs():
    import torch
    import paper_1310_4645_amd as lib
    assert torch.cuda.is_available()
    lib.load_library()
    return lib


def _sync():
    import torch
    torch.cuda.synchronize()


def _np(t):
    return t.cpu().numpy()


def _rel_ok(got, ref, rel=REL):
    return np.all(np.abs(got - ref) <= rel * np.abs(ref))


def _check_times(got, ref: O.BatchResult, exact):
    for key, r in (("greedy", ref.T_greedy), ("binomial", ref.T_binomial), ("pipeline", ref.T_pipeline),
                   ("binary", ref.T_binary), ("revopt", ref.T_revopt)):
        g = _np(got[key])
        if exact:
            assert np.array_equal(g, r), key
        else:
            assert _rel_ok(g, r), (key, np.max(np.abs(g - r) / np.abs(r)))
    assert _rel_ok(_np(got["butterfly"]), ref.T_butterfly)
    assert _rel_ok(_np(got["lower_bound"]), ref.T_lower_bound)
    assert np.array_equal(_np(got["q_eff"]), ref.q_eff)
    assert np.array_equal(_np(got["cfg_status"]), ref.status)


def _oracle_schedules(host, model):
    out = []
    for i in range(len(host)):
        sizes = O.equi_sizes(int(host.m[i]), int(host.q_req[i]))
        a, b, g = host.alpha[i].item(), host.beta[i].item(), host.gamma[i].item()
        fn = O.uni_greedy if model == O.UNI else O.bi_greedy
        kw = {} if model == O.UNI else {"mode": O.MODE_EVENT | O.MODE_PRUNE}
        out.append(fn(int(host.p[i]), sizes, a, b, g, host.cost, **kw))
    return out


def _check_schedules(prs, host, model, p_max, q_max, exact_t=True, tuning=None):
    dev = prs.DeviceConfigs.from_host(host)
    off = prs.prs_pair_offsets(dev, p_max, q_max)
    _sync()
    offh = _np(off)
    refs = _oracle_schedules(host, model)
    want_off = np.concatenate([[0], np.cumsum([len(r.src) for r in refs])])
    assert np.array_equal(offh, want_off)
    sch = prs.greedy_schedule_batch(dev, model, p_max, q_max, off, int(offh[-1]), tuning=tuning)
    _sync()
    src, dst, seg, t, T = (_np(sch[k]) for k in ("src", "dst", "seg", "t_start", "T_greedy"))
    assert np.all(_np(sch["cfg_status"]) == 0)
    for i, r in enumerate(refs):
        a, b = offh[i], offh[i + 1]
        ctx = (i, int(host.p[i]), int(host.q_req[i]), int(host.m[i]))
        assert np.array_equal(src[a:b], r.src), ("src", ctx)
        assert np.array_equal(dst[a:b], r.dst), ("dst", ctx)
        assert np.array_equal(seg[a:b], r.seg), ("seg", ctx)
        if exact_t:
            assert np.array_equal(t[a:b], r.t), ("t", ctx)
            assert T[i] == r.T, ("T", ctx)
        else:
            assert _rel_ok(t[a:b], r.t) and abs(T[i] - r.T) <= REL * abs(r.T), ("t", ctx)


# --------------------------------------------------------------------------- tiny sweep, integer costs
@pytest.mark.parametrize("model", [0, 1])
def test_tiny_sweep_times_bit_exact(prs, model):
    host = prs_inputs.tiny_sweep()
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, model, 16, 8)
    _sync()
    _check_times(got, O.simulate_batch(host, model), exact=True)


@pytest.mark.parametrize("model", [0, 1])
def test_tiny_sweep_schedules_bit_exact(prs, model):
    _check_schedules(prs, prs_inputs.tiny_sweep(), model, 16, 8)


@pytest.mark.parametrize("model", [0, 1])
def test_integer_costs_ragged_segments_and_larger_p(prs, model):
    rng = np.random.default_rng(2024 + model)
    n = 160
    p = rng.integers(2, 200, n).astype(np.int32)
    p[:8] = [2, 3, 63, 64, 65, 127, 128, 129]                  # word and tile boundaries
    m = rng.integers(1, 300, n).astype(np.int64)
    q = rng.integers(1, 24, n).astype(np.int32)
    host = prs_inputs.SweepConfigs(p, q, m, rng.integers(0, 12, n).astype(np.int64), rng.integers(0, 4, n).astype(np.int64),
                                   rng.integers(0, 4, n).astype(np.int64), "i64")
    host.alpha[host.beta == 0] += 1                                 # tcomm > 0
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, model, 256, 32)
    _sync()
    _check_times(got, O.simulate_batch(host, model), exact=True)
    _check_schedules(prs, host, model, 256, 32)


_BIG = 1000000000
# pair-count limits of the 1-, 4- (schedules: 8-) and 16-lane groups, and the binary logarithm of the pair count from which a
# configuration gets all 64 lanes: every group size in turn gets the whole batch
_GROUPINGS = {"64 lanes": {"uni_group_pairs": (0, 0, 0), "uni_wave_log2": 1},
              "64 and 32 lanes": {"uni_group_pairs": (0, 0, 0), "uni_wave_log2": 10},
              "32 lanes": {"uni_group_pairs": (0, 0, 0)},
              "16 lanes": {"uni_group_pairs": (0, 0, _BIG)},
              "4 or 8 lanes": {"uni_group_pairs": (0, _BIG, _BIG)},
              "1 lane": {"uni_group_pairs": (_BIG, _BIG, _BIG)}}


@pytest.mark.parametrize("grouping", list(_GROUPINGS))
def test_uni_every_group_size(prs, grouping):
    """Uni-greedy runs a configuration on 64, 32, 16, 4 or 1 lanes depending on its number of pairs; here every
    group size gets the same mixed batch (integer and fp64 costs, with fp64 rounding collisions)."""
    tuning = _GROUPINGS[grouping]
    rng = np.random.default_rng(77)
    n = 96
    p = rng.integers(2, 160, n).astype(np.int32)
    p[:8] = [2, 3, 31, 32, 33, 64, 65, 129]
    q = rng.integers(1, 80, n).astype(np.int32)
    q[:8] = [1, 70, 1, 33, 65, 31, 32, 5]
    m = (q.astype(np.int64) * rng.integers(1, 4, n) + rng.integers(0, 2, n)).astype(np.int64)
    host = prs_inputs.SweepConfigs(p, q, m, rng.integers(1, 12, n).astype(np.int64), rng.integers(0, 4, n).astype(np.int64),
                                   rng.integers(0, 4, n).astype(np.int64), "i64")
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, 0, 160, 80, tuning=tuning)
    _sync()
    _check_times(got, O.simulate_batch(host, 0), exact=True)
    _check_schedules(prs, host, 0, 160, 80, tuning=tuning)
    hostf = prs_inputs.SweepConfigs(p[:40], q[:40], m[:40], np.full(40, 1.0), np.full(40, 0.0), np.full(40, 2.0 ** -52), "f64")
    devf = prs.DeviceConfigs.from_host(hostf)
    gotf = prs.simulate_completion_batch(devf, 0, 160, 80, tuning=tuning)
    _sync()
    assert np.array_equal(_np(gotf["greedy"]), O.simulate_batch(hostf, 0).T_greedy)
    _check_schedules(prs, hostf, 0, 160, 80, tuning=tuning)


def test_uni_times_a_block_per_configuration(prs):
    """The kernel that gives a machine of thousands of processors a block of its own and forms many pairs of a
    segment at once, here fed with machines of every size (the limit lowered to two processors): completion
    times of the integer sweep, ragged integer cases, fp64 costs whose sums collide in rounding, and machines
    of a few thousand processors, against Algorithm 1 in the oracle, bit for bit."""
    tuning = {"uni_wide_procs": 2}
    host = prs_inputs.tiny_sweep()
    got = prs.simulate_completion_batch(prs.DeviceConfigs.from_host(host), 0, 16, 8, tuning=tuning)
    _sync()
    _check_times(got, O.simulate_batch(host, 0), exact=True)
    rng = np.random.default_rng(606)
    n = 80
    p = rng.integers(2, 300, n).astype(np.int32)
    p[:6] = [2, 3, 63, 64, 65, 257]
    q = rng.integers(1, 40, n).astype(np.int32)
    m = (q.astype(np.int64) * rng.integers(1, 4, n) + rng.integers(0, 2, n)).astype(np.int64)
    host = prs_inputs.SweepConfigs(p, q, m, rng.integers(1, 12, n).astype(np.int64), rng.integers(0, 4, n).astype(np.int64),
                                   rng.integers(0, 4, n).astype(np.int64), "i64")
    got = prs.simulate_completion_batch(prs.DeviceConfigs.from_host(host), 0, 300, 40, tuning=tuning)
    _sync()
    _check_times(got, O.simulate_batch(host, 0), exact=True)
    hostf = prs_inputs.SweepConfigs(p[:40], q[:40], m[:40], np.full(40, 1.0), np.full(40, 0.0), np.full(40, 2.0 ** -52), "f64")
    gotf = prs.simulate_completion_batch(prs.DeviceConfigs.from_host(hostf), 0, 300, 40, tuning=tuning)
    _sync()
    assert np.array_equal(_np(gotf["greedy"]), O.simulate_batch(hostf, 0).T_greedy)
    # more values under the bound than a round looks at (gamma large against the spacing of the ready times)
    pb = np.array([2500, 3000, 5000, 4097], np.int32)
    hostb = prs_inputs.SweepConfigs(pb, np.array([6, 3, 4, 9], np.int32), np.array([12, 9, 4, 27], np.int64), np.array([1, 0, 3, 2], np.int64),
                                    np.array([1, 1, 1, 2], np.int64), np.array([50, 7, 0, 1], np.int64), "i64")
    gotb = prs.simulate_completion_batch(prs.DeviceConfigs.from_host(hostb), 0, 8192, 16, tuning={"uni_wide_procs": 2048})
    _sync()
    want = [O.uni_greedy_time(int(pb[i]), O.equi_sizes(int(hostb.m[i]), int(hostb.q_req[i])), int(hostb.alpha[i]), int(hostb.beta[i]),
                              int(hostb.gamma[i])) for i in range(4)]
    assert list(_np(gotb["greedy"])) == want and np.all(_np(gotb["cfg_status"]) == 0)


# --------------------------------------------------------------------------- fp64 sweeps
def _fast_subset(host, budget, limit):
    """indices of configurations the plain oracle finishes quickly (cost ~ p^2 q)."""
    work = host.p.astype(np.float64) ** 2 * host.q_req
    idx = np.nonzero(work <= budget)[0][:limit]
    return idx


@pytest.mark.parametrize("model", [0, 1])
def test_fp64_sweep_sample_times(prs, model):
    full = prs_inputs.uni_sweep(4000)
    idx = _fast_subset(full, 4e6 if model == 0 else 3e5, 500)
    big = np.argsort(-(full.p.astype(np.float64) * full.q_req))[:3]             # a few heavy ones too
    host = full.take(np.concatenate([idx, big]))
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, model, 1024, 512)
    _sync()
    ref = O.simulate_batch(host, model)
    _check_times(got, ref, exact=False)
    # the arithmetic is the same sequence of roundings on both sides
    assert np.array_equal(_np(got["greedy"]), ref.T_greedy)


@pytest.mark.parametrize("model", [0, 1])
def test_fp64_sweep_sample_schedules(prs, model):
    full = prs_inputs.uni_sweep(3000)
    idx = _fast_subset(full, 6e5 if model == 0 else 1e5, 120)
    _check_schedules(prs, full.take(idx), model, 1024, 512)


def test_uni_schedules_with_long_runs_of_equal_values(prs):
    """Several hundred processors: the first segments send in runs of hundreds of equal values, B grows past
    what the kernel keeps in LDS, and late small indices are inserted far back (also exactly one LDS ring back)."""
    full = prs_inputs.uni_sweep(3000)
    work = full.p.astype(np.float64) ** 2 * full.q_req
    idx = np.nonzero((full.p >= 300) & (work <= 4e7))[0][:40]
    _check_schedules(prs, full.take(idx), 0, 1024, 512)


@pytest.mark.parametrize("model", [0, 1])
def test_fp64_rounding_ties(prs, model):
    # costs chosen so that sums produced at different times round to the same double
    n = 69
    p = np.arange(2, 2 + n).astype(np.int32)
    cases = [(1.0, 0.0, 2.0 ** -52), (1.0, 0.0, 2.0 ** -53), (0.75, 2.0 ** -54, 2.0 ** -51), (1.0, 2.0 ** -30, 0.0)]
    # few segments (batch kernels) and enough segments for the one-lane-per-segment kernels
    for q, m in ((5, 13), (9, 29)):
        for al, be, ga in cases:
            host = prs_inputs.SweepConfigs(p, np.full(n, q, np.int32), np.full(n, m, np.int64), np.full(n, al),
                                           np.full(n, be), np.full(n, ga), "f64")
            dev = prs.DeviceConfigs.from_host(host)
            got = prs.simulate_completion_batch(dev, model, 128, 16)
            _sync()
            ref = O.simulate_batch(host, model)
            assert np.array_equal(_np(got["greedy"]), ref.T_greedy), (q, al, be, ga)
            _check_schedules(prs, host, model, 128, 16)


def _mid_machines(cost, seed):
    """48 machines of 257..1024 processors (the bi-greedy kernel gives each 16 lanes) with 16..64 segments, half
    of them with a smaller last segment."""
    rng = np.random.default_rng(seed)
    n = 48
    p = rng.integers(257, 1025, n).astype(np.int32)
    p[:8] = [257, 511, 512, 513, 768, 1000, 1023, 1024]
    q = rng.integers(16, 65, n).astype(np.int32)
    per = rng.integers(2, 9, n).astype(np.int64) * (1 if cost == "i64" else 4096)
    m = q.astype(np.int64) * per
    m[1::2] -= rng.integers(1, per[1::2])                               # ragged: the last segment is smaller
    if cost == "i64":
        al, be, ga = rng.integers(0, 40, n).astype(np.int64), rng.integers(1, 4, n).astype(np.int64), rng.integers(0, 4, n).astype(np.int64)
    else:
        al, be, ga = 10.0 ** rng.uniform(-6, -4, n), 10.0 ** rng.uniform(-10, -8, n), 10.0 ** rng.uniform(-11, -9, n)
    return prs_inputs.SweepConfigs(p, q, m, al, be, ga, cost)


@pytest.mark.parametrize("cost", ["i64", "f64"])
def test_bi_schedules_of_machines_with_hundreds_of_processors(prs, cost):
    """Bi-greedy schedules pair for pair where a configuration occupies 16 lanes (p = 257..1024) and has many
    segments in flight: integer and fp64 costs, equal and smaller last segment."""
    host = _mid_machines(cost, 4242)
    q_eff = np.array([O.segmentation(int(host.m[i]), int(host.q_req[i]))[0] for i in range(len(host))])
    assert np.all(q_eff >= 16) and np.any(host.m % host.q_req != 0)
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, 1, 1024, 64)
    _sync()
    _check_times(got, O.simulate_batch(host, 1), exact=True)
    _check_schedules(prs, host, 1, 1024, 64)


@pytest.mark.parametrize("entries", [1, 3])
def test_bi_configurations_handed_over_to_the_general_kernel(prs, entries):
    """The kernel that runs several configurations per wavefront keeps a short list of running transfers per
    configuration; one that needs more is rerun by the one-configuration kernel.  With the list cut down to
    a few entries most of a mixed batch takes that road, times and schedules stay those of the oracle."""
    rng = np.random.default_rng(31 + entries)
    n = 90
    p = rng.integers(2, 400, n).astype(np.int32)
    p[:8] = [2, 3, 64, 65, 128, 129, 256, 257]                        # first and last machine of a group size
    q = rng.integers(1, 30, n).astype(np.int32)
    m = (q.astype(np.int64) * rng.integers(1, 5, n) - rng.integers(0, 2, n)).clip(1)
    host = prs_inputs.SweepConfigs(p, q, m, rng.integers(0, 12, n).astype(np.int64), rng.integers(1, 4, n).astype(np.int64),
                                   rng.integers(0, 4, n).astype(np.int64), "i64")
    tuning = {"bi_list_entries": entries}
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, 1, 512, 32, tuning=tuning)
    _sync()
    _check_times(got, O.simulate_batch(host, 1), exact=True)
    _check_schedules(prs, host, 1, 512, 32, tuning=tuning)
    hostf = _mid_machines("f64", 99).take(np.arange(0, 48, 4))
    _check_schedules(prs, hostf, 1, 1024, 64, tuning=tuning)


def test_costs_too_large_for_the_cost_type_are_refused(prs):
    """A configuration whose schedule would pass the range of the cost type (Table I's pipeline time, which
    bounds every greedy time) is reported as a bad parameter instead of being run: with doubles the sums would
    reach infinity, which the kernels use as "no value"."""
    p = np.array([8, 8, 8, 1000], np.int32)
    q = np.array([1, 1, 4, 4], np.int32)
    m = np.array([1, 1, 4, 4], np.int64)
    host = prs_inputs.SweepConfigs(p, q, m, np.array([1e308, 1e299, 1.0, 1e298]), np.zeros(4), np.zeros(4), "f64")
    dev = prs.DeviceConfigs.from_host(host)
    for model in (0, 1):
        got = prs.simulate_completion_batch(dev, model, 1024, 8)
        _sync()
        assert list(_np(got["cfg_status"])) == [1, 0, 0, 1]
        g = _np(got["greedy"])
        assert np.isnan(g[0]) and np.isnan(g[3]) and g[1] == 3e299 and np.isfinite(g[2])
    hosti = prs_inputs.SweepConfigs(p, q, m, np.array([1 << 61, 1 << 58, 1, 1 << 52], np.int64), np.ones(4, np.int64),
                                    np.zeros(4, np.int64), "i64")
    got = prs.simulate_completion_batch(prs.DeviceConfigs.from_host(hosti), 0, 1024, 8)
    _sync()
    assert list(_np(got["cfg_status"])) == [1, 0, 0, 1] and _np(got["greedy"])[1] == 3 * ((1 << 58) + 1)
    off = prs.prs_pair_offsets(dev, 1024, 8)
    _sync()
    assert list(_np(off)) == [0, 0, 7, 35, 35]


def test_invalid_configurations_are_reported_not_fatal(prs):
    p = np.array([1, 8, 8, 8, 8, 300, 8, 8], np.int32)
    q = np.array([2, 0, 2, 2, 2, 2, 99, 3], np.int32)
    m = np.array([4, 4, 0, 4, 4, 4, 400, 6], np.int64)
    al = np.array([1.0, 1.0, 1.0, -1.0, float("nan"), 1.0, 1.0, 2.0])
    host = prs_inputs.SweepConfigs(p, q, m, al, np.ones(8), np.ones(8), "f64")
    dev = prs.DeviceConfigs.from_host(host)
    for model in (0, 1):
        got = prs.simulate_completion_batch(dev, model, 64, 16)
        _sync()
        st = _np(got["cfg_status"])
        assert list(st) == [1, 1, 1, 1, 1, 2, 2, 0]
        g = _np(got["greedy"])
        assert np.all(np.isnan(g[:7]))
        sizes = O.equi_sizes(6, 3)
        want = (O.uni_greedy if model == 0 else O.bi_greedy)(8, sizes, 2.0, 1.0, 1.0, "f64").T
        assert g[7] == want
    off = prs.prs_pair_offsets(dev, 64, 16)
    _sync()
    assert list(_np(off)) == [0] * 8 + [21]
    # capacity too small for the only valid configuration
    sch = prs.greedy_schedule_batch(dev, 0, 64, 16, off, 20)
    _sync()
    assert _np(sch["cfg_status"])[7] == 2
    # call-level errors: nothing is enqueued
    with pytest.raises(prs.PrsError):
        prs.simulate_completion_batch(dev, 7, 64, 16)
    with pytest.raises(prs.PrsError):
        prs.simulate_completion_batch(dev, 0, 1, 16)


def test_empty_batch(prs):
    host = prs_inputs.tiny_sweep().take(np.arange(0))
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, 0, 16, 8)
    _sync()
    assert got["greedy"].numel() == 0


# --------------------------------------------------------------------------- full-size sweeps
@pytest.mark.parametrize("model", [0, 1])
def test_full_sweep_invariants_and_samples(prs, model):
    """The 100,000-configuration sweep in the launch shape the benchmark times: sampled configurations
    against the oracle, every configuration against what holds at any size."""
    host = prs_inputs.uni_sweep()
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, model, 1024, 512)
    _sync()
    T = _np(got["greedy"])
    assert np.all(_np(got["cfg_status"]) == 0) and np.all(np.isfinite(T))
    q = _np(got["q_eff"]).astype(np.int64)
    sz = -(-host.m // host.q_req)
    assert np.array_equal(q, -(-host.m // sz))
    L = np.ceil(np.log2(host.p)).astype(np.int64)
    r = (host.alpha + host.beta * sz) + host.gamma * sz
    if model == 0:
        # Theorem 1: no slower than the in-order pipeline and binary trees; Table II bounds
        assert np.all(T <= _np(got["pipeline"]) * (1 + 1e-12))
        assert np.all(T <= _np(got["binary"]) * (1 + 1e-12))
        assert np.all(T >= L * host.alpha)
        one = q == 1                                            # a single segment is the binomial tree
        assert _rel_ok(T[one], _np(got["binomial"])[one])
    else:
        # Section 6.2: equals the reversed optimal broadcast whenever all segments are equal
        eq = host.m % sz == 0
        assert eq.sum() > 1000
        assert _rel_ok(T[eq], ((L + q - 1) * r)[eq], 1e-11)
        assert np.all(T >= L * host.alpha)
    rng = np.random.default_rng(99)
    work = host.p.astype(np.float64) ** 2 * host.q_req
    cand = np.nonzero(work <= (2e7 if model == 0 else 1e6))[0]
    idx = np.sort(rng.choice(cand, 300, replace=False))
    ref = O.simulate_batch(host, model, index=idx)
    assert np.array_equal(T[idx], ref.T_greedy)
    assert _rel_ok(_np(got["butterfly"])[idx], ref.T_butterfly) and _rel_ok(_np(got["revopt"])[idx], ref.T_revopt)


def _large_p_subsample(max_pairs):
    """Every 61st configuration of the large-machine sweep (p in [1024, 65536], 64 to 4096 segments) whose
    schedule has at most max_pairs pairs, plus the first few with more than 32768 processors."""
    full = prs_inputs.large_p_sweep()
    q = np.array([O.segmentation(int(full.m[i]), int(full.q_req[i]))[0] for i in range(len(full))])
    pairs = (full.p.astype(np.int64) - 1) * q
    every = np.arange(0, len(full), 61)
    wide = np.nonzero((full.p > 32768) & (pairs <= max_pairs))[0][:6]
    idx = np.unique(np.concatenate([every[pairs[every] <= max_pairs], wide]))
    assert np.any(full.p[idx] > 32768) and len(idx) >= 60
    return full, idx


def test_large_machines_uni_times(prs):
    """Uni-greedy completion times on the large-machine sweep against the oracle's value-only form of
    Algorithm 1, bit for bit (same roundings), tens of thousands of processors included."""
    from concurrent.futures import ThreadPoolExecutor
    full, idx = _large_p_subsample(3e7)
    host = full.take(idx)
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, 0, 65536, 4096)
    _sync()
    assert np.all(_np(got["cfg_status"]) == 0)

    def one(i):
        return O.uni_greedy_time(int(host.p[i]), O.equi_sizes(int(host.m[i]), int(host.q_req[i])), float(host.alpha[i]),
                                 float(host.beta[i]), float(host.gamma[i]), "f64")
    with ThreadPoolExecutor(16) as ex:
        ref = np.array(list(ex.map(one, range(len(host)))))
    assert np.array_equal(_np(got["greedy"]), ref)
    assert np.all(ref <= _np(got["pipeline"]) * (1 + 1e-12)) and np.all(ref <= _np(got["binary"]) * (1 + 1e-12))   # Theorem 1


def test_large_machines_bi_times(prs):
    """Bi-greedy on the large-machine sweep.  (i) The draws of the subsample with the message size rounded up to
    a multiple of the segment count (equal segments): the time is that of the reversed optimal broadcast, Table
    III, up to 65536 processors.  (ii) Every 16th of the cheapest tenth of the sweep as drawn (mostly a smaller
    last segment) against the oracle, bit for bit."""
    full, idx = _large_p_subsample(1.2e7)
    host = full.take(idx)
    sz = -(-host.m // host.q_req)
    host.m = sz * host.q_req
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.simulate_completion_batch(dev, 1, 65536, 4096)
    _sync()
    assert np.all(_np(got["cfg_status"]) == 0) and np.array_equal(_np(got["q_eff"]), host.q_req)
    L = np.ceil(np.log2(host.p)).astype(np.int64)
    r = (host.alpha + host.beta * sz) + host.gamma * sz
    assert _rel_ok(_np(got["greedy"]), (L + host.q_req - 1) * r, 1e-11)
    assert _rel_ok(_np(got["greedy"]), _np(got["revopt"]), 1e-11)
    work = full.p.astype(np.float64) ** 2 * full.q_req
    cheap = np.sort(np.argsort(work)[: len(full) // 10])[::16]
    small = full.take(cheap)
    got = prs.simulate_completion_batch(prs.DeviceConfigs.from_host(small), 1, 65536, 4096)
    _sync()
    ref = O.simulate_batch(small, 1)
    assert np.array_equal(_np(got["greedy"]), ref.T_greedy) and np.all(_np(got["cfg_status"]) == 0)
    assert np.any(small.m % (-(-small.m // small.q_req)) != 0)


@pytest.mark.parametrize("model", [0, 1])
def test_schedules_beyond_1024_processors(prs, model):
    """Full schedules where the per-processor state no longer fits the small-machine kernels (bi-greedy: one
    wavefront per configuration with bit sets of many words; uni-greedy: streams far longer than the LDS ring),
    integer and fp64 costs, equal and ragged last segments."""
    p = np.array([1025, 2000, 3001, 1500], np.int32)
    q = np.array([3, 2, 5, 4], np.int32)
    m = np.array([9, 7, 20, 4], np.int64)
    host = prs_inputs.SweepConfigs(p, q, m, np.array([3, 0, 7, 2], np.int64), np.array([1, 2, 1, 3], np.int64),
                                   np.array([1, 1, 0, 2], np.int64), "i64")
    _check_schedules(prs, host, model, 4096, 8)
    _check_schedules(prs, host, model, 40000, 8)      # sized for tens of thousands of processors: other placement of the state
    hostf = prs_inputs.SweepConfigs(p[:3], q[:3], m[:3] * 1000 + 1, np.array([2e-6, 1e-5, 3e-6]), np.array([1e-9, 2e-9, 5e-10]),
                                    np.array([1e-10, 0.0, 3e-10]), "f64")
    _check_schedules(prs, hostf, model, 4096, 8)


# --------------------------------------------------------------------------- best segmentation per algorithm
@pytest.mark.parametrize("model", [0, 1])
@pytest.mark.parametrize("cost", ["i64", "f64"])
def test_optimal_segmentation_matches_trying_each_count(prs, model, cost):
    rng = np.random.default_rng(500 + model)
    n = 150
    p = rng.integers(2, 90, n).astype(np.int32)
    m = rng.integers(1, 3000, n).astype(np.int64)
    if cost == "i64":
        al, be, ga = (rng.integers(0, 60, n).astype(np.int64), rng.integers(1, 4, n).astype(np.int64),
                      rng.integers(0, 4, n).astype(np.int64))
    else:
        al, be, ga = 10.0 ** rng.uniform(-6, -4, n), 10.0 ** rng.uniform(-10, -8, n), 10.0 ** rng.uniform(-11, -9, n)
    p[:3] = [2, 3, 1]                                                   # the last one is not a valid problem
    host = prs_inputs.SweepConfigs(p, np.zeros(n, np.int32), m, al, be, ga, cost)
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.optimal_segmentation_batch(dev, model, 128, 32)
    _sync()
    ok = np.ones(n, bool); ok[2] = False
    ref = O.optimal_segmentation(host.take(np.nonzero(ok)[0]), model, 32)
    for key in ("greedy", "pipeline", "binary", "revopt"):
        assert np.array_equal(_np(got["T_" + key])[ok], ref["T_" + key]), key
        assert np.array_equal(_np(got["q_" + key])[ok], ref["q_" + key]), key
    st = _np(got["cfg_status"])
    assert st[2] == 1 and np.all(st[ok] == 0) and _np(got["q_greedy"])[2] == -1


def test_theoretical_experiment_grid_of_section_5_2(prs):
    """The parameter grid of the paper's theoretical experiments (alpha in {0,1,10,100,1000}, beta = 1,
    gamma in {0,1}, p = 4..1024, m = 4..65536 bytes, powers of two), every algorithm at its best
    power-of-two segment count, on the GPU: no standard algorithm ever beats uni-greedy (Theorem 1), small
    messages are reduced best unsegmented, where greedy is the binomial tree, and at p = 64, alpha = 10,
    gamma = 0 the largest gain over the best standard algorithm is about 50 % (Figure 4).  A sample of
    the grid is compared with the oracle trying each count."""
    probs = [(p, m, a, g) for a in (0, 1, 10, 100, 1000) for g in (0, 1) for p in (2 ** k for k in range(2, 11))
             for m in (2 ** k for k in range(2, 17))]
    n = len(probs)
    host = prs_inputs.SweepConfigs(np.array([x[0] for x in probs], np.int32), np.zeros(n, np.int32),
                                   np.array([x[1] for x in probs], np.int64), np.array([x[2] for x in probs], np.int64),
                                   np.ones(n, np.int64), np.array([x[3] for x in probs], np.int64), "i64")
    dev = prs.DeviceConfigs.from_host(host)
    best = prs.optimal_segmentation_batch(dev, prs.PRS_UNI, 1024, 65536)
    one = prs.DeviceConfigs.from_host(prs_inputs.SweepConfigs(host.p, np.ones(n, np.int32), host.m, host.alpha, host.beta,
                                                               host.gamma, "i64"))
    unsegmented = prs.simulate_completion_batch(one, prs.PRS_UNI, 1024, 1)
    _sync()
    assert np.all(_np(best["cfg_status"]) == 0)
    tg, tp, ty = (_np(best[k]).astype(np.float64) for k in ("T_greedy", "T_pipeline", "T_binary"))
    tb = _np(unsegmented["binomial"]).astype(np.float64)
    assert np.array_equal(_np(unsegmented["greedy"]), _np(unsegmented["binomial"]))      # q = 1: greedy is the binomial tree
    ratio = np.minimum(np.minimum(tb, tp), ty) / tg
    assert np.all(ratio >= 1.0)
    fig4 = [i for i, x in enumerate(probs) if x[0] == 64 and x[2] == 10 and x[3] == 0]
    r4 = {probs[i][1]: ratio[i] for i in fig4}
    assert r4[4] == 1.0 and r4[16] == 1.0 and _np(best["q_greedy"])[fig4[0]] == 1
    assert 1.4 <= max(r4.values()) <= 1.65 and max(r4, key=r4.get) in (256, 512, 1024)
    assert r4[65536] < r4[16384] < r4[4096] and r4[65536] < 1.1                         # the pipeline catches up
    # the region of the largest gain widens with p (Figure 5): count the message sizes with a gain above 30 %
    wide = {p: sum(1 for i, x in enumerate(probs) if x[0] == p and x[2] == 10 and x[3] == 0 and ratio[i] > 1.3)
            for p in (16, 64, 256, 1024)}
    assert wide[16] <= wide[64] <= wide[256] <= wide[1024] and wide[1024] > wide[16]
    idx = np.array([i for i, x in enumerate(probs) if x[0] <= 32 and x[1] <= 256][::3])
    ref = O.optimal_segmentation(host.take(idx), O.UNI, 65536)
    for key in ("greedy", "pipeline", "binary", "revopt"):
        assert np.array_equal(_np(best["T_" + key])[idx], ref["T_" + key]), key
        assert np.array_equal(_np(best["q_" + key])[idx], ref["q_" + key]), key


def test_theoretical_experiment_bidirectional_section_6_1(prs):
    """Section 6.1 with the machine of Figure 6 (alpha = 50000, beta = 6, gamma = 1), p = 4..1024, m = 2^10..2^27,
    every algorithm at its best power-of-two segment count up to 512: bi-greedy needs exactly the rounds of the
    reversed optimal broadcast (Table III), no tree algorithm beats it, it equals the binomial tree for small
    messages, the pipeline approaches it for large ones, and the butterfly comes close only for mid-size
    messages.  A sample is compared with the oracle trying each count."""
    probs = [(p, m) for p in (2 ** k for k in range(2, 11)) for m in (2 ** k for k in range(10, 28))]
    n = len(probs)
    host = prs_inputs.SweepConfigs(np.array([x[0] for x in probs], np.int32), np.zeros(n, np.int32),
                                   np.array([x[1] for x in probs], np.int64), np.full(n, 50000, np.int64),
                                   np.full(n, 6, np.int64), np.ones(n, np.int64), "i64")
    dev = prs.DeviceConfigs.from_host(host)
    best = prs.optimal_segmentation_batch(dev, prs.PRS_BI, 1024, 512)
    one = prs.DeviceConfigs.from_host(prs_inputs.SweepConfigs(host.p, np.ones(n, np.int32), host.m, host.alpha, host.beta,
                                                               host.gamma, "i64"))
    uns = prs.simulate_completion_batch(one, prs.PRS_BI, 1024, 1)
    _sync()
    assert np.all(_np(best["cfg_status"]) == 0)
    assert np.array_equal(_np(best["T_greedy"]), _np(best["T_revopt"])) and np.array_equal(_np(best["q_greedy"]), _np(best["q_revopt"]))
    tg = _np(best["T_greedy"]).astype(np.float64)
    rb, rp, ry = (_np(t).astype(np.float64) / tg for t in (uns["binomial"], best["T_pipeline"], best["T_binary"]))
    rf = _np(uns["butterfly"]) / tg
    assert np.all(np.minimum(np.minimum(rb, rp), ry) >= 1.0)
    row = [i for i, x in enumerate(probs) if x[0] == 64]
    assert rb[row[0]] == 1.0 and rb[row[1]] == 1.0 and np.all(np.diff(rb[row]) >= 0) and rb[row[-1]] > 5
    assert np.all(np.diff(rp[row]) < 0) and rp[row[-1]] < 1.2 and rp[row[0]] > 5
    assert np.all(ry[row] == 2.0)                                        # twice the rounds, whatever the segment size
    lowest = int(np.argmin(rf[row]))
    assert 0 < lowest < len(row) - 1 and 1.0 < rf[row][lowest] < 1.1 and rf[row[0]] > 1.5 and rf[row[-1]] > 1.5
    idx = np.array([i for i, x in enumerate(probs) if x[0] <= 16 and x[1] <= 2 ** 15][::2])
    ref = O.optimal_segmentation(host.take(idx), O.BI, 512)
    for key in ("greedy", "pipeline", "binary", "revopt"):
        assert np.array_equal(_np(best["T_" + key])[idx], ref["T_" + key]), key
        assert np.array_equal(_np(best["q_" + key])[idx], ref["q_" + key]), key


@pytest.mark.parametrize("p", [64, 1024])
def test_butterfly_threshold_by_bisection(prs, p):
    """Section 6.1: the largest beta/gamma for which some message size lets the butterfly beat the reversed
    optimal broadcast (= bi-greedy), found by bisection over the library's closed forms (every segment count
    1..512 for message sizes 2^4..2^22), takes the same steps as the bisection over the oracle's closed forms,
    stays below 5 and within a tenth of the closed form of the line."""
    ms = [2 ** k for k in range(4, 23)]
    mq = [(m, q) for m in ms for q in range(1, min(512, m) + 1)]
    n = len(mq)
    m_arr = np.array([x[0] for x in mq], np.int64)
    q_arr = np.array([x[1] for x in mq], np.int32)
    first = np.concatenate([[0], np.nonzero(np.diff(m_arr))[0] + 1])          # where each message size starts

    def wins_on_gpu(r):
        host = prs_inputs.SweepConfigs(np.full(n, p, np.int32), q_arr, m_arr, np.full(n, 1000.0), np.full(n, r), np.ones(n), "f64")
        got = prs.simulate_completion_batch(prs.DeviceConfigs.from_host(host), prs.PRS_BI, 1024, 512)
        _sync()
        rev, bf = _np(got["revopt"]), _np(got["butterfly"])
        best = np.minimum.reduceat(rev, first)
        return bool(np.any(bf[first] < best))

    lo_g = lo_o = 0.25
    hi_g = hi_o = 16.0
    for _ in range(8):
        mid = math.sqrt(lo_g * hi_g)
        lo_g, hi_g = (mid, hi_g) if wins_on_gpu(mid) else (lo_g, mid)
        mid = math.sqrt(lo_o * hi_o)
        lo_o, hi_o = (mid, hi_o) if O.butterfly_wins_somewhere(p, 1000.0, mid, 1.0, ms, 512) else (lo_o, mid)
    assert (lo_g, hi_g) == (lo_o, hi_o)
    assert hi_g < 5 and abs(math.sqrt(lo_g * hi_g) / O.butterfly_threshold_closed_form(p) - 1) < 0.1


def test_butterfly_threshold_entry_point(prs):
    """Section 6.1 on the device: the bracket of the largest beta/gamma at which the butterfly still beats
    bi-greedy's time for some message size, bisection step for step against the oracle's (same midpoints, same
    closed forms, so the brackets are equal bit for bit); for 4 to 1024 processors the line stays below 5, as the
    section says, and within a tenth of its closed form; a machine of one processor is reported, not run."""
    import torch
    ps = [4, 8, 16, 32, 64, 100, 128, 256, 512, 1000, 1024, 1]
    got = prs.butterfly_threshold_batch(torch.tensor(ps, dtype=torch.int32, device="cuda"), 1000.0, 512, 4, 22, 0.25, 16.0, 12)
    _sync()
    lo, hi, st = _np(got["ratio_below"]), _np(got["ratio_above"]), _np(got["cfg_status"])
    assert list(st) == [0] * 11 + [1] and np.isnan(lo[11]) and np.isnan(hi[11])
    for i in (1, 4, 5, 10):                                              # p = 8, 64, 100, 1024
        assert (lo[i], hi[i]) == O.butterfly_threshold_bisect(ps[i], 1000.0, 512, 4, 22, 0.25, 16.0, 12), ps[i]
    assert np.all(hi[:11] < 5) and np.all(hi[:11] - lo[:11] == (16.0 - 0.25) / 4096)
    for i in range(2, 11):                                               # from 16 processors on the line rises with p
        assert abs(0.5 * (lo[i] + hi[i]) / O.butterfly_threshold_closed_form(ps[i]) - 1) < 0.1, ps[i]
    grow = [0.5 * (lo[i] + hi[i]) for i in (2, 3, 4, 6, 7, 8, 10)]
    assert all(a < b for a, b in zip(grow, grow[1:]))
    # no steps: the caller's bracket comes back; another latency against the oracle as well
    same = prs.butterfly_threshold_batch(torch.tensor([64], dtype=torch.int32, device="cuda"), 10.0, 512, 4, 22, 0.25, 16.0, 0)
    other = prs.butterfly_threshold_batch(torch.tensor([64], dtype=torch.int32, device="cuda"), 10.0, 512, 4, 22, 0.25, 16.0, 9)
    _sync()
    assert (_np(same["ratio_below"])[0], _np(same["ratio_above"])[0]) == (0.25, 16.0)
    assert (_np(other["ratio_below"])[0], _np(other["ratio_above"])[0]) == O.butterfly_threshold_bisect(64, 10.0, 512, 4, 22, 0.25, 16.0, 9)
    with pytest.raises(prs.PrsError):
        prs.butterfly_threshold_batch(torch.tensor([64], dtype=torch.int32, device="cuda"), 10.0, 512, 4, 22, 16.0, 0.25, 3)


# --------------------------------------------------------------------------- unequal segmentation (Section 8)
_SUMMARY = ("T_best", "cuts_best", "n_best", "T_equi", "cuts_equi", "equi_optimal")


@pytest.mark.parametrize("grouping", [None, "64 lanes", "32 lanes", "16 lanes", "4 or 8 lanes"])
@pytest.mark.parametrize("cost", ["i64", "f64"])
def test_unequal_segmentation_matches_the_oracle(prs, cost, grouping):
    """Every segmentation of short messages of mixed length through uni-greedy, at every group size: all
    2^(m-1) times and the per-problem summary against the oracle running the segmentations one by one."""
    tuning = None if grouping is None else _GROUPINGS[grouping]
    rng = np.random.default_rng(808)
    n = 36
    p = rng.integers(2, 70, n).astype(np.int32)
    m = rng.integers(1, 10, n).astype(np.int64)
    p[:4] = [2, 3, 64, 65]; m[:4] = [9, 1, 9, 2]
    if cost == "i64":
        al, be, ga = (rng.integers(0, 12, n).astype(np.int64), rng.integers(1, 3, n).astype(np.int64),
                      rng.integers(0, 3, n).astype(np.int64))
    else:
        al, be, ga = 10.0 ** rng.uniform(-6, -5, n), 10.0 ** rng.uniform(-7, -5, n), 10.0 ** rng.uniform(-7, -5, n)
        al[5:9] = 1.0; be[5:9] = 0.0; ga[5:9] = 2.0 ** -52              # sums that collide in rounding
    p[4] = 1                                                            # not a valid problem
    m[9] = 12                                                           # longer than m_max
    host = prs_inputs.SweepConfigs(p, np.zeros(n, np.int32), m, al, be, ga, cost)
    dev = prs.DeviceConfigs.from_host(host)
    m_max = 9
    got = prs.unequal_segmentation_batch(dev, 70, m_max, tuning=tuning)
    _sync()
    st = _np(got["cfg_status"])
    T_all = _np(got["T_all"])
    for i in range(n):
        if i in (4, 9):
            assert st[i] == 1 and _np(got["n_best"])[i] == 0
            assert np.all(T_all[i] == -1) if cost == "i64" else np.all(np.isnan(T_all[i]))
            continue
        assert st[i] == 0
        ref = O.unequal_segmentation(int(p[i]), int(m[i]), al[i].item(), be[i].item(), ga[i].item(), cost)
        nc = 1 << (int(m[i]) - 1)
        assert np.array_equal(T_all[i, :nc], ref["T_all"]), i
        assert np.all(T_all[i, nc:] == -1) if cost == "i64" else np.all(np.isnan(T_all[i, nc:]))
        for key in _SUMMARY:
            assert _np(got[key])[i].item() == ref[key], (i, key)


def test_unequal_segmentation_of_one_unit(prs):
    """m_max = 1: one segmentation per problem, the unsegmented message, which is the binomial tree."""
    p = np.array([2, 3, 17, 64, 1000], np.int32)
    n = len(p)
    host = prs_inputs.SweepConfigs(p, np.zeros(n, np.int32), np.ones(n, np.int64), np.full(n, 3, np.int64),
                                   np.full(n, 2, np.int64), np.ones(n, np.int64), "i64")
    got = prs.unequal_segmentation_batch(prs.DeviceConfigs.from_host(host), 1024, 1)
    _sync()
    want = np.array([math.ceil(math.log2(x)) * (3 + 2 + 1) for x in p])
    assert np.array_equal(_np(got["T_all"])[:, 0], want) and np.array_equal(_np(got["T_best"]), want)
    assert np.array_equal(_np(got["T_equi"]), want) and np.all(_np(got["n_best"]) == 1)
    assert np.all(_np(got["equi_optimal"]) == 3) and np.all(_np(got["cuts_best"]) == 0)


def test_unequal_segmentation_reproduces_table4(prs):
    """The paper's experiment at full size (m = 10, beta = 1, 29 values of alpha, gamma in {0, 1}, 17 values of
    p up to 1024: 986 problems x 512 segmentations) on the GPU, checked against the printed table: the same 61
    problems are optimised only by unequal segmentations, with the printed optimal sets, best
    equi-segmentations and ratios, a largest gain of 7.3 % and a mean gain of 2.0 %."""
    import os
    alphas = list(range(0, 11)) + list(range(20, 101, 10)) + list(range(200, 1001, 100))
    ps = sorted([2 ** k for k in range(2, 11)] + [3 * 2 ** k for k in range(1, 9)])
    probs = [(p, a, g) for p in ps for a in alphas for g in (0, 1)]
    assert len(probs) == 986
    n = len(probs)
    host = prs_inputs.SweepConfigs(np.array([x[0] for x in probs], np.int32), np.zeros(n, np.int32), np.full(n, 10, np.int64),
                                   np.array([x[1] for x in probs], np.int64), np.ones(n, np.int64),
                                   np.array([x[2] for x in probs], np.int64), "i64")
    dev = prs.DeviceConfigs.from_host(host)
    got = prs.unequal_segmentation_batch(dev, 1024, 10)
    _sync()
    assert np.all(_np(got["cfg_status"]) == 0)
    T_all, T_best, T_equi = _np(got["T_all"]), _np(got["T_best"]), _np(got["T_equi"])
    flags, n_best, cuts_equi = _np(got["equi_optimal"]), _np(got["n_best"]), _np(got["cuts_equi"])
    comps = O.compositions(10)
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table4_unequal_segmentation.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p, a, g, ratio, equi, opt = line.split()
            rows[(int(p), int(a), int(g))] = (ratio, tuple(map(int, equi.split(","))),
                                              sorted(tuple(map(int, s.split(","))) for s in opt.split(";")))
    unequal_only = [i for i in range(n) if not flags[i] & 2]
    assert sorted(probs[i] for i in unequal_only) == sorted(rows)
    gains = []
    for i in unequal_only:
        ratio, equi, opt = rows[probs[i]]
        assert f"{T_equi[i] / T_best[i]:.4f}" == ratio
        assert sorted(comps[c] for c in np.nonzero(T_all[i] == T_best[i])[0]) == opt and n_best[i] == len(opt)
        assert T_all[i, comps.index(equi)] == T_equi[i] and comps.index(equi) >= cuts_equi[i]
        gains.append(T_equi[i] / T_best[i] - 1.0)
    assert f"{max(gains) * 100:.1f}" == "7.3" and f"{sum(gains) / len(gains) * 100:.1f}" == "2.0"
    # where an equi-segmentation is optimal in the section's wider sense, the ones cut from a count may still lose
    assert np.all(T_equi >= T_best) and np.all((flags & 1) == (T_equi == T_best))
    # sampled problems element by element against the oracle
    for i in (0, 57, 200, 333, 640):
        p, a, g = probs[i]
        if p > 96:
            continue
        ref = O.unequal_segmentation(p, 10, a, 1, g)
        assert np.array_equal(T_all[i], ref["T_all"])
    big = [i for i in range(n) if probs[i][0] == 1024][:2]
    for i in big:                                                       # two of the largest, a few segmentations each
        p, a, g = probs[i]
        for c in (0, 1, 255, 300, 511):
            assert T_all[i, c] == O.uni_greedy(p, list(comps[c]), a, 1, g, want_schedule=False).T


# --------------------------------------------------------------------------- replay
def _replay_case(prs, p, sizes, model, seg_off, dtype, cost=("i64", 2, 1, 1), strided=False):
    import torch
    cst, a, b, g = cost
    s = (O.uni_greedy if model == 0 else O.bi_greedy)(p, sizes, a, b, g, cst)
    n = int(seg_off[-1])
    buf = prs_inputs.replay_buffers(p, n, dtype)
    want = O.replay(p, seg_off, s.src, s.dst, s.seg, buf)
    dbuf = torch.from_numpy(buf).cuda()
    if strided:
        wide = torch.zeros((p, n + 3), dtype=dbuf.dtype, device="cuda")
        wide[:, :n] = dbuf
        dbuf = wide[:, :n]
    out, st = prs.replay_reduction(p, len(sizes), seg_off, torch.from_numpy(s.src).cuda(), torch.from_numpy(s.dst).cuda(),
                                   torch.from_numpy(s.seg).cuda(), dbuf)
    _sync()
    assert int(st.item()) == 0
    assert _np(out).tobytes() == want.tobytes(), (p, model, dtype)


@pytest.mark.parametrize("dtype", ["i32", "f32"])
@pytest.mark.parametrize("model", [0, 1])
def test_replay_small_ragged(prs, model, dtype):
    q = 5
    off = np.array([0, 1000, 2000, 3000, 4000, 4321], np.int64)          # aligned starts, ragged end
    _replay_case(prs, 23, [4] * 4 + [2], model, off, dtype)
    off = np.array([0, 37, 74, 111, 148, 150], np.int64)                 # unaligned starts: scalar path
    _replay_case(prs, 37, [4] * 4 + [1], model, off, dtype)
    _replay_case(prs, 2, [3], model, np.array([0, 5], np.int64), dtype)
    _replay_case(prs, 130, [4] * q, model, np.arange(q + 1, dtype=np.int64) * 2048, dtype, strided=True)


def _replay_pairs(prs, p, q, pairs, seg_off, dtype, op="sum", strided=False, special=False):
    """One replay of a given pair list: the library against the oracle, bit for bit."""
    import torch
    src, dst, seg = pairs
    n = int(seg_off[-1])
    buf = prs_inputs.replay_buffers(p, n, dtype)
    if special:                                                         # signed zeros and a NaN in floating-point columns
        buf[:, 0] = -0.0; buf[p // 2, 0] = 0.0
        buf[:, 1] = -0.0
        buf[p - 1, 2] = np.nan
    want = O.replay(p, seg_off, src, dst, seg, buf, op)
    dbuf = torch.from_numpy(buf).cuda()
    if strided:
        wide = torch.zeros((p, n + 6), dtype=dbuf.dtype, device="cuda")
        wide[:, :n] = dbuf
        dbuf = wide[:, :n]
    out, st = prs.replay_reduction(p, q, seg_off, torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda(),
                                   torch.from_numpy(seg).cuda(), dbuf, op=prs.PRS_OP_MAX if op == "max" else prs.PRS_OP_SUM)
    _sync()
    assert int(st.item()) == 0
    assert _np(out).tobytes() == want.tobytes(), (p, q, dtype, op)


@pytest.mark.parametrize("op", ["sum", "max"])
@pytest.mark.parametrize("dtype", ["i32", "f32", "i64", "f64"])
def test_replay_element_types_and_operations(prs, dtype, op):
    """Uni- and bi-greedy schedules on 32- and 64-bit integers and floating point, summed or maximised:
    vector path (aligned segments), scalar path (unaligned), ragged ends, strided rows."""
    q = 5
    sizes = [4] * 4 + [2]
    for model in (0, 1):
        s = (O.uni_greedy if model == 0 else O.bi_greedy)(29, sizes, 2, 1, 1)
        pairs = (s.src, s.dst, s.seg)
        _replay_pairs(prs, 29, q, pairs, np.array([0, 1000, 2000, 3000, 4000, 4321], np.int64), dtype, op)
        _replay_pairs(prs, 29, q, pairs, np.array([0, 37, 74, 111, 148, 151], np.int64), dtype, op)
        _replay_pairs(prs, 29, q, pairs, np.arange(q + 1, dtype=np.int64) * 1536, dtype, op, strided=True)
    if dtype in ("f32", "f64") and op == "max":
        s = O.uni_greedy(29, sizes, 2, 1, 1)
        _replay_pairs(prs, 29, q, (s.src, s.dst, s.seg), np.arange(q + 1, dtype=np.int64) * 512, dtype, op, special=True)


@pytest.mark.parametrize("tree", ["pipeline", "binomial", "binary"])
def test_replay_of_baseline_trees(prs, tree):
    """The same kernel on the trees of Section 4 (pipeline chain: the deepest combine tree there is;
    binomial; binary), every segment through the same tree."""
    import baseline_trees as B
    build = getattr(B, tree)
    for p, q, per in ((2, 1, 5), (13, 3, 1000), (64, 4, 2048), (200, 2, 700)):
        off = np.arange(q + 1, dtype=np.int64) * per
        for dtype in ("f32", "i32", "f64"):
            _replay_pairs(prs, p, q, build(p, q), off, dtype)


def test_replay_rejects_a_schedule_that_is_not_a_tree(prs):
    import torch
    p, q = 4, 1
    src = torch.tensor([1, 1, 3], dtype=torch.int32).cuda()             # processor 1 sends twice, 2 never
    dst = torch.tensor([0, 2, 0], dtype=torch.int32).cuda()
    seg = torch.zeros(3, dtype=torch.int32).cuda()
    buf = torch.ones((p, 8), dtype=torch.float32).cuda()
    out, st = prs.replay_reduction(p, q, np.array([0, 8], np.int64), src, dst, seg, buf)
    _sync()
    assert int(st.item()) == 1


@pytest.mark.parametrize("dtype", ["i32", "f32"])
def test_replay_full_size_sampled_columns(prs, dtype):
    """p = 256, 64 segments, 2^22 elements per buffer: the benchmark's replay.  Buffers are drawn on
    the device; the oracle replays sampled element columns copied back from it."""
    import torch
    host = prs_inputs.replay_config()
    p, q, n = 256, 64, 1 << 22
    sizes = O.equi_sizes(int(host.m[0]), q)
    s = O.uni_greedy(p, sizes, 1e-5, 1e-9, 1e-10, "f64")
    gen = torch.Generator(device="cuda").manual_seed(prs_inputs.SEED_REPLAY)
    if dtype == "i32":
        buf = torch.randint(-2 ** 20, 2 ** 20 + 1, (p, n), dtype=torch.int32, device="cuda", generator=gen)
    else:
        buf = torch.randn((p, n), dtype=torch.float32, device="cuda", generator=gen)
    seg_off = np.arange(q + 1, dtype=np.int64) * (n // q)
    dev = prs.DeviceConfigs.from_host(host)
    off = prs.prs_pair_offsets(dev, 256, 64)
    sch = prs.greedy_schedule_batch(dev, 0, 256, 64, off, (p - 1) * q)
    _sync()
    assert np.array_equal(_np(sch["src"]), s.src) and np.array_equal(_np(sch["dst"]), s.dst)
    out, st = prs.replay_reduction(p, q, seg_off, sch["src"], sch["dst"], sch["seg"], buf)
    _sync()
    assert int(st.item()) == 0
    rng = np.random.default_rng(7)
    cols = np.unique(np.concatenate([rng.integers(0, n, 3000), seg_off[:-1], seg_off[1:] - 1]))
    sub = buf[:, torch.from_numpy(cols).cuda()].cpu().numpy()
    col_seg = np.searchsorted(seg_off, cols, side="right") - 1
    # replay the sampled columns: one pseudo-segment per original segment, columns grouped by it
    order = np.argsort(col_seg, kind="stable")
    sub = np.ascontiguousarray(sub[:, order])
    sub_off = np.concatenate([[0], np.cumsum(np.bincount(col_seg, minlength=q))]).astype(np.int64)
    want = O.replay(p, sub_off, s.src, s.dst, s.seg, sub)
    got = _np(out)[cols[order]]
    assert got.tobytes() == want.tobytes()
    if dtype == "i32":
        assert np.array_equal(got, sub.sum(axis=0, dtype=np.int64).astype(np.int32))
