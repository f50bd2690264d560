"""TEST INFRASTRUCTURE: ctypes front end of the CPU oracle (oracle/prs_oracle.c).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It never imports the GPU package, and the GPU package never imports
it.  `build()` compiles the C file with gcc; loading builds on demand.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, "prs_oracle.c"), os.path.join(_HERE, "greedy_body.inc")]
_LIB_PATH = os.path.join(_HERE, "_build", "libprs_oracle.so")
_lib = None

UNI, BI = 0, 1
MODE_LITERAL, MODE_EVENT, MODE_PRUNE, MODE_LISTING_ONLY = 0, 1, 2, 4


def build(force: bool = False) -> str:
    """Compile the oracle.  No FMA contraction, no fast-math: every product and
    sum is rounded on its own, as the cost model is stated."""
    os.makedirs(os.path.dirname(_LIB_PATH), exist_ok=True)
    stale = force or not os.path.exists(_LIB_PATH) or any(
        os.path.getmtime(s) > os.path.getmtime(_LIB_PATH) for s in _SRC)
    if stale:
        tmp = _LIB_PATH + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fwrapv",
                               "-Wall", "-Wextra", "-shared", "-fPIC", "-o", tmp, _SRC[0]])
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_exhaustive_uni_i64.restype = C.c_int64
        _lib.orc_ceil_log2.restype = C.c_int32
        for suf in ("_i64", "_f64"):
            getattr(_lib, "orc_binomial_construct" + suf).restype = C.c_int64 if suf == "_i64" else C.c_double
            getattr(_lib, "orc_pipeline_construct" + suf).restype = C.c_int64 if suf == "_i64" else C.c_double
            getattr(_lib, "orc_binary_construct" + suf).restype = C.c_int64 if suf == "_i64" else C.c_double
            getattr(_lib, "orc_butterfly_steps" + suf).restype = C.c_double
    return _lib


def _ptr(a, ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def _ct(cost):
    if cost == "i64":
        return np.int64, C.c_int64, "_i64"
    if cost == "f64":
        return np.float64, C.c_double, "_f64"
    raise ValueError(cost)


def ceil_log2(v: int) -> int:
    return int(lib().orc_ceil_log2(C.c_int64(v)))


def segmentation(m: int, q_req: int):
    """(q_eff, sz_full, sz_last) of the equi-segmentation of m."""
    q, s, l = C.c_int64(), C.c_int64(), C.c_int64()
    lib().orc_segmentation(C.c_int64(int(m)), C.c_int64(int(q_req)), C.byref(q), C.byref(s), C.byref(l))
    return q.value, s.value, l.value


def equi_sizes(m: int, q_req: int) -> np.ndarray:
    q, s, l = segmentation(m, q_req)
    sizes = np.full(q, s, dtype=np.int64)
    sizes[-1] = l
    return sizes


@dataclass
class Schedule:
    src: np.ndarray
    dst: np.ndarray
    seg: np.ndarray
    t: np.ndarray
    T: object
    status: int = 0
    x_final: np.ndarray | None = None
    root_done: np.ndarray | None = None
    n_visits: int = 0


def uni_greedy(p, sizes, alpha, beta, gamma, cost="i64", want_schedule=True) -> Schedule:
    npt, ct, suf = _ct(cost)
    sizes = np.ascontiguousarray(sizes, dtype=np.int64)
    q = int(sizes.shape[0])
    n = (p - 1) * q if want_schedule else 0
    src = np.empty(n, np.int32) if want_schedule else None
    dst = np.empty(n, np.int32) if want_schedule else None
    seg = np.empty(n, np.int32) if want_schedule else None
    t = np.empty(n, npt) if want_schedule else None
    xf = np.empty(p, npt)
    T = ct()
    rc = getattr(lib(), "orc_uni_greedy" + suf)(
        C.c_int32(p), C.c_int32(q), _ptr(sizes, C.c_int64), ct(alpha), ct(beta), ct(gamma),
        _ptr(src, C.c_int32), _ptr(dst, C.c_int32), _ptr(seg, C.c_int32), _ptr(t, ct), _ptr(xf, ct), C.byref(T))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return Schedule(src, dst, seg, t, T.value, 0, xf)


def uni_greedy_time(p, sizes, alpha, beta, gamma, cost="i64"):
    """Completion time of uni-greedy from the ready times alone (a heap of values, no processor identities):
    for machines of tens of thousands of processors."""
    _, ct, suf = _ct(cost)
    sizes = np.ascontiguousarray(sizes, dtype=np.int64)
    T = ct()
    rc = getattr(lib(), "orc_uni_greedy_values" + suf)(C.c_int32(p), C.c_int32(int(sizes.shape[0])), _ptr(sizes, C.c_int64),
                                                       ct(alpha), ct(beta), ct(gamma), C.byref(T))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return T.value


def bi_greedy(p, sizes, alpha, beta, gamma, cost="i64", mode=MODE_EVENT, want_schedule=True) -> Schedule:
    npt, ct, suf = _ct(cost)
    sizes = np.ascontiguousarray(sizes, dtype=np.int64)
    q = int(sizes.shape[0])
    n = (p - 1) * q if want_schedule else 0
    src = np.empty(n, np.int32) if want_schedule else None
    dst = np.empty(n, np.int32) if want_schedule else None
    seg = np.empty(n, np.int32) if want_schedule else None
    t = np.empty(n, npt) if want_schedule else None
    rd = np.zeros(q, npt)
    T = ct()
    npairs, nvis = C.c_int64(), C.c_int64()
    rc = getattr(lib(), "orc_bi_greedy" + suf)(
        C.c_int32(p), C.c_int32(q), _ptr(sizes, C.c_int64), ct(alpha), ct(beta), ct(gamma), C.c_int(mode),
        C.c_int64(n), _ptr(src, C.c_int32), _ptr(dst, C.c_int32), _ptr(seg, C.c_int32), _ptr(t, ct),
        _ptr(rd, ct), C.byref(npairs), C.byref(nvis), C.byref(T))
    if rc < 0:
        raise MemoryError("oracle allocation failed")
    if want_schedule and rc == 0:
        assert npairs.value == n, (npairs.value, n)
    return Schedule(src, dst, seg, t, T.value, rc, None, rd, nvis.value)


def closed_forms(model, p, q, m, sz, alpha, beta, gamma, cost="i64"):
    """dict of the closed-form times: binomial, pipeline, binary, revopt (cost
    type), butterfly and lower_bound (always float)."""
    npt, ct, suf = _ct(cost)
    out = np.empty(4, npt)
    getattr(lib(), "orc_closed_forms" + suf)(C.c_int(model), C.c_int32(p), C.c_int32(q), C.c_int64(int(m)),
                                             C.c_int64(int(sz)), ct(alpha), ct(beta), ct(gamma), _ptr(out, ct))
    o2 = np.empty(2, np.float64)
    lib().orc_butterfly_and_bound(C.c_int(model), C.c_int32(p), C.c_int64(int(m)), C.c_double(float(alpha)),
                                  C.c_double(float(beta)), C.c_double(float(gamma)), _ptr(o2, C.c_double))
    return {"binomial": out[0].item(), "pipeline": out[1].item(), "binary": out[2].item(),
            "revopt": out[3].item(), "butterfly": float(o2[0]), "lower_bound": float(o2[1])}


def binomial_construct(p, m, alpha, beta, gamma, cost="i64"):
    _, ct, suf = _ct(cost)
    return getattr(lib(), "orc_binomial_construct" + suf)(C.c_int32(p), C.c_int64(int(m)), ct(alpha), ct(beta), ct(gamma))


def pipeline_construct(p, sizes, alpha, beta, gamma, cost="i64"):
    _, ct, suf = _ct(cost)
    sizes = np.ascontiguousarray(sizes, dtype=np.int64)
    return getattr(lib(), "orc_pipeline_construct" + suf)(C.c_int32(p), C.c_int32(sizes.shape[0]), _ptr(sizes, C.c_int64),
                                                          ct(alpha), ct(beta), ct(gamma))


def binary_construct(model, p, sizes, alpha, beta, gamma, cost="i64"):
    """Completion time of the binary tree of Section 4 built pair by pair (heap-shaped tree, two senders per
    receiver in turn, segments in order), under either port model."""
    _, ct, suf = _ct(cost)
    sizes = np.ascontiguousarray(sizes, dtype=np.int64)
    return getattr(lib(), "orc_binary_construct" + suf)(C.c_int(model), C.c_int32(p), C.c_int32(sizes.shape[0]),
                                                        _ptr(sizes, C.c_int64), ct(alpha), ct(beta), ct(gamma))


def butterfly_steps(p, m, alpha, beta, gamma, cost="f64"):
    _, ct, suf = _ct(cost)
    return getattr(lib(), "orc_butterfly_steps" + suf)(C.c_int32(p), C.c_int64(int(m)), ct(alpha), ct(beta), ct(gamma))


def exhaustive_uni(p, sizes, alpha, beta, gamma) -> int:
    sizes = np.ascontiguousarray(sizes, dtype=np.int64)
    return int(lib().orc_exhaustive_uni_i64(C.c_int32(p), C.c_int32(sizes.shape[0]), _ptr(sizes, C.c_int64),
                                            C.c_int64(alpha), C.c_int64(beta), C.c_int64(gamma)))


def total_order_key(x: np.ndarray) -> np.ndarray:
    """IEEE total order of floating-point values as signed integers: the bit pattern read as sign and
    magnitude (-NaN < -inf < ... < -0 < +0 < ... < +inf < +NaN)."""
    it = np.int32 if x.dtype == np.float32 else np.int64
    bits = x.view(it)
    mag = it(np.iinfo(it).max)                                  # every bit but the sign
    return np.where(bits < 0, bits ^ mag, bits)


def replay(p, seg_elem_offset, src, dst, seg, buf: np.ndarray, op: str = "sum") -> np.ndarray:
    """Section 4: the receiver of a pair combines the segment it received with its own.  Applies
    buf[dst, segment] = buf[dst, segment] (+ or max) buf[src, segment] pair by pair, in the order given, on a
    copy of buf (p rows); returns row 0.  int32 and float32 sums run in the C oracle; the other element
    types and the maximum are the same loop with numpy's element-wise operations (wrapping integer add,
    IEEE add, maximum in the IEEE total order for floating point)."""
    work = np.ascontiguousarray(buf).copy()
    assert work.shape[0] == p
    off = np.ascontiguousarray(seg_elem_offset, dtype=np.int64)
    src = np.ascontiguousarray(src, np.int32); dst = np.ascontiguousarray(dst, np.int32)
    seg = np.ascontiguousarray(seg, np.int32)
    if op == "sum" and work.dtype in (np.int32, np.float32):
        fn, ct = (lib().orc_replay_i32, C.c_int32) if work.dtype == np.int32 else (lib().orc_replay_f32, C.c_float)
        fn(C.c_int32(p), C.c_int64(work.shape[1]), _ptr(off, C.c_int64), C.c_int64(src.shape[0]),
           _ptr(src, C.c_int32), _ptr(dst, C.c_int32), _ptr(seg, C.c_int32), _ptr(work, ct))
        return work[0].copy()
    if work.dtype not in (np.int32, np.int64, np.float32, np.float64) or op not in ("sum", "max"):
        raise TypeError((work.dtype, op))
    floating = work.dtype in (np.float32, np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        for s, d, k in zip(src.tolist(), dst.tolist(), seg.tolist()):
            a, b = work[d, off[k]:off[k + 1]], work[s, off[k]:off[k + 1]]
            if op == "sum":
                a += b                                            # numpy integer addition wraps, floating point is IEEE
            elif floating:
                a[...] = np.where(total_order_key(a) < total_order_key(b), b, a)
            else:
                np.maximum(a, b, out=a)
    return work[0].copy()


# ---------------------------------------------------------------------------
# Batch front end: one configuration after another, results in the layout the
# C-ABI library uses, so tests can compare array against array.
# ---------------------------------------------------------------------------
@dataclass
class BatchResult:
    T_greedy: np.ndarray
    T_binomial: np.ndarray
    T_pipeline: np.ndarray
    T_binary: np.ndarray
    T_revopt: np.ndarray
    T_butterfly: np.ndarray
    T_lower_bound: np.ndarray
    q_eff: np.ndarray
    status: np.ndarray


def simulate_batch(cfgs, model, mode=MODE_EVENT | MODE_PRUNE, index=None) -> BatchResult:
    """Completion times and baselines for every configuration (or those in
    `index`), computed one by one."""
    npt, _, _ = _ct(cfgs.cost)
    idx = np.arange(len(cfgs)) if index is None else np.asarray(index)
    n = idx.shape[0]
    res = BatchResult(*(np.zeros(n, npt) for _ in range(5)), np.zeros(n), np.zeros(n),
                      np.zeros(n, np.int32), np.zeros(n, np.int32))
    for o, i in enumerate(idx):
        p, m, qr = int(cfgs.p[i]), int(cfgs.m[i]), int(cfgs.q_req[i])
        a, b, g = cfgs.alpha[i].item(), cfgs.beta[i].item(), cfgs.gamma[i].item()
        q, sz, _ = segmentation(m, qr)
        sizes = equi_sizes(m, qr)
        if model == UNI:
            s = uni_greedy(p, sizes, a, b, g, cfgs.cost, want_schedule=False)
        else:
            s = bi_greedy(p, sizes, a, b, g, cfgs.cost, mode=mode, want_schedule=False)
        cf = closed_forms(model, p, q, m, sz, a, b, g, cfgs.cost)
        res.T_greedy[o] = s.T
        res.T_binomial[o] = cf["binomial"]; res.T_pipeline[o] = cf["pipeline"]
        res.T_binary[o] = cf["binary"]; res.T_revopt[o] = cf["revopt"]
        res.T_butterfly[o] = cf["butterfly"]; res.T_lower_bound[o] = cf["lower_bound"]
        res.q_eff[o] = q
        res.status[o] = s.status
    return res


def optimal_segmentation(cfgs, model, q_max, mode=MODE_EVENT | MODE_PRUNE):
    """Sections 5.2 and 6.1: every algorithm is compared at the segmentation that suits it best.  For each
    problem (p, m, alpha, beta, gamma) -- cfgs.q_req is not read -- the segment counts 1, 2, 4, ... <= q_max are
    tried one after the other with the equi-segmentation of Section 2; per algorithm (greedy of `model`,
    pipeline, binary tree, reversed optimal broadcast) the smallest completion time and the first count that
    reaches it are returned as dict(T_greedy, q_greedy, ...)."""
    import copy
    cands = []
    q = 1
    while q <= q_max:
        cands.append(q)
        q *= 2
    n = len(cfgs)
    names = ("greedy", "pipeline", "binary", "revopt")
    best_T = {a: None for a in names}
    best_q = {a: np.zeros(n, np.int32) for a in names}
    for q in cands:
        trial = copy.copy(cfgs)
        trial.q_req = np.full(n, q, np.int32)
        r = simulate_batch(trial, model, mode)
        cols = {"greedy": r.T_greedy, "pipeline": r.T_pipeline, "binary": r.T_binary, "revopt": r.T_revopt}
        for a in names:
            if best_T[a] is None:
                best_T[a] = cols[a].copy()
                best_q[a][:] = q
            else:
                better = cols[a] < best_T[a]                      # strictly: ties keep the smaller count
                best_T[a][better] = cols[a][better]
                best_q[a][better] = q
    out = {}
    for a in names:
        out["T_" + a] = best_T[a]
        out["q_" + a] = best_q[a]
    return out


def compositions(m: int):
    """The 2^(m-1) ways of cutting m units into consecutive segments, indexed by cut pattern: bit b of the
    index set = a segment ends after unit b+1.  Index 0 is (m,), index 2^(m-1)-1 is (1, ..., 1)."""
    out = []
    for cuts in range(1 << (m - 1)):
        parts, cur = [], 1
        for b in range(m - 1):
            if cuts >> b & 1:
                parts.append(cur)
                cur = 1
            else:
                cur += 1
        parts.append(cur)
        out.append(tuple(parts))
    return out


def unequal_segmentation(p, m, alpha, beta, gamma, cost="i64"):
    """Section 8: the message is m units long and every segmentation of it is run through uni-greedy, one
    after the other.  Returns dict(T_all, T_best, cuts_best, n_best, T_equi, cuts_equi, equi_optimal):
    T_best the smallest time, cuts_best the smallest cut pattern reaching it, n_best how many do; T_equi /
    cuts_equi the same over the equi-segmentations (those Section 2 cuts from a segment count 1..m);
    equi_optimal bit 0: T_equi == T_best, bit 1: some optimal segmentation has equal sizes except a last
    one that is not larger (the section's wording of "equi-segmentation")."""
    comps = compositions(m)
    T_all = [uni_greedy(p, list(c), alpha, beta, gamma, cost, want_schedule=False).T for c in comps]
    T_best = min(T_all)
    winners = [i for i, t in enumerate(T_all) if t == T_best]
    by_count = {tuple(int(v) for v in equi_sizes(m, k)) for k in range(1, m + 1)}
    equi = [i for i, c in enumerate(comps) if c in by_count]
    T_equi = min(T_all[i] for i in equi)
    cuts_equi = min(i for i in equi if T_all[i] == T_equi)
    wide = any(all(x == comps[i][0] for x in comps[i][:-1]) and comps[i][-1] <= comps[i][0] for i in winners)
    return dict(T_all=np.array(T_all), T_best=T_best, cuts_best=winners[0], n_best=len(winners), T_equi=T_equi,
                cuts_equi=cuts_equi, equi_optimal=(1 if T_equi == T_best else 0) | (2 if wide else 0))


def butterfly_threshold_closed_form(p: int) -> float:
    """Section 6.1 (the figure of parameters for which the butterfly can beat the reversed optimal broadcast, i.e.
    bi-greedy): the largest beta/gamma for which some message size lets the butterfly win, with the segment count
    treated as a real number.  From Table III, with L = ceil(log2 p): the broadcast-based time at its best
    segment size is (sqrt((L-1) alpha) + sqrt((beta+gamma) m))^2, the butterfly's is
    2 L alpha + (2 beta + gamma)(p-1)/p m.  Their difference is A + B x^2 - C x in x = sqrt(m) with
    A = (L+1) alpha, B = beta (p-2)/p - gamma/p, C = 2 sqrt((L-1) alpha (beta+gamma)); it is negative for some
    x exactly when C^2 > 4 A B, in which alpha cancels:
        (L-1)(beta+gamma) > (L+1)(beta (p-2)/p - gamma/p).
    Solved for beta/gamma this gives the value returned.  (p >= 4.)"""
    L = ceil_log2(p)
    return ((L - 1) + (L + 1) / p) / ((L + 1) * (p - 2) / p - (L - 1))


def butterfly_wins_somewhere(p, alpha, beta, gamma, m_values, q_max) -> bool:
    """True if for one of the message sizes the butterfly's time (Table III) is below the reversed optimal
    broadcast's time at the best of the segment counts 1..q_max, each tried in turn."""
    for m in m_values:
        best, butterfly = None, None
        for q_req in range(1, min(q_max, m) + 1):
            q, sz, _ = segmentation(m, q_req)
            cf = closed_forms(BI, p, q, m, sz, alpha, beta, gamma, "f64")
            butterfly = cf["butterfly"]
            best = cf["revopt"] if best is None or cf["revopt"] < best else best
        if butterfly < best:
            return True
    return False


def butterfly_threshold_bisect(p, alpha, q_max, m_log2_first, m_log2_last, lo, hi, steps):
    """Section 6.1: bracket of the largest beta/gamma (gamma = 1) at which the butterfly beats the reversed optimal
    broadcast for some message size 2^k, by bisection from [lo, hi] (wins at lo, not at hi): `steps` times the
    midpoint lo + (hi - lo)/2 replaces lo if the butterfly wins there, else hi.  Returns (lo, hi)."""
    ms = [2 ** k for k in range(m_log2_first, m_log2_last + 1)]
    for _ in range(steps):
        mid = lo + (hi - lo) * 0.5
        if butterfly_wins_somewhere(p, float(alpha), mid, 1.0, ms, q_max):
            lo = mid
        else:
            hi = mid
    return lo, hi
