"""Schedule validator used by the tests: written from the machine model of the
paper (Section 2 and Section 5, first paragraphs), independent of both the
oracle and the GPU library.  It checks a list of (segment, src, dst, t_start)
pairs, it does not construct one."""
from __future__ import annotations

from collections import defaultdict


def validate(model, p, c, g, seg, src, dst, t, in_order=None, check_overlap=True, check_comm_comp=True):
    """model: 'uni' or 'bi'.  c[j], g[j]: tcomm / tcomp of segment j.
    Returns (completion_time, list_of_problems)."""
    q = len(c)
    if in_order is None:
        in_order = model == "uni"
    problems = []
    n = len(seg)
    if n != (p - 1) * q:
        problems.append(f"pair count {n} != (p-1)q = {(p - 1) * q}")
    sends = defaultdict(list)      # proc -> [(start, end, seg)]
    recvs = defaultdict(list)      # proc -> [(start, comm_end, comp_end, seg)]
    sent = set()
    for e in range(n):
        j, a, b, ts = int(seg[e]), int(src[e]), int(dst[e]), t[e]
        if not (0 <= j < q and 0 <= a < p and 0 <= b < p):
            problems.append(f"pair {e}: out of range"); continue
        if a == 0:
            problems.append(f"pair {e}: the root sends")
        if a == b:
            problems.append(f"pair {e}: self send")
        if (a, j) in sent:
            problems.append(f"pair {e}: processor {a} sends segment {j} twice")
        sent.add((a, j))
        if (b, j) in sent and b != a:
            # receiver must still hold segment j
            if any(s[2] == j and s[0] <= ts for s in sends[b]):
                problems.append(f"pair {e}: receiver {b} already sent segment {j}")
        sends[a].append((ts, ts + c[j], j))
        recvs[b].append((ts, ts + c[j], (ts + c[j]) + g[j], j))
    for i in range(1, p):
        for j in range(q):
            if (i, j) not in sent:
                problems.append(f"processor {i} never sends segment {j}")

    def overlap(a0, a1, b0, b1):
        return a0 < b1 and b0 < a1

    for i in range(p):
        sv, rv = sorted(sends[i]), sorted(recvs[i])
        if not check_overlap:
            break
        for k in range(len(sv) - 1):
            if sv[k][1] > sv[k + 1][0]:
                problems.append(f"proc {i}: two sends overlap")
        for k in range(len(rv) - 1):
            if rv[k][2] > rv[k + 1][0]:
                problems.append(f"proc {i}: receive/combine intervals overlap")
        for s in sv:
            for r in rv:
                if model == "uni" and overlap(s[0], s[1], r[0], r[2]):
                    problems.append(f"proc {i}: sends while receiving/combining (one port)")
                if model == "bi" and check_comm_comp and r[1] < r[2] and overlap(s[0], s[1], r[1], r[2]):
                    problems.append(f"proc {i}: communication overlaps computation")
    # a processor forwards segment j only after every contribution it received for j is combined
    for i in range(1, p):
        send_time = {s[2]: s[0] for s in sends[i]}
        for r in recvs[i]:
            if r[3] in send_time and r[2] > send_time[r[3]]:
                problems.append(f"proc {i}: sends segment {r[3]} before combining a received part")
    if in_order:
        for i in range(p):
            ev = [(s[0], s[1], s[2]) for s in sends[i]] + [(r[0], r[2], r[3]) for r in recvs[i]]
            last_end = defaultdict(lambda: None)
            first_start = defaultdict(lambda: None)
            for (a0, a1, j) in ev:
                last_end[j] = a1 if last_end[j] is None else max(last_end[j], a1)
                first_start[j] = a0 if first_start[j] is None else min(first_start[j], a0)
            js = sorted(last_end)
            for u, v in zip(js, js[1:]):
                if last_end[u] > first_start[v]:
                    problems.append(f"proc {i}: segment {v} touched before segment {u} is done")
    completion = max((r[2] for r in recvs[0]), default=0)
    return completion, problems
