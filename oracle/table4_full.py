"""TEST INFRASTRUCTURE: re-runs the paper's unequal-segmentation experiment
(Section 8, Table IV) with the CPU oracle: m = 10, beta = 1, gamma in {0,1},
29 values of alpha, 17 values of p, all 512 segmentations of m through
uni-greedy.  Prints every experiment whose optimum is reached by no
equi-segmentation, in the format of tests/golden/table4_unequal_segmentation.txt,
and the aggregate figures the section quotes (count, largest and mean gain).

Run:  python -m oracle.table4_full [max_p]
It calls nothing but the oracle and takes a few minutes on 8 cores.
"""
from __future__ import annotations

import sys
from concurrent.futures import ThreadPoolExecutor

import oracle as O

M = 10
ALPHAS = list(range(0, 11)) + list(range(20, 101, 10)) + list(range(200, 1001, 100))
PS = sorted([2 ** n for n in range(2, 11)] + [3 * 2 ** n for n in range(1, 9)])


def compositions(m):
    for bits in range(1 << (m - 1)):
        parts, cur = [], 1
        for i in range(m - 1):
            if bits >> i & 1:
                parts.append(cur); cur = 1
            else:
                cur += 1
        parts.append(cur)
        yield tuple(parts)


COMPS = list(compositions(M))
# "same size for all segments except possibly a smaller last one"
EQUI_ANY = [c for c in COMPS if all(x == c[0] for x in c[:-1]) and c[-1] <= c[0]]
# equi-segmentations obtained from a segment count: size ceil(m / count)
EQUI_BY_COUNT = sorted({tuple(int(v) for v in O.equi_sizes(M, k)) for k in range(1, M + 1)})


def experiment(args):
    p, a, g = args
    T = {c: O.uni_greedy(p, list(c), a, 1, g, want_schedule=False).T for c in COMPS}
    best = min(T.values())
    opt = [c for c in COMPS if T[c] == best]
    be = min(T[c] for c in EQUI_BY_COUNT)
    bes = [c for c in EQUI_BY_COUNT if T[c] == be]
    return p, a, g, best, opt, be, bes, any(c in EQUI_ANY for c in opt)


def main():
    max_p = int(sys.argv[1]) if len(sys.argv) > 1 else 1 << 30
    jobs = [(p, a, g) for p in PS if p <= max_p for a in ALPHAS for g in (0, 1)]
    with ThreadPoolExecutor(8) as ex:
        res = list(ex.map(experiment, jobs))
    rows = [r for r in res if not r[7]]
    gains = [r[5] / r[3] - 1.0 for r in rows]
    for p, a, g, best, opt, be, bes, _ in rows:
        print(p, a, g, f"{be / best:.4f}", ";".join(",".join(map(str, c)) for c in bes),
              ";".join(",".join(map(str, c)) for c in sorted(opt, key=lambda c: COMPS.index(c))))
    print(f"# experiments {len(jobs)}  improved {len(rows)}  max gain {max(gains) * 100:.1f}%  "
          f"mean gain {sum(gains) / len(gains) * 100:.1f}%  largest alpha {max(r[1] for r in rows)}")


if __name__ == "__main__":
    main()
