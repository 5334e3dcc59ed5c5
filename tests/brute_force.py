"""Pure-Python enumerator of block-size choices, used to pin the oracle's search.

Independent of ``oracle/`` (no shared code): it evaluates EVERY candidate
block size of a segment with full sorts and no early exit, then applies the
max-form of the decision rule (Eq. gk_star), whereas the oracle walks the
candidates downwards and stops at the first accepted one (Alg. 2).  It also
reports the smallest relative gap among all the comparisons that decided the
result, which the parity tests use to explain a disagreement between two
floating-point evaluations of the same segment.
"""

from __future__ import annotations

from typing import Dict, List, Sequence, Tuple


def top_b(st: Sequence[float], B: int) -> List[int]:
    order = sorted(range(len(st)), key=lambda t: (-st[t], t))
    return sorted(order[: max(min(B, len(st)), 0)])


def _rel_gap(x: float, y: float) -> float:
    d = abs(x - y)
    m = max(abs(x), abs(y))
    return d / m if m > 0 else 0.0


def fill(st: Sequence[float], a: int, b: int, g: int, bk: int) -> Tuple[List[int], float, float]:
    """T_k(g) (ascending), Score_k(g), and the smallest relative gap between
    neighbours in the two rankings that were used."""
    blocks = [(sum(st[lo:min(lo + g, b)]), m, lo, min(lo + g, b))
              for m, lo in enumerate(range(a, b, g))]
    ranked = sorted(blocks, key=lambda x: (-x[0], x[1]))
    gap = min([_rel_gap(ranked[i][0], ranked[i + 1][0]) for i in range(len(ranked) - 1)] or [1.0])
    chosen: List[int] = []
    for phi, m, lo, hi in ranked:
        if len(chosen) + (hi - lo) <= bk:
            chosen.extend(range(lo, hi))
        else:
            rem = bk - len(chosen)
            toks = sorted(range(lo, hi), key=lambda t: (-st[t], t))
            gap = min([gap] + [_rel_gap(st[toks[i]], st[toks[i + 1]]) for i in range(len(toks) - 1)])
            chosen.extend(toks[:rem])
            break
    chosen.sort()
    return chosen, sum(st[t] for t in chosen), gap


def enumerate_segment(st: Sequence[float], a: int, b: int, in_top: Sequence[int], cand: Sequence[int],
                      tau: float) -> Dict:
    """All candidates of one segment.  ``in_top``: the Top-B tokens inside [a,b)."""
    bk = len(in_top)
    base = sum(st[t] for t in in_top)
    out = dict(bk=bk, base=base, R={}, sets={}, g_star=0, gap=1.0)
    if bk == 0:
        return out
    feasible = [g for g in cand if 1 <= g <= min(b - a, bk)]
    for g in feasible:
        toks, sc, gap = fill(st, a, b, g, bk)
        out["sets"][g] = toks
        out["R"][g] = (sc, base)
        out["gap"] = min(out["gap"], gap)
        if g > 1:
            out["gap"] = min(out["gap"], _rel_gap(sc, tau * base))
    ok = [g for g in feasible if g == 1 or out["R"][g][0] >= tau * base]
    out["g_star"] = max(ok)
    return out


def run(st: Sequence[float], seg_off: Sequence[int], cand: Sequence[int], B: int, tau: float) -> Dict:
    """Whole per-head search + selection by enumeration."""
    st = [float(x) for x in st]
    T = seg_off[-1]
    top = top_b(st[:T], B)
    top_set = set(top)
    order = sorted(range(T), key=lambda t: (-st[t], t))
    nB = min(B, T)
    boundary_gap = _rel_gap(st[order[nB - 1]], st[order[nB]]) if 0 < nB < T else 1.0
    res = dict(b=[], g=[], idx=[], segs=[], boundary_gap=boundary_gap)
    for k in range(len(seg_off) - 1):
        a, b = seg_off[k], seg_off[k + 1]
        r = enumerate_segment(st, a, b, [t for t in range(a, b) if t in top_set], cand, tau)
        res["b"].append(r["bk"])
        res["g"].append(r["g_star"])
        if r["g_star"]:
            res["idx"].extend(r["sets"][r["g_star"]])
        res["segs"].append(r)
    return res
