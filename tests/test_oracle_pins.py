"""Pins for the fp64 CPU oracle: what the paper and the mathematics fix.

None of these tests re-types the oracle's own formula as the expected value:
they use library routines on special cases, closed forms, hand-computed
examples (numbers worked out on paper and written here as literals),
brute-force enumeration and the invariants the paper states.
"""

import math

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import brute_force as bf

RNG = np.random.default_rng(20251022)


# ------------------------------------------------------------------ score
def test_score_single_row_is_library_softmax(oracle):
    # G = 1, W = 1: the one window query sees every key, so s is one softmax row of K q / sqrt(D) (Eq. 1)
    D, L = 24, 57
    q = RNG.normal(size=(1, 1, D))
    k = RNG.normal(size=(L, D))
    s, e = oracle.score(q, k, eps=1e-6)
    np.testing.assert_allclose(s, sp_softmax(k @ q[0, 0] / math.sqrt(D)), rtol=1e-12, atol=1e-15)
    # one query => Ahat == 1 for every key => e_t = -ln(1 + eps)
    np.testing.assert_allclose(e, -math.log1p(1e-6), rtol=1e-9)


def test_score_matches_library_matmul_softmax_mean(oracle):
    # general case through library routines: matmul, masked softmax, mean over heads, sum over queries
    G, W, D, L = 3, 5, 16, 41
    T = L - W
    q = RNG.normal(size=(G, W, D))
    k = RNG.normal(size=(L, D))
    logits = np.einsum("gwd,ld->gwl", q, k) / math.sqrt(D)
    for i in range(W):
        logits[:, i, T + i + 1:] = -np.inf
    abar = sp_softmax(logits, axis=-1).mean(axis=0)
    s, e = oracle.score(q, k, eps=1e-6)
    np.testing.assert_allclose(s, abar.sum(axis=0), rtol=1e-12)
    ahat = abar / abar.sum(axis=0, keepdims=True)
    from scipy.special import xlogy
    # -sum a*ln(a+eps) written with xlogy(a, a+eps) (0 where a == 0)
    np.testing.assert_allclose(e, -xlogy(ahat, ahat + 1e-6).sum(axis=0), rtol=1e-10, atol=1e-14)


def test_score_zero_queries_closed_form(oracle):
    # Q == 0 => every visible key gets 1/(T+i+1) from query i
    G, W, D, L = 2, 4, 8, 30
    T = L - W
    eps = 1e-6
    s, e = oracle.score(np.zeros((G, W, D)), RNG.normal(size=(L, D)), eps=eps)
    w = np.array([1.0 / (T + i + 1) for i in range(W)])
    for t in range(L):
        first = max(0, t - T)            # queries first..W-1 see key t
        st = w[first:].sum()
        assert s[t] == pytest.approx(st, rel=1e-13)
        ah = w[first:] / st
        assert e[t] == pytest.approx(-(ah * np.log(ah + eps)).sum(), rel=1e-12)
    # compressible keys: identical score, entropy just under ln W
    assert np.ptp(s[:T]) < 1e-15
    assert math.log(W) - 1e-2 < e[0] <= math.log(W) + 1e-9


def test_score_columns_sum_to_window(oracle):
    G, W, D, L = 2, 6, 16, 100
    s, e = oracle.score(RNG.normal(size=(G, W, D)) * 2, RNG.normal(size=(L, D)), eps=1e-6)
    assert s.sum() == pytest.approx(W, rel=1e-12)           # every softmax row sums to one
    assert (s >= 0).all()
    assert (e >= -W * 1e-6 - 1e-12).all() and (e <= math.log(W) + 1e-9).all()


def test_score_one_hot_limit(oracle):
    # orthogonal keys c*I and queries aligned with key t0: all mass on t0 as c grows
    D = L = 16
    W, t0, c = 3, 5, 12.0
    k = c * np.eye(L, D)
    q = np.zeros((1, W, D))
    q[0, :, t0] = c
    s, e = oracle.score(q, k, eps=1e-6)
    assert s[t0] == pytest.approx(W, abs=1e-10)
    assert np.delete(s, t0).max() < 1e-10
    # all W queries attend t0 equally: its Ahat is uniform over W
    assert e[t0] == pytest.approx(math.log(W), abs=1e-5)


def test_score_head_mean_is_linear_in_heads(oracle):
    # s under a group of G heads equals the mean of the single-head scores (Eq. barA then Eq. st)
    G, W, D, L = 4, 3, 8, 25
    q = RNG.normal(size=(G, W, D))
    k = RNG.normal(size=(L, D))
    s, _ = oracle.score(q, k)
    singles = np.stack([oracle.score(q[h:h + 1], k)[0] for h in range(G)])
    np.testing.assert_allclose(s, singles.mean(axis=0), rtol=1e-12)
    # G identical heads reduce to one head, entropy included
    s1, e1 = oracle.score(q[:1], k)
    s4, e4 = oracle.score(np.repeat(q[:1], 4, axis=0), k)
    np.testing.assert_allclose(s4, s1, rtol=1e-12)
    np.testing.assert_allclose(e4, e1, rtol=1e-10, atol=1e-14)


def test_score_scale_uses_head_dim(oracle):
    # doubling D by zero padding changes only the 1/sqrt(D) scale: equals scaling q by 1/sqrt(2)
    G, W, D, L = 1, 2, 8, 20
    q = RNG.normal(size=(G, W, D))
    k = RNG.normal(size=(L, D))
    qp = np.concatenate([q, np.zeros_like(q)], axis=-1)
    kp = np.concatenate([k, np.zeros_like(k)], axis=-1)
    np.testing.assert_allclose(oracle.score(qp, kp)[0], oracle.score(q / math.sqrt(2), k)[0], rtol=1e-12)


# ------------------------------------------------------------------ refine
def test_refine_hand_example(oracle):
    # two segments of three tokens, alpha = 0.5, eta = 2; worked by hand:
    # seg 1: I = .2, D = 1   -> omega = .2 * (1 + 2)   = .6 -> factor 1.3
    # seg 2: I = .2, D = .5  -> omega = .2 * (1 + 1)   = .4 -> factor 1.2
    s = [0.1, 0.3, 0.2, 0.4, 0.0, 0.2]
    e = [1.0, 2.0, 0.0, 0.5, 0.5, 0.5]
    st, om = oracle.refine(s, e, [0, 3, 6], alpha=0.5, eta=2.0)
    np.testing.assert_allclose(om, [0.6, 0.4], rtol=1e-14)
    np.testing.assert_allclose(st, [0.13, 0.39, 0.26, 0.48, 0.0, 0.24], rtol=1e-14)


def test_refine_special_cases(oracle):
    T = 200
    s = RNG.random(T)
    e = RNG.random(T) * 3
    off = np.array([0, 7, 8, 50, 120, 200], dtype=np.int32)
    st0, _ = oracle.refine(s, e, off, alpha=0.0, eta=1.0)
    np.testing.assert_array_equal(st0, s)                               # alpha = 0: no change
    _, om = oracle.refine(s, e, off, alpha=0.9, eta=0.0)                # eta = 0: omega = I_k
    np.testing.assert_allclose(om, [s[a:b].mean() for a, b in zip(off[:-1], off[1:])], rtol=1e-13)
    st, om = oracle.refine(s, e, off, alpha=0.9, eta=1.0)
    for a, b in zip(off[:-1], off[1:]):                                 # order inside a segment unchanged
        np.testing.assert_array_equal(np.argsort(-st[a:b], kind="stable"), np.argsort(-s[a:b], kind="stable"))
        ratio = st[a:b] / s[a:b]
        assert np.ptp(ratio) < 1e-12 and ratio[0] > 1.0
    # one segment over everything: a single closed-form factor
    st1, _ = oracle.refine(s, e, [0, T], alpha=0.9, eta=1.0)
    c = 1.0 + 0.9 * s.mean() * (1.0 + e.mean())
    np.testing.assert_allclose(st1, c * s, rtol=1e-13)


# ------------------------------------------------------------------ search / select
HAND = [9, 1, 1, 8, 7, 6, 1, 1, 5, 0.5, 0.5, 4]
HAND_OFF = [0, 8, 12]


@pytest.mark.parametrize("tau,g_exp,idx_exp", [
    # worked by hand: Top-6 = {0,3,4,5,8,11}; b = (4, 2); base = (30, 9)
    # seg 1: R(4) = 19/30, R(2) = 23/30; seg 2: R(2) = 5.5/9
    (0.85, [1, 1], [0, 3, 4, 5, 8, 11]),
    (0.75, [2, 1], [0, 1, 4, 5, 8, 11]),
    (0.60, [4, 2], [0, 1, 2, 3, 8, 9]),
])
def test_search_hand_example(oracle, tau, g_exp, idx_exp):
    b, g = oracle.search_blocks(HAND, HAND_OFF, [1, 2, 4], 6, tau)
    assert b.tolist() == [4, 2]
    assert g.tolist() == g_exp
    idx, n = oracle.select(HAND, HAND_OFF, b, g, 6)
    assert n == 6 and idx.tolist() == idx_exp


def test_search_partial_block_and_short_tail_by_hand(oracle):
    # one segment, B = 3: Top-3 = {5, 0, 1}, base 16; g = 4 infeasible (> b_k);
    # g = 2: blocks 6, 4, 11 -> take {4,5}, then the best token of {0,1} (tie -> 0): 14/16 = .875
    st = [3, 3, 3, 1, 1, 10]
    b, g = oracle.search_blocks(st, [0, 6], [1, 2, 4], 3, 0.85)
    assert (b.tolist(), g.tolist()) == ([3], [2])
    assert oracle.select(st, [0, 6], b, g, 3)[0].tolist() == [0, 4, 5]
    # short last block competes with its own (smaller) sum: blocks 2, 2, 9 -> {4}, then token 0
    st = [1, 1, 1, 1, 9]
    b, g = oracle.search_blocks(st, [0, 5], [1, 2], 2, 0.85)
    assert (b.tolist(), g.tolist()) == ([2], [2])
    assert oracle.select(st, [0, 5], b, g, 2)[0].tolist() == [0, 4]
    sc, take = oracle.segment_score(st, 0, 5, 2, 2)
    assert sc == 10.0 and take.tolist() == [True, False, False, False, True]


def test_search_accepts_at_equality_with_the_threshold(oracle):
    # Eq. gk_star and Alg. 2 accept a block size when R_k(g) >= tau, equality included.  One segment, B = 2: the
    # Top-2 tokens are the first block of size 2, so T_k(2) is the Top-B set itself and R_k(2) = 1 exactly; with
    # tau = 1 the answer is g = 2 (a strict comparison would fall back to g = 1).  Second case by hand at
    # tau = 0.75 exactly: Top-2 = {0, 3}, base 16; g = 2 takes block {0, 1} = 12, R = 12/16 = 0.75.
    st = [9, 9, 1, 1, 1, 1, 1, 1]
    b, g = oracle.search_blocks(st, [0, 8], [1, 2, 4], 2, 1.0)
    assert (b.tolist(), g.tolist()) == ([2], [2])
    st = [8, 4, 3, 8, 0, 0]
    b, g = oracle.search_blocks(st, [0, 6], [1, 2], 2, 0.75)
    assert (b.tolist(), g.tolist()) == ([2], [2])
    assert oracle.select(st, [0, 6], b, g, 2)[0].tolist() == [0, 1]
    b, g = oracle.search_blocks(st, [0, 6], [1, 2], 2, 0.7500001)
    assert g.tolist() == [1]


def _random_case(rng, T, mean_len, levels=None):
    lens = []
    while sum(lens) < T:
        lens.append(int(rng.integers(1, 2 * mean_len)))
    off = np.minimum(np.concatenate([[0], np.cumsum(lens)]), T)
    off = np.unique(off).astype(np.int32)
    st = rng.random(T) ** 4
    if levels:                          # few distinct values: exercises every tie-break
        st = np.round(st * levels) / levels
    return st, off


@pytest.mark.parametrize("seed", range(12))
def test_search_equals_brute_force_enumeration(oracle, seed):
    rng = np.random.default_rng(seed)
    T = int(rng.integers(40, 400))
    st, off = _random_case(rng, T, int(rng.integers(3, 40)), levels=(8 if seed % 3 == 0 else None))
    cand = [[1, 2, 4, 8], [1, 2, 3, 5, 7, 9, 11, 13], [1, 3, 4], [1]][seed % 4]
    B = int(rng.integers(1, T))
    tau = [0.85, 0.6, 0.95, 1.0][seed % 4]
    b, g = oracle.search_blocks(st, off, cand, B, tau)
    idx, n = oracle.select(st, off, b, g, B)
    ref = bf.run(st, off.tolist(), cand, B, tau)
    assert b.tolist() == ref["b"]
    assert g.tolist() == ref["g"]            # Alg. 2's descending walk == Eq. gk_star's max-form
    assert idx[:n].tolist() == ref["idx"]
    # invariants the paper states
    assert n == min(B, T) == int(b.sum())
    assert (np.diff(idx[:n]) > 0).all()
    for r in ref["segs"]:
        for gg, (sc, base) in r["R"].items():
            assert sc <= base * (1 + 1e-12)                      # baseline is the maximum: R <= 1
            assert len(r["sets"][gg]) == r["bk"]                 # every candidate fills b_k exactly
        if r["bk"]:
            assert r["R"][1][0] == pytest.approx(r["base"], rel=1e-13)   # R_k(1) = 1


def test_topb_is_library_sort(oracle):
    rng = np.random.default_rng(7)
    T, B = 500, 123
    st = np.round(rng.random(T) * 50) / 50           # many ties
    off = np.arange(0, T + 1, 10, dtype=np.int32)
    b, g = oracle.search_blocks(st, off, [1], B, 0.85)
    order = np.lexsort((np.arange(T), -st))[:B]       # value descending, index ascending
    counts = np.bincount(order // 10, minlength=T // 10)
    assert b.tolist() == counts.tolist()
    idx, n = oracle.select(st, off, b, g, B)
    assert idx[:n].tolist() == sorted(order.tolist())   # candidates {1}: plain token-level top-k


def test_search_tau_extremes_and_budget_edges(oracle):
    rng = np.random.default_rng(3)
    st, off = _random_case(rng, 300, 20)
    cand = [1, 2, 4, 8, 16]
    b, g = oracle.search_blocks(st, off, cand, 150, 0.0)      # tau = 0: largest feasible candidate
    lens = np.diff(off)
    for bk, gk, ln in zip(b, g, lens):
        assert gk == (max(c for c in cand if c <= min(bk, ln)) if bk else 0)
    b, g = oracle.search_blocks(st, off, cand, 10 ** 6, 0.85)  # B >= T: everything kept
    assert b.tolist() == lens.tolist()
    idx, n = oracle.select(st, off, b, g, 300)
    assert n == 300 and idx.tolist() == list(range(300))
    b, g = oracle.search_blocks(st, off, cand, 0, 0.85)        # B = 0: nothing kept
    assert not b.any() and not g.any()
    assert oracle.select(st, off, b, g, 0)[1] == 0
    # tau > 1: only candidates that reproduce the baseline exactly survive; g = 1 always does
    b, g = oracle.search_blocks(st, off, cand, 100, 1.5)
    assert set(g[b > 0].tolist()) <= set(cand) and (g[b > 0] >= 1).all()


def test_blocks_never_cross_segments(oracle):
    # selected tokens of a segment with g* > 1 are whole aligned blocks plus at most one partial block
    rng = np.random.default_rng(11)
    st, off = _random_case(rng, 600, 30)
    b, g = oracle.search_blocks(st, off, [1, 2, 4, 8], 300, 0.5)
    idx, n = oracle.select(st, off, b, g, 300)
    sel = np.zeros(600, dtype=bool)
    sel[idx[:n]] = True
    assert (g > 1).sum() > 3
    for k in range(len(off) - 1):
        a, e_ = int(off[k]), int(off[k + 1])
        assert sel[a:e_].sum() == b[k]
        if g[k] > 1:
            partial = 0
            for lo in range(a, e_, int(g[k])):
                cnt = sel[lo:min(lo + g[k], e_)].sum()
                if 0 < cnt < min(lo + g[k], e_) - lo:
                    partial += 1
            assert partial <= 1


def test_block_size_trend_with_budget_and_tau(oracle):
    # sanity only (Sec. 3.3 / block-size trends): larger budget or smaller tau => larger blocks on average
    rng = np.random.default_rng(5)
    st, off = _random_case(rng, 4000, 32)
    cand = [1, 2, 4, 8, 16]

    def mean_g(B, tau):
        b, g = oracle.search_blocks(st, off, cand, B, tau)
        return (g * b).sum() / max(b.sum(), 1)

    assert mean_g(100, 0.85) < mean_g(800, 0.85) < mean_g(3000, 0.85)
    assert mean_g(800, 0.95) <= mean_g(800, 0.85) <= mean_g(800, 0.6)


# ------------------------------------------------------------------ compact
def test_compact_is_fancy_indexing(oracle):
    rng = np.random.default_rng(9)
    L, W, D, B = 90, 6, 16, 20
    k = rng.integers(0, 2 ** 16, size=(L, D), dtype=np.uint16)
    v = rng.integers(0, 2 ** 16, size=(L, D), dtype=np.uint16)
    idx = np.sort(rng.choice(L - W, size=13, replace=False)).astype(np.int32)
    full = np.concatenate([idx, -np.ones(B - 13, dtype=np.int32)])
    ko, vo = oracle.compact(k, v, W, full, 13, B, append_window=True)
    assert ko.shape == (B + W, D)
    np.testing.assert_array_equal(ko[:13], k[idx])
    np.testing.assert_array_equal(vo[:13], v[idx])
    assert not ko[13:B].any() and not vo[13:B].any()
    np.testing.assert_array_equal(ko[B:], k[L - W:])
    np.testing.assert_array_equal(vo[B:], v[L - W:])
    ko2, _ = oracle.compact(k.view(np.float16), v.view(np.float16), W, full, 13, B, append_window=False)
    assert ko2.shape == (B, D)
    np.testing.assert_array_equal(ko2.view(np.uint16)[:13], k[idx])


# ------------------------------------------------------------------ whole path on the tiny workload
def test_pipeline_tiny_invariants(oracle):
    from paper_2510_22556_amd import synth

    w = synth.WORKLOADS["tiny"]
    q, k, v = synth.host_layer(w)
    off, ptr = synth.workload_segments(w)
    B = w.budget()
    for j in range(w.n_kv_heads):
        r = oracle.pipeline_head(q[j * w.G:(j + 1) * w.G], k[j], v[j], off, w.cand, B,
                                 w.eps, w.alpha, w.eta, w.tau)
        assert r["s"].sum() == pytest.approx(w.window, rel=1e-12)
        assert r["n_sel"] == B and int(r["b"].sum()) == B
        assert r["k_out"].shape == (B + w.window, w.head_dim)       # retained entries == cache budget
        assert B + w.window <= w.cache_budgets[0]
        np.testing.assert_array_equal(r["k_out"][:B], k[j][r["idx"]])
        np.testing.assert_array_equal(r["v_out"][B:], v[j][w.T:])
        ref = bf.run(r["s_tilde"], off.tolist(), list(w.cand), B, w.tau)
        assert r["g"].tolist() == ref["g"] and r["idx"].tolist() == ref["idx"]


# ---------------------------------------------------------------- segmentation (Sec. 3.1)
def test_segment_hand_examples(oracle):
    # "a , b c . d" with delimiters {",", "."}: [a ,] [b c .] [d]
    np.testing.assert_array_equal(oracle.segment([5, 11, 7, 8, 13, 9], [11, 13]), [0, 2, 5, 6])
    # a delimiter as the last token closes the last segment without opening an empty one
    np.testing.assert_array_equal(oracle.segment([5, 11, 7, 13], [11, 13]), [0, 2, 4])
    # no delimiter at all / no delimiter set: one segment
    np.testing.assert_array_equal(oracle.segment([1, 2, 3], [11]), [0, 3])
    np.testing.assert_array_equal(oracle.segment([1, 2, 3], []), [0, 3])
    # consecutive delimiters: one-token segments
    np.testing.assert_array_equal(oracle.segment([11, 11, 11, 4], [11]), [0, 1, 2, 3, 4])
    np.testing.assert_array_equal(oracle.segment([11], [11]), [0, 1])


def test_segment_against_library_routines(oracle):
    from paper_2510_22556_amd import synth

    ids = synth.token_ids(11, 3, 5003, 24.0)
    for row in ids:
        off = oracle.segment(row, synth.DELIMS)
        interior = np.flatnonzero(np.isin(row[:-1], synth.DELIMS)) + 1          # library formulation
        np.testing.assert_array_equal(off, np.concatenate([[0], interior, [len(row)]]))
        assert (np.diff(off) >= 1).all()
        # every segment but the last ends with a delimiter and holds no other one
        for a, b in zip(off[:-1], off[1:]):
            assert not np.isin(row[a:b - 1], synth.DELIMS).any()
            assert b == len(row) or row[b - 1] in synth.DELIMS
        assert 16 < np.diff(off).mean() < 36                                       # the generator's mean length


# ---------------------------------------------------------------- decode attention (Sec. 2.1, Eq. 1)
def test_decode_attention_pins(oracle):
    from scipy.special import softmax

    rng = np.random.default_rng(3)
    G, D, R = 4, 16, 37
    q, k, v = rng.standard_normal((G, D)), rng.standard_normal((R, D)), rng.standard_normal((R, D))
    out = oracle.decode_attention(q, k, v)
    # library routines: softmax of the scaled logits, then a matrix product
    np.testing.assert_allclose(out, softmax(q @ k.T / 4.0, axis=1) @ v, rtol=1e-12, atol=1e-14)
    # q = 0: uniform weights, the mean of V; a single row: that row of V
    np.testing.assert_allclose(oracle.decode_attention(np.zeros((G, D)), k, v), np.tile(v.mean(axis=0), (G, 1)), rtol=1e-12)
    np.testing.assert_allclose(oracle.decode_attention(q, k[:1], v[:1]), np.tile(v[0], (G, 1)), rtol=1e-12)
    # one-hot limit: a key aligned with the query and scaled up takes all the weight (transposed operands or a
    # missing scale would pick another row or blur the weights)
    k2 = k.copy(); k2[5] = 200.0 * q[2] / np.linalg.norm(q[2])
    np.testing.assert_allclose(oracle.decode_attention(q, k2, v)[2], v[5], rtol=1e-9, atol=1e-12)
    # the 1/sqrt(D) scale: zero-padding D -> 4D divides the logits by 2 = logits of (q/2, k) at the old D
    pad = lambda a: np.concatenate([a, np.zeros((a.shape[0], 3 * D))], axis=1)
    np.testing.assert_allclose(oracle.decode_attention(pad(q), pad(k), v), oracle.decode_attention(q / 2, k, v), rtol=1e-12)
    # invariances: order of the rows, a common shift of the logits (k + c*q/|q|^2 direction per head is head-specific,
    # so shift through an extra constant column instead)
    perm = rng.permutation(R)
    np.testing.assert_allclose(oracle.decode_attention(q, k[perm], v[perm]), out, rtol=1e-12, atol=1e-14)
    q1 = np.concatenate([q, np.ones((G, 1))], axis=1); k1 = np.concatenate([k, np.full((R, 1), 7.0)], axis=1)
    ref = softmax(q @ k.T / np.sqrt(D + 1.0), axis=1) @ v
    np.testing.assert_allclose(oracle.decode_attention(q1, k1, v), ref, rtol=1e-12, atol=1e-14)
    assert (oracle.decode_attention(q, k[:0], v[:0]) == 0).all()


# ---------------------------------------------------------------- attention of the window queries (Sec. 2.1, Eq. 1)
def test_window_attention_pins(oracle):
    from scipy.special import logsumexp, softmax

    rng = np.random.default_rng(8)
    G, W, D, L = 3, 5, 12, 41
    T = L - W
    q, k, v = rng.standard_normal((G, W, D)), rng.standard_normal((L, D)), rng.standard_normal((L, 7))
    out, lse = oracle.window_attention(q, k, v)
    # library routines on the masked logits: softmax then a matrix product; logsumexp for the denominator
    for g in range(G):
        x = q[g] @ k.T / np.sqrt(D)
        x[np.arange(L)[None, :] > T + np.arange(W)[:, None]] = -np.inf        # query i sees keys t <= T + i
        np.testing.assert_allclose(out[g], softmax(x, axis=1) @ v, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse[g], logsumexp(x, axis=1), rtol=1e-13)
    # the mask matters and sits where it should: changing a key or value row that query i cannot see changes nothing
    # for queries <= i and something for the later ones
    k2, v2 = k.copy(), v.copy()
    k2[T + 3] += 1.0; v2[T + 3] -= 2.0
    out2, lse2 = oracle.window_attention(q, k2, v2)
    assert np.array_equal(out2[:, :3], out[:, :3]) and np.array_equal(lse2[:, :3], lse[:, :3])
    assert (np.abs(out2[:, 3:] - out[:, 3:]).max(axis=2) > 1e-6).all() and (lse2[:, 3:] != lse[:, 3:]).all()
    # q = 0: uniform weights over the T + i + 1 visible keys -> the running mean of V, lse = log(T + i + 1)
    out0, lse0 = oracle.window_attention(np.zeros((1, W, D)), k, v)
    for i in range(W):
        np.testing.assert_allclose(out0[0, i], v[:T + i + 1].mean(axis=0), rtol=1e-12)
        np.testing.assert_allclose(lse0[0, i], np.log(T + i + 1.0), rtol=1e-13)
    # the same denominators as the scoring step: its attention rows are exp(logit - lse), so the column sums of
    # exp(logit - lse) over the window rows of the G heads, averaged over the heads, are the oracle's scores
    s_ref, _ = oracle.score(q, k, 1e-6)
    acc = np.zeros(L)
    for g in range(G):
        x = q[g] @ k.T / np.sqrt(D)
        a = np.exp(x - lse[g][:, None])
        a[np.arange(L)[None, :] > T + np.arange(W)[:, None]] = 0.0
        acc += a.sum(axis=0)
    np.testing.assert_allclose(acc / G, s_ref, rtol=1e-10, atol=1e-14)
    # a decode step is the window of one query at the end: both oracle functions agree there
    o1, _ = oracle.window_attention(q[:, -1:, :], k, v)
    np.testing.assert_allclose(o1[:, 0], oracle.decode_attention(q[:, -1], k, v), rtol=1e-12, atol=1e-14)
    # the 1/sqrt(D) scale: zero-padding D -> 4D halves the logits
    pad = lambda a: np.concatenate([a, np.zeros(a.shape[:-1] + (3 * D,))], axis=-1)
    o_pad, l_pad = oracle.window_attention(pad(q), pad(k), v)
    o_half, l_half = oracle.window_attention(q / 2, k, v)
    np.testing.assert_allclose(o_pad, o_half, rtol=1e-12); np.testing.assert_allclose(l_pad, l_half, rtol=1e-12)


# ---------------------------------------------------------------- head mean over all heads of a layer (Eq. barA, literal)
def test_score_layer_pins(oracle):
    from scipy.special import softmax

    rng = np.random.default_rng(17)
    Hq, Hkv, W, D, L = 6, 3, 5, 8, 41
    T = L - W
    q, k = rng.standard_normal((Hq, W, D)), rng.standard_normal((Hkv, L, D))
    s, e = oracle.score_layer(q, k, 1e-6)
    # library routines: masked softmax per head, mean over all six heads, column sums, entropy of the
    # column-normalised means
    abar = np.zeros((W, L))
    for h in range(Hq):
        x = q[h] @ k[h // (Hq // Hkv)].T / np.sqrt(D)
        for i in range(W):
            abar[i, :T + i + 1] += softmax(x[i, :T + i + 1]) / Hq
    np.testing.assert_allclose(s, abar.sum(axis=0), rtol=1e-12, atol=1e-15)
    ah = abar / abar.sum(axis=0)
    np.testing.assert_allclose(e, -(ah * np.log(ah + 1e-6)).sum(axis=0), rtol=1e-11, atol=1e-14)
    assert abs(s.sum() - W) < 1e-12
    # one KV head: the per-KV-head score is the same thing
    s1, e1 = oracle.score_layer(q[:2], k[:1], 1e-6)
    s0, e0 = oracle.score(q[:2], k[0], 1e-6)
    np.testing.assert_allclose(s1, s0, rtol=1e-14, atol=0)
    np.testing.assert_allclose(e1, e0, rtol=1e-13, atol=1e-16)
    # the mean over heads of per-KV-head column sums (linear), though the entropy is not linear
    per = [oracle.score(q[g * 2:(g + 1) * 2], k[g], 1e-6)[0] for g in range(Hkv)]
    np.testing.assert_allclose(s, np.mean(per, axis=0), rtol=1e-12, atol=1e-15)
    # a wrong head-to-KV-head map would show: make KV head 2 special
    k2 = k.copy(); k2[2] *= 3.0
    s2, _ = oracle.score_layer(q, k2, 1e-6)
    per2 = [oracle.score(q[g * 2:(g + 1) * 2], k2[g], 1e-6)[0] for g in range(Hkv)]
    np.testing.assert_allclose(s2, np.mean(per2, axis=0), rtol=1e-12, atol=1e-15)
