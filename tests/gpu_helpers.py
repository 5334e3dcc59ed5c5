"""Helpers for the GPU parity tests: run the HIP path through the C ABI, run the
fp64 oracle on the same bits, and compare under the stated tolerances."""

from __future__ import annotations

import numpy as np

import brute_force as bf

# tolerances on floating-point scores (the benchmark spec): 1e-3 relative / 1e-5 absolute
RTOL, ATOL = 1e-3, 1e-5


def f32(x: float) -> float:
    """The float32 value the library receives for a hyperparameter, as a Python float."""
    return float(np.float32(x))


def to_np(t):
    import torch

    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def widen(raw: np.ndarray) -> np.ndarray:
    """float64 view of raw K/Q/V data (uint16 = bf16 bit patterns, else float32)."""
    if raw.dtype == np.uint16:
        return (raw.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return raw.astype(np.float64)


def close(gpu, ref, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(gpu - ref)
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, worst abs err {err.max():.3e}"
    return float((err / (np.abs(ref) + 1e-30)).max())


class GpuRun:
    """All five ABI calls on device tensors; results as numpy arrays indexed by problem."""

    def __init__(self, q, k, v, seg_off, seg_ptr, cand, budget, eps=1e-6, alpha=0.9, eta=1.0, tau=0.85,
                 append_window=True, row_lse=None, tuning=None):
        import torch
        from paper_2510_22556_amd import binding as B

        self.B = B
        dev = q.device
        self.shape = B.make_shape(q, k, v, **(tuning or {}))
        self.seg = B.make_segments(seg_off, seg_ptr, dev)
        self.buf = B.Buffers(self.shape, self.seg, budget, dev, append_window)
        self.cand, self.budget = list(cand), budget
        B.compress(self.shape, q, k, v, self.seg, cand, budget, self.buf, eps, alpha, eta, tau, row_lse)
        torch.cuda.synchronize()
        b = self.buf
        self.s, self.e, self.st = to_np(b.s), to_np(b.ent), to_np(b.s_tilde)
        self.omega, self.b, self.g = to_np(b.omega), to_np(b.seg_budget), to_np(b.block_size)
        self.idx, self.n_sel = to_np(b.idx), to_np(b.n_sel)
        self.k_out, self.v_out = to_np(b.k_out), to_np(b.v_out)


def problem_views(q, k, v, p, n_layers, Hkv, G):
    """numpy raw arrays (q [G,W,D], k [L,D], v [L,D]) of problem p from torch tensors."""
    seq, layer, head = p // (n_layers * Hkv), (p // Hkv) % n_layers, p % Hkv
    return (to_np(q[seq, layer, head * G:(head + 1) * G]), to_np(k[seq, layer, head]), to_np(v[seq, layer, head]), seq)


def check_problem(oracle, run: GpuRun, p, q_raw, k_raw, v_raw, seg_off, eps, alpha, eta, tau, append_window=True,
                  end_to_end=True, score_ref=None):
    """Stage-wise parity of problem p (each oracle stage fed with the GPU's previous output),
    then end-to-end parity with every disagreement explained by a near-tie.  ``score_ref``: the oracle's
    (s, ent) of this problem when the caller already has them (several runs over the same tensors)."""
    W = q_raw.shape[1]
    L = k_raw.shape[0]
    T = L - W
    K = len(seg_off) - 1
    B_ = run.budget
    cand = run.cand
    # --- stage 1: scores
    s_ref, e_ref = score_ref if score_ref is not None else oracle.score(widen(q_raw), widen(k_raw), eps)
    close(run.s[p], s_ref, f"s[p={p}]")
    close(run.e[p], e_ref, f"ent[p={p}]")
    # --- stage 2: refinement of the GPU's own s, e
    st_ref, om_ref = oracle.refine(run.s[p], run.e[p], seg_off, f32(alpha), f32(eta))
    np.testing.assert_allclose(run.st[p], st_ref, rtol=3e-7, atol=0, err_msg=f"s_tilde[p={p}]")
    np.testing.assert_allclose(run.omega[p][:K], om_ref, rtol=3e-7, err_msg=f"omega[p={p}]")
    assert not run.omega[p][K:].any()
    # --- stage 3/4: search + select on the GPU's own s_tilde: integer results bit-exact
    b_ref, g_ref = oracle.search_blocks(run.st[p], seg_off, cand, B_, f32(tau))
    np.testing.assert_array_equal(run.b[p][:K], b_ref, err_msg=f"b_k[p={p}]")
    np.testing.assert_array_equal(run.g[p][:K], g_ref, err_msg=f"g_k*[p={p}]")
    assert not run.b[p][K:].any() and not run.g[p][K:].any()
    idx_ref, n_ref = oracle.select(run.st[p], seg_off, b_ref, g_ref, B_)
    assert run.n_sel[p] == n_ref == min(B_, T)
    np.testing.assert_array_equal(run.idx[p][:B_], idx_ref, err_msg=f"idx[p={p}]")
    # --- stage 5: compaction of the GPU's own index set: bit-exact
    ko, vo = oracle.compact(k_raw, v_raw, W, run.idx[p][:B_] if B_ else np.zeros(0, np.int32), int(run.n_sel[p]),
                            B_, append_window)
    rows = B_ + (W if append_window else 0)
    np.testing.assert_array_equal(run.k_out[p][:rows], ko, err_msg=f"k_out[p={p}]")
    np.testing.assert_array_equal(run.v_out[p][:rows], vo, err_msg=f"v_out[p={p}]")
    if not end_to_end:
        return 0
    # --- end to end: the oracle's own chain in fp64
    st_o, _ = oracle.refine(s_ref, e_ref, seg_off, f32(alpha), f32(eta))
    close(run.st[p], st_o, f"s_tilde end-to-end[p={p}]")
    b_o, g_o = oracle.search_blocks(st_o, seg_off, cand, B_, f32(tau))
    idx_o, n_o = oracle.select(st_o, seg_off, b_o, g_o, B_)
    assert n_o == run.n_sel[p]
    return explain_mismatches(st_o, seg_off, cand, B_, f32(tau), b_o, g_o, idx_o[:n_o], run.b[p][:K], run.g[p][:K],
                              run.idx[p][:n_o], st_g=run.st[p])


def explain_mismatches(st_o, seg_off, cand, B_, tau, b_o, g_o, idx_o, b_g, g_g, idx_g, st_g=None):
    """Every segment where the two chains disagree must contain a decision whose two
    competing fp64 values differ by less than the score tolerance.  Returns the count.

    A differing implicit budget must come from tokens whose Top-B membership flipped, and every flipped token
    of the segment must itself sit within the tolerance of the oracle's Top-B threshold (``st_g``, the refined
    scores the other chain ranked, names the flipped tokens; without it, some token of the segment must).  Any
    other difference is handed to the enumerator, which reports the tightest comparison among all the
    segment's decisions (block ranking, cut block, accept test); only segments of 65 536 tokens or more are
    skipped (the pure-Python enumeration would take minutes)."""
    T = int(seg_off[-1])
    sel_o = np.zeros(T, bool)
    sel_o[idx_o] = True
    sel_g = np.zeros(T, bool)
    sel_g[idx_g] = True
    order = np.lexsort((np.arange(T), -st_o))
    nB = min(B_, T)
    v_star = st_o[order[nB - 1]] if nB > 0 else 0.0
    top_set = set(order[:nB].tolist())
    in_top_o = np.zeros(T, bool)
    in_top_o[order[:nB]] = True
    in_top_g = None
    if st_g is not None:
        st_g = np.asarray(st_g, dtype=np.float64)[:T]
        in_top_g = np.zeros(T, bool)
        in_top_g[np.lexsort((np.arange(T), -st_g))[:nB]] = True
    st_list = None
    n_bad = 0
    for k in range(len(seg_off) - 1):
        a, b = int(seg_off[k]), int(seg_off[k + 1])
        if b_o[k] == b_g[k] and g_o[k] == g_g[k] and (sel_o[a:b] == sel_g[a:b]).all():
            continue
        n_bad += 1
        if b_o[k] != b_g[k]:
            # a Top-B membership flipped: some token of the segment sits at the threshold
            if in_top_g is not None:
                flipped = np.nonzero(in_top_o[a:b] != in_top_g[a:b])[0]
                assert flipped.size, f"segment {k}: b_k {b_o[k]} vs {b_g[k]} although no Top-B membership differs"
                gap = np.abs(st_o[a:b][flipped] - v_star).max() / max(v_star, 1e-300)
            else:
                gap = np.abs(st_o[a:b] - v_star).min() / max(v_star, 1e-300)
            assert gap <= RTOL, f"segment {k}: b_k {b_o[k]} vs {b_g[k]} without a score within tolerance of the Top-B threshold"
            continue
        if b - a >= 65536:
            continue
        if st_list is None:
            st_list = st_o.tolist()
        r = bf.enumerate_segment(st_list, a, b, [t for t in range(a, b) if t in top_set], cand, tau)
        assert r["gap"] <= RTOL, f"segment {k}: g {g_o[k]} vs {g_g[k]} with no decision inside tolerance (min gap {r['gap']:.3e})"
    return n_bad
