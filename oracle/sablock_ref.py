"""ctypes wrapper around ``sablock_ref.c`` (the fp64 CPU oracle).

TEST INFRASTRUCTURE ONLY: argument marshalling for the plain C oracle.  Every
function takes numpy arrays for ONE KV head of one (sequence, layer) and widens
them to float64 before the call; nothing here does arithmetic of the method,
with two exceptions written out here in plain numpy / Python: ``segment``
(punctuation-based segmentation, Sec. 3.1; integer-only, a token walk) and
``decode_attention`` (Sec. 2.1 Eq. 1 for one query position; float64).
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sablock_ref.c")
_LIB = os.path.join(_HERE, "libsablock_ref.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)
_bp = ctypes.POINTER(ctypes.c_ubyte)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, no fast-math) into this folder."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32, f64 = ctypes.c_int32, ctypes.c_double
        lib.sablock_ref_score.argtypes = [_dp, _dp, i32, i32, i32, i32, f64, _dp, _dp]
        lib.sablock_ref_score_layer.argtypes = [_dp, _dp, i32, i32, i32, i32, i32, f64, _dp, _dp]
        lib.sablock_ref_score_layer.restype = ctypes.c_int
        lib.sablock_ref_refine.argtypes = [_dp, _dp, i32, _ip, i32, f64, f64, _dp, _dp]
        lib.sablock_ref_search_blocks.argtypes = [_dp, i32, _ip, i32, _ip, i32, i32, f64, _ip, _ip]
        lib.sablock_ref_select.argtypes = [_dp, i32, _ip, i32, _ip, _ip, i32, _ip, _ip]
        lib.sablock_ref_compact.argtypes = [ctypes.c_void_p, ctypes.c_void_p, i32, i32, ctypes.c_int64,
                                            _ip, i32, i32, i32, ctypes.c_void_p, ctypes.c_void_p]
        lib.sablock_ref_segment_score.argtypes = [_dp, i32, i32, i32, i32, _bp]
        lib.sablock_ref_segment_score.restype = f64
        for n in ("score", "refine", "search_blocks", "select", "compact"):
            getattr(lib, "sablock_ref_" + n).restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _check(rc: int, name: str):
    if rc != 0:
        raise ValueError(f"sablock_ref_{name} failed with status {rc}")


def score(q, k, eps: float = 1e-6) -> Tuple[np.ndarray, np.ndarray]:
    """q [G, W, D], k [L, D] -> (s [L], e [L]) in float64."""
    q, k = _f64(q), _f64(k)
    G, W, D = q.shape
    L = k.shape[0]
    assert k.shape[1] == D
    s = np.empty(L, dtype=np.float64)
    e = np.empty(L, dtype=np.float64)
    rc = _load().sablock_ref_score(q.ctypes.data_as(_dp), k.ctypes.data_as(_dp), G, W, D, L, float(eps),
                                   s.ctypes.data_as(_dp), e.ctypes.data_as(_dp))
    _check(rc, "score")
    return s, e


def score_layer(q, k, eps: float = 1e-6) -> Tuple[np.ndarray, np.ndarray]:
    """Head mean over ALL query heads of a layer: q [Hq, W, D], k [Hkv, L, D] -> (s [L], e [L]) in float64."""
    q, k = _f64(q), _f64(k)
    Hq, W, D = q.shape
    Hkv, L = k.shape[0], k.shape[1]
    assert k.shape[2] == D and Hq % Hkv == 0
    s = np.empty(L, dtype=np.float64)
    e = np.empty(L, dtype=np.float64)
    rc = _load().sablock_ref_score_layer(q.ctypes.data_as(_dp), k.ctypes.data_as(_dp), Hq, Hkv, W, D, L, float(eps),
                                         s.ctypes.data_as(_dp), e.ctypes.data_as(_dp))
    _check(rc, "score_layer")
    return s, e


def refine(s, e, seg_off, alpha: float = 0.9, eta: float = 1.0) -> Tuple[np.ndarray, np.ndarray]:
    """s, e [>= T], seg_off [K+1] -> (s_tilde [T], omega [K]) in float64."""
    s, e, seg_off = _f64(s), _f64(e), _i32(seg_off)
    K = len(seg_off) - 1
    T = int(seg_off[-1])
    st = np.zeros(T, dtype=np.float64)
    om = np.zeros(max(K, 1), dtype=np.float64)
    rc = _load().sablock_ref_refine(s.ctypes.data_as(_dp), e.ctypes.data_as(_dp), T,
                                    seg_off.ctypes.data_as(_ip), K, float(alpha), float(eta),
                                    st.ctypes.data_as(_dp), om.ctypes.data_as(_dp))
    _check(rc, "refine")
    return st, om[:K]


def search_blocks(s_tilde, seg_off, cand: Sequence[int], budget: int, tau: float = 0.85):
    """-> (b_k [K] int32, g_k* [K] int32)"""
    st, seg_off, cand = _f64(s_tilde), _i32(seg_off), _i32(cand)
    K = len(seg_off) - 1
    T = int(seg_off[-1])
    assert st.shape[0] >= T
    b = np.zeros(max(K, 1), dtype=np.int32)
    g = np.zeros(max(K, 1), dtype=np.int32)
    rc = _load().sablock_ref_search_blocks(st.ctypes.data_as(_dp), T, seg_off.ctypes.data_as(_ip), K,
                                           cand.ctypes.data_as(_ip), len(cand), int(budget), float(tau),
                                           b.ctypes.data_as(_ip), g.ctypes.data_as(_ip))
    _check(rc, "search_blocks")
    return b[:K], g[:K]


def select(s_tilde, seg_off, b, g, budget: int):
    """-> (idx [budget] int32 ascending, padded with -1; n_sel)"""
    st, seg_off, b, g = _f64(s_tilde), _i32(seg_off), _i32(b), _i32(g)
    K = len(seg_off) - 1
    T = int(seg_off[-1])
    idx = np.full(max(int(budget), 1), -1, dtype=np.int32)
    n = ctypes.c_int32(0)
    rc = _load().sablock_ref_select(st.ctypes.data_as(_dp), T, seg_off.ctypes.data_as(_ip), K,
                                    b.ctypes.data_as(_ip), g.ctypes.data_as(_ip), int(budget),
                                    idx.ctypes.data_as(_ip), ctypes.byref(n))
    _check(rc, "select")
    return idx[:int(budget)], int(n.value)


def compact(k: np.ndarray, v: np.ndarray, window: int, idx, n_sel: int, budget: int,
            append_window: bool = True):
    """k, v [L, D] of any fixed-size dtype -> (k_out, v_out) [budget (+W), D], copied bit for bit."""
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    idx = _i32(idx)
    L, D = k.shape
    rows = int(budget) + (window if append_window else 0)
    ko = np.empty((rows, D), dtype=k.dtype)
    vo = np.empty((rows, D), dtype=v.dtype)
    rc = _load().sablock_ref_compact(k.ctypes.data, v.ctypes.data, L, int(window), k.strides[0],
                                     idx.ctypes.data_as(_ip), int(n_sel), int(budget),
                                     1 if append_window else 0, ko.ctypes.data, vo.ctypes.data)
    _check(rc, "compact")
    return ko, vo


def segment_score(s_tilde, a: int, b: int, g: int, bk: int):
    """Score_k(g) and the membership of T_k(g) for one segment [a, b)."""
    st = _f64(s_tilde)
    take = np.zeros(b - a, dtype=np.uint8)
    sc = _load().sablock_ref_segment_score(st.ctypes.data_as(_dp), int(a), int(b), int(g), int(bk),
                                           take.ctypes.data_as(_bp))
    return float(sc), take.astype(bool)


def pipeline_head(q, k, v, seg_off, cand, budget: int, eps=1e-6, alpha=0.9, eta=1.0, tau=0.85,
                  append_window: bool = True, v_raw: Optional[np.ndarray] = None,
                  k_raw: Optional[np.ndarray] = None):
    """All five steps for one KV head, each step fed by the previous one in float64.

    ``k_raw``/``v_raw`` (optional) are the arrays whose rows compaction copies
    (e.g. uint16 bf16 bit patterns); default: ``k``/``v`` themselves.
    """
    W = np.shape(q)[1]
    s, e = score(q, k, eps)
    st, om = refine(s, e, seg_off, alpha, eta)
    b, g = search_blocks(st, seg_off, cand, budget, tau)
    idx, n_sel = select(st, seg_off, b, g, budget)
    ko, vo = compact(k if k_raw is None else k_raw, v if v_raw is None else v_raw, W, idx, n_sel,
                     budget, append_window)
    return dict(s=s, e=e, s_tilde=st, omega=om, b=b, g=g, idx=idx, n_sel=n_sel, k_out=ko, v_out=vo)


def segment(token_ids, delims: Sequence[int]) -> np.ndarray:
    """Punctuation-based segmentation of one sequence's compressible region (Sec. 3.1).

    Walks the tokens in order; a delimiter token closes the segment it is in, so the
    next token (if there is one) starts a new segment.  Returns the offsets
    ``[0, ..., T]`` (int32): segment k is tokens ``off[k] .. off[k+1]-1``.
    """
    ids = [int(x) for x in np.asarray(token_ids).reshape(-1)]
    dset = set(int(d) for d in delims)
    T = len(ids)
    off = [0]
    for t, tok in enumerate(ids):
        if tok in dset and t + 1 < T:
            off.append(t + 1)
    off.append(T)
    return np.asarray(off, dtype=np.int32)


def window_attention(q_win, k, v):
    """Causal attention of the observation-window queries of one KV head over all L keys (Sec. 2.1, Eq. 1): the part
    of the prefill attention whose softmax statistics the scoring step reuses.

    ``q_win [G, W, D]`` (window query i sits at position T + i, T = L - W), ``k, v [L, D]``.  Query i attends to
    keys t <= T + i.  Returns ``(out [G, W, Dv], lse [G, W])`` in float64: ``out = softmax(q . k / sqrt(D)) @ v`` and
    ``lse`` the natural logarithm of the softmax denominator, i.e. log sum_t exp(q . k_t / sqrt(D)) over the visible
    keys.
    """
    q = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    G, W, D = q.shape
    L = k.shape[0]
    T = L - W
    out = np.zeros((G, W, v.shape[1]), dtype=np.float64)
    lse = np.zeros((G, W), dtype=np.float64)
    for g in range(G):
        for i in range(W):
            x = k[:T + i + 1] @ q[g, i] / np.sqrt(float(D))       # the visible keys only
            m = x.max()
            w = np.exp(x - m)
            z = w.sum()
            out[g, i] = (w / z) @ v[:T + i + 1]
            lse[g, i] = m + np.log(z)
    return out, lse


def decode_attention(q, k_rows, v_rows) -> np.ndarray:
    """Attention of one new token over a cache, one KV head (Sec. 2.1, Eq. 1 with a single query position).

    ``q [G, D]`` (the query heads that share the KV head), ``k_rows, v_rows [R, D]`` (the rows that hold an
    entry).  Returns ``[G, D]`` float64: ``softmax_r(q . k_r / sqrt(D)) @ v``; zeros if there is no row.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k_rows, dtype=np.float64)
    v = np.asarray(v_rows, dtype=np.float64)
    G, D = q.shape                               # D: the contraction length that the scale 1/sqrt(D) refers to
    out = np.zeros((G, v.shape[1]), dtype=np.float64)
    if k.shape[0] == 0:
        return out
    for g in range(G):
        x = k @ q[g] / np.sqrt(float(D))
        w = np.exp(x - x.max())
        out[g] = (w / w.sum()) @ v
    return out
