"""Thin ctypes binding of ``libsablock.so``: argument marshalling only.

Function names mirror the C ABI (``include/sablock.h``).  Tensors are torch
tensors on the GPU (device memory and the current stream are the only things
torch provides); every step of the path runs in the library's HIP kernels.
There is no CPU fallback: if the library is missing, loading raises.
"""

from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsablock.so")
_lib = None

SABLOCK_OK = 0
STATUS_NAMES = {0: "OK", 1: "INVALID_ARG", 2: "UNSUPPORTED", 3: "WORKSPACE_TOO_SMALL", 4: "DEVICE"}
SABLOCK_F32, SABLOCK_BF16 = 0, 1

EXPORTS = ("sablock_version", "sablock_last_error", "sablock_workspace_bytes", "sablock_score",
           "sablock_refine", "sablock_search_blocks", "sablock_select", "sablock_compact",
           "sablock_segment_count", "sablock_segment_offsets", "sablock_decode_workspace_bytes",
           "sablock_decode_attention", "sablock_score_all_heads_workspace_bytes", "sablock_score_all_heads",
           "sablock_compact_shared", "sablock_search_select", "sablock_window_attention_workspace_bytes",
           "sablock_window_attention", "sablock_score_static", "sablock_stream_probe", "sablock_validate_segments")


class SablockError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"sablock status {status} ({STATUS_NAMES.get(status, '?')}): {msg}")
        self.status = status


class CTuning(ctypes.Structure):
    """Launch parameters (``sablock_tuning``); all zero = the library's own plan."""

    _fields_ = [("compute_units", ctypes.c_int32), ("score_chunk", ctypes.c_int32), ("window_chunk", ctypes.c_int32),
                ("topb_slices", ctypes.c_int32), ("stats_per_key", ctypes.c_int32), ("reserved", ctypes.c_int32 * 3)]


class CShape(ctypes.Structure):
    _fields_ = [("n_seq", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("seq_len", ctypes.c_int32),
                ("window", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("q_stride", ctypes.c_int64 * 4), ("k_stride", ctypes.c_int64 * 4), ("v_stride", ctypes.c_int64 * 4),
                ("tuning", CTuning)]


class CHparams(ctypes.Structure):
    _fields_ = [("eps", ctypes.c_float), ("alpha", ctypes.c_float), ("eta", ctypes.c_float), ("tau", ctypes.c_float)]


def load():
    """Load the HIP library (built in-tree by ``paper_2510_22556_amd.build``); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2510_22556_amd.build` "
                "(there is no fallback path)")
        # torch first: it ships its own copy of the HIP runtime, and a process must hold one runtime only (device
        # pointers and streams of torch are meaningless to a second copy loaded through this library)
        import torch  # noqa: F401

        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        sp = ctypes.POINTER(CShape)
        lib.sablock_version.restype = ctypes.c_char_p
        lib.sablock_last_error.restype = ctypes.c_char_p
        lib.sablock_workspace_bytes.argtypes = [sp, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
        lib.sablock_score.argtypes = [sp, vp, vp, vp, f32, vp, vp, vp, ctypes.c_size_t, vp]
        lib.sablock_score_static.argtypes = [sp, vp, vp, vp, f32, vp, vp, vp]
        lib.sablock_stream_probe.argtypes = [sp, vp, i32, vp, vp, vp, vp]
        lib.sablock_refine.argtypes = [sp, vp, vp, vp, ctypes.POINTER(i32), i32, ctypes.POINTER(CHparams),
                                       vp, vp, vp, ctypes.c_size_t, vp]
        lib.sablock_search_blocks.argtypes = [sp, vp, vp, ctypes.POINTER(i32), i32, ctypes.POINTER(i32), i32,
                                              i32, f32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.sablock_select.argtypes = [sp, vp, vp, ctypes.POINTER(i32), i32, vp, vp, vp, i32, vp, vp, vp,
                                       ctypes.c_size_t, vp]
        lib.sablock_compact.argtypes = [sp, vp, vp, vp, vp, i32, i32, vp, vp, vp]
        lib.sablock_search_select.argtypes = [sp, vp, vp, ctypes.POINTER(i32), i32, ctypes.POINTER(i32), i32, i32, f32,
                                              vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.sablock_segment_count.argtypes = [vp, ctypes.c_int64, i32, i32, ctypes.POINTER(i32), i32, vp, vp]
        lib.sablock_segment_offsets.argtypes = [vp, ctypes.c_int64, i32, i32, ctypes.POINTER(i32), i32,
                                                ctypes.POINTER(i32), vp, vp]
        lib.sablock_validate_segments.argtypes = [vp, ctypes.POINTER(i32), i32, i32, vp, vp]
        lib.sablock_decode_workspace_bytes.argtypes = [sp, ctypes.POINTER(ctypes.c_size_t)]
        lib.sablock_decode_attention.argtypes = [sp, vp, vp, vp, vp, i32, vp, vp, ctypes.c_size_t, vp]
        lib.sablock_score_all_heads_workspace_bytes.argtypes = [sp, ctypes.POINTER(ctypes.c_size_t)]
        lib.sablock_score_all_heads.argtypes = [sp, vp, vp, vp, f32, vp, vp, vp, ctypes.c_size_t, vp]
        lib.sablock_compact_shared.argtypes = [sp, vp, vp, vp, vp, i32, i32, vp, vp, vp]
        lib.sablock_window_attention_workspace_bytes.argtypes = [sp, ctypes.POINTER(ctypes.c_size_t)]
        lib.sablock_window_attention.argtypes = [sp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        for n in EXPORTS[2:]:
            getattr(lib, n).restype = ctypes.c_int
        _lib = lib
    return _lib


def _check(status: int):
    if status != SABLOCK_OK:
        raise SablockError(status, load().sablock_last_error().decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def make_shape(q, k, v=None, **tuning) -> CShape:
    """Shape descriptor from ``q [n_seq, n_layers, Hq, W, D]`` and ``k, v [n_seq, n_layers, Hkv, L, D]``;
    keyword arguments set fields of ``shape.tuning`` (e.g. ``score_chunk=2048``)."""
    import torch

    assert q.dim() == 5 and k.dim() == 5 and q.stride(-1) == 1 and k.stride(-1) == 1
    assert q.dtype == k.dtype and q.dtype in (torch.float32, torch.bfloat16)
    s = CShape()
    s.n_seq, s.n_layers, s.n_q_heads, s.window, s.head_dim = q.shape
    s.n_kv_heads, s.seq_len = k.shape[2], k.shape[3]
    s.dtype = SABLOCK_F32 if q.dtype == torch.float32 else SABLOCK_BF16
    vv = k if v is None else v
    for a in range(4):
        s.q_stride[a] = q.stride(a)
        s.k_stride[a] = k.stride(a)
        s.v_stride[a] = vv.stride(a)
    for name, val in tuning.items():
        setattr(s.tuning, name, int(val))
    return s


@dataclass
class Segments:
    """Segment offsets: ``seg_off`` device int32 CSR, ``seg_ptr`` host ints, ``max_segments`` row stride."""

    seg_off: "object"
    seg_ptr: Sequence[int]
    max_segments: int

    def c_ptr(self):
        return (ctypes.c_int32 * len(self.seg_ptr))(*[int(x) for x in self.seg_ptr])


def make_segments(seg_off_host, seg_ptr_host, device) -> Segments:
    import numpy as np
    import torch

    ptr = [int(x) for x in seg_ptr_host]
    mx = max(ptr[i + 1] - ptr[i] - 1 for i in range(len(ptr) - 1))
    return Segments(torch.as_tensor(np.asarray(seg_off_host, dtype=np.int32)).to(device), ptr, mx)


def sablock_workspace_bytes(shape: CShape, max_segments: int, budget: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().sablock_workspace_bytes(ctypes.byref(shape), max_segments, budget, ctypes.byref(out)))
    return int(out.value)


def n_problems(shape: CShape) -> int:
    return shape.n_seq * shape.n_layers * shape.n_kv_heads


def sablock_score(shape: CShape, q, k, s_out, ent_out, ws, eps: float = 1e-6, row_lse=None, stream=None):
    _check(load().sablock_score(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(row_lse), eps, _ptr(s_out),
                                _ptr(ent_out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def sablock_stream_probe(shape: CShape, k, sink, read_lds: bool = False, s_out=None, ent_out=None, stream=None):
    """Measurement aid: K through the scoring kernels' load ring, no arithmetic; with ``s_out`` / ``ent_out`` also
    the column pass's stores."""
    _check(load().sablock_stream_probe(ctypes.byref(shape), _ptr(k), 1 if read_lds else 0, _ptr(s_out), _ptr(ent_out),
                                       _ptr(sink), _stream(stream)))


STATIC_SCRATCH_BYTES = 8 << 20


def sablock_score_static(shape: CShape, q, k, s_out, ent_out, eps: float = 1e-6, row_lse=None, stream=None):
    """``sablock_score`` without a workspace argument: the row statistics live in the library's own static array."""
    _check(load().sablock_score_static(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(row_lse), eps, _ptr(s_out),
                                       _ptr(ent_out), _stream(stream)))


def sablock_refine(shape: CShape, s, ent, seg: Segments, s_tilde_out, ws, alpha=0.9, eta=1.0,
                   omega_out=None, stream=None):
    hp = CHparams(0.0, alpha, eta, 0.0)
    _check(load().sablock_refine(ctypes.byref(shape), _ptr(s), _ptr(ent), _ptr(seg.seg_off), seg.c_ptr(),
                                 seg.max_segments, ctypes.byref(hp), _ptr(s_tilde_out), _ptr(omega_out),
                                 _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def sablock_search_blocks(shape: CShape, s_tilde, seg: Segments, cand: Sequence[int], budget: int, tau: float,
                          seg_budget_out, block_size_out, ws, stream=None, topb_out=None):
    c = (ctypes.c_int32 * len(cand))(*[int(x) for x in cand])
    _check(load().sablock_search_blocks(ctypes.byref(shape), _ptr(s_tilde), _ptr(seg.seg_off), seg.c_ptr(),
                                        seg.max_segments, c, len(cand), budget, tau, _ptr(seg_budget_out),
                                        _ptr(block_size_out), _ptr(topb_out), _ptr(ws),
                                        ws.numel() * ws.element_size(), _stream(stream)))


def sablock_select(shape: CShape, s_tilde, seg: Segments, seg_budget, block_size, budget: int,
                   idx_out, n_sel_out, ws, stream=None, topb=None):
    _check(load().sablock_select(ctypes.byref(shape), _ptr(s_tilde), _ptr(seg.seg_off), seg.c_ptr(),
                                 seg.max_segments, _ptr(seg_budget), _ptr(block_size), _ptr(topb), budget,
                                 _ptr(idx_out), _ptr(n_sel_out), _ptr(ws), ws.numel() * ws.element_size(),
                                 _stream(stream)))


def sablock_search_select(shape: CShape, s_tilde, seg: Segments, cand: Sequence[int], budget: int, tau: float,
                          seg_budget_out, block_size_out, idx_out, n_sel_out, ws, stream=None, topb_out=None):
    c = (ctypes.c_int32 * len(cand))(*[int(x) for x in cand])
    _check(load().sablock_search_select(ctypes.byref(shape), _ptr(s_tilde), _ptr(seg.seg_off), seg.c_ptr(),
                                        seg.max_segments, c, len(cand), budget, tau, _ptr(seg_budget_out),
                                        _ptr(block_size_out), _ptr(topb_out), _ptr(idx_out), _ptr(n_sel_out),
                                        _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def sablock_compact(shape: CShape, k, v, idx, n_sel, budget: int, append_window: bool, k_out, v_out,
                    stream=None):
    _check(load().sablock_compact(ctypes.byref(shape), _ptr(k), _ptr(v), _ptr(idx), _ptr(n_sel), budget,
                                  1 if append_window else 0, _ptr(k_out), _ptr(v_out), _stream(stream)))


def sablock_segment_count(token_ids, delims: Sequence[int], seg_count_out, stream=None):
    """``token_ids [n_seq, T]`` int32 (row stride in elements taken from the tensor) -> ``seg_count_out [n_seq]``."""
    d = (ctypes.c_int32 * max(len(delims), 1))(*[int(x) for x in delims])
    _check(load().sablock_segment_count(_ptr(token_ids), token_ids.stride(0), token_ids.shape[0], token_ids.shape[1],
                                        d, len(delims), _ptr(seg_count_out), _stream(stream)))


def sablock_segment_offsets(token_ids, delims: Sequence[int], seg_ptr: Sequence[int], seg_off_out, stream=None):
    d = (ctypes.c_int32 * max(len(delims), 1))(*[int(x) for x in delims])
    sp = (ctypes.c_int32 * len(seg_ptr))(*[int(x) for x in seg_ptr])
    _check(load().sablock_segment_offsets(_ptr(token_ids), token_ids.stride(0), token_ids.shape[0],
                                          token_ids.shape[1], d, len(delims), sp, _ptr(seg_off_out), _stream(stream)))


def sablock_validate_segments(seg_off, seg_ptr: Sequence[int], n_tokens: int, n_bad_out, stream=None):
    sp = (ctypes.c_int32 * len(seg_ptr))(*[int(x) for x in seg_ptr])
    _check(load().sablock_validate_segments(_ptr(seg_off), sp, len(seg_ptr) - 1, int(n_tokens), _ptr(n_bad_out),
                                            _stream(stream)))


def segment(token_ids, delims: Sequence[int]) -> "Segments":
    """Both segmentation calls and the host step between them (one read-back of n_seq counts)."""
    import torch

    assert token_ids.dim() == 2 and token_ids.dtype == torch.int32 and token_ids.stride(1) == 1
    counts = torch.empty((token_ids.shape[0],), dtype=torch.int32, device=token_ids.device)
    sablock_segment_count(token_ids, delims, counts)
    c = counts.cpu().tolist()
    ptr = [0]
    for n in c:
        ptr.append(ptr[-1] + n + 1)
    seg_off = torch.empty((ptr[-1],), dtype=torch.int32, device=token_ids.device)
    sablock_segment_offsets(token_ids, delims, ptr, seg_off)
    return Segments(seg_off, ptr, max(c))


def layer_shape(shape: CShape) -> CShape:
    """The shape to pass to refine / search_blocks / select when scores are per (sequence, layer)."""
    s = CShape.from_buffer_copy(shape)
    s.n_q_heads = s.n_kv_heads = 1
    return s


def sablock_score_all_heads_workspace_bytes(shape: CShape) -> int:
    out = ctypes.c_size_t(0)
    _check(load().sablock_score_all_heads_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return int(out.value)


def sablock_score_all_heads(shape: CShape, q, k, s_out, ent_out, ws, eps: float = 1e-6, row_lse=None, stream=None):
    _check(load().sablock_score_all_heads(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(row_lse), eps, _ptr(s_out),
                                          _ptr(ent_out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def sablock_compact_shared(shape: CShape, k, v, idx, n_sel, budget: int, append_window: bool, k_out, v_out,
                           stream=None):
    _check(load().sablock_compact_shared(ctypes.byref(shape), _ptr(k), _ptr(v), _ptr(idx), _ptr(n_sel), budget,
                                         1 if append_window else 0, _ptr(k_out), _ptr(v_out), _stream(stream)))


def sablock_window_attention_workspace_bytes(shape: CShape) -> int:
    out = ctypes.c_size_t(0)
    _check(load().sablock_window_attention_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return int(out.value)


def sablock_window_attention(shape: CShape, q, k, v, out, row_lse_out, ws, stream=None):
    _check(load().sablock_window_attention(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(row_lse_out),
                                           _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def make_cache_shape(q, k_cache, v_cache=None) -> CShape:
    """Shape of a decode call: ``q [n_seq, n_layers, Hq, D]`` and a cache ``[n_seq, n_layers, Hkv, rows, D]``
    (any strides on the four outer axes; a compacted cache ``[P, rows, D]`` is viewed that way by the caller)."""
    import torch

    assert q.dim() == 4 and k_cache.dim() == 5 and q.is_contiguous() and k_cache.stride(-1) == 1
    assert q.dtype == k_cache.dtype and q.dtype in (torch.float32, torch.bfloat16)
    s = CShape()
    s.n_seq, s.n_layers, s.n_q_heads, s.head_dim = q.shape
    s.n_kv_heads, s.seq_len = k_cache.shape[2], k_cache.shape[3]
    s.window = 1
    s.dtype = SABLOCK_F32 if q.dtype == torch.float32 else SABLOCK_BF16
    vv = k_cache if v_cache is None else v_cache
    for a in range(4):
        s.q_stride[a] = 0
        s.k_stride[a] = k_cache.stride(a)
        s.v_stride[a] = vv.stride(a)
    return s


def sablock_decode_workspace_bytes(shape: CShape) -> int:
    out = ctypes.c_size_t(0)
    _check(load().sablock_decode_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return int(out.value)


def sablock_decode_attention(shape: CShape, q, k_cache, v_cache, out, ws, n_sel=None, budget: int = 0, stream=None):
    _check(load().sablock_decode_attention(ctypes.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(n_sel),
                                           budget, _ptr(out), _ptr(ws), ws.numel() * ws.element_size(),
                                           _stream(stream)))


class Buffers:
    """Device buffers for one call geometry: outputs of every step plus the workspace.

    Allocation happens here, once; the five ``sablock_*`` calls then only enqueue kernels.
    """

    def __init__(self, shape: CShape, seg: Segments, budget: int, device, append_window: bool = True,
                 dtype=None):
        import torch

        P, L, W, D = n_problems(shape), shape.seq_len, shape.window, shape.head_dim
        T = L - W
        ms = max(seg.max_segments, 1)
        dt = dtype or (torch.float32 if shape.dtype == SABLOCK_F32 else torch.bfloat16)
        self.budget, self.append_window = budget, append_window
        self.s = torch.empty((P, L), dtype=torch.float32, device=device)
        self.ent = torch.empty((P, L), dtype=torch.float32, device=device)
        self.s_tilde = torch.empty((P, T), dtype=torch.float32, device=device)
        self.omega = torch.empty((P, ms), dtype=torch.float32, device=device)
        self.seg_budget = torch.empty((P, ms), dtype=torch.int32, device=device)
        self.block_size = torch.empty((P, ms), dtype=torch.int32, device=device)
        self.idx = torch.empty((P, max(budget, 1)), dtype=torch.int32, device=device)
        self.n_sel = torch.empty((P,), dtype=torch.int32, device=device)
        self.topb = torch.empty((P, 2), dtype=torch.int32, device=device)
        rows = budget + (W if append_window else 0)
        self.k_out = torch.empty((P, max(rows, 1), D), dtype=dt, device=device)
        self.v_out = torch.empty((P, max(rows, 1), D), dtype=dt, device=device)
        self.ws = torch.empty((sablock_workspace_bytes(shape, seg.max_segments, budget),), dtype=torch.uint8,
                              device=device)


def compress(shape: CShape, q, k, v, seg: Segments, cand: Sequence[int], budget: int, buf: Buffers,
             eps=1e-6, alpha=0.9, eta=1.0, tau=0.85, row_lse=None, stream=None, fused=True) -> Buffers:
    """The whole hot path: score, refine, search_blocks + select (one call for both, or the two separate calls with
    ``fused=False``: same results), compact."""
    sablock_score(shape, q, k, buf.s, buf.ent, buf.ws, eps, row_lse, stream)
    sablock_refine(shape, buf.s, buf.ent, seg, buf.s_tilde, buf.ws, alpha, eta, buf.omega, stream)
    if fused:
        sablock_search_select(shape, buf.s_tilde, seg, cand, budget, tau, buf.seg_budget, buf.block_size, buf.idx,
                              buf.n_sel, buf.ws, stream, topb_out=buf.topb)
    else:
        sablock_search_blocks(shape, buf.s_tilde, seg, cand, budget, tau, buf.seg_budget, buf.block_size, buf.ws,
                              stream, topb_out=buf.topb)
        sablock_select(shape, buf.s_tilde, seg, buf.seg_budget, buf.block_size, budget, buf.idx, buf.n_sel, buf.ws,
                       stream, topb=buf.topb)
    sablock_compact(shape, k, v, buf.idx, buf.n_sel, budget, buf.append_window, buf.k_out, buf.v_out, stream)
    return buf
