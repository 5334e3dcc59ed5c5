"""Seeded synthetic inputs for the SABlock compression path.

This module only *makes inputs*: window queries, keys, values and segment
offsets with the shapes and statistics of the workloads.  It contains none of
the method's arithmetic (no scoring, refinement, search or selection) and is
the only code shared by the HIP path's tests/benchmarks and the CPU oracle's.

Random numbers come from a counter-based generator written here (splitmix64 of
``(seed, stream, element index)`` -> two uniforms -> Box-Muller), so the bits do
not depend on a library's RNG implementation.  Two back ends produce the same
hash stream: numpy (host, small configurations) and torch (device, large
configurations).  Transcendentals may differ in the last ulp between back
ends; wherever the oracle and the HIP path are compared they both read the
bits of one realised tensor.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1

BASE_SEED = 0x5AB10C00

# stream ids: one per tensor kind so tensors of one configuration are independent
STREAM_Q, STREAM_K, STREAM_V, STREAM_SEG, STREAM_HEAVY, STREAM_TOK = 1, 2, 3, 4, 5, 6


# --------------------------------------------------------------------------
# counter-based hash, numpy back end
# --------------------------------------------------------------------------
def _mix_np(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        x = x + np.uint64(_GOLDEN)
        x = (x ^ (x >> np.uint64(30))) * np.uint64(_M1)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(_M2)
        x = x ^ (x >> np.uint64(31))
    return x


def _key(seed: int, stream: int) -> int:
    """Scalar key derived from (seed, stream); python ints, reduced mod 2^64."""
    x = (seed * 0xD1342543DE82EF95 + stream * 0xA0761D6478BD642F + 0x1234567) & _MASK64
    x = (x + _GOLDEN) & _MASK64
    x = ((x ^ (x >> 30)) * _M1) & _MASK64
    x = ((x ^ (x >> 27)) * _M2) & _MASK64
    return x ^ (x >> 31)


def hash_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """uint64 hash of counters ``start .. start+count-1`` under (seed, stream)."""
    ctr = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix_np(ctr * np.uint64(_GOLDEN) ^ np.uint64(_key(seed, stream)))


def uniform01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 uniforms in the open interval (0, 1)."""
    h = hash_u64(seed, stream, start, count)
    return ((h >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal_f32(seed: int, stream: int, shape: Sequence[int], start: int = 0) -> np.ndarray:
    """Standard normals, float32, element e built from counters 2e and 2e+1."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    step = 1 << 22
    for lo in range(0, n, step):
        m = min(step, n - lo)
        u = uniform01(seed, stream, 2 * (start + lo), 2 * m)
        u1, u2 = u[0::2], u[1::2]
        out[lo:lo + m] = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)).astype(np.float32)
    return out.reshape(tuple(shape))


# --------------------------------------------------------------------------
# counter-based hash, torch back end (host or device)
# --------------------------------------------------------------------------
def _to_i64(x: int) -> int:
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(x, s: int):
    """logical right shift of an int64 torch tensor"""
    return (x >> s) & ((1 << (64 - s)) - 1)


def hash_i64_torch(seed: int, stream: int, start: int, count: int, device):
    """Same hash as :func:`hash_u64`, as int64 bit patterns in a torch tensor."""
    import torch

    ctr = torch.arange(start, start + count, dtype=torch.int64, device=device)
    x = (ctr * _to_i64(_GOLDEN)) ^ _to_i64(_key(seed, stream))
    x = x + _to_i64(_GOLDEN)
    x = (x ^ _lsr(x, 30)) * _to_i64(_M1)
    x = (x ^ _lsr(x, 27)) * _to_i64(_M2)
    return x ^ _lsr(x, 31)


def normal_torch(seed: int, stream: int, shape: Sequence[int], device, dtype=None, start: int = 0):
    """Standard normals as a torch tensor on ``device`` (float32, or rounded once to ``dtype``)."""
    import torch

    n = int(np.prod(shape))
    out = torch.empty(n, dtype=dtype or torch.float32, device=device)
    step = 1 << 24
    for lo in range(0, n, step):
        m = min(step, n - lo)
        h = hash_i64_torch(seed, stream, 2 * (start + lo), 2 * m, device)
        u = (_lsr(h, 11).to(torch.float64) + 0.5) * (1.0 / 9007199254740992.0)
        u1, u2 = u[0::2], u[1::2]
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)
        out[lo:lo + m] = z.to(torch.float32).to(out.dtype)
    return out.reshape(tuple(shape))


# --------------------------------------------------------------------------
# bf16 bit helpers (numpy has no bf16 type)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# segments
# --------------------------------------------------------------------------
def segment_offsets(seed: int, T: int, mean: float, min_len: int = 2,
                    max_len: Optional[int] = None, stream: int = STREAM_SEG) -> np.ndarray:
    """Offsets ``0 = o_0 < o_1 < ... < o_K = T`` of contiguous segments.

    Lengths are ``min_len + Geometric(p)`` with ``p = 1/(mean - min_len + 1)``,
    clamped to ``max_len``, laid end to end; the last one is truncated at ``T``
    and merged into its predecessor if it would be shorter than ``min_len``.
    """
    if T <= 0:
        return np.zeros(1, dtype=np.int32)
    p = 1.0 / (mean - min_len + 1.0)
    n_guess = int(T / max(mean, 1.0) * 1.5) + 64
    offs: List[int] = [0]
    ctr = 0
    while offs[-1] < T:
        u = uniform01(seed, stream, ctr, n_guess)
        ctr += n_guess
        if p >= 1.0:
            extra = np.zeros(n_guess, dtype=np.int64)
        else:
            extra = np.floor(np.log(u) / math.log1p(-p)).astype(np.int64)
        lens = min_len + extra
        if max_len is not None:
            lens = np.minimum(lens, max_len)
        for ln in lens.tolist():
            nxt = offs[-1] + ln
            if nxt >= T:
                if T - offs[-1] < min_len and len(offs) > 1:
                    offs[-1] = T
                else:
                    offs.append(T)
                break
            offs.append(nxt)
    return np.asarray(offs, dtype=np.int32)


# --------------------------------------------------------------------------
# rotary position embedding (input preparation for configuration 2)
# --------------------------------------------------------------------------
# Delimiter ids of the synthetic prompts (stand-ins for a tokenizer's comma, period, semicolon, ... ids; the real
# sets belong to tokenizers that are not available here).
DELIMS = (11, 13, 26, 30, 198, 0)


def token_ids(seed: int, n_seq: int, T: int, mean: float, vocab: int = 128256,
              delims: Sequence[int] = DELIMS) -> np.ndarray:
    """Synthetic prompts ``[n_seq, T]`` int32: each token is a delimiter with probability 1/mean (so segment
    lengths are geometric with that mean), otherwise a non-delimiter id below ``vocab``."""
    out = np.empty((n_seq, T), dtype=np.int32)
    dl = np.asarray(delims, dtype=np.int64)
    dset = set(int(d) for d in delims)
    for s in range(n_seq):
        h = hash_u64(seed + 7919 * s, STREAM_TOK, 0, 2 * T)
        u = (h[:T] >> np.uint64(11)).astype(np.float64) / float(1 << 53)
        r = h[T:]
        ids = (r % np.uint64(vocab)).astype(np.int64)
        for d in dset:                                   # keep ordinary tokens off the delimiter ids
            ids[ids == d] = (d + 1) % vocab if ((d + 1) % vocab) not in dset else (d + 7) % vocab
        is_d = u < 1.0 / mean
        ids[is_d] = dl[(r[is_d] >> np.uint64(32)).astype(np.int64) % len(dl)]
        out[s] = ids.astype(np.int32)
    return out


def apply_rope(x: np.ndarray, positions: np.ndarray, base: float = 500000.0) -> np.ndarray:
    """Rotate ``x[..., pos, D]`` by position; half-split pairing (d, d + D/2)."""
    D = x.shape[-1]
    half = D // 2
    inv = base ** (-np.arange(half, dtype=np.float64) / half)
    ang = positions.astype(np.float64)[:, None] * inv[None, :]
    c, s = np.cos(ang), np.sin(ang)
    x1 = x[..., :half].astype(np.float64)
    x2 = x[..., half:].astype(np.float64)
    out = np.empty_like(x, dtype=np.float32)
    out[..., :half] = (x1 * c - x2 * s).astype(np.float32)
    out[..., half:] = (x1 * s + x2 * c).astype(np.float32)
    return out


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    """One benchmark configuration (shapes and recipe, no data)."""

    name: str
    cfg: int
    n_seq: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int
    window: int
    dtype: str                      # "f32" or "bf16"
    cand: Tuple[int, ...]
    cache_budgets: Tuple[int, ...]  # total retained entries (selected + window)
    seg_means: Tuple[float, ...]    # per sequence (cycled)
    seg_min: int = 2
    seg_max: Optional[int] = None   # None: 8 x mean
    rope: bool = False
    heavy_rows: int = 0
    heavy_scale: float = 4.0
    # paper hyperparameters (Implementation Details, Sec. 4.1)
    eps: float = 1e-6
    alpha: float = 0.9
    eta: float = 1.0
    tau: float = 0.85

    @property
    def T(self) -> int:
        return self.seq_len - self.window

    @property
    def G(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def budget(self, i: int = 0) -> int:
        """Entries to choose from the compressible region: cache budget minus the window."""
        return max(self.cache_budgets[i] - self.window, 0)

    def seed(self, layer: int = 0, seq: int = 0) -> int:
        return BASE_SEED + 256 * self.cfg + layer + 7919 * seq


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 1, 1, 1, 4, 2, 64, 2048, 16, "f32", (1, 2, 4, 8), (128,),
                     (24.0,), 2, 128),
    "llama8b_8k": Workload("llama8b_8k", 2, 1, 1, 32, 8, 128, 8192, 32, "bf16",
                           (1, 2, 4, 8, 16, 32), (1024,), (32.0,), 2, 256, rope=True),
    "llama8b_32k_heavy": Workload("llama8b_32k_heavy", 3, 1, 32, 32, 8, 128, 32768, 32, "bf16",
                                  (1, 2, 4, 8, 16, 32), (96, 256, 1024), (48.0,), 2, 384,
                                  heavy_rows=64),
    "llama8b_128k": Workload("llama8b_128k", 4, 1, 32, 32, 8, 128, 131072, 32, "bf16",
                             (1, 2, 4, 8, 16, 32, 64), (1024,), (64.0,), 2, 512),
    "llama8b_4x64k": Workload("llama8b_4x64k", 5, 4, 32, 32, 8, 128, 65536, 64, "bf16",
                              (1, 2, 4, 8, 16, 32, 64), (2048,), (16.0, 64.0, 256.0, 16.0), 2, None),
    # the paper's own settings (Implementation Details, Sec. 4.1; block sizes of Sec. 4.4): window of 8 recent
    # tokens, candidate block sizes up to g_max = 13, on the same head shape; mean segment of 28 tokens, the
    # length at which a block of 7 crosses a boundary about 21.65 % of the time (Sec. 2.2)
    "paper_defaults_32k": Workload("paper_defaults_32k", 6, 1, 32, 32, 8, 128, 32768, 8, "bf16",
                                   (1, 2, 3, 5, 7, 9, 11, 13), (96, 128, 1024), (28.0,), 2, 224, rope=True),
    # a head shape whose group size is no power of two (28 query / 4 KV heads, 28 layers: seven heads per KV head,
    # 112 window-query rows in four row tiles, the last one half padding), outside the paper's models
    "gqa7_32k": Workload("gqa7_32k", 7, 1, 28, 28, 4, 128, 32768, 16, "bf16",
                         (1, 2, 4, 8, 16, 32), (1024,), (32.0,), 2, 256, rope=True),
}


def workload_segments(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Segment offsets for every sequence, concatenated (CSR).

    Returns ``(seg_off, seg_ptr)``: sequence ``s`` owns
    ``seg_off[seg_ptr[s] : seg_ptr[s+1]]`` (its first entry 0, its last ``T``).
    """
    parts, ptr = [], [0]
    for s in range(w.n_seq):
        mean = w.seg_means[s % len(w.seg_means)]
        mx = w.seg_max if w.seg_max is not None else int(8 * mean)
        o = segment_offsets(w.seed(0, s), w.T, mean, w.seg_min, mx)
        parts.append(o)
        ptr.append(ptr[-1] + len(o))
    return np.concatenate(parts).astype(np.int32), np.asarray(ptr, dtype=np.int32)


def heavy_positions(w: Workload, layer: int, seq: int = 0) -> np.ndarray:
    """Distinct seeded key positions in [0, T) whose K rows are scaled up."""
    if w.heavy_rows <= 0:
        return np.zeros(0, dtype=np.int64)
    h = hash_u64(w.seed(layer, seq), STREAM_HEAVY, 0, 4 * w.heavy_rows)
    pos, seen = [], set()
    for v in (h % np.uint64(w.T)).tolist():
        if v not in seen:
            seen.add(v)
            pos.append(v)
        if len(pos) == w.heavy_rows:
            break
    return np.asarray(sorted(pos), dtype=np.int64)


def host_layer(w: Workload, layer: int = 0, seq: int = 0):
    """Q window, K, V of one (sequence, layer) on the host.

    Returns float32 arrays ``q [Hq, W, D]``, ``k [Hkv, L, D]``, ``v [Hkv, L, D]``;
    for bf16 workloads the values are already rounded to bf16 (representable
    exactly), so ``f32_to_bf16_bits`` of them is lossless.
    """
    seed = w.seed(layer, seq)
    q = normal_f32(seed, STREAM_Q, (w.n_q_heads, w.window, w.head_dim))
    k = normal_f32(seed, STREAM_K, (w.n_kv_heads, w.seq_len, w.head_dim))
    v = normal_f32(seed, STREAM_V, (w.n_kv_heads, w.seq_len, w.head_dim))
    if w.rope:
        q = apply_rope(q, np.arange(w.T, w.seq_len))
        k = apply_rope(k, np.arange(w.seq_len))
    hp = heavy_positions(w, layer, seq)
    if hp.size:
        k[:, hp, :] *= np.float32(w.heavy_scale)
    if w.dtype == "bf16":
        q = bf16_bits_to_f32(f32_to_bf16_bits(q))
        k = bf16_bits_to_f32(f32_to_bf16_bits(k))
        v = bf16_bits_to_f32(f32_to_bf16_bits(v))
    return q, k, v


def device_tensors(w: Workload, device, n_layers: Optional[int] = None, with_v: bool = True):
    """Q window, K, V of the whole workload as torch tensors on ``device``.

    Layouts: ``q [n_seq, n_layers, Hq, W, D]``, ``k, v [n_seq, n_layers, Hkv, L, D]``,
    dtype float32 or bfloat16 per the workload.  Generated per (sequence, layer)
    with the same counter streams as :func:`host_layer`.
    """
    import torch

    nl = w.n_layers if n_layers is None else n_layers
    dt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    q = torch.empty((w.n_seq, nl, w.n_q_heads, w.window, w.head_dim), dtype=dt, device=device)
    k = torch.empty((w.n_seq, nl, w.n_kv_heads, w.seq_len, w.head_dim), dtype=dt, device=device)
    v = torch.empty_like(k) if with_v else None
    for s in range(w.n_seq):
        for l in range(nl):
            seed = w.seed(l, s)
            qf = normal_torch(seed, STREAM_Q, q.shape[2:], device)
            kf = normal_torch(seed, STREAM_K, k.shape[2:], device)
            if w.rope:
                qf = _rope_torch(qf, torch.arange(w.T, w.seq_len, device=device))
                kf = _rope_torch(kf, torch.arange(w.seq_len, device=device))
            hp = heavy_positions(w, l, s)
            if hp.size:
                kf[:, torch.as_tensor(hp, device=device), :] *= w.heavy_scale
            q[s, l] = qf.to(dt)
            k[s, l] = kf.to(dt)
            if with_v:
                v[s, l] = normal_torch(seed, STREAM_V, k.shape[2:], device).to(dt)
    return q, k, v


def _rope_torch(x, positions, base: float = 500000.0):
    import torch

    D = x.shape[-1]
    half = D // 2
    inv = base ** (-torch.arange(half, dtype=torch.float64, device=x.device) / half)
    ang = positions.to(torch.float64)[:, None] * inv[None, :]
    c, s = torch.cos(ang), torch.sin(ang)
    x1 = x[..., :half].to(torch.float64)
    x2 = x[..., half:].to(torch.float64)
    return torch.cat([(x1 * c - x2 * s).to(torch.float32), (x1 * s + x2 * c).to(torch.float32)], dim=-1)
