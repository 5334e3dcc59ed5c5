"""CPU-side checks of the HIP library: it loads, exports what the header declares,
and rejects bad host arguments before anything is enqueued (no GPU needed)."""

import ctypes
import os
import re
import sys

import numpy as np
import pytest

from paper_2510_22556_amd import binding as B
from paper_2510_22556_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2510_22556_amd.build import build
        build()
    return B.load()


def _shape(**kw):
    s = B.CShape()
    s.n_seq, s.n_layers, s.n_q_heads, s.n_kv_heads = 1, 1, 4, 2
    s.head_dim, s.seq_len, s.window, s.dtype = 64, 2048, 16, B.SABLOCK_F32
    s.tuning.compute_units = 256            # plans are made for this count: no device is asked
    for a, (qv, kv) in enumerate([(4 * 16 * 64, 2 * 2048 * 64), (4 * 16 * 64, 2 * 2048 * 64), (16 * 64, 2048 * 64), (64, 64)]):
        s.q_stride[a], s.k_stride[a], s.v_stride[a] = qv, kv, kv
    for k, v in kw.items():
        setattr(s.tuning if hasattr(B.CTuning, k) else s, k, v)
    return s


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "sablock.h")).read()
    declared = re.findall(r"SABLOCK_API\s+[\w\s\*]+?\b(sablock_\w+)\s*\(", hdr)
    assert sorted(declared) == sorted(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.sablock_version().decode().startswith("sablock")


def test_struct_layout_matches_header():
    # 8 int32, 3 x 4 int64, then the 8 int32 of the launch parameters: no padding surprises
    assert ctypes.sizeof(B.CShape) == 8 * 4 + 12 * 8 + 8 * 4
    assert B.CShape.q_stride.offset == 32 and B.CShape.v_stride.offset == 96 and B.CShape.tuning.offset == 128
    assert ctypes.sizeof(B.CTuning) == 32 and B.CTuning.stats_per_key.offset == 16
    assert ctypes.sizeof(B.CHparams) == 16
    hdr = open(os.path.join(ROOT, "include", "sablock.h")).read()
    body = re.search(r"typedef struct \{([^}]*)\} sablock_tuning;", hdr).group(1)
    fields = re.findall(r"int32_t\s+(\w+)", body)
    assert fields == [f[0] for f in B.CTuning._fields_]


def test_workspace_bytes_and_shape_validation(lib):
    n = B.sablock_workspace_bytes(_shape(), 100, 112)
    assert n > 0 and n % 256 == 0
    for bad, status in [(dict(n_q_heads=3), 1), (dict(window=2048), 1), (dict(window=0), 1), (dict(dtype=7), 1),
                        (dict(head_dim=60), 2), (dict(head_dim=512), 2), (dict(window=65), 2), (dict(n_seq=0), 1)]:
        with pytest.raises(B.SablockError) as ei:
            B.sablock_workspace_bytes(_shape(**bad), 100, 112)
        assert ei.value.status == status, bad
    with pytest.raises(B.SablockError):
        B.sablock_workspace_bytes(_shape(), -1, 10)


def test_launch_parameters_are_validated_and_change_only_the_plan(lib):
    # out-of-range launch parameters are refused; valid ones change workspace sizes, never the status
    llama = dict(dtype=B.SABLOCK_BF16, head_dim=128, n_q_heads=32, n_kv_heads=8, seq_len=131072, window=32)
    def shape(**kw):                        # dense strides for the Llama geometry
        s = _shape(**kw)
        for a, (qv, kv) in enumerate([(32 * 32 * 128, 8 * 131072 * 128), (32 * 32 * 128, 8 * 131072 * 128),
                                      (32 * 128, 131072 * 128), (128, 128)]):
            s.q_stride[a], s.k_stride[a], s.v_stride[a] = qv, kv, kv
        return s

    for bad in (dict(compute_units=-1), dict(score_chunk=64), dict(score_chunk=1 << 20), dict(window_chunk=8),
                dict(topb_slices=65), dict(topb_slices=-2), dict(stats_per_key=3), dict(stats_per_key=-1)):
        with pytest.raises(B.SablockError) as ei:
            B.sablock_workspace_bytes(shape(**llama, **bad), 100, 112)
        assert ei.value.status == 1, bad
    s = shape(**llama)
    s.tuning.reserved[1] = 3
    with pytest.raises(B.SablockError):
        B.sablock_workspace_bytes(s, 100, 112)
    base = B.sablock_workspace_bytes(shape(**llama), 2100, 992)
    # shorter chunks = more chunk partials of the row statistics; more compute units = more chunks per problem
    few = B.sablock_workspace_bytes(shape(**llama), 0, 0)
    assert B.sablock_workspace_bytes(shape(**llama, score_chunk=1024), 0, 0) > few
    assert B.sablock_workspace_bytes(shape(**llama, compute_units=4096), 0, 0) > few
    assert B.sablock_workspace_bytes(shape(**llama, topb_slices=1), 2100, 992) < base      # no sliced Top-B lists
    # the library reads no environment variable
    os.environ["SABLOCK_SCORE_CHUNK"] = "1024"
    try:
        assert B.sablock_workspace_bytes(shape(**llama), 0, 0) == few
    finally:
        del os.environ["SABLOCK_SCORE_CHUNK"]
    src = os.path.join(ROOT, "paper_2510_22556_amd", "csrc")
    for f in os.listdir(src):
        assert "getenv" not in open(os.path.join(src, f)).read(), f


def test_calls_reject_bad_host_arguments_before_launch(lib):
    s = _shape()
    sp = ctypes.byref(s)
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    ptr2 = (ctypes.c_int32 * 2)(0, 5)
    cand_bad = (ctypes.c_int32 * 3)(2, 4, 8)
    cand_ok = (ctypes.c_int32 * 3)(1, 2, 4)
    cand_desc = (ctypes.c_int32 * 3)(1, 4, 2)
    hp = B.CHparams(1e-6, 0.9, 1.0, 0.85)
    assert lib.sablock_score(sp, None, fake, None, 1e-6, fake, fake, fake, 1 << 30, None) == 1
    assert lib.sablock_score(sp, fake, fake, None, 1e-6, fake, fake, fake, 16, None) == 3       # workspace too small
    assert b"workspace" in lib.sablock_last_error()
    assert lib.sablock_score(sp, ctypes.c_void_p(0x1004), fake, None, 1e-6, fake, fake, fake, 1 << 30, None) == 1
    assert lib.sablock_refine(sp, fake, fake, fake, None, 4, ctypes.byref(hp), fake, None, fake, 0, None) == 1
    assert lib.sablock_refine(sp, fake, fake, fake, ptr2, 2, ctypes.byref(hp), fake, None, fake, 0, None) == 1  # 4 segs > 2
    assert lib.sablock_search_blocks(sp, fake, fake, ptr2, 4, cand_bad, 3, 10, 0.85, fake, fake, None, fake, 1 << 20, None) == 1
    assert lib.sablock_search_blocks(sp, fake, fake, ptr2, 4, cand_desc, 3, 10, 0.85, fake, fake, None, fake, 1 << 20, None) == 1
    assert lib.sablock_search_blocks(sp, fake, fake, ptr2, 4, cand_ok, 3, -1, 0.85, fake, fake, None, fake, 1 << 20, None) == 1
    assert lib.sablock_search_blocks(sp, fake, fake, ptr2, 4, cand_ok, 0, 10, 0.85, fake, fake, None, fake, 1 << 20, None) == 1
    assert lib.sablock_search_blocks(sp, fake, fake, ptr2, 4, cand_ok, 3, 10, 0.85, fake, fake, None, fake, 0, None) == 3
    big = (ctypes.c_int32 * 2)(1, 128)
    assert lib.sablock_search_blocks(sp, fake, fake, ptr2, 4, big, 2, 10, 0.85, fake, fake, None, fake, 1 << 20, None) == 2
    assert lib.sablock_search_select(sp, fake, fake, ptr2, 4, cand_bad, 3, 10, 0.85, fake, fake, None, fake, fake, fake, 1 << 20, None) == 1
    assert lib.sablock_search_select(sp, fake, fake, ptr2, 4, cand_ok, 3, -1, 0.85, fake, fake, None, fake, fake, fake, 1 << 20, None) == 1
    assert lib.sablock_search_select(sp, fake, fake, ptr2, 4, cand_ok, 3, 10, 0.85, fake, fake, None, None, fake, fake, 1 << 20, None) == 1
    assert lib.sablock_search_select(sp, fake, fake, ptr2, 4, cand_ok, 3, 10, 0.85, fake, fake, None, fake, fake, fake, 64, None) == 3
    assert lib.sablock_search_select(sp, fake, fake, ptr2, 4, big, 2, 10, 0.85, fake, fake, None, fake, fake, fake, 1 << 20, None) == 2
    assert lib.sablock_select(sp, fake, fake, ptr2, 4, fake, fake, None, -5, fake, fake, fake, 1 << 20, None) == 1
    assert lib.sablock_select(sp, fake, fake, ptr2, 4, fake, fake, None, 5, fake, fake, fake, 8, None) == 3
    assert lib.sablock_compact(sp, fake, None, fake, fake, 8, 1, fake, fake, None) == 1
    assert lib.sablock_compact(sp, fake, fake, fake, fake, -8, 1, fake, fake, None) == 1
    assert lib.sablock_score(None, fake, fake, None, 1e-6, fake, fake, fake, 0, None) == 1
    # eps keeps the logarithm of a masked or underflowed entry finite: zero, negative and NaN are refused
    for bad_eps in (0.0, -1e-6, float("nan")):
        assert lib.sablock_score(sp, fake, fake, None, bad_eps, fake, fake, fake, 1 << 30, None) == 1
        assert lib.sablock_score_static(sp, fake, fake, None, bad_eps, fake, fake, None) == 1
    assert b"eps" in lib.sablock_last_error()
    # the measurement aid validates like the calls it imitates
    assert lib.sablock_stream_probe(sp, fake, 0, None, None, fake, None) == 2          # fp32, D 64: unsupported
    assert lib.sablock_stream_probe(sp, None, 0, None, None, fake, None) == 1
    assert lib.sablock_stream_probe(sp, fake, 0, fake, None, fake, None) == 1          # only one of the two output rows
    # segmentation
    dl = (ctypes.c_int32 * 2)(11, 13)
    many = (ctypes.c_int32 * 65)(*range(65))
    assert lib.sablock_segment_count(None, 100, 1, 100, dl, 2, fake, None) == 1
    assert lib.sablock_segment_count(fake, 50, 1, 100, dl, 2, fake, None) == 1              # stride < n_tokens
    assert lib.sablock_segment_count(fake, 100, 1, 0, dl, 2, fake, None) == 1
    assert lib.sablock_segment_count(fake, 100, 1, 100, many, 65, fake, None) == 2
    assert lib.sablock_segment_count(fake, 100, 65, 100, dl, 2, fake, None) == 2
    assert lib.sablock_segment_offsets(fake, 100, 1, 100, dl, 2, None, fake, None) == 1
    assert lib.sablock_validate_segments(None, (ctypes.c_int32 * 2)(0, 3), 1, 100, fake, None) == 1
    assert lib.sablock_validate_segments(fake, (ctypes.c_int32 * 2)(0, 3), 1, 100, None, None) == 1
    assert lib.sablock_validate_segments(fake, (ctypes.c_int32 * 2)(0, 1), 1, 100, fake, None) == 1               # < 2 offsets
    assert lib.sablock_validate_segments(fake, (ctypes.c_int32 * 2)(0, 200), 1, 100, fake, None) == 1             # > T + 1
    assert lib.sablock_validate_segments(fake, (ctypes.c_int32 * 2)(0, 3), 65, 100, fake, None) == 2
    assert lib.sablock_segment_offsets(fake, 100, 1, 100, dl, 2, (ctypes.c_int32 * 2)(0, 1), fake, None) == 1     # < 2 offsets
    assert lib.sablock_segment_offsets(fake, 100, 1, 100, dl, 2, (ctypes.c_int32 * 2)(0, 200), fake, None) == 1   # > T + 1


def test_decode_calls_validate_host_arguments(lib):
    def cache_shape(**kw):
        s = _shape(dtype=B.SABLOCK_BF16, head_dim=128, n_q_heads=8, n_kv_heads=2, seq_len=1056, window=1)
        for a, st in enumerate([2 * 1056 * 128, 2 * 1056 * 128, 1056 * 128, 128]):
            s.k_stride[a] = s.v_stride[a] = st
        for k, v in kw.items():
            setattr(s, k, v)
        return s

    n = B.sablock_decode_workspace_bytes(cache_shape())
    assert n > 0 and n % 256 == 0
    fake = ctypes.c_void_p(0x1000)
    sp = ctypes.byref(cache_shape())
    assert lib.sablock_decode_attention(sp, None, fake, fake, None, 0, fake, fake, n, None) == 1
    assert lib.sablock_decode_attention(sp, fake, fake, fake, None, 0, fake, fake, 16, None) == 3
    assert lib.sablock_decode_attention(sp, fake, fake, fake, fake, 2000, fake, fake, n, None) == 1      # budget > rows
    assert lib.sablock_decode_attention(sp, ctypes.c_void_p(0x1008), fake, fake, None, 0, fake, fake, n, None) == 1
    assert B.sablock_decode_workspace_bytes(cache_shape(n_q_heads=6)) > 0                                 # G = 3
    for bad, status in [(dict(n_q_heads=18), 2), (dict(head_dim=24), 2), (dict(seq_len=1), 1), (dict(n_q_heads=7), 1)]:
        with pytest.raises(B.SablockError) as ei:
            B.sablock_decode_workspace_bytes(cache_shape(**bad))
        assert ei.value.status == status, bad


def test_all_head_calls_validate_host_arguments(lib):
    def llama_shape(**kw):
        T, W, D = 4096, 32, 128
        s = _shape(dtype=B.SABLOCK_BF16, head_dim=D, n_q_heads=8, n_kv_heads=2, seq_len=T, window=W)
        for a, (qv, kv) in enumerate([(8 * W * D, 2 * T * D), (8 * W * D, 2 * T * D), (W * D, T * D), (D, D)]):
            s.q_stride[a], s.k_stride[a], s.v_stride[a] = qv, kv, kv
        for k, v in kw.items():
            setattr(s, k, v)
        return s

    n = B.sablock_score_all_heads_workspace_bytes(llama_shape())
    L = 4096 - 32
    assert n >= 2 * L * 32 * 4            # at least the head-group means of both KV heads
    fake = ctypes.c_void_p(0x1000)
    sp = ctypes.byref(llama_shape())
    assert lib.sablock_score_all_heads(sp, None, fake, None, 1e-6, fake, fake, fake, n, None) == 1
    assert lib.sablock_score_all_heads(sp, fake, fake, None, 1e-6, fake, fake, fake, n - 1, None) == 3
    assert lib.sablock_score_all_heads(sp, fake, fake, None, 1e-6, fake, fake, None, n, None) == 3
    assert lib.sablock_score_all_heads(sp, fake, ctypes.c_void_p(0x1008), None, 1e-6, fake, fake, fake, n, None) == 1
    assert lib.sablock_score_all_heads(sp, fake, fake, None, -1.0, fake, fake, fake, n, None) == 1
    for bad in (dict(dtype=B.SABLOCK_F32), dict(head_dim=64), dict(window=64)):
        with pytest.raises(B.SablockError) as ei:
            B.sablock_score_all_heads_workspace_bytes(llama_shape(**bad))
        assert ei.value.status == 2, bad
    # attention of the window queries (same shape family): validation only, nothing is launched
    nw = B.sablock_window_attention_workspace_bytes(llama_shape())
    assert nw >= 256
    assert lib.sablock_window_attention(sp, None, fake, fake, fake, fake, fake, nw, None) == 1
    assert lib.sablock_window_attention(sp, fake, fake, fake, fake, None, fake, nw, None) == 1
    assert lib.sablock_window_attention(sp, fake, fake, ctypes.c_void_p(0x1008), fake, fake, fake, nw, None) == 1
    assert lib.sablock_window_attention(sp, fake, fake, fake, fake, fake, fake, nw - 1, None) == 3
    assert lib.sablock_window_attention(sp, fake, fake, fake, fake, fake, None, nw, None) == 3
    for ok in (dict(window=8), dict(window=16), dict(window=64), dict(n_q_heads=16), dict(n_q_heads=4), dict(n_q_heads=2),
               dict(n_q_heads=6), dict(n_q_heads=14), dict(n_q_heads=10, window=8)):
        assert B.sablock_window_attention_workspace_bytes(llama_shape(**ok)) >= 256, ok
    for bad in (dict(dtype=B.SABLOCK_F32), dict(head_dim=64), dict(window=24), dict(window=128), dict(n_q_heads=18), dict(n_q_heads=32)):
        with pytest.raises(B.SablockError) as ei:
            B.sablock_window_attention_workspace_bytes(llama_shape(**bad))
        assert ei.value.status == 2, bad
    assert lib.sablock_compact_shared(sp, fake, None, fake, fake, 8, 1, fake, fake, None) == 1
    assert lib.sablock_compact_shared(sp, fake, fake, fake, fake, -8, 1, fake, fake, None) == 1
    assert lib.sablock_compact_shared(sp, fake, fake, None, fake, 8, 1, fake, fake, None) == 1
    assert lib.sablock_compact_shared(sp, fake, fake, fake, fake, 8, 1, None, fake, None) == 1
    ls = B.layer_shape(llama_shape())
    assert (ls.n_q_heads, ls.n_kv_heads, ls.seq_len, ls.window) == (1, 1, 4096, 32)


def test_binding_refuses_missing_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        B.load()


def test_synth_backends_agree_and_recipes_hold():
    import torch

    a = synth.hash_u64(77, synth.STREAM_K, 5, 4096)
    b = synth.hash_i64_torch(77, synth.STREAM_K, 5, 4096, "cpu").numpy().view(np.uint64)
    assert (a == b).all()
    x = synth.normal_f32(3, synth.STREAM_Q, (256, 128))
    y = synth.normal_torch(3, synth.STREAM_Q, (256, 128), "cpu").numpy()
    np.testing.assert_allclose(x, y, rtol=1e-6, atol=1e-7)
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1) < 0.02
    bits = synth.f32_to_bf16_bits(x)
    assert (torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16) == bits).all()
    np.testing.assert_array_equal(synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(bits)), bits)
    for w in synth.WORKLOADS.values():
        off, ptr = synth.workload_segments(w)
        assert len(ptr) == w.n_seq + 1
        for s in range(w.n_seq):
            o = off[ptr[s]:ptr[s + 1]]
            assert o[0] == 0 and o[-1] == w.T and (np.diff(o) >= 1).all()
            mean = w.seg_means[s % len(w.seg_means)]
            assert 0.7 * mean < np.diff(o).mean() < 1.3 * mean
            if w.seg_max:
                assert np.diff(o).max() <= w.seg_max + w.seg_min
        assert w.budget() + w.window == w.cache_budgets[0]


def test_paper_defaults_in_workloads():
    vals = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "hyperparameters.txt")):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            vals[k] = v
    w = synth.WORKLOADS["llama8b_128k"]
    assert (w.eps, w.alpha, w.eta, w.tau) == tuple(float(vals[k][0]) for k in ("eps", "alpha", "eta", "tau"))


def test_bench_refuses_more_than_one_gpu():
    # this build runs on one GPU: bench.py says so and exits before it touches a device
    import subprocess

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_algorithmic_bytes_match_the_stated_formulas():
    # algorithmic bytes of a step as bench.py counts them (K once, Q, the score outputs, refine's three arrays,
    # one read of the refined scores, the gathered rows twice): config 4 must come to 2 240 B per token and layer
    # plus the compaction, the figure the roofline fractions are quoted against
    sys.path.insert(0, ROOT)
    import bench

    w = synth.WORKLOADS["llama8b_128k"]
    alg = bench.algorithmic_bytes(w, w.budget())
    per_layer = sum(alg.values()) / w.n_layers
    assert alg["score"] > 0.9 * sum(alg.values())
    k_bytes = w.n_kv_heads * w.seq_len * w.head_dim * 2
    assert abs(alg["score"] / w.n_layers - (k_bytes + w.n_q_heads * w.window * w.head_dim * 2
                                            + 2 * 4 * w.n_kv_heads * w.seq_len)) < 1
    assert 0.29e9 < per_layer < 0.32e9
