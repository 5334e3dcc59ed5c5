"""The scoring entry point that allocates nothing (``sablock_score_static``): same bits as ``sablock_score``.

Its scratch memory is one static array per GPU that keeps the previous call's contents, so the test makes two
calls in a row, the second on a smaller input, and checks each against the call that takes a workspace; a third
call covers the 256-row shape, a fourth the generic kernels, and an oversized call must be refused before
anything is launched.
"""

import ctypes

import numpy as np
import pytest

from paper_2510_22556_amd import synth

pytestmark = pytest.mark.gpu


def _both(torch, B, q, k, eps=1e-6):
    shape = B.make_shape(q, k)
    P, L = B.n_problems(shape), shape.seq_len
    ws = torch.empty((B.sablock_workspace_bytes(shape, 1, 1),), dtype=torch.uint8, device="cuda")
    out = [torch.full((P, L), float("nan"), dtype=torch.float32, device="cuda") for _ in range(4)]
    B.sablock_score(shape, q, k, out[0], out[1], ws, eps)
    B.sablock_score_static(shape, q, k, out[2], out[3], eps)
    torch.cuda.synchronize()
    assert torch.equal(out[0], out[2]) and torch.equal(out[1], out[3])          # bit for bit (NaN would fail too)
    s = out[2].double().sum(dim=1).cpu().numpy()
    np.testing.assert_allclose(s, shape.window, rtol=1e-4)                      # every softmax row sums to one
    return shape


def test_static_scratch_scoring_equals_workspace_scoring():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2510_22556_amd import binding as B

    B.load()
    torch.cuda.set_device(0)
    bf = torch.bfloat16
    # first call: Llama shape, several chunks per problem (row statistics of 3 x 4 problems x 5 chunks in the array)
    G, Hkv, W, D, L = 4, 4, 32, 128, 20000 + 77
    q = synth.normal_torch(901, 1, (1, 3, G * Hkv, W, D), "cuda", bf)
    k = synth.normal_torch(901, 2, (1, 3, Hkv, L, D), "cuda", bf)
    k[0, 1, 2, 12345, :] = (q[0, 1, 2 * G + 1, 7, :].float() * 6.0).to(bf)    # a row whose reference moves
    _both(torch, B, q, k)
    # second call, right behind it, on a smaller input: stale statistics of the first call must not leak in
    L2 = 3000 + 13
    q2 = synth.normal_torch(902, 1, (1, 1, G * 2, W, D), "cuda", bf)
    k2 = synth.normal_torch(902, 2, (1, 1, 2, L2, D), "cuda", bf)
    _both(torch, B, q2, k2)
    # the 256-row shape (its statistics come from another kernel with its own chunking) and the generic kernels
    q3 = synth.normal_torch(903, 1, (2, 1, G * 2, 64, D), "cuda", bf)
    k3 = synth.normal_torch(903, 2, (2, 1, 2, 4000 + 64, D), "cuda", bf)
    _both(torch, B, q3, k3)
    q4 = synth.normal_torch(904, 1, (1, 2, 6, 7, 40), "cuda", torch.float32)
    k4 = synth.normal_torch(904, 2, (1, 2, 2, 1003, 40), "cuda", torch.float32)
    _both(torch, B, q4, k4)
    # with the rows' log-sum-exp given no scratch is needed; result = sablock_score's for the same input
    shape = B.make_shape(q2, k2)
    lse = torch.empty((1, 1, G * 2, W), dtype=torch.float32, device="cuda")
    wws = torch.empty((B.sablock_window_attention_workspace_bytes(shape),), dtype=torch.uint8, device="cuda")
    wout = torch.empty((1, 1, G * 2, W, D), dtype=torch.float32, device="cuda")
    B.sablock_window_attention(shape, q2, k2, k2, wout, lse, wws)
    o = [torch.empty((2, L2), dtype=torch.float32, device="cuda") for _ in range(4)]
    B.sablock_score(shape, q2, k2, o[0], o[1], wws, 1e-6, row_lse=lse)
    B.sablock_score_static(shape, q2, k2, o[2], o[3], 1e-6, row_lse=lse)
    torch.cuda.synchronize()
    assert torch.equal(o[0], o[2]) and torch.equal(o[1], o[3])
    # a call whose statistics exceed the static array is refused with UNSUPPORTED and launches nothing
    big = B.make_shape(q, k, score_chunk=128)
    big.seq_len = 1 << 20
    big.n_layers = 64
    for a, st in enumerate([64 * Hkv * (1 << 20) * D, Hkv * (1 << 20) * D, (1 << 20) * D, D]):
        big.k_stride[a] = big.v_stride[a] = st
    assert B.sablock_workspace_bytes(big, 1, 1) > B.STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: the size check comes first
    lib = B.load()
    assert lib.sablock_score_static(ctypes.byref(big), fake, fake, None, 1e-6, fake, fake, None) == 2
    assert b"static array" in lib.sablock_last_error()
    assert lib.sablock_score_static(ctypes.byref(shape), None, fake, None, 1e-6, fake, fake, None) == 1


def test_static_scratch_scoring_replays_in_a_hip_graph():
    # the callers the entry point is for: a captured graph cannot allocate.  After one eager call on the device (which
    # asks for the array's address) the call only enqueues kernels, so it can be captured; several replays, with eager
    # work and synchronisations between them and the outputs cleared before each, reproduce the eager run bit for bit
    import torch

    from paper_2510_22556_amd import binding as B

    B.load()
    w = synth.WORKLOADS["llama8b_8k"]
    q, k, v = synth.device_tensors(w, "cuda")
    shape = B.make_shape(q, k, v)
    P, L = B.n_problems(shape), shape.seq_len
    s, e = (torch.empty((P, L), dtype=torch.float32, device="cuda") for _ in range(2))
    B.sablock_score_static(shape, q, k, s, e, w.eps)
    torch.cuda.synchronize()
    eager = [s.clone(), e.clone()]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.sablock_score_static(shape, q, k, s, e, w.eps)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        B.sablock_score_static(shape, q, k, s, e, w.eps)
    for rep in range(3):
        s.zero_()
        e.zero_()
        (q.float().sum() + k.float().sum()).item()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(s, eager[0]) and torch.equal(e, eager[1]), f"replay {rep} differs from the eager run"
