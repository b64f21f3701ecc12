"""paep_predict_static (the entry point that allocates nothing) against paep_predict, through the C ABI:
same kernels, its workspace being the library's built-in buffer, so every output must agree bit for bit.
Two calls in a row on the same device, the second with a smaller input, so that whatever the first left
in the buffer is in the way; then the size limit."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2511_10676_amd import binding as B

pytestmark = pytest.mark.gpu


def _inputs(seed, L, T, d, r, E):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x = torch.randn((L, T, d), device="cuda", generator=g).to(torch.bfloat16)
    W1 = (torch.randn((L, r, d), device="cuda", generator=g) / d ** 0.5).to(torch.bfloat16)
    W2 = (torch.randn((L, E, r), device="cuda", generator=g) / r ** 0.5).to(torch.bfloat16)
    return x, W1, W2


def _both_ways(x, W1, W2, k):
    """(reference through paep_predict with its own workspace, result of paep_predict_static), raw C calls."""
    L, T, d = x.shape
    r, E = W1.shape[1], W2.shape[1]
    lib = B.lib()
    desc = B.make_desc(T, d, r, E, k, L, B.BF16)
    need = B.predict_workspace_bytes(desc)
    assert 0 < need <= B.STATIC_SCRATCH_BYTES, need            # the case must exercise the scratch buffer
    mk = lambda: (torch.full((L, T, k), -7, dtype=torch.int32, device="cuda"),
                  torch.full((L, T, k), -7.0, dtype=torch.float32, device="cuda"),
                  torch.full((L, T, E), -7.0, dtype=torch.float32, device="cuda"))
    ref, got = mk(), mk()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    st = lib.paep_predict(ctypes.byref(desc), p(x), p(W1), p(W2), None, None, p(ref[0]), p(ref[1]), p(ref[2]),
                          p(ws), need, stream)
    assert st == 0
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    st = lib.paep_predict_static(ctypes.byref(desc), p(x), p(W1), p(W2), None, None, p(got[0]), p(got[1]), p(got[2]),
                                 stream)
    assert st == 0
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return ref, got


@pytest.mark.parametrize("first,second", [
    # decode path: fp32 partial scores of every slice of r go through the scratch buffer
    (dict(L=6, T=64, d=512, r=512, E=64, k=6), dict(L=3, T=5, d=512, r=256, E=48, k=4)),
    # prefill path with r split over workgroups: score tiles and tickets go through it
    (dict(L=2, T=700, d=256, r=1024, E=128, k=8), dict(L=1, T=130, d=256, r=512, E=40, k=8)),
    # one after the other across the two families
    (dict(L=2, T=300, d=256, r=512, E=64, k=6), dict(L=26, T=1, d=256, r=128, E=64, k=6)),
])
def test_static_scratch_predict_equals_predict_twice_in_a_row(first, second):
    assert B.lib().paep_static_init() == 0
    for i, c in enumerate((first, second)):
        k = c.pop("k")
        x, W1, W2 = _inputs(40 + i, **c)
        ref, got = _both_ways(x, W1, W2, k)
        for a, b, name in zip(ref, got, ("idx", "probs", "logits")):
            assert torch.equal(a, b), f"call {i}: {name} differs"
        assert bool((got[0] >= 0).all())
        c["k"] = k


def test_static_scratch_predict_refuses_what_does_not_fit_and_launches_nothing():
    # Qwen3-sized bank at 64 tokens: 48 layers x 32 slices x 64 tokens x 128 experts of fp32 partial scores
    desc = B.make_desc(64, 2048, 2048, 128, 8, 48, B.BF16)
    assert B.predict_workspace_bytes(desc) > B.STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)
    st = B.lib().paep_predict_static(ctypes.byref(desc), fake, fake, fake, None, None, fake, fake, None, None)
    assert st == 6                                               # PAEP_ERR_WORKSPACE
    bad = B.make_desc(64, 2048, 2048, 128, 0, 48, B.BF16)
    assert B.lib().paep_predict_static(ctypes.byref(bad), fake, fake, fake, None, None, fake, fake, None, None) == 3


def test_binding_wrapper_runs_on_caller_buffers():
    x, W1, W2 = _inputs(50, L=4, T=8, d=512, r=256, E=64)
    ref = B.predict(x, W1, W2, 6)
    out = B.Prediction(torch.empty_like(ref.idx), torch.empty_like(ref.probs), None, "")
    got = B.predict_static(x, W1, W2, 6, out)
    torch.cuda.synchronize()
    assert got.path == "decode" and torch.equal(got.idx, ref.idx) and torch.equal(got.probs, ref.probs)
