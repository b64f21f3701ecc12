"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before any HIP
call (the pointers used here are never dereferenced)."""
import ctypes
import os
import re

import pytest

from paper_2511_10676_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, E_NULL, E_SHAPE, E_K, E_DTYPE, E_ALIGN, E_WS, E_HIP, E_UNSUP = range(9)
FAKE = ctypes.c_void_p(0x10000)          # aligned, never touched: every case fails validation or is empty
ODD = ctypes.c_void_p(0x10008)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "paep.h")).read()
    declared = set(re.findall(r"\b(paep_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.paep_version() >= 100
    assert lib.paep_status_string(0) == b"ok"
    for s in range(1, 9):
        assert len(lib.paep_status_string(s)) > 3


def _predict(desc, x=FAKE, W1=FAKE, W2=FAKE, idx=FAKE, probs=FAKE, ws=None, ws_bytes=0):
    d = ctypes.byref(desc) if desc is not None else None
    return B.lib().paep_predict(d, x, W1, W2, None, None, idx, probs, None, ws, ws_bytes, None)


def _desc(**kw):
    base = dict(T=0, d=256, r=64, E=16, k=2, L=1, dtype=B.F32)
    base.update(kw)
    return B.make_desc(**base)


def test_predict_rejects_bad_descriptors():
    assert _predict(None) == E_NULL
    assert _predict(_desc(dtype=7)) == E_DTYPE
    bad_act = _desc()
    bad_act.act = 9
    assert _predict(bad_act) == E_DTYPE
    bad_path = _desc()
    bad_path.path = 9
    assert _predict(bad_path) == E_UNSUP
    bad_prob = _desc()
    bad_prob.prob = 3
    assert _predict(bad_prob) == E_DTYPE
    for kw in (dict(T=-1), dict(L=0), dict(d=260), dict(d=0), dict(r=12), dict(E=0), dict(E=1025)):
        assert _predict(_desc(**kw)) == E_SHAPE, kw
    for kw in (dict(k=0), dict(k=17), dict(E=64, k=33)):
        assert _predict(_desc(**kw)) == E_K, kw
    assert _predict(_desc(T=8, L=2, x_layer_stride=8 * 256 - 8)) == E_SHAPE
    assert _predict(_desc(T=8, L=2, w1_layer_stride=64 * 256 + 4)) == E_ALIGN
    assert _predict(_desc(T=8, L=2, w2_layer_stride=-8)) == E_SHAPE


def test_predict_rejects_bad_pointers_and_paths():
    assert _predict(_desc(T=8), x=None) == E_NULL
    assert _predict(_desc(T=8), idx=None) == E_NULL
    assert _predict(_desc(T=0), W2=None) == E_NULL
    assert _predict(_desc(T=0), x=None, idx=None, probs=None) == OK
    assert _predict(_desc(), W1=ODD) == E_ALIGN
    assert _predict(_desc(path="prefill")) == E_UNSUP          # fp32 storage has no matrix-core path
    assert _predict(_desc(path="decode")) == E_UNSUP
    big = _desc(dtype=B.BF16, d=2048, r=2048, E=64, k=6, L=26, T=8)
    need = B.predict_workspace_bytes(big)
    assert need == 4 * 26 * (2048 // 64) * 8 * 64
    assert _predict(big, ws=None, ws_bytes=0) == E_WS
    assert _predict(big, ws=FAKE, ws_bytes=need - 1) == E_WS
    assert _predict(big, ws=ODD, ws_bytes=need) == E_WS


def test_empty_call_is_valid_and_touches_nothing():
    assert _predict(_desc(T=0)) == OK
    assert _predict(_desc(T=0, dtype=B.BF16, d=2048, r=2048, E=64, k=6, L=26)) == OK


def test_path_resolution_by_shape():
    ds = dict(dtype=B.BF16, d=2048, r=2048, E=64, k=6, L=26)
    assert B.resolve_path(_desc(T=1, **ds)) == "decode"
    assert B.resolve_path(_desc(T=64, **ds)) == "decode"
    assert B.resolve_path(_desc(T=65, **ds)) == "prefill"
    assert B.resolve_path(_desc(T=4096, **ds)) == "prefill"
    assert B.resolve_path(_desc(T=512)) == "simple"
    assert B.resolve_path(_desc(T=4096, dtype=B.BF16, d=72, r=40, E=13, k=5)) == "simple"
    assert B.resolve_path(_desc(T=4096, dtype=B.BF16, d=2048, r=4096, E=256, k=8)) == "prefill"
    assert B.resolve_path(_desc(k=0)) == "invalid"
    # with a whole number of rounds of 256 token tiles prefill needs no workspace (32 layers x 16 tiles), nor
    # when the tiles beyond the last full round are too many for cutting them to pay (26 x 16 = 256 + 160) ...
    assert B.predict_workspace_bytes(_desc(T=4096, **dict(ds, L=32))) == 0
    assert B.predict_workspace_bytes(_desc(T=4096, **ds)) == 0
    # ... otherwise those tiles (20 x 16 = 256 + 64) are cut along r into 4 pieces each, whose score tiles of
    # 256 x E fp32 meet in the workspace, plus a ticket per tile ...
    assert B.predict_workspace_bytes(_desc(T=4096, **dict(ds, L=20))) == 64 * 4 * 256 * 64 * 4 + 64 * 4
    # ... and with long rows (d >= 4096) r is split over two co-scheduled workgroups for every tile
    phi = dict(dtype=B.BF16, d=4096, r=1024, E=16, k=2, L=32)
    tiles = (8192 // 256) * 32
    assert B.predict_workspace_bytes(_desc(T=8192, **phi)) == tiles * 2 * 256 * 16 * 4 + tiles * 4
    # few tiles (32 of 128 tokens): r is split over all 8 chunks so that the whole chip streams the weights
    assert B.predict_workspace_bytes(_desc(T=100, **phi)) == 32 * 8 * 128 * 16 * 4 + 32 * 4
    assert B.predict_workspace_bytes(_desc(k=0)) == 0


def _group(idx=FAKE, L=1, T=0, k=2, E=16, outs=(FAKE,) * 6, ws=FAKE, ws_bytes=1 << 20):
    return B.lib().paep_group_by_expert(idx, L, T, k, E, *outs, ws, ws_bytes, None)


def test_group_rejects_bad_arguments():
    assert _group(L=0) == E_SHAPE
    assert _group(T=-1) == E_SHAPE
    assert _group(E=0) == E_SHAPE
    assert _group(E=1025) == E_SHAPE
    assert _group(k=0) == E_K
    assert _group(k=33) == E_K
    assert _group(T=1 << 29, k=2) == E_SHAPE
    assert _group(outs=(None,) + (FAKE,) * 5) == E_NULL
    assert _group(T=4, idx=None) == E_NULL
    # more than 32768 selections per layer: the parts' counts meet in a workspace, (parts + 1) rows of E + 1
    assert _group(T=8192, k=8, E=256, ws=None) == E_WS
    assert _group(T=8192, k=8, E=256, ws_bytes=16) == E_WS
    assert _group(T=8192, k=8, E=256, ws=ODD) == E_WS
    assert B.group_workspace_bytes(1, 8192, 8, 256) == 4 * 9 * 257
    assert B.group_workspace_bytes(3, 8192, 8, 256) == 3 * 4 * 9 * 257
    assert B.group_workspace_bytes(1, 32768, 8, 256) == 4 * 33 * 257
    assert B.group_workspace_bytes(1, 70000, 8, 64) == 4 * 36 * 65              # 35 parts of 16384
    assert B.group_workspace_bytes(1, 262200, 8, 64) == 4 * 66 * 65             # 65 parts of 32768
    assert B.group_workspace_bytes(2, 66000, 16, 1024) == 2 * 4 * 66 * 1025     # 1024 experts: parts of 16384 at most
    # shorter layers run in one launch out of LDS and need none (a NULL workspace is then accepted:
    # checked with real buffers in the GPU tests, since every valid call launches)
    assert B.group_workspace_bytes(1, 4096, 8, 256) == 0
    assert B.group_workspace_bytes(3, 0, 8, 256) == 0
    assert B.group_workspace_bytes(0, 1, 1, 1) == 0


def test_score_rejects_bad_arguments():
    f = B.lib().paep_score
    assert f(FAKE, 2, FAKE, 2, 0, 4, 16, FAKE, None) == E_SHAPE
    assert f(FAKE, 2, FAKE, 2, 1, -4, 16, FAKE, None) == E_SHAPE
    assert f(FAKE, 2, FAKE, 2, 1, 4, 2000, FAKE, None) == E_SHAPE
    assert f(FAKE, 0, FAKE, 2, 1, 4, 16, FAKE, None) == E_K
    assert f(FAKE, 2, FAKE, 40, 1, 4, 16, FAKE, None) == E_K
    assert f(FAKE, 2, FAKE, 2, 1, 4, 16, None, None) == E_NULL
    assert f(None, 2, FAKE, 2, 1, 4, 16, FAKE, None) == E_NULL


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libpaep.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()


def test_score_rows_and_confidence_select_reject_bad_arguments():
    f = B.lib().paep_score_rows
    assert f(FAKE, 2, None, FAKE, 2, 1, 4, 16, FAKE, None) == E_NULL          # widths missing
    assert f(FAKE, 2, FAKE, FAKE, 2, 1, 4, 2000, FAKE, None) == E_SHAPE
    assert f(FAKE, 0, FAKE, FAKE, 2, 1, 4, 16, FAKE, None) == E_K
    assert f(None, 2, None, None, 2, 1, 0, 16, None, None) == E_NULL         # counters missing
    g = B.lib().paep_confidence_select
    import ctypes
    r = ctypes.c_float
    assert g(FAKE, FAKE, 1, 4, 6, 6, r(2.0), FAKE, FAKE, FAKE, None) == E_K      # k_base must be < k_pred
    assert g(FAKE, FAKE, 1, 4, 6, 0, r(2.0), FAKE, FAKE, FAKE, None) == E_K
    assert g(FAKE, FAKE, 1, 4, 1, 1, r(2.0), FAKE, FAKE, FAKE, None) == E_K
    assert g(FAKE, FAKE, 1, 4, 6, 2, r(0.5), FAKE, FAKE, FAKE, None) == E_SHAPE  # ratio below 1
    assert g(FAKE, FAKE, 1, 4, 6, 2, r(float("nan")), FAKE, FAKE, FAKE, None) == E_SHAPE
    assert g(FAKE, FAKE, 0, 4, 6, 2, r(2.0), FAKE, FAKE, FAKE, None) == E_SHAPE
    assert g(FAKE, None, 1, 4, 6, 2, r(2.0), FAKE, FAKE, FAKE, None) == E_NULL
    assert g(FAKE, FAKE, 1, 4, 6, 2, r(2.0), FAKE, FAKE, None, None) == E_NULL


def test_counted_predict_needs_its_counts():
    d = _desc(T=4)
    f = B.lib().paep_predict_counted
    assert f(ctypes.byref(d), FAKE, FAKE, FAKE, None, None, FAKE, FAKE, None, None, FAKE, 1 << 30, None) == E_NULL
    assert f(ctypes.byref(_desc(T=4, k=0)), FAKE, FAKE, FAKE, None, None, FAKE, FAKE, None, FAKE, FAKE, 1 << 30, None) == E_K


def test_plan_reports_the_family_and_the_tile_choice():
    # DeepSeek-V2-Lite-shaped prefill: 256 x 256 tiles, every workgroup walks all eight chunks of r
    p = B.predict_plan(B.make_desc(4096, 2048, 2048, 64, 6, 26, B.BF16))
    assert p == B.Plan("prefill", "256x256", 1, 8)
    # a single layer of the same: too few tiles, r is split over workgroups that meet in the workspace
    p1 = B.predict_plan(B.make_desc(4096, 2048, 2048, 64, 6, 1, B.BF16))
    assert p1.path == "prefill" and p1.groups > 1 and p1.groups * p1.chunks_per_group * 128 in (2048, 4096)
    assert B.predict_plan(B.make_desc(8, 2048, 2048, 64, 6, 26, B.BF16)).path == "decode"
    assert B.predict_plan(B.make_desc(512, 256, 64, 16, 2, 1, B.F32)) == B.Plan("simple", "", 1, 0)
    # a margin output makes the matrix-core family keep one more candidate: k = 16 no longer fits there
    d16 = B.make_desc(4096, 2048, 2048, 64, 16, 26, B.BF16)
    assert B.predict_plan(d16).path == "prefill" and B.predict_plan(d16, want_margin=True).path == "simple"
    bad = B.make_desc(4096, 2048, 2048, 64, 0, 26, B.BF16)
    out = (ctypes.c_int32 * 4)()
    assert B.lib().paep_predict_plan(ctypes.byref(bad), 0, ctypes.byref(out)) == E_K
    assert B.lib().paep_predict_plan(ctypes.byref(d16), 0, None) == E_NULL


def test_confidence_predict_and_fold_reject_bad_arguments():
    f = B.lib().paep_predict_confidence
    d = _desc(T=4)
    assert f(ctypes.byref(d), None, FAKE, FAKE, None, None, FAKE, FAKE, None, None, FAKE, None, 0, None) == E_NULL
    assert f(ctypes.byref(_desc(T=4, k=40, E=64)), FAKE, FAKE, FAKE, None, None, FAKE, FAKE, None, None, FAKE, None, 0, None) == E_K
    pf = B.make_desc(4096, 2048, 2048, 64, 16, 26, B.BF16, path="prefill")
    assert f(ctypes.byref(pf), FAKE, FAKE, FAKE, None, None, FAKE, FAKE, None, None, FAKE, None, 0, None) == E_UNSUP
    g = B.lib().paep_fold_batchnorm
    eps = ctypes.c_float(1e-5)
    assert g(FAKE, None, FAKE, FAKE, FAKE, FAKE, eps, 0, 8, 8, B.F32, FAKE, FAKE, None) == E_SHAPE
    assert g(FAKE, None, FAKE, FAKE, FAKE, FAKE, eps, 1, 8, 8, 5, FAKE, FAKE, None) == E_DTYPE
    assert g(FAKE, None, FAKE, FAKE, FAKE, FAKE, ctypes.c_float(-1.0), 1, 8, 8, B.F32, FAKE, FAKE, None) == E_SHAPE
    assert g(FAKE, None, None, FAKE, FAKE, FAKE, eps, 1, 8, 8, B.F32, FAKE, FAKE, None) == E_NULL
    assert g(FAKE, None, FAKE, FAKE, FAKE, FAKE, eps, 1, 8, 8, B.F32, FAKE, None, None) == E_NULL
