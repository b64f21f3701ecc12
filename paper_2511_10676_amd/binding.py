"""Python binding of the C-ABI library declared in ``include/paep.h``.

Argument marshalling only: tensors (PyTorch-ROCm, used for device memory and
streams and nothing else) are checked, their device pointers and the current
HIP stream are handed to the C entry points of the same names, and a non-zero
status becomes an exception.  There is no fallback: if ``libpaep.so`` has not
been built (``python -m paper_2511_10676_amd.build``), loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpaep.so")

# enums of paep.h
F32, BF16 = 0, 1
ACT = {"none": 0, "silu": 1, "gelu": 2}
PATH = {"auto": 0, "simple": 1, "decode": 2, "prefill": 3}
PATH_NAME = {v: k for k, v in PATH.items()}
PROB = {"softmax": 0, "softmax_topk": 1, "sigmoid": 2}
TILE_CFG = {0: "128x128", 1: "128x128 wide", 2: "256x256", 3: "256x128", 4: "256x256 wide"}
MAX_K, MAX_E = 32, 1024

STATUS_NAMES = ["PAEP_OK", "PAEP_ERR_NULL", "PAEP_ERR_SHAPE", "PAEP_ERR_K", "PAEP_ERR_DTYPE",
                "PAEP_ERR_ALIGN", "PAEP_ERR_WORKSPACE", "PAEP_ERR_HIP", "PAEP_ERR_UNSUPPORTED"]

STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = ["paep_predict_workspace_bytes", "paep_predict_resolve_path", "paep_predict_plan", "paep_predict",
           "paep_static_init", "paep_predict_static",
           "paep_predict_counted", "paep_predict_confidence", "paep_fold_batchnorm",
           "paep_group_workspace_bytes", "paep_group_by_expert", "paep_score",
           "paep_score_rows", "paep_confidence_select", "paep_activation_profile", "paep_probe_read",
           "paep_probe_mfma", "paep_status_string", "paep_version"]


class PredictDesc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("r", ctypes.c_int32),
                ("E", ctypes.c_int32), ("k", ctypes.c_int32), ("L", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("act", ctypes.c_int32), ("path", ctypes.c_int32),
                ("prob", ctypes.c_int32),
                ("x_layer_stride", ctypes.c_int64), ("w1_layer_stride", ctypes.c_int64),
                ("w2_layer_stride", ctypes.c_int64)]


class PaepError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        try:
            msg = lib().paep_status_string(status).decode()
        except Exception:  # pragma: no cover
            msg = ""
        super().__init__(f"{where}: {name} ({msg})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2511_10676_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        dp = ctypes.POINTER(PredictDesc)
        L.paep_predict_workspace_bytes.argtypes = [dp]
        L.paep_predict_workspace_bytes.restype = sz
        L.paep_predict_resolve_path.argtypes = [dp]
        L.paep_predict_resolve_path.restype = ctypes.c_int
        L.paep_predict.argtypes = [dp] + [vp] * 9 + [sz, vp]
        L.paep_predict.restype = ctypes.c_int
        L.paep_predict_counted.argtypes = [dp] + [vp] * 10 + [sz, vp]
        L.paep_predict_counted.restype = ctypes.c_int
        L.paep_predict_confidence.argtypes = [dp] + [vp] * 11 + [sz, vp]
        L.paep_predict_confidence.restype = ctypes.c_int
        L.paep_predict_static.argtypes = [dp] + [vp] * 8 + [vp]
        L.paep_predict_static.restype = ctypes.c_int
        L.paep_static_init.argtypes = []
        L.paep_static_init.restype = ctypes.c_int
        L.paep_predict_plan.argtypes = [dp, i32, ctypes.POINTER(ctypes.c_int32 * 4)]
        L.paep_predict_plan.restype = ctypes.c_int
        L.paep_fold_batchnorm.argtypes = [vp] * 6 + [ctypes.c_float] + [i32] * 4 + [vp] * 3
        L.paep_fold_batchnorm.restype = ctypes.c_int
        L.paep_group_workspace_bytes.argtypes = [i32] * 4
        L.paep_group_workspace_bytes.restype = sz
        L.paep_group_by_expert.argtypes = [vp] + [i32] * 4 + [vp] * 7 + [sz, vp]
        L.paep_group_by_expert.restype = ctypes.c_int
        L.paep_score.argtypes = [vp, i32, vp, i32, i32, i32, i32, vp, vp]
        L.paep_score.restype = ctypes.c_int
        L.paep_score_rows.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, vp, vp]
        L.paep_score_rows.restype = ctypes.c_int
        L.paep_confidence_select.argtypes = [vp, vp, i32, i32, i32, i32, ctypes.c_float, vp, vp, vp, vp]
        L.paep_confidence_select.restype = ctypes.c_int
        L.paep_activation_profile.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.paep_activation_profile.restype = ctypes.c_int
        L.paep_probe_read.argtypes = [vp, sz, vp, sz, vp]
        L.paep_probe_read.restype = ctypes.c_int
        L.paep_probe_mfma.argtypes = [i32, i32, vp, sz, vp, ctypes.POINTER(ctypes.c_double)]
        L.paep_probe_mfma.restype = ctypes.c_int
        L.paep_status_string.argtypes = [ctypes.c_int]
        L.paep_status_string.restype = ctypes.c_char_p
        L.paep_version.restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _on(stream):
    """Context in which torch allocates on `stream` (its caching allocator ties a block to the stream that
    was current when it was handed out): temporaries made for a call must belong to the stream the call's
    kernels are enqueued on, or the allocator may hand them to someone else while those kernels still run."""
    import contextlib
    return contextlib.nullcontext() if stream is None else torch.cuda.stream(stream)


def _storage_dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported storage dtype {t.dtype}; use float32 or bfloat16")


def _need_device(*tensors):
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("every tensor must be a contiguous device tensor")


class Prepared:
    """One library call with its arguments marshalled once.  Calling the object enqueues the work on
    `stream` (default: torch's current stream) at the cost of a single foreign call -- for loops that
    repeat the same call on the same buffers (a decode step per token)."""

    __slots__ = ("_fn", "_name", "_args", "_keep", "result")

    def __init__(self, fn, name, args, keep, result):
        self._fn, self._name, self._args, self._keep, self.result = fn, name, args, keep, result

    def __call__(self, stream=None):
        st = self._fn(*self._args, _stream_ptr(stream))
        if st != 0:
            raise PaepError(st, self._name)
        return self.result


class Prediction(NamedTuple):
    idx: torch.Tensor                 # [L, T, k] int32
    probs: torch.Tensor               # [L, T, k] float32
    logits: Optional[torch.Tensor]    # [L, T, E] float32 or None
    path: str
    margin: Optional[torch.Tensor] = None   # [L, T] float32: last selected score minus the best one left out


class Plan(NamedTuple):
    path: str
    tile: str                 # prefill tile configuration ("" on the other paths)
    groups: int               # workgroups sharing one token tile (r split between them)
    chunks_per_group: int


def make_desc(T, d, r, E, k, L, dtype, act="none", path="auto",
              x_layer_stride=None, w1_layer_stride=None, w2_layer_stride=None, prob="softmax") -> PredictDesc:
    return PredictDesc(T=T, d=d, r=r, E=E, k=k, L=L, dtype=dtype, act=ACT[act], path=PATH[path], prob=PROB[prob],
                       x_layer_stride=T * d if x_layer_stride is None else x_layer_stride,
                       w1_layer_stride=r * d if w1_layer_stride is None else w1_layer_stride,
                       w2_layer_stride=E * r if w2_layer_stride is None else w2_layer_stride)


def predict_workspace_bytes(desc: PredictDesc) -> int:
    return int(lib().paep_predict_workspace_bytes(ctypes.byref(desc)))


def resolve_path(desc: PredictDesc) -> str:
    p = int(lib().paep_predict_resolve_path(ctypes.byref(desc)))
    return PATH_NAME.get(p, "invalid")


def predict_plan(desc: PredictDesc, want_margin: bool = False) -> Plan:
    """How paep_predict will run this shape (kernel family, prefill tile configuration, r split)."""
    out = (ctypes.c_int32 * 4)()
    st = lib().paep_predict_plan(ctypes.byref(desc), int(bool(want_margin)), ctypes.byref(out))
    if st != 0:
        raise PaepError(st, "paep_predict_plan")
    path = PATH_NAME.get(out[0], "invalid")
    return Plan(path, TILE_CFG.get(out[1], "?") if path == "prefill" else "", int(out[2]), int(out[3]))


def _check_predict_inputs(x, W1, W2, k, b1, b2, act, path, prob):
    """Shape and dtype checks shared by the predict calls; returns the 3-D views and the descriptor."""
    if W1.dim() == 2:
        W1 = W1.unsqueeze(0)
    if W2.dim() == 2:
        W2 = W2.unsqueeze(0)
    if x.dim() == 2:
        x = x.unsqueeze(0)
    _need_device(x, W1, W2, b1, b2)
    L, r, d = W1.shape
    L2, E, r2 = W2.shape
    Lx, T, dx = x.shape
    if L2 != L or r2 != r or dx != d or Lx not in (1, L):
        raise ValueError(f"shape mismatch: x{tuple(x.shape)} W1{tuple(W1.shape)} W2{tuple(W2.shape)}")
    dt = _storage_dtype(x)
    if _storage_dtype(W1) != dt or _storage_dtype(W2) != dt:
        raise TypeError("x, W1 and W2 must share one storage dtype")
    for b, n in ((b1, r), (b2, E)):
        if b is not None and (b.numel() != L * n or _storage_dtype(b) != dt):
            raise ValueError("bias must be [L, r] / [L, E] in the storage dtype")
    desc = make_desc(T, d, r, E, k, L, dt, act, path, x_layer_stride=(T * d if Lx == L and L > 1 else 0), prob=prob)
    if L == 1:
        desc.x_layer_stride = T * d
    return x, W1, W2, desc, (L, T, E)


def prepare_predict(x: torch.Tensor, W1: torch.Tensor, W2: torch.Tensor, k: int, *,
                    b1: Optional[torch.Tensor] = None, b2: Optional[torch.Tensor] = None,
                    act: str = "none", path: str = "auto", want_logits: bool = False,
                    out: Optional[Prediction] = None, workspace: Optional[torch.Tensor] = None,
                    counts: Optional[torch.Tensor] = None, prob: str = "softmax",
                    want_margin: bool = False) -> Prepared:
    """Check and marshal one predict call; the returned object runs it (see `predict` for the arguments)."""
    x, W1, W2, desc, (L, T, E) = _check_predict_inputs(x, W1, W2, k, b1, b2, act, path, prob)
    dev = x.device
    if out is None:
        idx = torch.empty((L, T, k), dtype=torch.int32, device=dev)
        probs = torch.empty((L, T, k), dtype=torch.float32, device=dev)
        logits = torch.empty((L, T, E), dtype=torch.float32, device=dev) if want_logits else None
        margin = torch.empty((L, T), dtype=torch.float32, device=dev) if want_margin else None
    else:
        idx, probs, logits, margin = out.idx, out.probs, out.logits, out.margin
        _need_device(idx, probs, logits, margin)
        if margin is not None and (tuple(margin.shape) != (L, T) or margin.dtype != torch.float32):
            raise ValueError("margin buffer has the wrong shape or dtype")
        if tuple(idx.shape) != (L, T, k) or tuple(probs.shape) != (L, T, k) or idx.dtype != torch.int32 \
                or probs.dtype != torch.float32:
            raise ValueError("out buffers have the wrong shape or dtype")
        if logits is not None and (tuple(logits.shape) != (L, T, E) or logits.dtype != torch.float32):
            raise ValueError("logits buffer has the wrong shape or dtype")
    need = predict_workspace_bytes(desc)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if counts is not None:
        _need_device(counts)
        if counts.dtype != torch.int32 or tuple(counts.shape) != (L, E):
            raise ValueError("counts must be int32 [L, E]")
    if margin is not None:
        # the family is chosen knowing that one more candidate per row is kept
        args = (ctypes.byref(desc), _ptr(x), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(b2),
                _ptr(idx), _ptr(probs), _ptr(logits), _ptr(counts), _ptr(margin), _ptr(workspace), ws_bytes)
        fam = predict_plan(desc, True).path
        return Prepared(lib().paep_predict_confidence, "paep_predict_confidence", args,
                        (desc, x, W1, W2, b1, b2, workspace, counts), Prediction(idx, probs, logits, fam, margin))
    result = Prediction(idx, probs, logits, resolve_path(desc))
    if counts is not None:
        args = (ctypes.byref(desc), _ptr(x), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(b2),
                _ptr(idx), _ptr(probs), _ptr(logits), _ptr(counts), _ptr(workspace), ws_bytes)
        return Prepared(lib().paep_predict_counted, "paep_predict_counted", args,
                        (desc, x, W1, W2, b1, b2, workspace, counts), result)
    args = (ctypes.byref(desc), _ptr(x), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(b2),
            _ptr(idx), _ptr(probs), _ptr(logits), _ptr(workspace), ws_bytes)
    return Prepared(lib().paep_predict, "paep_predict", args, (desc, x, W1, W2, b1, b2, workspace), result)


def predict(x: torch.Tensor, W1: torch.Tensor, W2: torch.Tensor, k: int, *,
            b1: Optional[torch.Tensor] = None, b2: Optional[torch.Tensor] = None,
            act: str = "none", path: str = "auto", want_logits: bool = False,
            out: Optional[Prediction] = None, workspace: Optional[torch.Tensor] = None,
            counts: Optional[torch.Tensor] = None, prob: str = "softmax", want_margin: bool = False,
            stream=None) -> Prediction:
    """predict(x[L|1,T,d], W1[L,r,d], W2[L,E,r], k) -> idx[L,T,k], probs[L,T,k].

    2-D inputs are taken as one layer.  x with a leading dimension of 1 (or
    2-D x with 3-D weights) feeds the same tokens to every layer.  `out` and
    `workspace` let a caller reuse buffers; otherwise they are allocated here.
    `counts` (int32 [L, E]) is increased by the activation counts of this call.
    `prob` picks what probs holds ("softmax" over all E, "softmax_topk" over the k selected, "sigmoid");
    `want_margin` adds margin[L, T], the last selected score minus the best one left out.
    Buffers allocated here are allocated on `stream`, the stream the kernels run on.
    """
    with _on(stream):
        prep = prepare_predict(x, W1, W2, k, b1=b1, b2=b2, act=act, path=path, want_logits=want_logits, out=out,
                               workspace=workspace, counts=counts, prob=prob, want_margin=want_margin)
    return prep(stream)


def static_init() -> None:
    """Bind the library's built-in scratch buffer on the current device (once per device, before graph capture)."""
    st = lib().paep_static_init()
    if st != 0:
        raise PaepError(st, "paep_static_init")


def predict_static(x: torch.Tensor, W1: torch.Tensor, W2: torch.Tensor, k: int, out: Prediction, *,
                   b1: Optional[torch.Tensor] = None, b2: Optional[torch.Tensor] = None,
                   act: str = "none", path: str = "auto", prob: str = "softmax", stream=None) -> Prediction:
    """paep_predict_static: predict into caller-provided `out` buffers using the library's built-in scratch
    buffer; nothing is allocated (shapes that need more than STATIC_SCRATCH_BYTES of workspace raise)."""
    x, W1, W2, desc, (L, T, E) = _check_predict_inputs(x, W1, W2, k, b1, b2, act, path, prob)
    _need_device(out.idx, out.probs, out.logits)
    if tuple(out.idx.shape) != (L, T, k) or tuple(out.probs.shape) != (L, T, k) or out.idx.dtype != torch.int32 \
            or out.probs.dtype != torch.float32:
        raise ValueError("out buffers have the wrong shape or dtype")
    if out.logits is not None and (tuple(out.logits.shape) != (L, T, E) or out.logits.dtype != torch.float32):
        raise ValueError("logits buffer has the wrong shape or dtype")
    st = lib().paep_predict_static(ctypes.byref(desc), _ptr(x), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(b2),
                                   _ptr(out.idx), _ptr(out.probs), _ptr(out.logits), _stream_ptr(stream))
    if st != 0:
        raise PaepError(st, "paep_predict_static")
    return Prediction(out.idx, out.probs, out.logits, resolve_path(desc))


class Grouping(NamedTuple):
    counts: torch.Tensor      # [L, E] int32
    offsets: torch.Tensor     # [L, E+1] int32
    token_pos: torch.Tensor   # [L, T*k] int32
    active: torch.Tensor      # [L, E] int32
    n_active: torch.Tensor    # [L] int32
    n_invalid: torch.Tensor   # [L] int32


def group_workspace_bytes(L: int, T: int, k: int, E: int) -> int:
    return int(lib().paep_group_workspace_bytes(L, T, k, E))


def alloc_grouping(L: int, T: int, k: int, E: int, device) -> Grouping:
    i32 = dict(dtype=torch.int32, device=device)
    return Grouping(torch.empty((L, E), **i32), torch.empty((L, E + 1), **i32),
                    torch.empty((L, T * k), **i32), torch.empty((L, E), **i32),
                    torch.empty((L,), **i32), torch.empty((L,), **i32))


def prepare_group_by_expert(idx: torch.Tensor, E: int, *, out: Optional[Grouping] = None,
                            workspace: Optional[torch.Tensor] = None) -> Prepared:
    """Check and marshal one group_by_expert call; the returned object runs it."""
    if idx.dim() == 2:
        idx = idx.unsqueeze(0)
    _need_device(idx)
    if idx.dtype != torch.int32 or idx.dim() != 3:
        raise TypeError("idx must be int32 [L, T, k]")
    L, T, k = idx.shape
    if out is None:
        out = alloc_grouping(L, T, k, E, idx.device)
    need = group_workspace_bytes(L, T, k, E)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=idx.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    args = (_ptr(idx), L, T, k, E, _ptr(out.counts), _ptr(out.offsets), _ptr(out.token_pos), _ptr(out.active),
            _ptr(out.n_active), _ptr(out.n_invalid), _ptr(workspace), ws_bytes)
    return Prepared(lib().paep_group_by_expert, "paep_group_by_expert", args, (idx, workspace), out)


def group_by_expert(idx: torch.Tensor, E: int, *, out: Optional[Grouping] = None,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> Grouping:
    """group_by_expert(idx[L,T,k]) -> counts[L,E], offsets[L,E+1], token lists, prefetch list."""
    with _on(stream):
        prep = prepare_group_by_expert(idx, E, out=out, workspace=workspace)
    return prep(stream)


def prepare_score(idx: torch.Tensor, ref_idx: torch.Tensor, E: int, *, k_row: Optional[torch.Tensor] = None,
                  out: Optional[torch.Tensor] = None) -> Prepared:
    """Check and marshal one score call; the returned object runs it."""
    if idx.dim() == 2:
        idx = idx.unsqueeze(0)
    if ref_idx.dim() == 2:
        ref_idx = ref_idx.unsqueeze(0)
    _need_device(idx, ref_idx)
    if idx.dtype != torch.int32 or ref_idx.dtype != torch.int32:
        raise TypeError("idx and ref_idx must be int32")
    L, T, k_pred = idx.shape
    if ref_idx.shape[0] != L or ref_idx.shape[1] != T:
        raise ValueError("idx and ref_idx must agree on [L, T]")
    k_ref = ref_idx.shape[2]
    if out is None:
        out = torch.empty((L, 4), dtype=torch.int64, device=idx.device)
    if k_row is None:
        return Prepared(lib().paep_score, "paep_score",
                        (_ptr(idx), k_pred, _ptr(ref_idx), k_ref, L, T, E, _ptr(out)), (idx, ref_idx), out)
    _need_device(k_row)
    if k_row.dtype != torch.int32 or k_row.numel() != L * T or not k_row.is_contiguous():
        raise TypeError("k_row must be contiguous int32 [L, T]")
    return Prepared(lib().paep_score_rows, "paep_score_rows",
                    (_ptr(idx), k_pred, _ptr(k_row), _ptr(ref_idx), k_ref, L, T, E, _ptr(out)),
                    (idx, ref_idx, k_row), out)


def score(idx: torch.Tensor, ref_idx: torch.Tensor, E: int, *, k_row: Optional[torch.Tensor] = None,
          out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """score(idx[L,T,k_pred], ref_idx[L,T,k_ref]) -> int64 [L,4]: n_exact, n_hit, n_cover, n_top1.
    With k_row[L,T] (int32) each row uses only its first k_row predicted ids."""
    with _on(stream):
        prep = prepare_score(idx, ref_idx, E, k_row=k_row, out=out)
    return prep(stream)


class Widened(NamedTuple):
    idx: torch.Tensor         # [L, T, k_pred] int32, -1 past each row's width
    k_row: torch.Tensor       # [L, T] int32
    n_wide: torch.Tensor      # [L] int32


def confidence_select(idx: torch.Tensor, probs: torch.Tensor, k_base: int, ratio: float, stream=None) -> Widened:
    """Keep k_base predictions on confident rows (probs[k_base-1] >= ratio * probs[k_base]), all of them elsewhere."""
    if idx.dim() == 2:
        idx, probs = idx.unsqueeze(0), probs.unsqueeze(0)
    _need_device(idx, probs)
    if idx.dtype != torch.int32 or probs.dtype != torch.float32 or idx.shape != probs.shape \
            or not idx.is_contiguous() or not probs.is_contiguous():
        raise TypeError("idx int32 and probs float32 must be contiguous and of one shape [L, T, k_pred]")
    L, T, k_pred = idx.shape
    with _on(stream):
        out = Widened(torch.empty_like(idx), torch.empty((L, T), dtype=torch.int32, device=idx.device),
                      torch.empty((L,), dtype=torch.int32, device=idx.device))
    st = lib().paep_confidence_select(_ptr(idx), _ptr(probs), L, T, k_pred, k_base, float(ratio), _ptr(out.idx),
                                      _ptr(out.k_row), _ptr(out.n_wide), _stream_ptr(stream))
    if st != 0:
        raise PaepError(st, "paep_confidence_select")
    return out


class ActivationProfile(NamedTuple):
    order: torch.Tensor       # [L, E] int32: experts by descending count, then -1
    n_active: torch.Tensor    # [L] int32
    entropy: torch.Tensor     # [L] float64: normalised Shannon entropy of the activation distribution


def activation_profile(counts: torch.Tensor, stream=None) -> ActivationProfile:
    """activation_profile(counts[L,E]) -> popularity-ordered expert list and entropy per layer."""
    if counts.dim() == 1:
        counts = counts.unsqueeze(0)
    _need_device(counts)
    if counts.dtype != torch.int32 or not counts.is_contiguous():
        raise TypeError("counts must be contiguous int32")
    L, E = counts.shape
    with _on(stream):
        out = ActivationProfile(torch.empty((L, E), dtype=torch.int32, device=counts.device),
                                torch.empty((L,), dtype=torch.int32, device=counts.device),
                                torch.empty((L,), dtype=torch.float64, device=counts.device))
    st = lib().paep_activation_profile(_ptr(counts), L, E, _ptr(out.order), _ptr(out.n_active), _ptr(out.entropy),
                                       _stream_ptr(stream))
    if st != 0:
        raise PaepError(st, "paep_activation_profile")
    return out


def fold_batchnorm(W1: torch.Tensor, b1: Optional[torch.Tensor], gamma: torch.Tensor, beta: torch.Tensor,
                   mean: torch.Tensor, var: torch.Tensor, eps: float = 1e-5, stream=None):
    """BatchNorm (inference form) folded into the first linear layer: returns (W1', b1') such that
    act(BN(W1 x + b1)) = act(W1' x + b1').  W1 [L, r, d] (or [r, d]), b1 [L, r] or None in the storage
    dtype; gamma, beta, mean, var [L, r] float32."""
    squeeze = W1.dim() == 2
    if squeeze:
        W1 = W1.unsqueeze(0)
    L, r, d = W1.shape
    stats = [t.reshape(L, r) for t in (gamma, beta, mean, var)]
    _need_device(W1, b1, *stats)
    if any(t.dtype != torch.float32 for t in stats):
        raise TypeError("gamma, beta, mean, var must be float32")
    dt = _storage_dtype(W1)
    if b1 is not None and (_storage_dtype(b1) != dt or b1.numel() != L * r):
        raise ValueError("b1 must be [L, r] in the storage dtype of W1")
    with _on(stream):
        W1o = torch.empty_like(W1)
        b1o = torch.empty((L, r), dtype=W1.dtype, device=W1.device)
    st = lib().paep_fold_batchnorm(_ptr(W1), _ptr(b1), *[_ptr(t) for t in stats], float(eps), L, r, d, dt,
                                   _ptr(W1o), _ptr(b1o), _stream_ptr(stream))
    if st != 0:
        raise PaepError(st, "paep_fold_batchnorm")
    return (W1o[0], b1o[0]) if squeeze else (W1o, b1o)


def probe_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """One launch of the streaming-read probe over all of `src` (device ceilings, not part of the method)."""
    _need_device(src, sink)
    st = lib().paep_probe_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                               sink.numel() * sink.element_size(), _stream_ptr(stream))
    if st != 0:
        raise PaepError(st, "paep_probe_read")


def probe_mfma(workgroups: int, iters: int, sink: torch.Tensor, stream=None) -> float:
    """One launch of the register-only matrix-instruction probe; returns the flops of the launch."""
    _need_device(sink)
    flops = ctypes.c_double(0.0)
    st = lib().paep_probe_mfma(workgroups, iters, _ptr(sink), sink.numel() * sink.element_size(),
                               _stream_ptr(stream), ctypes.byref(flops))
    if st != 0:
        raise PaepError(st, "paep_probe_mfma")
    return flops.value
