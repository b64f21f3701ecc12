"""Workload shapes for the pre-attention expert predictor.

Each entry gives the number of MoE layers L (one predictor per layer, paper
section 4.2), hidden size d, predictor inner width r (the paper uses 2048,
section 1), expert count E and selected experts k (paper Table 2), the storage
dtype, and the token counts the workload is run at.  `k_over` is the
over-provisioned prediction width the paper evaluates (section 5.2:
10 / 12 / 3 for k = 6 / 8 / 2).

This module holds shapes only; it performs no arithmetic of the method.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    L: int
    d: int
    r: int
    E: int
    k: int
    dtype: str                      # "f32" or "bf16"
    decode_T: Tuple[int, ...] = ()
    prefill_T: Tuple[int, ...] = ()
    k_over: int = 0                 # over-provisioned k' (0: not evaluated)
    rms_scale: bool = True          # rows of x divided by their RMS
    n_outlier: int = 0              # 0 -> max(4, d // 512)
    zipf_bias: bool = False         # b2 carries a Zipf(s=1.2) expert skew
    near_tie_frac: float = 0.0      # fraction of rows with a tiny k/(k+1) gap
    exact_tie_rows: int = 0         # rows per layer whose k/(k+1) logits tie exactly

    @property
    def outliers(self) -> int:
        return self.n_outlier if self.n_outlier else max(4, self.d // 512)


WORKLOADS = {
    w.name: w
    for w in (
        Workload("toy", 0, L=1, d=256, r=64, E=16, k=2, dtype="f32",
                 prefill_T=(512,), k_over=3, rms_scale=False, n_outlier=4),
        Workload("deepseek_v2_lite", 1, L=26, d=2048, r=2048, E=64, k=6, dtype="bf16",
                 decode_T=(1, 8, 64), prefill_T=(4096,), k_over=10),
        Workload("qwen3_30b_a3b", 2, L=48, d=2048, r=2048, E=128, k=8, dtype="bf16",
                 decode_T=(1, 16, 64), prefill_T=(8192,), k_over=12),
        Workload("phi_mini_moe", 3, L=32, d=4096, r=1024, E=16, k=2, dtype="bf16",
                 decode_T=(1, 32), prefill_T=(8192,), k_over=3, zipf_bias=True),
        Workload("stress", 4, L=48, d=2048, r=4096, E=256, k=8, dtype="bf16",
                 prefill_T=(32768,), k_over=12, near_tie_frac=0.01, exact_tie_rows=16),
    )
}


def get(name: str) -> Workload:
    try:
        return WORKLOADS[name]
    except KeyError:
        raise KeyError(f"unknown workload {name!r}; have {sorted(WORKLOADS)}") from None
