"""LKV-H at inference time (Sec. 3.3), fp64, CPU.

TEST INFRASTRUCTURE, NOT PRODUCT: only tests, the smoke check and the CPU leg
of the benchmark may use this module.

What is computed, in the paper's order:

* ``head_scores`` -- "Head Embeddings and Scoring": every KV head (l, h) owns
  an embedding e^{(l,h)} and one shared network maps it to a scalar
  s^{(l,h)} = MLP_head(e^{(l,h)}).  Table 5 fixes the network as
  128 -> 64 -> 1 with SiLU and 8,320 parameters, i.e. a hidden bias and no
  output bias (128*64 + 64 + 64).  An output bias is accepted anyway; it
  cannot change the ratios because ST_k is translation invariant.
* ``head_ratios`` -- "Global 1D Competition": the scores of all L*H heads,
  flattened, go through the Soft-TopK operator with k = R_agg = R L H and
  temperature 1; the result r sums to R L H and every r lies in (0, 1).
* ``head_budgets`` -- "Zero-Overhead Budgeting at Inference":
  b^{(l,h)} = floor(r^{(l,h)} t).

Reading where the paper is silent: the flattening order is layer-major
(index l * H + h); any fixed order gives the same ratios per head.

Pins: tests/test_oracle_lkv_h.py (parameter count of Table 5, hand-computed
tiny network, equal embeddings give r = R for every head, the antisymmetric
two-head closed form, sum / range / order properties, total budget bound).
"""
from __future__ import annotations

import numpy as np

from . import soft_topk as _st


def predictor_param_count(d_e: int, hidden: int, out_bias: bool) -> int:
    return d_e * hidden + hidden + hidden + (1 if out_bias else 0)


def head_scores(emb: np.ndarray, mlp: dict) -> np.ndarray:
    """emb [n_heads, d_e]; mlp: w1 [hidden, d_e], b1 [hidden], w2 [hidden], b2 scalar or None."""
    e = np.asarray(emb, dtype=np.float64)
    w1 = np.asarray(mlp["w1"], dtype=np.float64)
    b1 = np.asarray(mlp["b1"], dtype=np.float64)
    w2 = np.asarray(mlp["w2"], dtype=np.float64)
    z = e @ w1.T + b1                       # [n_heads, hidden]
    a = z / (1.0 + np.exp(-z))              # SiLU
    s = a @ w2
    if mlp.get("b2") is not None:
        s = s + float(mlp["b2"])
    return s


def head_ratios(s: np.ndarray, R: float) -> np.ndarray:
    s = np.asarray(s, dtype=np.float64).reshape(-1)
    return _st.soft_topk(s, R * s.size, tau=1.0)


def head_budgets(r: np.ndarray, t: int) -> np.ndarray:
    return np.floor(np.asarray(r, dtype=np.float64) * float(t)).astype(np.int64)
