"""Seeded synthetic inputs for the LKV eviction hot path.

This module only *draws inputs*: cache contents, scorer weights, head budgets,
query vectors, sequence lengths.  It contains none of the method's arithmetic
(no scoring, no selection, no attention) and is the one piece of code that the
CPU oracle's tests and the HIP path's tests both use, so that both sides see
the same bytes.

The five workload shapes follow the benchmark configurations of this build;
they take the *shapes* of the paper's evaluation (Llama-3.1-8B: 32 layers x 8
KV heads, d = 128, App. C.1; contexts of 4k-32k and 200k+, Sec. 4.3 / 4.5;
retention 0.15 / 0.10, Sec. 4.2) and stand in for LongBench / RULER prompts and
for trained LKV weights, none of which are available.  No benchmark item is
reproduced here.

Recipe
------
* K, V, q: i.i.d. N(0,1), rounded to bf16 (round-to-nearest-even).
  - ``outliers='x10'``: per (layer, head) 4 of the 256 [k;v] feature channels
    are multiplied by 10 before rounding.
  - ``outliers='student_t'``: per (layer, head) round(0.02*256) = 5 feature
    channels get additive Student-t(3) noise per token before rounding.
  The channel set is drawn per (layer, head) and shared by all sequences.
* Scorer weights ~ N(0, 0.02^2) (0.02 is the standard deviation).  The first
  layer (or the linear weight vector) is rounded to bf16; biases and the output
  vector stay fp32.  One scorer per layer, shared by its heads, unless
  ``per_head`` is set (the paper's one-MLP-per-head arrangement, Sec. 3.4).
* Budgets: B_total = floor(R L H T); p ~ Dirichlet(alpha) over the flattened
  L*H heads (the paper's LKV-H competes over the flattened head vector, Sec.
  3.3); every head gets ``b_min`` and floor(p_h * rest) of what remains, with
  water-filling when a head would exceed T.  Hence b_min <= b <= T and
  sum(b) <= B_total.
* Training-time attention (``draw_training_attention``): q, k, v, dO i.i.d. N(0,1) in bf16 (one
  layer of one sequence; the paper trains on 2k-16k token samples of its own corpus, App. C.2,
  which is not available); soft mask m = x^4 with x ~ U(0,1) (mean 0.2, most weights small, as
  late in the annealing of Sec. 3.4), 10 % of the weights set to exactly 0 and 5 % to exactly 1,
  the first key of every head kept above 0.25 so that every causal prefix carries weight.
* Observation-window queries (``draw_window_queries``): i.i.d. N(0,1) in bf16 like the decode
  queries; on top, per (layer, query head) four "needle" positions of the prefix are drawn and each
  window row, with probability 1/2, gets half of one needle's key row added before rounding (a logit
  about 5.7 above the rest), so that the votes have the few-heavy-tokens shape attention over a
  prompt has and the pooling has peaks to spread.
* Sub-streams are keyed by (seed, config id, tensor tag, sequence, layer) so
  that any single layer can be regenerated on its own.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Tuple, Union

import numpy as np

D_HEAD = 128

_TAGS = {"kv": 1, "q": 2, "scorer": 3, "budget": 4, "seqlen": 5, "chan": 6, "noise": 7, "headpred": 8, "train": 9, "win": 10}


@dataclasses.dataclass(frozen=True)
class Workload:
    cid: int
    name: str
    n_seq: int
    L: int
    H: int
    Hq: int
    T: Union[int, Tuple[int, int]]      # fixed length, or (lo, hi) inclusive for a uniform draw
    scorer: str                         # 'linear' or 'mlp'
    hidden: int
    act: str                            # 'gelu' or 'silu' (mlp only)
    R: float
    alpha: float
    b_min: int
    outliers: Optional[str] = None      # None, 'x10', 'student_t'
    shared_budgets: bool = False        # one budget table for all sequences
    per_head: bool = False
    out_bias: bool = True               # False: the paper's arrangement (Table 5: no output bias)
    d: int = D_HEAD

    @property
    def g(self) -> int:
        return self.Hq // self.H


CONFIGS = (
    Workload(0, "cfg0-L1-H8-T4096-linear", 1, 1, 8, 32, 4096, "linear", 0, "gelu", 0.15, 1.0, 32),
    Workload(1, "cfg1-L32-H8-T32768-linear", 1, 32, 8, 32, 32768, "linear", 0, "gelu", 0.15, 0.5, 64,
             outliers="x10"),
    Workload(2, "cfg2-L32-H8-T131072-mlp64gelu", 1, 32, 8, 32, 131072, "mlp", 64, "gelu", 0.10, 0.3, 128),
    Workload(3, "cfg3-16seq-T4096..16384-linear", 16, 32, 8, 32, (4096, 16384), "linear", 0, "gelu",
             0.15, 0.5, 32),
    Workload(4, "cfg4-8seq-L28-H4-g7-T65536-mlp64gelu", 8, 28, 4, 28, 65536, "mlp", 64, "gelu", 0.05, 0.1, 32,
             outliers="student_t", shared_budgets=True),
    # not one of the five benchmark configurations: the scorer exactly as the paper builds it
    # (Sec. 3.4 / Table 5: one 256 -> 128 -> 1 SiLU network per (layer, head), no output bias)
    # on the Llama-3.1-8B cache shape of its App. C.1
    Workload(5, "paper-L32-H8-T32768-mlp128silu-per-head", 1, 32, 8, 32, 32768, "mlp", 128, "silu", 0.15, 0.5, 64,
             per_head=True, out_bias=False),
    # the same scorer on the other model shape of App. C.1 (36 layers x 8 KV heads: 288 scorers, Table 5)
    Workload(6, "paper-L36-H8-T32768-mlp128silu-per-head", 1, 36, 8, 32, 32768, "mlp", 128, "silu", 0.15, 0.5, 64,
             per_head=True, out_bias=False),
)


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (for small test cases)."""
    return dataclasses.replace(w, **kw)


def _rng(seed: int, cid: int, tag: str, seq: int = 0, layer: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(cid), _TAGS[tag], int(seq), int(layer)])


# --------------------------------------------------------------------------
# bf16 storage helpers (storage format only)
# --------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = np.isnan(x)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    rounded = np.where(nan, np.uint32(0x7FC0), rounded)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# host-side draws (small tensors, and everything that is small at any size)
# --------------------------------------------------------------------------


def seq_lengths(w: Workload, seed: int = 0) -> np.ndarray:
    if isinstance(w.T, int):
        return np.full(w.n_seq, w.T, dtype=np.int64)
    lo, hi = w.T
    return _rng(seed, w.cid, "seqlen").integers(lo, hi + 1, size=w.n_seq).astype(np.int64)


def outlier_channels(w: Workload, seed: int = 0) -> Optional[np.ndarray]:
    """[L, H, n_ch] indices into the 256-wide [k;v] feature vector, or None."""
    if w.outliers is None:
        return None
    n_ch = 4 if w.outliers == "x10" else int(round(0.02 * 2 * w.d))
    rng = _rng(seed, w.cid, "chan")
    out = np.empty((w.L, w.H, n_ch), dtype=np.int64)
    for l in range(w.L):
        for h in range(w.H):
            out[l, h] = np.sort(rng.choice(2 * w.d, size=n_ch, replace=False))
    return out


def draw_budgets(w: Workload, T: int, seq: int = 0, seed: int = 0) -> np.ndarray:
    """Integer per-head budgets [L, H] for one sequence of length T."""
    if w.shared_budgets:
        seq = 0
    rng = _rng(seed, w.cid, "budget", seq)
    n = w.L * w.H
    B_total = int(math.floor(w.R * n * T))
    b_min = min(w.b_min, T)
    rest = B_total - n * b_min
    if rest < 0:
        raise ValueError("b_min does not fit the total budget")
    p = rng.dirichlet(np.full(n, w.alpha, dtype=np.float64))
    extra = np.zeros(n, dtype=np.int64)
    free = np.ones(n, dtype=bool)
    cap = T - b_min
    while True:
        psum = p[free].sum()
        if psum <= 0 or rest <= 0:
            break
        share = np.floor(p * (rest / psum)).astype(np.int64)
        over = free & (share > cap)
        if not over.any():
            extra[free] = share[free]
            break
        extra[over] = cap
        free &= ~over
        rest -= int(over.sum()) * cap
    b = (b_min + extra).reshape(w.L, w.H)
    assert b.min() >= b_min and b.max() <= T and int(b.sum()) <= B_total
    return b.astype(np.int32)


def draw_scorer(w: Workload, seed: int = 0) -> dict:
    """Scorer parameters.

    linear: w1 uint16(bf16) [L, Hs, 2d], b1 fp32 [L, Hs]
    mlp   : w1 uint16(bf16) [L, Hs, hidden, 2d] (one row per hidden unit),
            b1 fp32 [L, Hs, hidden], w2 fp32 [L, Hs, hidden], b2 fp32 [L, Hs] or None
    """
    rng = _rng(seed, w.cid, "scorer")
    Hs = w.H if w.per_head else 1
    std = 0.02
    if w.scorer == "linear":
        w1 = rng.normal(0.0, std, size=(w.L, Hs, 2 * w.d)).astype(np.float32)
        b1 = rng.normal(0.0, std, size=(w.L, Hs)).astype(np.float32)
        return {"kind": "linear", "act": w.act, "hidden": 0, "per_head": w.per_head,
                "w1": f32_to_bf16_bits(w1), "b1": b1, "w2": None, "b2": None}
    w1 = rng.normal(0.0, std, size=(w.L, Hs, w.hidden, 2 * w.d)).astype(np.float32)
    b1 = rng.normal(0.0, std, size=(w.L, Hs, w.hidden)).astype(np.float32)
    w2 = rng.normal(0.0, std, size=(w.L, Hs, w.hidden)).astype(np.float32)
    b2 = rng.normal(0.0, std, size=(w.L, Hs)).astype(np.float32) if w.out_bias else None
    return {"kind": "mlp", "act": w.act, "hidden": w.hidden, "per_head": w.per_head,
            "w1": f32_to_bf16_bits(w1), "b1": b1, "w2": w2, "b2": b2}


def draw_head_predictor(w: Workload, seed: int = 0, d_e: int = 128, hidden: int = 64,
                        out_bias: bool = False, spread: float = 0.5):
    """LKV-H inputs: head embeddings fp32 [L * H, d_e] and the shared predictor
    (w1 fp32 [hidden, d_e], b1 fp32 [hidden], w2 fp32 [hidden], b2 float or None).

    No trained embeddings exist here, so the draw is shaped to give what trained ones give in
    the paper's figures: head scores a few units apart, so ratios from a few percent to near one.
    """
    rng = _rng(seed, w.cid, "headpred")
    n = w.L * w.H
    emb = rng.standard_normal(size=(n, d_e)).astype(np.float32)
    w1 = (rng.standard_normal(size=(hidden, d_e)) / np.sqrt(d_e)).astype(np.float32)
    b1 = rng.normal(0.0, 0.1, size=hidden).astype(np.float32)
    w2 = (rng.standard_normal(size=hidden) * (spread * 4.0 / np.sqrt(hidden))).astype(np.float32)
    b2 = float(np.float32(rng.normal(0.0, 0.1))) if out_bias else None
    return emb, {"w1": w1, "b1": b1, "w2": w2, "b2": b2, "d_e": d_e, "hidden": hidden}


def draw_kv_layer(w: Workload, T: int, seq: int, layer: int, seed: int = 0,
                  channels: Optional[np.ndarray] = None):
    """K and V of one layer on the host: uint16(bf16) [H, T, d] each."""
    rng = _rng(seed, w.cid, "kv", seq, layer)
    x = rng.standard_normal(size=(w.H, T, 2 * w.d), dtype=np.float32)
    if w.outliers is not None:
        if channels is None:
            channels = outlier_channels(w, seed)
        for h in range(w.H):
            ch = channels[layer, h]
            if w.outliers == "x10":
                x[h][:, ch] *= np.float32(10.0)
            else:
                nrng = _rng(seed, w.cid, "noise", seq, layer * w.H + h)
                x[h][:, ch] += nrng.standard_t(3.0, size=(T, ch.size)).astype(np.float32)
    bits = f32_to_bf16_bits(x)
    return np.ascontiguousarray(bits[:, :, :w.d]), np.ascontiguousarray(bits[:, :, w.d:])


def draw_kv(w: Workload, T: int, seq: int = 0, seed: int = 0):
    """K and V of one sequence on the host: uint16(bf16) [L, H, T, d] each."""
    ch = outlier_channels(w, seed)
    K = np.empty((w.L, w.H, T, w.d), dtype=np.uint16)
    V = np.empty_like(K)
    for l in range(w.L):
        K[l], V[l] = draw_kv_layer(w, T, seq, l, seed, ch)
    return K, V


def draw_q(w: Workload, seq: int = 0, seed: int = 0) -> np.ndarray:
    """Decode-step query vectors of one sequence: uint16(bf16) [L, Hq, d]."""
    rng = _rng(seed, w.cid, "q", seq)
    return f32_to_bf16_bits(rng.standard_normal(size=(w.L, w.Hq, w.d), dtype=np.float32))


def draw_window_queries(w: Workload, K: np.ndarray, window: int, seq: int = 0, seed: int = 0) -> np.ndarray:
    """Queries of the last `window` prompt positions of one sequence: uint16(bf16) [L, Hq, window, d].
    K is the sequence's key cache as bf16 bit patterns [L, H, T, d] (the needles are rows of it)."""
    L, H, T, d = K.shape
    G = w.Hq // H
    rng = _rng(seed, w.cid, "win", seq, window)
    q = rng.standard_normal(size=(L, w.Hq, window, d), dtype=np.float32)
    prefix = T - window
    if prefix > 0:
        needles = rng.integers(0, prefix, size=(L, w.Hq, 4))
        which = rng.integers(0, 4, size=(L, w.Hq, window))
        planted = rng.uniform(size=(L, w.Hq, window)) < 0.5
        for l in range(L):
            for hq in range(w.Hq):
                rows = bf16_bits_to_f32(K[l, hq // G, needles[l, hq, which[l, hq]]])     # [window, d]
                q[l, hq] += np.float32(0.5) * rows * planted[l, hq][:, None]
    return f32_to_bf16_bits(q)


# --------------------------------------------------------------------------
# device-side draws for the full-size workloads (torch is plumbing here)
# --------------------------------------------------------------------------


def draw_training_attention(Hq: int, H: int, T: int, seed: int = 0, d: int = D_HEAD):
    """Inputs of one layer of training-time attention: bf16 bit patterns q, dO [Hq, T, d],
    k, v [H, T, d] and the fp32 soft mask m [H, T] (see the recipe above)."""
    rng = _rng(seed, 100, "train", Hq * 1000 + H, T)
    q = f32_to_bf16_bits(rng.standard_normal((Hq, T, d), dtype=np.float32))
    k = f32_to_bf16_bits(rng.standard_normal((H, T, d), dtype=np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((H, T, d), dtype=np.float32))
    d_o = f32_to_bf16_bits(rng.standard_normal((Hq, T, d), dtype=np.float32))
    x = rng.uniform(size=(H, T)).astype(np.float32)
    m = (x * x) * (x * x)
    pick = rng.uniform(size=(H, T))
    m[pick < 0.10] = 0.0
    m[pick > 0.95] = 1.0
    m[:, 0] = np.maximum(m[:, 0], np.float32(0.25))
    return q, k, v, m.astype(np.float32), d_o


def device_kv(w: Workload, T: int, seq: int, device, seed: int = 0):
    """K and V of one sequence drawn on the GPU: torch bf16 [L, H, T, d] each.

    Same distribution as ``draw_kv`` but a different random stream (the GPU's
    generator); the oracle is fed by copying slices of these tensors back to
    the host, so both sides always see identical bytes.
    """
    import torch

    gen = torch.Generator(device=device)
    K = torch.empty((w.L, w.H, T, w.d), dtype=torch.bfloat16, device=device)
    V = torch.empty_like(K)
    channels = outlier_channels(w, seed)
    for l in range(w.L):
        gen.manual_seed(int(_rng(seed, w.cid, "kv", seq, l).integers(0, 2**62)))
        x = torch.randn((w.H, T, 2 * w.d), dtype=torch.float32, device=device, generator=gen)
        if channels is not None:
            for h in range(w.H):
                ch = torch.as_tensor(channels[l, h], device=device)
                if w.outliers == "x10":
                    x[h, :, ch] *= 10.0
                else:
                    z = torch.randn((4, T, ch.numel()), dtype=torch.float32, device=device, generator=gen)
                    chi = (z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0
                    x[h, :, ch] += z[0] / torch.sqrt(chi)
        K[l] = x[:, :, :w.d].to(torch.bfloat16)
        V[l] = x[:, :, w.d:].to(torch.bfloat16)
        del x
    return K, V
