"""Plain fp64 CPU oracle of LKV's inference-time eviction path.

TEST INFRASTRUCTURE, NOT PRODUCT.  This module is the slow, obviously-correct
statement of what the hot path computes.  It is written from the paper's
definitions with numpy only; it shares no code, table or helper with the HIP
kernels and is never reached from the product path.

What is computed, and where the paper defines it:

* ``score``   -- LKV-T intrinsic token score, Sec. 3.4 ("Head-Specific
  Intrinsic Scoring"): ``u_i = MLP_token([k_i ; v_i])``.  Table 5 fixes the
  paper's network as 256 -> 128 -> 1 with SiLU and 33,024 parameters, which
  means a hidden bias and no output bias.  The benchmark workloads also use a
  single linear layer ``w.x + b`` and a 256 -> 64 -> 1 GELU network.
* ``integer_budgets`` / ``total_budget`` -- Sec. 3.3 ("Zero-Overhead Budgeting
  at Inference"): ``b = floor(r * t)``; Sec. 3.1: ``B_total = floor(R L H t)``.
* ``select``  -- Sec. 3.4, inference: ``m = TopK(u, b)``, a hard top-k on the
  raw scores that keeps exactly ``b`` tokens.
* ``compact`` -- Sec. 4.5: the kept K/V rows are flattened into one padding-free
  buffer with per-head segment offsets.
* ``decode_attn`` -- Eq. 1 restricted to the kept tokens; the mask is per KV
  head, so every query head of a GQA group sees the same segment (Sec. 3.1).
* ``masked_attention_full`` -- App. B.2: ``p_i = e^{s_i} m_i / sum_j e^{s_j} m_j``
  over the *uncompacted* cache.  With a 0/1 mask this must equal
  ``decode_attn`` over the compacted cache; it is kept here as a second,
  independently written route to the same numbers.

Readings where the paper is silent (they are also listed in the design notes):

* concatenation order is key first, then value, as the paper writes [k; v];
* GELU is the exact erf form 0.5 z (1 + erf(z / sqrt 2));
* ties in TopK go to the lower token index; a NaN score ranks as -inf; scores
  are ordered by the IEEE-754 total order of their fp32 bit patterns, so
  -0.0 ranks below +0.0;
* query head ``hq`` reads KV head ``hq // g`` (contiguous groups);
* a head with budget 0 is legal: its decode output is all zero, its
  log-sum-exp is -inf.

All floating-point arithmetic is fp64 on inputs converted exactly (every bf16
value is an fp64 value).  A score is rounded once, to fp32, at the end, because
the top-k is defined on fp32 scores.

Pin status: every function below is pinned by tests/test_oracle_*.py against
closed forms, brute force, library routines used as independent checks, and
the paper's own arithmetic (parameter counts, storage sizes).  Agreement with
the paper's *task quality* numbers is "parity unpinned": that needs datasets
and trained weights that are not available.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

# --------------------------------------------------------------------------
# exact input conversion
# --------------------------------------------------------------------------


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp64, exactly.

    A bf16 number is the upper half of an fp32 number, so placing the 16 bits
    in the high half of a 32-bit word and widening is lossless.
    """
    bits = np.ascontiguousarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError("bf16 bit patterns must be uint16")
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# Sec. 3.4 / Table 5: the scorer
# --------------------------------------------------------------------------


def scorer_param_count(d_in: int, hidden: int) -> int:
    """Parameters of one LKV-T / LKV-H predictor ``d_in -> hidden -> 1``.

    Table 5: a weight matrix, a hidden bias and an output weight vector; no
    output bias.  (256,128) must give 33,024 and (128,64) must give 8,320.
    """
    return d_in * hidden + hidden + hidden


def silu(z: np.ndarray) -> np.ndarray:
    """SiLU, z * sigmoid(z) (Table 5 caption: all MLPs use SiLU)."""
    z = np.asarray(z, dtype=np.float64)
    # sigmoid written so that neither branch overflows
    pos = z >= 0
    ez = np.exp(np.where(pos, -z, z))
    sig = np.where(pos, 1.0 / (1.0 + ez), ez / (1.0 + ez))
    return z * sig


def gelu_erf(z: np.ndarray) -> np.ndarray:
    """Exact GELU, 0.5 z (1 + erf(z / sqrt 2))."""
    z = np.asarray(z, dtype=np.float64)
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


_ACTS = {"silu": silu, "gelu": gelu_erf}


def score(K: np.ndarray, V: np.ndarray, scorer: dict) -> np.ndarray:
    """Token scores for one sequence (Sec. 3.4).

    K, V   : fp64 [L, H, T, d]   (exactly converted cache contents)
    scorer : dict with
        kind   'linear' or 'mlp'
        w1     linear: fp64 [L, Hs, 2d]; mlp: fp64 [L, Hs, hidden, 2d]
               (Hs is H for one scorer per head as in the paper, or 1 for one
               scorer per layer shared by its heads)
        b1     linear: fp64 [L, Hs]  (the scalar bias); mlp: fp64 [L, Hs, hidden]
        w2     mlp: fp64 [L, Hs, hidden]
        b2     mlp: fp64 [L, Hs] or None (the paper has no output bias)
        act    'silu' or 'gelu' (mlp only)
    returns fp32 [L, H, T]: the fp64 result rounded once to fp32.
    """
    L, H, T, d = K.shape
    assert V.shape == K.shape
    w1 = np.asarray(scorer["w1"], dtype=np.float64)
    Hs = w1.shape[1]
    assert Hs in (1, H)
    u = np.empty((L, H, T), dtype=np.float64)
    for l in range(L):
        for h in range(H):
            hs = h if Hs == H else 0
            x = np.concatenate([K[l, h], V[l, h]], axis=1)  # [T, 2d], key first
            if scorer["kind"] == "linear":
                u[l, h] = x @ w1[l, hs] + float(scorer["b1"][l][hs])
            elif scorer["kind"] == "mlp":
                act = _ACTS[scorer["act"]]
                pre = x @ w1[l, hs].T + np.asarray(scorer["b1"], dtype=np.float64)[l, hs]
                hid = act(pre)
                out = hid @ np.asarray(scorer["w2"], dtype=np.float64)[l, hs]
                if scorer.get("b2") is not None:
                    out = out + float(scorer["b2"][l][hs])
                u[l, h] = out
            else:
                raise ValueError(scorer["kind"])
    return u.astype(np.float32)


# --------------------------------------------------------------------------
# Sec. 3.1 / 3.3: budgets
# --------------------------------------------------------------------------


def total_budget(R: float, L: int, H: int, t: int) -> int:
    """B_total = floor(R * L * H * t)  (Sec. 3.1)."""
    return int(math.floor(R * L * H * t))


def integer_budgets(r: np.ndarray, t: int) -> np.ndarray:
    """b = floor(r * t) per head (Sec. 3.3, applied at inference only)."""
    return np.floor(np.asarray(r, dtype=np.float64) * t).astype(np.int64)


def segment_offsets(budgets: np.ndarray) -> np.ndarray:
    """Exclusive prefix sum of the budgets in (sequence, layer, head) order.

    offsets[s] is the first packed row of segment s; offsets[-1] is the number
    of kept rows.  No padding between segments (Sec. 4.5).
    """
    b = np.asarray(budgets, dtype=np.int64).reshape(-1)
    off = np.zeros(b.size + 1, dtype=np.int64)
    np.cumsum(b, out=off[1:])
    return off


def packed_cache_bytes(budgets: np.ndarray, d: int, bytes_per_el: int = 2) -> int:
    """Bytes of the padding-free K and V buffers: sum(b) * 2 * d * bytes."""
    return int(np.asarray(budgets, dtype=np.int64).sum()) * 2 * d * bytes_per_el


# --------------------------------------------------------------------------
# Sec. 3.4 (inference): hard top-k
# --------------------------------------------------------------------------


def order_key(u: np.ndarray) -> np.ndarray:
    """fp32 scores -> uint32 keys whose unsigned order is the score order.

    NaN is first replaced by -inf.  Then the IEEE-754 bit pattern is mapped so
    that unsigned comparison of keys equals the total order of the floats:
    non-negative floats get their sign bit set, negative floats are inverted.
    """
    u = np.ascontiguousarray(u, dtype=np.float32)
    u = np.where(np.isnan(u), np.float32(-np.inf), u).astype(np.float32)
    bits = u.view(np.uint32)
    neg = (bits >> np.uint32(31)).astype(bool)
    return np.where(neg, ~bits, bits | np.uint32(0x80000000)).astype(np.uint32)


def select(u: np.ndarray, b: int) -> np.ndarray:
    """TopK(u, b) for one head: the kept token indices, ascending (int32).

    The definition, written out: sort all tokens by (score descending, index
    ascending), keep the first b, report them in ascending index order.
    """
    u = np.asarray(u, dtype=np.float32).reshape(-1)
    T = u.size
    if not 0 <= b <= T:
        raise ValueError("budget outside [0, T]")
    key = order_key(u).astype(np.int64)
    # a stable sort on the negated key leaves equal keys in index order
    ranked = np.argsort(-key, kind="stable")
    return np.sort(ranked[:b]).astype(np.int32)


def select_all(u: np.ndarray, budgets: np.ndarray):
    """Top-k for every head of one sequence.

    u [L, H, T] fp32, budgets [L, H] -> (idx int32 [sum b], offsets int64 [L*H+1])
    with segments in (layer, head) order.
    """
    L, H, T = u.shape
    budgets = np.asarray(budgets).reshape(L, H)
    off = segment_offsets(budgets)
    idx = np.empty(int(off[-1]), dtype=np.int32)
    for l in range(L):
        for h in range(H):
            s = l * H + h
            idx[off[s]:off[s + 1]] = select(u[l, h], int(budgets[l, h]))
    return idx, off


# --------------------------------------------------------------------------
# Sec. 4.5: padding-free compaction
# --------------------------------------------------------------------------


def compact(K: np.ndarray, V: np.ndarray, idx: np.ndarray, offsets: np.ndarray):
    """Gather the kept rows of every head into flat [sum b, d] buffers.

    K, V may be any dtype (bit patterns are copied, not interpreted);
    shape [L, H, T, d].  Segment s = l*H + h occupies rows
    offsets[s]:offsets[s+1], in ascending original token order.
    """
    L, H, T, d = K.shape
    n = int(offsets[-1])
    Kp = np.empty((n, d), dtype=K.dtype)
    Vp = np.empty((n, d), dtype=V.dtype)
    for l in range(L):
        for h in range(H):
            s = l * H + h
            rows = idx[offsets[s]:offsets[s + 1]]
            Kp[offsets[s]:offsets[s + 1]] = K[l, h, rows]
            Vp[offsets[s]:offsets[s + 1]] = V[l, h, rows]
    return Kp, Vp


# --------------------------------------------------------------------------
# Eq. 1 on the compacted cache; App. B.2 on the full cache
# --------------------------------------------------------------------------


def decode_attn(q: np.ndarray, Kp: np.ndarray, Vp: np.ndarray, offsets: np.ndarray,
                H: int, scale: float):
    """One decode step over the ragged packed cache of one sequence (Eq. 1).

    q       fp64 [L, Hq, d]
    Kp, Vp  fp64 [sum b, d]
    offsets [L*H + 1]
    returns (o fp64 [L, Hq, d], lse fp64 [L, Hq]); lse = log sum_j exp(s_j).
    """
    L, Hq, d = q.shape
    g = Hq // H
    assert g * H == Hq
    o = np.zeros((L, Hq, d), dtype=np.float64)
    lse = np.full((L, Hq), -np.inf, dtype=np.float64)
    for l in range(L):
        for hq in range(Hq):
            h = hq // g
            lo, hi = int(offsets[l * H + h]), int(offsets[l * H + h + 1])
            if hi == lo:
                continue
            s = (Kp[lo:hi] @ q[l, hq]) * scale
            m = s.max()
            e = np.exp(s - m)
            z = e.sum()
            o[l, hq] = (e / z) @ Vp[lo:hi]
            lse[l, hq] = m + math.log(z)
    return o, lse


def masked_attention_full(q: np.ndarray, K: np.ndarray, V: np.ndarray,
                          mask: np.ndarray, scale: float):
    """App. B.2: raw softmax over the whole cache, multiply by the mask,
    renormalise.  q [d], K, V [T, d], mask [T] in [0, 1].  Returns o [d]."""
    s = (K @ q) * scale
    p_raw = np.exp(s - s.max())
    p_raw = p_raw / p_raw.sum()
    p_tilde = p_raw * mask
    p = p_tilde / p_tilde.sum()
    return p @ V


def mask_from_indices(idx: np.ndarray, T: int) -> np.ndarray:
    """Retention mask m in {0,1}^T of one head from its kept indices."""
    m = np.zeros(T, dtype=np.float64)
    m[np.asarray(idx, dtype=np.int64)] = 1.0
    return m
