"""Plain fp64 CPU oracle of the observation-window token scorer.

TEST INFRASTRUCTURE, NOT PRODUCT.  Written with numpy only; it shares no code with the HIP
kernels and is never reached from the product path.

Where it comes from.  The ablation of Sec. 4.4 feeds the head-wise budgets of LKV-H to token
selection policies other than LKV-T; the first of them scores a token by the attention it
receives from a local observation window at the end of the prompt (Sec. 2 describes it so, and
the complexity table of Sec. 4.5 lists it as O(W T), W the window size).  The paper names the
policy and refers to its publication for the rule; it prints no formula, no window size and no
smoothing width of its own, so what follows is this build's reading of that published rule,
stated here in full, and every parameter is an argument.  There is no value in the paper to pin
it to: parity unpinned against the paper, pinned against library routines and identities
(tests/test_oracle_window_score.py).

What is computed, for one layer of one sequence with T cached tokens:

    window      the last W positions, T - W ... T - 1; query row i of the window stands at
                position T - W + i and, being causal, sees keys 0 ... T - W + i
    a[hq, i, :] = softmax over those keys of  scale * q[hq, i] . k[h, j],   h = hq // (Hq // H)
    vote[h, j]  = (1 / G) sum over the G query heads of the group, sum over i, of a[hq, i, j]
                  for the prefix tokens j < T - W      (group mean: one score per KV head, since
                  the heads of a GQA group share the cache entry they would evict)
    pooled      a 1-D pooling of vote[h, :] along j, width `pool_width` (odd), stride 1, centred:
                  'max'  the largest vote inside the part of [j - c, j + c] that lies in the prefix
                  'avg'  the sum over that part divided by pool_width (positions outside the
                         prefix count as zeros, the library default for padded average pooling)
                  with c = (pool_width - 1) / 2; width 1 leaves the votes as they are
    scores[h, j] = pooled[h, j] for j < T - W,  +inf for the window tokens themselves

A hard top-k over these scores with a budget b >= W therefore keeps the window and the b - W
prefix tokens with the largest pooled votes, which is the published selection rule; with b < W
the tie rule of the top-k (lower index first) decides among the window tokens.
"""
from __future__ import annotations

import numpy as np


def window_attention(Qw: np.ndarray, K: np.ndarray, scale: float) -> np.ndarray:
    """Attention weights of the window queries: a [Hq, W, T] (zero where a key lies after the query).

    Qw [Hq, W, d] are the queries of the last W positions, K [H, T, d] all keys."""
    Qw = np.asarray(Qw, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    Hq, W, _ = Qw.shape
    H, T, _ = K.shape
    if Hq % H != 0:
        raise ValueError("the number of query heads must be a multiple of the number of KV heads")
    if not 1 <= W <= T:
        raise ValueError("the window must hold between 1 and T tokens")
    G = Hq // H
    a = np.zeros((Hq, W, T))
    for hq in range(Hq):
        k = K[hq // G]
        for i in range(W):
            last = T - W + i                      # position of this query = last key it sees
            s = scale * (k[:last + 1] @ Qw[hq, i])
            e = np.exp(s - s.max())
            a[hq, i, :last + 1] = e / e.sum()
    return a


def window_log_normalisers(Qw: np.ndarray, K: np.ndarray, scale: float) -> np.ndarray:
    """lse [Hq, W]: natural logarithm of the softmax denominators of the window rows, i.e. what a causal
    attention kernel returns next to its output for these queries."""
    Qw = np.asarray(Qw, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    Hq, W, _ = Qw.shape
    H, T, _ = K.shape
    G = Hq // H
    lse = np.empty((Hq, W))
    for hq in range(Hq):
        for i in range(W):
            s = scale * (K[hq // G, :T - W + i + 1] @ Qw[hq, i])
            lse[hq, i] = s.max() + np.log(np.exp(s - s.max()).sum())
    return lse


def window_votes(Qw: np.ndarray, K: np.ndarray, scale: float) -> np.ndarray:
    """vote [H, T - W]: attention mass each prefix token receives from the window, summed over the
    window rows and averaged over the query heads of the group."""
    a = window_attention(Qw, K, scale)
    Hq, W, T = a.shape
    H = K.shape[0]
    G = Hq // H
    vote = np.zeros((H, T - W))
    for hq in range(Hq):
        for i in range(W):
            vote[hq // G] += a[hq, i, :T - W]
    return vote / G


def pool1d(x: np.ndarray, width: int, kind: str) -> np.ndarray:
    """Centred 1-D pooling of each row of x [H, n], stride 1, same length out as in."""
    if width < 1 or width % 2 == 0:
        raise ValueError("the pooling width must be odd and positive")
    if kind not in ("max", "avg"):
        raise ValueError("kind is 'max' or 'avg'")
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[-1]
    c = (width - 1) // 2
    out = np.empty_like(x)
    for j in range(n):
        part = x[..., max(0, j - c):min(n, j + c + 1)]
        out[..., j] = part.max(axis=-1) if kind == "max" else part.sum(axis=-1) / width
    return out


def window_scores(Qw: np.ndarray, K: np.ndarray, scale: float, pool_width: int = 1, kind: str = "max") -> np.ndarray:
    """scores [H, T]: pooled votes on the prefix, +inf on the window tokens."""
    W = np.asarray(Qw).shape[1]
    H, T, _ = np.asarray(K).shape
    scores = np.full((H, T), np.inf)
    if T > W:
        scores[:, :T - W] = pool1d(window_votes(Qw, K, scale), pool_width, kind)
    return scores
