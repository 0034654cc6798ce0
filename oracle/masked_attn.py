"""Plain fp64 CPU oracle of the training-time attention with a multiplicative soft mask.

TEST INFRASTRUCTURE, NOT PRODUCT.  Written from App. B of the paper with numpy only; it
shares no code with the HIP kernels and is never reached from the product path.

What is computed (App. B.2, "Proposed Multiplicative Formulation"), for every query i of a
causal self-attention over T tokens and every key j <= i of the query head's KV head:

    p_raw = softmax(s),  s_j = scale * q_i . k_j           (raw softmax over the causal prefix)
    p~_j  = p_raw_j * m_j                                   (multiplicative mask, m per KV head and key)
    p_j   = p~_j / sum_k p~_k                               (re-normalisation)
    o_i   = sum_j p_j v_j

which equals softmax(s + log m) (the proof in App. B.2) wherever the latter is defined.
``forward`` takes these three steps in that order.  ``backward`` walks the same graph in
reverse, node by node as App. B.3 does: through the re-normalisation (its Jacobian is
(delta_jk - p_j) / Z~), through the product p~ = p_raw * m (the factor towards the mask is
p_raw, never 1 / m, which is the point of the formulation), and through the raw softmax.

Layout: Q [Hq, T, d], K and V [H, T, d], m [H, T]; query head hq reads KV head hq // (Hq // H)
(Sec. 3.1: the heads of a GQA group share one KV head and therefore one mask).

Readings where the paper is silent:
* a query whose causal prefix carries no weight at all (every m_j = 0) has no defined
  distribution (0 / 0); the paper keeps m inside (0, 1) so the case cannot arise there.  Here
  its output and all its gradient contributions are zero and its log-normaliser is -inf.
* the log-normaliser returned next to the output is that of the masked weights,
  log sum_j e^{s_j} m_j, the quantity a backward pass needs to rebuild p from s.
"""
from __future__ import annotations

import numpy as np


def _group(Hq: int, H: int) -> int:
    if Hq % H != 0:
        raise ValueError("the number of query heads must be a multiple of the number of KV heads")
    return Hq // H


def forward(Q: np.ndarray, K: np.ndarray, V: np.ndarray, m: np.ndarray, scale: float, rows=None):
    """Causal attention with the multiplicative mask.  Returns (O [Hq, T, d], lse [Hq, T]).

    ``rows``: the query positions to compute (default all); the others stay 0 / -inf.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    Hq, T, d = Q.shape
    g = _group(Hq, K.shape[0])
    O = np.zeros((Hq, T, d))
    lse = np.full((Hq, T), -np.inf)
    for hq in range(Hq):
        h = hq // g
        for i in (range(T) if rows is None else rows):
            s = scale * (K[h, : i + 1] @ Q[hq, i])
            top = s.max()
            e = np.exp(s - top)
            p_raw = e / e.sum()                       # step 1: raw softmax
            p_tilde = p_raw * m[h, : i + 1]           # step 2: multiplicative mask
            z_tilde = p_tilde.sum()
            if z_tilde > 0.0:
                p = p_tilde / z_tilde                 # step 3: re-normalisation
                O[hq, i] = p @ V[h, : i + 1]
                lse[hq, i] = top + np.log(e.sum()) + np.log(z_tilde)
    return O, lse


def backward(Q: np.ndarray, K: np.ndarray, V: np.ndarray, m: np.ndarray, scale: float, dO: np.ndarray, rows=None):
    """Gradients of sum(O * dO) with respect to Q, K, V and m (App. B.3's graph, reversed).

    ``rows``: only these query positions contribute (default all).  With rows = range(j, T) the
    gradients of the keys j .. T - 1 and of those queries are complete, since earlier queries do
    not see these keys.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    Hq, T, d = Q.shape
    g = _group(Hq, K.shape[0])
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    dm = np.zeros_like(m)
    for hq in range(Hq):
        h = hq // g
        for i in (range(T) if rows is None else rows):
            n = i + 1
            s = scale * (K[h, :n] @ Q[hq, i])
            e = np.exp(s - s.max())
            p_raw = e / e.sum()
            p_tilde = p_raw * m[h, :n]
            z_tilde = p_tilde.sum()
            if not z_tilde > 0.0:
                continue
            p = p_tilde / z_tilde
            # o = p V
            dp = V[h, :n] @ dO[hq, i]
            dV[h, :n] += np.outer(p, dO[hq, i])
            # p = p~ / Z~ : d p_k / d p~_j = (delta_jk - p_k) / Z~
            dp_tilde = (dp - p @ dp) / z_tilde
            # p~ = p_raw * m : the factor towards m is p_raw, towards p_raw it is m
            dm[h, :n] += dp_tilde * p_raw
            dp_raw = dp_tilde * m[h, :n]
            # p_raw = softmax(s)
            ds = p_raw * (dp_raw - p_raw @ dp_raw)
            # s = scale * K q
            dQ[hq, i] += scale * (ds @ K[h, :n])
            dK[h, :n] += scale * np.outer(ds, Q[hq, i])
    return dQ, dK, dV, dm
