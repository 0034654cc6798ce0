"""Decode-time growth of the compacted cache, fp64 / exact copies, CPU, one sequence.

TEST INFRASTRUCTURE, NOT PRODUCT: only tests, the smoke check and the CPU leg
of the benchmark may use this module.

The paper evicts during prefill (Sec. 1) and defines decoding as q_t attending
to every cached token up to t (Eq. 1); the inference-time budget of a head at
step t is floor(r t) (Sec. 3.3).  It does not say how the compacted cache
follows t during decoding.  The reading taken here:

* every segment of the packed cache is given `slack` spare rows behind its
  kept rows; segment s then owns rows cap_offsets[s] .. cap_offsets[s+1] of
  which the first lengths[s] are in use;
* a decode step appends the new token's key and value (and its LKV-T score,
  which depends on that token alone, Sec. 3.4) to every segment;
* attention reads the rows in use, i.e. the kept prefill tokens and all
  tokens generated since (App. B.2 with a 0/1 mask that is 1 on them);
* when the slack is used up the cache is re-evicted: with the budgets
  b' = floor(r t') of the new length t', each head keeps the b' rows it holds
  with the largest stored scores (same hard top-k and tie rule as at prefill;
  "position" is the position among the held rows, which is time order), and
  gets fresh slack.  Tokens dropped earlier do not come back.

Each function works on plain arrays; a segment is s = l * H + h.

Pins: tests/test_oracle_growth.py (the decode over a grown cache equals the
masked attention of App. B.2 over the whole history; no slack and no appends
is the plain compacted cache; re-eviction against a brute-force ranking of
the held scores with token identities tracked separately; keeping everything
is the identity).
"""
from __future__ import annotations

import numpy as np

from . import lkv_oracle as O


def grown_layout(budgets: np.ndarray, slack: int):
    """cap_offsets [n_seg + 1] and lengths [n_seg] of a cache with `slack` spare rows per segment."""
    b = np.asarray(budgets, dtype=np.int64).reshape(-1)
    cap = np.zeros(b.size + 1, dtype=np.int64)
    cap[1:] = np.cumsum(b + int(slack))
    return cap, b.copy()


def compact_with_slack(K, V, u, idx, offsets, slack):
    """Packed cache with slack.  K, V [L, H, T, d] (any dtype, copied bit for bit), u fp32 [L, H, T],
    idx / offsets as written by select_all.  Unused rows are zero."""
    L, H, T, d = K.shape
    budgets = np.diff(np.asarray(offsets, dtype=np.int64))
    cap, lengths = grown_layout(budgets, slack)
    Kp = np.zeros((int(cap[-1]), d), dtype=K.dtype)
    Vp = np.zeros((int(cap[-1]), d), dtype=V.dtype)
    up = np.zeros(int(cap[-1]), dtype=np.float32)
    for l in range(L):
        for h in range(H):
            s = l * H + h
            rows = idx[offsets[s]:offsets[s + 1]]
            Kp[cap[s]:cap[s] + lengths[s]] = K[l, h, rows]
            Vp[cap[s]:cap[s] + lengths[s]] = V[l, h, rows]
            up[cap[s]:cap[s] + lengths[s]] = u[l, h, rows]
    return Kp, Vp, up, cap, lengths


def append(Kp, Vp, up, cap, lengths, k_new, v_new, u_new):
    """One generated token: k_new, v_new [n_seg, d], u_new [n_seg].  In place.  A full segment
    is left as it is; returns True if any segment was full."""
    overflow = False
    for s in range(lengths.size):
        row = cap[s] + lengths[s]
        if row >= cap[s + 1]:
            overflow = True
            continue
        Kp[row] = k_new[s]
        Vp[row] = v_new[s]
        up[row] = u_new[s]
        lengths[s] += 1
    return overflow


def tight(Kp, Vp, cap, lengths):
    """The rows in use, packed without gaps, and their offsets."""
    off = np.zeros(lengths.size + 1, dtype=np.int64)
    off[1:] = np.cumsum(lengths)
    rows = np.concatenate([np.arange(cap[s], cap[s] + lengths[s]) for s in range(lengths.size)] + [np.zeros(0, dtype=np.int64)])
    rows = rows.astype(np.int64)
    return Kp[rows], Vp[rows], off


def decode_grown(q, Kp64, Vp64, cap, lengths, H, scale):
    """Eq. 1 over the rows in use of every segment.  q fp64 [L, Hq, d]; Kp64, Vp64 fp64."""
    Kt, Vt, off = tight(Kp64, Vp64, cap, lengths)
    return O.decode_attn(q, Kt, Vt, off, H, scale)


def reevict(Kp, Vp, up, cap, lengths, new_budgets, slack):
    """Keep, per segment, the new_budgets[s] held rows with the largest stored scores (ties to the
    earlier row), in their order, and lay the result out with fresh slack.  Returns the new
    (Kp, Vp, up, cap, lengths) and, per segment, the positions among the old held rows that stay."""
    nb = np.asarray(new_budgets, dtype=np.int64).reshape(-1)
    assert np.all(nb <= lengths) and np.all(nb >= 0)
    cap2, len2 = grown_layout(nb, slack)
    K2 = np.zeros((int(cap2[-1]), Kp.shape[1]), dtype=Kp.dtype)
    V2 = np.zeros((int(cap2[-1]), Vp.shape[1]), dtype=Vp.dtype)
    u2 = np.zeros(int(cap2[-1]), dtype=np.float32)
    kept = []
    for s in range(lengths.size):
        held = up[cap[s]:cap[s] + lengths[s]]
        pos = O.select(held, int(nb[s]))
        kept.append(pos)
        K2[cap2[s]:cap2[s] + nb[s]] = Kp[cap[s] + pos]
        V2[cap2[s]:cap2[s] + nb[s]] = Vp[cap[s] + pos]
        u2[cap2[s]:cap2[s] + nb[s]] = held[pos]
    return K2, V2, u2, cap2, len2, kept
