"""Pins of the oracle for the training-time attention with a multiplicative mask (App. B).

Each test checks oracle/masked_attn.py against something other than itself: a library
attention routine, automatic differentiation of the log-space formulation the paper proves
equivalent, finite differences, or an identity that follows from the formula.
"""
import numpy as np
import torch

from oracle import masked_attn as ma


def _draw(seed, Hq=4, H=2, T=11, d=8, zero_frac=0.0):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((Hq, T, d))
    K = rng.standard_normal((H, T, d))
    V = rng.standard_normal((H, T, d))
    m = rng.uniform(0.05, 1.0, size=(H, T))
    if zero_frac > 0:
        m[rng.uniform(size=m.shape) < zero_frac] = 0.0
        m[:, 0] = np.maximum(m[:, 0], 0.3)     # every causal prefix keeps some weight
    dO = rng.standard_normal((Hq, T, d))
    return Q, K, V, m, dO, 1.0 / np.sqrt(d)


def _torch_logspace(Q, K, V, m, scale):
    """softmax(s + log m) with a causal mask, plain torch ops in fp64 (App. B.1's formulation)."""
    Hq, T, _ = Q.shape
    g = Hq // K.shape[0]
    Kx = K.repeat_interleave(g, dim=0)
    Vx = V.repeat_interleave(g, dim=0)
    mx = m.repeat_interleave(g, dim=0)
    s = scale * Q @ Kx.transpose(1, 2) + torch.log(mx)[:, None, :]
    causal = torch.ones(T, T, dtype=torch.bool).tril()
    s = s.masked_fill(~causal, float("-inf"))
    return torch.softmax(s, dim=-1) @ Vx, torch.logsumexp(s, dim=-1)


def test_all_ones_mask_is_plain_causal_attention():
    # m = 1 everywhere: the three steps collapse to Eq. 1 with a causal mask, a library routine
    Q, K, V, m, _, scale = _draw(1)
    m[:] = 1.0
    O, lse = ma.forward(Q, K, V, m, scale)
    g = Q.shape[0] // K.shape[0]
    tq, tk, tv = (torch.from_numpy(x) for x in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk.repeat_interleave(g, 0)[None], tv.repeat_interleave(g, 0)[None], is_causal=True, scale=scale)[0]
    assert np.allclose(O, ref.numpy(), rtol=0, atol=1e-12)
    s = scale * tq @ tk.repeat_interleave(g, 0).transpose(1, 2)
    s = s.masked_fill(~torch.ones(s.shape[-2:], dtype=torch.bool).tril(), float("-inf"))
    assert np.allclose(lse, torch.logsumexp(s, -1).numpy(), rtol=0, atol=1e-12)


def test_binary_mask_is_attention_over_the_kept_keys():
    # m in {0, 1}: the masked, re-normalised softmax is attention restricted to the kept keys
    # (the identity eviction rests on), here through the library routine's boolean mask
    Q, K, V, m, _, scale = _draw(2, zero_frac=0.5)
    m = (m > 0).astype(np.float64)
    O, _ = ma.forward(Q, K, V, m, scale)
    Hq, T, _ = Q.shape
    g = Hq // K.shape[0]
    keep = torch.from_numpy(m > 0).repeat_interleave(g, 0)[:, None, :] & torch.ones(T, T, dtype=torch.bool).tril()
    tq, tk, tv = (torch.from_numpy(x) for x in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk.repeat_interleave(g, 0)[None], tv.repeat_interleave(g, 0)[None], attn_mask=keep[None], scale=scale)[0]
    assert np.allclose(O, ref.numpy(), rtol=0, atol=1e-12)


def test_forward_equals_logspace_softmax():
    # the algebraic equivalence proved in App. B.2, outputs and log-normaliser
    Q, K, V, m, _, scale = _draw(3)
    O, lse = ma.forward(Q, K, V, m, scale)
    ref, ref_lse = _torch_logspace(*(torch.from_numpy(x) for x in (Q, K, V, m)), scale)
    assert np.allclose(O, ref.numpy(), rtol=0, atol=1e-12)
    assert np.allclose(lse, ref_lse.numpy(), rtol=0, atol=1e-12)


def test_backward_equals_autograd_of_the_logspace_form():
    # where m > 0 both formulations are the same function, so their gradients agree; the
    # log-space one is differentiated by torch, which shares nothing with the oracle
    Q, K, V, m, dO, scale = _draw(4)
    tq, tk, tv, tm = (torch.from_numpy(x).requires_grad_(True) for x in (Q, K, V, m))
    out, _ = _torch_logspace(tq, tk, tv, tm, scale)
    (out * torch.from_numpy(dO)).sum().backward()
    dQ, dK, dV, dm = ma.backward(Q, K, V, m, scale, dO)
    for mine, ref in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad), (dm, tm.grad)):
        assert np.allclose(mine, ref.numpy(), rtol=0, atol=1e-11)


def test_backward_by_finite_differences_also_at_zero_mask():
    # the forward is a rational function of m, smooth through m = 0: central differences hold there too
    Q, K, V, m, dO, scale = _draw(5, Hq=2, H=1, T=7, d=4, zero_frac=0.4)
    assert (m == 0).any()
    grads = ma.backward(Q, K, V, m, scale, dO)
    args = [Q, K, V, m]

    def loss():
        return float((ma.forward(*args, scale)[0] * dO).sum())

    rng = np.random.default_rng(0)
    step = 1e-6
    for which in range(4):
        x = args[which]
        picks = [tuple(rng.integers(0, n) for n in x.shape) for _ in range(12)]
        if which == 3:
            picks += [tuple(p) for p in np.argwhere(m == 0)[:4]]
        for at in picks:
            keep = x[at]
            x[at] = keep + step
            up = loss()
            x[at] = keep - step
            down = loss()
            x[at] = keep
            assert abs((up - down) / (2 * step) - grads[which][at]) < 1e-7, (which, at)


def test_mask_gradient_is_finite_where_the_logspace_form_breaks():
    # App. B.1 against B.3: at m_i = 0 the log-space graph multiplies by 1 / m_i and yields no
    # usable number, the multiplicative one scales by p_raw and stays finite
    Q, K, V, m, dO, scale = _draw(6, zero_frac=0.4)
    tq, tk, tv, tm = (torch.from_numpy(x).requires_grad_(True) for x in (Q, K, V, m))
    out, _ = _torch_logspace(tq, tk, tv, tm, scale)
    (out * torch.from_numpy(dO)).sum().backward()
    assert not torch.isfinite(tm.grad[tm.detach() == 0]).all()
    dm = ma.backward(Q, K, V, m, scale, dO)[3]
    assert np.isfinite(dm).all()
    # closed form at an evicted key j of a single-query problem: e^{s_j} (dO . v_j - dO . o) / Z
    i = Q.shape[1] - 1
    Q1, dO1 = Q[:1, i:i + 1], dO[:1, i:i + 1]
    # a one-query problem is the last row of a causal one: put the query last by truncating nothing
    s = scale * K[0] @ Q1[0, 0]
    w = np.exp(s) * m[0]
    o = (w / w.sum()) @ V[0]
    expect = np.exp(s) * (V[0] @ dO1[0, 0] - o @ dO1[0, 0]) / w.sum()
    full = np.zeros_like(dO[:1])
    full[0, i] = dO1[0, 0]
    dm_one = ma.backward(Q[:1], K[:1], V[:1], m[:1], scale, full)[3]
    assert np.allclose(dm_one[0], expect, rtol=0, atol=1e-12)


def test_mask_gradient_is_orthogonal_to_the_mask():
    # p is unchanged when a head's whole mask is multiplied by a constant, so the directional
    # derivative along m vanishes: sum_j m_j dL/dm_j = 0 for every KV head
    Q, K, V, m, dO, scale = _draw(7, zero_frac=0.2)
    dm = ma.backward(Q, K, V, m, scale, dO)[3]
    assert np.allclose((dm * m).sum(axis=1), 0.0, atol=1e-12)
    O1, _ = ma.forward(Q, K, V, m, scale)
    O2, _ = ma.forward(Q, K, V, 0.37 * m, scale)
    assert np.allclose(O1, O2, rtol=0, atol=1e-13)


def test_first_query_and_empty_prefix():
    Q, K, V, m, dO, scale = _draw(8)
    O, lse = ma.forward(Q, K, V, m, scale)
    g = Q.shape[0] // K.shape[0]
    for hq in range(Q.shape[0]):
        # the first query sees one key: its output is that value row whatever the mask weight
        assert np.allclose(O[hq, 0], V[hq // g, 0], rtol=0, atol=1e-14)
        assert np.isclose(lse[hq, 0], scale * Q[hq, 0] @ K[hq // g, 0] + np.log(m[hq // g, 0]))
    # a prefix without any weight: zero output, -inf normaliser, no gradient from those queries
    m[:, :3] = 0.0
    O, lse = ma.forward(Q, K, V, m, scale)
    assert (O[:, :3] == 0).all() and np.isneginf(lse[:, :3]).all() and np.isfinite(lse[:, 3:]).all()
    only_early = np.zeros_like(dO)
    only_early[:, :3] = dO[:, :3]
    for grad in ma.backward(Q, K, V, m, scale, only_early):
        assert (grad == 0).all()


def test_group_heads_share_their_kv_head():
    # the heads of a GQA group with equal queries give equal outputs, and the KV-side gradients
    # add up over the group
    Q, K, V, m, dO, scale = _draw(9, Hq=4, H=2)
    Q[1] = Q[0]
    O, _ = ma.forward(Q, K, V, m, scale)
    assert np.array_equal(O[0], O[1])
    _, dK, dV, dm = ma.backward(Q, K, V, m, scale, dO)
    parts = [ma.backward(Q[h:h + 1], K[:1], V[:1], m[:1], scale, dO[h:h + 1]) for h in (0, 1)]
    assert np.allclose(dK[0], parts[0][1][0] + parts[1][1][0], atol=1e-13)
    assert np.allclose(dV[0], parts[0][2][0] + parts[1][2][0], atol=1e-13)
    assert np.allclose(dm[0], parts[0][3][0] + parts[1][3][0], atol=1e-13)


def test_row_subsets():
    # computing some query rows only gives those rows of the full result, and the key-side gradients
    # of the last keys are complete once every query at or after them is included
    Q, K, V, m, dO, scale = _draw(11, T=13)
    O, lse = ma.forward(Q, K, V, m, scale)
    pick = [2, 7, 12]
    Os, ls = ma.forward(Q, K, V, m, scale, rows=pick)
    assert np.array_equal(Os[:, pick], O[:, pick]) and np.array_equal(ls[:, pick], lse[:, pick])
    rest = [i for i in range(13) if i not in pick]
    assert (Os[:, rest] == 0).all() and np.isneginf(ls[:, rest]).all()
    full = ma.backward(Q, K, V, m, scale, dO)
    tail = ma.backward(Q, K, V, m, scale, dO, rows=range(9, 13))
    assert np.allclose(tail[0][:, 9:], full[0][:, 9:], rtol=0, atol=1e-14)      # dQ of those queries
    for a, b in zip(tail[1:], full[1:]):                                         # dK, dV, dm of keys 9..12
        assert np.allclose(a[:, 9:], b[:, 9:], rtol=0, atol=1e-14)
