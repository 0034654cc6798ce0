"""Pins of the oracle for the observation-window scorer (the attention-based selection policy of
the ablation grid, Sec. 4.4; complexity O(W T) in the table of Sec. 4.5).

The paper prints no values for it, so every pin is a library routine, a closed form or an
identity: the window's attention weights against the library attention routine applied to an
identity value matrix, the pooling against the library's pooling layers, softmax identities,
a case worked out by hand, and the selection the scores lead to.
"""
import numpy as np
import pytest
import torch

from oracle import lkv_oracle as O
from oracle import window_score as ws


def _draw(seed, Hq=4, H=2, T=23, W=5, d=8):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((Hq, W, d)), rng.standard_normal((H, T, d)), 1.0 / np.sqrt(d)


def test_weights_are_the_last_rows_of_causal_attention():
    # with the identity as value matrix the library's attention returns the weights themselves;
    # the window rows are the last W rows of full causal self-attention
    Qw, K, scale = _draw(1)
    Hq, W, d = Qw.shape
    H, T, _ = K.shape
    G = Hq // H
    rng = np.random.default_rng(11)
    Qfull = rng.standard_normal((Hq, T, d))
    Qfull[:, T - W:] = Qw
    tk = torch.from_numpy(K).repeat_interleave(G, 0)
    eye = torch.eye(T, dtype=torch.float64).expand(Hq, T, T)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Qfull)[None], tk[None], eye[None], is_causal=True, scale=scale)[0]
    a = ws.window_attention(Qw, K, scale)
    assert np.allclose(a, ref[:, T - W:].numpy(), rtol=0, atol=1e-14)
    # votes: column sums of those rows over the prefix, group mean
    vote = ref[:, T - W:, :T - W].sum(1).reshape(H, G, T - W).mean(1)
    assert np.allclose(ws.window_votes(Qw, K, scale), vote.numpy(), rtol=0, atol=1e-14)


def test_single_query_window_is_a_plain_softmax():
    # W = 1, one head: the votes are the softmax of the last query over all T keys, cut to the prefix
    Qw, K, scale = _draw(2, Hq=1, H=1, T=9, W=1)
    p = torch.softmax(torch.from_numpy(scale * K[0] @ Qw[0, 0]), dim=0).numpy()
    s = ws.window_scores(Qw, K, scale, 1, "max")
    assert np.allclose(s[0, :8], p[:8], rtol=0, atol=1e-15)
    assert np.isposinf(s[0, 8])


def test_case_worked_by_hand():
    # d = 1, T = 3, W = 2, keys 0, ln 2, ln 3, both queries 1, scale 1:
    #   row 0 (position 1) sees keys 0, 1: weights e^0, e^{ln 2}    -> 1/3, 2/3
    #   row 1 (position 2) sees keys 0, 1, 2: weights 1, 2, 3 over 6 -> 1/6, 1/3, 1/2
    # the one prefix token collects 1/3 + 1/6 = 1/2
    K = np.log(np.array([1.0, 2.0, 3.0])).reshape(1, 3, 1)
    Qw = np.ones((1, 2, 1))
    a = ws.window_attention(Qw, K, 1.0)
    assert np.allclose(a[0], [[1 / 3, 2 / 3, 0], [1 / 6, 1 / 3, 1 / 2]], rtol=0, atol=1e-15)
    s = ws.window_scores(Qw, K, 1.0)
    assert np.isclose(s[0, 0], 0.5, rtol=0, atol=1e-15) and np.isposinf(s[0, 1:]).all()


def test_rows_are_distributions_and_mass_is_conserved():
    Qw, K, scale = _draw(3)
    a = ws.window_attention(Qw, K, scale)
    Hq, W, T = a.shape
    assert np.allclose(a.sum(-1), 1.0, rtol=0, atol=1e-14)
    for i in range(W):                                    # nothing on keys after the query
        assert (a[:, i, T - W + i + 1:] == 0).all() and (a[:, i, :T - W + i + 1] > 0).all()
    # prefix votes plus the mass that stays inside the window add up to W per KV head
    inside = a[:, :, T - W:].sum((1, 2)).reshape(K.shape[0], -1).mean(1)
    assert np.allclose(ws.window_votes(Qw, K, scale).sum(1) + inside, W, rtol=0, atol=1e-13)


def test_softmax_identities():
    Qw, K, scale = _draw(4)
    base = ws.window_votes(Qw, K, scale)
    # a shift of all keys along a direction orthogonal to every window query changes no logit
    q_flat = Qw.reshape(-1, Qw.shape[-1])
    _, _, vt = np.linalg.svd(q_flat, full_matrices=True)
    if q_flat.shape[0] < q_flat.shape[1]:
        assert np.allclose(ws.window_votes(Qw, K + 3.0 * vt[-1], scale), base, rtol=0, atol=1e-12)
    # adding the same vector to all keys shifts each row's logits by a constant: no change either
    assert np.allclose(ws.window_votes(Qw, K + np.arange(K.shape[-1]) * 0.1, scale), base, rtol=0, atol=1e-12)
    # scale and query magnitude are interchangeable
    assert np.allclose(ws.window_votes(2.0 * Qw, K, 0.5 * scale), base, rtol=0, atol=1e-12)
    # a duplicated prefix key collects exactly what its twin collects
    K2 = K.copy()
    K2[:, 7] = K2[:, 3]
    v2 = ws.window_votes(Qw, K2, scale)
    assert np.array_equal(v2[:, 7], v2[:, 3])
    # zero queries: uniform attention, row i spreads 1 / (T - W + i + 1) on each visible key
    Hq, W, _ = Qw.shape
    T = K.shape[1]
    flat = ws.window_votes(np.zeros_like(Qw), K, scale)
    assert np.allclose(flat, sum(1.0 / (T - W + i + 1) for i in range(W)), rtol=0, atol=1e-14)


def test_group_mean():
    # the score of a KV head is the mean of what its query heads would give alone
    Qw, K, scale = _draw(5, Hq=6, H=2)
    both = ws.window_votes(Qw, K, scale)
    for h in range(2):
        parts = [ws.window_votes(Qw[hq:hq + 1], K[h:h + 1], scale)[0] for hq in range(3 * h, 3 * h + 3)]
        assert np.allclose(both[h], np.mean(parts, axis=0), rtol=0, atol=1e-15)


@pytest.mark.parametrize("width", [1, 3, 5, 7, 13])
def test_pooling_against_the_library_layers(width):
    rng = np.random.default_rng(width)
    for n in (1, 2, 6, 40):
        x = rng.uniform(size=(3, n))
        tx = torch.from_numpy(x)[None]
        ref_max = torch.nn.functional.max_pool1d(tx, width, stride=1, padding=width // 2)[0].numpy()
        ref_avg = torch.nn.functional.avg_pool1d(tx, width, stride=1, padding=width // 2)[0].numpy()
        assert np.array_equal(ws.pool1d(x, width, "max"), ref_max)
        assert np.allclose(ws.pool1d(x, width, "avg"), ref_avg, rtol=0, atol=1e-15)
    with pytest.raises(ValueError):
        ws.pool1d(np.zeros((1, 4)), 4, "max")


def test_scores_keep_the_window_and_the_heaviest_prefix_tokens():
    Qw, K, scale = _draw(6, T=40, W=4)
    H, T, _ = K.shape
    W = Qw.shape[1]
    s = ws.window_scores(Qw, K, scale, 5, "avg")
    assert s.shape == (H, T) and np.isposinf(s[:, T - W:]).all() and np.isfinite(s[:, :T - W]).all()
    assert np.array_equal(s[:, :T - W], ws.pool1d(ws.window_votes(Qw, K, scale), 5, "avg"))
    for h in range(H):
        kept = O.select(s[h].astype(np.float32), 10)
        assert set(range(T - W, T)) <= set(kept.tolist())
        best = np.argsort(-s[h, :T - W], kind="stable")[:6]
        assert set(best.tolist()) <= set(kept.tolist())
    # the whole prompt inside the window: nothing to vote on
    Qall, Kall, _ = _draw(7, T=5, W=5)
    assert np.isposinf(ws.window_scores(Qall, Kall, scale, 3, "max")).all()
    with pytest.raises(ValueError):
        ws.window_attention(Qall, Kall[:, :4], scale)


def test_log_normalisers_against_the_library_logsumexp():
    Qw, K, scale = _draw(8)
    Hq, W, _ = Qw.shape
    H, T, _ = K.shape
    G = Hq // H
    lse = ws.window_log_normalisers(Qw, K, scale)
    for hq in range(Hq):
        logits = torch.from_numpy(scale * Qw[hq] @ K[hq // G].T)                    # [W, T]
        for i in range(W):
            assert np.isclose(lse[hq, i], float(torch.logsumexp(logits[i, :T - W + i + 1], 0)), rtol=0, atol=1e-13)
    # and they are the normalisers of the weights: a = exp(logit - lse)
    a = ws.window_attention(Qw, K, scale)
    for hq in range(Hq):
        logits = scale * Qw[hq] @ K[hq // G].T
        for i in range(W):
            n = T - W + i + 1
            assert np.allclose(a[hq, i, :n], np.exp(logits[i, :n] - lse[hq, i]), rtol=1e-12, atol=0)
