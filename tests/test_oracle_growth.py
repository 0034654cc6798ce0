"""Pins of the decode-time growth oracle against the definitions it must reduce to."""
import numpy as np
import pytest

from oracle import lkv_growth as GR
from oracle import lkv_oracle as O
from paper_2605_06676_amd import workloads as W


def _small(seed, T=90, L=2, H=3, Hq=6, slack=5, n_new=5):
    w = W.scaled(W.CONFIGS[0], L=L, H=H, Hq=Hq, b_min=2)
    Kb, Vb = W.draw_kv(w, T, 0, seed)
    sc = W.draw_scorer(w, seed)
    K64, V64 = O.bf16_bits_to_f64(Kb), O.bf16_bits_to_f64(Vb)
    sco = {"kind": sc["kind"], "act": sc["act"], "w1": O.bf16_bits_to_f64(sc["w1"]),
           "b1": np.asarray(sc["b1"], np.float64), "w2": None, "b2": None}
    u = O.score(K64, V64, sco)
    budgets = W.draw_budgets(w, T, 0, seed)
    idx, off = O.select_all(u, budgets)
    # generated tokens: fresh rows drawn with another seed, scored by the same scorer
    w_new = W.scaled(w, cid=77)
    Kn, Vn = W.draw_kv(w_new, n_new, 0, seed + 1)           # [L, H, n_new, d]
    un = O.score(O.bf16_bits_to_f64(Kn), O.bf16_bits_to_f64(Vn), sco)
    q = O.bf16_bits_to_f64(W.draw_q(w, 0, seed))
    return w, Kb, Vb, u, budgets, idx, off, Kn, Vn, un, q


def test_no_slack_no_append_is_the_plain_packed_cache():
    w, Kb, Vb, u, budgets, idx, off, *_ = _small(0, slack=0)
    Kp, Vp, up, cap, lengths = GR.compact_with_slack(Kb, Vb, u, idx, off, 0)
    Kt, Vt = O.compact(Kb, Vb, idx, off)
    assert np.array_equal(Kp, Kt) and np.array_equal(Vp, Vt)
    assert np.array_equal(cap, off) and np.array_equal(lengths, budgets.reshape(-1))


@pytest.mark.parametrize("seed", range(3))
def test_decode_over_a_grown_cache_is_masked_attention_over_the_whole_history(seed):
    # Eq. 1 / App. B.2: the step after n generated tokens attends the kept prefill tokens and
    # every generated token, i.e. a 0/1 mask over the T + n tokens of the history
    slack, n_new = 6, 4
    w, Kb, Vb, u, budgets, idx, off, Kn, Vn, un, q = _small(seed, slack=slack, n_new=n_new)
    Kp, Vp, up, cap, lengths = GR.compact_with_slack(Kb, Vb, u, idx, off, slack)
    n_seg = w.L * w.H
    for j in range(n_new):
        full = GR.append(Kp, Vp, up, cap, lengths, Kn[:, :, j].reshape(n_seg, -1), Vn[:, :, j].reshape(n_seg, -1),
                         un[:, :, j].reshape(n_seg))
        assert not full
    assert np.array_equal(lengths, budgets.reshape(-1) + n_new)
    scale = 1.0 / np.sqrt(w.d)
    o, lse = GR.decode_grown(q, O.bf16_bits_to_f64(Kp), O.bf16_bits_to_f64(Vp), cap, lengths, w.H, scale)
    T = Kb.shape[2]
    K_hist = np.concatenate([O.bf16_bits_to_f64(Kb), O.bf16_bits_to_f64(Kn)], axis=2)
    V_hist = np.concatenate([O.bf16_bits_to_f64(Vb), O.bf16_bits_to_f64(Vn)], axis=2)
    mask = np.zeros((w.L, w.H, T + n_new))
    for s in range(n_seg):
        mask[s // w.H, s % w.H, idx[off[s]:off[s + 1]]] = 1.0
    mask[:, :, T:] = 1.0
    g = w.Hq // w.H
    for l in range(w.L):
        for hq in range(w.Hq):
            h = hq // g
            if mask[l, h].sum() == 0:
                continue
            o_ref = O.masked_attention_full(q[l, hq], K_hist[l, h], V_hist[l, h], mask[l, h], scale)
            assert np.allclose(o[l, hq], o_ref, rtol=1e-10, atol=1e-12)


def test_append_to_a_full_segment_is_refused_and_reported():
    w, Kb, Vb, u, budgets, idx, off, Kn, Vn, un, q = _small(1, slack=1, n_new=2)
    Kp, Vp, up, cap, lengths = GR.compact_with_slack(Kb, Vb, u, idx, off, 1)
    n_seg = w.L * w.H
    args = lambda j: (Kn[:, :, j].reshape(n_seg, -1), Vn[:, :, j].reshape(n_seg, -1), un[:, :, j].reshape(n_seg))
    assert not GR.append(Kp, Vp, up, cap, lengths, *args(0))
    before = (Kp.copy(), Vp.copy(), up.copy(), lengths.copy())
    assert GR.append(Kp, Vp, up, cap, lengths, *args(1))
    assert all(np.array_equal(a, b) for a, b in zip(before, (Kp, Vp, up, lengths)))


@pytest.mark.parametrize("seed", range(3))
def test_reeviction_against_brute_force_with_token_identities(seed):
    slack, n_new = 4, 4
    w, Kb, Vb, u, budgets, idx, off, Kn, Vn, un, q = _small(seed, slack=slack, n_new=n_new)
    Kp, Vp, up, cap, lengths = GR.compact_with_slack(Kb, Vb, u, idx, off, slack)
    n_seg, T = w.L * w.H, Kb.shape[2]
    for j in range(n_new):
        GR.append(Kp, Vp, up, cap, lengths, Kn[:, :, j].reshape(n_seg, -1), Vn[:, :, j].reshape(n_seg, -1),
                  un[:, :, j].reshape(n_seg))
    rng = np.random.default_rng(seed)
    nb = np.array([int(rng.integers(0, lengths[s] + 1)) for s in range(n_seg)])
    K2, V2, u2, cap2, len2, kept = GR.reevict(Kp, Vp, up, cap, lengths, nb, 3)
    assert np.array_equal(len2, nb) and np.array_equal(np.diff(cap2), nb + 3)
    u_hist = np.concatenate([u, un], axis=2)                  # scores of the whole history, by token id
    K_hist = np.concatenate([Kb, Kn], axis=2)
    for s in range(n_seg):
        l, h = divmod(s, w.H)
        ids = np.concatenate([idx[off[s]:off[s + 1]], T + np.arange(n_new)])      # token ids held, in time order
        # brute force: rank the held ids by (score descending, id ascending), keep nb[s], restore time order
        ranked = sorted(ids, key=lambda t: (-float(u_hist[l, h, t]), t))
        want = np.array(sorted(ranked[:nb[s]]), dtype=np.int64)
        got = ids[kept[s]]
        if np.unique(u_hist[l, h, ids]).size == ids.size:
            assert np.array_equal(got, want)
        assert np.array_equal(K2[cap2[s]:cap2[s] + nb[s]], K_hist[l, h, got])
        assert np.array_equal(u2[cap2[s]:cap2[s] + nb[s]], u_hist[l, h, got])
    # keeping everything changes nothing but the slack
    K3, V3, u3, cap3, len3, kept3 = GR.reevict(Kp, Vp, up, cap, lengths, lengths, slack)
    for s in range(n_seg):
        assert np.array_equal(kept3[s], np.arange(lengths[s]))
        assert np.array_equal(K3[cap3[s]:cap3[s] + len3[s]], Kp[cap[s]:cap[s] + lengths[s]])
