"""Pins of the LKV-H oracle (Sec. 3.3; Table 5) against what the paper and the mathematics fix."""
import math
import os

import numpy as np
import pytest

from oracle import lkv_h as H
from oracle import lkv_oracle as O
from oracle import soft_topk as ST
from paper_2605_06676_amd import workloads as W



def golden_constants(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = [p.strip() for p in line.split("=")]
                vals[k] = float(v)
    return vals


def test_predictor_parameter_count_is_table_5(golden_dir):
    g = golden_constants(golden_dir)
    assert H.predictor_param_count(128, 64, out_bias=False) == g["lkv_h_unit_params"]
    assert H.predictor_param_count(128, 64, out_bias=True) != g["lkv_h_unit_params"]
    assert g["llama_layers"] * g["llama_kv_heads"] * g["head_dim"] == g["lkv_h_embed_llama"]
    assert g["qwen3_layers"] * g["llama_kv_heads"] * g["head_dim"] == g["lkv_h_embed_qwen3"]


def test_head_scores_tiny_network_by_hand():
    # two heads, d_e = 3, two hidden units; every number below is worked out term by term
    emb = np.array([[1.0, -2.0, 0.5], [0.0, 3.0, -1.0]])
    mlp = {"w1": np.array([[0.5, 0.25, -1.0], [-1.5, 0.0, 2.0]]), "b1": np.array([0.1, -0.2]),
           "w2": np.array([2.0, -3.0]), "b2": None}
    def silu(z):
        return z / (1.0 + math.exp(-z))
    z00 = 0.5 * 1.0 + 0.25 * -2.0 + -1.0 * 0.5 + 0.1       # head 0, unit 0
    z01 = -1.5 * 1.0 + 0.0 * -2.0 + 2.0 * 0.5 + -0.2       # head 0, unit 1
    z10 = 0.5 * 0.0 + 0.25 * 3.0 + -1.0 * -1.0 + 0.1
    z11 = -1.5 * 0.0 + 0.0 * 3.0 + 2.0 * -1.0 + -0.2
    want = np.array([2.0 * silu(z00) - 3.0 * silu(z01), 2.0 * silu(z10) - 3.0 * silu(z11)])
    got = H.head_scores(emb, mlp)
    assert np.allclose(got, want, rtol=1e-14)
    # an output bias shifts every score by the same amount
    mlp_b = dict(mlp, b2=0.75)
    assert np.allclose(H.head_scores(emb, mlp_b), want + 0.75, rtol=1e-14)
    # a transposed w1 or a dropped bias must show: the four pre-activations are all different
    assert len({round(v, 9) for v in (z00, z01, z10, z11)}) == 4


def test_head_scores_zero_first_layer_is_closed_form():
    rng = np.random.default_rng(0)
    emb = rng.standard_normal((7, 128))
    b1 = rng.standard_normal(64)
    w2 = rng.standard_normal(64)
    s = H.head_scores(emb, {"w1": np.zeros((64, 128)), "b1": b1, "w2": w2, "b2": None})
    want = sum(w2[j] * b1[j] / (1.0 + math.exp(-b1[j])) for j in range(64))
    assert np.allclose(s, want, rtol=1e-13)


@pytest.mark.parametrize("R", [0.05, 0.15, 0.5, 0.9])
def test_equal_heads_all_get_the_global_ratio(R):
    # identical scores: by symmetry every head receives k / n = R
    r = H.head_ratios(np.full(256, 1.2345), R)
    assert np.allclose(r, R, rtol=1e-12)


@pytest.mark.parametrize("a", [0.1, 1.0, 4.0])
def test_two_antisymmetric_heads_closed_form(a):
    # n = 2, k = 1, scores (a, -a): the threshold is 0 by symmetry, so r = (1 - e^-a / 2, e^-a / 2)
    r = H.head_ratios(np.array([a, -a]), 0.5)
    assert r[0] == pytest.approx(1.0 - 0.5 * math.exp(-a), rel=1e-13)
    assert r[1] == pytest.approx(0.5 * math.exp(-a), rel=1e-13)


@pytest.mark.parametrize("cid,R", [(1, 0.15), (2, 0.10), (4, 0.3)])
def test_ratios_and_budgets_properties_on_workload_draws(cid, R):
    w = W.CONFIGS[cid]
    emb, mlp = W.draw_head_predictor(w)
    n = w.L * w.H
    assert emb.shape == (n, 128) and mlp["w1"].shape == (64, 128)
    s = H.head_scores(emb, mlp)
    r = H.head_ratios(s, R)
    assert r.shape == (n,)
    assert np.all((r > 0) & (r < 1))
    assert r.sum() == pytest.approx(R * n, rel=1e-12)                 # sum of ratios = R L H
    order = np.argsort(s)
    assert np.all(np.diff(r[order]) >= 0)                              # a higher score never gets less
    assert r.max() / r.min() > 3                                       # the draw is heterogeneous
    # the ratios are the Laplace CDF of the scores around one common threshold
    lam, _ = ST.soft_topk_lambda(s, R * n)
    assert np.allclose(r, np.where(s >= lam, 1 - 0.5 * np.exp(lam - s), 0.5 * np.exp(s - lam)), rtol=1e-12)
    for t in (1, 1000, 32768, 131072):
        b = H.head_budgets(r, t)
        assert np.array_equal(b, O.integer_budgets(r, t))
        assert np.all((b >= 0) & (b < t))
        total = O.total_budget(R, w.L, w.H, t)
        assert total - n < b.sum() <= total                            # B_total = floor(R L H t), Sec. 3.1
