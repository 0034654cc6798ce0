"""Pins for the oracle's scorer (Sec. 3.4, Table 5).  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import lkv_oracle as O
from paper_2605_06676_amd import workloads as W


def _golden(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = [s.strip() for s in line.split("=")]
                vals[k] = float(v)
    return vals


def test_param_counts_match_table5(golden_dir):
    g = _golden(golden_dir)
    d = int(g["head_dim"])
    unit_t = O.scorer_param_count(2 * d, 128)
    unit_h = O.scorer_param_count(d, 64)
    assert unit_t == g["lkv_t_unit_params"]
    assert unit_h == g["lkv_h_unit_params"]
    n_llama = int(g["llama_layers"] * g["llama_kv_heads"])
    n_qwen = int(g["qwen3_layers"] * g["llama_kv_heads"])
    assert unit_t * n_llama == g["lkv_t_total_llama"]
    assert unit_t * n_qwen == g["lkv_t_total_qwen3"]
    assert d * n_llama == g["lkv_h_embed_llama"]
    assert d * n_qwen == g["lkv_h_embed_qwen3"]
    assert round((unit_t * n_llama + d * n_llama + unit_h) / 1e6, 2) == g["total_added_llama_M"]
    assert round((unit_t * n_qwen + d * n_qwen + unit_h) / 1e6, 2) == g["total_added_qwen3_M"]
    # a hidden bias plus an output bias, or no bias at all, would not give Table 5's number
    assert 256 * 128 + 128 + 128 + 1 != g["lkv_t_unit_params"]
    assert 256 * 128 + 128 != g["lkv_t_unit_params"]


def _small_kv(L=2, H=3, T=37, d=128, seed=1):
    rng = np.random.default_rng(seed)
    Kb = W.f32_to_bf16_bits(rng.standard_normal((L, H, T, d), dtype=np.float32))
    Vb = W.f32_to_bf16_bits(rng.standard_normal((L, H, T, d), dtype=np.float32))
    return Kb, Vb, O.bf16_bits_to_f64(Kb), O.bf16_bits_to_f64(Vb)


def test_bf16_conversion_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x0000, 0x8000, 0x4049, 0x7F80, 0x0001], dtype=np.uint16)
    got = O.bf16_bits_to_f64(bits)
    want = [1.0, -1.0, 0.0, -0.0, 3.140625, math.inf, 2.0 ** -133]
    assert got.tolist() == want
    assert math.copysign(1.0, got[3]) == -1.0
    # every bf16 pattern equals torch's own widening
    allb = np.arange(65536, dtype=np.uint16)
    t = torch.from_numpy(allb.astype(np.int32)).to(torch.int16).view(torch.bfloat16).to(torch.float64).numpy()
    mine = O.bf16_bits_to_f64(allb)
    both_nan = np.isnan(t) & np.isnan(mine)
    assert np.array_equal(t[~both_nan], mine[~both_nan])


@pytest.mark.parametrize("c", [0, 5, 127, 128, 200, 255])
def test_linear_one_hot_weight_reads_that_channel(c):
    # w = e_c: the score is feature c of [k ; v] exactly -- pins the k-then-v order
    Kb, Vb, K, V = _small_kv()
    L, H = K.shape[:2]
    w = np.zeros((L, 1, 256)); w[:, :, c] = 1.0
    u = O.score(K, V, {"kind": "linear", "w1": w, "b1": np.zeros((L, 1))})
    src = K[..., c] if c < 128 else V[..., c - 128]
    assert np.array_equal(u, src.astype(np.float32))


def test_linear_bias_and_brute_force():
    Kb, Vb, K, V = _small_kv(L=1, H=2, T=5)
    rng = np.random.default_rng(3)
    w = rng.normal(0, 0.02, (1, 2, 256)); b = rng.normal(0, 0.02, (1, 2))
    u = O.score(K, V, {"kind": "linear", "w1": w, "b1": b})
    for h in range(2):
        for i in range(5):
            acc = math.fsum([w[0, h, c] * K[0, h, i, c] for c in range(128)]
                            + [w[0, h, 128 + c] * V[0, h, i, c] for c in range(128)]) + b[0, h]
            assert u[0, h, i] == pytest.approx(acc, rel=1e-6, abs=1e-7)


def test_activation_closed_forms():
    # Phi(1) and the logistic function at 1, from their definitions
    assert O.gelu_erf(np.array([1.0]))[0] == pytest.approx(0.8413447460685429, rel=1e-14)
    assert O.gelu_erf(np.array([-1.0]))[0] == pytest.approx(-0.15865525393145707, rel=1e-13)
    assert O.gelu_erf(np.array([0.0]))[0] == 0.0
    assert O.silu(np.array([1.0]))[0] == pytest.approx(1.0 / (1.0 + math.exp(-1.0)), rel=1e-15)
    assert O.silu(np.array([-745.0, 745.0]))[1] == pytest.approx(745.0)
    assert O.silu(np.array([0.0]))[0] == 0.0
    # the erf form is not the tanh approximation
    z = 1.5
    tanh_form = 0.5 * z * (1 + math.tanh(math.sqrt(2 / math.pi) * (z + 0.044715 * z ** 3)))
    assert abs(O.gelu_erf(np.array([z]))[0] - tanh_form) > 1e-5


@pytest.mark.parametrize("act", ["silu", "gelu"])
def test_mlp_zero_first_layer_gives_constant(act):
    Kb, Vb, K, V = _small_kv()
    L, H = K.shape[:2]
    hidden = 16
    rng = np.random.default_rng(5)
    b1 = rng.normal(0, 1, (L, H, hidden)); w2 = rng.normal(0, 1, (L, H, hidden)); b2 = rng.normal(0, 1, (L, H))
    sc = {"kind": "mlp", "act": act, "w1": np.zeros((L, H, hidden, 256)), "b1": b1, "w2": w2, "b2": b2}
    u = O.score(K, V, sc)
    f = (lambda z: z / (1 + math.exp(-z))) if act == "silu" else (lambda z: 0.5 * z * (1 + math.erf(z / math.sqrt(2))))
    for l in range(L):
        for h in range(H):
            want = sum(w2[l, h, j] * f(b1[l, h, j]) for j in range(hidden)) + b2[l, h]
            assert np.all(u[l, h] == np.float32(want)) or np.allclose(u[l, h], want, rtol=1e-6)
    # no output bias (the paper's arrangement)
    sc["b2"] = None
    u0 = O.score(K, V, sc)
    assert np.allclose(u0.astype(np.float64) + b2[:, :, None], u, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("act,hidden", [("silu", 128), ("gelu", 64)])
def test_mlp_against_torch_fp64(act, hidden):
    # torch's linear / gelu / silu on CPU in fp64: an independent library route
    Kb, Vb, K, V = _small_kv(L=2, H=2, T=19)
    L, H = 2, 2
    rng = np.random.default_rng(7)
    w1 = rng.normal(0, 0.05, (L, H, hidden, 256)); b1 = rng.normal(0, 0.05, (L, H, hidden))
    w2 = rng.normal(0, 0.5, (L, H, hidden))
    u = O.score(K, V, {"kind": "mlp", "act": act, "w1": w1, "b1": b1, "w2": w2, "b2": None})
    F = torch.nn.functional
    for l in range(L):
        for h in range(H):
            x = torch.from_numpy(np.concatenate([K[l, h], V[l, h]], axis=1))
            pre = F.linear(x, torch.from_numpy(w1[l, h]), torch.from_numpy(b1[l, h]))
            hid = F.silu(pre) if act == "silu" else F.gelu(pre, approximate="none")
            want = F.linear(hid, torch.from_numpy(w2[l, h])[None, :])[:, 0].numpy()
            assert np.allclose(u[l, h], want, rtol=2e-7, atol=1e-9)


def test_channel_permutation_invariance():
    Kb, Vb, K, V = _small_kv(L=1, H=1, T=23)
    rng = np.random.default_rng(11)
    hidden = 32
    w1 = rng.normal(0, 0.05, (1, 1, hidden, 256)); b1 = rng.normal(0, 0.05, (1, 1, hidden)); w2 = rng.normal(0, 1, (1, 1, hidden))
    base = O.score(K, V, {"kind": "mlp", "act": "gelu", "w1": w1, "b1": b1, "w2": w2, "b2": None})
    perm = rng.permutation(256)
    x = np.concatenate([K, V], axis=-1)[..., perm]
    Kp, Vp = x[..., :128], x[..., 128:]
    got = O.score(Kp, Vp, {"kind": "mlp", "act": "gelu", "w1": w1[..., perm], "b1": b1, "w2": w2, "b2": None})
    assert np.allclose(base, got, rtol=1e-6, atol=1e-8)
    # swapping K and V without swapping the weight halves must change the result
    swapped = O.score(V, K, {"kind": "mlp", "act": "gelu", "w1": w1, "b1": b1, "w2": w2, "b2": None})
    assert not np.allclose(base, swapped, rtol=1e-3)


def test_per_layer_scorer_is_shared_by_heads():
    Kb, Vb, K, V = _small_kv(L=2, H=3, T=9)
    rng = np.random.default_rng(13)
    w = rng.normal(0, 0.02, (2, 1, 256)); b = rng.normal(0, 0.02, (2, 1))
    shared = O.score(K, V, {"kind": "linear", "w1": w, "b1": b})
    tiled = O.score(K, V, {"kind": "linear", "w1": np.repeat(w, 3, axis=1), "b1": np.repeat(b, 3, axis=1)})
    assert np.array_equal(shared, tiled)
