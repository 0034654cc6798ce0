"""The input generators: determinism, storage rounding, shapes.  CPU only."""
import numpy as np
import torch

from paper_2605_06676_amd import workloads as W


def test_bf16_rounding_matches_torch_rne():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, np.inf, -np.inf, 3.3895e38], np.float32)])
    mine = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(mine, ref)
    assert np.array_equal(W.bf16_bits_to_f32(mine), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_draws_are_seeded_and_layer_sliceable():
    w = W.scaled(W.CONFIGS[1], L=3, H=2, T=64)
    K1, V1 = W.draw_kv(w, 64)
    K2, V2 = W.draw_kv(w, 64)
    assert np.array_equal(K1, K2) and np.array_equal(V1, V2)
    k_l, v_l = W.draw_kv_layer(w, 64, 0, 2)
    assert np.array_equal(k_l, K1[2]) and np.array_equal(v_l, V1[2])
    K3, _ = W.draw_kv(w, 64, seed=1)
    assert not np.array_equal(K1, K3)


def test_outlier_channels_are_scaled():
    w = W.scaled(W.CONFIGS[1], L=1, H=2, T=4096)
    K, V = W.draw_kv(w, 4096)
    ch = W.outlier_channels(w)
    x = np.concatenate([W.bf16_bits_to_f32(K), W.bf16_bits_to_f32(V)], axis=-1)
    for h in range(2):
        std = x[0, h].std(axis=0)
        hot = np.zeros(256, bool); hot[ch[0, h]] = True
        assert np.all(std[hot] > 8) and np.all(std[~hot] < 1.2)


def test_config_table_shapes():
    n_ht = [1 * 8 * 4096, 32 * 8 * 32768, 32 * 8 * 131072]
    for w, n in zip(W.CONFIGS[:3], n_ht):
        assert w.L * w.H * int(W.seq_lengths(w)[0]) == n
    w3 = W.CONFIGS[3]
    Ts = W.seq_lengths(w3)
    assert Ts.size == 16 and Ts.min() >= 4096 and Ts.max() <= 16384
    assert W.CONFIGS[4].g == 7 and W.CONFIGS[1].g == 4
    paper = W.draw_scorer(W.scaled(W.CONFIGS[5], L=2))
    assert paper["w1"].shape == (2, 8, 128, 256) and paper["b2"] is None and paper["act"] == "silu"
    sc = W.draw_scorer(W.CONFIGS[2])
    assert sc["w1"].shape == (32, 1, 64, 256) and sc["w1"].dtype == np.uint16
    assert abs(W.bf16_bits_to_f32(sc["w1"]).std() - 0.02) < 1e-3


def test_training_attention_draw():
    q, k, v, m, d_o = W.draw_training_attention(8, 2, 500, seed=3)
    assert q.shape == d_o.shape == (8, 500, 128) and k.shape == v.shape == (2, 500, 128) and m.shape == (2, 500)
    assert q.dtype == np.uint16 and m.dtype == np.float32
    again = W.draw_training_attention(8, 2, 500, seed=3)
    assert all(np.array_equal(a, b) for a, b in zip((q, k, v, m, d_o), again))
    assert not np.array_equal(m, W.draw_training_attention(8, 2, 500, seed=4)[3])
    assert m.min() >= 0.0 and m.max() <= 1.0 and (m == 0).any() and (m == 1).any() and (m[:, 0] >= 0.25).all()
    assert 0.1 < m.mean() < 0.35                       # most weights small, as late in the annealing
    assert abs(W.bf16_bits_to_f32(k).std() - 1.0) < 0.02


def test_window_queries_draw():
    w = W.scaled(W.CONFIGS[0], L=2, H=2, Hq=8, T=300, b_min=1)
    K, _ = W.draw_kv(w, 300, 0, 3)
    q = W.draw_window_queries(w, K, 32, 0, 3)
    assert q.shape == (2, 8, 32, 128) and q.dtype == np.uint16
    assert np.array_equal(q, W.draw_window_queries(w, K, 32, 0, 3))
    assert not np.array_equal(q, W.draw_window_queries(w, K, 32, 0, 4))
    # about half of the rows carry a needle: their norm is above that of a plain N(0, 1) row
    qf, kf = W.bf16_bits_to_f32(q), W.bf16_bits_to_f32(K)
    logits = np.einsum("lgwd,lgtd->lgwt", qf.reshape(2, 2, 4 * 32, 128), kf[:, :, :268]) / np.sqrt(128.0)
    peaked = (logits.max(-1) > 4.0).mean()
    assert 0.3 < peaked < 0.7
    # a window as long as the prompt has no prefix to plant needles in
    assert W.draw_window_queries(w, K, 300, 0, 3).shape == (2, 8, 300, 128)
