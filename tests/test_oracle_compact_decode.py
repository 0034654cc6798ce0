"""Pins for the oracle's compaction (Sec. 4.5) and decode attention (Eq. 1, App. B.2).  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import lkv_oracle as O
from paper_2605_06676_amd import workloads as W


def test_storage_arithmetic_of_sec_4_5(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = [s.strip() for s in line.split("=")]
                vals[k] = float(v)
    L, H, d = int(vals["llama_layers"]), int(vals["llama_kv_heads"]), int(vals["head_dim"])
    t = 204800                                    # "200k" with k = 1024
    full = O.packed_cache_bytes(np.full((L, H), t), d)
    assert full / 2 ** 30 == vals["kv_full_gb_at_200k"]
    # any budget table that spends B_total = floor(R L H t) packs to R * full: no padding
    B = O.total_budget(vals["retention"], L, H, t)
    rng = np.random.default_rng(0)
    p = rng.dirichlet(np.ones(L * H))
    b = np.floor(p * B).astype(np.int64)
    b[0] += B - b.sum()
    assert O.packed_cache_bytes(b, d) / 2 ** 30 == vals["kv_lkv_gb_at_200k"]
    assert math.floor(full / O.packed_cache_bytes(b, d) * 10) / 10 == vals["kv_reduction_x"]
    off = O.segment_offsets(b)
    assert off[-1] * 2 * d * 2 == O.packed_cache_bytes(b, d)


def test_compact_is_a_stable_bit_exact_gather():
    rng = np.random.default_rng(1)
    L, H, T, d = 2, 3, 50, 128
    K = rng.integers(0, 65536, (L, H, T, d)).astype(np.uint16)   # arbitrary bit patterns, NaNs included
    V = rng.integers(0, 65536, (L, H, T, d)).astype(np.uint16)
    b = np.array([[0, 50, 7], [1, 13, 25]])
    u = rng.standard_normal((L, H, T)).astype(np.float32)
    idx, off = O.select_all(u, b)
    Kp, Vp = O.compact(K, V, idx, off)
    assert Kp.shape == (b.sum(), d) and Kp.dtype == np.uint16
    r = 0
    for l in range(L):
        for h in range(H):
            for i in idx[off[l * H + h]:off[l * H + h + 1]]:
                assert Kp[r].tobytes() == K[l, h, i].tobytes()
                assert Vp[r].tobytes() == V[l, h, i].tobytes()
                r += 1
    assert r == b.sum()
    # b = T keeps the head unchanged and in order
    assert np.array_equal(Kp[off[1]:off[2]], K[0, 1])


def _kv(T, d=128, seed=0):
    rng = np.random.default_rng(seed)
    K = O.bf16_bits_to_f64(W.f32_to_bf16_bits(rng.standard_normal((T, d), dtype=np.float32)))
    V = O.bf16_bits_to_f64(W.f32_to_bf16_bits(rng.standard_normal((T, d), dtype=np.float32)))
    q = O.bf16_bits_to_f64(W.f32_to_bf16_bits(rng.standard_normal((d,), dtype=np.float32)))
    return q, K, V


SCALE = 1.0 / math.sqrt(128.0)


def test_decode_brute_force_loops():
    q, K, V = _kv(11)
    o, lse = O.decode_attn(q[None, None, :], K, V, np.array([0, 11]), H=1, scale=SCALE)
    s = [sum(q[c] * K[j, c] for c in range(128)) * SCALE for j in range(11)]
    z = sum(math.exp(x) for x in s)
    want = [sum(math.exp(s[j]) / z * V[j, c] for j in range(11)) for c in range(128)]
    assert np.allclose(o[0, 0], want, rtol=1e-12, atol=1e-14)
    assert lse[0, 0] == pytest.approx(math.log(z), rel=1e-13)


def test_decode_special_cases():
    q, K, V = _kv(40, seed=2)
    # one kept token: the output is that value row, whatever the query
    o, lse = O.decode_attn(q[None, None], K[:1], V[:1], np.array([0, 1]), 1, SCALE)
    assert np.array_equal(o[0, 0], V[0])
    assert lse[0, 0] == pytest.approx(float(K[0] @ q) * SCALE, rel=1e-14)
    # zero query: uniform weights
    o, lse = O.decode_attn(np.zeros((1, 1, 128)), K, V, np.array([0, 40]), 1, SCALE)
    assert np.allclose(o[0, 0], V.mean(axis=0), rtol=1e-13, atol=1e-15)
    assert lse[0, 0] == pytest.approx(math.log(40))
    # empty segment: zero output, lse = -inf; the neighbour is unaffected
    qq = np.stack([q, q])[None]                       # L=1, Hq=2, H=2, g=1
    o, lse = O.decode_attn(qq, K, V, np.array([0, 0, 40]), 2, SCALE)
    assert np.all(o[0, 0] == 0) and lse[0, 0] == -np.inf
    assert np.isfinite(lse[0, 1])
    # weights are a probability vector: the output lies in the per-channel hull of V
    assert np.all(o[0, 1] <= V.max(axis=0) + 1e-12) and np.all(o[0, 1] >= V.min(axis=0) - 1e-12)


def test_decode_dense_equals_torch_sdpa():
    # b = T: plain Eq. 1, which torch implements independently
    L, H, g, T, d = 2, 2, 4, 33, 128
    rng = np.random.default_rng(4)
    K = rng.standard_normal((L, H, T, d)); V = rng.standard_normal((L, H, T, d))
    q = rng.standard_normal((L, H * g, d))
    off = np.arange(L * H + 1) * T
    o, lse = O.decode_attn(q, K.reshape(-1, d), V.reshape(-1, d), off, H, SCALE)
    tq = torch.from_numpy(q)[:, :, None, :]                                   # [L, Hq, 1, d]
    tk = torch.from_numpy(K).repeat_interleave(g, dim=1)                      # contiguous groups
    tv = torch.from_numpy(V).repeat_interleave(g, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, :, 0, :].numpy()
    assert np.allclose(o, want, rtol=1e-10, atol=1e-12)
    want_lse = torch.logsumexp((tq @ tk.transpose(-1, -2))[:, :, 0, :] * SCALE, dim=-1).numpy()
    assert np.allclose(lse, want_lse, rtol=1e-12)


def test_gqa_group_shares_the_kv_head():
    L, H, g, d = 1, 2, 4, 128
    rng = np.random.default_rng(6)
    Kp = rng.standard_normal((30, d)); Vp = rng.standard_normal((30, d))
    off = np.array([0, 12, 30])
    q1 = rng.standard_normal(d)
    q = np.tile(q1, (L, H * g, 1))
    o, lse = O.decode_attn(q, Kp, Vp, off, H, SCALE)
    for hq in range(1, g):
        assert np.array_equal(o[0, hq], o[0, 0]) and np.array_equal(o[0, g + hq], o[0, g])
    assert not np.allclose(o[0, 0], o[0, g])          # the two groups read different segments
    # head 3 belongs to KV head 0, head 4 to KV head 1 (contiguous groups)
    single, _ = O.decode_attn(q1[None, None], Kp[12:], Vp[12:], np.array([0, 18]), 1, SCALE)
    assert np.allclose(o[0, 4], single[0, 0], rtol=1e-13)


@pytest.mark.parametrize("seed", range(3))
def test_compacted_attention_equals_masked_full_attention(seed):
    # App. B.2 with a 0/1 mask: renormalised masked softmax over the full cache
    T = 200
    q, K, V = _kv(T, seed=10 + seed)
    rng = np.random.default_rng(seed)
    u = rng.standard_normal(T).astype(np.float32)
    b = int(rng.integers(1, T))
    idx = O.select(u, b)
    Kp, Vp = O.compact(K[None, None], V[None, None], idx, np.array([0, b]))
    o, _ = O.decode_attn(q[None, None], Kp, Vp, np.array([0, b]), 1, SCALE)
    want = O.masked_attention_full(q, K, V, O.mask_from_indices(idx, T), SCALE)
    assert np.allclose(o[0, 0], want, rtol=1e-11, atol=1e-13)
    # and equals softmax(s + log m) with the mask as an additive bias
    with np.errstate(divide="ignore"):
        s = K @ q * SCALE + np.log(O.mask_from_indices(idx, T))
    p = np.exp(s - s.max()); p /= p.sum()
    assert np.allclose(o[0, 0], p @ V, rtol=1e-11, atol=1e-13)


def test_masked_attention_with_a_soft_mask_is_softmax_of_scores_plus_log_mask():
    # App. B.2: multiplying the exponentiated scores by m and renormalising is softmax(s + log m)
    from scipy.special import logsumexp
    rng = np.random.default_rng(42)
    T, d = 300, 128
    q = rng.standard_normal(d)
    K = rng.standard_normal((T, d))
    V = rng.standard_normal((T, d))
    m = rng.uniform(0.0, 1.0, T)
    m[::7] = 0.0
    got = O.masked_attention_full(q, K, V, m, SCALE)
    s = K @ q * SCALE
    with np.errstate(divide="ignore"):
        z = s + np.log(m)
    p = np.exp(z - logsumexp(z))
    assert np.allclose(got, p @ V, rtol=1e-12, atol=1e-14)
    assert np.all(p[::7] == 0.0)
