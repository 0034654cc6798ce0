"""The relaxed forward of one layer as LKV trains it (Sec. 3.4, 3.5), composed from library calls only:
token scores (lkv_score) -> noisy scores -> per-head soft masks m = ST_b((u + g) / tau) (lkv_soft_topk_batched) ->
causal attention with the multiplicative mask (lkv_masked_attn_forward), its backward pass, and the backward pass of
the Soft-TopK operator (lkv_soft_topk_backward_batched), which turns the mask gradient into a gradient of the scores.  Checked
against the same chain of oracle functions.  As for the hard selection, the oracle's mask is taken on the
GPU's own fp32 scores, so that the comparison is about each step, not about score rounding shifting the
threshold.  The Gumbel noise is an input (a seeded draw), added with a plain torch / numpy addition."""
import numpy as np
import pytest
import torch

from oracle import lkv_oracle as O
from oracle import masked_attn as MA
from oracle import soft_topk as ST
from paper_2605_06676_amd import lkv
from paper_2605_06676_amd import workloads as W

import gpu_util as G
from test_gpu_masked_attn import assert_rows_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = lkv.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("tau", [1.0, 0.05])
def test_relaxed_layer_forward_and_backward(ctx, tau):
    # the paper's scorer shape: one 256 -> 128 -> 1 SiLU network per head, no output bias
    w = W.scaled(W.CONFIGS[5], L=1, H=2, Hq=8, T=700, b_min=8)
    T, H, Hq = 700, w.H, w.Hq
    K, V = W.draw_kv(w, T, 0, 2)                       # uint16 [1, H, T, 128]
    sc = W.draw_scorer(w, 2)
    q, _, _, _, d_o = W.draw_training_attention(Hq, H, T, seed=9)
    rng = np.random.default_rng(21)
    gumbel = (-np.log(-np.log(rng.uniform(1e-6, 1.0 - 1e-6, size=(H, T))))).astype(np.float32) * np.float32(0.05)
    r = np.array([0.1, 0.3])                           # retention ratios of the two heads; the soft budget r t is not rounded

    # ---- GPU ----
    tk, tv = G.bits_to_bf16_gpu(K[0]), G.bits_to_bf16_gpu(V[0])
    cache = lkv.Cache([tk[None]], [tv[None]], Hq)
    scores = [torch.empty((1, H, T), dtype=torch.float32, device="cuda")]
    lkv.lkv_score(ctx, cache, G.scorer_to_gpu(sc), scores)
    noisy = scores[0][0] + torch.from_numpy(gumbel).cuda()
    m64 = torch.empty((H, T), dtype=torch.float64, device="cuda")
    st_info = torch.empty((H, 2), dtype=torch.float64, device="cuda")
    soft_budgets = torch.from_numpy(r * T).cuda()          # fp64 [H], on the device as LKV-H would leave them
    lkv.lkv_soft_topk_batched(ctx, noisy.contiguous(), soft_budgets, tau, m64, st_info)   # all heads in one launch
    m = m64.to(torch.float32)
    tq, tg = G.bits_to_bf16_gpu(q), G.bits_to_bf16_gpu(d_o)
    o = torch.empty((Hq, T, 128), dtype=torch.float32, device="cuda")
    lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
    lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, m, G.SCALE, o, lse)
    dq = torch.empty_like(o)
    dk = torch.empty((H, T, 128), dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    dm = torch.empty_like(m)
    ws = torch.empty(lkv.lkv_masked_attn_backward_workspace_bytes(Hq, H, T), dtype=torch.uint8, device="cuda")
    lkv.lkv_masked_attn_backward(ctx, tq, tk, tv, m, o, lse, tg, G.SCALE, dq, dk, dv, dm, ws)
    dm64 = dm.to(torch.float64)
    du = torch.empty((H, T), dtype=torch.float64, device="cuda")           # gradient of the noisy scores
    d_budget = torch.empty((H,), dtype=torch.float64, device="cuda")       # gradient of the soft budgets r t
    lkv.lkv_soft_topk_backward_batched(ctx, noisy.contiguous(), tau, st_info, dm64.contiguous(), du, d_budget)
    torch.cuda.synchronize()

    # ---- oracle, step by step ----
    Kf, Vf = O.bf16_bits_to_f64(K[0]), O.bf16_bits_to_f64(V[0])
    u_ref = O.score(Kf[None], Vf[None], G.scorer_to_oracle(sc))[0]
    G.assert_scores_close(scores[0][0].cpu().numpy(), u_ref, "scores")
    noisy_host = noisy.cpu().numpy()
    assert np.array_equal(noisy_host, scores[0][0].cpu().numpy() + gumbel)
    m_ref = np.stack([ST.soft_topk(noisy_host[h], float(r[h] * T), tau) for h in range(H)])
    assert np.abs(m64.cpu().numpy() - m_ref).max() <= 1e-9
    assert np.allclose(m_ref.sum(axis=1), r * T, rtol=1e-12)
    m_host = m.cpu().numpy()                            # the fp32 mask both attention routes use
    qf, gf = O.bf16_bits_to_f64(q), O.bf16_bits_to_f64(d_o)
    o_ref, lse_ref = MA.forward(qf, Kf, Vf, m_host, G.SCALE)
    G.assert_decode_close(o.cpu().numpy().reshape(-1, 128), lse.cpu().numpy().reshape(-1), o_ref.reshape(-1, 128),
                          lse_ref.reshape(-1), f"relaxed forward tau={tau}")
    rq, rk, rv, rm = MA.backward(qf, Kf, Vf, m_host, G.SCALE, gf)
    assert_rows_close(dq.cpu().numpy(), rq, "dQ")
    assert_rows_close(dk.cpu().numpy(), rk, "dK")
    assert_rows_close(dv.cpu().numpy(), rv, "dV")
    assert_rows_close(dm.cpu().numpy(), rm, "dm")
    # the Soft-TopK backward on the GPU's own mask gradient (App. A.2), per head
    dm_host = dm64.cpu().numpy()
    for h in range(H):
        du_ref, db_ref = ST.soft_topk_backward(noisy_host[h], float(r[h] * T), tau, dm_host[h])
        scale = max(1.0, float(np.abs(dm_host[h]).max()))
        assert np.abs(du[h].cpu().numpy() - du_ref).max() <= 1e-8 * scale / tau
        assert abs(float(d_budget[h]) - db_ref) <= 1e-8 * scale
