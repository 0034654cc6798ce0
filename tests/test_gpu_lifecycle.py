"""One sequence through its whole life on the GPU, every stage checked against the oracle:
LKV-H budgets -> layer-by-layer eviction during prefill -> packed cache with spare rows ->
decode steps that append the generated token -> re-eviction with the budgets of the longer
context -> more decode steps."""
import numpy as np
import pytest
import torch

from oracle import lkv_growth as GR
from oracle import lkv_h as OH
from oracle import lkv_oracle as O
from paper_2605_06676_amd import lkv
from paper_2605_06676_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


def test_prefill_to_decode_lifecycle():
    ctx = lkv.Context(0)
    w = W.scaled(W.CONFIGS[5], L=3, H=4, Hq=8, T=1800, hidden=128, b_min=4)     # the paper's scorer shape, small
    T, R, slack, n_seg = 1800, 0.2, 8, 3 * 4
    # 1. budgets from LKV-H
    emb, mlp = W.draw_head_predictor(w, spread=0.4)
    r_d = torch.empty(n_seg, dtype=torch.float64, device="cuda")
    b_d = torch.empty(n_seg, dtype=torch.int32, device="cuda")
    pred = {k: torch.from_numpy(np.ascontiguousarray(mlp[k], dtype=np.float32)).cuda() for k in ("w1", "b1", "w2")}
    pred["b2"] = None
    lkv.lkv_head_budgets(ctx, torch.from_numpy(emb).cuda(), pred, R, T, r_d, b_d)
    torch.cuda.synchronize()
    r_ref = OH.head_ratios(OH.head_scores(emb, mlp), R)
    budgets = b_d.cpu().numpy()
    assert np.array_equal(budgets, OH.head_budgets(r_ref, T))
    B = [budgets.reshape(w.L, w.H).astype(np.int32)]

    # 2. layer-by-layer eviction, 3. into a cache with spare rows
    K, V = W.draw_kv(w, T, 0, 9)
    Q, sc = W.draw_q(w, 0, 9), W.draw_scorer(w, 9)
    run = G.LayerwiseRun(ctx, [K], [V], [Q], sc, B, w.Hq)
    run.run_all()
    G.check_against_oracle(run, [K], [V], [Q], sc, B, "layer by layer with LKV-H budgets")
    rows = run.total + n_seg * slack
    kp = torch.zeros((rows, w.d), dtype=torch.bfloat16, device="cuda")
    vp = torch.zeros_like(kp)
    up = torch.zeros((rows,), dtype=torch.float32, device="cuda")
    cap = torch.empty((n_seg + 1,), dtype=torch.int32, device="cuda")
    ln = torch.empty((n_seg,), dtype=torch.int32, device="cuda")
    overflow = torch.zeros((1,), dtype=torch.int32, device="cuda")
    lkv.lkv_compact_grow(ctx, run.cache, run.scores, run.idx, run.offsets, run.total, slack, kp, vp, up, cap, ln)
    torch.cuda.synchronize()
    u_gpu = run.scores[0].cpu().numpy()
    idx_ref, off_ref = O.select_all(u_gpu, B[0])
    state = list(GR.compact_with_slack(K, V, u_gpu, idx_ref, off_ref, slack))

    def decode_and_check(kp, vp, cap, ln, rows, q_bits, what):
        out = torch.full((1, w.L, w.Hq, w.d), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((1, w.L, w.Hq), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.empty((max(lkv.lkv_decode_workspace_bytes(n_seg, rows, w.Hq, w.H), 256),), dtype=torch.uint8, device="cuda")
        lkv.lkv_decode_attn_grown(ctx, 1, w.L, w.H, w.Hq, w.d, G.bits_to_bf16_gpu(q_bits)[None].contiguous(), kp, vp, cap, ln,
                                  rows, G.SCALE, out, lse, ws)
        torch.cuda.synchronize()
        o_ref, lse_ref = GR.decode_grown(O.bf16_bits_to_f64(q_bits), O.bf16_bits_to_f64(state[0]), O.bf16_bits_to_f64(state[1]),
                                         state[3], state[4], w.H, G.SCALE)
        G.assert_decode_close(out[0].cpu().numpy().reshape(-1, w.d), lse[0].cpu().numpy().reshape(-1),
                              o_ref.reshape(-1, w.d), lse_ref.reshape(-1), what)

    def append(kp, vp, up, cap, ln, step):
        wn = W.scaled(w, cid=60 + step)
        kn, vn = W.draw_kv(wn, 1, 0, step)                        # [L, H, 1, d]
        kn, vn = np.ascontiguousarray(kn[:, :, 0]), np.ascontiguousarray(vn[:, :, 0])
        cap_h, ln_h = cap.cpu().numpy(), ln.cpu().numpy()
        lkv.lkv_append(ctx, 1, w.L, w.H, w.d, run.scorer, G.bits_to_bf16_gpu(kn[None]), G.bits_to_bf16_gpu(vn[None]), kp, vp, up,
                       cap, ln, overflow)
        torch.cuda.synchronize()
        u_new = up.cpu().numpy()[cap_h[:-1] + ln_h]               # the scores the GPU gave the new token
        assert not GR.append(state[0], state[1], state[2], state[3], state[4], kn.reshape(n_seg, -1), vn.reshape(n_seg, -1), u_new)

    # 4. decode steps, each appending its token
    for step in range(slack):
        decode_and_check(kp, vp, cap, ln, rows, W.draw_q(w, 0, 100 + step), f"decode step {step}")
        append(kp, vp, up, cap, ln, step)
    assert int(overflow.item()) == 0
    assert np.array_equal(ln.cpu().numpy(), budgets + slack)

    # 5. the spare rows are used up: re-evict with floor(r t') on the ratios LKV-H gave
    t2 = T + slack
    nb = np.minimum(OH.head_budgets(r_ref, t2), state[4])
    total2 = int(nb.sum())
    rows2 = total2 + n_seg * slack
    kp2 = torch.zeros((rows2, w.d), dtype=torch.bfloat16, device="cuda")
    vp2 = torch.zeros_like(kp2)
    up2 = torch.zeros((rows2,), dtype=torch.float32, device="cuda")
    cap2, ln2 = torch.empty_like(cap), torch.empty_like(ln)
    idx2 = torch.empty((max(total2, 1),), dtype=torch.int32, device="cuda")
    off2 = torch.empty((n_seg + 1,), dtype=torch.int32, device="cuda")
    assert lkv.lkv_reevict(ctx, w.d, kp, vp, up, cap, ln, state[4], nb, slack, idx2, off2, kp2, vp2, up2, cap2, ln2) == total2
    torch.cuda.synchronize()
    K2, V2, u2, c2, l2, _ = GR.reevict(state[0], state[1], state[2], state[3], state[4], nb, slack)
    state[:] = [K2, V2, u2, c2, l2]
    cap2_h = cap2.cpu().numpy()
    assert np.array_equal(cap2_h, c2) and np.array_equal(ln2.cpu().numpy(), l2)
    kb, vb, ub = G.bf16_gpu_to_bits(kp2), G.bf16_gpu_to_bits(vp2), up2.cpu().numpy()
    for s in range(n_seg):
        a, n = int(c2[s]), int(l2[s])
        assert np.array_equal(kb[a:a + n], K2[a:a + n]) and np.array_equal(vb[a:a + n], V2[a:a + n])
        assert np.array_equal(ub[a:a + n], u2[a:a + n])

    # 6. and on it goes
    for step in range(3):
        decode_and_check(kp2, vp2, cap2, ln2, rows2, W.draw_q(w, 0, 200 + step), f"after re-eviction, step {step}")
        append(kp2, vp2, up2, cap2, ln2, 50 + step)
    assert int(overflow.item()) == 0
    ctx.close()
