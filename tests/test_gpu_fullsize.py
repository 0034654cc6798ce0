"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The whole workload is generated on the GPU and run through the four calls exactly as in
bench.py.  The oracle cannot redo tens of millions of rows in test time, so it recomputes a
sample: whole (layer, head) segments -- the first and last layer plus the heads with the
smallest and the largest budget -- copied back to the host, so both sides see identical bytes.
For every sampled head the scores are compared to the stated tolerance, the kept indices and
the packed rows must match bit for bit (selection on the GPU's own scores), and the decode
output of its query heads must match to the stated tolerance.  Properties that hold at any
size are checked over the whole output: offsets, index ranges and order, finite outputs.
"""

import numpy as np
import pytest
import torch

from oracle import lkv_oracle as O
from paper_2605_06676_amd import lkv
from paper_2605_06676_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _run_full(w):
    dev = torch.device("cuda:0")
    ctx = lkv.Context(0)
    Ts = [int(t) for t in W.seq_lengths(w)]
    Ks, Vs = [], []
    for s, T in enumerate(Ts):
        k, v = W.device_kv(w, T, s, dev)
        Ks.append(k); Vs.append(v)
    cache = lkv.Cache(Ks, Vs, w.Hq)
    sc = W.draw_scorer(w)
    scorer = G.scorer_to_gpu(sc)
    budgets = [W.draw_budgets(w, T, s) for s, T in enumerate(Ts)]
    flat = np.concatenate([b.reshape(-1) for b in budgets]).astype(np.int32)
    total = int(flat.sum())
    scores = [torch.empty((w.L, w.H, T), dtype=torch.float32, device=dev) for T in Ts]
    idx = torch.empty((total,), dtype=torch.int32, device=dev)
    offsets = torch.empty((cache.n_segments + 1,), dtype=torch.int32, device=dev)
    kp = torch.empty((total, w.d), dtype=torch.bfloat16, device=dev)
    vp = torch.empty_like(kp)
    qbits = [W.draw_q(w, s) for s in range(w.n_seq)]
    q = torch.stack([G.bits_to_bf16_gpu(x) for x in qbits]).contiguous()
    out = torch.full((w.n_seq, w.L, w.Hq, w.d), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((w.n_seq, w.L, w.Hq), float("nan"), dtype=torch.float32, device=dev)
    ws = torch.empty((lkv.lkv_decode_workspace_bytes(cache.n_segments, total, w.Hq, w.H),), dtype=torch.uint8, device=dev)
    lkv.lkv_score(ctx, cache, scorer, scores)
    lkv.lkv_select(ctx, cache, scores, flat, idx, offsets)
    lkv.lkv_compact(ctx, cache, idx, offsets, total, kp, vp)
    lkv.lkv_decode_attn(ctx, w.n_seq, w.L, w.H, w.Hq, w.d, q, kp, vp, offsets, total, G.SCALE, out, lse, ws)
    torch.cuda.synchronize()
    return dict(w=w, Ts=Ts, Ks=Ks, Vs=Vs, sc=sc, budgets=budgets, flat=flat, total=total, scores=scores, idx=idx,
                offsets=offsets, kp=kp, vp=vp, qbits=qbits, out=out, lse=lse, ctx=ctx)


def _check_global_properties(r):
    w = r["w"]
    off = r["offsets"].cpu().numpy().astype(np.int64)
    assert np.array_equal(off, np.concatenate([[0], np.cumsum(r["flat"].astype(np.int64))]))
    idx = r["idx"]
    # indices inside every segment are strictly ascending and inside [0, T)
    seg_T = np.repeat(np.asarray(r["Ts"]), w.L * w.H)
    assert int(idx.min()) >= 0
    d = (idx[1:] - idx[:-1]).cpu().numpy()
    starts = off[1:-1]
    inner = np.ones(d.size, dtype=bool)
    inner[starts[(starts > 0) & (starts < idx.numel())] - 1] = False
    assert np.all(d[inner] > 0)
    last = idx.cpu().numpy()[np.maximum(off[1:] - 1, 0)]
    assert np.all((last < seg_T) | (r["flat"] == 0))
    assert bool(torch.isfinite(r["out"]).all())
    assert bool(torch.isfinite(r["lse"]).all()) or (r["flat"] == 0).any()
    assert r["total"] / sum(w.L * w.H * T for T in r["Ts"]) <= w.R


def _check_sampled_heads(r, seq, heads):
    w = r["w"]
    T = r["Ts"][seq]
    off = r["offsets"].cpu().numpy().astype(np.int64)
    sc_o = G.scorer_to_oracle(r["sc"])
    Hs = r["sc"]["w1"].shape[1]
    worst_s = worst_d = 0.0
    inter = union = 0
    for (l, h) in heads:
        seg = (seq * w.L + l) * w.H + h
        Kb = _bits(r["Ks"][seq][l, h])[None, None]          # [1, 1, T, d]
        Vb = _bits(r["Vs"][seq][l, h])[None, None]
        hs = h if Hs == w.H else 0
        one = {"kind": sc_o["kind"], "act": sc_o["act"], "w1": sc_o["w1"][l:l + 1, hs:hs + 1],
               "b1": sc_o["b1"][l:l + 1, hs:hs + 1],
               "w2": None if sc_o["w2"] is None else sc_o["w2"][l:l + 1, hs:hs + 1],
               "b2": None if sc_o["b2"] is None else sc_o["b2"][l:l + 1, hs:hs + 1]}
        u_ref = O.score(O.bf16_bits_to_f64(Kb), O.bf16_bits_to_f64(Vb), one)[0, 0]
        u_gpu = r["scores"][seq][l, h].cpu().numpy()
        worst_s = max(worst_s, G.assert_scores_close(u_gpu[None], u_ref[None], f"seq {seq} layer {l} head {h}"))
        b = int(r["budgets"][seq][l, h])
        idx_ref = O.select(u_gpu, b)
        lo, hi = int(off[seg]), int(off[seg + 1])
        assert hi - lo == b
        assert np.array_equal(r["idx"][lo:hi].cpu().numpy(), idx_ref), f"indices of segment {seg}"
        # informative, not gating: how far the kept set moves when the oracle ranks its own scores instead of
        # the GPU's (tokens within rounding distance of the threshold can change sides)
        idx_own = O.select(u_ref, b)
        inter += np.intersect1d(idx_ref, idx_own, assume_unique=True).size
        union += np.union1d(idx_ref, idx_own).size
        Kp_ref, Vp_ref = O.compact(Kb, Vb, idx_ref, np.array([0, b]))
        assert np.array_equal(_bits(r["kp"][lo:hi]), Kp_ref), f"packed K of segment {seg}"
        assert np.array_equal(_bits(r["vp"][lo:hi]), Vp_ref), f"packed V of segment {seg}"
        g = w.g
        qh = O.bf16_bits_to_f64(r["qbits"][seq][l, h * g:(h + 1) * g])[None]      # [1, g, d]
        o_ref, lse_ref = O.decode_attn(qh, O.bf16_bits_to_f64(Kp_ref), O.bf16_bits_to_f64(Vp_ref),
                                       np.array([0, b]), 1, G.SCALE)
        o_gpu = r["out"][seq, l, h * g:(h + 1) * g].cpu().numpy()
        lse_gpu = r["lse"][seq, l, h * g:(h + 1) * g].cpu().numpy()
        worst_d = max(worst_d, G.assert_decode_close(o_gpu, lse_gpu, o_ref[0], lse_ref[0], f"decode of segment {seg}"))
    r.setdefault("overlap", [0, 0])
    r["overlap"][0] += inter
    r["overlap"][1] += union
    return worst_s, worst_d


def _report_overlap(r, what):
    inter, union = r["overlap"]
    print(f"{what}: selection on GPU scores vs selection on oracle scores, sampled heads: Jaccard overlap "
          f"{inter / max(union, 1):.6f} ({union - inter} of {union} kept tokens differ)")


def _sample(r, seq, n_layers_sample=2):
    w = r["w"]
    b = r["budgets"][seq]
    heads = {(0, h) for h in range(w.H)} | {(w.L - 1, h) for h in range(w.H)}
    lmin, hmin = np.unravel_index(np.argmin(b), b.shape)
    lmax, hmax = np.unravel_index(np.argmax(b), b.shape)
    heads |= {(int(lmin), int(hmin)), (int(lmax), int(hmax)), (w.L // 2, 0)}
    return sorted(heads)


# 5 and 6: the paper's own scorer shape (one 256 -> 128 -> 1 SiLU network per head) on its two model shapes
# (32 x 8 and 36 x 8 KV heads: 256 and 288 scorers, Table 5)
@pytest.mark.parametrize("cid", [1, 2, 5, 6])
def test_full_size_single_sequence(cid):
    w = W.CONFIGS[cid]
    r = _run_full(w)
    _check_global_properties(r)
    ws, wd = _check_sampled_heads(r, 0, _sample(r, 0))
    print(f"cfg{cid}: kept {r['total']}, worst score error {ws:.3g} x tol, worst decode error {wd:.3g} x tol")
    _report_overlap(r, w.name)
    r["ctx"].close()


def test_full_size_batched_heterogeneous():
    w = W.CONFIGS[3]
    r = _run_full(w)
    _check_global_properties(r)
    for seq in (0, w.n_seq - 1, int(np.argmin(r["Ts"])), int(np.argmax(r["Ts"]))):
        b = r["budgets"][seq]
        lmax, hmax = np.unravel_index(np.argmax(b), b.shape)
        _check_sampled_heads(r, seq, [(0, 0), (w.L - 1, w.H - 1), (int(lmax), int(hmax))])
    _report_overlap(r, w.name)
    r["ctx"].close()


def test_full_size_group7_shared_budgets():
    w = W.CONFIGS[4]
    r = _run_full(w)
    _check_global_properties(r)
    b = r["budgets"][0]
    assert int(b.max()) == w.T      # at least one head keeps everything: the b = T path at full size
    lmax, hmax = np.unravel_index(np.argmax(b), b.shape)
    lmin, hmin = np.unravel_index(np.argmin(b), b.shape)
    for seq in (0, w.n_seq - 1):
        _check_sampled_heads(r, seq, [(0, 0), (int(lmax), int(hmax)), (int(lmin), int(hmin)), (w.L - 1, w.H - 1)])
    _report_overlap(r, w.name)
    r["ctx"].close()


def test_full_size_growth_and_reeviction():
    """Workload 1 with 128 spare rows per segment: three generated tokens are appended, the decode
    reads the rows in use, then the cache is re-evicted with the budgets floor(r t') of the longer
    context.  Sampled heads are rebuilt by the oracle from the same bytes."""
    from oracle import lkv_growth as GR

    w = W.CONFIGS[1]
    r = _run_full(w)
    ctx, dev = r["ctx"], torch.device("cuda:0")
    T, n_seg, slack, n_new = r["Ts"][0], w.L * w.H, 128, 3
    cache = lkv.Cache(r["Ks"], r["Vs"], w.Hq)
    rows = r["total"] + n_seg * slack
    kp = torch.zeros((rows, w.d), dtype=torch.bfloat16, device=dev)
    vp = torch.zeros_like(kp)
    up = torch.zeros((rows,), dtype=torch.float32, device=dev)
    cap = torch.empty((n_seg + 1,), dtype=torch.int32, device=dev)
    ln = torch.empty((n_seg,), dtype=torch.int32, device=dev)
    overflow = torch.zeros((1,), dtype=torch.int32, device=dev)
    scorer = G.scorer_to_gpu(r["sc"])
    lkv.lkv_compact_grow(ctx, cache, r["scores"], r["idx"], r["offsets"], r["total"], slack, kp, vp, up, cap, ln)
    gen = torch.Generator(device=dev); gen.manual_seed(123)
    new_k = [torch.randn((1, w.L, w.H, w.d), device=dev, generator=gen).to(torch.bfloat16) for _ in range(n_new)]
    new_v = [torch.randn((1, w.L, w.H, w.d), device=dev, generator=gen).to(torch.bfloat16) for _ in range(n_new)]
    for kn, vn in zip(new_k, new_v):
        lkv.lkv_append(ctx, 1, w.L, w.H, w.d, scorer, kn, vn, kp, vp, up, cap, ln, overflow)
    q = torch.stack([G.bits_to_bf16_gpu(x) for x in r["qbits"]]).contiguous()
    out = torch.full((1, w.L, w.Hq, w.d), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((1, w.L, w.Hq), float("nan"), dtype=torch.float32, device=dev)
    ws = torch.empty((lkv.lkv_decode_workspace_bytes(n_seg, rows, w.Hq, w.H),), dtype=torch.uint8, device=dev)
    lkv.lkv_decode_attn_grown(ctx, 1, w.L, w.H, w.Hq, w.d, q, kp, vp, cap, ln, rows, G.SCALE, out, lse, ws)
    torch.cuda.synchronize()
    assert int(overflow.item()) == 0
    cap_h, len_h = cap.cpu().numpy().astype(np.int64), ln.cpu().numpy().astype(np.int64)
    assert np.array_equal(len_h, r["flat"] + n_new)
    assert np.array_equal(cap_h, np.concatenate([[0], np.cumsum(r["flat"].astype(np.int64) + slack)]))
    assert bool(torch.isfinite(out).all())

    # re-eviction with the budgets of the longer context
    ratios = r["flat"].astype(np.float64) / T
    nb = np.minimum(np.floor(ratios * (T + n_new)).astype(np.int64), len_h)
    total2 = int(nb.sum())
    rows2 = total2 + n_seg * slack
    kp2 = torch.zeros((rows2, w.d), dtype=torch.bfloat16, device=dev)
    vp2 = torch.zeros_like(kp2)
    up2 = torch.zeros((rows2,), dtype=torch.float32, device=dev)
    cap2 = torch.empty_like(cap); len2 = torch.empty_like(ln)
    idx2 = torch.empty((total2,), dtype=torch.int32, device=dev)
    off2 = torch.empty((n_seg + 1,), dtype=torch.int32, device=dev)
    assert lkv.lkv_reevict(ctx, w.d, kp, vp, up, cap, ln, len_h, nb, slack, idx2, off2, kp2, vp2, up2, cap2, len2) == total2
    torch.cuda.synchronize()
    cap2_h = cap2.cpu().numpy().astype(np.int64)
    assert np.array_equal(len2.cpu().numpy(), nb)

    sc_o = G.scorer_to_oracle(r["sc"])
    off = r["offsets"].cpu().numpy().astype(np.int64)
    for (l, h) in _sample(r, 0):
        seg = l * w.H + h
        a, n = int(cap_h[seg]), int(len_h[seg])
        b = int(r["flat"][seg])
        # rows in use: the kept prefill rows (bit for bit, checked against the tight cache) then the new tokens
        assert torch.equal(kp[a:a + b].view(torch.int16), r["kp"][off[seg]:off[seg + 1]].view(torch.int16))
        assert torch.equal(vp[a:a + b].view(torch.int16), r["vp"][off[seg]:off[seg + 1]].view(torch.int16))
        u_head = r["scores"][0][l, h]
        assert torch.equal(up[a:a + b], u_head[r["idx"][off[seg]:off[seg + 1]].long()])
        one = {"kind": sc_o["kind"], "act": sc_o["act"], "w1": sc_o["w1"][l:l + 1, 0:1], "b1": sc_o["b1"][l:l + 1, 0:1],
               "w2": None, "b2": None}
        rms = float(u_head.double().pow(2).mean().sqrt())
        for j in range(n_new):
            assert torch.equal(kp[a + b + j].view(torch.int16), new_k[j][0, l, h].view(torch.int16))
            assert torch.equal(vp[a + b + j].view(torch.int16), new_v[j][0, l, h].view(torch.int16))
            u_ref = O.score(O.bf16_bits_to_f64(_bits(new_k[j][0, l, h]))[None, None, None],
                            O.bf16_bits_to_f64(_bits(new_v[j][0, l, h]))[None, None, None], one)[0, 0, 0]
            assert abs(float(up[a + b + j]) - float(u_ref)) <= G.SCORE_RTOL * max(abs(float(u_ref)), rms)
        # decode over the rows in use
        Kh, Vh = _bits(kp[a:a + n]), _bits(vp[a:a + n])
        g = w.g
        qh = O.bf16_bits_to_f64(r["qbits"][0][l, h * g:(h + 1) * g])[None]
        o_ref, lse_ref = O.decode_attn(qh, O.bf16_bits_to_f64(Kh), O.bf16_bits_to_f64(Vh), np.array([0, n]), 1, G.SCALE)
        G.assert_decode_close(out[0, l, h * g:(h + 1) * g].cpu().numpy(), lse[0, l, h * g:(h + 1) * g].cpu().numpy(),
                              o_ref[0], lse_ref[0], f"grown decode of segment {seg}")
        # re-eviction of this segment, by the oracle, on the scores the GPU holds
        u_held = up[a:a + n].cpu().numpy()
        K2, V2, u2, c2, l2, pos = GR.reevict(Kh, Vh, u_held, np.array([0, n]), np.array([n]), np.array([nb[seg]]), 0)
        a2 = int(cap2_h[seg])
        assert np.array_equal(_bits(kp2[a2:a2 + nb[seg]]), K2), f"re-evicted K of segment {seg}"
        assert np.array_equal(_bits(vp2[a2:a2 + nb[seg]]), V2), f"re-evicted V of segment {seg}"
        assert np.array_equal(up2[a2:a2 + nb[seg]].cpu().numpy(), u2), f"re-evicted scores of segment {seg}"
    ctx.close()


def test_full_size_masked_attention_identity():
    """App. B.2 at full size: attention over the whole 4.3 GB cache with the 0/1 retention mask must
    give, for every query head, what the decode over the compacted cache gives (a property that
    holds at any size; both routes are GPU results, the oracle checks sampled heads of each)."""
    w = W.CONFIGS[1]
    r = _run_full(w)
    ctx, dev = r["ctx"], torch.device("cuda:0")
    T = r["Ts"][0]
    cache = lkv.Cache(r["Ks"], r["Vs"], w.Hq)
    seg_of_row = torch.repeat_interleave(torch.arange(w.L * w.H, device=dev),
                                         torch.from_numpy(r["flat"].astype(np.int64)).to(dev))
    mask = torch.zeros((w.L * w.H * T,), dtype=torch.float32, device=dev)
    mask[seg_of_row * T + r["idx"].long()] = 1.0
    assert int(mask.sum().item()) == r["total"]
    q = torch.stack([G.bits_to_bf16_gpu(x) for x in r["qbits"]]).contiguous()
    out = torch.full((1, w.L, w.Hq, w.d), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((1, w.L, w.Hq), float("nan"), dtype=torch.float32, device=dev)
    ws = torch.empty((lkv.lkv_masked_decode_workspace_bytes(cache),), dtype=torch.uint8, device=dev)
    lkv.lkv_masked_decode_attn(ctx, cache, q, [mask.view(w.L, w.H, T)], G.SCALE, out, lse, ws)
    torch.cuda.synchronize()
    a, b = out.double(), r["out"].double()
    scale = torch.maximum(b.abs().amax(dim=-1), b.pow(2).mean(dim=-1).sqrt())
    err = (a - b).abs().amax(dim=-1)
    # each route is within DECODE_RTOL of the exact result, so two routes are within twice that of each other
    assert bool((err <= 2 * G.DECODE_RTOL * scale).all()), f"worst {(err / scale).max().item():.3g}"
    assert bool(((lse.double() - r["lse"].double()).abs() <= 2 * G.LSE_ATOL).all())
    print(f"masked vs compacted decode over {w.L * w.Hq} query heads: worst relative difference {(err / scale).max().item():.3g}")
    ctx.close()
