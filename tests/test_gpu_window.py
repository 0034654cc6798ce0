"""GPU parity of the observation-window scorer (lkv_score_window) against oracle/window_score.py, and of the
selection it feeds: the same seeded keys and window queries go to both sides; the scores are compared to a
tolerance, the window tokens must be +inf exactly, and the hard top-k on the GPU's own scores must be the
oracle's top-k on those scores, bit for bit.

Tolerance.  Both sides multiply the same bf16 values; the GPU accumulates the 128-term dot products and the
softmax sums in fp32 and uses the hardware exp2 / log2 (about 1 ulp).  A weight exp2(x - lse) with |x|, |lse| up
to a few tens carries a relative error of a few 1e-6 from the rounding of its exponent, the normaliser the
same, so a vote is good to about 1e-5 relative; the test asks for 1e-3 of max(|score|, rms of the head's
scores), a tenth of the 1e-2 the LKV-T scores are held to.
"""
import numpy as np
import pytest
import torch

from oracle import lkv_oracle as O
from oracle import window_score as WS
from paper_2605_06676_amd import lkv
from paper_2605_06676_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu

RTOL = 1e-3


@pytest.fixture(scope="module")
def ctx():
    c = lkv.Context(0)
    yield c
    c.close()


def run_gpu(ctx, Kbits, Qbits, Hq, window, pool, kind, scale=G.SCALE):
    """Kbits: list of uint16 [L, H, T, d]; Qbits: list of uint16 [L, Hq, window, d].  Returns the scores as numpy."""
    k = [G.bits_to_bf16_gpu(x) for x in Kbits]
    cache = lkv.Cache(k, k, Hq)                                   # the value cache is not read
    q = [G.bits_to_bf16_gpu(x) for x in Qbits]
    scores = [torch.full(x.shape[:3], float("nan"), dtype=torch.float32, device="cuda") for x in Kbits]
    ws = torch.empty(lkv.lkv_score_window_workspace_bytes(cache), dtype=torch.uint8, device="cuda")
    lkv.lkv_score_window(ctx, cache, q, window, pool, kind, scale, scores, ws)
    torch.cuda.synchronize()
    return cache, scores


def check_against_oracle(s_gpu, Kbits, Qbits, window, pool, kind, scale=G.SCALE, what=""):
    L, H, T, _ = Kbits.shape
    worst = 0.0
    for l in range(L):
        ref = WS.window_scores(O.bf16_bits_to_f64(Qbits[l]), O.bf16_bits_to_f64(Kbits[l]), scale, pool,
                               "max" if kind == lkv.POOL_MAX else "avg")
        got = s_gpu[l]
        assert np.isposinf(got[:, T - window:]).all(), f"{what}: window tokens must score +inf"
        if T > window:
            r, g = ref[:, :T - window], got[:, :T - window].astype(np.float64)
            assert np.isfinite(g).all() and (g >= 0).all(), what
            rms = np.sqrt((r ** 2).mean(axis=-1, keepdims=True))
            ratio = np.abs(g - r) / (RTOL * np.maximum(np.abs(r), rms))
            assert ratio.max() <= 1.0, f"{what}: layer {l}: worst error {ratio.max():.3g} of the tolerance"
            worst = max(worst, float(ratio.max()))
    return worst


SHAPES = [
    # L, H, Hq, T, window, pool, kind
    (2, 2, 8, 700, 32, 7, lkv.POOL_MAX),      # 128 query rows per KV head: the full fragment set, several blocks
    (1, 2, 6, 333, 5, 5, lkv.POOL_AVG),       # 15 rows: one M tile with a padding row, second wave all padding
    (1, 1, 8, 1025, 16, 1, lkv.POOL_MAX),     # group of 8, no pooling
    (2, 3, 6, 257, 40, 13, lkv.POOL_AVG),     # 80 rows: three M tiles per wave, the last half padding
    (1, 2, 2, 130, 64, 3, lkv.POOL_MAX),      # one query head per KV head, window longer than 4 tiles
    (1, 1, 4, 40, 7, 63, lkv.POOL_AVG),       # pooling wider than the prefix
    (1, 2, 4, 33, 32, 3, lkv.POOL_MAX),       # a prefix of one token
    (1, 1, 4, 32, 32, 3, lkv.POOL_MAX),       # the window is the whole prompt
    (1, 1, 1, 1, 1, 1, lkv.POOL_MAX),         # one token
    (1, 1, 16, 100, 8, 5, lkv.POOL_MAX),      # group of 16
]


@pytest.mark.parametrize("L,H,Hq,T,window,pool,kind", SHAPES)
def test_scores_match_the_oracle(ctx, L, H, Hq, T, window, pool, kind):
    w = W.scaled(W.CONFIGS[0], L=L, H=H, Hq=Hq, T=T, b_min=1)
    K, _ = W.draw_kv(w, T, 0, 3)
    Q = W.draw_window_queries(w, K, window, 0, 3)
    _, scores = run_gpu(ctx, [K], [Q], Hq, window, pool, kind)
    check_against_oracle(scores[0].cpu().numpy(), K, Q, window, pool, kind, what=f"T={T} W={window}")


def test_several_sequences_and_selection(ctx):
    # three sequences of different lengths in one call; then the hard top-k under per-head budgets
    w = W.scaled(W.CONFIGS[0], L=2, H=2, Hq=8, T=900, b_min=1)
    lens = [900, 129, 2051]
    window = 32
    Ks = [W.draw_kv(w, T, s, 4)[0] for s, T in enumerate(lens)]
    Qs = [W.draw_window_queries(w, K, window, s, 4) for s, K in enumerate(Ks)]
    cache, scores = run_gpu(ctx, Ks, Qs, w.Hq, window, 7, lkv.POOL_MAX)
    for s, T in enumerate(lens):
        check_against_oracle(scores[s].cpu().numpy(), Ks[s], Qs[s], window, 7, lkv.POOL_MAX, what=f"sequence {s}")
    rng = np.random.default_rng(5)
    budgets = np.concatenate([rng.integers(window, T // 2, size=w.L * w.H) for T in lens]).astype(np.int32)
    idx = torch.empty(int(budgets.sum()), dtype=torch.int32, device="cuda")
    offsets = torch.empty(budgets.size + 1, dtype=torch.int32, device="cuda")
    lkv.lkv_select(ctx, cache, scores, budgets, idx, offsets)
    torch.cuda.synchronize()
    idx_h, off_h = idx.cpu().numpy(), offsets.cpu().numpy()
    seg = 0
    for s, T in enumerate(lens):
        u = scores[s].cpu().numpy().reshape(-1, T)
        for lh in range(w.L * w.H):
            kept = idx_h[off_h[seg]:off_h[seg + 1]]
            assert np.array_equal(kept, O.select(u[lh], int(budgets[seg])))
            assert np.array_equal(kept[-window:], np.arange(T - window, T))       # the window survives
            seg += 1


def test_runaway_logits_move_the_references(ctx):
    # logits spread over hundreds of binary orders of magnitude, largest ones late in the prefix: the first pass
    # has to move its references many times, and the weights still have to come out right
    w = W.scaled(W.CONFIGS[0], L=1, H=2, Hq=8, T=1500, b_min=1)
    T, window = 1500, 32
    K, _ = W.draw_kv(w, T, 0, 6)
    Q = W.draw_window_queries(w, K, window, 0, 6)
    ramp = np.linspace(0.05, 3.0, T, dtype=np.float32)[None, None, :, None]
    K = W.f32_to_bf16_bits(W.bf16_bits_to_f32(K) * ramp)
    for scale in (G.SCALE * 40.0, G.SCALE * 4.0):
        _, scores = run_gpu(ctx, [K], [Q], w.Hq, window, 1, lkv.POOL_MAX, scale)
        check_against_oracle(scores[0].cpu().numpy(), K, Q, window, 1, lkv.POOL_MAX, scale, what=f"scale {scale:.3g}")


def test_reproducible_and_workspace_is_scratch(ctx):
    w = W.scaled(W.CONFIGS[0], L=1, H=2, Hq=8, T=777, b_min=1)
    K, _ = W.draw_kv(w, 777, 0, 7)
    Q = W.draw_window_queries(w, K, 32, 0, 7)
    k = G.bits_to_bf16_gpu(K)
    cache = lkv.Cache([k], [k], w.Hq)
    q = G.bits_to_bf16_gpu(Q)
    outs = []
    for fill in (0, 255):
        ws = torch.full((lkv.lkv_score_window_workspace_bytes(cache),), fill, dtype=torch.uint8, device="cuda")
        s = torch.empty((1, 2, 777), dtype=torch.float32, device="cuda")
        lkv.lkv_score_window(ctx, cache, [q], 32, 7, lkv.POOL_AVG, G.SCALE, [s], ws)
        torch.cuda.synchronize()
        outs.append(s.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


def test_argument_errors(ctx):
    w = W.scaled(W.CONFIGS[0], L=1, H=2, Hq=8, T=200, b_min=1)
    K, _ = W.draw_kv(w, 200, 0, 8)
    k = G.bits_to_bf16_gpu(K)
    cache = lkv.Cache([k], [k], w.Hq)
    q = torch.zeros((1, 8, 64, 128), dtype=torch.bfloat16, device="cuda")
    s = torch.empty((1, 2, 200), dtype=torch.float32, device="cuda")
    ws = torch.empty(lkv.lkv_score_window_workspace_bytes(cache), dtype=torch.uint8, device="cuda")

    def status(**kw):
        a = dict(window=32, pool=7, kind=lkv.POOL_MAX, scale=G.SCALE, ws=ws)
        a.update(kw)
        with pytest.raises(lkv.LkvError) as e:
            lkv.lkv_score_window(ctx, cache, [q], a["window"], a["pool"], a["kind"], a["scale"], [s], a["ws"])
        return e.value.status

    assert status(window=0) == 1
    assert status(window=201) == 1
    assert status(window=33) == 2                      # 4 x 33 query rows per KV head
    assert status(pool=4) == 1 and status(pool=65) == 1 and status(pool=0) == 1
    assert status(kind=2) == 1
    assert status(scale=0.0) == 1 and status(scale=float("inf")) == 1
    assert status(ws=None) == 3 and status(ws=ws[:ws.numel() - 256]) == 3
    assert status(ws=ws[1:]) == 3                      # misaligned
    lkv.lkv_score_window(ctx, cache, [q], 32, 7, lkv.POOL_MAX, G.SCALE, [s], ws)    # and the good call goes through
    torch.cuda.synchronize()
    want = s.clone()
    cache.c.v = None                                   # the value table is not read and may be absent
    s.fill_(float("nan"))
    lkv.lkv_score_window(ctx, cache, [q], 32, 7, lkv.POOL_MAX, G.SCALE, [s], ws)
    torch.cuda.synchronize()
    assert torch.equal(s, want)


def test_full_size_sampled_heads(ctx):
    # the 32k workload (32 layers x 8 KV heads, 32 query heads, T = 32768), window 32, in the launch configuration
    # the benchmark times: three heads against the oracle, every head against what holds at any size
    w = W.CONFIGS[1]
    T, window = 32768, 32
    k, _ = W.device_kv(w, T, 0, "cuda")
    cache = lkv.Cache([k], [k], w.Hq)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(12)
    q = torch.randn((w.L, w.Hq, window, w.d), device="cuda", generator=gen)
    # plant needles: some window rows lean towards a prefix key of their KV head
    grp = w.Hq // w.H
    for l, hq, row, j in ((0, 0, 3, 17), (5, 9, 31, 30000), (31, 31, 0, 32735), (17, 14, 8, 12345)):
        q[l, hq, row] += 0.5 * k[l, hq // grp, j].float()
    q = q.to(torch.bfloat16).contiguous()
    ws = torch.empty(lkv.lkv_score_window_workspace_bytes(cache), dtype=torch.uint8, device="cuda")
    plain = torch.empty((w.L, w.H, T), dtype=torch.float32, device="cuda")
    pooled = torch.empty_like(plain)
    lkv.lkv_score_window(ctx, cache, [q], window, 1, lkv.POOL_MAX, G.SCALE, [plain], ws)
    lkv.lkv_score_window(ctx, cache, [q], window, 7, lkv.POOL_MAX, G.SCALE, [pooled], ws)
    torch.cuda.synchronize()
    # any size: +inf exactly on the window; unpooled votes are non-negative and a head cannot hand out more than the
    # W units of attention mass its window rows have; max pooling never lowers a score and is the max of 7 neighbours
    assert torch.isposinf(plain[:, :, T - window:]).all() and torch.isposinf(pooled[:, :, T - window:]).all()
    v = plain[:, :, :T - window]
    assert torch.isfinite(v).all() and (v >= 0).all()
    mass = v.double().sum(-1)
    assert (mass <= window * (1 + 1e-4)).all() and (mass > 0).all()
    ref_pool = torch.nn.functional.max_pool1d(v.reshape(1, -1, T - window), 7, stride=1, padding=3).reshape(v.shape)
    assert torch.equal(pooled[:, :, :T - window], ref_pool)
    for l, h in ((0, 0), (5, 2), (31, 7)):
        Kb = G.bf16_gpu_to_bits(k[l, h])[None, None]
        Qb = G.bf16_gpu_to_bits(q[l, h * grp:(h + 1) * grp])[None]
        check_against_oracle(pooled[l, h][None, None].cpu().numpy(), Kb, Qb, window, 7, lkv.POOL_MAX, what=f"layer {l} head {h}")
        check_against_oracle(plain[l, h][None, None].cpu().numpy(), Kb, Qb, window, 1, lkv.POOL_MAX, what=f"layer {l} head {h}, unpooled")


def test_more_sequences_than_one_launch_table_holds(ctx):
    # 35 short sequences of different lengths: the call splits them over two launch tables and walks the workspace on
    w = W.scaled(W.CONFIGS[0], L=1, H=2, Hq=4, T=64, b_min=1)
    rng = np.random.default_rng(9)
    lens = [int(t) for t in rng.integers(9, 140, size=35)]
    window = 8
    Ks = [W.draw_kv(w, T, s, 9)[0] for s, T in enumerate(lens)]
    Qs = [W.draw_window_queries(w, K, window, s, 9) for s, K in enumerate(Ks)]
    _, scores = run_gpu(ctx, Ks, Qs, w.Hq, window, 3, lkv.POOL_AVG)
    for s in range(len(lens)):
        check_against_oracle(scores[s].cpu().numpy(), Ks[s], Qs[s], window, 3, lkv.POOL_AVG, what=f"sequence {s}")


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes(ctx, seed):
    # groups, windows, lengths, pooling and logit scales drawn at random; now and then the window is the whole prompt
    rng = np.random.default_rng(500 + seed)
    L, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    g = int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
    window = int(rng.integers(1, 128 // g + 1))
    n_seq = int(rng.integers(1, 4))
    Ts = [int(rng.integers(window, 3000)) for _ in range(n_seq)]
    if rng.random() < 0.15:
        Ts[0] = window
    pool, kind = int(rng.choice([1, 3, 5, 7, 9, 13, 31, 63])), int(rng.integers(0, 2))
    scale = G.SCALE * float(rng.choice([1.0, 1.0, 3.0, 12.0]))
    w = W.scaled(W.CONFIGS[0], L=L, H=H, Hq=H * g, n_seq=n_seq, T=64, b_min=1)
    Ks = [W.draw_kv(w, T, s, seed)[0] for s, T in enumerate(Ts)]
    Qs = [W.draw_window_queries(w, K, window, s, seed) for s, K in enumerate(Ks)]
    _, scores = run_gpu(ctx, Ks, Qs, w.Hq, window, pool, kind, scale)
    for s in range(n_seq):
        check_against_oracle(scores[s].cpu().numpy(), Ks[s], Qs[s], window, pool, kind, scale, what=f"random {seed}, sequence {s}")


def test_layer_by_layer_eviction_with_window_scores(ctx):
    # the prefill-time flow with this scorer: per layer, score the layer view, then lkv_evict_layer without a scorer
    # (top-k and compaction of given scores); the packed cache must equal what the whole-cache top-k and compaction
    # make of the same scores, bit for bit
    w = W.scaled(W.CONFIGS[0], L=3, H=2, Hq=8, T=64, b_min=1)
    lens, window = [1500, 260], 32
    Ks, Vs = zip(*[W.draw_kv(w, T, s, 13) for s, T in enumerate(lens)])
    Qs = [W.draw_window_queries(w, K, window, s, 13) for s, K in enumerate(Ks)]
    tk, tv = [G.bits_to_bf16_gpu(x) for x in Ks], [G.bits_to_bf16_gpu(x) for x in Vs]
    tq = [G.bits_to_bf16_gpu(x) for x in Qs]
    rng = np.random.default_rng(13)
    budgets = np.concatenate([rng.integers(window, T // 2, size=w.L * w.H) for T in lens]).astype(np.int32)
    total = int(budgets.sum())
    n_seg = budgets.size

    def buffers():
        return (torch.full((total,), -1, dtype=torch.int32, device="cuda"), torch.full((n_seg + 1,), -1, dtype=torch.int32, device="cuda"),
                torch.zeros((total, 128), dtype=torch.bfloat16, device="cuda"), torch.zeros((total, 128), dtype=torch.bfloat16, device="cuda"))

    cache = lkv.Cache(tk, tv, w.Hq)
    whole_scores = [torch.empty((w.L, w.H, T), dtype=torch.float32, device="cuda") for T in lens]
    ws = torch.empty(lkv.lkv_score_window_workspace_bytes(cache), dtype=torch.uint8, device="cuda")
    lkv.lkv_score_window(ctx, cache, tq, window, 7, lkv.POOL_MAX, G.SCALE, whole_scores, ws)
    # layer by layer, in some order
    idx2, offsets2, kp2, vp2 = buffers()
    assert lkv.lkv_plan_offsets(ctx, budgets, offsets2) == total
    layer_scores = [torch.empty((w.H, T), dtype=torch.float32, device="cuda") for T in lens]
    scores = [torch.empty((w.L, w.H, T), dtype=torch.float32, device="cuda") for T in lens]
    for l in (2, 0, 1):
        view = lkv.Cache([k[l:l + 1] for k in tk], [v[l:l + 1] for v in tv], w.Hq)
        lkv.lkv_score_window(ctx, view, [q[l:l + 1].contiguous() for q in tq], window, 7, lkv.POOL_MAX, G.SCALE,
                             [s[None] for s in layer_scores], ws)
        lkv.lkv_evict_layer(ctx, view, l, w.L, None, budgets, offsets2, layer_scores, idx2, kp2, vp2)
        torch.cuda.synchronize()
        for s in range(len(lens)):
            scores[s][l].copy_(layer_scores[s])
            # a launch over one layer may split the keys into other blocks than a launch over all of them, which
            # changes the order of the fp32 sums and nothing else
            pre = slice(0, lens[s] - window)
            assert torch.allclose(layer_scores[s][:, pre], whole_scores[s][l][:, pre], rtol=1e-5, atol=1e-9)
    # the whole-cache top-k and compaction of the same scores
    idx, offsets, kp, vp = buffers()
    lkv.lkv_select(ctx, cache, scores, budgets, idx, offsets)
    lkv.lkv_compact(ctx, cache, idx, offsets, total, kp, vp)
    torch.cuda.synchronize()
    assert torch.equal(offsets2, offsets) and torch.equal(idx2, idx)
    assert torch.equal(kp2.view(torch.int16), kp.view(torch.int16)) and torch.equal(vp2.view(torch.int16), vp.view(torch.int16))


@pytest.mark.parametrize("L,H,Hq,T,window,pool,kind", [(2, 2, 8, 1700, 32, 7, lkv.POOL_MAX), (1, 3, 6, 333, 20, 5, lkv.POOL_AVG),
                                                     (1, 1, 4, 32, 32, 3, lkv.POOL_MAX)])
def test_with_the_callers_log_normalisers(ctx, L, H, Hq, T, window, pool, kind):
    # the prefill's attention kernel has the normalisers of the window rows already: given them, the call reads the
    # keys once and must give the scores of the two-pass route to the rounding of the normalisers (fp32 here)
    w = W.scaled(W.CONFIGS[0], L=L, H=H, Hq=Hq, T=T, b_min=1)
    K, _ = W.draw_kv(w, T, 0, 21)
    Q = W.draw_window_queries(w, K, window, 0, 21)
    lse = np.stack([WS.window_log_normalisers(O.bf16_bits_to_f64(Q[l]), O.bf16_bits_to_f64(K[l]), G.SCALE) for l in range(L)])
    k = G.bits_to_bf16_gpu(K)
    cache = lkv.Cache([k], [k], Hq)
    q = G.bits_to_bf16_gpu(Q)
    ws = torch.empty(lkv.lkv_score_window_workspace_bytes(cache), dtype=torch.uint8, device="cuda")
    two_pass = torch.empty((L, H, T), dtype=torch.float32, device="cuda")
    one_pass = torch.full((L, H, T), float("nan"), dtype=torch.float32, device="cuda")
    lkv.lkv_score_window(ctx, cache, [q], window, pool, kind, G.SCALE, [two_pass], ws)
    ws.fill_(255)                                          # nothing of the first call may be needed
    lkv.lkv_score_window(ctx, cache, [q], window, pool, kind, G.SCALE, [one_pass], ws,
                         lse_win=[torch.from_numpy(lse.astype(np.float32)).cuda()])
    torch.cuda.synchronize()
    check_against_oracle(one_pass.cpu().numpy(), K, Q, window, pool, kind, what="with given normalisers")
    pre = slice(0, T - window)
    assert torch.allclose(one_pass[:, :, pre], two_pass[:, :, pre], rtol=2e-5, atol=1e-12)
    assert torch.isposinf(one_pass[:, :, T - window:]).all()


def test_normalisers_from_the_attention_kernel(ctx):
    # the chain a serving engine would run: causal attention over the prompt (here lkv_masked_attn_forward with
    # m = 1) returns the log-normaliser of every query; those of the last W queries feed the window scorer
    Hq, H, T, window = 8, 2, 900, 32
    q, k, v, _, _ = W.draw_training_attention(Hq, H, T, seed=31)
    tq, tk, tv = (G.bits_to_bf16_gpu(x) for x in (q, k, v))
    ones = torch.ones((H, T), dtype=torch.float32, device="cuda")
    o = torch.empty((Hq, T, 128), dtype=torch.float32, device="cuda")
    lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
    lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, ones, G.SCALE, o, lse)
    cache = lkv.Cache([tk[None]], [tv[None]], Hq)
    q_win = tq[:, T - window:].contiguous()[None]                      # [1, Hq, W, 128]
    lse_win = lse[:, T - window:].contiguous()[None]                   # [1, Hq, W]
    ws = torch.empty(lkv.lkv_score_window_workspace_bytes(cache), dtype=torch.uint8, device="cuda")
    s = torch.empty((1, H, T), dtype=torch.float32, device="cuda")
    lkv.lkv_score_window(ctx, cache, [q_win], window, 7, lkv.POOL_MAX, G.SCALE, [s], ws, lse_win=[lse_win])
    torch.cuda.synchronize()
    check_against_oracle(s.cpu().numpy(), k[None], q[:, T - window:][None], window, 7, lkv.POOL_MAX, what="normalisers from attention")


def test_long_context_sampled_heads(ctx):
    # 131072 tokens per head (the length of the second benchmark workload; four layers of it), 128 blocks per head
    # and pass: two heads against the oracle, with and without the caller's normalisers
    w = W.scaled(W.CONFIGS[2], L=4)
    T, window = 131072, 32
    k, _ = W.device_kv(w, T, 0, "cuda")
    cache = lkv.Cache([k], [k], w.Hq)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(14)
    q = torch.randn((w.L, w.Hq, window, w.d), device="cuda", generator=gen)
    grp = w.Hq // w.H
    q[1, 5, 7] += 0.5 * k[1, 5 // grp, 100000].float()
    q[3, 30, 31] += 0.5 * k[3, 30 // grp, 7].float()
    q = q.to(torch.bfloat16).contiguous()
    ws = torch.empty(lkv.lkv_score_window_workspace_bytes(cache), dtype=torch.uint8, device="cuda")
    s = torch.empty((w.L, w.H, T), dtype=torch.float32, device="cuda")
    lkv.lkv_score_window(ctx, cache, [q], window, 7, lkv.POOL_AVG, G.SCALE, [s], ws)
    torch.cuda.synchronize()
    assert torch.isposinf(s[:, :, T - window:]).all() and torch.isfinite(s[:, :, :T - window]).all()
    lse = torch.zeros((w.L, w.Hq, window), dtype=torch.float32, device="cuda")
    picks = ((1, 5 // grp), (3, 30 // grp))
    for l, h in picks:
        Kb = G.bf16_gpu_to_bits(k[l, h])[None, None]
        Qb = G.bf16_gpu_to_bits(q[l, h * grp:(h + 1) * grp])[None]
        check_against_oracle(s[l, h][None, None].cpu().numpy(), Kb, Qb, window, 7, lkv.POOL_AVG, what=f"layer {l} head {h}")
        ref_lse = WS.window_log_normalisers(O.bf16_bits_to_f64(Qb[0]), O.bf16_bits_to_f64(Kb[0]), G.SCALE)
        lse[l, h * grp:(h + 1) * grp] = torch.from_numpy(ref_lse.astype(np.float32)).cuda()
    one = torch.empty_like(s)
    lkv.lkv_score_window(ctx, cache, [q], window, 7, lkv.POOL_AVG, G.SCALE, [one], ws, lse_win=[lse])
    torch.cuda.synchronize()
    for l, h in picks:      # only these heads were given true normalisers
        Kb = G.bf16_gpu_to_bits(k[l, h])[None, None]
        Qb = G.bf16_gpu_to_bits(q[l, h * grp:(h + 1) * grp])[None]
        check_against_oracle(one[l, h][None, None].cpu().numpy(), Kb, Qb, window, 7, lkv.POOL_AVG, what=f"layer {l} head {h}, given normalisers")
