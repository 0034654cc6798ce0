"""The hot calls only enqueue kernels on the caller's stream, so a step can be captured into a HIP
graph and replayed: every replay must reproduce the eager result (replays are interleaved with
eager work and synchronisations, as a serving loop would)."""
import numpy as np
import pytest
import torch

from paper_2605_06676_amd import lkv
from paper_2605_06676_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = lkv.Context(0)
    yield c
    c.close()


def test_captured_step_replays_to_the_eager_result(ctx):
    w = W.scaled(W.CONFIGS[0], L=4, H=4, Hq=16, b_min=8)      # 16 segments: offsets ride in the kernel arguments
    T = 3000
    K, V = W.draw_kv(w, T, 0, 1)
    Q, sc, B = W.draw_q(w, 0, 1), W.draw_scorer(w, 1), W.draw_budgets(w, T, 0, 1)
    run = G.GpuRun(ctx, [K], [V], [Q], sc, [B], w.Hq)
    run.run_all()
    G.check_against_oracle(run, [K], [V], [Q], sc, [B], "eager")
    want = {k: getattr(run, k).clone() for k in ("idx", "offsets", "kp", "vp", "out", "lse")}
    want_scores = run.scores[0].clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run.score(); run.select(); run.compact(); run.decode()      # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run.score(); run.select(); run.compact(); run.decode()
    torch.cuda.synchronize()
    for rep in range(4):
        # eager work between replays: scribble over every output, then replay
        for k in want:
            getattr(run, k).fill_(-3 if getattr(run, k).dtype == torch.int32 else float("nan"))
        run.scores[0].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(run.scores[0], want_scores), f"replay {rep}: scores"
        for k in ("idx", "offsets"):
            assert torch.equal(getattr(run, k), want[k]), f"replay {rep}: {k}"
        for k in ("kp", "vp"):
            assert torch.equal(getattr(run, k).view(torch.int16), want[k].view(torch.int16)), f"replay {rep}: {k}"
        for k in ("out", "lse"):
            assert torch.equal(getattr(run, k), want[k]), f"replay {rep}: {k}"


def test_captured_training_attention_replays_to_the_eager_result(ctx):
    # forward and backward of the training-time attention only enqueue kernels: captured, every replay
    # must give the bits of the eager run (the backward pass has no atomics)
    Hq, H, T = 8, 2, 700
    q, k, v, m, d_o = W.draw_training_attention(Hq, H, T, 5)
    tq, tk, tv, tg = (G.bits_to_bf16_gpu(x) for x in (q, k, v, d_o))
    tm = torch.from_numpy(m).cuda()
    outs = {"o": torch.empty((Hq, T, 128), dtype=torch.float32, device="cuda"),
            "lse": torch.empty((Hq, T), dtype=torch.float32, device="cuda"),
            "dq": torch.empty((Hq, T, 128), dtype=torch.float32, device="cuda"),
            "dk": torch.empty((H, T, 128), dtype=torch.float32, device="cuda"),
            "dv": torch.empty((H, T, 128), dtype=torch.float32, device="cuda"),
            "dm": torch.empty((H, T), dtype=torch.float32, device="cuda")}
    ws = torch.empty(lkv.lkv_masked_attn_backward_workspace_bytes(Hq, H, T), dtype=torch.uint8, device="cuda")

    def both():
        lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, tm, G.SCALE, outs["o"], outs["lse"])
        lkv.lkv_masked_attn_backward(ctx, tq, tk, tv, tm, outs["o"], outs["lse"], tg, G.SCALE, outs["dq"], outs["dk"],
                                     outs["dv"], outs["dm"], ws)

    both()
    torch.cuda.synchronize()
    want = {name: t.clone() for name, t in outs.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        both()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            both()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs.values():
            t.fill_(float("nan"))
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t in outs.items():
            assert torch.equal(t, want[name]), f"replay {rep}: {name}"


def test_captured_window_scoring_replays_to_the_eager_result(ctx):
    # the observation-window scorer is four kernel launches and no copy: captured together with the top-k it feeds,
    # every replay must give the bits of the eager run
    w = W.scaled(W.CONFIGS[0], L=2, H=2, Hq=8, b_min=8)
    T, window = 1900, 32
    K, _ = W.draw_kv(w, T, 0, 2)
    Q = W.draw_window_queries(w, K, window, 0, 2)
    tk, tq = G.bits_to_bf16_gpu(K), G.bits_to_bf16_gpu(Q)
    cache = lkv.Cache([tk], [tk], w.Hq)
    budgets = np.full(w.L * w.H, 300, dtype=np.int32)
    scores = torch.empty((w.L, w.H, T), dtype=torch.float32, device="cuda")
    idx = torch.empty(int(budgets.sum()), dtype=torch.int32, device="cuda")
    offsets = torch.empty(budgets.size + 1, dtype=torch.int32, device="cuda")
    ws = torch.empty(lkv.lkv_score_window_workspace_bytes(cache), dtype=torch.uint8, device="cuda")

    def both():
        lkv.lkv_score_window(ctx, cache, [tq], window, 7, lkv.POOL_MAX, G.SCALE, [scores], ws)
        lkv.lkv_select(ctx, cache, [scores], budgets, idx, offsets)

    both()
    torch.cuda.synchronize()
    want = (scores.clone(), idx.clone(), offsets.clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        both()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            both()
    torch.cuda.synchronize()
    for rep in range(3):
        scores.fill_(float("nan"))
        idx.fill_(-3)
        offsets.fill_(-3)
        ws.fill_(255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(scores, want[0]) and torch.equal(idx, want[1]) and torch.equal(offsets, want[2]), f"replay {rep}"
