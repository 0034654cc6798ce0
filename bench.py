#!/usr/bin/env python3
"""Benchmark of the LKV eviction hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch that is already
resident in HBM: lkv_score -> lkv_select -> lkv_compact -> lkv_decode_attn.
Prints ONE JSON line.  `value` is KV entries evicted per second over the three
eviction calls ((head-tokens - kept) / time); the decode leg is reported as
achieved HBM GB/s in `decode`.  The `roofline` object is for the kernel that
moves most of the bytes, the token scorer.

With no --config the headline (top-level keys) is the 131072-token workload
(32 x 8 heads, MLP 256 -> 64 GELU scorer) and `per_workload` carries the same
keys for the 32768-token workload, the 16-sequence batch and the 8 x 65536
batch, measured one after the other in the same process.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
HEADLINE_CONFIG = 2
ALSO_BY_DEFAULT = (1, 3, 4)

# HBM bytes per launch of the score kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, each scaled by what
# the same counter reads for a plain 1 GiB copy (the profiles/ file named next to each figure).  Hardware counters
# cannot be read from inside this script, so the figure is carried per workload together with the hash of the
# kernel's sources at the time of the measurement; when the sources have changed since, `traffic` is null.
SCORE_KERNEL_SOURCES = {
    "score_linear_kernel": ("score_linear.hip", "lkv_common.h"),
    "score_mlp_kernel": ("score_mlp.hip", "lkv_act.h", "lkv_common.h"),
    "score_mlp_wide_kernel": ("score_mlp.hip", "lkv_act.h", "lkv_common.h"),
}
MEASURED_SCORE_TRAFFIC = {
    # workload name: (bytes per launch, sha256[:16] of the kernel's sources, profile)
    "cfg1-L32-H8-T32768-linear": (4328897267, "8df6ec869a771fd8", "profiles/all_kernels__cfg1-L32-H8-T32768-linear.md"),
    "cfg2-L32-H8-T131072-mlp64gelu": (17337369377, "8610e17d31f2b4e3", "profiles/all_kernels__cfg2-L32-H8-T131072-mlp64gelu.md"),
    "cfg3-16seq-T4096..16384-linear": (22846926438, "8df6ec869a771fd8", "profiles/all_kernels__cfg3-16seq-T4096-16384-linear.md"),
    "cfg4-8seq-L28-H4-g7-T65536-mlp64gelu": (30386206836, "8610e17d31f2b4e3", "profiles/all_kernels__cfg4-8seq-L28-H4-g7-T65536-mlp64gelu.md"),
    "paper-L32-H8-T32768-mlp128silu-per-head": (4469725727, "8610e17d31f2b4e3", "profiles/all_kernels__paper-L32-H8-T32768-mlp128silu-per-head.md"),
    "paper-L36-H8-T32768-mlp128silu-per-head": (5028391389, "8610e17d31f2b4e3", "profiles/all_kernels__paper-L36-H8-T32768-mlp128silu-per-head.md"),
}


def kernel_source_hash(kernel: str) -> str:
    h = hashlib.sha256()
    for name in SCORE_KERNEL_SOURCES[kernel]:
        with open(os.path.join(ROOT, "paper_2605_06676_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, kernel: str):
    rec = MEASURED_SCORE_TRAFFIC.get(workload)
    if rec is None:
        return None, None
    nbytes, src_hash, profile = rec
    if src_hash != kernel_source_hash(kernel):
        return None, None          # the kernel has changed since the counters were read
    return nbytes, profile


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=None,
                    help="measure this workload only (0..6); default: the 131072-token workload as the headline and "
                         "workloads 1, 3 and 4 under `per_workload`")
    ap.add_argument("--seq-len", type=int, default=0, metavar="T",
                    help="override the context length of a fixed-length workload (the paper's overhead run is at 200k, Sec. 4.5)")
    ap.add_argument("--budgets", choices=("recipe", "lkvh"), default="recipe",
                    help="per-head budgets: the seeded recipe of the workload, or LKV-H computed on the GPU")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plain-select", action="store_true",
                    help="never let the scoring kernel count for the top-k (default: it does for the MLP scorers, whose "
                         "kernels count at no cost; lkv_score_counted / lkv_select_counted)")
    ap.add_argument("--decode-per-layer", action="store_true",
                    help="also time the decode as one launch per layer (single-sequence workloads); adds the key "
                         "`decode_per_layer_launches`")
    ap.add_argument("--growth", action="store_true",
                    help="also measure decode-time growth (compaction with slack, append, grown decode, re-eviction); "
                         "adds the key `growth`")
    ap.add_argument("--train-attn", type=int, nargs="?", const=16384, default=0, metavar="T",
                    help="also time the training-time attention with the multiplicative mask (forward and backward) "
                         "over T tokens (default 16384) for the workload's head counts; adds the key `training_attention`")
    ap.add_argument("--window-score", type=int, nargs="?", const=32, default=0, metavar="W",
                    help="also time the observation-window scorer (window W, default 32) and the eviction it feeds")
    ap.add_argument("--layerwise", action="store_true",
                    help="also measure layer-by-layer eviction during prefill; adds the key `layerwise` (a list: one entry "
                         "per --layerwise-shape)")
    ap.add_argument("--layerwise-producer", choices=("normal", "attention"), default="normal",
                    help="what produces a layer's K/V on the other stream in --layerwise: in-place normal_() (a stand-in "
                         "that costs about what the eviction costs, so the overlap is visible), or the layer's causal "
                         "attention over the prompt (lkv_masked_attn_forward with m = 1; single-sequence workloads, one "
                         "layer per call)")
    ap.add_argument("--layerwise-selector", choices=("lkv-t", "window"), default="lkv-t",
                    help="with --layerwise-producer attention: score with the workload's LKV-T scorer, or with the "
                         "observation-window scorer fed by the attention's log-normalisers (window 32, max pooling 7)")
    ap.add_argument("--layerwise-shape", action="append", default=None, metavar="STREAMS,LAYERS",
                    help="eviction streams and layers per lkv_evict_layer call for --layerwise (repeatable; "
                         "default 2,1 and 4,1 and 2,4)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy before the timed region (a kernel of known "
                         "traffic for scaling hardware byte counters under rocprofv3 --pmc)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="time cap of the oracle sample")
    return ap.parse_args()


def count_in_scorer(w, args):
    return w.scorer == "mlp" and w.hidden <= 64 and not args.plain_select


def count_for_layerwise(W, w, args):
    """Layer by layer, a call covers few heads, and the top-k of long heads is split over workgroups when it is given
    the first-level counts.  The 64-unit MLP scorer counts for free; the linear scorer needs a counting pass over
    its scores, which pays from about 131072 tokens per head on (measured: 6.84 against 7.19 ms at 204800 tokens,
    2.52 against 2.45 ms at 65536); the wide scorer's in-kernel counting costs what the split saves."""
    if args.plain_select:
        return False
    return count_in_scorer(w, args) or (w.scorer == "linear" and max(int(t) for t in W.seq_lengths(w)) >= 131072)


def to_dev(a, dev, bf16=False):
    import torch

    if a is None:
        return None
    if bf16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(dev)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)


def run_workload(ctx, lkv, W, w, args, dev, headline):
    """Times the step on workload `w`; returns the keys that describe one workload.  The extras that the
    command line asks for (growth, layer-by-layer, ...) and the oracle baseline are measured for the
    headline workload only."""
    import torch

    layerwise_result = None
    sc_host = W.draw_scorer(w)
    scorer = {"kind": sc_host["kind"], "act": sc_host["act"], "hidden": sc_host["hidden"],
              "per_head": sc_host["per_head"], "w1": to_dev(sc_host["w1"], dev, True), "b1": to_dev(sc_host["b1"], dev),
              "w2": to_dev(sc_host["w2"], dev), "b2": to_dev(sc_host["b2"], dev)}
    # ---- layer-by-layer mode first, while the whole cache does not exist yet ---------------
    if headline and args.layerwise:
        shapes = [tuple(int(x) for x in sh.split(",")) for sh in (args.layerwise_shape or ["2,1", "4,1", "2,4"])]
        layerwise_result = []
        for n_streams, per_call in shapes:
            layerwise_result.append(layerwise(ctx, lkv, W, w, scorer, dev, n_streams, per_call,
                                              counted=count_for_layerwise(W, w, args), producer=args.layerwise_producer,
                                              selector=args.layerwise_selector))
            torch.cuda.empty_cache()

    # ---- inputs, resident in HBM before the timed region --------------------------------
    Ts = [int(t) for t in W.seq_lengths(w)]
    Ks, Vs = [], []
    for s, T in enumerate(Ts):
        k, v = W.device_kv(w, T, s, dev)
        Ks.append(k); Vs.append(v)
    cache = lkv.Cache(Ks, Vs, w.Hq)
    # LKV-H (Sec. 3.3): ratios are computed once from static parameters; timed apart from the step
    emb_h, mlp_h = W.draw_head_predictor(w)
    emb_d = to_dev(emb_h, dev)
    pred_d = {k: to_dev(mlp_h[k], dev) for k in ("w1", "b1", "w2")}
    pred_d["b2"] = None
    r_d = torch.empty((w.L * w.H,), dtype=torch.float64, device=dev)
    b_d = torch.empty((w.L * w.H,), dtype=torch.int32, device=dev)
    lkv.lkv_head_budgets(ctx, emb_d, pred_d, w.R, Ts[0], r_d, b_d)
    torch.cuda.synchronize()
    eh = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    eh[0].record()
    for _ in range(20):
        lkv.lkv_head_budgets(ctx, emb_d, pred_d, w.R, Ts[0], r_d, b_d)
    eh[1].record()
    torch.cuda.synchronize()
    lkv_h_us = eh[0].elapsed_time(eh[1]) * 1e3 / 20
    if args.budgets == "lkvh":
        budgets = []
        for T in Ts:
            lkv.lkv_head_budgets(ctx, emb_d, pred_d, w.R, T, r_d, b_d)
            torch.cuda.synchronize()
            budgets.append(b_d.cpu().numpy().reshape(w.L, w.H).astype(np.int32))
    else:
        budgets = [W.draw_budgets(w, T, s) for s, T in enumerate(Ts)]
    budgets_flat = np.concatenate([b.reshape(-1) for b in budgets]).astype(np.int32)
    total = int(budgets_flat.sum())
    N = sum(w.L * w.H * T for T in Ts)
    scores = [torch.empty((w.L, w.H, T), dtype=torch.float32, device=dev) for T in Ts]
    idx = torch.empty((total,), dtype=torch.int32, device=dev)
    offsets = torch.empty((cache.n_segments + 1,), dtype=torch.int32, device=dev)
    kp = torch.empty((total, w.d), dtype=torch.bfloat16, device=dev)
    vp = torch.empty_like(kp)
    q = torch.stack([to_dev(W.draw_q(w, s), dev, True) for s in range(w.n_seq)]).contiguous()
    out = torch.empty((w.n_seq, w.L, w.Hq, w.d), dtype=torch.float32, device=dev)
    lse = torch.empty((w.n_seq, w.L, w.Hq), dtype=torch.float32, device=dev)
    ws = torch.empty((lkv.lkv_decode_workspace_bytes(cache.n_segments, total, w.Hq, w.H),), dtype=torch.uint8, device=dev)
    scale = 1.0 / math.sqrt(w.d)

    # The packed layout follows from the budgets alone, and those are static (Sec. 3.3: b = floor(r t) with frozen
    # ratios), so the offsets are planned once per (model, context length), before the timed region; inside it
    # lkv_select reads them from the device: no copy and no host wait, whatever the number of segments.
    t0 = time.perf_counter()
    planned = lkv.lkv_plan_offsets(ctx, budgets_flat, offsets)
    torch.cuda.synchronize()
    plan_us = (time.perf_counter() - t0) * 1e6
    assert planned == total

    # MLP scorers up to 64 hidden units: the scoring kernel counts the first radix level of the top-k on its way out
    # (free there: the kernel waits for HBM; the wider scorer is bound by instruction issue and pays 3 % for it)
    counted = count_in_scorer(w, args)
    counts = None
    if counted:
        counts = torch.empty((cache.n_segments, 2048), dtype=torch.int32, device=dev)
        lkv.lkv_clear_counts(ctx, counts, cache.n_segments)      # once: every select leaves the counters zero again

    def step(ev=(None,) * 5):
        if ev[0] is not None: ev[0].record()
        if counted:
            lkv.lkv_score_counted(ctx, cache, scorer, scores, counts)
        else:
            lkv.lkv_score(ctx, cache, scorer, scores)
        if ev[1] is not None: ev[1].record()
        if counted:
            lkv.lkv_select_counted(ctx, cache, scores, None, counts, idx, offsets)
        else:
            lkv.lkv_select(ctx, cache, scores, None, idx, offsets)
        if ev[2] is not None: ev[2].record()
        lkv.lkv_compact(ctx, cache, idx, offsets, total, kp, vp)
        if ev[3] is not None: ev[3].record()
        lkv.lkv_decode_attn(ctx, w.n_seq, w.L, w.H, w.Hq, w.d, q, kp, vp, offsets, total, scale, out, lse, ws)
        if ev[4] is not None: ev[4].record()

    if headline and args.calibrate_copy:
        src = torch.zeros((1 << 28,), dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # ---- the timed region: exactly K whole steps, nothing but the library's calls between the two synchronisations ----
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # ---- the same K steps again with events, for the breakdown.  An event record is not free: two records with
    # nothing between them are `event_pair_us` apart (about 4 us here), and whatever they bracket carries that much.
    # First with three events per step (before the eviction, after it, after the decode): the eviction's time inside
    # the step, from which `value` is taken, carries one such pair in a millisecond or more.  Then with an event
    # after every call for the per-call figures, of which the short ones (top-k, decode) are visibly inflated; the
    # decode is therefore also timed as K calls between one pair of events further down.  (The kernels are enqueued
    # on torch's current stream, which is also where these events are recorded.)
    def timed_steps(marks):
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        for i in range(args.steps):
            step([e if j in marks else None for j, e in enumerate(evs[i])])
        torch.cuda.synchronize()
        ms = sorted(marks)
        return np.array([[ev[ms[j]].elapsed_time(ev[ms[j + 1]]) for j in range(len(ms) - 1)] for ev in evs]).mean(axis=0)

    t_evict, t_decode = timed_steps({0, 3, 4})
    t_score, t_select, t_compact, t_decode_call = timed_steps({0, 1, 2, 3, 4})
    pairs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(50)]
    for a_, b_ in pairs:
        a_.record(); b_.record()
    torch.cuda.synchronize()
    event_pair_us = float(np.median([a_.elapsed_time(b_) for a_, b_ in pairs])) * 1e3
    rho = total / N
    evict_bytes = N * 520 + total * 1032
    decode_bytes = total * 512 + w.n_seq * w.L * w.Hq * w.d * (2 + 4)
    score_bytes = N * 516
    kernel = "score_linear_kernel" if w.scorer == "linear" else ("score_mlp_kernel" if w.hidden <= 64 else "score_mlp_wide_kernel")
    launches = 1 if w.n_seq <= 32 else math.ceil(w.n_seq / 32)
    traffic, traffic_profile = (None, None) if args.seq_len or args.budgets != "recipe" else measured_traffic(w.name, kernel)

    result = {
        "value": (N - total) / (t_evict * 1e-3),
        "ms_per_step": wall * 1e3 / args.steps,
        "config": {"workload": w.name, "n_seq": w.n_seq, "layers": w.L, "kv_heads": w.H, "q_heads": w.Hq,
                   "seq_len": Ts if len(set(Ts)) > 1 else Ts[0], "head_tokens": N, "kept": total,
                   "retention": rho, "scorer": w.scorer if w.scorer == "linear" else f"mlp256-{w.hidden}-{w.act}",
                   "budgets": "lkv-h on the GPU" if args.budgets == "lkvh" else "seeded recipe",
                   "offsets": "planned once before the timed region (budgets are static); lkv_select reads them from the device",
                   "plan_offsets_us": plan_us,
                   "top_k_first_level": "counted by the scoring kernel" if counted else "counted by the top-k kernel"},
        "phases_ms": {"score": t_score, "select": t_select, "compact": t_compact, "decode": t_decode_call,
                      "evict": t_evict, "step_gpu": t_evict + t_decode, "event_pair_us": event_pair_us,
                      "note": "score, select, compact, decode: steps with an event after every call, each figure includes "
                              "one event_pair_us; evict: steps with events around the three eviction calls only"},
        "evict": {"bytes": evict_bytes, "GBps": evict_bytes / (t_evict * 1e6),
                  "frac_of_peak": evict_bytes / (t_evict * 1e6) / HBM_PEAK_GBS,
                  "context_tokens_per_s": sum(Ts) / (t_evict * 1e-3)},
        "decode": {"bytes": decode_bytes, "in_step_ms": t_decode, "in_step_GBps": decode_bytes / (t_decode * 1e6),
                   "in_step_frac_of_peak": decode_bytes / (t_decode * 1e6) / HBM_PEAK_GBS},
        # achieved = algorithmic bytes of one launch (516 B per head-token) over the kernel's average duration,
        # from the events that bracket lkv_score on the stream it runs on (the call is `launches` launches back to back)
        "roofline": {"kernel": kernel, "bound": "hbm", "achieved": score_bytes / (t_score * 1e6), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": score_bytes / (t_score * 1e6) / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_profile": traffic_profile, "kernel_source_sha256_16": kernel_source_hash(kernel),
                     "launches_per_step": launches, "bytes_per_launch": score_bytes // launches},
    }

    # decode: K calls back to back between one pair of events, which is also what a serving loop sees between
    # evictions (the in-step figure above carries an event pair and follows the compaction's writes)
    es = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    es[0].record()
    for _ in range(args.steps):
        lkv.lkv_decode_attn(ctx, w.n_seq, w.L, w.H, w.Hq, w.d, q, kp, vp, offsets, total, scale, out, lse, ws)
    es[1].record()
    torch.cuda.synchronize()
    t_steady = es[0].elapsed_time(es[1]) / args.steps
    result["decode"]["ms"] = t_steady
    result["decode"]["GBps"] = decode_bytes / (t_steady * 1e6)
    result["decode"]["frac_of_peak"] = decode_bytes / (t_steady * 1e6) / HBM_PEAK_GBS
    if not headline:
        return result

    # ---- context figures: a plain device copy on this machine, and decode launched once per layer ----
    src = torch.empty((1 << 28,), dtype=torch.float32, device=dev)      # 1 GiB
    dst = torch.empty_like(src)
    dst.copy_(src)
    ec = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ec[0].record()
    for _ in range(5):
        dst.copy_(src)
    ec[1].record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * src.numel() * 4 / (ec[0].elapsed_time(ec[1]) * 1e6)
    del src, dst
    result["device_copy_GBps"] = copy_gbps
    if w.n_seq == 1 and args.decode_per_layer:
        # a real model runs its layers one after the other, so decode is one launch per layer there
        off_h = offsets.cpu().numpy().astype(np.int64)
        lay_off = [torch.from_numpy((off_h[l * w.H:(l + 1) * w.H + 1] - off_h[l * w.H]).astype(np.int32)).to(dev)
                   for l in range(w.L)]
        lay_rows = [int(off_h[(l + 1) * w.H] - off_h[l * w.H]) for l in range(w.L)]
        def decode_layers():
            for l in range(w.L):
                r0 = int(off_h[l * w.H])
                lkv.lkv_decode_attn(ctx, 1, 1, w.H, w.Hq, w.d, q[0, l], kp[r0:], vp[r0:], lay_off[l], lay_rows[l],
                                    scale, out[0, l], lse[0, l], ws)
        decode_layers()
        torch.cuda.synchronize()
        ec[0].record()
        for _ in range(5):
            decode_layers()
        ec[1].record()
        torch.cuda.synchronize()
        t_layers = ec[0].elapsed_time(ec[1]) / 5
        # the same 2 L launches captured once into a HIP graph and replayed: no per-launch host cost
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            decode_layers()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                decode_layers()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ec[0].record()
        for _ in range(5):
            graph.replay()
        ec[1].record()
        torch.cuda.synchronize()
        t_graph = ec[0].elapsed_time(ec[1]) / 5
        result["decode_per_layer_launches"] = {"ms_all_layers": t_layers, "us_per_layer": t_layers * 1e3 / w.L,
                                               "GBps": decode_bytes / (t_layers * 1e6),
                                               "hip_graph_ms_all_layers": t_graph,
                                               "hip_graph_us_per_layer": t_graph * 1e3 / w.L,
                                               "hip_graph_GBps": decode_bytes / (t_graph * 1e6),
                                               "note": "launch-latency bound at batch 1: one layer is ~20-54 MB"}
    result["lkv_h"] = {"n_heads": w.L * w.H, "us_per_call": lkv_h_us, "dtype": "f64",
                       "note": "head scores + Soft-TopK + floor(r t); computed once, outside the step"}
    if layerwise_result is not None:
        result["layerwise"] = layerwise_result
    if args.growth:
        result["growth"] = growth(ctx, lkv, w, cache, scorer, scores, idx, offsets, budgets_flat, total, Ts, q, scale, dev)
    if args.train_attn:
        result["training_attention"] = training_attention(ctx, lkv, w, args.train_attn, dev)
    if args.window_score:
        result["window_scorer"] = window_scorer(ctx, lkv, w, cache, scores, budgets_flat, idx, offsets, total, kp, vp,
                                                Ts, args.window_score, scale, dev)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, Ts, Ks, Vs, sc_host, budgets, q, args.cpu_seconds)
    return result


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every (sequence, layer, head) is independent, "
              "so more GPUs would just take disjoint heads); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2605_06676_amd import lkv
    from paper_2605_06676_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    head_id = HEADLINE_CONFIG if args.config is None else args.config
    others = ALSO_BY_DEFAULT if args.config is None and not args.seq_len else ()
    w = W.CONFIGS[head_id]
    if args.seq_len:
        if not isinstance(w.T, int):
            print("bench.py: --seq-len needs a workload with one fixed length", file=sys.stderr)
            sys.exit(2)
        w = W.scaled(w, T=args.seq_len, name=f"{w.name}-T{args.seq_len}")
    ctx = lkv.Context(0)

    head = run_workload(ctx, lkv, W, w, args, dev, headline=True)
    result = {
        "metric": "KV tokens evicted/sec (score+select+compact); ragged decode-attn HBM GB/s in `decode`",
        "value": head.pop("value"),
        "unit": "evicted KV entries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "accumulate": "f32", "data": "synthetic",
    }
    result.update(head)
    if others:
        per = {}
        for cid in others:
            torch.cuda.empty_cache()
            r = run_workload(ctx, lkv, W, W.CONFIGS[cid], args, dev, headline=False)
            r["unit"] = "evicted KV entries/s"
            per[r["config"]["workload"]] = r
        result["per_workload"] = per
    print(json.dumps(result))


MFMA_BF16_PEAK_TFLOPS = 2500.0


def training_attention(ctx, lkv, w, T, dev, reps=10):
    """Causal attention with the multiplicative mask (App. B) for one layer of one sequence of T tokens, the
    workload's query and KV head counts: forward, and backward (dQ, dK, dV, dm).  FLOPs are the algorithmic
    ones of the causal triangle: 2 products for the forward, 5 for the backward (the backward kernels execute
    7, because s and dP are recomputed in both of them)."""
    import torch

    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    q = torch.randn((w.Hq, T, w.d), device=dev, generator=gen).to(torch.bfloat16)
    k = torch.randn((w.H, T, w.d), device=dev, generator=gen).to(torch.bfloat16)
    v = torch.randn((w.H, T, w.d), device=dev, generator=gen).to(torch.bfloat16)
    d_o = torch.randn((w.Hq, T, w.d), device=dev, generator=gen).to(torch.bfloat16)
    m = torch.rand((w.H, T), device=dev, generator=gen) ** 4
    o = torch.empty((w.Hq, T, w.d), dtype=torch.float32, device=dev)
    lse = torch.empty((w.Hq, T), dtype=torch.float32, device=dev)
    dq = torch.empty_like(o)
    dk = torch.empty((w.H, T, w.d), dtype=torch.float32, device=dev)
    dv = torch.empty_like(dk)
    dm = torch.empty_like(m)
    ws = torch.empty((lkv.lkv_masked_attn_backward_workspace_bytes(w.Hq, w.H, T),), dtype=torch.uint8, device=dev)
    scale = 1.0 / math.sqrt(w.d)

    def timed(fn):
        for _ in range(2):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(reps):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / reps

    t_fwd = timed(lambda: lkv.lkv_masked_attn_forward(ctx, q, k, v, m, scale, o, lse))
    t_bwd = timed(lambda: lkv.lkv_masked_attn_backward(ctx, q, k, v, m, o, lse, d_o, scale, dq, dk, dv, dm, ws))
    product = 2.0 * w.d * (T * (T + 1) / 2) * w.Hq      # one causal (query, key) product over d channels, all heads
    out = {"tokens": T, "n_q_heads": w.Hq, "n_kv_heads": w.H, "dtype": "bf16", "accumulate": "f32"}
    for name, t, n_products, executed in (("forward", t_fwd, 2, 2), ("backward", t_bwd, 5, 7)):
        tf = n_products * product / (t * 1e9)
        out[name] = {"ms": t, "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                                           "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
                     "executed_TFLOPs": executed * product / (t * 1e9)}
    return out


def window_scorer(ctx, lkv, w, cache, scores, budgets_flat, idx, offsets, total, kp, vp, Ts, window, scale, dev, reps=10):
    """The observation-window scorer (the attention-based selection policy of the ablation, Sec. 4.4) on the
    workload's cache with the workload's budgets: the scoring call alone, and scoring + top-k + compaction.
    Algorithmic bytes: every key row once (the kernels read them twice, once per softmax pass), the window
    queries, the scores; the eviction adds the index and packed-cache traffic of the main path."""
    import torch

    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    q_win = [torch.randn((w.L, w.Hq, window, w.d), device=dev, generator=gen).to(torch.bfloat16) for _ in Ts]
    ws = torch.empty((lkv.lkv_score_window_workspace_bytes(cache),), dtype=torch.uint8, device=dev)
    budgets = np.maximum(budgets_flat, window).astype(np.int32)      # the rule keeps the window on top of its picks
    budgets = np.minimum(budgets, np.repeat(np.asarray(Ts, dtype=np.int32), w.L * w.H))
    extra = int(budgets.sum()) - total
    if extra > 0:
        kp = torch.empty((total + extra, w.d), dtype=torch.bfloat16, device=dev)
        vp = torch.empty_like(kp)
        idx = torch.empty((total + extra,), dtype=torch.int32, device=dev)

    def score():
        lkv.lkv_score_window(ctx, cache, q_win, window, 7, lkv.POOL_MAX, scale, scores, ws)

    def evict():
        score()
        lkv.lkv_select(ctx, cache, scores, budgets, idx, offsets)
        lkv.lkv_compact(ctx, cache, idx, offsets, int(budgets.sum()), kp, vp)

    def timed(fn):
        for _ in range(2):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(reps):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / reps

    t_score, t_evict = timed(score), timed(evict)
    # the same with the window rows' log-normalisers supplied, as a serving engine would have them from the prefill's
    # attention kernel (computed here with torch, outside the timed region): the keys are then read once
    G = w.Hq // w.H
    lse_win = []
    for s_i, T in enumerate(Ts):
        lse = torch.empty((w.L, w.Hq, window), dtype=torch.float32, device=dev)
        causal = (torch.arange(T, device=dev)[None, :] > (T - window + torch.arange(window, device=dev))[:, None])
        for l in range(w.L):
            kl = cache.k[s_i][l].float()                                                  # [H, T, d]
            ql = q_win[s_i][l].float().reshape(w.H, G * window, w.d)                      # [H, G W, d]
            logits = torch.einsum("hrd,htd->hrt", ql, kl) * scale
            logits = logits.reshape(w.H, G, window, T).masked_fill(causal[None, None], float("-inf"))
            lse[l] = torch.logsumexp(logits, dim=-1).reshape(w.Hq, window)
        lse_win.append(lse)
    del logits, kl, ql

    def score_given_lse():
        lkv.lkv_score_window(ctx, cache, q_win, window, 7, lkv.POOL_MAX, scale, scores, ws, lse_win=lse_win)

    t_score_lse = timed(score_given_lse)
    N = sum(w.L * w.H * T for T in Ts)
    kept = int(budgets.sum())
    score_bytes = N * (2 * w.d + 4) + len(Ts) * w.L * w.Hq * window * w.d * 2
    evict_bytes = score_bytes + N * 4 + kept * 4 + kept * 2 * w.d * 2 * 2
    return {"window": window, "pool": "max, width 7", "dtype": "bf16", "accumulate": "f32",
            "score_ms": t_score, "evict_ms": t_evict,
            "roofline": {"bound": "hbm", "achieved": score_bytes / (t_score * 1e6), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": score_bytes / (t_score * 1e6) / HBM_PEAK_GBS, "traffic": None},
            "keys_read_twice_GBps": (score_bytes + N * 2 * w.d) / (t_score * 1e6),
            "given_prefill_normalisers": {"score_ms": t_score_lse, "GBps": score_bytes / (t_score_lse * 1e6),
                                          "frac": score_bytes / (t_score_lse * 1e6) / HBM_PEAK_GBS,
                                          "note": "log-normalisers of the window rows passed in: one pass over the keys"},
            "evict_GBps": evict_bytes / (t_evict * 1e6),
            "note": "the two softmax passes are bound by vector and matrix issue (one exponential per logit and "
                    "pass), not by HBM"}


def growth(ctx, lkv, w, cache, scorer, scores, idx, offsets, budgets_flat, total, Ts, q, scale, dev, slack=128, n_new=64):
    """Decode-time growth (spare rows per segment): compaction with slack, n_new appended tokens,
    decode over the rows in use, then a re-eviction with the budgets floor(r t') of the longer context."""
    import torch

    n_seg = cache.n_segments
    rows = total + n_seg * slack
    kp = torch.empty((rows, w.d), dtype=torch.bfloat16, device=dev)
    vp = torch.empty_like(kp)
    up = torch.empty((rows,), dtype=torch.float32, device=dev)
    cap = torch.empty((n_seg + 1,), dtype=torch.int32, device=dev)
    ln = torch.empty((n_seg,), dtype=torch.int32, device=dev)
    out = torch.empty((w.n_seq, w.L, w.Hq, w.d), dtype=torch.float32, device=dev)
    lse = torch.empty((w.n_seq, w.L, w.Hq), dtype=torch.float32, device=dev)
    ws = torch.empty((lkv.lkv_decode_workspace_bytes(n_seg, rows, w.Hq, w.H),), dtype=torch.uint8, device=dev)
    k_new = torch.randn((w.n_seq, w.L, w.H, w.d), device=dev).to(torch.bfloat16)
    v_new = torch.randn((w.n_seq, w.L, w.H, w.d), device=dev).to(torch.bfloat16)

    def timed(fn, reps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(reps):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / reps

    def compact():
        lkv.lkv_compact_grow(ctx, cache, scores, idx, offsets, total, slack, kp, vp, up, cap, ln)

    compact()
    t_compact = timed(compact, 5)
    t_append = timed(lambda: lkv.lkv_append(ctx, w.n_seq, w.L, w.H, w.d, scorer, k_new, v_new, kp, vp, up, cap, ln), n_new)
    used = total + n_seg * n_new
    dec = lambda: lkv.lkv_decode_attn_grown(ctx, w.n_seq, w.L, w.H, w.Hq, w.d, q, kp, vp, cap, ln, rows, scale, out, lse, ws)
    dec()
    t_decode = timed(dec, 10)
    seg_T = np.repeat(np.asarray(Ts, dtype=np.float64), w.L * w.H)
    len_h = budgets_flat.astype(np.int64) + n_new
    nb = np.minimum(np.floor(budgets_flat / seg_T * (seg_T + n_new)).astype(np.int64), len_h)
    total2 = int(nb.sum())
    rows2 = total2 + n_seg * slack
    kp2 = torch.empty((rows2, w.d), dtype=torch.bfloat16, device=dev)
    vp2 = torch.empty_like(kp2)
    up2 = torch.empty((rows2,), dtype=torch.float32, device=dev)
    cap2, len2 = torch.empty_like(cap), torch.empty_like(ln)
    idx2 = torch.empty((total2,), dtype=torch.int32, device=dev)
    off2 = torch.empty((n_seg + 1,), dtype=torch.int32, device=dev)
    re = lambda: lkv.lkv_reevict(ctx, w.d, kp, vp, up, cap, ln, len_h, nb, slack, idx2, off2, kp2, vp2, up2, cap2, len2)
    re()
    t_reevict = timed(re, 5)
    re_bytes = used * 4 + total2 * (4 + 4 + 4 + 4 + 1024)
    return {"slack": slack, "appended": n_new, "rows_in_use": int(used),
            "compact_with_slack_ms": t_compact, "append_us_per_token": t_append * 1e3,
            "decode_ms": t_decode, "decode_GBps": used * 512 / (t_decode * 1e6),
            "decode_frac_of_peak": used * 512 / (t_decode * 1e6) / HBM_PEAK_GBS,
            "reevict_ms": t_reevict, "reevict_kept": total2, "reevict_GBps": re_bytes / (t_reevict * 1e6)}


def layerwise(ctx, lkv, W, w, scorer, dev, n_streams=2, layers_per_call=1, counted=False, producer="normal",
              selector="lkv-t", reps=3):
    """Layer-by-layer eviction during prefill (Sec. 1): a stand-in producer fills the K/V of the next
    `layers_per_call` layers on one stream (it takes the place of the prefill compute), the eviction of
    earlier layers runs on `n_streams` other streams in turn; n_streams buffers of layers_per_call layers
    are alive at any time instead of L layers.  Reports time and peak memory."""
    import torch

    Ts = [int(t) for t in W.seq_lengths(w)]
    if len(Ts) > 32:
        return None
    attention = producer == "attention"
    if attention and (len(Ts) != 1 or layers_per_call != 1):
        return None
    m = layers_per_call
    calls = [(l, min(m, w.L - l)) for l in range(0, w.L, m)]
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    budgets = np.concatenate([W.draw_budgets(w, T, s).reshape(-1) for s, T in enumerate(Ts)]).astype(np.int32)
    n_seg = budgets.size
    total = int(budgets.sum())
    ring = [([torch.empty((m, w.H, T, w.d), dtype=torch.bfloat16, device=dev) for T in Ts],
             [torch.empty((m, w.H, T, w.d), dtype=torch.bfloat16, device=dev) for T in Ts]) for _ in range(n_streams)]

    def view(slot, n):
        return lkv.Cache([k[:n] for k in ring[slot][0]], [v[:n] for v in ring[slot][1]], w.Hq)

    views = {(slot, n): view(slot, n) for slot in range(n_streams) for n in {c[1] for c in calls}}
    # the eviction streams take the calls in turn (each with its own score scratch) so that the latency-bound
    # top-k of one call overlaps the bandwidth-bound scoring of the next
    scratch = [[torch.empty((m, w.H, T), dtype=torch.float32, device=dev) for T in Ts] for _ in range(n_streams)]
    idx = torch.empty((total,), dtype=torch.int32, device=dev)
    offsets = torch.empty((n_seg + 1,), dtype=torch.int32, device=dev)
    kp = torch.empty((total, w.d), dtype=torch.bfloat16, device=dev)
    vp = torch.empty_like(kp)
    s_fill, s_evicts = torch.cuda.Stream(), [torch.cuda.Stream() for _ in range(n_streams)]
    counts = None
    if counted:
        # counters plus room for the bitmaps that let a call over few long heads split every head over several workgroups
        counts = torch.empty((lkv.lkv_counts_bytes_split(n_seg, max(Ts)) // 4,), dtype=torch.int32, device=dev)
        lkv.lkv_clear_counts(ctx, counts, n_seg)
        torch.cuda.synchronize()

    if attention:
        # the layer's own attention over the prompt: queries of all positions (a stand-in draw; K/V keep what the
        # first fill wrote), output and log-normalisers; the last `window` queries and their normalisers feed the
        # observation-window scorer when that is the selector
        T0, window = Ts[0], 32
        q_all = torch.randn((w.Hq, T0, w.d), device=dev).to(torch.bfloat16)
        ones = torch.ones((w.H, T0), dtype=torch.float32, device=dev)
        att_o = torch.empty((w.Hq, T0, w.d), dtype=torch.float32, device=dev)
        att_lse = [torch.empty((w.Hq, T0), dtype=torch.float32, device=dev) for _ in range(n_streams)]
        q_win = q_all[:, T0 - window:].contiguous()[None]
        win_ws = torch.empty((lkv.lkv_score_window_workspace_bytes(views[(0, 1)]),), dtype=torch.uint8, device=dev)
        for slot in range(n_streams):
            for t in ring[slot][0] + ring[slot][1]:
                t.normal_()
        att_scale = 1.0 / math.sqrt(w.d)

    def fill(slot):
        if attention:
            lkv.lkv_masked_attn_forward(ctx, q_all, ring[slot][0][0][0], ring[slot][1][0][0], ones, att_scale, att_o,
                                        att_lse[slot], stream=s_fill)
            return
        for t in ring[slot][0] + ring[slot][1]:
            t.normal_()

    def run(evict=True, produce=True):
        n = len(calls)
        filled = [torch.cuda.Event() for _ in range(n)]
        evicted = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        started = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if evict:
            lkv.lkv_plan_offsets(ctx, budgets, offsets, stream=s_evicts[0])
            planned = torch.cuda.Event()
            planned.record(s_evicts[0])
            for s_e in s_evicts[1:]:
                s_e.wait_event(planned)
        for i, (l, nl) in enumerate(calls):
            slot = i % n_streams
            s_evict = s_evicts[slot]
            if produce:
                with torch.cuda.stream(s_fill):
                    if evict and i >= n_streams:
                        s_fill.wait_event(evicted[i - n_streams])     # the buffer's previous layers have left it
                    fill(slot)
                    filled[i].record(s_fill)
            if evict:
                if produce:
                    s_evict.wait_event(filled[i])
                started[i].record(s_evict)
                if attention and selector == "window":
                    with torch.cuda.stream(s_evict):
                        lse_win = att_lse[slot][:, T0 - window:].contiguous()[None]
                    lkv.lkv_score_window(ctx, views[(slot, 1)], [q_win], window, 7, lkv.POOL_MAX, att_scale,
                                         [scratch[slot][0][:1]], win_ws, stream=s_evict, lse_win=[lse_win])
                    lkv.lkv_evict_layer(ctx, views[(slot, 1)], l, w.L, None, budgets, offsets, [scratch[slot][0][0]],
                                        idx, kp, vp, stream=s_evict)
                else:
                    lkv.lkv_evict_layer(ctx, views[(slot, nl)], l, w.L, scorer, budgets, offsets,
                                        [t[:nl] for t in scratch[slot]], idx, kp, vp, stream=s_evict, counts=counts)
                evicted[i].record(s_evict)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        per_call = float(np.mean([started[i].elapsed_time(evicted[i]) for i in range(n)])) if evict else 0.0
        return wall, per_call

    run()                                   # warm-up
    both = min(run()[0] for _ in range(reps))
    produce_only = min(run(evict=False)[0] for _ in range(reps))
    for slot in range(n_streams):
        fill(slot)
    evict_only, per_call = min(run(produce=False) for _ in range(reps))
    peak = torch.cuda.max_memory_allocated() - base
    layer_bytes = sum(2 * w.H * T * w.d * 2 for T in Ts)
    N = sum(w.L * w.H * T for T in Ts)
    gbps = (N * 520 + total * 1032) / (evict_only * 1e6)
    return {"eviction_streams": n_streams, "layers_per_call": m, "layer_buffers_alive": n_streams * m,
            "top_k_first_level": ("counted by the top-k kernel" if not counted else
                                  "counted by a pass over the scores, top-k split over workgroups" if w.scorer == "linear" else
                                  "counted by the scoring kernel"),
            "ms_producer_and_eviction": both, "ms_producer_alone": produce_only, "ms_eviction_alone": evict_only,
            "ms_per_call_eviction": per_call,
            "evict_GBps_eviction_alone": gbps, "evict_frac_of_peak_eviction_alone": gbps / HBM_PEAK_GBS,
            "peak_bytes": int(peak), "peak_bytes_whole_cache_path": int(w.L * layer_bytes + total * 1032 + N * 4),
            "producer": "causal attention over the prompt, lkv_masked_attn_forward with m = 1" if attention
                        else "in-place normal_() of the layers' K/V on another stream, standing in for prefill",
            "selector": ("observation window fed by the attention's log-normalisers" if selector == "window" else "lkv-t")
                        if attention else "lkv-t",
            "note": "wall-clock times from the first enqueue to the last completion"}


def cpu_baseline(w, Ts, Ks, Vs, sc_host, budgets, q, cap_s):
    """The oracle as it stands, timed on the host cores over whole layers of sequence 0 until the cap."""
    import torch
    from threadpoolctl import threadpool_info

    from oracle import lkv_oracle as O

    T = Ts[0]
    done_tokens = done_kept = 0
    layers = 0
    spent = 0.0
    evict_s = 0.0
    scale = 1.0 / math.sqrt(w.d)
    qh = q[0].view(torch.int16).cpu().numpy().view(np.uint16)
    while layers < w.L and spent < cap_s:
        l = layers
        Kb = Ks[0][l].view(torch.int16).cpu().numpy().view(np.uint16)[None]     # [1, H, T, d]
        Vb = Vs[0][l].view(torch.int16).cpu().numpy().view(np.uint16)[None]
        sc = {"kind": sc_host["kind"], "act": sc_host["act"], "w1": sc_host["w1"][l:l + 1],
              "b1": sc_host["b1"][l:l + 1], "w2": None if sc_host["w2"] is None else sc_host["w2"][l:l + 1],
              "b2": None if sc_host["b2"] is None else sc_host["b2"][l:l + 1]}
        t0 = time.perf_counter()
        sco = dict(sc)
        sco["w1"] = O.bf16_bits_to_f64(sc["w1"])
        u = O.score(O.bf16_bits_to_f64(Kb), O.bf16_bits_to_f64(Vb), sco)
        b = budgets[0][l:l + 1]
        idx, off = O.select_all(u, b)
        Kp, Vp = O.compact(Kb, Vb, idx, off)
        t_ev = time.perf_counter() - t0
        O.decode_attn(O.bf16_bits_to_f64(qh[l:l + 1]), O.bf16_bits_to_f64(Kp), O.bf16_bits_to_f64(Vp), off, w.H, scale)
        spent += time.perf_counter() - t0
        done_tokens += w.H * T
        done_kept += int(b.sum())
        layers += 1
        evict_s += t_ev
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    cpu_model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next((line.split(":", 1)[1].strip() for line in f if line.startswith("model name")), cpu_model)
    except OSError:
        pass
    return {"value": (done_tokens - done_kept) / evict_s, "unit": "evicted KV entries/s",
            "cores": threads, "kind": "oracle",
            "sample": f"layers 0..{layers - 1} of sequence 0 ({done_tokens} head-tokens), numpy fp64, "
                      f"{spent:.1f} s including the decode leg",
            "host_cpus": os.cpu_count(), "cpu_model": cpu_model}


if __name__ == "__main__":
    main()
