"""lkv_decode_attn_static: the decode call that takes no workspace and allocates nothing (its split-K partials
go to a static device array inside the library).  It runs the kernels of lkv_decode_attn, so its output must
equal that call's bit for bit, on two calls in a row, the second with a smaller input (the array then still
holds the first call's partials)."""
import ctypes as C

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


def _case(ctx, w, Ts, seed):
    Ks, Vs, Qs, Bs = [], [], [], []
    for s, T in enumerate(Ts):
        K, V = W.draw_kv(w, T, s, seed)
        Ks.append(K); Vs.append(V); Qs.append(W.draw_q(w, s, seed)); Bs.append(W.draw_budgets(w, T, s, seed))
    sc = W.draw_scorer(w, seed)
    run = G.GpuRun(ctx, Ks, Vs, Qs, sc, Bs, w.Hq)
    run.run_all()                                   # score, select, compact, and lkv_decode_attn with a workspace
    G.check_against_oracle(run, Ks, Vs, Qs, sc, Bs, w.name)
    return run


def _decode_static(ctx, run):
    """One call through the C ABI; returns (out, lse) as new tensors."""
    c = run.cache
    out = torch.full_like(run.out, float("nan"))
    lse = torch.full_like(run.lse, float("nan"))
    lib = lkv.load_library()
    st = lib.lkv_decode_attn_static(ctx.h, c.n_seq, c.L, c.H, c.Hq, c.d, run.q.data_ptr(), run.kp.data_ptr(),
                                    run.vp.data_ptr(), run.offsets.data_ptr(), run.total, C.c_float(G.SCALE),
                                    out.data_ptr(), lse.data_ptr(), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == lkv.LKV_OK, lib.lkv_last_error(ctx.h).decode()
    torch.cuda.synchronize()
    return out, lse


def test_static_scratch_decode_equals_the_workspace_decode_twice_in_a_row(ctx):
    # first call: segments long enough to be split over several chunks (partials merged through the scratch)
    big = _case(ctx, W.scaled(W.CONFIGS[1], L=3, H=4, Hq=16, b_min=8, R=0.5), [9000], seed=21)
    # second call: fewer, shorter segments, an empty one among them
    small_w = W.scaled(W.CONFIGS[0], L=2, H=2, Hq=14, b_min=0, R=0.3)
    small = _case(ctx, small_w, [700, 300], seed=22)
    for name, run in (("first (large)", big), ("second (smaller)", small)):
        out, lse = _decode_static(ctx, run)
        assert torch.equal(out, run.out), f"{name}: output differs from lkv_decode_attn"
        assert torch.equal(lse, run.lse), f"{name}: lse differs from lkv_decode_attn"
    # and once more the large one, after the small one has left its partials behind
    out, lse = _decode_static(ctx, big)
    assert torch.equal(out, big.out) and torch.equal(lse, big.lse)


def test_static_scratch_decode_refuses_what_does_not_fit(ctx):
    # 2^17 segments x 16 query heads per KV head need far more than the static array holds; refused on the host
    lib = lkv.load_library()
    n_seq, L, H, Hq = 64, 64, 32, 512
    need = lkv.lkv_decode_workspace_bytes(n_seq * L * H, 0, Hq, H)
    assert need > lkv.DECODE_STATIC_SCRATCH_BYTES
    one = torch.zeros(256, dtype=torch.int32, device="cuda")
    st = lib.lkv_decode_attn_static(ctx.h, n_seq, L, H, Hq, 128, one.data_ptr(), one.data_ptr(), one.data_ptr(),
                                    one.data_ptr(), 0, C.c_float(G.SCALE), one.data_ptr(), None, None)
    assert st == 3 and b"static array" in lib.lkv_last_error(ctx.h)
