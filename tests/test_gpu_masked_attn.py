"""GPU parity of the training-time attention with a multiplicative mask (App. B) against the
fp64 oracle, through the C ABI.  The bound on the outputs is the decode bound (2e-2 of the
output scale of the query row); the log-normaliser is held to 1e-3 absolute."""
import numpy as np
import pytest
import torch

from oracle import lkv_oracle as O
from oracle import masked_attn as MA
from paper_2605_06676_amd import lkv
from paper_2605_06676_amd import workloads as W
from tests.gpu_util import SCALE, assert_decode_close, bf16_gpu_to_bits, bits_to_bf16_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = lkv.Context(0)
    yield c
    c.close()


def run_forward(ctx, q, k, v, m):
    tq, tk, tv = (bits_to_bf16_gpu(x) for x in (q, k, v))
    tm = torch.from_numpy(m).cuda()
    o = torch.full(tq.shape, float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full(tq.shape[:2], float("nan"), dtype=torch.float32, device="cuda")
    lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, tm, SCALE, o, lse)
    torch.cuda.synchronize()
    return o.cpu().numpy(), lse.cpu().numpy()


def check_forward(ctx, Hq, H, T, seed=0, mask=None):
    q, k, v, m, _ = W.draw_training_attention(Hq, H, T, seed)
    if mask is not None:
        m = mask(m)
    o_gpu, lse_gpu = run_forward(ctx, q, k, v, m)
    o_ref, lse_ref = MA.forward(*(O.bf16_bits_to_f64(x) for x in (q, k, v)), m, SCALE)
    return assert_decode_close(o_gpu.reshape(-1, 128), lse_gpu.reshape(-1), o_ref.reshape(-1, 128), lse_ref.reshape(-1),
                               f"Hq{Hq} H{H} T{T}")


@pytest.mark.parametrize("Hq,H,T", [(4, 2, 300), (2, 2, 1), (1, 1, 33), (4, 1, 128), (2, 1, 129), (7, 1, 257), (8, 2, 1000), (16, 1, 70), (3, 3, 64),
                                    (6, 2, 513)])
def test_forward_small(ctx, Hq, H, T):
    check_forward(ctx, Hq, H, T)


def test_forward_wide_blocks(ctx):
    # long enough for the 256-query blocks, ragged against every tile size
    check_forward(ctx, 2, 1, 8192 + 77)


def test_forward_mask_edge_cases(ctx):
    def zero_prefix(m):
        m = m.copy()
        m[:, :37] = 0.0          # the first 37 queries see no weight at all: zero output, lse = -inf
        return m

    check_forward(ctx, 4, 2, 200, mask=zero_prefix)
    check_forward(ctx, 4, 2, 200, mask=lambda m: np.ones_like(m))                       # plain causal attention
    check_forward(ctx, 4, 2, 200, mask=lambda m: (m > 0.2).astype(np.float32))   # 0/1 mask, first key kept


def test_forward_rejects_bad_arguments(ctx):
    q, k, v, m, _ = W.draw_training_attention(4, 2, 64)
    tq, tk, tv = (bits_to_bf16_gpu(x) for x in (q, k, v))
    tm = torch.from_numpy(m).cuda()
    o = torch.empty(tq.shape, dtype=torch.float32, device="cuda")
    lse = torch.empty(tq.shape[:2], dtype=torch.float32, device="cuda")
    with pytest.raises(lkv.LkvError):
        lkv.lkv_masked_attn_forward(ctx, tq, tk[:1].repeat(3, 1, 1), tv, tm, SCALE, o, lse)   # 4 query heads, 3 KV heads
    with pytest.raises(lkv.LkvError):
        lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, tm, 0.0, o, lse)
    with pytest.raises(lkv.LkvError):
        lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, None, SCALE, o, lse)
    with pytest.raises(lkv.LkvError):
        lkv.lkv_masked_attn_forward(ctx, tq[:, :, :64].contiguous(), tk, tv, tm, SCALE, o, lse)   # head_dim 64


# ---- backward -------------------------------------------------------------------------------------
# Every gradient element is an fp32 sum of products in which one factor (P or dS) was rounded to bf16 on
# its way through the matrix cores (relative error up to 2^-9).  On top of that the per-query quantities the
# backward pass takes from the forward one (o_i in D_i = dO_i . o_i, and lse_i) carry the forward pass's own
# rounding of P, and an error dD_i enters every dS_ij of the row as p_ij dD_i whatever the size of the
# row's own gradient (the second query has two keys whose dS cancel: its dQ is small, the inherited error
# is not).  Hence a relative and an absolute part: per row, max error <= 2e-2 * (scale of the row: the
# larger of its biggest entry and its rms) + 2e-3 * (rms of the whole gradient tensor).
GRAD_RTOL = 2e-2
GRAD_ATOL_OF_RMS = 2e-3


def assert_rows_close(got, ref, what):
    ref = ref.reshape(-1, ref.shape[-1]).astype(np.float64)
    got = got.reshape(ref.shape).astype(np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    err = np.abs(got - ref).max(axis=-1)
    scale = np.maximum(np.abs(ref).max(axis=-1), np.sqrt((ref ** 2).mean(axis=-1)))
    if not np.any(ref):
        # a gradient that vanishes identically (a single key: dS = 0) comes out at the rounding level of
        # o = (p v) * (1 / l); the inputs are N(0, 1), so 1e-4 is far below any real gradient
        assert err.max() <= 1e-4, f"{what}: a gradient that must vanish is {err.max():.3g}"
        return
    tol = GRAD_RTOL * scale + GRAD_ATOL_OF_RMS * np.sqrt((ref ** 2).mean())
    bad = err > tol
    assert not bad.any(), f"{what}: {bad.sum()} rows out of tolerance, worst ratio {(err / tol).max():.3g}"


def run_backward(ctx, q, k, v, m, d_o):
    tq, tk, tv, tg = (bits_to_bf16_gpu(x) for x in (q, k, v, d_o))
    tm = torch.from_numpy(m).cuda()
    o = torch.empty(tq.shape, dtype=torch.float32, device="cuda")
    lse = torch.empty(tq.shape[:2], dtype=torch.float32, device="cuda")
    lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, tm, SCALE, o, lse)
    nan = float("nan")
    dq = torch.full(tq.shape, nan, dtype=torch.float32, device="cuda")
    dk = torch.full(tk.shape, nan, dtype=torch.float32, device="cuda")
    dv = torch.full(tk.shape, nan, dtype=torch.float32, device="cuda")
    dm = torch.full(tm.shape, nan, dtype=torch.float32, device="cuda")
    ws = torch.empty(lkv.lkv_masked_attn_backward_workspace_bytes(tq.shape[0], tk.shape[0], tq.shape[1]), dtype=torch.uint8, device="cuda")
    lkv.lkv_masked_attn_backward(ctx, tq, tk, tv, tm, o, lse, tg, SCALE, dq, dk, dv, dm, ws)
    torch.cuda.synchronize()
    return [x.cpu().numpy() for x in (dq, dk, dv, dm)]


def check_backward(ctx, Hq, H, T, seed=0, mask=None):
    q, k, v, m, d_o = W.draw_training_attention(Hq, H, T, seed)
    if mask is not None:
        m = mask(m)
    dq, dk, dv, dm = run_backward(ctx, q, k, v, m, d_o)
    rq, rk, rv, rm = MA.backward(*(O.bf16_bits_to_f64(x) for x in (q, k, v)), m, SCALE, O.bf16_bits_to_f64(d_o))
    tag = f"Hq{Hq} H{H} T{T}"
    assert_rows_close(dq, rq, tag + " dQ")
    assert_rows_close(dk, rk, tag + " dK")
    assert_rows_close(dv, rv, tag + " dV")
    assert_rows_close(dm, rm, tag + " dm")   # one row per KV head: the mask gradient of a head is judged as a vector


@pytest.mark.parametrize("Hq,H,T", [(4, 2, 300), (2, 2, 1), (1, 1, 33), (4, 1, 128), (2, 1, 129), (7, 1, 257), (8, 2, 1000), (16, 1, 70), (3, 3, 64),
                                    (6, 2, 513)])
def test_backward_small(ctx, Hq, H, T):
    check_backward(ctx, Hq, H, T)


def test_backward_mask_edge_cases(ctx):
    def zero_prefix(m):
        m = m.copy()
        m[:, :37] = 0.0          # 37 queries without any weight: they contribute nothing, and dm stays finite
        return m

    check_backward(ctx, 4, 2, 200, mask=zero_prefix)
    check_backward(ctx, 4, 2, 200, mask=lambda m: np.ones_like(m))
    check_backward(ctx, 4, 2, 200, mask=lambda m: (m > 0.2).astype(np.float32))


def test_backward_is_reproducible(ctx):
    # no atomics: two runs give the same bits
    q, k, v, m, d_o = W.draw_training_attention(8, 2, 777, 3)
    a = run_backward(ctx, q, k, v, m, d_o)
    b = run_backward(ctx, q, k, v, m, d_o)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_backward_rejects_small_workspace(ctx):
    q, k, v, m, d_o = W.draw_training_attention(4, 2, 64)
    tq, tk, tv, tg = (bits_to_bf16_gpu(x) for x in (q, k, v, d_o))
    tm = torch.from_numpy(m).cuda()
    o = torch.zeros(tq.shape, dtype=torch.float32, device="cuda")
    lse = torch.zeros(tq.shape[:2], dtype=torch.float32, device="cuda")
    dq = torch.empty(tq.shape, dtype=torch.float32, device="cuda")
    dk = torch.empty(tk.shape, dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    dm = torch.empty_like(tm)
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(lkv.LkvError) as e:
        lkv.lkv_masked_attn_backward(ctx, tq, tk, tv, tm, o, lse, tg, SCALE, dq, dk, dv, dm, ws)
    assert e.value.status == 3


@pytest.mark.parametrize("Hq,H,T", [(32, 8, 16384), (4, 1, 131072 + 5)])
def test_full_size_sampled(ctx, Hq, H, T):
    """Llama-3.1-8B's attention shape (32 query heads, 8 KV heads) at the longest training length of
    the paper (16k tokens, App. C.2), in the launch configuration bench.py times.  Checked on what the
    oracle can compute row by row: forward rows and dQ rows of sampled queries, dK / dV / dm of the last
    keys (complete once every later query is included), and two identities that hold at any size:
    sum_j dV_j = sum_i dO_i over the group's queries (the weights of a row sum to 1) and
    sum_j m_j dm_j = 0 (scaling a head's mask changes nothing).  The second case is one GQA group over a
    context eight times longer, ragged against every tile size (index arithmetic at length)."""
    G = Hq // H
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20260506)
    tq = torch.randn((Hq, T, 128), device="cuda", generator=gen).to(torch.bfloat16)
    tk = torch.randn((H, T, 128), device="cuda", generator=gen).to(torch.bfloat16)
    tv = torch.randn((H, T, 128), device="cuda", generator=gen).to(torch.bfloat16)
    tg = torch.randn((Hq, T, 128), device="cuda", generator=gen).to(torch.bfloat16)
    x = torch.rand((H, T), device="cuda", generator=gen)
    pick = torch.rand((H, T), device="cuda", generator=gen)
    tm = (x * x) * (x * x)
    tm[pick < 0.10] = 0.0
    tm[pick > 0.95] = 1.0
    tm[:, 0] = torch.clamp(tm[:, 0], min=0.25)
    o = torch.empty((Hq, T, 128), dtype=torch.float32, device="cuda")
    lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
    lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, tm, SCALE, o, lse)
    dq = torch.empty_like(o)
    dk = torch.empty((H, T, 128), dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    dm = torch.empty_like(tm)
    ws = torch.empty(lkv.lkv_masked_attn_backward_workspace_bytes(Hq, H, T), dtype=torch.uint8, device="cuda")
    lkv.lkv_masked_attn_backward(ctx, tq, tk, tv, tm, o, lse, tg, SCALE, dq, dk, dv, dm, ws)
    torch.cuda.synchronize()

    # identities over everything
    dv_sum = dv.double().sum(dim=1)                                            # [H, 128]
    do_sum = tg.double().view(H, G, T, 128).sum(dim=(1, 2))
    scale_dv = tg.double().abs().view(H, G, T, 128).sum(dim=(1, 2))
    assert (dv_sum - do_sum).abs().max().item() <= 2.0 ** -9 * scale_dv.max().item()
    along = (dm.double() * tm.double()).sum(dim=1)
    assert along.abs().max().item() <= 2.0 ** -9 * (dm.double() * tm.double()).abs().sum(dim=1).max().item()

    # one KV head and its group on the host; the last `tail` queries and a few scattered ones
    tail = 150
    for h in (0, H - 1):
        heads = slice(h * G, (h + 1) * G)
        q, g = (O.bf16_bits_to_f64(bf16_gpu_to_bits(x[heads])) for x in (tq, tg))
        k, v = (O.bf16_bits_to_f64(bf16_gpu_to_bits(x[h:h + 1])) for x in (tk, tv))
        m = tm[h:h + 1].cpu().numpy()
        rows = [0, 1, 63, 64, 255, 256, 4097, 9000, T // 2 + 1] + list(range(T - tail, T))
        o_ref, lse_ref = MA.forward(q, k, v, m, SCALE, rows=rows)
        assert_decode_close(o[heads][:, rows].cpu().numpy().reshape(-1, 128), lse[heads][:, rows].cpu().numpy().reshape(-1),
                            o_ref[:, rows].reshape(-1, 128), lse_ref[:, rows].reshape(-1), f"full size head {h} forward")
        rq, rk, rv, rm = MA.backward(q, k, v, m, SCALE, g, rows=rows)
        assert_rows_close(dq[heads][:, rows].cpu().numpy(), rq[:, rows], f"full size head {h} dQ")
        keys = slice(T - tail, T)
        assert_rows_close(dk[h:h + 1, keys].cpu().numpy(), rk[:, keys], f"full size head {h} dK")
        assert_rows_close(dv[h:h + 1, keys].cpu().numpy(), rv[:, keys], f"full size head {h} dV")
        assert_rows_close(dm[h:h + 1, keys].cpu().numpy(), rm[:, keys], f"full size head {h} dm")


def test_random_shapes(ctx):
    # seeded draws of head counts and lengths, forward and backward, every element against the oracle
    rng = np.random.default_rng(7)
    for case in range(12):
        H = int(rng.integers(1, 4))
        G = int(rng.choice([1, 2, 3, 4, 8]))
        T = int(rng.integers(1, 420))
        check_forward(ctx, H * G, H, T, seed=100 + case)
        check_backward(ctx, H * G, H, T, seed=100 + case)
