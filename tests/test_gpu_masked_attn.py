"""GPU parity of the training-time attention with a multiplicative mask (App. B) against the
fp64 oracle, through the C ABI.  Outputs are bf16: the bound is the decode bound (2e-2 of the
output scale of the query row); the log-normaliser is fp32 and held to 1e-3 absolute."""
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
    o = torch.full(tq.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full(tq.shape[:2], float("nan"), dtype=torch.float32, device="cuda")
    lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, tm, SCALE, o, lse)
    torch.cuda.synchronize()
    return O.bf16_bits_to_f64(bf16_gpu_to_bits(o)), lse.cpu().numpy()


def check_forward(ctx, Hq, H, T, seed=0, mask=None):
    q, k, v, m, _ = W.draw_training_attention(Hq, H, T, seed)
    if mask is not None:
        m = mask(m)
    o_gpu, lse_gpu = run_forward(ctx, q, k, v, m)
    o_ref, lse_ref = MA.forward(*(O.bf16_bits_to_f64(x) for x in (q, k, v)), m, SCALE)
    return assert_decode_close(o_gpu.reshape(-1, 128), lse_gpu.reshape(-1), o_ref.reshape(-1, 128), lse_ref.reshape(-1),
                               f"Hq{Hq} H{H} T{T}")


@pytest.mark.parametrize("Hq,H,T", [(4, 2, 300), (2, 2, 1), (1, 1, 33), (4, 1, 128), (2, 1, 129), (7, 1, 257), (8, 2, 1000)])
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
    o = torch.empty_like(tq)
    lse = torch.empty(tq.shape[:2], dtype=torch.float32, device="cuda")
    with pytest.raises(lkv.LkvError):
        lkv.lkv_masked_attn_forward(ctx, tq, tk[:1].repeat(3, 1, 1), tv, tm, SCALE, o, lse)   # 4 query heads, 3 KV heads
    with pytest.raises(lkv.LkvError):
        lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, tm, 0.0, o, lse)
    with pytest.raises(lkv.LkvError):
        lkv.lkv_masked_attn_forward(ctx, tq, tk, tv, None, SCALE, o, lse)
    with pytest.raises(lkv.LkvError):
        lkv.lkv_masked_attn_forward(ctx, tq[:, :, :64].contiguous(), tk, tv, tm, SCALE, o, lse)   # head_dim 64
