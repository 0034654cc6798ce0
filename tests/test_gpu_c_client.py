"""The four hot calls driven from plain C (tests/c_abi_gpu_client.c): device memory from the HIP runtime's C
interface, no PyTorch in the process that computes.  The client also checks, on a live context, that the hot
calls refuse bad arguments before enqueueing anything.  Its results are compared with the oracle here, to the same
bar as everywhere else: scores to tolerance, selection and packed rows bit for bit on the GPU's own scores, decode
outputs to tolerance."""
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

from oracle import lkv_oracle as O  # noqa: E402
from paper_2605_06676_amd import lkv, workloads as W  # noqa: E402

pytestmark = pytest.mark.gpu


def _build(tmp_path):
    lkv.load_library()                                    # raises if the library has not been built
    libdir = os.path.dirname(lkv.LIB_PATH)
    exe = str(tmp_path / "c_abi_gpu_client")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
                    os.path.join(ROOT, "tests", "c_abi_gpu_client.c"), "-L", libdir, "-llkv", "-L", "/opt/rocm/lib",
                    "-lamdhip64", "-lm", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True)
    return exe


@pytest.mark.parametrize("kind,hidden,act,per_head,out_bias,T,g", [
    ("linear", 0, "gelu", False, False, 777, 4),
    ("mlp", 64, "gelu", False, True, 1301, 2),
    ("mlp", 128, "silu", True, False, 530, 4),
])
def test_hot_path_from_plain_c(tmp_path, kind, hidden, act, per_head, out_bias, T, g):
    import gpu_util as G

    L, H = 2, 2
    w = W.scaled(W.CONFIGS[0], L=L, H=H, Hq=H * g, T=T, scorer=kind, hidden=hidden, act=act, per_head=per_head,
                 out_bias=out_bias)
    Kb, Vb = W.draw_kv(w, T, 0)
    qb = W.draw_q(w, 0)
    sc = W.draw_scorer(w)
    budgets = W.draw_budgets(w, T).astype(np.int32)
    budgets[0, 0] = 0                                     # an empty head and a head kept whole
    budgets[1, 1] = T
    has_b2 = int(kind == "mlp" and sc["b2"] is not None)
    head = np.array([L, H, H * g, T, int(kind == "mlp"), hidden, int(act == "gelu"), int(per_head), has_b2], dtype=np.int32)
    src = tmp_path / "in.bin"
    with open(src, "wb") as f:
        f.write(head.tobytes())
        f.write(np.ascontiguousarray(Kb).tobytes())
        f.write(np.ascontiguousarray(Vb).tobytes())
        f.write(np.ascontiguousarray(sc["w1"]).tobytes())
        f.write(np.ascontiguousarray(sc["b1"], dtype=np.float32).tobytes())
        if kind == "mlp":
            f.write(np.ascontiguousarray(sc["w2"], dtype=np.float32).tobytes())
            if has_b2:
                f.write(np.ascontiguousarray(sc["b2"], dtype=np.float32).tobytes())
        f.write(np.ascontiguousarray(budgets).tobytes())
        f.write(np.ascontiguousarray(qb).tobytes())
    dst = tmp_path / "out.bin"
    res = subprocess.run([_build(tmp_path), str(src), str(dst)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0 and "c gpu client ok" in res.stdout, res.stderr

    raw = open(dst, "rb").read()
    pos = 0

    def take(dtype, n):
        nonlocal pos
        a = np.frombuffer(raw, dtype=dtype, count=n, offset=pos)
        pos += a.nbytes
        return a

    total = int(take(np.int64, 1)[0])
    assert total == int(budgets.sum())
    u_gpu = take(np.float32, L * H * T).reshape(L, H, T)
    off_gpu = take(np.int32, L * H + 1)
    idx_gpu = take(np.int32, total)
    kp_gpu = take(np.uint16, total * 128).reshape(total, 128)
    vp_gpu = take(np.uint16, total * 128).reshape(total, 128)
    o_gpu = take(np.float32, L * H * g * 128).reshape(-1, 128)
    lse_gpu = take(np.float32, L * H * g)
    assert pos == len(raw)

    u_ref = O.score(O.bf16_bits_to_f64(Kb), O.bf16_bits_to_f64(Vb), G.scorer_to_oracle(sc))
    G.assert_scores_close(u_gpu, u_ref, "plain C client: scores")
    idx_ref, off_ref = O.select_all(u_gpu, budgets)
    assert np.array_equal(off_gpu, off_ref) and np.array_equal(idx_gpu, idx_ref)
    Kp_ref, Vp_ref = O.compact(Kb, Vb, idx_ref, off_ref)
    assert np.array_equal(kp_gpu, Kp_ref) and np.array_equal(vp_gpu, Vp_ref)
    o_ref, lse_ref = O.decode_attn(O.bf16_bits_to_f64(qb), O.bf16_bits_to_f64(Kp_ref), O.bf16_bits_to_f64(Vp_ref), off_ref,
                                   H, G.SCALE)
    G.assert_decode_close(o_gpu, lse_gpu, o_ref.reshape(-1, 128), lse_ref.reshape(-1), "plain C client: decode")
