"""Pins for the oracle's budgets and hard top-k (Sec. 3.1, 3.3, 3.4) and for the
Soft-TopK helper that serves as an independent check (Sec. 3.2, App. A.1).  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import lkv_oracle as O
from oracle import soft_topk as ST
from paper_2605_06676_amd import workloads as W


# ----- budgets --------------------------------------------------------------

def test_budget_floor_rule_and_total():
    r = np.array([[0.5, 0.1], [0.0999, 0.9999]])
    b = O.integer_budgets(r, 1000)
    assert b.tolist() == [[500, 100], [99, 999]]
    # sum of floors never exceeds the floor of the sum (the constraint of Sec. 3.1)
    rng = np.random.default_rng(0)
    for _ in range(50):
        L, H, t = 4, 8, int(rng.integers(100, 5000))
        R = float(rng.uniform(0.05, 0.5))
        p = rng.dirichlet(np.ones(L * H))
        r = np.minimum(p * R * L * H, 0.999)
        assert int(O.integer_budgets(r, t).sum()) <= O.total_budget(R, L, H, t)
    assert O.total_budget(0.15, 32, 8, 204800) == 7864320


def test_offsets_are_exclusive_prefix_sums():
    off = O.segment_offsets(np.array([[3, 0], [5, 1]]))
    assert off.tolist() == [0, 3, 3, 8, 9]


@pytest.mark.parametrize("cid", [0, 1, 2, 3, 4])
def test_workload_budget_generator_invariants(cid):
    w = W.CONFIGS[cid]
    T = int(W.seq_lengths(w)[0])
    b = W.draw_budgets(w, T)
    assert b.shape == (w.L, w.H)
    assert b.min() >= w.b_min and b.max() <= T
    assert int(b.sum()) <= O.total_budget(w.R, w.L, w.H, T)
    assert int(b.sum()) >= O.total_budget(w.R, w.L, w.H, T) - w.L * w.H
    if cid == 4:
        assert b.max() == T  # alpha = 0.1 drives at least one head into the cap


# ----- order key --------------------------------------------------------------

def test_order_key_is_monotone_and_handles_specials():
    vals = np.array([-np.inf, -3.5, -1e-40, -0.0, 0.0, 1e-40, 2.0, np.inf], dtype=np.float32)
    keys = O.order_key(vals)
    assert np.all(np.diff(keys.astype(np.int64)) > 0)        # strictly increasing, -0 < +0
    assert O.order_key(np.array([np.nan], dtype=np.float32))[0] == keys[0]  # NaN ranks as -inf
    rng = np.random.default_rng(1)
    x = rng.standard_normal(1000).astype(np.float32)
    k = O.order_key(x).astype(np.int64)
    i, j = rng.integers(0, 1000, 500), rng.integers(0, 1000, 500)
    assert np.array_equal(np.sign(x[i] - x[j]), np.sign(k[i] - k[j]))


# ----- hard top-k ------------------------------------------------------------

def _brute(u, b):
    ranked = sorted(range(len(u)), key=lambda i: (-float(u[i]), i))
    return sorted(ranked[:b])


@pytest.mark.parametrize("seed", range(6))
def test_select_matches_brute_force_sort(seed):
    rng = np.random.default_rng(seed)
    T = int(rng.integers(1, 300))
    u = rng.standard_normal(T).astype(np.float32)
    if seed % 2:
        u = np.round(u * 2) / 2          # many exact ties
    for b in {0, 1, T // 3, T - 1 if T > 1 else 0, T}:
        assert O.select(u, b).tolist() == _brute(u, b)


def _check_invariants(u, b, idx):
    T = u.size
    assert idx.dtype == np.int32 and idx.size == b
    assert np.all(np.diff(idx) > 0)
    if b:
        assert 0 <= idx[0] and idx[-1] < T
    kept = np.zeros(T, bool); kept[idx] = True
    key = O.order_key(u).astype(np.int64)
    if 0 < b < T:
        thr = key[kept].min()
        assert thr >= key[~kept].max()
        eq_kept = np.flatnonzero(kept & (key == thr))
        eq_drop = np.flatnonzero(~kept & (key == thr))
        if eq_drop.size:
            assert eq_kept.max() < eq_drop.min()


def test_select_invariants_on_workload_scores():
    w = W.scaled(W.CONFIGS[0], L=1, H=4, T=1024, b_min=8)
    K, V = W.draw_kv(w, 1024)
    sc = W.draw_scorer(w)
    u = O.score(O.bf16_bits_to_f64(K), O.bf16_bits_to_f64(V),
                {"kind": "linear", "w1": O.bf16_bits_to_f64(sc["w1"]), "b1": sc["b1"]})
    b = W.draw_budgets(w, 1024)
    idx, off = O.select_all(u, b)
    assert off[-1] == b.sum() and idx.size == b.sum()
    assert b.sum() / (w.L * w.H * 1024) <= w.R
    for h in range(4):
        _check_invariants(u[0, h], int(b[0, h]), idx[off[h]:off[h + 1]])


def test_select_forced_ties_keep_lowest_indices():
    u = np.full(100, 0.25, dtype=np.float32)
    assert O.select(u, 17).tolist() == list(range(17))
    # duplicated rows: the copy with the lower index wins
    u = np.array([1.0, 5.0, 3.0, 5.0, 3.0, 3.0, 0.0], dtype=np.float32)
    assert O.select(u, 1).tolist() == [1]
    assert O.select(u, 3).tolist() == [1, 2, 3]
    assert O.select(u, 4).tolist() == [1, 2, 3, 4]


def test_select_specials():
    u = np.array([np.nan, -np.inf, 0.0, -0.0, np.inf, np.nan], dtype=np.float32)
    assert O.select(u, 1).tolist() == [4]
    assert O.select(u, 2).tolist() == [2, 4]          # +0 before -0
    assert O.select(u, 3).tolist() == [2, 3, 4]
    assert O.select(u, 4).tolist() == [0, 2, 3, 4]    # NaN ties with -inf, lower index first
    assert O.select(u, 5).tolist() == [0, 1, 2, 3, 4]
    with pytest.raises(ValueError):
        O.select(u, 7)


def test_select_invariant_under_order_preserving_maps():
    rng = np.random.default_rng(5)
    u = rng.standard_normal(500).astype(np.float32)
    base = O.select(u, 77)
    assert np.array_equal(O.select(u * np.float32(4.0), 77), base)       # exact scaling by 2^2
    assert np.array_equal(O.select(np.exp(u.astype(np.float64)).astype(np.float32), 77), base)
    perm = rng.permutation(500)
    assert np.array_equal(np.sort(perm[O.select(u[perm], 77)]), base)     # relabelling tokens (tie-free)


# ----- Soft-TopK helper and its hard limit ------------------------------------

@pytest.mark.parametrize("seed", range(4))
def test_soft_topk_properties(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(5, 60))
    x = rng.standard_normal(n) * 2
    k = float(rng.uniform(0.5, n - 0.5))
    y = ST.soft_topk(x, k)
    assert np.all((y > 0) & (y < 1))
    assert y.sum() == pytest.approx(k, rel=1e-12)                          # normalisation
    order = np.argsort(x)
    assert np.all(np.diff(y[order]) >= -1e-15)                             # order preservation
    assert np.allclose(ST.soft_topk(x + 3.7, k), y, rtol=1e-10)             # translation invariance
    # the threshold solves the constraint as a root of sum f(x - lam) - k
    lam, m = ST.soft_topk_lambda(x, k)
    lo, hi = x.min() - 50, x.max() + 50
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if ST.laplace_cdf(x - mid).sum() > k:
            lo = mid
        else:
            hi = mid
    assert lam == pytest.approx(0.5 * (lo + hi), abs=1e-9)
    # and agrees with the printed closed form when the split index is interior
    if 1 <= m < n:
        xs = np.sort(x)[::-1]
        s1, s2 = np.exp(-xs[:m]).sum(), np.exp(xs[m:]).sum()
        assert lam == pytest.approx(math.log((math.sqrt((k - m) ** 2 + s1 * s2) - (k - m)) / s1), abs=1e-9)


def test_soft_topk_k1_is_softmax():
    rng = np.random.default_rng(9)
    x = rng.standard_normal(40) * 0.5      # flat enough: largest softmax probability < 1/2
    sm = np.exp(x - x.max()); sm /= sm.sum()
    assert sm.max() < 0.5
    assert np.allclose(ST.soft_topk(x, 1.0), sm, rtol=1e-12)


@pytest.mark.parametrize("seed", range(5))
def test_hard_topk_is_the_zero_temperature_limit_of_soft_topk(seed):
    rng = np.random.default_rng(100 + seed)
    T = int(rng.integers(20, 200))
    u = rng.standard_normal(T).astype(np.float32)
    assert np.unique(u).size == T          # tie-free
    b = int(rng.integers(1, T))
    soft = ST.soft_topk(u.astype(np.float64), float(b), tau=1e-4)
    mask = np.zeros(T); mask[O.select(u, b)] = 1.0
    assert np.array_equal(np.round(soft), mask)
    assert soft.sum() == pytest.approx(b, rel=1e-9)


def test_total_budget_is_a_floor():
    # B_total = floor(R L H t), Sec. 3.1: products that are not integers must round down
    assert O.total_budget(0.15, 32, 8, 32768) == 1258291          # 1258291.2
    assert O.total_budget(0.15, 32, 8, 1001) == 38438              # 38438.4
    assert O.total_budget(0.10, 32, 8, 131072) == 3355443          # 3355443.2
    assert O.total_budget(0.5, 1, 1, 7) == 3                       # 3.5
    assert np.array_equal(O.integer_budgets(np.array([0.5, 0.999, 0.25]), 7), [3, 6, 1])


# ---- Soft-TopK backward (App. A.2) ----------------------------------------------------------------

def _torch_closed_form(x, k, m):
    """y = f(x - lambda) with lambda from the closed form of App. A.1 at a fixed split index m, in torch (fp64):
    differentiating this expression is the route App. A.2 says it avoids, so autograd through it is independent
    of the implicit-function formulas the oracle uses."""
    xs, _ = torch.sort(x, descending=True)
    s1 = torch.exp(-xs[:m]).sum()
    s2 = torch.exp(xs[m:]).sum()
    d = k - m
    lam = torch.log((torch.sqrt(d * d + s1 * s2) - d) / s1)
    z = x - lam
    e = 0.5 * torch.exp(-z.abs())
    return torch.where(z >= 0, 1.0 - e, e), lam


@pytest.mark.parametrize("seed", range(4))
def test_soft_topk_backward_against_autograd_of_the_closed_form(seed):
    rng = np.random.default_rng(seed)
    n = 23
    x = rng.standard_normal(n) * 2.0
    k = float(rng.uniform(1.5, n - 1.5))
    g = rng.standard_normal(n)
    lam, m = ST.soft_topk_lambda(x, k)
    assert 1 <= m < n
    tx = torch.from_numpy(x).requires_grad_(True)
    tk = torch.tensor(k, dtype=torch.float64, requires_grad=True)
    y, tlam = _torch_closed_form(tx, tk, m)
    assert abs(float(tlam.detach()) - lam) < 1e-12
    (y * torch.from_numpy(g)).sum().backward()
    dx, dk = ST.soft_topk_backward(x, k, 1.0, g)
    assert np.allclose(dx, tx.grad.numpy(), rtol=0, atol=1e-12)
    assert abs(dk - float(tk.grad)) < 1e-12


def test_threshold_derivatives_of_app_a2_by_finite_differences():
    rng = np.random.default_rng(7)
    x = rng.standard_normal(17) * 1.5
    k = 5.3
    lam, _ = ST.soft_topk_lambda(x, k)
    w = ST.threshold_weights(x - lam)
    assert np.isclose(w.sum(), 1.0, rtol=0, atol=1e-14) and (w > 0).all()
    h = 1e-6
    for j in range(x.size):
        up, dn = x.copy(), x.copy()
        up[j] += h
        dn[j] -= h
        fd = (ST.soft_topk_lambda(up, k)[0] - ST.soft_topk_lambda(dn, k)[0]) / (2 * h)
        assert abs(fd - w[j]) < 1e-8                                     # d lambda / d x_j
    fd_k = (ST.soft_topk_lambda(x, k + h)[0] - ST.soft_topk_lambda(x, k - h)[0]) / (2 * h)
    assert abs(fd_k + 1.0 / ST.laplace_pdf(x - lam).sum()) < 1e-8        # d lambda / d k


@pytest.mark.parametrize("tau", [1.0, 0.3, 0.05])
def test_soft_topk_backward_by_finite_differences_and_identities(tau):
    rng = np.random.default_rng(11)
    n = 19
    x = rng.standard_normal(n)
    k, g = 6.25, rng.standard_normal(n)
    dx, dk = ST.soft_topk_backward(x, k, tau, g)
    h = 1e-6 * tau

    def loss(xx, kk):
        return float((ST.soft_topk(xx, kk, tau) * g).sum())

    for j in range(n):
        up, dn = x.copy(), x.copy()
        up[j] += h
        dn[j] -= h
        assert abs((loss(up, k) - loss(dn, k)) / (2 * h) - dx[j]) < 2e-7 / tau
    assert abs((loss(x, k + 1e-6) - loss(x, k - 1e-6)) / 2e-6 - dk) < 1e-7
    # the outputs always sum to k: a constant upstream gradient gives no input gradient and dL/dk = that constant
    dx1, dk1 = ST.soft_topk_backward(x, k, tau, np.full(n, 2.5))
    assert np.allclose(dx1, 0.0, atol=1e-15 / tau) and abs(dk1 - 2.5) < 1e-14
    # translation invariance of the forward: the input gradient sums to zero
    assert abs(dx.sum()) < 1e-12 / tau
    # linear in g
    dx2, dk2 = ST.soft_topk_backward(x, k, tau, 3.0 * g)
    assert np.allclose(dx2, 3.0 * dx, rtol=1e-13) and np.isclose(dk2, 3.0 * dk, rtol=1e-13)


def test_soft_topk_backward_cold_limit_stays_finite():
    # tau -> 0+: every f'(z) underflows, the hard top-k has zero gradient, and dL/dk is g at the element(s) nearest the threshold
    x = np.array([3.0, -1.0, 0.5, 2.0, -2.5])
    g = np.array([1.0, 2.0, 3.0, 4.0, 5.0])
    dx, dk = ST.soft_topk_backward(x, 2.0, 1e-4, g)
    assert np.isfinite(dx).all() and np.isfinite(dk) and np.allclose(dx, 0.0, atol=1e-300)
    # k = 2 puts the threshold midway (in x / tau) between the 2nd and 3rd largest inputs, 2.0 and 0.5: both weigh 1/2
    assert abs(dk - 0.5 * (4.0 + 3.0)) < 1e-9
