"""The HIP library against facts that do not pass through the CPU oracle: the hand-derived
two-iteration example, the closed forms the paper's propositions give, a library optimizer at
scale 1.  The oracle and the library's scalar kernel state the same formulas, so agreement
between the two says little about the reading of App. B.3 they share; these tests pin the
library's side of it directly (the oracle's side has its own pins)."""
import math
import os

import numpy as np
import pytest
import torch

import harness as H
from paper_2007_05105_amd import EST_NORM_RATIO, F32, FORCE_FUSED, FORCE_GENERAL, FORCE_STREAMING, LAGGED_R, AdaScale, Tuning

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(autouse=True, params=["fused", "three_kernel", "general"])
def tuning(request):
    return Tuning(force_path={"fused": FORCE_FUSED, "three_kernel": FORCE_STREAMING, "general": FORCE_GENERAL}[request.param])


def dev(a):
    return torch.tensor(np.asarray(a, dtype=np.float32), device="cuda:0")


def test_hand_derived_two_step_example(tuning):
    """tests/golden/two_step_example.txt: estimates, eps clamp, mean of the samples before the
    exponential average takes over, lr index floor(tau_t), momentum, tau (App. B.3, Sec. 3.2).
    Every quantity of the example is exact in fp32 storage except w (compared to fp32 rounding)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "two_step_example.txt")) if l[0].isdigit()]
    g = [([1, 2], [3, 0]), ([2, 2], [2, 2])]
    ada = AdaScale([2], 2, [0.125, 0.0625], momentum=0.9, weight_decay=0.0, theta=0.9, eps=1e-6, tuning=tuning)
    w, v = [dev([0, 0])], [dev([0, 0])]
    for row, (g1, g2) in zip(rows, g):
        ada.step(w, v, [[dev(g1)], [dev(g2)]])
        st = ada.get_state()
        exp = [float(x) for x in row[1:]]
        got = [st.sum_sq, st.sq_mean, st.sigma2_hat, st.mu2_hat, st.sigma2_bar, st.mu2_bar, st.r, st.lr_eff]
        np.testing.assert_allclose(got, exp[:8], rtol=1e-14, atol=1e-15)
        np.testing.assert_allclose(st.tau, exp[12], rtol=1e-14)
        np.testing.assert_allclose(v[0].cpu().numpy(), exp[8:10], rtol=2e-7)
        np.testing.assert_allclose(w[0].cpu().numpy(), exp[10:12], rtol=3e-7)
    ada.close()


@pytest.mark.parametrize("S", [2, 4, 16])
def test_identical_gradients_closed_form(S, tuning):
    """Zero variance (Prop. 1's setting): sigma2_hat = 0 is clamped to eps, mu2_hat = B, and with
    theta = 0 the gain is (eps + B)/(eps/S + B)."""
    d, eps = 3000, 1e-3
    g = np.random.default_rng(S).normal(size=d).astype(np.float32)
    B = float((g.astype(np.float64) ** 2).sum())
    ada = AdaScale([d], S, [0.1], theta=0.0, eps=eps, tuning=tuning)
    w, v = [torch.zeros(d, device="cuda:0")], [torch.zeros(d, device="cuda:0")]
    ada.step(w, v, [[dev(g)] for _ in range(S)])
    st = ada.get_state()
    assert abs(st.sigma2_hat) <= 1e-9 * B
    np.testing.assert_allclose([st.sq_mean, st.mu2_hat, st.sigma2_bar], [B, B, eps], rtol=1e-9)
    np.testing.assert_allclose(st.r, (eps + B) / (eps / S + B), rtol=1e-12)
    np.testing.assert_allclose(w[0].cpu().numpy(), -np.float32(st.lr_eff) * g, rtol=3e-7, atol=1e-12)
    ada.close()


@pytest.mark.parametrize("S", [2, 8])
def test_opposite_gradients_give_the_full_gain(S, tuning):
    """Mean gradient exactly zero: mu2_hat = -sigma2_hat/S < 0 is clamped to 0 and r = S exactly
    (the linear-scaling end of eq. 3); the mean of the samples then keeps it there."""
    d = 2000
    g = np.random.default_rng(3).normal(size=d).astype(np.float32)
    ada = AdaScale([d], S, [0.1, 0.05, 0.01], theta=0.5, tuning=tuning)
    w, v = [torch.ones(d, device="cuda:0")], [torch.zeros(d, device="cuda:0")]
    grads = [[dev(g if i % 2 == 0 else -g)] for i in range(S)]
    for t in range(2):
        ada.step(w, v, grads)
        st = ada.get_state()
        assert st.sq_mean == 0.0 and st.mu2_bar == 0.0 and st.r == float(S) and st.tau == float(S * (t + 1))
        np.testing.assert_allclose(st.sigma2_hat, S * float((g.astype(np.float64) ** 2).sum()) / (S - 1), rtol=1e-12)
    assert torch.equal(w[0], torch.ones(d, device="cuda:0"))        # a zero mean gradient moves nothing
    ada.close()


def test_ratio_of_norms_at_theta_zero(tuning):
    """Sec. 3.4: with no averaging and no clamp active r_t = (A/S)/B, A and B from numpy; both
    estimators agree on it, and sigma2_hat is the summed per-coordinate sample variance."""
    S, d = 6, 5000
    g = (np.random.default_rng(7).normal(size=(S, d)) + 0.5).astype(np.float32)
    g64 = g.astype(np.float64)
    A, B = (g64 ** 2).sum(), (g64.mean(axis=0) ** 2).sum()
    for flags, eps in ((0, 1e-6), (EST_NORM_RATIO, 1e-6)):
        ada = AdaScale([d], S, [0.1], theta=0.0, eps=eps, flags=flags, tuning=tuning)
        w, v = [torch.zeros(d, device="cuda:0")], [torch.zeros(d, device="cuda:0")]
        ada.step(w, v, [[dev(g[i])] for i in range(S)])
        st = ada.get_state()
        np.testing.assert_allclose([st.sum_sq, st.sq_mean], [A, B], rtol=1e-12)
        np.testing.assert_allclose(st.sigma2_hat, g64.var(axis=0, ddof=1).sum(), rtol=1e-10)
        want = (A / S + eps) / (B + eps) if flags else (A / S) / B
        np.testing.assert_allclose(st.r, want, rtol=1e-10)
        ada.close()


@pytest.mark.parametrize("wd", [0.0, 5e-4])
def test_scale_one_is_momentum_sgd(wd, tuning):
    """S = 1: r = 1, tau = t, and the trajectory is that of torch.optim.SGD (dampening 0, coupled
    L2) with lr(t) changing every step -- in fp32 on both sides, compared to a few roundings."""
    T, d, rho = 12, 4099, 0.9
    lr = (0.3 * 0.8 ** np.arange(T)).astype(np.float32)
    rng = np.random.default_rng(11)
    w0 = (rng.normal(size=d) * 0.1).astype(np.float32)
    g = [rng.normal(size=d).astype(np.float32) for _ in range(T)]
    ada = AdaScale([d], 1, lr, momentum=rho, weight_decay=wd, tuning=tuning)
    w, v = [dev(w0)], [torch.zeros(d, device="cuda:0")]
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=1.0, momentum=rho, weight_decay=wd)
    for t in range(T):
        ada.step(w, v, [[dev(g[t])]])
        st = ada.get_state()
        assert st.r == 1.0 and st.tau == float(t + 1) and st.sigma2_hat == 0.0
        np.testing.assert_allclose(st.lr_eff, float(lr[t]), rtol=1e-15)
        for grp in opt.param_groups:
            grp["lr"] = float(lr[t])
        p.grad = torch.tensor(g[t], dtype=torch.float64)
        opt.step()
    ref = p.detach().numpy()
    assert np.abs(w[0].cpu().numpy() - ref).max() <= 2e-6 * np.abs(ref).max()
    ada.close()


def test_lagged_gain_is_the_previous_iterations_gain(tuning):
    """App. B.3's own variant: r_t from the averages of prior iterations, r_0 = 1."""
    S, d, T = 4, 3000, 5
    rng = np.random.default_rng(5)
    gs = [(rng.normal(size=(S, d)) + 0.3).astype(np.float32) for _ in range(T)]
    cur = AdaScale([d], S, [0.01], theta=0.7, tuning=tuning)
    lag = AdaScale([d], S, [0.01], theta=0.7, flags=LAGGED_R, tuning=tuning)
    wc, vc = [torch.zeros(d, device="cuda:0")], [torch.zeros(d, device="cuda:0")]
    wl, vl = [torch.zeros(d, device="cuda:0")], [torch.zeros(d, device="cuda:0")]
    prev = 1.0
    for t in range(T):
        grads = [[dev(gs[t][i])] for i in range(S)]
        cur.step(wc, vc, grads)
        lag.step(wl, vl, grads)
        sc, sl = cur.get_state(), lag.get_state()
        # the gain the other variant had one step earlier (the two sum their partials in different orders)
        np.testing.assert_allclose(sl.r, prev, rtol=1e-12)
        np.testing.assert_allclose([sl.sigma2_bar, sl.mu2_bar], [sc.sigma2_bar, sc.mu2_bar], rtol=1e-12)
        prev = sc.r
    cur.close()
    lag.close()


def test_many_fused_launches_are_reproducible(tuning):
    """Six hundred steps, twice: the per-workgroup partials cross the grid barrier through
    memory-side atomics, and a partial read before it was written would show as a sum that
    differs between the runs (compared bit for bit every 25 steps, stopping at the first
    difference)."""
    from workloads import Inputs, custom
    wl = custom([(600000,), (999,), (70001,)], 8, weight_decay=1e-4, theta=0.9, steps=1, seed=13)
    logs = []
    for _ in range(2):
        inp = Inputs(wl, "cuda:0")
        inp.fill_grads(0)
        g = H.make_gpu(wl, tuning=tuning)
        log = []
        for t in range(600):
            g.step(inp.w, inp.v, inp.g)
            if t % 25 == 24:
                st = g.get_state()
                log.append((st.sum_sq, st.sq_mean, st.r, st.tau, float(inp.w_flat.double().sum())))
                if logs:
                    assert log[-1] == logs[0][len(log) - 1], f"runs differ at step {t}"
        logs.append(log)
        g.close()
