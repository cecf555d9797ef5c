"""Dataset-free end-to-end run: a noisy quadratic (PL, smooth, bounded gradient variance: the
setting of Theorems 1-2) trained with AdaScale at several scales until tau >= T_SI.  Checks the
driver loop and stopping rule, the iteration bounds of Sec. 3.2, that the final objective does
not degrade with S (the scale-invariance claim), and agreement with the CPU oracle fed the same
gradients."""
import math

import numpy as np
import pytest
import torch

import workloads as W
from oracle.oracle import Oracle
from paper_2007_05105_amd import AdaScale, run_until_done

pytestmark = pytest.mark.gpu

D, L = 20000, 400


def problem():
    rng = np.random.default_rng(0)
    h = torch.tensor(rng.uniform(0.5, 2.0, D), dtype=torch.float32, device="cuda:0")
    c = torch.tensor(rng.normal(size=D), dtype=torch.float32, device="cuda:0")
    lr = W.lr_exponential_decay(0.05, L, 0.1)
    return h, c, lr


def train(S, with_oracle):
    h, c, lr = problem()
    w = [torch.zeros(D, device="cuda:0")]
    v = [torch.zeros(D, device="cuda:0")]
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(100 + S)
    ada = AdaScale([D], S, lr, momentum=0.9)
    orc = Oracle(S, lr, momentum=0.9) if with_oracle else None
    w64, v64 = [np.zeros(D)], [np.zeros(D)]
    grads = [[torch.empty(D, device="cuda:0")] for _ in range(S)]
    log = []

    def make_grads(t):
        base = h * (w[0] - c)                      # gradient of 0.5 * sum h (w - c)^2 at the current w
        for i in range(S):
            grads[i][0].copy_(base + torch.randn(D, generator=gen, device="cuda:0"))
        return grads

    def on_step(t, st):
        if orc is not None:
            ost = orc.step(w64, v64, [[g[0].cpu().numpy()] for g in grads])
            log.append((st.r, ost.r, st.tau, ost.tau, st.done, ost.done))

    steps = run_until_done(ada, w, v, make_grads, max_steps=L + 5, on_step=on_step)
    st = ada.get_state()
    loss = float(0.5 * torch.sum(h * (w[0] - c) ** 2))
    ada.close()
    return steps, loss, st, log, (w[0].cpu().numpy(), w64[0])


def test_noisy_quadratic_reaches_t_si_at_every_scale():
    h, c, _ = problem()
    f0 = float(0.5 * torch.sum(h * c ** 2))
    results = {S: train(S, with_oracle=(S in (1, 16))) for S in (1, 4, 16)}
    steps = {S: r[0] for S, r in results.items()}
    loss = {S: r[1] for S, r in results.items()}
    print("iterations", steps, "final objective", loss, "initial", f0, flush=True)
    for S, (n, f, st, log, (w_gpu, w_or)) in results.items():
        assert st.done and st.tau >= L
        assert math.ceil(L / S) <= n <= L                        # iteration bounds, Sec. 3.2
        assert st.tau - st.r < L                                 # stopped at the first iteration past T_SI
        assert f < 0.05 * f0
        for r_gpu, r_or, tau_gpu, tau_or, d_gpu, d_or in log:    # same gradients into the oracle
            assert abs(r_gpu - r_or) <= 1e-5 * r_or and abs(tau_gpu - tau_or) <= 1e-5 * tau_or and d_gpu == d_or
        if log:
            assert np.abs(w_gpu - w_or).max() <= 2e-5 * np.abs(w_or).max()
    assert steps[1] == L and steps[1] > steps[4] > steps[16]     # S = 1: r = 1, tau = t
    assert loss[4] <= 1.1 * loss[1] and loss[16] <= 1.1 * loss[1]   # quality does not degrade with scale


def test_linear_scaling_baseline_runs_through_a_scale_one_context():
    """The comparison run of Sec. 4 (linear scaling with warm-up) through the same library: a
    scale-1 context (gain 1, clock = iteration count) given the LSW table and the mean of the S
    gradients.  Checks the plumbing -- ceil(T/S) iterations, eta_t = table[t] -- and prints the
    objective next to AdaScale's; no claim is tested on it."""
    from paper_2007_05105_amd import schedules as SCH
    S = 16
    h, c, lr = problem()
    table = SCH.lsw_schedule(lr, S)
    assert len(table) == math.ceil(L / S)
    w, v = [torch.zeros(D, device="cuda:0")], [torch.zeros(D, device="cuda:0")]
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(100 + S)
    ada = AdaScale([D], 1, table, momentum=0.9)
    gbar = [[torch.empty(D, device="cuda:0")]]
    seen = []

    def make_grads(t):
        base = h * (w[0] - c)
        noise = torch.randn(S, D, generator=gen, device="cuda:0").mean(dim=0)
        gbar[0][0].copy_(base + noise)
        return gbar

    steps = run_until_done(ada, w, v, make_grads, max_steps=L, on_step=lambda t, st: seen.append((t, st.r, st.tau, st.lr_eff)))
    ada.close()
    assert steps == len(table)
    for t, r, tau, eta in seen:
        assert r == 1.0 and tau == t and eta == float(table[t - 1])
    loss_lsw = float(0.5 * torch.sum(h * (w[0] - c) ** 2))
    _, loss_as, _, _, _ = train(S, with_oracle=False)
    print("S = 16: LSW objective", loss_lsw, "after", steps, "iterations; AdaScale", loss_as, flush=True)
    assert math.isfinite(loss_lsw)


def test_noisy_quadratic_sits_under_the_bound_of_theorem_2():
    """Theorem 2 (Sec. 3.3): for an alpha-PL, beta-smooth objective with gradient variance at most
    V, constant lr(t) = eta < 2/beta and S <= 1/gamma, AdaScale SGD (no momentum) ends with
        E[F(w_T) - F*] <= (1 - gamma)^(rbar T) [F(w_0) - F*] + Delta,
        gamma = eta alpha (2 - eta beta),  Delta = eta^2 beta V / (2 gamma),
    where rbar T = tau_T: the same bound, with the same constants, at every scale.  Here
    F(w) = 1/2 sum_j h_j (w_j - c_j)^2 with h_j in [0.5, 2] (alpha = 0.5, beta = 2), per-batch
    gradients = the exact gradient + N(0, 1) noise per coordinate (V = d), F* = 0.  F is a sum over
    20000 independent coordinates, so one run sits within about a percent of its expectation.  The
    run stops when tau >= T_SI, so the bound is evaluated at the tau the run ended with; it is
    checked at two budgets: the first term shrinks with T_SI, the floor Delta does not depend on S."""
    h, c, _ = problem()
    alpha, beta, eta, V = 0.5, 2.0, 0.05, float(D)
    assert float(h.min()) >= alpha and float(h.max()) <= beta
    gamma = eta * alpha * (2.0 - eta * beta)
    delta = eta ** 2 * beta * V / (2.0 * gamma)
    f0 = float(0.5 * torch.sum(h * c ** 2))
    seen = {}
    for budget in (100, 400):
        for S in (1, 4, 16):
            assert S <= 1.0 / gamma                                     # the theorem's condition on the scale
            w, v = [torch.zeros(D, device="cuda:0")], [torch.zeros(D, device="cuda:0")]
            gen = torch.Generator(device="cuda:0")
            gen.manual_seed(1000 * budget + S)
            ada = AdaScale([D], S, np.full(budget, eta, dtype=np.float32), momentum=0.0)
            grads = [[torch.empty(D, device="cuda:0")] for _ in range(S)]

            def make_grads(t):
                base = h * (w[0] - c)
                for i in range(S):
                    grads[i][0].copy_(base + torch.randn(D, generator=gen, device="cuda:0"))
                return grads

            steps = run_until_done(ada, w, v, make_grads, max_steps=budget)
            st = ada.get_state()
            ada.close()
            f = float(0.5 * torch.sum(h * (w[0] - c) ** 2))
            bound = (1.0 - gamma) ** st.tau * f0 + delta
            seen[(budget, S)] = (steps, st.tau, f, bound)
            print(f"T_SI {budget} S {S}: {steps} iterations, tau {st.tau:.1f}, F - F* = {f:.1f}, bound {bound:.1f} "
                  f"(floor {delta:.1f}, start {f0:.1f})", flush=True)
            assert st.done and math.ceil(budget / S) <= steps <= budget
            assert f <= bound
    # the bound says something: its floor is a small part of the initial gap, and at the larger
    # budget the first term has gone, so every scale sits under the same number
    assert delta < 0.1 * f0
    assert max(seen[(400, S)][3] for S in (1, 4, 16)) <= 1.0001 * delta
    assert seen[(400, 16)][0] < seen[(400, 4)][0] < seen[(400, 1)][0] == 400


def test_run_log_has_one_record_per_poll(tmp_path):
    """The per-step log of the driver loop: iteration, gain, learning rate, clock, estimates."""
    import json
    S, budget = 4, 40
    h, c, _ = problem()
    w, v = [torch.zeros(D, device="cuda:0")], [torch.zeros(D, device="cuda:0")]
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(5)
    ada = AdaScale([D], S, np.full(budget, 0.05, dtype=np.float32))
    grads = [[torch.empty(D, device="cuda:0")] for _ in range(S)]

    def make_grads(t):
        base = h * (w[0] - c)
        for i in range(S):
            grads[i][0].copy_(base + torch.randn(D, generator=gen, device="cuda:0"))
        return grads

    path = tmp_path / "run.jsonl"
    steps = run_until_done(ada, w, v, make_grads, max_steps=budget, log_path=str(path))
    final = ada.get_state()
    ada.close()
    rows = [json.loads(l) for l in open(path)]
    assert [r["iteration"] for r in rows] == list(range(1, steps + 1))
    assert all(1.0 <= r["r"] <= S and r["step"] == r["iteration"] for r in rows)
    assert all(b["tau"] == a["tau"] + b["r"] for a, b in zip(rows, rows[1:]))      # tau_{t+1} = tau_t + r_t
    assert rows[-1]["done"] == 1 and rows[-1]["tau"] == final.tau and all(r["done"] == 0 for r in rows[:-1])
