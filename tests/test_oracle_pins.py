"""Pins for the CPU oracle: facts the paper and the mathematics fix, each chosen so that a
plausible mistake in the oracle (dropped term, wrong sign, wrong index, swapped operand)
fails at least one of them.  CPU only.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle.oracle import BF16, EST_M1M2, F32, LAGGED_R, Oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed=0):
    return np.random.default_rng(seed)


def f32(a):
    return np.asarray(a, dtype=np.float32)


def run(S, grads_per_step, d=None, lr=(0.1,), w0=None, v0=None, **kw):
    """grads_per_step: list over steps of array [S, d] (single tensor).  Returns states, w, v."""
    d = grads_per_step[0].shape[1] if d is None else d
    o = Oracle(S, f32(lr), **kw)
    w = [np.zeros(d) if w0 is None else np.array(w0, dtype=np.float64)]
    v = [np.zeros(d) if v0 is None else np.array(v0, dtype=np.float64)]
    states = []
    for g in grads_per_step:
        st = o.step(w, v, [[f32(g[i])] for i in range(S)])
        states.append(st.as_dict())
    return states, w[0], v[0]


# ----------------------------------------------------------------------------- golden
def test_hand_derived_two_step_example():
    """Hand-derived example (tests/golden/two_step_example.txt): pins the estimates, the
    eps clamp, the running-mean warm start, the lr index floor(tau_t), momentum and tau."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "two_step_example.txt")) if l[0].isdigit()]
    g = [np.array([[1, 2], [3, 0]], float), np.array([[2, 2], [2, 2]], float)]
    o = Oracle(2, f32([0.125, 0.0625]), momentum=0.9, weight_decay=0.0, theta=0.9, eps=1e-6)
    w, v = [np.zeros(2)], [np.zeros(2)]
    for row, gt in zip(rows, g):
        st = o.step(w, v, [[f32(gt[0])], [f32(gt[1])]])
        exp = [float(x) for x in row[1:]]
        got = [st.sum_sq, st.sq_mean, st.sigma2_hat, st.mu2_hat, st.sigma2_bar, st.mu2_bar, st.r,
               st.lr_eff, v[0][0], v[0][1], w[0][0], w[0][1], st.tau]
        np.testing.assert_allclose(got, exp, rtol=1e-14, atol=1e-15)


# ------------------------------------------------------- S = 1 (proof of Theorem 1)
def test_scale_one_gives_unit_gain_and_plain_clock():
    g = [rng(t).normal(size=(1, 37)) for t in range(12)]
    states, _, _ = run(1, g, lr=np.linspace(0.5, 0.1, 12), theta=0.5)
    for t, st in enumerate(states):
        assert st["r"] == 1.0
        assert st["tau"] == float(t + 1)
        assert st["sigma2_hat"] == 0.0 and st["sigma2_bar"] == 0.0   # no eps clamp at S = 1
        assert st["mu2_hat"] == st["sq_mean"]


@pytest.mark.parametrize("wd", [0.0, 5e-4])
def test_scale_one_matches_library_momentum_sgd(wd):
    """With S = 1 AdaScale is Algorithm 1, i.e. momentum-SGD with lr(t): compare with
    torch.optim.SGD in fp64 (dampening 0, coupled L2), lr changing every step."""
    T, d, rho = 15, 23, 0.9
    lr = f32(0.3 * 0.8 ** np.arange(T))
    r = rng(3)
    w0 = r.normal(size=d) * 0.1
    g = [f32(r.normal(size=(1, d))) for _ in range(T)]
    _, w, v = run(1, g, lr=lr, w0=w0, momentum=rho, weight_decay=wd)
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=1.0, momentum=rho, weight_decay=wd)
    for t in range(T):
        for grp in opt.param_groups:
            grp["lr"] = float(lr[t])
        p.grad = torch.tensor(g[t][0], dtype=torch.float64)
        opt.step()
    np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-13, atol=1e-15)


# ------------------------------------------- zero variance (Proposition 1 setting)
def test_identical_gradients_closed_form():
    S, d, eps = 8, 50, 1e-6
    m = f32(rng(1).normal(size=d))
    B = float(np.dot(m.astype(np.float64), m.astype(np.float64)))
    states, _, _ = run(S, [np.tile(m, (S, 1))], theta=0.0, eps=eps)
    st = states[0]
    assert abs(st["sigma2_hat"]) <= 1e-12 * S * B          # exact zero up to rounding of A - S B
    assert st["sigma2_bar"] == eps                        # clamped
    np.testing.assert_allclose(st["mu2_hat"], B, rtol=1e-13)
    np.testing.assert_allclose(st["r"], (eps + B) / (eps / S + B), rtol=1e-12)
    assert 1.0 <= st["r"] < 1.0 + 1e-6


def test_deterministic_gradients_follow_the_single_batch_trajectory():
    """Zero gradient variance: scale S with AdaScale retraces S = 1 (identity scaling,
    Proposition 1) up to the eps clamp, whose effect on r is at most eps (1 - 1/S) / B."""
    T, d = 10, 16
    r = rng(5)
    gs = [f32(r.normal(size=d)) for _ in range(T)]
    lr = np.full(64, 0.05)
    _, w1, _ = run(1, [g[None, :] for g in gs], lr=lr, weight_decay=1e-3)
    _, w4, _ = run(4, [np.tile(g, (4, 1)) for g in gs], lr=lr, weight_decay=1e-3)
    np.testing.assert_allclose(w4, w1, rtol=0, atol=1e-5 * np.abs(w1).max())


# ------------------------------------------------- estimator identities (Sec. 3.4 / B.3)
@pytest.mark.parametrize("S", [2, 3, 5, 16])
def test_estimates_are_the_ratio_of_norms(S):
    """With theta = 0 and no clamp active, sigma2+mu2 = A/S, sigma2/S+mu2 = B and therefore
    r = (A/S)/B, the ratio-of-norms form of the gain (Sec. 3.4)."""
    d = 200
    g = f32(rng(S).normal(size=(S, d)) + 0.7)
    g64 = g.astype(np.float64)
    A = float((g64 ** 2).sum())
    gbar = g64.mean(axis=0)
    B = float((gbar ** 2).sum())
    st = run(S, [g], theta=0.0)[0][0]
    np.testing.assert_allclose(st["sum_sq"], A, rtol=1e-14)
    np.testing.assert_allclose(st["sq_mean"], B, rtol=1e-14)
    np.testing.assert_allclose(st["sigma2_hat"] + st["mu2_hat"], A / S, rtol=1e-12)
    np.testing.assert_allclose(st["sigma2_hat"] / S + st["mu2_hat"], B, rtol=1e-12)
    np.testing.assert_allclose(st["r"], (A / S) / B, rtol=1e-12)


@pytest.mark.parametrize("S,d", [(2, 1), (2, 16), (3, 7), (5, 16), (8, 3)])
def test_brute_force_small(S, d):
    """sigma2_hat is the sum over coordinates of the unbiased sample variance of the S
    values (sigma^2 = tr(Sigma)); mu2_hat = ||mean||^2 - sigma2_hat / S."""
    g = f32(rng(10 * S + d).normal(size=(S, d)) * 3 + 1)
    g64 = g.astype(np.float64)
    var = sum(np.var(g64[:, j], ddof=1) for j in range(d))
    mean = np.array([np.mean(g64[:, j]) for j in range(d)])
    o = Oracle(S, f32([0.1]), theta=0.0)
    w, v = [np.zeros(d)], [np.zeros(d)]
    st = o.step(w, v, [[g[i]] for i in range(S)])
    np.testing.assert_allclose(o.last_gbar[0], mean, rtol=1e-15)
    np.testing.assert_allclose(st.sigma2_hat, var, rtol=1e-12)
    np.testing.assert_allclose(st.mu2_hat, float(mean @ mean) - var / S, rtol=1e-11, atol=1e-13)
    # the first update from v = 0 is w = -eta * gbar
    np.testing.assert_allclose(w[0], -st.lr_eff * mean, rtol=1e-14)


def test_unbiasedness_monte_carlo():
    """E[sigma2_hat] = s^2 d and E[mu2_hat] = ||m||^2 (App. B.3) within 4 standard errors."""
    S, d, s, trials = 4, 64, 0.5, 4000
    r = rng(7)
    m = r.normal(size=d)
    sig, mu = [], []
    o = Oracle(S, f32([0.1]), theta=0.0)
    w, v = [np.zeros(d)], [np.zeros(d)]
    for _ in range(trials):
        g = f32(m + s * r.normal(size=(S, d)))
        st = o.step(w, v, [[g[i]] for i in range(S)])
        sig.append(st.sigma2_hat)
        mu.append(st.mu2_hat)
    for sample, truth in ((sig, s * s * d), (mu, float(m @ m))):
        se = np.std(sample, ddof=1) / math.sqrt(trials)
        assert abs(np.mean(sample) - truth) < 4 * se, (np.mean(sample), truth, se)


# --------------------------------------------------------------- range and extremes
def test_gain_stays_in_range():
    r = rng(11)
    for S in (2, 3, 7, 64):
        for signal in (0.0, 1e-3, 1.0, 1e3):
            for theta in (0.0, 0.9):
                g = [f32(signal + r.normal(size=(S, 9)) * r.choice([1e-20, 1.0, 1e3])) for _ in range(6)]
                for st in run(S, g, theta=theta)[0]:     # up to the rounding of one division
                    assert 1.0 - 1e-15 <= st["r"] <= S * (1 + 1e-15), (S, signal, theta, st)


def test_zero_mean_estimate_gives_linear_scaling():
    """mu2 clamped to 0 means r = S exactly (linear scaling); zero-mean iid noise comes close."""
    g1 = f32(rng(2).normal(size=33))
    st = run(2, [np.stack([g1, -g1])], theta=0.0)[0][0]
    assert st["sq_mean"] == 0.0 and st["mu2_hat"] < 0 and st["mu2_bar"] == 0.0
    assert st["r"] == 2.0
    S, d = 8, 20000
    st = run(S, [f32(rng(4).normal(size=(S, d)))], theta=0.0)[0][0]
    assert S * (1 - 6 / math.sqrt(d)) <= st["r"] <= S


def test_all_zero_gradients():
    st = run(4, [np.zeros((4, 5))], theta=0.0)[0][0]
    assert st["sigma2_bar"] == 1e-6 and st["mu2_bar"] == 0.0 and st["r"] == 4.0
    st = run(1, [np.zeros((1, 5))])[0][0]
    assert st["r"] == 1.0 and st["tau"] == 1.0


# ----------------------------------------------------------------------- symmetries
def test_scaling_invariance():
    S, d = 5, 40
    g = f32(rng(8).normal(size=(S, d)) + 0.3)
    a = run(S, [g], theta=0.0)[0][0]
    b = run(S, [g * 4.0], theta=0.0)[0][0]     # power of two: exact in floating point
    assert b["sigma2_hat"] == 16 * a["sigma2_hat"] and b["mu2_hat"] == 16 * a["mu2_hat"]
    assert b["r"] == a["r"]


def test_permutation_invariance_and_tensor_splitting():
    S, d = 6, 120
    r = rng(9)
    g = f32(r.normal(size=(S, d)) + 0.2)
    base = run(S, [g], theta=0.0)[0][0]
    perm_rep = run(S, [g[r.permutation(S)]], theta=0.0)[0][0]
    perm_el = run(S, [g[:, r.permutation(d)]], theta=0.0)[0][0]
    for other in (perm_rep, perm_el):
        for key in ("sigma2_hat", "mu2_hat", "r"):
            np.testing.assert_allclose(other[key], base[key], rtol=1e-12)
    # one tensor vs the same coordinates cut into four tensors: one global r (w in R^d)
    cuts = [0, 1, 50, 51, d]
    o = Oracle(S, f32([0.1]), theta=0.0)
    w = [np.zeros(cuts[i + 1] - cuts[i]) for i in range(4)]
    v = [np.zeros_like(x) for x in w]
    st = o.step(w, v, [[g[i, cuts[k]:cuts[k + 1]] for k in range(4)] for i in range(S)])
    for key in ("sum_sq", "sq_mean", "sigma2_hat", "mu2_hat", "r"):
        np.testing.assert_allclose(getattr(st, key), base[key], rtol=1e-13)
    _, w_one, _ = run(S, [g], theta=0.0)
    np.testing.assert_allclose(np.concatenate(w), w_one, rtol=1e-13)


# ------------------------------------------------------------ moving average, clock
def test_moving_average_is_mean_of_samples_then_exponential():
    """theta = 0.75: 1/(1-theta) = 4, so the first four averages are plain means of the
    samples so far, afterwards xbar <- theta xbar + (1 - theta) x."""
    S, d, theta, T = 2, 2, 0.75, 9
    r = rng(12)
    gs = [f32(r.integers(-4, 5, size=(S, d))) + np.array([[3.0, 3.0]]) for _ in range(T)]
    states = run(S, gs, theta=theta)[0]
    samples = [max(st["mu2_hat"], 0.0) for st in states]
    ssig = [max(st["sigma2_hat"], 1e-6) for st in states]
    avg_m = avg_s = None
    for t, st in enumerate(states):
        if t < 4:
            avg_m, avg_s = np.mean(samples[:t + 1]), np.mean(ssig[:t + 1])
        else:
            avg_m = theta * avg_m + (1 - theta) * samples[t]
            avg_s = theta * avg_s + (1 - theta) * ssig[t]
        np.testing.assert_allclose(st["mu2_bar"], avg_m, rtol=1e-13)
        np.testing.assert_allclose(st["sigma2_bar"], avg_s, rtol=1e-13)
        np.testing.assert_allclose(st["r"], (avg_s + avg_m) / (avg_s / S + avg_m), rtol=1e-13)


def test_default_theta_follows_scale():
    """theta = max(1 - S/1000, 0): S >= 1000 means no averaging, S = 500 means alpha = 0.5."""
    S, T = 4, 5
    gs = [f32(rng(t).normal(size=(S, 6)) + 1) for t in range(T)]
    a = run(S, gs, theta=-1.0)[0]
    b = run(S, gs, theta=1 - S / 1000)[0]
    assert [x["r"] for x in a] == [x["r"] for x in b]


def test_learning_rate_uses_floor_of_tau_before_the_step():
    S, T = 4, 12
    lr = f32(np.arange(1, 9) * 0.01)                     # distinct entries, L = 8
    gs = [f32(rng(t).normal(size=(S, 30)) * 2 + 0.5) for t in range(T)]
    states = run(S, gs, lr=lr, theta=0.5)[0]
    tau = 0.0
    for st in states:
        idx = min(int(math.floor(tau)), len(lr) - 1)
        np.testing.assert_allclose(st["lr_eff"], st["r"] * float(lr[idx]), rtol=1e-15)
        tau += st["r"]
        np.testing.assert_allclose(st["tau"], tau, rtol=1e-15)
        assert st["done"] == (tau >= len(lr))


@pytest.mark.parametrize("S", [1, 4, 16])
def test_iteration_count_bounds(S):
    """Reaching tau >= T_SI takes between ceil(T_SI / S) and T_SI iterations (Sec. 3.2)."""
    L, d = 40, 25
    o = Oracle(S, np.full(L, 0.01, dtype=np.float32), theta=0.0)
    w, v = [np.zeros(d)], [np.zeros(d)]
    r = rng(S)
    t = 0
    while not o.state().done:
        g = f32(r.normal(size=(S, d)) + 0.4)
        o.step(w, v, [[g[i]] for i in range(S)])
        t += 1
        assert t <= L
    assert math.ceil(L / S) <= t <= L


# ------------------------------------------------------------------ update equation
def test_weight_decay_is_outside_the_statistics_and_inside_the_update():
    S, d, lam, rho = 3, 10, 0.1, 0.5
    r = rng(13)
    g = f32(r.normal(size=(S, d)))
    w0, v0 = r.normal(size=d), r.normal(size=d)
    a = run(S, [g], w0=w0, v0=v0, weight_decay=0.0, momentum=rho, theta=0.0)
    b = run(S, [g], w0=w0, v0=v0, weight_decay=lam, momentum=rho, theta=0.0)
    assert a[0][0]["r"] == b[0][0]["r"] and a[0][0]["sigma2_hat"] == b[0][0]["sigma2_hat"]
    eta = b[0][0]["lr_eff"]
    gbar = g.astype(np.float64).mean(axis=0)
    v_exp = rho * v0 + gbar + lam * w0
    np.testing.assert_allclose(b[2], v_exp, rtol=1e-14)
    np.testing.assert_allclose(b[1], w0 - eta * v_exp, rtol=1e-13, atol=1e-15)


# -------------------------------------------------------------------- bf16 widening
def test_bf16_gradients_are_widened_exactly():
    S, d = 2, 64
    t = torch.randn(S, d, generator=torch.Generator().manual_seed(0)).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    exact = t.to(torch.float64).numpy()
    o = Oracle(S, f32([0.1]), theta=0.0, grad_dtype=BF16)
    w, v = [np.zeros(d)], [np.zeros(d)]
    st = o.step(w, v, [[bits[i]] for i in range(S)])
    np.testing.assert_allclose(o.last_gbar[0], exact.mean(axis=0), rtol=1e-15)
    np.testing.assert_allclose(st.sum_sq, (exact ** 2).sum(), rtol=1e-14)


# ------------------------------------------------- the two other variants in the paper
def test_lagged_gain_is_the_previous_iterations_current_gain():
    """App. B.3: the lagged variant plugs in averages of prior iterations and starts at r_0 = 1;
    the averages themselves do not depend on r, so lagged r_t = current-mode r_{t-1}."""
    S, T = 4, 8
    gs = [f32(rng(t).normal(size=(S, 20)) + 0.5) for t in range(T)]
    cur = run(S, gs, theta=0.8)[0]
    lag = run(S, gs, theta=0.8, flags=LAGGED_R)[0]
    assert lag[0]["r"] == 1.0
    for t in range(1, T):
        assert lag[t]["r"] == cur[t - 1]["r"]
        assert lag[t]["sigma2_bar"] == cur[t]["sigma2_bar"]
    np.testing.assert_allclose(lag[-1]["tau"], 1.0 + sum(c["r"] for c in cur[:-1]), rtol=1e-15)


def test_norm_ratio_estimator_matches_when_no_clamp_is_active():
    """Sec. 3.4: r = (m1 + eps)/(m2 + eps) with moving averages of A/S and B; App. B.3 calls the
    two estimators algebraically equivalent apart from the stability measures."""
    S, T, theta, eps = 4, 7, 0.7, 1e-6
    gs = [f32(rng(t).normal(size=(S, 50)) + 1.0) for t in range(T)]
    a = run(S, gs, theta=theta)[0]
    b = run(S, gs, theta=theta, flags=EST_M1M2, eps=eps)[0]
    for x, y in zip(a, b):
        assert x["mu2_hat"] > 0 and x["sigma2_hat"] > eps          # no clamp active
        m1, m2 = y["sigma2_bar"], y["mu2_bar"]
        np.testing.assert_allclose(m1, x["sigma2_bar"] + x["mu2_bar"], rtol=1e-12)
        np.testing.assert_allclose(m2, x["sigma2_bar"] / S + x["mu2_bar"], rtol=1e-12)
        np.testing.assert_allclose(y["r"], (m1 + eps) / (m2 + eps), rtol=1e-15)
        np.testing.assert_allclose(y["r"], x["r"], rtol=1e-6)
    # theta = 0: the literal one-sample form
    g = gs[0].astype(np.float64)
    A, B = (g ** 2).sum(), (g.mean(axis=0) ** 2).sum()
    y = run(S, [gs[0]], theta=0.0, flags=EST_M1M2, eps=eps)[0][0]
    np.testing.assert_allclose(y["r"], (A / S + eps) / (B + eps), rtol=1e-13)


def test_elastic_scale_change_keeps_state():
    """Elastic AdaScaling (Sec. 4): S changes mid-run; tau keeps accumulating and the gain
    re-enters [1, S']."""
    d = 30
    o = Oracle(4, np.full(100, 0.01, dtype=np.float32), theta=0.5)
    w, v = [np.zeros(d)], [np.zeros(d)]
    r = rng(21)
    taus = []
    for S in (4, 4, 8, 8, 2, 2):
        if S != o.S:
            o.set_scale(S, 0.5)
        g = f32(r.normal(size=(S, d)) + 0.3)
        st = o.step(w, v, [[g[i]] for i in range(S)])
        assert 1.0 <= st.r <= S
        taus.append(st.tau)
    assert all(b > a for a, b in zip(taus, taus[1:]))


# ------------------------------------------------- resuming and changing the scale
def _numpy_sample(g):
    """A, B and the two raw estimates of App. B.3 for one [S, d] sample, from numpy."""
    g = np.asarray(g, dtype=np.float64)
    S = g.shape[0]
    A, B = (g ** 2).sum(), (g.mean(axis=0) ** 2).sum()
    sig = g.var(axis=0, ddof=1).sum() if S >= 2 else 0.0     # summed per-coordinate sample variance
    return A, B, sig, B - sig / S


@pytest.mark.parametrize("flags", [0, LAGGED_R, EST_M1M2])
def test_resume_from_the_saved_state_continues_the_same_run(flags):
    """The state of Algorithm 2 is (w, v, tau) plus the two averages of App. B.3 and their sample
    count: a fresh oracle given exactly those continues an interrupted run bit for bit."""
    S, d, T = 4, 40, 6
    lr = f32(0.2 * 0.7 ** np.arange(12))
    gs = [f32(rng(50 + t).normal(size=(S, d)) + 0.4) for t in range(T)]
    kw = dict(theta=0.8, weight_decay=1e-3, momentum=0.9, flags=flags)
    straight, w_a, v_a = run(S, gs, lr=lr, **kw)

    o = Oracle(S, lr, **kw)
    w, v = [np.zeros(d)], [np.zeros(d)]
    for g in gs[:3]:
        o.step(w, v, [[g[i]] for i in range(S)])
    saved = o.state()
    o2 = Oracle(S, lr, **kw)
    o2.set_state(saved.step, saved.tau, saved.sigma2_bar, saved.mu2_bar, saved.r)
    w2, v2 = [w[0].copy()], [v[0].copy()]
    for t, g in enumerate(gs[3:], start=3):
        st = o2.step(w2, v2, [[g[i]] for i in range(S)]).as_dict()
        assert st == straight[t]
    assert np.array_equal(w2[0], w_a) and np.array_equal(v2[0], v_a)


def test_set_state_fields_land_where_the_next_step_reads_them():
    """One step after set_state(k, tau, s, m), against numpy: the averages move by
    alpha = max(1 - theta, 1/(k+1)) towards the new (clamped) sample, the learning rate is read at
    floor(tau), the clock becomes tau + r and the count k + 1 (Sec. 3.2, App. B.3).  The four
    values are all different, so a swapped or dropped field shows."""
    S, d, theta, eps = 4, 25, 0.75, 1e-6
    lr = f32(np.linspace(1.0, 0.1, 10))
    g = f32(rng(61).normal(size=(S, d)) * 0.7 + 0.5)
    A, B, sig, mu = _numpy_sample(g)
    assert sig > eps and mu > 0
    for k, tau, s0, m0 in ((2, 5.25, 3.5, 0.125), (40, 7.9, 0.25, 6.0)):
        o = Oracle(S, lr, theta=theta, eps=eps)
        o.set_state(k, tau, s0, m0)
        w, v = [np.zeros(d)], [np.zeros(d)]
        st = o.step(w, v, [[g[i]] for i in range(S)])
        alpha = max(1 - theta, 1.0 / (k + 1))
        s1, m1 = s0 + alpha * (sig - s0), m0 + alpha * (mu - m0)
        r = (s1 + m1) / (s1 / S + m1)
        np.testing.assert_allclose([st.sigma2_bar, st.mu2_bar, st.r], [s1, m1, r], rtol=1e-13)
        np.testing.assert_allclose(st.lr_eff, r * float(lr[int(math.floor(tau))]), rtol=1e-13)
        np.testing.assert_allclose(st.tau, tau + r, rtol=1e-14)
        assert st.step == k + 1
        np.testing.assert_allclose(w[0], -st.lr_eff * g.astype(np.float64).mean(axis=0), rtol=1e-12)


@pytest.mark.parametrize("S_old,S_new", [(4, 8), (8, 3), (2, 5)])
def test_scale_change_uses_the_new_scale_in_the_estimator(S_old, S_new):
    """Elastic AdaScaling (Sec. 4): after the scale changes, sigma2_hat divides by S' - 1, mu2_hat
    and the gain ratio use S' (App. B.3, eq. 3).  With theta = 0 the next gain is the plain ratio
    of norms (A/S')/B of Sec. 3.4 -- taken here from numpy."""
    d = 30
    o = Oracle(S_old, f32([0.05]), theta=0.6)
    w, v = [np.zeros(d)], [np.zeros(d)]
    for t in range(3):
        g = f32(rng(70 + t).normal(size=(S_old, d)) + 0.3)
        o.step(w, v, [[g[i]] for i in range(S_old)])
    tau_before = o.state().tau
    o.set_scale(S_new, 0.0)
    g = f32(rng(80).normal(size=(S_new, d)) + 0.3)
    st = o.step(w, v, [[g[i]] for i in range(S_new)])
    A, B, sig, mu = _numpy_sample(g)
    assert sig > 1e-6 and mu > 0                                  # no clamp active
    np.testing.assert_allclose([st.sum_sq, st.sq_mean, st.sigma2_hat, st.mu2_hat], [A, B, sig, mu], rtol=1e-12)
    np.testing.assert_allclose(st.r, (A / S_new) / B, rtol=1e-12)
    np.testing.assert_allclose([st.sigma2_bar, st.mu2_bar], [sig, mu], rtol=1e-12)   # theta = 0: no memory
    np.testing.assert_allclose(st.tau, tau_before + st.r, rtol=1e-14)
    assert st.step == 4                                           # the count carries on


@pytest.mark.parametrize("S_new", [16, 100, 1500])
def test_scale_change_default_theta_follows_the_new_scale(S_new):
    """theta = max(1 - S'/1000, 0) after a change of scale (Sec. 3.4, Sec. 4): asking for the
    default gives the same run as passing that value, and the averages move by
    alpha = max(1 - theta, 1/k) = max(min(S'/1000, 1), 1/k)."""
    d, S_old = 12, 2
    explicit = max(1.0 - S_new / 1000.0, 0.0)
    outs = []
    for theta in (-1.0, explicit):
        o = Oracle(S_old, f32([0.05]), theta=0.3)
        w, v = [np.zeros(d)], [np.zeros(d)]
        o.set_state(50, 11.0, 2.0, 0.5)
        o.set_scale(S_new, theta)
        g = f32(rng(90).normal(size=(S_new, d)) + 0.3)
        st = o.step(w, v, [[g[i]] for i in range(S_new)])
        outs.append((st.as_dict(), w[0].copy()))
    assert outs[0][0] == outs[1][0] and np.array_equal(outs[0][1], outs[1][1])
    A, B, sig, mu = _numpy_sample(g)
    alpha = max(min(S_new / 1000.0, 1.0), 1.0 / 51)
    np.testing.assert_allclose(outs[0][0]["sigma2_bar"], 2.0 + alpha * (max(sig, 1e-6) - 2.0), rtol=1e-12)
    np.testing.assert_allclose(outs[0][0]["mu2_bar"], 0.5 + alpha * (max(mu, 0.0) - 0.5), rtol=1e-12)


def test_openmp_build_agrees():
    S, d = 5, 1000
    g = f32(rng(30).normal(size=(S, d)) + 0.1)
    outs = []
    for omp in (False, True):
        o = Oracle(S, f32([0.1]), theta=0.0, weight_decay=1e-3, openmp=omp)
        w, v = [np.full(d, 0.5)], [np.zeros(d)]
        st = o.step(w, v, [[g[i]] for i in range(S)])
        outs.append((st.as_dict(), w[0].copy()))
    for key in ("sum_sq", "sq_mean", "sigma2_hat", "mu2_hat", "r", "tau"):
        np.testing.assert_allclose(outs[0][0][key], outs[1][0][key], rtol=1e-14)
    np.testing.assert_allclose(outs[0][1], outs[1][1], rtol=1e-14)
