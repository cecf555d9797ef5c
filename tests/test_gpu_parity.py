"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Tolerances are the ones of the benchmark definition: relative error <= 1e-5 on
sigma2_hat, mu2_hat (against max(|value|, 1e-4 A/S)), r and tau; |dw| <= 1e-6 max|w| per step.
The same 1e-6 bar is applied to bf16-gradient runs (the definition allows 1e-2 there) and to v.
"""
import ctypes as C
import math

import numpy as np
import pytest
import torch

import harness as H
import workloads as W
from paper_2007_05105_amd import (BF16, COOPERATIVE_LAUNCH, EST_NORM_RATIO, F32, FORCE_FUSED, FORCE_GENERAL,
                                  FORCE_STREAMING, LAGGED_R, NO_POINTER_CHECK, AdaScale, AdaScaleError, Tuning)

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)


@pytest.fixture(autouse=True, params=["fused", "three_kernel", "general"])
def step_path(request, monkeypatch):
    """Every test runs once per implementation of the step, forced here even where the library
    would choose another: the fused persistent launch (the mean gradient stays on chip as far as
    it fits), the three-kernel step with the streaming reduce kernel (what parameter lists far
    larger than the chip get), and the general three-kernel step (any scale; the other two stop
    at S = 4096)."""
    force = {"fused": FORCE_FUSED, "three_kernel": FORCE_STREAMING, "general": FORCE_GENERAL}[request.param]
    monkeypatch.setattr(H, "DEFAULT_TUNING", Tuning(force_path=force))
    return request.param


def expect_path(gpu, step_path, dtype=F32):
    fused = step_path == "fused"
    assert gpu.uses_fused_step() == fused
    assert gpu.step_path() == ("fused" if fused else "general" if step_path == "general" else "streaming")


# ------------------------------------------------------------------ small shapes, every path
SMALL_SHAPES = [(5000,), (1,), (1023,), (1024,), (1025,), (3, 7, 11), (4096,), (64,), (2, 2049), (7,)]


@pytest.mark.parametrize("S", [1, 2, 3, 4, 5, 8, 16, 17, 33, 64])
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_small_multi_tensor_all_scales(S, dtype):
    """Several tiles, ragged tails, 1-element tensors; S below, at and off the load-group sizes."""
    wl = W.custom(SMALL_SHAPES, S, grad_dtype=dtype, weight_decay=1e-3, theta=0.5,
                  lr_table=W.lr_step_decay(0.1, 8), steps=4, seed=S)
    rep = H.run_teacher_forced(wl, log=log)
    H.assert_report(rep)


@pytest.mark.parametrize("S,dtype", [(1, F32), (2, F32), (3, F32), (4, F32), (7, F32), (8, F32), (13, F32), (16, F32),
                                     (23, F32), (32, F32), (33, F32), (57, F32),
                                     (1, BF16), (4, BF16), (6, BF16), (16, BF16), (27, BF16), (32, BF16), (51, BF16), (64, BF16),
                                     (65, BF16), (130, BF16)])
def test_fused_step_spills_to_hbm_when_the_chip_is_full(S, dtype, step_path, monkeypatch):
    """Two workgroups only, so most tiles overflow registers + LDS: their sweep updates the
    momentum in place and phase 2 only applies it."""
    if step_path != "fused":
        pytest.skip("fused step only")
    monkeypatch.setattr(H, "DEFAULT_TUNING", Tuning(force_path=FORCE_FUSED, fused_max_grid=2))
    wl = W.custom([(150001,), (5,), (300000,), (2048,), (77777,)], S, grad_dtype=dtype, weight_decay=1e-3, theta=0.5,
                  steps=3, seed=S)
    g = H.make_gpu(wl)
    assert g.uses_fused_step()
    g.close()
    H.assert_report(H.run_teacher_forced(wl, log=log))


@pytest.mark.parametrize("skew", [1, 3])
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_element_aligned_pointers(skew, dtype):
    """Tensor starts that are only element aligned (views into a flat buffer at odd offsets)."""
    wl = W.custom(SMALL_SHAPES, 4, grad_dtype=dtype, weight_decay=1e-3, steps=3, seed=5)
    rep = H.run_teacher_forced(wl, skew_elems=skew, log=log)
    H.assert_report(rep)


@pytest.mark.parametrize("S,dtype", [(4, F32), (16, F32), (32, BF16)])
def test_one_allocation_per_replica(S, dtype):
    """The S gradient buffers in allocations of their own (the other tests pass rows of one allocation)."""
    wl = W.custom(SMALL_SHAPES + [(300, 1000)], S, grad_dtype=dtype, weight_decay=1e-3, theta=0.5,
                  lr_table=W.lr_step_decay(0.1, 8), steps=3, seed=40 + S)
    inp = W.Inputs(wl, "cuda:0", one_allocation=False)
    assert len({g.untyped_storage().data_ptr() for g in inp.g_flat}) == S
    rep = H.run_teacher_forced(wl, inputs=inp, log=log)
    H.assert_report(rep)


@pytest.mark.parametrize("recipe,S", [("identical", 4), ("zero_mean", 8), ("zeros", 4), ("zeros", 1),
                                      ("identical", 1)])
def test_degenerate_gradients(recipe, S):
    """Zero variance (r -> 1), zero mean (r -> S), all-zero gradients (B = 0)."""
    wl = W.custom([(3000,), (17,)], S, theta=0.0, steps=3, recipe=recipe, seed=3)
    rep = H.run_teacher_forced(wl, log=log)
    H.assert_report(rep)
    for s in rep.steps:
        assert 1.0 - 1e-12 <= s.r <= S * (1 + 1e-12)


def test_empty_tensors_and_empty_list():
    """numel 0 tensors are skipped; an empty parameter list still advances the clock."""
    wl = W.custom([(0,), (300,), (0,), (0,), (5,)], 3, steps=2, seed=9)
    H.assert_report(H.run_teacher_forced(wl, log=log))
    g = AdaScale([], 4, [0.1], theta=0.0, tuning=H.DEFAULT_TUNING)
    assert not g.uses_fused_step()
    g.step([], [], [[], [], [], []])
    st = g.get_state()
    assert st.step == 1 and st.sum_sq == 0.0 and st.sq_mean == 0.0 and st.r == 4.0 and st.tau == 4.0


def test_huge_dynamic_range():
    """Per-tensor gradient scales spread over many decades: the sums must not lose the small tensors."""
    wl = W.custom([(20000,), (20000,), (20000,)], 8, theta=0.0, steps=2, recipe="per_tensor_scale", seed=4)
    H.assert_report(H.run_teacher_forced(wl, log=log))


def test_lr_table_overrun_clamps_to_last_entry():
    wl = W.custom([(2000,)], 8, theta=0.0, lr_table=np.array([0.1, 0.05, 0.025], np.float32), steps=4,
                  recipe="zero_mean", seed=2)
    rep = H.run_teacher_forced(wl, log=log)
    H.assert_report(rep)
    assert rep.steps[-1].tau > 3.0          # past the table: the library kept stepping


@pytest.mark.parametrize("flags", [LAGGED_R, EST_NORM_RATIO, LAGGED_R | EST_NORM_RATIO])
def test_variants_of_the_estimator(flags):
    """Prior-iteration gain (App. B.3) and the norm-ratio estimator (Sec. 3.4)."""
    wl = W.custom(SMALL_SHAPES, 8, weight_decay=1e-3, theta=0.7, steps=5, seed=11)
    H.assert_report(H.run_teacher_forced(wl, flags=flags, log=log))


@pytest.mark.parametrize("S,dtype", [(16, F32), (4, F32), (32, BF16), (5, F32), (64, BF16), (29, F32), (40, F32)])
def test_lagged_gain_single_pass_medium(S, dtype, step_path):
    """Prior-iteration gain on shapes that span many tiles per workgroup (fused step: without its
    grid barrier at S = 4, 5, where a workgroup's share of the step is short, with it at the
    larger scales; streaming reduce, scalars, update; beyond their scales one sweep that reduces
    and updates, then the scalars)."""
    wl = W.custom([(3_000_000,), (70001,), (513,), (1_200_000,)], S, grad_dtype=dtype, weight_decay=1e-4, theta=0.9,
                  lr_table=W.lr_step_decay(0.1, 64), steps=3, seed=41)
    H.assert_report(H.run_teacher_forced(wl, flags=LAGGED_R, log=log))


def test_cooperative_launch_flag(step_path):
    wl = W.custom([(300000,), (999,), (5000,)], 8, weight_decay=1e-3, theta=0.5, steps=3, seed=21)
    H.assert_report(H.run_teacher_forced(wl, flags=COOPERATIVE_LAUNCH, log=log))


def test_two_contexts_on_two_streams(step_path):
    """Steps of two contexts issued alternately on two streams without host synchronisation give
    exactly what each context gives alone (fused launches of one process are chained per device)."""
    wls = [W.custom([(400000,), (77,)], 16, weight_decay=1e-4, theta=0.9, steps=4, seed=31),
           W.custom([(250001,), (3000,)], 4, weight_decay=0.0, theta=0.5, steps=4, seed=32)]

    def run(interleaved):
        inps = [W.Inputs(wl, "cuda:0") for wl in wls]
        for inp in inps:
            inp.fill_grads(0)
        gpus = [H.make_gpu(wl) for wl in wls]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()] if interleaved else [torch.cuda.current_stream()] * 2
        torch.cuda.synchronize()
        for t in range(4):
            for g, inp, st in zip(gpus, inps, streams):
                g.step(inp.w, inp.v, inp.g, stream=st)
        torch.cuda.synchronize()
        out = [(g.get_state(st).as_dict(), inp.w_flat.clone()) for g, inp, st in zip(gpus, inps, streams)]
        for g in gpus:
            g.close()
        return out

    a, b = run(False), run(True)
    for (sa, wa), (sb, wb) in zip(a, b):
        assert sa == sb and torch.equal(wa, wb)


# ------------------------------------------------------------ nothing outside the tensors
@pytest.mark.parametrize("skew", [0, 1, 3])
@pytest.mark.parametrize("S,dtype,flags", [(4, F32, 0), (5, F32, 0), (4, BF16, 0), (11, BF16, 0), (16, F32, LAGGED_R),
                                           (6, BF16, LAGGED_R)])
def test_poisoned_padding_is_neither_read_nor_written(skew, S, dtype, flags):
    """Every element between the tensors (and between the gradient rows) holds a NaN: an
    out-of-extent read at a ragged tail would put it into A or B, an out-of-extent write would
    replace the sentinel in w or v (checked bit for bit after every step, with the gradient
    buffers, which the library must never write)."""
    wl = W.custom(SMALL_SHAPES, S, grad_dtype=dtype, weight_decay=1e-3, theta=0.5, steps=3, seed=50 + S)
    rep = H.run_teacher_forced(wl, skew_elems=skew, flags=flags, poison=True, log=log)
    H.assert_report(rep)


@pytest.mark.parametrize("skew", [0, 1])
@pytest.mark.parametrize("S,dtype", [(3, F32), (16, F32), (8, BF16), (33, BF16)])
def test_poisoned_padding_with_tiles_beyond_the_chip(skew, S, dtype, step_path, monkeypatch):
    """The same with two workgroups only, so that most tiles take the momentum-in-the-sweep path of
    the fused step, and on the streaming kernel's many pairs per workgroup."""
    if step_path == "fused":
        monkeypatch.setattr(H, "DEFAULT_TUNING", Tuning(force_path=FORCE_FUSED, fused_max_grid=2))
    wl = W.custom([(150001,), (5,), (300000,), (2048,), (77777,)], S, grad_dtype=dtype, weight_decay=1e-3, theta=0.5,
                  steps=2, seed=60 + S)
    H.assert_report(H.run_teacher_forced(wl, skew_elems=skew, poison=True, log=log))


# ------------------------------------------------------------------------------ write bursts
@pytest.mark.parametrize("keep,ticks", [(3, 100), (18, 10 ** 8), (1, 64), (5, 300)],
                         ids=["short_windows", "ring_fills_first", "one_tile", "five_tiles"])
@pytest.mark.parametrize("S,dtype", [(3, F32), (16, F32), (8, BF16), (33, BF16)])
def test_write_bursts_leave_the_same_bits(keep, ticks, S, dtype, step_path, monkeypatch):
    """Sweeps that write as they read keep finished tiles in LDS and write them in clock windows
    (by default only from 32 gradient bytes per parameter upwards).  Forced here at every scale,
    with windows of 1 us (nearly every tile written at once), 3 us, and so long that only a full
    ring is ever written: parity with the oracle, poisoned padding intact, and w, v bit for bit
    what the same steps give with every tile written at once."""
    if step_path == "general":
        pytest.skip("the general kernels write at once")
    base = dict(force_path=FORCE_FUSED, fused_max_grid=2) if step_path == "fused" else dict(force_path=FORCE_STREAMING)
    wl = W.custom([(150001,), (5,), (300000,), (2048,), (77777,)], S, grad_dtype=dtype, weight_decay=1e-3, theta=0.5,
                  steps=3, seed=70 + S)
    monkeypatch.setattr(H, "DEFAULT_TUNING", Tuning(burst_tiles=keep, burst_window_ticks=ticks, **base))
    H.assert_report(H.run_teacher_forced(wl, skew_elems=1, poison=True, log=log))
    outs = []
    for tun in (Tuning(burst_tiles=keep, burst_window_ticks=ticks, **base), Tuning(burst_tiles=-1, **base)):
        inp = W.Inputs(wl, "cuda:0")
        gpu = H.make_gpu(wl, tuning=tun)
        for t in range(3):
            inp.fill_grads(t)
            gpu.step(inp.w, inp.v, inp.g)
        st = gpu.get_state()
        outs.append((st.tau, st.r, inp.w_flat.clone(), inp.v_flat.clone()))
        gpu.close()
    assert outs[0][:2] == outs[1][:2]
    assert torch.equal(outs[0][2], outs[1][2]) and torch.equal(outs[0][3], outs[1][3])


# ---------------------------------------------------------------- pointer sets and failure
def test_alternating_pointer_sets(step_path):
    """A caller that rotates between three (w, v) pairs and two sets of gradient buffers (six
    distinct pointer sets, more than the library keeps tables for) gets bit for bit what a caller
    with one fixed set of buffers gets when the same data is copied in and out of them."""
    wl = W.custom([(70000,), (513,), (4096, 3)], 4, weight_decay=1e-3, theta=0.5, lr_table=W.lr_step_decay(0.1, 16),
                  steps=12, seed=71)
    sets = [W.Inputs(wl, "cuda:0") for _ in range(3)]
    for j, inp in enumerate(sets):
        inp.w_flat.mul_(1.0 + j)
    gsets = [W.Inputs(wl, "cuda:0"), W.Inputs(wl, "cuda:0")]
    gsets[0].fill_grads(0)
    gsets[1].fill_grads(1)
    start = [(inp.w_flat.clone(), inp.v_flat.clone()) for inp in sets]

    rot = H.make_gpu(wl)
    for t in range(wl.steps):
        rot.step(sets[t % 3].w, sets[t % 3].v, gsets[t % 2].g)
    st_rot = rot.get_state().as_dict()
    rot.close()
    got = [(inp.w_flat.clone(), inp.v_flat.clone()) for inp in sets]

    fixed = W.Inputs(wl, "cuda:0")
    cur = [(w.clone(), v.clone()) for w, v in start]
    one = H.make_gpu(wl)
    for t in range(wl.steps):
        fixed.w_flat.copy_(cur[t % 3][0])
        fixed.v_flat.copy_(cur[t % 3][1])
        for dst, src in zip(fixed.g_flat, gsets[t % 2].g_flat):
            dst.copy_(src)
        one.step(fixed.w, fixed.v, fixed.g)
        cur[t % 3] = (fixed.w_flat.clone(), fixed.v_flat.clone())
    st_one = one.get_state().as_dict()
    one.close()
    assert st_rot == st_one
    for (w1, v1), (w2, v2) in zip(got, cur):
        assert torch.equal(w1, w2) and torch.equal(v1, v2)


@pytest.mark.parametrize("flags", [0, COOPERATIVE_LAUNCH])
def test_grid_barrier_that_gives_up_is_reported_and_recoverable(flags, step_path):
    """The failure path of the fused step, forced from the host: the barrier of one step waits for
    an arrival that never comes, with a wait of a few hundred polls, so every workgroup gives up
    and every kernel exits normally.  The step must leave w and v alone (all tiles are on chip
    here), adascale_get_state and further steps must report ESTATE, and after adascale_set_state
    the run continues exactly like one that never failed."""
    if step_path != "fused":
        pytest.skip("fused step only")
    wl = W.custom([(300000,), (999,), (5000,)], 8, weight_decay=1e-3, theta=0.5, steps=3, seed=21)
    tun = Tuning(force_path=FORCE_FUSED, barrier_spin_limit=300)

    def run(fail_at):
        inp = W.Inputs(wl, "cuda:0")
        g = H.make_gpu(wl, flags=flags, tuning=tun)
        for t in range(wl.steps):
            inp.fill_grads(t)
            if t == fail_at:
                st = g.get_state()
                w0, v0 = inp.w_flat.clone(), inp.v_flat.clone()
                g.fail_next_barrier()
                g.step(inp.w, inp.v, inp.g)                     # queued; the failure shows at the next query
                with pytest.raises(AdaScaleError) as e:
                    g.get_state()
                assert e.value.code == 4
                assert torch.equal(inp.w_flat, w0) and torch.equal(inp.v_flat, v0)
                with pytest.raises(AdaScaleError) as e:
                    g.step(inp.w, inp.v, inp.g)
                assert e.value.code == 4
                g.set_state(st.step, st.tau, st.sigma2_bar, st.mu2_bar)
            g.step(inp.w, inp.v, inp.g)
        out = (g.get_state().as_dict(), inp.w_flat.clone(), inp.v_flat.clone())
        g.close()
        return out

    a, b = run(None), run(1)
    assert a[0] == b[0] and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])
    # a context without a barrier has nothing to fail
    g = H.make_gpu(wl, flags=LAGGED_R, tuning=tun)
    with pytest.raises(AdaScaleError) as e:
        g.fail_next_barrier()
    assert e.value.code == 4
    g.close()


def test_free_running_small():
    wl = W.custom(SMALL_SHAPES, 4, weight_decay=1e-3, theta=0.9, steps=20, seed=6)
    rel, drift, gst, ost = H.run_free(wl)
    log(f"free-running 20 steps: rel={rel} drift={drift:.3g}")
    assert max(rel[k] for k in ("r", "tau")) <= 1e-5
    assert drift <= 2e-5


def test_bitwise_determinism():
    """No atomics: two runs on the same inputs give identical scalars and weights."""
    wl = W.custom([(100000,), (333,), (70001,)], 16, weight_decay=1e-4, theta=0.9, steps=3, seed=8)
    outs = []
    for _ in range(2):
        inp = W.Inputs(wl, "cuda:0")
        g = H.make_gpu(wl)
        for t in range(wl.steps):
            inp.fill_grads(t)
            g.step(inp.w, inp.v, inp.g)
        st = g.get_state()
        outs.append((st.as_dict(), inp.w_flat.clone(), inp.v_flat.clone()))
        g.close()
    assert outs[0][0] == outs[1][0]
    assert torch.equal(outs[0][1], outs[1][1]) and torch.equal(outs[0][2], outs[1][2])


def test_elastic_scale_and_checkpoint_resume():
    """S changes mid-run (elastic AdaScaling, Sec. 4) and a run resumed from (w, v, state)
    continues exactly like the uninterrupted one."""
    shapes = [(5000,), (77,)]
    wls = {S: W.custom(shapes, S, theta=0.5, weight_decay=1e-3, lr_table=W.lr_constant(0.05, 64), seed=12)
           for S in (4, 8, 2)}
    gpu = H.make_gpu(wls[4])
    orc = H.make_oracle(wls[4])
    inp = {S: W.Inputs(wls[S], "cuda:0") for S in wls}
    w_flat, v_flat = inp[4].w_flat, inp[4].v_flat
    w = W.views(w_flat, wls[4].numel, inp[4].offs32)
    v = W.views(v_flat, wls[4].numel, inp[4].offs32)
    w64 = [x.cpu().numpy().astype(np.float64) for x in w]
    v64 = [x.cpu().numpy().astype(np.float64) for x in v]
    snap = None
    for t, S in enumerate([4, 4, 8, 8, 2, 2]):
        if gpu.S != S:
            gpu.set_scale(S, 0.5)
            orc.set_scale(S, 0.5)
        inp[S].fill_grads(t)
        gpu.step(w, v, inp[S].g)
        ost = orc.step(w64, v64, H.grads_to_numpy(inp[S]))
        gst = gpu.get_state()
        rel = H.compare_step(gst, ost, S)
        assert max(rel[k] for k in ("sigma2_hat", "mu2_hat", "r", "tau")) <= 1e-5, rel
        assert 1.0 <= gst.r <= S
        if t == 2:
            snap = (gst, w_flat.clone(), v_flat.clone())
    final = (gpu.get_state(), w_flat.clone())
    gpu.close()
    # resume from the snapshot taken after step 2 (S = 8 at that point)
    gst, w_flat2, v_flat2 = snap
    g2 = H.make_gpu(wls[8])
    g2.set_scale(8, 0.5)
    g2.set_state(gst.step, gst.tau, gst.sigma2_bar, gst.mu2_bar)
    w2 = W.views(w_flat2, wls[8].numel, inp[8].offs32)
    v2 = W.views(v_flat2, wls[8].numel, inp[8].offs32)
    for t, S in list(enumerate([4, 4, 8, 8, 2, 2]))[3:]:
        if g2.S != S:
            g2.set_scale(S, 0.5)
        inp[S].fill_grads(t)
        g2.step(w2, v2, inp[S].g)
    st2 = g2.get_state()
    assert st2.tau == final[0].tau and st2.r == final[0].r and st2.step == final[0].step
    assert torch.equal(w_flat2, final[1])
    g2.close()


@pytest.mark.parametrize("scales", [(32, 64, 128), (128, 64, 32)], ids=["growing", "shrinking"])
def test_elastic_scale_changes_at_quarter_and_half_of_the_budget(scales, step_path):
    """Elastic AdaScaling as the paper runs it (Sec. 4): the scale doubles (or halves) when tau
    passes T_SI/4 and T_SI/2, theta follows the scale (max(1 - S/1000, 0)), and the run ends at
    tau >= T_SI.  bf16 gradients over several tensors; S = 128 has no fused instance, so the run
    also crosses from one step path to the other.  The oracle runs freely beside the GPU."""
    shapes = [(300, 1000), (4099,), (2048 * 3,), (17, 31)]
    L = 600
    wls = {S: W.custom(shapes, S, grad_dtype=BF16, theta=-1.0, weight_decay=1e-4,
                       lr_table=W.lr_step_decay(0.05, L), steps=30, seed=21)
           for S in scales}
    inp = {S: W.Inputs(wls[S], "cuda:0") for S in scales}
    first = inp[scales[0]]
    w = W.views(first.w_flat, first.wl.numel, first.offs32)
    v = W.views(first.v_flat, first.wl.numel, first.offs32)
    w64 = [x.cpu().numpy().astype(np.float64) for x in w]
    v64 = [x.cpu().numpy().astype(np.float64) for x in v]
    w0 = [x.copy() for x in w64]
    gpu = H.make_gpu(wls[scales[0]])
    orc = H.make_oracle(wls[scales[0]])
    tau, t, seen = 0.0, 0, []
    while tau < L:
        assert t < 60, "the run should reach tau >= T_SI within a few dozen iterations"
        S = scales[0] if tau < L / 4 else scales[1] if tau < L / 2 else scales[2]
        if gpu.S != S:
            gpu.set_scale(S, -1.0)
            orc.set_scale(S, -1.0)
        inp[S].fill_grads(t)
        gpu.step(w, v, inp[S].g)
        ost = orc.step(w64, v64, H.grads_to_numpy(inp[S]))
        gst = gpu.get_state()
        rel = H.compare_step(gst, ost, S)
        assert max(rel[k] for k in ("sigma2_hat", "mu2_hat", "r", "tau", "lr_eff")) <= H.TOL_SCALAR, (t, S, rel)
        assert 1.0 <= gst.r <= S * (1 + 1e-12)
        tau, t = gst.tau, t + 1
        seen.append(S)
    assert gst.done == 1 and ost.done == 1
    assert list(dict.fromkeys(seen)) == list(scales)          # all three scales were visited, in order
    assert math.ceil(L / max(scales)) <= t <= L               # iteration bounds of Sec. 3.2
    # free-running drift of w over the whole run (fp32 storage against the fp64 oracle)
    assert H.tensor_err(first.w_flat, w64, w0, first.wl.numel, first.offs32) <= 2e-5
    gpu.close()


def test_scale_beyond_every_512_lane_shape_and_back(step_path):
    """S = 4100 has no fused or streaming instance: the context moves to the general kernels (and
    only then allocates the full mean-gradient scratch), then back."""
    shapes = [(2500,), (5,)]
    wls = {S: W.custom(shapes, S, theta=0.5, weight_decay=1e-3, lr_table=W.lr_constant(0.05, 8), seed=77) for S in (8, 4100)}
    inp = {S: W.Inputs(wls[S], "cuda:0") for S in wls}
    first = inp[8]
    w = W.views(first.w_flat, first.wl.numel, first.offs32)
    v = W.views(first.v_flat, first.wl.numel, first.offs32)
    w64 = [x.cpu().numpy().astype(np.float64) for x in w]
    v64 = [x.cpu().numpy().astype(np.float64) for x in v]
    gpu, orc = H.make_gpu(wls[8]), H.make_oracle(wls[8])
    paths = []
    for t, S in enumerate([8, 8, 4100, 4100, 8]):
        if gpu.S != S:
            gpu.set_scale(S, 0.5)
            orc.set_scale(S, 0.5)
        paths.append(gpu.step_path())
        inp[S].fill_grads(t)
        gpu.step(w, v, inp[S].g)
        ost = orc.step(w64, v64, H.grads_to_numpy(inp[S]))
        rel = H.compare_step(gpu.get_state(), ost, S)
        assert max(rel[k] for k in ("sigma2_hat", "mu2_hat", "r", "tau", "lr_eff")) <= H.TOL_SCALAR, (t, S, rel)
    assert paths[2] == paths[3] == "general"
    assert paths[0] == paths[4] == {"fused": "fused", "three_kernel": "streaming", "general": "general"}[step_path]
    assert H.tensor_err(first.w_flat, w64, w64, first.wl.numel, first.offs32) <= 1e-5
    gpu.close()


def test_error_paths_launch_nothing():
    """Bad arguments come back as codes; the pointer check refuses host memory and short buffers."""
    with pytest.raises(AdaScaleError) as e:
        AdaScale([10], 0, [0.1])
    assert e.value.code == 1
    with pytest.raises(AdaScaleError):
        AdaScale([10], 2, [0.1], momentum=1.0)
    with pytest.raises(AdaScaleError):
        AdaScale([10], 2, [0.1], theta=1.0)
    with pytest.raises(AdaScaleError):
        AdaScale([-1], 2, [0.1])
    with pytest.raises(AdaScaleError):
        AdaScale([10], 2, [])
    g = AdaScale([1000], 2, [0.1], tuning=H.DEFAULT_TUNING)
    w = torch.zeros(1000, device="cuda:0")
    v = torch.zeros(1000, device="cuda:0")
    ok = [torch.ones(1000, device="cuda:0"), torch.ones(1000, device="cuda:0")]
    stream = int(torch.cuda.current_stream().cuda_stream)
    arr = lambda ptrs: (C.c_void_p * len(ptrs))(*ptrs)
    pw, pv = arr([w.data_ptr()]), arr([v.data_ptr()])
    assert g.step_raw(pw, pv, arr([ok[0].data_ptr(), 0]), stream) == 1            # null gradient
    host = torch.ones(1000)
    assert g.step_raw(pw, pv, arr([ok[0].data_ptr(), host.data_ptr()]), stream) == 1   # host memory
    small = torch.ones(10, device="cuda:0")
    own = torch.empty(1 << 22, device="cuda:0")      # make `small`'s segment end well before 1000 floats
    del own
    assert g.step_raw(pw, pv, arr([ok[0].data_ptr(), ok[1].data_ptr() + 2]), stream) == 1  # misaligned
    assert g.step_raw(None, pv, arr([ok[0].data_ptr(), ok[1].data_ptr()]), stream) == 1
    assert "pointer" in g.last_error() or "null" in g.last_error()
    torch.cuda.synchronize()
    assert g.get_state().step == 0 and float(w.abs().max()) == 0.0          # nothing ran
    assert g.step_raw(pw, pv, arr([ok[0].data_ptr(), ok[1].data_ptr()]), stream) == 0
    assert g.get_state().step == 1
    g.close()


def test_default_choice_of_step_path(step_path, monkeypatch):
    """Left alone, the library takes the fused step while at least 8 % of the mean gradient fits
    on chip (cfg3 entirely, cfg4 54 %, cfg5 9 %) and the three-kernel step with the streaming
    reduce kernel beyond (three times cfg5's list: 3 %)."""
    if step_path != "fused":
        pytest.skip("one run is enough")
    monkeypatch.setattr(H, "DEFAULT_TUNING", None)
    import torch
    from paper_2007_05105_amd import binding
    prop = torch.cuda.get_device_properties(0)
    for cfg, path in ((1, "fused"), (2, "fused"), (3, "fused"), (4, "fused"), (5, "fused"), (6, "streaming")):
        wl = W.config(min(cfg, 5))
        if cfg == 6:        # 1.05 G parameters; a context needs the list, not the tensors
            wl = W.custom([tuple(s) for s in wl.shapes] * 3, wl.S, grad_dtype=wl.grad_dtype, lr_table=wl.lr_table)
        g = H.make_gpu(wl)
        assert g.step_path() == path and g.uses_fused_step() == (path == "fused"), cfg
        # bytes the kernels move, against a count in Python: on-chip tiles 16 per parameter, tiles whose
        # sweep leaves the momentum in v 20 (24 with weight decay), ragged tiles through the scratch
        full = sum(n // 2048 * 2048 for n in wl.numel)
        keep = {1: 1.0, 2: 1.0, 3: 1.0, 6: 0.0}.get(cfg)
        if keep is not None:
            per = 16 if keep else (24 if wl.weight_decay else 20)
            ragged = 24 if path == "fused" else 32
            assert g.step_moved_bytes() == wl.S * wl.d * wl.grad_bytes + per * full + ragged * (wl.d - full), cfg
        assert g.step_moved_bytes() <= g.step_bytes() + 12 * (wl.d - full)
        # the host-only plan for a device of this size says the same
        plan = binding.plan(wl.numel, wl.S, wl.grad_dtype, compute_units=prop.multi_processor_count,
                            lds_bytes=prop.shared_memory_per_block)
        assert plan["path"] == path, (cfg, plan)
        g.close()
    assert (prop.multi_processor_count, prop.shared_memory_per_block) == (256, 160 * 1024)   # what plan() assumes by default
    wl = W.config(5)
    g = AdaScale(wl.numel * 3, 128, wl.lr_table, grad_dtype=BF16)  # run-time number of half-groups
    assert g.step_path() == "streaming"
    g.close()
    g = AdaScale(W.config(3).numel, 128, wl.lr_table, grad_dtype=BF16)
    assert g.step_path() == "fused"
    g.close()
    g = AdaScale([1000], 5000, [0.1])                             # beyond every 512-lane shape
    assert g.step_path() == "general"
    g.close()


@pytest.mark.parametrize("S,dtype", [(1, F32), (3, F32), (16, F32), (32, F32), (33, F32), (50, F32), (2, BF16), (11, BF16),
                                     (64, BF16), (65, BF16), (128, BF16), (150, BF16)])
@pytest.mark.parametrize("bursts", [None, (3, 200), (2, 10 ** 8)], ids=["default", "ring_of_3", "ring_of_2_fills_first"])
def test_streaming_reduce_many_pairs_per_workgroup(S, dtype, bursts, step_path, monkeypatch):
    """Three-kernel step on a list with thousands of tile pairs (each workgroup claims dozens),
    an odd number of whole tiles, ragged tails and tensors smaller than a tile; with the default
    write bursts (on from 32 gradient bytes per parameter) and with small rings forced at every
    scale, written in 2 us windows or only when full."""
    if step_path != "three_kernel":
        pytest.skip("three-kernel step only")
    if bursts:
        monkeypatch.setattr(H, "DEFAULT_TUNING", Tuning(force_path=FORCE_STREAMING, burst_tiles=bursts[0],
                                                        burst_window_ticks=bursts[1]))
    wl = W.custom([(2048 * 1501 + 3,), (5,), (2048 * 700,), (2047,), (2048 * 302 + 2047,)], S, grad_dtype=dtype,
                  weight_decay=1e-3, theta=0.5, steps=2, seed=100 + S)
    H.assert_report(H.run_teacher_forced(wl, log=log))


@pytest.mark.timeout(600)
def test_one_tensor_beyond_two_to_the_31_elements(step_path):
    """Maximum sizes: a single tensor of 2^31 + 6149 elements (element offsets beyond 32 bits, byte
    offsets beyond 2^33, a ragged last tile), S = 2 bf16 gradients.  The oracle takes the tensor
    in chunks through its C entry points (the norms are global, so chunks are just more tensors
    to it); w and v are compared element by element on the first chunk, the two chunks around
    element 2^31 and the last one, the scalars on everything."""
    import ctypes
    from oracle.oracle import Oracle
    n = 2 ** 31 + 3 * 2048 + 5
    wl = W.custom([(n,)], 2, grad_dtype=BF16, weight_decay=1e-4, theta=0.0, lr_table=W.lr_constant(0.05), steps=1, seed=17)
    inp = W.Inputs(wl, "cuda:0")
    inp.fill_grads(0)
    gpu = H.make_gpu(wl)
    chunk = 1 << 26
    bounds = [(lo, min(lo + chunk, n)) for lo in range(0, n, chunk)]
    sampled = sorted({0, 2 ** 31 // chunk - 1, 2 ** 31 // chunk, len(bounds) - 1})
    before = {c: (inp.w_flat[lo:hi].cpu().numpy().astype(np.float64), inp.v_flat[lo:hi].cpu().numpy().astype(np.float64))
              for c in sampled for lo, hi in [bounds[c]]}
    gpu.step(inp.w, inp.v, inp.g)
    got = gpu.get_state()
    log(f"path {gpu.step_path()}: r={got.r:.6g} A={got.sum_sq:.6g} B={got.sq_mean:.6g}")

    orc = Oracle(wl.S, wl.lr_table, wl.momentum, wl.weight_decay, wl.theta, wl.eps, wl.grad_dtype, 0, openmp=True)
    lib, h = orc._l, orc._h
    lib.oracle_begin_step(h)
    gbar = {}
    for c, (lo, hi) in enumerate(bounds):
        rows = [inp.g_flat[i][lo:hi].view(torch.int16).cpu().numpy().view(np.uint16) for i in range(wl.S)]
        ptrs = (ctypes.c_void_p * wl.S)(*[r.ctypes.data for r in rows])
        gb = np.empty(hi - lo, dtype=np.float64)
        lib.oracle_accumulate(h, hi - lo, ptrs, gb.ctypes.data)
        if c in sampled:
            gbar[c] = gb
    lib.oracle_gain(h)
    for c in sampled:
        lo, hi = bounds[c]
        w64, v64 = before[c]
        lib.oracle_apply(h, hi - lo, w64.ctypes.data, v64.ctypes.data, gbar[c].ctypes.data)
        for name, flat, ref in (("w", inp.w_flat, w64), ("v", inp.v_flat, v64)):
            err = np.abs(flat[lo:hi].cpu().numpy().astype(np.float64) - ref).max() / np.abs(ref).max()
            log(f"chunk {c} [{lo}, {hi}): {name} err {err:.3g}")
            assert err <= H.TOL_W, (c, name, err)
    lib.oracle_advance(h)
    rel = H.compare_step(got, orc.state(), wl.S)
    assert max(v for k, v in rel.items() if not k.endswith("_plain")) <= H.TOL_SCALAR, rel
    gpu.close()


@pytest.mark.parametrize("S,dtype", [(4096, BF16), (4095, F32), (1000, F32)])
def test_largest_scales_of_the_512_lane_kernels(S, dtype, step_path):
    """The run-time half-group count at its upper end: S = 4096 is the largest scale the fused and
    streaming kernels take (512 half-groups of 8 bf16 loads, 1024 of 4 fp32 loads), 4095 and 1000
    leave padding slots in the last pair of half-groups."""
    wl = W.custom([(2048 * 3 + 77,), (5,), (2048,)], S, grad_dtype=dtype, weight_decay=1e-3, theta=0.5, steps=2, seed=S)
    g = H.make_gpu(wl)
    assert g.step_path() == {"fused": "fused", "three_kernel": "streaming", "general": "general"}[step_path]
    g.close()
    H.assert_report(H.run_teacher_forced(wl, log=log))


def _random_case(seed):
    rng = np.random.default_rng(seed)
    sizes = []
    for _ in range(int(rng.integers(1, 9))):
        kind = rng.integers(0, 6)
        if kind == 0:
            sizes.append(int(rng.integers(0, 4)))                                  # empty or tiny
        elif kind == 1:
            sizes.append(int(rng.integers(1, 5000)))
        elif kind == 2:
            sizes.append(int(2048 * rng.integers(1, 40) + rng.integers(-3, 4)))   # around whole tiles
        elif kind == 3:
            sizes.append(int(rng.integers(100_000, 600_000)))
        else:
            sizes.append(int(1024 * rng.integers(1, 64)))
    S = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 20, 24, 31, 32, 33, 48, 64, 72, 80]))
    dtype = int(rng.integers(0, 2))
    flags = int(rng.choice([0, 0, LAGGED_R, EST_NORM_RATIO, LAGGED_R | EST_NORM_RATIO]))
    wl = W.custom([(n,) for n in sizes], S, grad_dtype=dtype, momentum=float(rng.choice([0.0, 0.9, 0.99])),
                  weight_decay=float(rng.choice([0.0, 1e-4, 1e-2])), theta=float(rng.choice([-1.0, 0.0, 0.5, 0.9])),
                  lr_table=W.lr_step_decay(float(rng.choice([0.01, 0.1])), 16), steps=3, seed=int(seed),
                  recipe=str(rng.choice(["shared_fresh_signal", "decaying_signal", "per_tensor_scale", "zero_mean"])))
    return wl, flags, int(rng.integers(0, 4))


@pytest.mark.parametrize("seed", range(1000, 1016))
def test_random_shapes_scales_and_flags(seed):
    """Seeded random parameter lists (empty, tiny, around whole tiles, large), scales, gradient
    types, estimator flags, hyper-parameters and pointer alignments."""
    wl, flags, skew = _random_case(seed)
    log(f"seed {seed}: numel={wl.numel} S={wl.S} dtype={wl.grad_dtype} flags={flags} skew={skew} "
        f"rho={wl.momentum} lambda={wl.weight_decay} theta={wl.theta} recipe={wl.recipe}")
    H.assert_report(H.run_teacher_forced(wl, flags=flags, skew_elems=skew, log=log))


# ------------------------------------------------------------------------- the five configs
def test_config1_every_step_teacher_forced_and_free(step_path):
    wl = W.config(1)
    g = H.make_gpu(wl)
    expect_path(g, step_path)
    g.close()
    rep = H.run_teacher_forced(wl, log=log)
    H.assert_report(rep)
    assert 3.5 < rep.steps[-1].r < 4.0
    rel, drift, gst, ost = H.run_free(wl)
    log(f"cfg1 free-running: rel={rel} drift={drift:.3g}")
    assert max(rel[k] for k in ("sigma2_hat", "mu2_hat", "r", "tau")) <= 1e-5 and drift <= 1e-5


@pytest.mark.timeout(600)
def test_config2_full_run_sampled_steps():
    """All 200 steps run on the GPU while the signal decays 1.0 -> 0.05 (the one-sample gain would
    sweep about 1.8 -> 7.9; the theta = 0.992 average follows it with a lag); the oracle checks a
    sample of the steps."""
    wl = W.config(2)
    rep = H.run_teacher_forced(wl, check_steps=[0, 1, 2, 49, 99, 149, 199], openmp=True, log=log)
    H.assert_report(rep)
    assert rep.steps[0].r < 2.0 and rep.steps[-1].r > 3.5


@pytest.mark.timeout(600)
def test_config3_benchmark_shape(step_path):
    """The configuration the benchmark times: d = 25.6M in 161 tensors, S = 16."""
    wl = W.config(3)
    g = H.make_gpu(wl)
    expect_path(g, step_path)
    g.close()
    rep = H.run_teacher_forced(wl, n_steps=6, check_steps=[0, 1, 5], openmp=True, log=log)
    H.assert_report(rep)


@pytest.mark.timeout(900)
def test_config4_bf16(step_path):
    wl = W.config(4)
    g = H.make_gpu(wl)
    expect_path(g, step_path, BF16)
    g.close()
    rep = H.run_teacher_forced(wl, n_steps=4, check_steps=[0, 3], openmp=True, log=log)
    H.assert_report(rep)


@pytest.mark.timeout(1100)
def test_config5_bf16_45GB(step_path):
    """d = 351M, S = 64: 45 GB of bf16 gradients resident; the oracle (OpenMP build) checks the two
    ends of the signal-to-noise sweep: iteration 0 (signal dominated, gain near 1) and iteration 49
    (noise dominated, one-sample gain near 60)."""
    wl = W.config(5)
    inp = W.Inputs(wl, "cuda:0")
    rep = H.run_teacher_forced(wl, step_ids=[0, 49], openmp=True, inputs=inp, log=log)
    H.assert_report(rep)
    assert rep.steps[0].r < 1.2 and rep.steps[1].r > rep.steps[0].r
