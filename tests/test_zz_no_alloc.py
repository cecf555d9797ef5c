"""The entry point that allocates nothing (adascale_step_flat, for callers under graph capture or
otherwise unable to call hipMalloc) against adascale_step on a context with the same single
tensor: same inputs, results to the tolerances of the parity tests (the two sum in different
orders), on two runs in a row, the second smaller than the first, so that whatever the first left
in the library's fixed scratch block is there when the second runs."""
import ctypes as C

import numpy as np
import pytest
import torch

import harness as H
import workloads as W
from paper_2007_05105_amd import BF16, EST_NORM_RATIO, F32, LAGGED_R, AdaScaleError, State, step_flat

pytestmark = pytest.mark.gpu


def read_state(buf: torch.Tensor) -> State:
    raw = buf.cpu().numpy().tobytes()
    return State.from_buffer_copy(raw[:C.sizeof(State)])


def both_ways(numel, S, dtype, flags, wd, steps, seed):
    wl = W.custom([(numel,)], S, grad_dtype=dtype, weight_decay=wd, theta=0.5, lr_table=W.lr_step_decay(0.1, 12),
                  steps=steps, seed=seed)
    a, b = W.Inputs(wl, "cuda:0"), W.Inputs(wl, "cuda:0")
    assert torch.equal(a.w_flat, b.w_flat)
    ctx = H.make_gpu(wl, flags=flags)
    lr_dev = torch.tensor(wl.lr_table, device="cuda:0")
    state = torch.zeros(16, dtype=torch.float64, device="cuda:0")      # 128 bytes >= sizeof(adascale_state)
    assert C.sizeof(State) <= state.numel() * 8
    for t in range(steps):
        a.fill_grads(t)
        b.fill_grads(t)
        ctx.step(a.w, a.v, a.g)
        step_flat(b.w[0], b.v[0], [g[0] for g in b.g], lr_dev, state, wl.momentum, wl.weight_decay, wl.theta, wl.eps,
                  dtype, flags)
        ref, got = ctx.get_state(), read_state(state)
        rel = H.compare_step(got, ref, S)
        worst = max(v for k, v in rel.items() if not k.endswith("_plain"))
        ew = float((a.w_flat - b.w_flat).abs().max() / a.w_flat.abs().max())
        ev = float((a.v_flat - b.v_flat).abs().max() / a.v_flat.abs().max())
        print(f"numel {numel} S {S} dtype {dtype} flags {flags} step {t}: scalars {worst:.3g} w {ew:.3g} v {ev:.3g} "
              f"r {got.r:.6g} tau {got.tau:.6g}", flush=True)
        assert worst <= H.TOL_SCALAR and got.step == ref.step == t + 1 and got.done == ref.done
        assert ew <= H.TOL_W and ev <= H.TOL_W
    ctx.close()


def test_flat_step_matches_the_context_step_twice_in_a_row_second_smaller():
    both_ways(1_300_001, 16, F32, 0, 1e-3, 3, 5)         # 318 tiles over 318 workgroups... and a ragged tail
    both_ways(5003, 3, BF16, 0, 0.0, 3, 6)               # smaller: fewer partial slots than the block still holds
    both_ways(3_000_000, 64, BF16, LAGGED_R, 1e-4, 2, 7)  # more tiles than workgroups
    both_ways(77, 1, F32, EST_NORM_RATIO, 1e-3, 2, 8)


def test_flat_step_rejects_what_its_fixed_scratch_cannot_hold():
    w = torch.zeros(100, device="cuda:0")
    v = torch.zeros(100, device="cuda:0")
    g = [torch.ones(100, device="cuda:0") for _ in range(65)]
    lr = torch.tensor([0.1], device="cuda:0")
    state = torch.zeros(16, dtype=torch.float64, device="cuda:0")
    with pytest.raises(AdaScaleError) as e:
        step_flat(w, v, g, lr, state)
    assert e.value.code == 1 and "64" in str(e.value)
    with pytest.raises(AdaScaleError) as e:
        step_flat(w, v, g[:2], lr, state, numel=1 << 40)
    assert e.value.code == 1 and "elements" in str(e.value)
    with pytest.raises(AdaScaleError) as e:
        step_flat(w, v, [g[0], torch.ones(100)], lr, state)   # a gradient in host memory
    assert e.value.code == 1 and "device memory" in str(e.value)
    torch.cuda.synchronize()
    assert float(w.abs().max()) == 0.0 and float(state.abs().max()) == 0.0     # nothing ran
