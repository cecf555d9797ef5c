"""A step captured into a HIP graph and replayed against the same steps issued directly: bit for
bit the same state and weights after every replay, with the program's own eager work (new
gradients written into the same buffers) and synchronisations between the replays.  What changes
from step to step lives on the device and is advanced by the kernels, so the captured launch
arguments stay valid."""
import pytest
import torch

import harness as H
import workloads as W
from paper_2007_05105_amd import (BF16, EST_NORM_RATIO, F32, FORCE_FUSED, FORCE_GENERAL, FORCE_STREAMING, LAGGED_R,
                                  AdaScaleError, Tuning)

pytestmark = pytest.mark.gpu

# the three implementations of the step, and the two sweeps that write as they read with their write
# bursts forced (small rings, 2 us clock windows): the fused step on two workgroups, so that most
# tiles lie beyond the chip's capacity, and the streaming sweep
PATHS = {"fused": dict(force_path=FORCE_FUSED), "three_kernel": dict(force_path=FORCE_STREAMING),
         "general": dict(force_path=FORCE_GENERAL),
         "fused_beyond_capacity_bursts": dict(force_path=FORCE_FUSED, fused_max_grid=2, burst_tiles=3, burst_window_ticks=200),
         "three_kernel_bursts": dict(force_path=FORCE_STREAMING, burst_tiles=3, burst_window_ticks=200)}


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("S,dtype,flags", [(8, F32, 0), (8, F32, LAGGED_R), (5, BF16, EST_NORM_RATIO)])
def test_captured_step_replays_like_direct_steps(path, S, dtype, flags):
    T = 7
    tun = Tuning(**PATHS[path])
    wl = W.custom([(300000,), (999,), (70001,), (2048 * 40,)], S, grad_dtype=dtype, weight_decay=1e-3, theta=0.7,
                  lr_table=W.lr_step_decay(0.1, 40), steps=T, seed=91)

    direct, inp = H.make_gpu(wl, flags=flags, tuning=tun), W.Inputs(wl, "cuda:0")
    want = []
    for t in range(T):
        inp.fill_grads(t)
        direct.step(inp.w, inp.v, inp.g)
        want.append((direct.get_state().as_dict(), inp.w_flat.clone(), inp.v_flat.clone()))
    direct.close()

    gpu, inp = H.make_gpu(wl, flags=flags, tuning=tun), W.Inputs(wl, "cuda:0")
    inp.fill_grads(0)
    gpu.step(inp.w, inp.v, inp.g)                      # outside the capture: uploads the pointer table
    assert gpu.get_state().as_dict() == want[0][0] and torch.equal(inp.w_flat, want[0][1])
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        gpu.step(inp.w, inp.v, inp.g)                  # recorded on the capturing stream, not run
    torch.cuda.synchronize()
    assert gpu.get_state().as_dict() == want[0][0] and torch.equal(inp.w_flat, want[0][1])
    for t in range(1, T):
        inp.fill_grads(t)                              # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = gpu.get_state().as_dict()
        assert got == want[t][0], (path, t, got, want[t][0])
        assert torch.equal(inp.w_flat, want[t][1]) and torch.equal(inp.v_flat, want[t][2]), (path, t)
    # direct steps and replays mix: one more of each
    inp.fill_grads(0)
    gpu.step(inp.w, inp.v, inp.g)
    graph.replay()
    torch.cuda.synchronize()
    assert gpu.get_state().step == T + 2
    del graph
    gpu.close()


def test_capture_refuses_what_it_cannot_replay():
    """During capture nothing is uploaded: a set of tensor pointers the context has not seen is
    refused, and nothing is recorded for it."""
    wl = W.custom([(5000,), (77,)], 4, steps=2, seed=3)
    a, b = W.Inputs(wl, "cuda:0"), W.Inputs(wl, "cuda:0")
    a.fill_grads(0)
    b.fill_grads(0)
    gpu = H.make_gpu(wl)
    gpu.step(a.w, a.v, a.g)
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        with pytest.raises(AdaScaleError) as e:
            gpu.step(b.w, b.v, b.g)
        gpu.step(a.w, a.v, a.g)
    assert e.value.code == 4 and "capture" in str(e.value)
    w_b = b.w_flat.clone()
    graph.replay()
    torch.cuda.synchronize()
    assert gpu.get_state().step == 2 and torch.equal(b.w_flat, w_b)
    del graph
    gpu.close()
