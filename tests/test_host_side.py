"""CPU checks of host-side pieces that hold none of the method's arithmetic: the baseline schedule
tables (linear scaling with warm-up and its stretched form) and the layout of the synthetic inputs."""
import math

import numpy as np
import pytest

from paper_2007_05105_amd import schedules as SCH


def step_table(L=800, lr0=0.1):
    t = np.full(L, lr0, dtype=np.float32)
    t[L // 2:] *= 0.1
    t[3 * L // 4:] *= 0.1
    return t


@pytest.mark.parametrize("S", [1, 2, 8, 16, 64])
def test_lsw_length_warmup_and_scaled_tail(S):
    lr = step_table()
    out = SCH.lsw_schedule(lr, S)
    T_S = math.ceil(len(lr) / S)
    W = int(round(0.055 * T_S))
    assert out.dtype == np.float32 and len(out) == T_S                 # ceil(T / S) iterations (Sec. 3.1, Def. 2)
    assert out[0] == pytest.approx(lr[0])                              # warm-up starts at the single-batch rate
    if W > 0:
        d = np.diff(out[:W].astype(np.float64))
        assert np.allclose(d, (S - 1) * lr[0] / W, rtol=1e-4, atol=1e-9)   # and rises linearly ...
        assert out[W] == pytest.approx(S * lr[min(S * W, len(lr) - 1)])    # ... to the scaled schedule
    for t in range(W, T_S):
        assert out[t] == pytest.approx(S * lr[min(S * t, len(lr) - 1)], rel=1e-6)
    if S == 1:
        assert np.array_equal(out[W:], lr[W:])                         # scale 1: the single-batch schedule


def test_lsw_without_warmup_is_definition_2():
    lr = np.linspace(1.0, 0.1, 37).astype(np.float32)
    out = SCH.lsw_schedule(lr, 4, warmup_fraction=0.0)
    assert len(out) == 10
    assert np.allclose(out, 4 * lr[np.minimum(4 * np.arange(10), 36)])


def test_lsw_plus_stretches_to_the_given_length():
    lr = step_table()
    base = SCH.lsw_schedule(lr, 8)
    out = SCH.lsw_plus_schedule(lr, 8, 250)
    assert len(out) == 250 and out[0] == base[0] and out[-1] == base[-1]
    assert np.array_equal(SCH.lsw_plus_schedule(lr, 8, len(base)), base)      # same length: unchanged
    # every entry of LSW appears, in order
    assert np.array_equal(out[np.sort(np.unique(out, return_index=True)[1])],
                          base[np.sort(np.unique(base, return_index=True)[1])])


def test_bad_arguments():
    with pytest.raises(ValueError):
        SCH.lsw_schedule([], 2)
    with pytest.raises(ValueError):
        SCH.lsw_schedule([0.1], 0)
    with pytest.raises(ValueError):
        SCH.lsw_plus_schedule([0.1], 2, 0)


def test_gradient_buffers_are_rows_of_one_allocation():
    """Input layout (no arithmetic of the method): S rows of one allocation, disjoint, the same
    tensor offsets in every row; rows of 2 MiB or more start on 2 MiB boundaries."""
    import workloads as W
    wl = W.custom([(5000,), (3, 7), (1,)], 4, steps=1)
    inp = W.Inputs(wl, "cpu")
    base = inp.g_all.data_ptr()
    starts = [f.data_ptr() - base for f in inp.g_flat]
    assert starts == sorted(starts) and starts[0] == 0
    assert all(b - a >= inp.len_g * 4 and (b - a) % 256 == 0 for a, b in zip(starts, starts[1:]))
    for row in inp.g:
        assert [t.numel() for t in row] == list(wl.numel)
    assert [[t.data_ptr() - f.data_ptr() for t in row] for row, f in zip(inp.g, inp.g_flat)] == \
           [[o * 4 for o in inp.offs_g]] * 4
    big = W.custom([(600000,)], 3, steps=1)                      # 2.4 MB per row
    inp = W.Inputs(big, "cpu")
    starts = [f.data_ptr() - inp.g_all.data_ptr() for f in inp.g_flat]
    assert starts == [0, 4 << 20, 8 << 20]
    sep = W.Inputs(wl, "cpu", one_allocation=False)
    assert len({f.untyped_storage().data_ptr() for f in sep.g_flat}) == 4
