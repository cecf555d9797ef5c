"""CPU-side checks of the boundary: the library loads, exports every symbol the header
declares, and reports a missing GPU as an error code (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

from paper_2007_05105_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adascale_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.library_path()):
        pytest.skip("libadascale.so not built (run __graft_entry__.build())")
    lib = C.CDLL(binding.library_path())
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["adascale.h", "adascale_diag.h"]
    for header, exports in (("adascale.h", binding.EXPORTS), ("adascale_diag.h", binding.EXPORTS_DIAG)):
        names = declared_symbols(header)
        assert len(names) >= 7
        for n in names:
            assert hasattr(lib, n), n
        assert sorted(exports) == names          # the Python binding carries the same names


def test_library_reads_no_environment_variables():
    """What a call does depends on its arguments alone: the library does not import getenv."""
    import subprocess
    if not os.path.exists(binding.library_path()):
        pytest.skip("libadascale.so not built")
    out = subprocess.run(["nm", "-D", "--undefined-only", binding.library_path()], capture_output=True, text=True,
                         check=True).stdout
    assert "getenv" not in out


def test_struct_layouts_match_header(tmp_path):
    """Compile the header with gcc and compare sizes and offsets with the ctypes mirrors."""
    import subprocess
    src = tmp_path / "layout.c"
    fields_c = [n for n, _ in binding.Config._fields_]
    fields_s = [n for n, _ in binding.State._fields_]
    fields_p = [n for n, _ in binding.PlanInfo._fields_]
    fields_t = [n for n, _ in binding.Tuning._fields_]
    fields_f = [n for n, _ in binding.FlatStep._fields_]
    body = "".join(f'printf("%zu\\n", offsetof(adascale_config, {f}));' for f in fields_c)
    body += "".join(f'printf("%zu\\n", offsetof(adascale_state, {f}));' for f in fields_s)
    body += "".join(f'printf("%zu\\n", offsetof(adascale_plan_info, {f}));' for f in fields_p)
    body += 'printf("%zu\\n", sizeof(adascale_plan_info));'
    body += "".join(f'printf("%zu\\n", offsetof(adascale_tuning, {f}));' for f in fields_t)
    body += 'printf("%zu\\n", sizeof(adascale_tuning));'
    body += "".join(f'printf("%zu\\n", offsetof(adascale_flat_step, {f}));' for f in fields_f)
    body += 'printf("%zu\\n%d\\n%lld\\n", sizeof(adascale_flat_step), ADASCALE_FLAT_MAX_SCALE, (long long)ADASCALE_FLAT_MAX_NUMEL);'
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "adascale_diag.h"\nint main(void){'
                   'printf("%zu\\n%zu\\n", sizeof(adascale_config), sizeof(adascale_state));' + body + "return 0;}")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = [int(x) for x in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    assert out[0] == C.sizeof(binding.Config) and out[1] == C.sizeof(binding.State)
    got = [getattr(binding.Config, f).offset for f in fields_c] + [getattr(binding.State, f).offset for f in fields_s]
    got += [getattr(binding.PlanInfo, f).offset for f in fields_p] + [C.sizeof(binding.PlanInfo)]
    got += [getattr(binding.Tuning, f).offset for f in fields_t] + [C.sizeof(binding.Tuning)]
    got += [getattr(binding.FlatStep, f).offset for f in fields_f] + [C.sizeof(binding.FlatStep)]
    got += [binding.FLAT_MAX_SCALE, binding.FLAT_MAX_NUMEL]
    assert out[2:] == got


def test_init_argument_errors_need_no_gpu():
    if not os.path.exists(binding.library_path()):
        pytest.skip("libadascale.so not built")
    with pytest.raises(binding.AdaScaleError) as e:
        binding.AdaScale([10], 0, [0.1])
    assert e.value.code == 1 and "S" in str(e.value)
    with pytest.raises(binding.AdaScaleError):
        binding.AdaScale([10], 2, [0.1], momentum=1.5)


def test_every_scale_up_to_4096_has_a_kernel_shape_and_instances():
    """Host logic that picks the kernel instance: the half-groups cover S with less than one pair of
    half-groups of padding, loads per half-group stay within what the register buffers hold, and an
    instance exists for every scale in range (outside it the general kernels run)."""
    if not os.path.exists(binding.library_path()):
        pytest.skip("libadascale.so not built")
    for dtype, cap in ((0, 4), (1, 8)):
        for S in range(1, 4097):
            mask, (hg, nh, padded) = binding.kernel_shape(dtype, S)
            assert mask == 3, (dtype, S)
            assert 1 <= hg <= cap and hg & (hg - 1) == 0
            assert nh >= 2 and nh % 2 == 0
            assert padded == hg * nh and S <= padded < S + 2 * hg
            assert 2 * hg >= min(S, 2 * cap)          # the two buffers together hold S, or are full size
        for S in (0, -3, 4097, 1 << 20):
            assert binding.kernel_shape(dtype, S)[0] == 0
    assert binding.kernel_shape(7, 16)[0] == 0
    # the shapes the benchmark configurations run with
    assert binding.kernel_shape(0, 16)[1] == (4, 4, 16)
    assert binding.kernel_shape(0, 8)[1] == (4, 2, 8)
    assert binding.kernel_shape(1, 32)[1] == (8, 4, 32)
    assert binding.kernel_shape(1, 64)[1] == (8, 8, 64)


def test_plan_of_the_benchmark_configurations():
    """Host logic that lays a parameter list out over the chip (no device needed): tile counts
    against a count in Python, the split of the mean gradient between registers, LDS and memory,
    and the path, for the five workloads on an MI355X-sized device."""
    if not os.path.exists(binding.library_path()):
        pytest.skip("libadascale.so not built")
    import workloads as W
    expect = {1: "fused", 2: "fused", 3: "fused", 4: "fused", 5: "fused", 6: "streaming"}
    for cfg in range(1, 7):
        wl = W.config(min(cfg, 5))
        if cfg == 6:                                  # three times cfg5's list: 1.05 G parameters, 3 % of them on chip
            wl = W.custom([tuple(s) for s in wl.shapes] * 3, wl.S, grad_dtype=wl.grad_dtype)
        p = binding.plan(wl.numel, wl.S, wl.grad_dtype)
        full = sum(n // 2048 for n in wl.numel)
        ragged = sum(1 for n in wl.numel if n % 2048)
        assert (p["full_tiles"], p["ragged_tiles"]) == (full, ragged)
        assert p["path"] == expect[cfg], (cfg, p)
        assert p["stream_grid"] == min(256, max((full + 1) // 2, ragged, 1))
        if p["path"] == "fused":
            g = p["fused_grid"]
            assert g == min(256, max(full, ragged)) and p["tiles_per_workgroup"] == -(-full // g)
            assert p["register_tiles"] in (0, 10, 30, 44) and p["register_tiles"] <= full // g   # every workgroup fills them
            assert p["register_tiles"] + p["lds_tiles"] <= p["tiles_per_workgroup"]
            assert 0 <= p["lds_tiles"] <= 19                                                   # 19 tiles of 8 KB fit beside the static LDS
            kept = min(p["tiles_per_workgroup"], p["register_tiles"] + p["lds_tiles"])
            assert p["on_chip_percent"] == min(100, 100 * kept // p["tiles_per_workgroup"]) >= 8
    p3, p4 = binding.plan(W.config(3).numel, 16), binding.plan(W.config(4).numel, 32, binding.BF16)
    # cfg3's 49 tiles per workgroup fit with 30 in registers and 19 in LDS: the lowest level that keeps everything on chip
    assert (p3["register_tiles"], p3["lds_tiles"], p3["tiles_per_workgroup"], p3["on_chip_percent"]) == (30, 19, 49, 100)
    assert (p4["register_tiles"], p4["lds_tiles"], p4["tiles_per_workgroup"], p4["on_chip_percent"]) == (44, 19, 116, 54)
    p5 = binding.plan(W.config(5).numel, 64, binding.BF16)
    assert (p5["register_tiles"], p5["lds_tiles"], p5["tiles_per_workgroup"], p5["on_chip_percent"]) == (44, 19, 670, 9)
    # scales beyond the 512-lane kernels' range, an empty list, and the knobs of the tuning record
    assert binding.plan(W.config(3).numel, 5000)["path"] == "general"
    assert binding.plan([], 4) == dict(binding.plan([0, 0], 4), path="general")
    assert binding.plan([7], 4)["ragged_tiles"] == 1 and binding.plan([7], 4)["fused_grid"] == 1
    T = binding.Tuning
    assert binding.plan(W.config(3).numel, 16, tuning=T(force_path=binding.FORCE_STREAMING))["path"] == "streaming"
    assert binding.plan(W.config(3).numel, 16, tuning=T(force_path=binding.FORCE_GENERAL))["path"] == "general"
    forced = binding.plan(W.config(5).numel, 64, binding.BF16, tuning=T(force_path=binding.FORCE_FUSED))
    assert forced["path"] == "fused" and forced["on_chip_percent"] == 9
    big = [n for n in W.config(5).numel] * 3
    assert binding.plan(big, 64, binding.BF16)["path"] == "streaming"
    assert binding.plan(big, 64, binding.BF16, tuning=T(force_path=binding.FORCE_FUSED))["on_chip_percent"] == 3
    assert binding.plan(W.config(4).numel, 32, binding.BF16, tuning=T(fused_min_percent=60))["path"] == "streaming"
    assert binding.plan(W.config(5).numel, 64, binding.BF16, tuning=T(fused_min_percent=10))["path"] == "streaming"
    assert binding.plan(big, 64, binding.BF16, tuning=T(fused_min_percent=3))["path"] == "fused"
    few = binding.plan(W.config(1).numel, 4, tuning=T(fused_max_grid=2))
    assert few["fused_grid"] == 2 and few["tiles_per_workgroup"] == 244 and few["register_tiles"] + few["lds_tiles"] == 63
    os.environ["ADASCALE_FUSED"] = "2"              # the library does not read the environment
    try:
        assert binding.plan(W.config(3).numel, 16)["path"] == "fused"
    finally:
        del os.environ["ADASCALE_FUSED"]
    # a device with a quarter of the compute units keeps a quarter of the parameters on chip
    small = binding.plan(W.config(3).numel, 16, compute_units=64)
    assert small["fused_grid"] == 64 and small["on_chip_percent"] == 100 * 63 // small["tiles_per_workgroup"]
    with pytest.raises(binding.AdaScaleError):
        binding.plan([10], 0)
    with pytest.raises(binding.AdaScaleError):
        binding.plan([-1], 2)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "library_path", lambda: str(tmp_path / "libadascale.so"))
    with pytest.raises(ImportError):
        binding.load_library()


def test_bench_refuses_more_than_one_gpu():
    """This build is for one GPU: bench.py says so and exits before touching any device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
