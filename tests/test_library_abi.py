"""CPU-side checks of the boundary: the library loads, exports every symbol the header
declares, and reports a missing GPU as an error code (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

from paper_2007_05105_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "adascale.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adascale_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.library_path()):
        pytest.skip("libadascale.so not built (run __graft_entry__.build())")
    lib = C.CDLL(binding.library_path())
    names = declared_symbols()
    assert len(names) >= 8
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names      # the Python binding carries the same names


def test_struct_layouts_match_header(tmp_path):
    """Compile the header with gcc and compare sizes and offsets with the ctypes mirrors."""
    import subprocess
    src = tmp_path / "layout.c"
    fields_c = [n for n, _ in binding.Config._fields_]
    fields_s = [n for n, _ in binding.State._fields_]
    body = "".join(f'printf("%zu\\n", offsetof(adascale_config, {f}));' for f in fields_c)
    body += "".join(f'printf("%zu\\n", offsetof(adascale_state, {f}));' for f in fields_s)
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "adascale.h"\nint main(void){'
                   'printf("%zu\\n%zu\\n", sizeof(adascale_config), sizeof(adascale_state));' + body + "return 0;}")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = [int(x) for x in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    assert out[0] == C.sizeof(binding.Config) and out[1] == C.sizeof(binding.State)
    got = [getattr(binding.Config, f).offset for f in fields_c] + [getattr(binding.State, f).offset for f in fields_s]
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
