"""The C-ABI library loads and exports every symbol include/gensor.h declares (no compute
calls here: those need a GPU); host-side argument checks that return before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "gensor.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gensor_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2502_11407_amd import binding
    names = _declared()
    assert {"gensor_gemm", "gensor_bmm", "gensor_conv2d", "gensor_construct"} <= set(names)
    assert set(names) == set(binding.EXPORTS)
    raw = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert getattr(raw, n) is not None, n


def test_struct_layouts_match_the_header(tmp_path):
    """Compile the header with gcc and compare sizeof/offsetof with the ctypes mirrors."""
    import subprocess
    from paper_2502_11407_amd import binding
    src = tmp_path / "sz.c"
    src.write_text('#include "gensor.h"\n#include <stdio.h>\n#include <stddef.h>\nint main(void){printf("%zu %zu %zu %zu %zu %zu %zu\\n",'
                   'sizeof(gensor_problem), sizeof(gensor_schedule), sizeof(gensor_hw), sizeof(gensor_construct_opts),'
                   'offsetof(gensor_problem, stride), offsetof(gensor_schedule, seed), offsetof(gensor_hw, launch_us));return 0;}\n')
    exe = tmp_path / "sz"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    want = [ctypes.sizeof(binding.Problem), ctypes.sizeof(binding.Schedule), ctypes.sizeof(binding.Hw),
            ctypes.sizeof(binding.ConstructOpts), binding.Problem.stride.offset, binding.Schedule.seed.offset,
            binding.Hw.launch_us.offset]
    assert got == want
    assert binding.num_instances() > 50


def test_host_side_argument_checks_without_a_gpu():
    from paper_2502_11407_amd import binding as gs
    bad = gs.gemm_problem("f16", 0, 64, 64, 0, 1)
    buf = ctypes.create_string_buffer(64)
    addr = ctypes.addressof(buf)
    st = gs.lib.gensor_gemm(None, ctypes.byref(bad), 1.0, addr, 64, addr, 64, 0.0, addr, 64, None, 0, None)
    assert st == 1
    ok = gs.gemm_problem("f16", 64, 64, 64, 0, 1)
    assert gs.lib.gensor_gemm(None, ctypes.byref(ok), 1.0, None, 64, addr, 64, 0.0, addr, 64, None, 0, None) == 1
    assert gs.lib.gensor_gemm(None, ctypes.byref(ok), 1.0, addr, 8, addr, 64, 0.0, addr, 64, None, 0, None) == 1
    conv = gs.conv_problem("f16", 1, 4, 2, 2, 4, 3, 3, 1, 0)      # filter larger than the image
    assert gs.lib.gensor_conv2d(None, ctypes.byref(conv), addr, addr, addr, None, 0, None) == 1
    assert gs.status_string(3).startswith("no feasible schedule")
    assert gs.instance_schedule(0, gs.gemm_problem("f32", 8, 8, 8)) is None
