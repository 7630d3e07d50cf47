"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the constructor, the host side of the operator
entry points and the C oracle are compiled with -fsanitize=address,undefined (host only; the kernels are replaced
by stubs, the GPU toolchain's sanitizers are not involved) together with tests/sanitize_host.cpp, and the driver is
run on the CPU.  Any report makes it exit non-zero."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2502_11407_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]


def test_constructor_api_and_oracle_under_asan_ubsan(tmp_path):
    sys.path.insert(0, CSRC)
    import build as kernel_build
    import lattice
    kernel_build.generate()                       # the registry table of the current lattice
    stubs = ['#include "registry.hpp"', "namespace gensor {"]
    for d in lattice.lattice():
        stubs.append("hipError_t launch_%d(const KernelArgs&, hipStream_t) { return hipErrorNotSupported; }" % d["id"])
        if lattice.splittable(d):
            stubs.append("hipError_t launch_split_%d(const KernelArgs&, hipStream_t) { return hipErrorNotSupported; }" % d["id"])
    stubs.append("}\n")
    (tmp_path / "stubs.cpp").write_text("\n".join(stubs))
    objs = []
    hip_flags = ["-x", "hip", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-I", CSRC,
                 "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"] + SAN
    for src in (os.path.join(CSRC, "constructor.cpp"), os.path.join(CSRC, "gensor_api.cpp"), os.path.join(CSRC, "scan_kernels.cpp"),
                os.path.join(CSRC, "_build", "registry.hip"), str(tmp_path / "stubs.cpp"), os.path.join(ROOT, "tests", "sanitize_host.cpp")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        r = subprocess.run([HIPCC] + hip_flags + ["-c", src, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        objs.append(obj)
    obj = str(tmp_path / "oracle_ops.o")
    r = subprocess.run(["/opt/rocm/lib/llvm/bin/clang", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=undefined", "-c", os.path.join(ROOT, "oracle", "oracle_ops.c"), "-o", obj],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    objs.append(obj)
    exe = str(tmp_path / "host_check")
    r = subprocess.run([HIPCC, "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined"] + objs + ["-lm", "-o", exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    print(r.stdout[-2000:])
    print(r.stderr[-4000:])
    assert r.returncode == 0 and "sanitized host paths ok" in r.stdout
