"""Build libgensor.so for gfx950: one translation unit per group of kernel instances
(generated from lattice.py), the registry table, the constructor and the C ABI."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
PKG = os.path.dirname(HERE)
GEN = os.path.join(HERE, "_build")
LIB = os.path.join(PKG, "libgensor.so")
PROBE_LIB = os.path.join(PKG, "libgensor_probe.so")     # the benchmark's MFMA-only probe, a library of its own
sys.path.insert(0, HERE)
import lattice  # noqa: E402

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", HERE,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
# patch-staged convolution units only: accumulators stay in plain VGPRs (no copies to and from
# AGPRs around the tap loop)
CONV_FLAGS = ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]
PER_TU = 4


def _write_if_changed(path, text):
    if os.path.exists(path) and open(path).read() == text:
        return
    with open(path, "w") as f:
        f.write(text)


def generate():
    os.makedirs(GEN, exist_ok=True)
    L = lattice.lattice()
    tus = []
    # translation units hold instances of one kernel template only (they are built with different flags)
    ordered = [d for d in L if not d["units"]]
    ordered += [None] * (-len(ordered) % PER_TU) + [d for d in L if d["units"]]
    for t in range(0, len(ordered), PER_TU):
        group = [d for d in ordered[t:t + PER_TU] if d is not None]
        src = ['#include "registry.hpp"', "namespace gensor {"]
        for d in group:
            src.append("typedef %s C_%d;" % (lattice.cfg_type(d), d["id"]))
            src.append("hipError_t launch_%d(const KernelArgs& a, hipStream_t st) { return %s<C_%d>(a, st); }"
                       % (d["id"], "launch_conv_instance" if d["units"] else "launch_instance", d["id"]))
            if lattice.splittable(d):
                src.append("hipError_t launch_split_%d(const KernelArgs& a, hipStream_t st) { return launch_instance<C_%d, true>(a, st); }"
                           % (d["id"], d["id"]))
        src.append("}  // namespace gensor\n")
        path = os.path.join(GEN, "%s_%03d.hip" % ("conv" if group[0]["units"] else "inst", t // PER_TU))
        _write_if_changed(path, "\n".join(src))
        tus.append(path)
    for f in os.listdir(GEN):                      # units of an earlier lattice
        if f.endswith(".hip") and os.path.join(GEN, f) not in tus and f != "registry.hip":
            os.remove(os.path.join(GEN, f))
            if os.path.exists(os.path.join(GEN, f[:-4] + ".o")):
                os.remove(os.path.join(GEN, f[:-4] + ".o"))
    reg = ['#include "registry.hpp"', "#if !defined(__HIP_DEVICE_COMPILE__)", "namespace gensor {"]
    for d in L:
        reg.append("hipError_t launch_%d(const KernelArgs&, hipStream_t);" % d["id"])
        if lattice.splittable(d):
            reg.append("hipError_t launch_split_%d(const KernelArgs&, hipStream_t);" % d["id"])
    reg.append("const InstanceDesc g_instances[] = {")
    for d in L:
        es = 4 if d["dt"] == "f32" else 2
        kg = (64 // d["mb"]) * (16 // es)
        a_bytes = d["bm"] * d["bk"] * es if d["asrc"] == "KC" else d["bk"] * (d["bm"] * es + lattice.pad_m(d))
        b_bytes = d["bn"] * d["bk"] * es if (d["bsrc"] == "KC" or d["direct"]) else d["bk"] * (d["bn"] * es + lattice.pad_n(d))
        lds = 0 if d["units"] else (a_bytes + b_bytes) * d["stages"]
        threads = (d["bm"] // d["wm"]) * (d["bn"] // d["wn"]) * 64
        reg.append("  {%d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, launch_%d, %s}," % (
            d["id"], lattice.DT[d["dt"]], lattice.DT[d["out"]], d["bm"], d["bn"], d["bk"], d["wm"], d["wn"], d["mb"],
            d["vm"], d["vn"], lattice.BSRC[d["bsrc"]], lattice.ASRC[d["asrc"]], d["vec"], d["stages"], d["direct"], lds, threads, kg, d["units"], d["id"],
            ("launch_split_%d" % d["id"]) if lattice.splittable(d) else "nullptr"))
    reg.append("};")
    reg.append("const int g_num_instances = %d;" % len(L))
    reg.append("}  // namespace gensor")
    reg.append("#endif\n")
    path = os.path.join(GEN, "registry.hip")
    _write_if_changed(path, "\n".join(reg))
    tus.append(path)
    return tus


def _compile(src):
    obj = os.path.join(GEN, os.path.basename(src).rsplit(".", 1)[0] + ".o")
    deps = [src, os.path.join(HERE, "gemm_kernel.hpp"), os.path.join(HERE, "conv_kernel.hpp"), os.path.join(HERE, "registry.hpp"),
            os.path.join(HERE, "host_common.hpp"), os.path.join(PKG, "..", "include", "gensor.h")]
    if os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps if os.path.exists(d)):
        return obj
    # host sources: no fused multiply-add contraction, so the constructor's double arithmetic
    # is the plain IEEE sequence its tests compare against
    extra = ["-ffp-contract=off"] if src.endswith(".cpp") else []
    if os.path.basename(src).startswith("conv_"):
        extra += CONV_FLAGS
    cmd = [HIPCC] + FLAGS + extra + ["-x", "hip", "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(force=False, jobs=None):
    tus = generate()
    tus += [os.path.join(HERE, "gensor_api.cpp"), os.path.join(HERE, "constructor.cpp"), os.path.join(HERE, "scan_kernels.cpp")]
    probe = os.path.join(HERE, "probe.cpp")
    if force:
        for f in os.listdir(GEN):
            if f.endswith(".o"):
                os.remove(os.path.join(GEN, f))
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, tus + [probe]))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs[:-1], check=True)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBE_LIB, objs[-1]], check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
