"""The kernels that issue their LDS fragment reads from inline assembly (direct staging with an n-contiguous 16-bit
B operand) wait for those reads themselves, because the compiler's counter bookkeeping does not see them.  This test
compiles every such instance to assembly (this repository's own kernels, device code only, no GPU needed) and checks
the contract instruction by instruction: a register written by an LDS read is not touched by any instruction until
an `s_waitcnt lgkmcnt(k)` has executed with k no larger than the number of LDS operations issued after that read
(LDS operations complete in issue order), along every path through the kernel."""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2502_11407_amd", "csrc")
sys.path.insert(0, CSRC)

REG = re.compile(r"\b([va])\[(\d+):(\d+)\]|\b([va])(\d+)\b")


def _regs(text):
    out = set()
    for m in REG.finditer(text):
        if m.group(1):
            out.update((m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1))
        else:
            out.add((m.group(4), int(m.group(5))))
    return out


def check_function(lines):
    """lines: the instruction and label lines of one kernel.  Returns (violations, transposing reads seen)."""
    labels = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    entry_state = {}                       # label index -> {reg: younger LDS ops} merged over the paths found so far
    violations, reads = [], 0

    def merge(into, state):
        changed = False
        for r, age in state.items():
            if r not in into or age < into[r]:
                into[r] = age
                changed = True
        return changed

    work = [(0, {})]
    seen_reads = set()
    while work:
        i, pending = work.pop()
        pending = dict(pending)
        while i < len(lines):
            l = lines[i]
            if l.endswith(":"):
                st = entry_state.setdefault(i, None)
                if st is None:
                    entry_state[i] = dict(pending)
                elif not merge(st, pending):
                    break                                  # nothing new reaches this label
                pending = dict(entry_state[i])
                i += 1
                continue
            op, _, rest = l.partition(" ")
            if op == "s_waitcnt":
                m = re.search(r"lgkmcnt\((\d+)\)", rest)
                if m:
                    k = int(m.group(1))
                    pending = {r: age for r, age in pending.items() if age < k}
            elif op == "s_endpgm":
                break
            else:
                touched = _regs(rest) & set(pending)
                if touched:
                    violations.append((i, l, sorted(touched)))
                    for r in touched:
                        del pending[r]
                if op.startswith("ds_"):
                    pending = {r: age + 1 for r, age in pending.items()}
                    if op.startswith("ds_read"):
                        if i not in seen_reads:
                            seen_reads.add(i)
                            reads += 1
                        for r in _regs(rest.split(",")[0]):
                            pending[r] = 0
                if op.startswith("s_cbranch") or op == "s_branch":
                    target = rest.strip()
                    if target in labels:
                        work.append((labels[target], pending))
                    if op == "s_branch":
                        break
            i += 1
    return violations, reads


def _functions(asm):
    cur, out = None, []
    for raw in asm.splitlines():
        l = raw.split(";")[0].strip()
        if not l or l.startswith("."):
            if re.match(r"^\.LBB\d+_\d+:", l):
                if cur is not None:
                    cur.append(l)
            continue
        if l.endswith(":"):
            if "contraction_kernel" in l:
                cur = []
                out.append(cur)
            continue
        if cur is not None:
            cur.append(l)
            if l.startswith("s_endpgm") and False:
                cur = None
    return out


def test_checker_catches_an_early_use():
    good = ["ds_read_b64_tr_b16 v[4:5], v9", "ds_read_b128 v[10:13], v9", "s_waitcnt lgkmcnt(1)", "v_mov_b32_e32 v0, v4",
            "s_waitcnt lgkmcnt(0)", "v_mov_b32_e32 v1, v10", "s_endpgm"]
    assert check_function(good) == ([], 2)
    assert check_function(good[:4] + ["v_mov_b32_e32 v1, v10", "s_endpgm"])[0]          # the second read is still pending
    early = ["ds_read_b64_tr_b16 v[4:5], v9", "v_mov_b32_e32 v0, v4", "s_endpgm"]
    assert check_function(early)[0]
    weak = ["ds_read_b64_tr_b16 v[4:5], v9", "s_waitcnt lgkmcnt(1)", "v_mfma_f32_32x32x16_f16 v[16:31], v[0:3], v[4:7], v[16:31]", "s_endpgm"]
    assert check_function(weak)[0]
    loop = [".LBB0_1:", "v_mov_b32_e32 v0, v4", "ds_read_b64_tr_b16 v[4:5], v9", "s_cbranch_scc0 .LBB0_1", "s_endpgm"]
    assert check_function(loop)[0]                      # pending across the back edge
    loop_ok = [".LBB0_1:", "s_waitcnt lgkmcnt(0)", "v_mov_b32_e32 v0, v4", "ds_read_b64_tr_b16 v[4:5], v9", "s_cbranch_scc0 .LBB0_1",
               "s_waitcnt vmcnt(0) lgkmcnt(0)", "v_mov_b32_e32 v1, v5", "s_endpgm"]
    assert check_function(loop_ok)[0] == []


def test_every_instance_with_assembly_reads_waits_for_them(tmp_path):
    import build as kernel_build
    import lattice
    insts = [d for d in lattice.lattice() if d["bsrc"] == "NC" and d["direct"] and d["dt"] != "f32" and not d["units"]]
    assert len(insts) >= 20

    def one(d):
        src = tmp_path / ("i%d.hip" % d["id"])
        body = ['#include "registry.hpp"', "namespace gensor {", "typedef %s C_X;" % lattice.cfg_type(d),
                "hipError_t l0(const KernelArgs& a, hipStream_t st) { return launch_instance<C_X>(a, st); }"]
        if lattice.splittable(d):
            body.append("hipError_t l1(const KernelArgs& a, hipStream_t st) { return launch_instance<C_X, true>(a, st); }")
        body.append("}\n")
        src.write_text("\n".join(body))
        out = tmp_path / ("i%d.s" % d["id"])
        r = subprocess.run([kernel_build.HIPCC] + kernel_build.FLAGS + ["-x", "hip", "--cuda-device-only", "-S", str(src), "-o", str(out)],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        res = []
        for fn in _functions(out.read_text()):
            res.append(check_function(fn))
        return d["id"], res

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        results = list(ex.map(one, insts))
    for idx, res in results:
        assert res, idx
        for violations, reads in res:
            assert reads > 0, "instance %d: no LDS reads found" % idx
            assert not violations, "instance %d: %s" % (idx, violations[:3])
