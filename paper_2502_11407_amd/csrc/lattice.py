"""The compiled part of the schedule lattice: which (tile, wave tile, MFMA block, virtual
thread, staging) points exist as kernel instances for each element type and operand source.
build.py turns this list into one translation unit per instance plus the registry table."""
from itertools import product

DT = {"f32": 0, "f16": 1, "bf16": 2}
BSRC = {"KC": 0, "NC": 1, "CONV": 2, "NCS2": 3}
ASRC = {"KC": 0, "MC": 1}
CT = {"f32": "f32_t", "f16": "f16_t", "bf16": "bf16_t"}


def full_v(dt, bk, bsrc, asrc="KC"):
    """Virtual threads at which the fragment reads of both operand tiles are free of bank conflicts: a
    k-contiguous tile needs as many phases as it has 16-byte chunks per row; an n-contiguous one has its
    4 (16-bit) or 2 (fp32) k rows that are read together spread by the row pad."""
    es = 4 if dt == "f32" else 2
    cpr = bk * es // 16
    strided = 2 if dt == "f32" else 4
    return (cpr if asrc == "KC" else strided), (cpr if bsrc == "KC" else strided)


def _inst(dt, out, bm, bn, bk, wm, wn, mb, vm=None, vn=None, bsrc="KC", vec=1, stages=2, direct=0, units=0, asrc="KC"):
    fm, fn = (1, 1) if units else full_v(dt, bk, bsrc, asrc)
    return dict(dt=dt, out=out, bm=bm, bn=bn, bk=bk, wm=wm, wn=wn, mb=mb, vm=vm or fm, vn=vn or fn,
                bsrc=bsrc, vec=vec, stages=stages, direct=direct, units=units, asrc=asrc)


def _convp(dt, out, bm, bn, bkc, wm, wn, units, stages=2):
    """Convolution with the input patch staged in LDS (direct = 1 on the CONV source); bk = channels per stage;
    stages = LDS buffers (1: more workgroups per CU hide the load latency, 2: the next stage is written while
    this one is multiplied)."""
    return _inst(dt, out, bm, bn, bkc, wm, wn, 32, 1, 1, "CONV", 1, stages, 1, units)


def _pad(v, row_bytes):
    if v == 1:
        return 0
    t = 64 if v >= 4 else 32
    return (3 * t - row_bytes % (2 * t)) % (2 * t)


def pad_n(d):
    """Row pad in bytes of a register-staged n-contiguous B tile (the kernel's PAD_N)."""
    return _pad(d["vn"], d["bn"] * (4 if d["dt"] == "f32" else 2))


def pad_m(d):
    """Row pad in bytes of an m-contiguous A tile (the kernel's PAD_M)."""
    return _pad(d["vm"], d["bm"] * (4 if d["dt"] == "f32" else 2))


def splittable(d):
    """Instances also compiled with split tiles (split-k): plainly fetched operands, vector loads, double buffer."""
    return d["bsrc"] in ("KC", "NC") and d["vec"] == 1 and d["stages"] == 2 and not d["units"]


def lattice():
    out = []
    # 16-bit inputs, fp32 output: (BM, BN, BK, WM, WN, MB, VM, VN)
    tiles16 = [
        (256, 256, 64, 128, 128, 32, None, None),
        (256, 128, 64, 128, 64, 32, None, None),
        (128, 256, 64, 64, 128, 32, None, None),
        (128, 128, 64, 64, 64, 32, None, None),
        (128, 128, 64, 64, 64, 16, None, None),
        (128, 64, 64, 64, 32, 32, None, None),
        (64, 128, 64, 32, 64, 32, None, None),
        (64, 64, 64, 32, 32, 32, None, None),
        (64, 64, 64, 32, 32, 16, None, None),
        (32, 32, 64, 16, 16, 16, None, None),
        # eight waves per workgroup (two per SIMD)
        (256, 256, 64, 128, 64, 32, None, None),
        (256, 256, 64, 64, 128, 32, None, None),
        (256, 128, 64, 64, 64, 32, None, None),
        (128, 256, 64, 64, 64, 32, None, None),
        # other k depths
        (256, 256, 32, 128, 128, 32, None, None),
        (128, 128, 32, 64, 64, 32, None, None),
        (128, 128, 128, 64, 64, 32, None, None),
    ]
    for dt in ("f16", "bf16"):
        for bsrc in ("KC", "NC", "CONV"):
            for (bm, bn, bk, wm, wn, mb, vm, vn) in tiles16:
                out.append(_inst(dt, "f32", bm, bn, bk, wm, wn, mb, vm, vn, bsrc))
            # scalar-access instance: any alignment, any extents
            out.append(_inst(dt, "f32", 64, 64, 32, 32, 32, 16, None, None, bsrc, vec=0))
        # pointwise convolution with stride 2: the n-contiguous B operand sampled while it is fetched
        for (bm, bn, bk, wm, wn, mb, vm, vn) in tiles16:
            if bm * bn >= 64 * 64 and bk == 64 and mb == 32 and wm * wn < 128 * 128:
                out.append(_inst(dt, "f32", bm, bn, bk, wm, wn, mb, vm, vn, "NCS2"))
        # direct global->LDS staging for k-contiguous operands
        for (bm, bn, bk, wm, wn, mb, vm, vn) in tiles16:
            if bm * bn >= 128 * 128:
                out.append(_inst(dt, "f32", bm, bn, bk, wm, wn, mb, vm, vn, "KC", direct=1))
        # the same for an n-contiguous B (rows of at least 16 chunks: its swizzle needs them)
        for (bm, bn, bk, wm, wn, mb, vm, vn) in tiles16:
            if bm * bn >= 128 * 128 and bn >= 128:
                out.append(_inst(dt, "f32", bm, bn, bk, wm, wn, mb, vm, vn, "NC", direct=1))
        # a ring of three LDS stages (two k tiles in flight) for the mid-size eight-wave tiles; measured to pay
        # for k-contiguous operands only
        for (bm, bn) in ((128, 256), (256, 128)):
            out.append(_inst(dt, "f32", bm, bn, 64, 64, 64, 32, None, None, "KC", stages=3, direct=1))
        # one LDS stage: half the LDS, twice the resident workgroups, for contractions of a single k tile
        for bsrc in ("KC", "NC"):
            for (bm, bn, wm, wn) in ((128, 128, 64, 64), (128, 64, 64, 32)):
                out.append(_inst(dt, "f32", bm, bn, 64, wm, wn, 32, None, None, bsrc, stages=1))
        # 16-bit output variants
        out.append(_inst(dt, dt, 128, 128, 64, 64, 64, 32, None, None, "KC"))
        out.append(_inst(dt, dt, 128, 128, 64, 64, 64, 32, None, None, "NC"))
        out.append(_inst(dt, dt, 256, 256, 64, 128, 64, 32, None, None, "KC", direct=1))
        out.append(_inst(dt, dt, 128, 128, 64, 64, 64, 32, None, None, "KC", direct=1))
        out.append(_inst(dt, dt, 128, 256, 64, 64, 64, 32, None, None, "NC"))
        out.append(_inst(dt, dt, 256, 256, 64, 128, 64, 32, None, None, "NC"))
        out.append(_inst(dt, dt, 256, 256, 64, 128, 64, 32, None, None, "NCS2"))
        out.append(_inst(dt, dt, 64, 64, 32, 32, 32, 16, None, None, "KC", vec=0))
        out.append(_inst(dt, dt, 64, 64, 32, 32, 32, 16, None, None, "NC", vec=0))
        out.append(_inst(dt, dt, 128, 128, 64, 64, 64, 32, None, None, "CONV"))
        out.append(_inst(dt, dt, 64, 64, 32, 32, 32, 16, None, None, "CONV", vec=0))
        # patch-staged convolution: (BM filters, BN pixels, channels per stage, WM, WN, units)
        # two LDS stages (the 64x256 tile of 64x64 wave tiles compiles to one wave per SIMD with two stages
        # and is left out: its single-stage twin below is faster everywhere)
        for (bm, bn, bkc, wm, wn, units) in [(64, 128, 16, 32, 64, 1), (64, 64, 16, 32, 32, 1),
                                             (128, 128, 16, 64, 64, 1), (128, 256, 16, 64, 64, 1), (256, 128, 16, 64, 64, 1),
                                             (32, 256, 16, 32, 64, 1), (128, 128, 16, 64, 64, 2)]:
            out.append(_convp(dt, "f32", bm, bn, bkc, wm, wn, units))
        for (bm, bn, bkc, wm, wn, units) in [(64, 256, 16, 64, 64, 1), (64, 128, 16, 32, 64, 1), (64, 64, 16, 32, 32, 1),
                                             (32, 256, 16, 32, 64, 1), (32, 128, 16, 32, 32, 1), (64, 256, 16, 32, 64, 1),
                                             (64, 256, 16, 64, 64, 2), (128, 128, 16, 64, 64, 1), (128, 256, 16, 64, 64, 1),
                                             (128, 128, 16, 32, 64, 1)]:
            out.append(_convp(dt, "f32", bm, bn, bkc, wm, wn, units, stages=1))
        out.append(_convp(dt, dt, 64, 128, 16, 32, 64, 1))
        out.append(_convp(dt, dt, 64, 256, 16, 64, 64, 1, stages=1))
        out.append(_convp(dt, dt, 128, 256, 16, 64, 64, 1, stages=1))
    for (bm, bn, bkc, wm, wn, units) in [(64, 128, 8, 32, 64, 1), (64, 64, 8, 32, 32, 1), (128, 128, 8, 64, 64, 2)]:
        out.append(_convp("f32", "f32", bm, bn, bkc, wm, wn, units))
    tiles32 = [
        (128, 128, 32, 64, 64, 32, None, None),
        (64, 64, 32, 32, 32, 32, None, None),
        (64, 64, 32, 32, 32, 16, None, None),
        (32, 32, 32, 16, 16, 16, None, None),
        (64, 32, 32, 32, 16, 16, None, None),
    ]
    for (bm, bn, bk, wm, wn, mb, vm, vn) in tiles32[:3:2]:
        out.append(_inst("f32", "f32", bm, bn, bk, wm, wn, mb, vm, vn, "NCS2"))
    for bsrc in ("KC", "NC", "CONV"):
        for (bm, bn, bk, wm, wn, mb, vm, vn) in tiles32:
            out.append(_inst("f32", "f32", bm, bn, bk, wm, wn, mb, vm, vn, bsrc))
        out.append(_inst("f32", "f32", 64, 64, 16, 32, 32, 16, None, None, bsrc, vec=0))
    # 128x128 tiles of eight 64x32 waves (two workgroups, sixteen waves per CU), direct staging: the mid-size
    # shapes whose k loop waits on memory gain 3-6 % from the extra waves (appended last: ids above stay put)
    for dt in ("f16", "bf16"):
        for bsrc in ("KC", "NC"):
            out.append(_inst(dt, "f32", 128, 128, 64, 64, 32, 32, None, None, bsrc, direct=1))
    for dt in ("f16", "bf16"):
        for bsrc in ("KC", "NC"):
            out.append(_inst(dt, dt, 128, 128, 64, 64, 32, 32, None, None, bsrc, direct=1))
    # shallower virtual-thread interleaves of the tiles the benchmark shapes end in (fp16): what the walk can
    # reach when setVThread stops early, and all it can reach without setVThread (V = 1: the plain LDS layout)
    for bsrc in ("KC", "NC"):
        for (bm, bn, wm, wn) in ((256, 256, 128, 128), (256, 256, 128, 64), (128, 256, 64, 64), (256, 128, 64, 64),
                                 (128, 128, 64, 64), (128, 128, 64, 32)):
            for v in ((1, 2, 4) if (bm, bn, wm, wn) in ((256, 256, 128, 128), (128, 256, 64, 64), (128, 128, 64, 32)) else (1,)):
                out.append(_inst("f16", "f32", bm, bn, 64, wm, wn, 32, v, min(v, full_v("f16", 64, bsrc)[1]), bsrc, direct=1))
    for bsrc in ("KC", "NC"):
        out.append(_inst("f16", "f32", 128, 128, 64, 64, 64, 32, 1, 1, bsrc))
        out.append(_inst("f32", "f32", 64, 64, 32, 32, 32, 32, 1, 1, bsrc))
        out.append(_inst("f32", "f32", 32, 32, 32, 16, 16, 16, 1, 1, bsrc))
    out.append(_inst("f16", "f32", 256, 256, 64, 128, 64, 32, 1, 1, "NCS2"))
    out.append(_inst("f16", "f32", 128, 128, 64, 64, 64, 32, 1, 1, "CONV"))
    # A stored [k][m] (transA): register-staged instances, both B layouts
    for bsrc in ("KC", "NC"):
        for dt in ("f16", "bf16"):
            for (bm, bn, wm, wn, mb) in ((256, 256, 128, 64, 32), (256, 128, 64, 64, 32), (128, 256, 64, 64, 32), (128, 128, 64, 64, 32),
                                         (128, 128, 64, 64, 16), (64, 64, 32, 32, 32), (32, 32, 16, 16, 16)):
                out.append(_inst(dt, "f32", bm, bn, 64, wm, wn, mb, bsrc=bsrc, asrc="MC"))
            out.append(_inst(dt, "f32", 128, 128, 32, 64, 64, 32, bsrc=bsrc, asrc="MC"))
            out.append(_inst(dt, "f32", 128, 128, 64, 64, 64, 32, 1, 1, bsrc=bsrc, asrc="MC"))
            out.append(_inst(dt, "f32", 64, 64, 32, 32, 32, 16, bsrc=bsrc, vec=0, asrc="MC"))
            out.append(_inst(dt, dt, 128, 128, 64, 64, 64, 32, bsrc=bsrc, asrc="MC"))
            out.append(_inst(dt, dt, 64, 64, 32, 32, 32, 16, bsrc=bsrc, vec=0, asrc="MC"))
        for (bm, bn, wm, wn, mb) in ((128, 128, 64, 64, 32), (64, 64, 32, 32, 32), (64, 64, 32, 32, 16), (32, 32, 16, 16, 16)):
            out.append(_inst("f32", "f32", bm, bn, 32, wm, wn, mb, bsrc=bsrc, asrc="MC"))
        out.append(_inst("f32", "f32", 64, 64, 32, 32, 32, 32, 1, 1, bsrc=bsrc, asrc="MC"))
        out.append(_inst("f32", "f32", 64, 64, 16, 32, 32, 16, bsrc=bsrc, vec=0, asrc="MC"))
    # three-stage rings for an n-contiguous B (the mid-size eight-wave tiles), like the k-contiguous ones above
    for dt in ("f16", "bf16"):
        for (bm, bn) in ((128, 256), (256, 128)):
            out.append(_inst(dt, "f32", bm, bn, 64, 64, 64, 32, bsrc="NC", stages=3, direct=1))
    for i, d in enumerate(out):
        d["id"] = i
    keys = [(d["dt"], d["out"], d["bm"], d["bn"], d["bk"], d["wm"], d["wn"], d["mb"], d["vm"], d["vn"], d["bsrc"], d["vec"],
             d["stages"], d["direct"], d["units"], d["asrc"]) for d in out]
    assert len(set(keys)) == len(keys), "duplicate instance"
    return out


def cfg_type(d):
    if d["units"]:
        return "ConvCfg<%s, %s, %d, %d, %d, %d, %d, %d, %d, %d>" % (
            CT[d["dt"]], CT[d["out"]], d["bm"], d["bn"], d["bk"], d["wm"], d["wn"], d["mb"], d["units"], d["stages"])
    return ("Cfg<%s, %s, %d, %d, %d, %d, %d, %d, %d, %d, %d, %s, %d, %s, %d>" % (
        CT[d["dt"]], CT[d["out"]], d["bm"], d["bn"], d["bk"], d["wm"], d["wn"], d["mb"], d["vm"], d["vn"],
        BSRC[d["bsrc"]], "true" if d["vec"] else "false", d["stages"], "true" if d["direct"] else "false", ASRC[d["asrc"]]))


if __name__ == "__main__":
    L = lattice()
    print(len(L), "instances")
