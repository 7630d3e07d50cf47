"""GPU parity: the HIP kernels, called through the C ABI, against the CPU oracle.

Integer-valued inputs make every partial sum exact in fp32, so any summation order must
agree with the oracle bit for bit; real-valued inputs are held to the stated tolerances
(relative Frobenius error <= 1e-5 for fp32, <= 2e-3 for fp16/bf16 inputs with fp32 accumulate).
"""
import numpy as np
import pytest

from oracle import ops
from paper_2502_11407_amd import inputs

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}
DT_NAME = {0: "f32", 1: "f16", 2: "bf16"}


@pytest.fixture(scope="module")
def gs():
    from paper_2502_11407_amd import binding
    return binding


def _round_up(x, m):
    return (x + m - 1) // m * m


def run_gemm(gs, dtype, M, N, K, transB, sched, A, B, alpha=1.0, beta=0.0, C0=None, batch=1, out_dtype="f32", transA=0):
    import torch
    p = gs.gemm_problem(dtype, M, N, K, transA, transB, batch, out_dtype)
    dA, dB = gs.to_device(A, dtype), gs.to_device(B, dtype)
    shape = (batch, M, N) if batch > 1 else (M, N)
    if C0 is None:
        dC = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")   # beta = 0 must not read it
        if out_dtype != "f32":
            dC = dC.to({"f16": torch.float16, "bf16": torch.bfloat16}[out_dtype])
    else:
        dC = gs.to_device(C0, out_dtype)
    if batch > 1:
        gs.bmm(p, dA, dB, dC, alpha, beta, sched)
    else:
        gs.gemm(p, dA, dB, dC, alpha, beta, sched)
    torch.cuda.synchronize()
    return gs.to_host_f64(dC)


def instance_cases(gs):
    """(instance id, dtype, bsrc, vec, direct, bm, bn, bk) for every compiled instance."""
    out = []
    for idx in range(gs.num_instances()):
        for dt in ("f32", "f16", "bf16"):
            for out_dt in sorted({"f32", dt}):
                for tb, op in ((1, "gemm"), (0, "gemm"), (1, "gemm_ta"), (0, "gemm_ta"), (0, "conv"), (0, "conv1x1"), (0, "conv_pw2")):
                    if op == "conv1x1" and out and out[-1][0] == idx:
                        continue                      # already covered with 3x3 filters
                    if op == "conv_pw2":              # pointwise, stride 2: the sampling B source
                        p = gs.conv_problem(dt, 1, 8, 8, 16, 8, 1, 1, 2, 0, out_dt)
                    elif op.startswith("conv"):
                        p = gs.conv_problem(dt, 1, 8, 8, 8, 8, 3 if op == "conv" else 1, 3 if op == "conv" else 1, 1, 1, out_dt)
                    else:
                        p = gs.gemm_problem(dt, 64, 64, 64, 1 if op == "gemm_ta" else 0, tb, 1, out_dt)
                    s = gs.instance_schedule(idx, p)
                    if s is not None:
                        out.append((idx, dt, out_dt, op, tb, s))
    return out


def test_every_instance_bit_exact_on_integers(gs):
    """Each compiled instance on a problem with several tiles and ragged tails in m, n and k."""
    cases = instance_cases(gs)
    assert len(cases) == gs.num_instances()
    for (idx, dt, out_dt, op, tb, s) in cases:
        bm, bn, bk = s.tile[0][0], s.tile[1][0], s.tile[2][0]
        epc = 4 if dt == "f32" else 8
        vec = s.vec_bytes == 16
        print(f"instance {idx} {dt}->{out_dt} {op} transB={tb} tile {bm}x{bn}x{bk} vec={vec} direct={s.direct_lds}", flush=True)
        lim = 1 if out_dt == "bf16" else 4      # keep results exactly representable in the output type
        if op in ("gemm", "gemm_ta"):
            ta = 1 if op == "gemm_ta" else 0
            M = bm + (17 if not (ta and vec) else 16)          # an m-contiguous A read in vectors needs M in whole vectors
            N = bn + (8 if vec else 9)
            K = 2 * bk + (0 if s.direct_lds else (epc if vec else 5))
            A = inputs.small_ints(100 + idx, (K, M) if ta else (M, K), dt, -lim, lim)
            B = inputs.small_ints(200 + idx, (N, K) if tb else (K, N), dt, -lim, lim)
            want = ops.gemm(A, B, dt, transA=ta, transB=tb)
            got = run_gemm(gs, dt, M, N, K, tb, s, A, B, out_dtype=out_dt, transA=ta)
        else:
            import torch
            c, r = (8, 3) if vec else (5, 3)        # K = c*r*r: 72 (whole chunks) or 45
            if op == "conv1x1":
                c, r = 24, 1
            k = bm + 5
            n, h, w = 2, 9, max(7, bn // 8)
            stride, pad = 1, 1
            if op == "conv_pw2":                    # P = 9, Q = bn/8: P*Q spans a tile and a ragged tail
                c, r, stride, pad = 24, 1, 2, 0
                h, w = 17, 2 * max(8, bn // 8)
            I = inputs.small_ints(300 + idx, (n, c, h, w), dt, -min(lim, 2), min(lim, 2))
            W = inputs.small_ints(400 + idx, (k, c, r, r), dt, -min(lim, 2), min(lim, 2))
            want = ops.conv2d(I, W, dt, stride=stride, pad=pad)
            p = gs.conv_problem(dt, n, c, h, w, k, r, r, stride, pad, out_dt)
            dO = gs.empty_device(want.shape, out_dt)
            dO.fill_(float("nan"))
            gs.conv2d(p, gs.to_device(I, dt), gs.to_device(W, dt), dO, s, gs.conv_workspace(p, s))
            torch.cuda.synchronize()
            got = gs.to_host_f64(dO)
        assert np.abs(want).max() < (256 if out_dt == "bf16" else 2048)
        assert np.array_equal(got, want), f"instance {idx}: max abs diff {np.abs(got - want).max()}"


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("transB", [0, 1])
def test_gemm_real_values_default_schedule(gs, dtype, transB):
    M, N, K = 300, 264, 520
    A = inputs.uniform_pm1(1, (M, K), dtype)
    B = inputs.uniform_pm1(2, (N, K) if transB else (K, N), dtype)
    want = ops.gemm(A, B, dtype, transB=transB)
    got = run_gemm(gs, dtype, M, N, K, transB, None, A, B)
    err = ops.rel_frobenius(got, want)
    print(dtype, transB, "rel frobenius", err)
    assert err <= TOL[dtype]
    assert err <= 1e-5      # rounding alone is ~1e-7..1e-6 (see the CPU error-bound test)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_gemm_alpha_beta_and_unaligned_shapes(gs, dtype):
    M, N, K = 77, 53, 41        # nothing is a multiple of a chunk: scalar path
    A = inputs.small_ints(3, (M, K), dtype)
    B = inputs.small_ints(4, (K, N), dtype)
    C0 = inputs.small_ints(5, (M, N), "f32")
    want = ops.gemm(A, B, dtype, alpha=2.0, beta=-3.0, C0=C0)
    got = run_gemm(gs, dtype, M, N, K, 0, None, A, B, alpha=2.0, beta=-3.0, C0=C0)
    assert np.array_equal(got, want)
    got1 = run_gemm(gs, dtype, M, N, K, 0, None, A, B, alpha=0.0, beta=1.0, C0=C0)
    assert np.array_equal(got1, C0)


def test_gemm_degenerate_extents(gs):
    for (M, N, K) in [(1, 1, 1), (1, 300, 7), (300, 1, 8), (5, 5, 1024), (130, 2, 3)]:
        A = inputs.small_ints(6, (M, K), "f16")
        B = inputs.small_ints(7, (N, K), "f16")
        assert np.array_equal(run_gemm(gs, "f16", M, N, K, 1, None, A, B), ops.gemm(A, B, "f16", transB=1)), (M, N, K)


def test_bmm_strided_batches(gs):
    w = inputs.config4_bmm_scores(batch=5, seq=200, head=64)
    want = ops.bmm(w.A, w.B, "f16", transB=1, alpha=0.125)
    got = run_gemm(gs, "f16", 200, 200, 64, 1, None, w.A, w.B, alpha=0.125, batch=5)
    assert ops.rel_frobenius(got, want) <= 1e-5
    wt = inputs.config4_bmm_scores(batch=5, seq=200, head=64, materialised_kt=True)
    got2 = run_gemm(gs, "f16", 200, 200, 64, 0, None, wt.A, wt.B, alpha=0.125, batch=5)
    assert ops.rel_frobenius(got2, want) <= 1e-5


@pytest.mark.parametrize("which,n,hw", [("3x3", 2, 20), ("1x1s2", 2, 14)])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_conv_real_values(gs, which, n, hw, dtype):
    import torch
    w = inputs.config5_conv(which, n=n, dtype=dtype, hw=hw)
    want = ops.conv2d(w.I, w.W, dtype, stride=w.stride, pad=w.pad)
    p = gs.conv_problem(dtype, w.n, w.c, w.h, w.w, w.k, w.r, w.s, w.stride, w.pad)
    dO = gs.empty_device(want.shape)
    dO.fill_(float("nan"))
    gs.conv2d(p, gs.to_device(w.I, dtype), gs.to_device(w.W, dtype), dO, None, gs.conv_workspace(p))
    torch.cuda.synchronize()
    err = ops.rel_frobenius(gs.to_host_f64(dO), want)
    print(which, dtype, "rel frobenius", err)
    assert err <= min(TOL[dtype], 1e-5)


@pytest.mark.parametrize("stride,pad,r,s", [(1, 0, 3, 3), (2, 1, 3, 3), (2, 2, 5, 3), (3, 0, 1, 1), (1, 2, 1, 5)])
def test_conv_geometry_bit_exact(gs, stride, pad, r, s):
    import torch
    n, c, h, w, k = 3, 6, 13, 11, 10
    I = inputs.small_ints(8, (n, c, h, w), "f16", -2, 2)
    W = inputs.small_ints(9, (k, c, r, s), "f16", -2, 2)
    want = ops.conv2d(I, W, "f16", stride=stride, pad=pad)
    p = gs.conv_problem("f16", n, c, h, w, k, r, s, stride, pad)
    dO = gs.empty_device(want.shape)
    gs.conv2d(p, gs.to_device(I, "f16"), gs.to_device(W, "f16"), dO, None, gs.conv_workspace(p))
    torch.cuda.synchronize()
    assert np.array_equal(gs.to_host_f64(dO), want)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("geom", [
    # n, c, h, w, k, r, s, stride, pad
    (3, 24, 13, 11, 70, 3, 3, 1, 1),     # channel tail (24 = 16 + 8), W not a multiple of 8, tiles span images
    (2, 16, 9, 20, 33, 3, 3, 2, 1),      # stride 2
    (2, 40, 12, 12, 64, 1, 1, 2, 1),     # 1x1 stride 2 (with padding: without it the problem is a batched GEMM)
    (1, 8, 7, 30, 16, 1, 3, 1, 2),       # 1x3 filter, padding wider than the filter needs
    (4, 32, 6, 6, 130, 3, 3, 1, 0),      # valid convolution, tiny images: a tile covers several images
    (2, 16, 16, 16, 64, 2, 2, 1, 1),     # even filter
])
def test_conv_patch_instances_bit_exact(gs, dtype, geom):
    """Every patch-staged convolution instance that can run the geometry, bit-exact on integers."""
    import torch
    n, c, h, w, k, r, s, stride, pad = geom
    I = inputs.small_ints(11, (n, c, h, w), dtype, -2, 2)
    W = inputs.small_ints(12, (k, c, r, s), dtype, -2, 2)
    want = ops.conv2d(I, W, dtype, stride=stride, pad=pad)
    p = gs.conv_problem(dtype, n, c, h, w, k, r, s, stride, pad)
    dI, dW = gs.to_device(I, dtype), gs.to_device(W, dtype)
    ran = 0
    for idx in range(gs.num_instances()):
        sch = gs.instance_schedule(idx, p)
        if sch is None or not sch.direct_lds:
            continue
        print(f"conv patch instance {idx} tile {sch.tile[0][0]}x{sch.tile[1][0]}x{sch.tile[2][0]} geom {geom} {dtype}", flush=True)
        dO = gs.empty_device(want.shape)
        dO.fill_(float("nan"))
        gs.conv2d(p, dI, dW, dO, sch, gs.conv_workspace(p, sch))
        torch.cuda.synchronize()
        got = gs.to_host_f64(dO)
        assert np.array_equal(got, want), f"instance {idx}: max abs diff {np.nanmax(np.abs(got - want))}"
        ran += 1
    assert ran >= 2


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("geom", [
    # n, c, h, w, k, stride
    (3, 40, 12, 16, 70, 1),      # the input itself is the B operand (ldb = H*W)
    (3, 40, 12, 16, 70, 2),      # stride 2, rows of whole vectors: sampled while fetched, no workspace; P*Q = 48
    (2, 16, 16, 40, 300, 2),     # the same over several m and n tiles with ragged edges; P*Q = 160
    (2, 24, 13, 11, 33, 3),      # compacted through the workspace; P*Q = 20: scalar instances only
    (2, 16, 31, 31, 16, 2),      # compacted through the workspace; P*Q = 256, several n tiles
    (2, 8, 9, 24, 20, 2),        # could be sampled, but P*Q = 60 is no whole number of fp16 vectors: compacted
])
def test_pointwise_conv_is_a_batched_gemm(gs, dtype, geom):
    """1x1 filter, no padding: every n-contiguous-B GEMM instance that serves the per-image view,
    bit-exact on integers; then the default schedule with and without the workspace."""
    import torch
    n, c, h, w, k, stride = geom
    I = inputs.small_ints(21, (n, c, h, w), dtype, -2, 2)
    W = inputs.small_ints(22, (k, c, 1, 1), dtype, -2, 2)
    want = ops.conv2d(I, W, dtype, stride=stride, pad=0)
    p = gs.conv_problem(dtype, n, c, h, w, k, 1, 1, stride, 0)
    dI, dW = gs.to_device(I, dtype), gs.to_device(W, dtype)
    pq = want.shape[2] * want.shape[3]
    esize = 4 if dtype == "f32" else 2
    sampled = stride == 2 and w % (16 // esize) == 0          # instance_schedule then offers the sampling instances
    need = 0 if (stride == 1 or sampled) else n * c * pq * esize
    assert gs.workspace_bytes(p) >= need
    ran = 0
    for idx in range(gs.num_instances()):
        sch = gs.instance_schedule(idx, p)
        if sch is None or (sch.vec_bytes == 16 and pq % (16 // esize)):
            continue
        if sch.direct_lds and c % sch.tile[2][0]:
            continue                                            # direct staging takes whole k tiles only
        assert gs.workspace_bytes(p, sch) == need
        print(f"pointwise conv instance {idx} tile {sch.tile[0][0]}x{sch.tile[1][0]}x{sch.tile[2][0]} geom {geom} {dtype}", flush=True)
        dO = gs.empty_device(want.shape)
        dO.fill_(float("nan"))
        gs.conv2d(p, dI, dW, dO, sch, gs.conv_workspace(p, sch))
        torch.cuda.synchronize()
        got = gs.to_host_f64(dO)
        assert np.array_equal(got, want), f"instance {idx}: max abs diff {np.nanmax(np.abs(got - want))}"
        if need:
            with pytest.raises(gs.GensorError) as e:
                gs.conv2d(p, dI, dW, dO, sch)               # the schedule needs the compacted input
            assert e.value.status == 4
        ran += 1
    assert ran >= (2 if pq % (16 // esize) == 0 else (0 if sampled else 1))
    for ws in (gs.conv_workspace(p), None):                  # None: strided input falls back to the general view
        dO = gs.empty_device(want.shape)
        dO.fill_(float("nan"))
        gs.conv2d(p, dI, dW, dO, None, ws)
        torch.cuda.synchronize()
        assert np.array_equal(gs.to_host_f64(dO), want)


def test_conv_needs_no_workspace(gs):
    """Patch-staged and gather schedules run without any workspace (filters are reordered inside the
    kernel); only a pointwise convolution through the compaction pre-pass asks for one."""
    import torch
    n, c, h, w, k = 2, 16, 12, 12, 32
    I = inputs.small_ints(13, (n, c, h, w), "f16", -2, 2)
    W = inputs.small_ints(14, (k, c, 3, 3), "f16", -2, 2)
    want = ops.conv2d(I, W, "f16", stride=1, pad=1)
    p = gs.conv_problem("f16", n, c, h, w, k, 3, 3, 1, 1)
    dI, dW = gs.to_device(I, "f16"), gs.to_device(W, "f16")
    assert gs.workspace_bytes(p) == 0
    patch = [s for s in (gs.instance_schedule(i, p) for i in range(gs.num_instances())) if s is not None and s.direct_lds]
    assert patch and gs.workspace_bytes(p, patch[0]) == 0
    for sch in (patch[0], None):
        dO = gs.empty_device(want.shape)
        dO.fill_(float("nan"))
        gs.conv2d(p, dI, dW, dO, sch)
        torch.cuda.synchronize()
        assert np.array_equal(gs.to_host_f64(dO), want)
    pw = gs.conv_problem("f16", n, c, h, w, k, 1, 1, 3, 0)
    assert gs.workspace_bytes(pw) == n * c * 4 * 4 * 2


def test_error_paths_launch_nothing(gs):
    import torch
    p = gs.gemm_problem("f16", 64, 64, 64, 0, 1)
    A = torch.zeros((64, 64), dtype=torch.float16, device="cuda")
    Cc = torch.zeros((64, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(gs.GensorError) as e:
        gs.gemm(p, A, A, Cc, lda=32)           # leading dimension smaller than the row
    assert e.value.status == 1
    bad = gs.gemm_problem("f16", 0, 64, 64, 0, 1)
    with pytest.raises(gs.GensorError) as e:
        gs.gemm(bad, A, A, Cc)
    assert e.value.status == 1
    pt = gs.gemm_problem("f16", 64, 64, 64, 0, 1, 1, "bf16")     # output neither fp32 nor the input type: no kernel
    with pytest.raises(gs.GensorError) as e:
        gs.gemm(pt, A, A, Cc)
    assert e.value.status == 2
    s = gs.instance_schedule(0, p)
    s.tile[0][0] = 48                                  # not a lattice point
    s.kernel_id = -1
    with pytest.raises(gs.GensorError) as e:
        gs.gemm(p, A, A, Cc, schedule=s)
    assert e.value.status == 3


# ------------------------------------------------------------------ full benchmark sizes
def _full_size_case(gs, name):
    """The benchmark workload `name` (or a workload object) with the schedule bench.py would time
    (gensor_construct, seed 0)."""
    import torch
    w = inputs.all_configs()[name] if isinstance(name, str) else name
    if isinstance(w, inputs.GemmWorkload):
        p = gs.gemm_problem(w.dtype, w.M, w.N, w.K, w.transA, w.transB, w.batch)
        s = gs.construct(p, seed=0)
        out = gs.empty_device((w.batch, w.M, w.N) if w.batch > 1 else (w.M, w.N))
        out.fill_(float("nan"))
        dA, dB = gs.to_device(w.A, w.dtype), gs.to_device(w.B, w.dtype)
        (gs.bmm if w.batch > 1 else gs.gemm)(p, dA, dB, out, 1.0, 0.0, s, workspace=gs.gemm_workspace(p, s))
        torch.cuda.synchronize()
        co = inputs.sample_indices(21, (w.batch, w.M, w.N), 1500)
        # whole first / last rows and columns as well: tile edges and the ragged last tile
        edge = [(b, i, j) for b in (0, w.batch - 1) for i in (0, w.M - 1) for j in range(0, w.N, max(1, w.N // 97))]
        edge += [(b, i, j) for b in (0, w.batch - 1) for j in (0, w.N - 1) for i in range(0, w.M, max(1, w.M // 97))]
        co = np.concatenate([co, np.array(edge, dtype=np.int64)])
        want = ops.bmm_at(w.A, w.B, w.dtype, co, transA=w.transA, transB=w.transB)
        o3 = out if w.batch > 1 else out[None]
        idx = torch.from_numpy(co).cuda()
        got = o3[idx[:, 0], idx[:, 1], idx[:, 2]].double().cpu().numpy()
        finite = bool(torch.isfinite(out).all())
    else:
        p = gs.conv_problem(w.dtype, w.n, w.c, w.h, w.w, w.k, w.r, w.s, w.stride, w.pad)
        s = gs.construct(p, seed=0)
        out = gs.empty_device((w.n, w.k, w.p, w.q))
        out.fill_(float("nan"))
        gs.conv2d(p, gs.to_device(w.I, w.dtype), gs.to_device(w.W, w.dtype), out, s, gs.conv_workspace(p, s))
        torch.cuda.synchronize()
        co = inputs.sample_indices(22, (w.n, w.k, w.p, w.q), 1500)
        edge = [(n, k, p_, q_) for n in (0, w.n - 1) for k in (0, w.k - 1) for p_ in (0, w.p - 1) for q_ in range(w.q)]
        edge += [(n, k, p_, q_) for n in (0, w.n - 1) for k in (0, w.k - 1) for q_ in (0, w.q - 1) for p_ in range(w.p)]
        co = np.concatenate([co, np.array(edge, dtype=np.int64)])
        want = ops.conv2d_at(w.I, w.W, w.dtype, co, stride=w.stride, pad=w.pad)
        idx = torch.from_numpy(co).cuda()
        got = out[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].double().cpu().numpy()
        finite = bool(torch.isfinite(out).all())
    return w, s, got, want, finite


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3_up", "cfg3_down", "cfg4", "cfg5_3x3", "cfg5_1x1s2"])
def test_benchmark_shapes_full_size_sampled(gs, name):
    """All five benchmark configurations at full size with the constructed schedule: sampled
    entries plus tile-edge rows and columns against the oracle, every output finite (no entry
    left unwritten), and the per-entry error within the fp32-accumulation bound."""
    w, s, got, want, finite = _full_size_case(gs, name)
    err = ops.rel_frobenius(got, want)
    print(name, "kernel", s.kernel_id, "rel frobenius on samples", err)
    assert finite
    assert err <= TOL[w.dtype]
    assert err <= 2e-6
    scale = np.abs(want).max()
    assert np.abs(got - want).max() <= 1e-4 * scale


@pytest.mark.parametrize("index", range(len(inputs.UNBALANCED_GEMMS)))
def test_unbalanced_gemm_shapes_full_size_sampled(gs, index):
    """The paper's GEMM shapes with unbalanced dimensions (K = 4 ... 8192) at full size with the
    constructed schedule: sampled entries and tile edges against the oracle, nothing left unwritten."""
    w, s, got, want, finite = _full_size_case(gs, inputs.unbalanced_gemm(index))
    err = ops.rel_frobenius(got, want)
    print(w.name, "kernel", s.kernel_id, "rel frobenius on samples", err)
    assert finite
    assert err <= 1e-5          # fp32 accumulation of up to 8192 exact products; the stated bound is 2e-3


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_mfma_probe_counts_its_flops(gs, dtype):
    """The measurement aid really executes iters x 8 MFMAs per wavefront: with all-ones operands every
    accumulator element ends at 16 * iters, so a lane's sum over its 8 x 16 values is 2048 * iters."""
    import torch
    from paper_2502_11407_amd import probe
    ones = inputs.to_storage(np.ones(128 * 1024, dtype=np.float32), dtype)
    sink = torch.zeros(256 * 256, dtype=torch.float32, device="cuda")
    probe.mfma_probe(dtype, gs.to_device(ones, dtype), sink, 10, 256)
    torch.cuda.synchronize()
    assert torch.all(sink == 2048.0 * 10).item()
    with pytest.raises(gs.GensorError):
        probe.mfma_probe("f32", gs.to_device(np.ones(64 * 1024, dtype=np.float32), "f32"), sink, 10, 256)


# ------------------------------------------------------------------ GEMV and AvgPooling2d
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("M,N", [(1, 1), (7, 5), (8, 64), (37, 1000), (130, 520), (9, 20011), (16, 32768 + 8)])
def test_gemv_bit_exact_on_integers(gs, dtype, M, N):
    """Several workgroups, rows that are no multiple of 8, ragged vector tails, x longer than one LDS panel."""
    import torch
    A = inputs.small_ints(41, (M, N), dtype, -2, 2)
    x = inputs.small_ints(42, (N,), dtype, -2, 2)
    y0 = inputs.small_ints(43, (M,), "f32", -4, 4)
    dA, dx = gs.to_device(A, dtype), gs.to_device(x, dtype)
    y = torch.full((M,), float("nan"), dtype=torch.float32, device="cuda")          # beta = 0 must not read it
    gs.gemv(dtype, dA, dx, y)
    torch.cuda.synchronize()
    assert np.array_equal(gs.to_host_f64(y), ops.gemv(A, x, dtype))
    y = gs.to_device(y0, "f32")
    gs.gemv(dtype, dA, dx, y, alpha=2.0, beta=-3.0)
    torch.cuda.synchronize()
    assert np.array_equal(gs.to_host_f64(y), ops.gemv(A, x, dtype, alpha=2.0, beta=-3.0, y0=y0))


def test_gemv_unaligned_operands_and_errors(gs):
    """A view with an odd leading dimension and an offset start takes the element-load kernel."""
    import torch
    A = inputs.small_ints(44, (33, 77), "f16", -2, 2)
    x = inputs.small_ints(45, (77,), "f16", -2, 2)
    dA, dx = gs.to_device(A, "f16"), gs.to_device(np.concatenate([x[:1], x]), "f16")[1:]
    sub = dA[:, 3:70]                                        # lda = 77, start 6 bytes into a row
    y = torch.zeros(33, dtype=torch.float32, device="cuda")
    gs.gemv("f16", sub, dx[3:70], y)
    torch.cuda.synchronize()
    assert np.array_equal(gs.to_host_f64(y), ops.gemv(np.ascontiguousarray(A[:, 3:70]), x[3:70], "f16"))
    with pytest.raises(gs.GensorError) as e:
        gs.gemv("f16", dA, dx, y, lda=10)                    # lda < N
    assert e.value.status == 1


@pytest.mark.parametrize("index", range(3))
def test_gemv_paper_shapes_full_size(gs, index):
    import torch
    A, x = inputs.gemv_workload(index)
    y = torch.full((A.shape[0],), float("nan"), dtype=torch.float32, device="cuda")
    gs.gemv("f16", gs.to_device(A, "f16"), gs.to_device(x, "f16"), y)
    torch.cuda.synchronize()
    rows = inputs.sample_indices(46, (A.shape[0],), 400)[:, 0]
    want = ops.gemv(np.ascontiguousarray(A[rows]), x, "f16")
    got = gs.to_host_f64(y)
    err = ops.rel_frobenius(got[rows], want)
    print("gemv", A.shape, "rel frobenius on sampled rows", err)
    assert np.isfinite(got).all() and err <= 1e-5


@pytest.mark.parametrize("dtype,out_dtype", [("f32", "f32"), ("f16", "f32"), ("bf16", "f32"), ("f16", "f16")])
@pytest.mark.parametrize("n,c,h,w,f,stride", [(2, 3, 8, 10, 2, 2), (1, 5, 9, 7, 3, 2), (3, 2, 7, 9, 2, 2), (2, 2, 6, 6, 3, 1),
                                              (1, 1, 5, 300, 4, 4), (2, 4, 17, 33, 1, 1),
                                              (3, 37, 21, 21, 3, 2),        # many small planes per workgroup, ragged last group
                                              (1, 2, 150, 131, 2, 2),       # a plane larger than the LDS span: runs of output rows
                                              (1, 1, 3, 20000, 2, 1)])      # rows too long for the span: direct kernel
def test_avgpool_small_cases(gs, dtype, out_dtype, n, c, h, w, f, stride):
    """Window sums of small integers are exact in fp32; dividing by a power of two keeps them exact, so F in
    {1, 2, 4} must agree bit for bit; F = 3 divides by 9 and is held to one fp32 rounding."""
    import torch
    I = inputs.small_ints(47, (n, c, h, w), dtype, -8, 8)
    want = ops.avgpool2d(I, dtype, f, stride)
    O = gs.empty_device(want.shape, out_dtype)
    O.fill_(float("nan"))
    gs.avgpool2d(dtype, gs.to_device(I, dtype), O, f, stride, out_dtype)
    torch.cuda.synchronize()
    got = gs.to_host_f64(O)
    if out_dtype == "f32" and dtype == "f16":                # an input that does not start on a 16-byte boundary
        shifted = gs.to_device(np.concatenate([I.reshape(-1)[:1], I.reshape(-1)]), dtype)[1:].view(n, c, h, w)
        O2 = gs.empty_device(want.shape, out_dtype)
        gs.avgpool2d(dtype, shifted, O2, f, stride, out_dtype)
        torch.cuda.synchronize()
        assert np.array_equal(gs.to_host_f64(O2), got)
    if f in (1, 2, 4) and out_dtype == "f32":
        assert np.array_equal(got, want)
    else:
        tol = 2.0 ** -24 if out_dtype == "f32" else 2.0 ** -11
        assert np.abs(got - want).max() <= tol * max(1.0, np.abs(want).max())


@pytest.mark.parametrize("index", range(3))
def test_avgpool_paper_shapes_full_size(gs, index):
    import torch
    I, f, stride = inputs.pool_workload(index)
    shape = ops.pool_out_shape(*I.shape, f, stride)
    O = gs.empty_device(shape)
    O.fill_(float("nan"))
    gs.avgpool2d("f16", gs.to_device(I, "f16"), O, f, stride)
    torch.cuda.synchronize()
    co = inputs.sample_indices(48, shape, 3000)
    want = ops.avgpool2d_at(I, "f16", co, f, stride)
    idx = torch.from_numpy(co).cuda()
    got = O[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].double().cpu().numpy()
    err = ops.rel_frobenius(got, want)
    print("avgpool", I.shape, f, stride, "rel frobenius on samples", err)
    assert bool(torch.isfinite(O).all()) and err <= 1e-6


@pytest.mark.parametrize("index", range(3))
def test_paper_conv_shapes_full_size(gs, index):
    """Conv2d shapes C1-C3 of the operator table with the constructed schedule."""
    w, s, got, want, finite = _full_size_case(gs, inputs.paper_conv(index))
    err = ops.rel_frobenius(got, want)
    print(w.name, "kernel", s.kernel_id, "rel frobenius on samples", err)
    assert finite and err <= 1e-5


def test_shape_changes_reconstruct_within_a_latency_budget(gs):
    """Dynamic shapes: a call without a schedule constructs one for a shape it has not seen (a few
    milliseconds on the host) and reuses it afterwards; results stay exact across the shape changes."""
    import time
    import torch
    first, again = [], []
    for i, (M, N, K) in enumerate([(96 + 32 * j, 200 + 8 * j, 64 * (1 + j % 3)) for j in range(12)]):
        A = inputs.small_ints(60 + i, (M, K), "f16", -2, 2)
        B = inputs.small_ints(80 + i, (K, N), "f16", -2, 2)
        p = gs.gemm_problem("f16", M, N, K, 0, 0)
        dA, dB = gs.to_device(A, "f16"), gs.to_device(B, "f16")
        dC = gs.empty_device((M, N))
        torch.cuda.synchronize()
        for bucket in (first, again):
            t0 = time.perf_counter()
            gs.gemm(p, dA, dB, dC, 1.0, 0.0, None)
            torch.cuda.synchronize()
            bucket.append(time.perf_counter() - t0)
        assert np.array_equal(gs.to_host_f64(dC), ops.gemm(A, B, "f16"))
    print("first call per new shape: max %.1f ms, repeated: max %.2f ms" % (1e3 * max(first[1:]), 1e3 * max(again)))
    assert max(first[1:]) < 0.25            # construction plus launch (the very first call also loads the code object)
    assert max(again) < max(0.05, max(first[1:]))


@pytest.mark.gpu
@pytest.mark.parametrize("k_tiles", [1, 2, 3, 4, 7])
def test_multi_tile_schedules_across_k_depths(gs, k_tiles):
    """Instances whose loop looks further ahead than one k tile or one k step (rings of three LDS stages; the
    one-wave-per-SIMD tiles that read fragments two k steps ahead and fetch two tiles ahead): fewer k tiles than
    the look-ahead (everything happens in the prologue and the peeled tiles), exactly as many, and enough for
    the steady-state body, each with ragged m and n, bit-exact on integers."""
    ran = 0
    for idx in range(gs.num_instances()):
        for dt in ("f16", "bf16"):
            for tb in (1, 0):
                p0 = gs.gemm_problem(dt, 64, 64, 64, 0, tb, 1, "f32")
                s = gs.instance_schedule(idx, p0)
                if s is None:
                    continue
                deep = s.direct_lds and s.tile[0][1] * s.tile[1][1] >= 128 * 128
                if s.stages <= 2 and not deep:
                    continue
                bm, bn, bk = s.tile[0][0], s.tile[1][0], s.tile[2][0]
                M, N, K = 2 * bm + 17, bn + 8, k_tiles * bk
                print(f"instance {idx} {dt} transB={tb} stages {s.stages} tile {bm}x{bn}x{bk} K={K}", flush=True)
                A = inputs.small_ints(500 + idx, (M, K), dt, -2, 2)
                B = inputs.small_ints(600 + idx, (N, K) if tb else (K, N), dt, -2, 2)
                want = ops.gemm(A, B, dt, transB=tb)
                got = run_gemm(gs, dt, M, N, K, tb, s, A, B)
                assert np.abs(want).max() < 2048
                assert np.array_equal(got, want), f"instance {idx} K={K}: max abs diff {np.abs(got - want).max()}"
                ran += 1
    assert ran >= 6


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["cfg3_up", "cfg4", "cfg5_3x3", "cfg5_1x1s2"])
def test_benchmark_shapes_with_output_in_the_input_type(gs, name):
    """The 16-bit-input benchmark shapes with fp16 output (rounded once from the fp32 accumulator), full size,
    constructed schedule, sampled entries against the oracle."""
    import torch
    w = inputs.all_configs()[name]
    if isinstance(w, inputs.GemmWorkload):
        p = gs.gemm_problem(w.dtype, w.M, w.N, w.K, w.transA, w.transB, w.batch, "f16")
        out = gs.empty_device((w.batch, w.M, w.N) if w.batch > 1 else (w.M, w.N), "f16")
        out.fill_(float("nan"))
        dA, dB = gs.to_device(w.A, w.dtype), gs.to_device(w.B, w.dtype)
        (gs.bmm if w.batch > 1 else gs.gemm)(p, dA, dB, out, 1.0, 0.0, None)
        co = inputs.sample_indices(11, (w.batch, w.M, w.N), 400)
        want = ops.bmm_at(w.A, w.B, w.dtype, co, transA=w.transA, transB=w.transB)
        o3 = out if w.batch > 1 else out[None]
        idx = torch.from_numpy(co).cuda()
        got = o3[idx[:, 0], idx[:, 1], idx[:, 2]]
    else:
        p = gs.conv_problem(w.dtype, w.n, w.c, w.h, w.w, w.k, w.r, w.s, w.stride, w.pad, "f16")
        out = gs.empty_device((w.n, w.k, w.p, w.q), "f16")
        out.fill_(float("nan"))
        gs.conv2d(p, gs.to_device(w.I, w.dtype), gs.to_device(w.W, w.dtype), out, None, gs.conv_workspace(p))
        co = inputs.sample_indices(11, (w.n, w.k, w.p, w.q), 400)
        want = ops.conv2d_at(w.I, w.W, w.dtype, co, stride=w.stride, pad=w.pad)
        idx = torch.from_numpy(co).cuda()
        got = out[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]]
    torch.cuda.synchronize()
    assert not torch.isnan(out).any()
    assert ops.rel_frobenius(got.double().cpu().numpy(), want) <= 2e-3


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_random_gemm_shapes_with_constructed_schedules(gs, dtype):
    """Seeded random extents, layouts, batch counts and scalars, each with the schedule the constructor picks
    for it: whatever instance that is (vector or element loads, any tile) must be bit-exact on integers."""
    rng = np.random.default_rng(20250211)
    for case in range(24):
        M, N, K = (int(x) for x in rng.integers(1, 420, size=3))
        if case % 3 == 0:                       # whole 16-byte chunks: the vector paths
            N, K = max(8, N // 8 * 8), max(8, K // 8 * 8)
        tb = int(rng.integers(0, 2))
        batch = int(rng.integers(1, 4))
        alpha, beta = float(rng.integers(-2, 3)), float(rng.integers(-1, 2))
        print(f"case {case}: {dtype} {batch}x{M}x{N}x{K} transB={tb} alpha={alpha} beta={beta}", flush=True)
        A = inputs.small_ints(700 + case, (batch, M, K) if batch > 1 else (M, K), dtype, -2, 2)
        B = inputs.small_ints(800 + case, ((batch, N, K) if tb else (batch, K, N)) if batch > 1 else ((N, K) if tb else (K, N)),
                              dtype, -2, 2)
        C0 = inputs.small_ints(900 + case, (batch, M, N) if batch > 1 else (M, N), "f32", -3, 3)
        if batch > 1:
            want = np.stack([ops.gemm(A[b], B[b], dtype, transB=tb, alpha=alpha, beta=beta, C0=C0[b]) for b in range(batch)])
        else:
            want = ops.gemm(A, B, dtype, transB=tb, alpha=alpha, beta=beta, C0=C0)
        got = run_gemm(gs, dtype, M, N, K, tb, None, A, B, alpha=alpha, beta=beta, C0=C0, batch=batch)
        assert np.abs(want).max() < 2 ** 22
        assert np.array_equal(got, want), f"case {case}: max abs diff {np.abs(got - want).max()}"


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_random_conv_geometries_with_constructed_schedules(gs, dtype):
    """Seeded random convolution geometries (filter sizes 1-5, strides 1-3, paddings 0-2, channel counts with and
    without whole vectors), each with the constructed schedule: bit-exact on integers."""
    import torch
    rng = np.random.default_rng(11407)
    for case in range(16):
        r, s = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        stride, pad = int(rng.integers(1, 4)), int(rng.integers(0, 3))
        n, c, k = int(rng.integers(1, 4)), int(rng.integers(1, 5)) * (8 if case % 2 == 0 else 3), int(rng.integers(1, 90))
        h, w = int(rng.integers(max(r - 2 * pad, 1), 24)), int(rng.integers(max(s - 2 * pad, 1), 24))
        print(f"case {case}: {dtype} n={n} c={c} {h}x{w} k={k} {r}x{s} stride {stride} pad {pad}", flush=True)
        I = inputs.small_ints(1000 + case, (n, c, h, w), dtype, -2, 2)
        W = inputs.small_ints(1100 + case, (k, c, r, s), dtype, -2, 2)
        want = ops.conv2d(I, W, dtype, stride=stride, pad=pad)
        p = gs.conv_problem(dtype, n, c, h, w, k, r, s, stride, pad)
        dO = gs.empty_device(want.shape)
        dO.fill_(float("nan"))
        gs.conv2d(p, gs.to_device(I, dtype), gs.to_device(W, dtype), dO, None, gs.conv_workspace(p))
        torch.cuda.synchronize()
        assert np.array_equal(gs.to_host_f64(dO), want), f"case {case}"


# ----------------------------------------------------------------------------------------------------------
# split-k: tiles computed by several workgroups that exchange partial sums through the workspace
# ----------------------------------------------------------------------------------------------------------
def _split_schedules(gs, p, split, want_tiles):
    """Schedules of the instances that serve `p`, exist with split tiles and have one of the wanted (BM, BN)."""
    out = []
    for idx in range(gs.num_instances()):
        s = gs.instance_schedule(idx, p)
        if s is None or (s.tile[0][0], s.tile[1][0]) not in want_tiles:
            continue
        if s.direct_lds and p.K % s.tile[2][0]:
            continue                                   # direct staging takes whole k tiles only
        s.split_k = split
        if gs.workspace_bytes(p, s) > 0:
            out.append(s)
    return out


def _run_split(gs, p, s, dtype, A, B, ws, alpha=1.0, beta=0.0, C0=None, out_dtype="f32"):
    import torch
    batch = A.shape[0] if A.ndim == 3 else 1
    dA, dB = gs.to_device(A, dtype), gs.to_device(B, dtype)
    shape = (batch, p.M, p.N) if batch > 1 else (p.M, p.N)
    dC = gs.to_device(C0, out_dtype) if C0 is not None else gs.empty_device(shape, out_dtype).fill_(float("nan"))
    (gs.bmm if batch > 1 else gs.gemm)(p, dA, dB, dC, alpha, beta, s, workspace=ws)
    torch.cuda.synchronize()
    return gs.to_host_f64(dC)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,M,N,K,tb,batch,split,tiles", [
    ("f16", 256, 256, 2048, 1, 1, 8, {(256, 256), (128, 128), (64, 64)}),     # one to sixteen tiles, all split
    ("f16", 200, 136, 1000, 0, 1, 3, {(128, 128), (64, 64), (32, 32)}),       # ragged tiles, k tail, parts on different XCDs
    ("bf16", 192, 320, 1536, 1, 3, 2, {(128, 128), (64, 128), (64, 64)}),     # batched
    ("f32", 130, 72, 520, 0, 1, 4, {(64, 64), (32, 32)}),
    ("f16", 544, 544, 512, 1, 1, 2, {(32, 32)}),                              # 289 tiles: 256 whole, 33 split
    ("f16", 1024, 1088, 256, 0, 1, 4, {(64, 64)}),                            # 272 tiles: 256 whole, 16 split four ways
    ("f32", 64, 64, 4096, 1, 1, 16, {(64, 64), (32, 32)}),                    # the deepest split
])
def test_split_k_bit_exact_on_integers(gs, dtype, M, N, K, tb, batch, split, tiles):
    p = gs.gemm_problem(dtype, M, N, K, 0, tb, batch)
    scheds = _split_schedules(gs, p, split, tiles)
    assert scheds
    shp = lambda r, c: (batch, r, c) if batch > 1 else (r, c)
    A = inputs.small_ints(31, shp(M, K), dtype, -2, 2)
    B = inputs.small_ints(32, shp(N, K) if tb else shp(K, N), dtype, -2, 2)
    A2 = inputs.small_ints(33, shp(M, K), dtype, -2, 2)
    C0 = inputs.small_ints(34, shp(M, N), "f32", -3, 3)
    ref = lambda a: np.stack([ops.gemm(a[b], B[b], dtype, transB=tb, alpha=2.0, beta=-1.0, C0=C0[b]) for b in range(batch)]) \
        if batch > 1 else ops.gemm(a, B, dtype, transB=tb, alpha=2.0, beta=-1.0, C0=C0)
    want, want2 = ref(A), ref(A2)
    assert np.abs(want).max() < 2 ** 23
    for s in scheds:
        print("instance", s.kernel_id, s.describe()["tile_m"], s.describe()["tile_n"], "split", split, flush=True)
        ws = gs.gemm_workspace(p, s)
        ws.fill_(0xAB)                                  # whatever the workspace holds, counters included
        # the same workspace serves call after call: the second must not see what the first left in it
        assert np.array_equal(_run_split(gs, p, s, dtype, A2, B, ws, 2.0, -1.0, C0), want2)
        assert np.array_equal(_run_split(gs, p, s, dtype, A, B, ws, 2.0, -1.0, C0), want)


@pytest.mark.gpu
def test_split_k_real_values_and_16_bit_output(gs):
    M, N, K = 384, 256, 8192
    for dtype, out_dtype, tb in (("f16", "f32", 1), ("f16", "f16", 0), ("bf16", "bf16", 1), ("f32", "f32", 0)):
        p = gs.gemm_problem(dtype, M, N, K, 0, tb, 1, out_dtype)
        A = inputs.uniform_pm1(41, (M, K), dtype)
        B = inputs.uniform_pm1(42, (N, K) if tb else (K, N), dtype)
        want = ops.gemm(A, B, dtype, transB=tb)
        for split in (2, 5):
            for s in _split_schedules(gs, p, split, {(128, 128), (64, 64)})[:3]:
                got = _run_split(gs, p, s, dtype, A, B, gs.gemm_workspace(p, s), out_dtype=out_dtype)
                err = ops.rel_frobenius(got, want)
                print(dtype, out_dtype, "instance", s.kernel_id, "split", split, "rel frobenius", err, flush=True)
                assert err <= (TOL[dtype] if out_dtype == "f32" else 2e-3)
                # two parts are summed in one order, more parts in part order: the result is reproducible
                again = _run_split(gs, p, s, dtype, A, B, gs.gemm_workspace(p, s), out_dtype=out_dtype)
                assert np.array_equal(got, again)


@pytest.mark.gpu
def test_split_k_constructed_for_deep_k_and_workspace_rules(gs):
    import torch
    M, N, K = 512, 512, 16384
    p = gs.gemm_problem("f16", M, N, K, 0, 1)
    s = gs.construct(p)
    assert s.split_k > 1 and gs.workspace_bytes(p, s) > 0
    A, B = inputs.uniform_pm1(51, (M, K), "f16"), inputs.uniform_pm1(52, (N, K), "f16")
    want = ops.gemm(A, B, "f16", transB=1)
    ws = gs.gemm_workspace(p, s)
    assert ops.rel_frobenius(_run_split(gs, p, s, "f16", A, B, ws), want) <= TOL["f16"]
    # no schedule named: the library constructs one; with a workspace it may split, without one it does not
    assert ops.rel_frobenius(_run_split(gs, p, None, "f16", A, B, ws), want) <= TOL["f16"]
    assert ops.rel_frobenius(_run_split(gs, p, None, "f16", A, B, None), want) <= TOL["f16"]
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    assert ops.rel_frobenius(_run_split(gs, p, None, "f16", A, B, small), want) <= TOL["f16"]
    # a named split schedule needs its workspace: missing, too small, misaligned
    for bad in (None, small, ws[16:]):
        with pytest.raises(gs.GensorError) as e:
            _run_split(gs, p, s, "f16", A, B, bad)
        assert e.value.status == 4
    # more parts than k tiles, or an instance without the split path
    s.split_k = 16
    q = gs.gemm_problem("f16", M, N, 8 * s.tile[2][0], 0, 1)
    with pytest.raises(gs.GensorError) as e:
        _run_split(gs, q, s, "f16", A[:, :q.K].copy(), B[:, :q.K].copy(), ws)
    assert e.value.status == 3
    # a tile count that is a whole number of rounds has nothing to split: runs as it is, no workspace
    r = gs.gemm_problem("f16", 512, 512, 256, 0, 1)
    s32 = [x for x in (gs.instance_schedule(i, r) for i in range(gs.num_instances()))
           if x is not None and (x.tile[0][0], x.tile[1][0]) == (32, 32) and x.vec_bytes == 16 and x.stages == 2][0]
    s32.split_k = 2
    assert gs.workspace_bytes(r, s32) == 0
    Ar, Br = inputs.small_ints(53, (512, 256), "f16", -2, 2), inputs.small_ints(54, (512, 256), "f16", -2, 2)
    assert np.array_equal(_run_split(gs, r, s32, "f16", Ar, Br, None), ops.gemm(Ar, Br, "f16", transB=1))


@pytest.mark.gpu
@pytest.mark.parametrize("index", range(len(inputs.DEEP_K_GEMMS)))
def test_deep_k_shapes_full_size_sampled(gs, index):
    """The deep-k workloads bench.py times, with the constructed (split-k) schedule: sampled entries and tile
    edges against the oracle, no unwritten output."""
    w, s, got, want, finite = _full_size_case(gs, inputs.deep_k_gemm(index))
    assert s.split_k > 1
    err = ops.rel_frobenius(got, want)
    print(w.name, "kernel", s.kernel_id, "split", s.split_k, "rel frobenius", err)
    assert finite and err <= TOL[w.dtype]


@pytest.mark.gpu
def test_operators_captured_in_a_graph_replay_like_eager_calls(gs):
    """Every operator launch (the split-k pair of counter clear + kernel included) can be recorded into a HIP
    graph: each replay, with eager work and synchronisations in between and fresh inputs written into the
    captured buffers, gives what the eager call gives."""
    import torch
    M, N, K = 256, 192, 4096
    p = gs.gemm_problem("f16", M, N, K, 0, 1)
    s = [x for x in _split_schedules(gs, p, 4, {(64, 64)})][0]
    ws = gs.gemm_workspace(p, s)
    pc = gs.conv_problem("f16", 2, 16, 12, 12, 24, 3, 3, 1, 1)
    dA, dB = gs.empty_device((M, K), "f16"), gs.empty_device((N, K), "f16")
    dC, dC1 = gs.empty_device((M, N)), gs.empty_device((M, N))
    dI, dW, dO = gs.empty_device((2, 16, 12, 12), "f16"), gs.empty_device((24, 16, 3, 3), "f16"), gs.empty_device((2, 24, 12, 12))
    dx, dy = gs.empty_device((K,), "f16"), gs.empty_device((M,))
    dP = gs.empty_device((2, 16, 6, 6))
    cws = gs.conv_workspace(pc)

    def launch_all():
        gs.gemm(p, dA, dB, dC, 1.0, 0.0, s, workspace=ws)          # split-k: counter clear + kernel
        gs.gemm(p, dA, dB, dC1, 1.0, 0.0, None)                    # schedule looked up per shape
        gs.conv2d(pc, dI, dW, dO, None, cws)
        gs.gemv("f16", dA, dx, dy)
        gs.avgpool2d("f16", dI, dP, 2, 2)

    def fill(seed):
        dA.copy_(gs.to_device(inputs.small_ints(seed, (M, K), "f16", -2, 2), "f16"))
        dB.copy_(gs.to_device(inputs.small_ints(seed + 1, (N, K), "f16", -2, 2), "f16"))
        dI.copy_(gs.to_device(inputs.small_ints(seed + 2, (2, 16, 12, 12), "f16", -2, 2), "f16"))
        dW.copy_(gs.to_device(inputs.small_ints(seed + 3, (24, 16, 3, 3), "f16", -2, 2), "f16"))
        dx.copy_(gs.to_device(inputs.small_ints(seed + 4, (K,), "f16", -2, 2), "f16"))

    outs = (dC, dC1, dO, dy, dP)
    fill(60)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        launch_all()                                               # first use outside the capture (per-device set-up)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        launch_all()
    for rep in range(4):
        fill(70 + 10 * rep)
        launch_all()
        torch.cuda.synchronize()
        eager = [o.clone() for o in outs]
        for o in outs:
            o.fill_(float("nan"))
        ws.fill_(0x5A)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for name, o, e in zip(("gemm split-k", "gemm", "conv2d", "gemv", "avgpool2d"), outs, eager):
            assert torch.equal(o, e), (rep, name)
    # and the eager results are the oracle's (last inputs)
    A = inputs.small_ints(100, (M, K), "f16", -2, 2)
    B = inputs.small_ints(101, (N, K), "f16", -2, 2)
    assert np.array_equal(gs.to_host_f64(dC), ops.gemm(A, B, "f16", transB=1))


@pytest.mark.gpu
@pytest.mark.parametrize("M,N,K,split", [(384, 384, 2048, 3), (512, 512, 4096, 8), (192, 320, 1536, 5)])
def test_split_k_many_calls_on_one_workspace_stay_exact(gs, M, N, K, split):
    """Two hundred calls alternating between two input sets on one workspace, parts of a tile on one XCD
    (unit count a multiple of 8) and spread over several (not a multiple): every result is the oracle's,
    so no call ever reads a partial sum or a count that an earlier call left behind."""
    import torch
    p = gs.gemm_problem("f16", M, N, K, 0, 1)
    s = _split_schedules(gs, p, split, {(128, 128), (64, 64)})[0]
    ws = gs.gemm_workspace(p, s)
    sets = []
    for seed in (81, 91):
        A = inputs.small_ints(seed, (M, K), "f16", -2, 2)
        B = inputs.small_ints(seed + 1, (N, K), "f16", -2, 2)
        sets.append((gs.to_device(A, "f16"), gs.to_device(B, "f16"), torch.from_numpy(ops.gemm(A, B, "f16", transB=1)).float().cuda()))
    dC = gs.empty_device((M, N))
    bad = torch.zeros((), dtype=torch.int64, device="cuda")
    for it in range(200):
        dA, dB, want = sets[it & 1] if it % 7 else sets[1 - (it & 1)]
        gs.gemm(p, dA, dB, dC, 1.0, 0.0, s, workspace=ws)
        bad += (dC != want).sum()
    torch.cuda.synchronize()
    assert int(bad) == 0


# ----------------------------------------------------------------------------------------------------------
# transA: A stored [K][M]
# ----------------------------------------------------------------------------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("transB", [0, 1])
def test_gemm_with_a_stored_transposed(gs, dtype, transB):
    """C = alpha A^T-stored x op(B) + beta C under the constructed schedule: real values at the stated tolerance,
    integers exactly, aligned and unaligned extents, batched, and split along k."""
    import torch
    for (M, N, K, batch) in ((392, 264, 520, 1), (77, 53, 41, 1), (136, 200, 192, 3)):
        shp = lambda r, c: (batch, r, c) if batch > 1 else (r, c)
        A = inputs.uniform_pm1(41, shp(K, M), dtype)
        B = inputs.uniform_pm1(42, shp(N, K) if transB else shp(K, N), dtype)
        C0 = inputs.uniform_pm1(43, shp(M, N), "f32")
        got = run_gemm(gs, dtype, M, N, K, transB, None, A, B, 1.5, -0.5, C0, batch=batch, transA=1)
        ref = (lambda a, b, c: ops.gemm(a, b, dtype, transA=1, transB=transB, alpha=1.5, beta=-0.5, C0=c))
        want = np.stack([ref(A[i], B[i], C0[i]) for i in range(batch)]) if batch > 1 else ref(A, B, C0)
        err = ops.rel_frobenius(got, want)
        print(dtype, "transB", transB, (M, N, K, batch), "rel frobenius", err, flush=True)
        assert err <= TOL[dtype]
        Ai = inputs.small_ints(44, shp(K, M), dtype, -3, 3)
        Bi = inputs.small_ints(45, shp(N, K) if transB else shp(K, N), dtype, -3, 3)
        goti = run_gemm(gs, dtype, M, N, K, transB, None, Ai, Bi, batch=batch, transA=1)
        refi = lambda a, b: ops.gemm(a, b, dtype, transA=1, transB=transB)
        wanti = np.stack([refi(Ai[i], Bi[i]) for i in range(batch)]) if batch > 1 else refi(Ai, Bi)
        assert np.array_equal(goti, wanti)
    # split along k: few tiles, deep reduction
    M, N, K = 192, 136, 2048
    p = gs.gemm_problem(dtype, M, N, K, 1, transB)
    scheds = _split_schedules(gs, p, 4, {(128, 128), (64, 64)})
    assert scheds
    A = inputs.small_ints(46, (K, M), dtype, -2, 2)
    B = inputs.small_ints(47, (N, K) if transB else (K, N), dtype, -2, 2)
    want = ops.gemm(A, B, dtype, transA=1, transB=transB)
    for s in scheds[:3]:
        print("transA split-k instance", s.kernel_id, flush=True)
        assert np.array_equal(_run_split(gs, p, s, dtype, A, B, gs.gemm_workspace(p, s)), want)
