"""Workgroup -> tile maps, checked exhaustively: every output element of launches of several hundred tiles is
compared with the oracle on integer inputs (any summation order is exact), for the kernel instances the seven
benchmark configurations end in.  The launches cover a tile count that is a multiple of 8 (contiguous tile ranges
per XCD) and one that is not, more tile rows than a panel holds with a ragged last panel, ragged edge tiles, and
batches."""
import numpy as np
import pytest

from oracle import ops
from paper_2502_11407_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gs():
    from paper_2502_11407_amd import binding
    return binding


def _pick(gs, name):
    wl = inputs.all_configs()[name]
    if isinstance(wl, inputs.GemmWorkload):
        p = gs.gemm_problem(wl.dtype, wl.M, wl.N, wl.K, wl.transA, wl.transB, wl.batch)
    else:
        p = gs.conv_problem(wl.dtype, wl.n, wl.c, wl.h, wl.w, wl.k, wl.r, wl.s, wl.stride, wl.pad)
    return wl, gs.construct(p, seed=0)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3_up", "cfg3_down", "cfg4"])
def test_gemm_tile_map_every_element(gs, name):
    import torch
    wl, s0 = _pick(gs, name)
    bm, bn, bk = s0.tile[0][0], s0.tile[1][0], s0.tile[2][0]
    K = 2 * bk if bm * bn < 256 * 256 else bk          # (the map does not depend on k; the oracle's cost does)
    # (tile rows, tile columns, batch, ragged): 270 tiles (not a multiple of 8), 18 = 4 panels of 4 rows + 2; 256 tiles
    # (a multiple of 8); three batches of 90; two batches of 64
    for tm, tn, batch, ragged in ((18, 15, 1, True), (16, 16, 1, False), (10, 9, 3, True), (8, 8, 2, False)):
        M = tm * bm - (17 if ragged else 0)
        N = tn * bn - (8 if ragged else 0)
        p = gs.gemm_problem(wl.dtype, M, N, K, 0, wl.transB, batch)
        s = gs.instance_schedule(s0.kernel_id, p)
        assert s is not None and s.wg_remap == 4 and tm > s.wg_remap
        print(f"{name}: instance {s.kernel_id} tile {bm}x{bn}x{bk}: {tm}x{tn} tiles x {batch} batch(es), M={M} N={N} K={K}", flush=True)
        shp = lambda r, c: (batch, r, c) if batch > 1 else (r, c)
        A = inputs.small_ints(500 + tm, shp(M, K), wl.dtype, -3, 3)
        B = inputs.small_ints(600 + tn, shp(N, K) if wl.transB else shp(K, N), wl.dtype, -3, 3)
        dC = torch.full(shp(M, N), float("nan"), dtype=torch.float32, device="cuda")
        (gs.bmm if batch > 1 else gs.gemm)(p, gs.to_device(A, wl.dtype), gs.to_device(B, wl.dtype), dC, 1.0, 0.0, s)
        torch.cuda.synchronize()
        got = gs.to_host_f64(dC)
        want = np.stack([ops.gemm(A[b], B[b], wl.dtype, transB=wl.transB) for b in range(batch)]) if batch > 1 \
            else ops.gemm(A, B, wl.dtype, transB=wl.transB)
        assert np.array_equal(got, want), f"{name} {tm}x{tn}x{batch}: {np.count_nonzero(got != want)} elements differ"


def _conv_tile_px(bn, N, Q, tiles_m, cus=256):
    """The library's rule for the pixels of a patch-staged workgroup (whole output rows when rows are shorter than
    the tile, as many as fit or fewer when that deals the tiles more evenly), restated here only to choose
    geometries with the wanted tile counts; the comparison below does not depend on it."""
    import math
    if Q > bn:
        return bn
    cost = lambda px: math.ceil(math.ceil(N / px) * tiles_m / cus) * (0.55 * bn + 0.45 * px)
    best = bn // Q * Q
    for r in range(bn // Q - 1, 0, -1):
        if cost(r * Q) < cost(best):
            best = r * Q
    return best


@pytest.mark.parametrize("tiles_m,whole_octets,ragged", [(4, False, True), (4, True, False)])
def test_conv_patch_tile_map_every_element(gs, tiles_m, whole_octets, ragged):
    """The patch-staged convolution instance of the 3x3 benchmark shape over a few hundred tiles, every output element
    compared: once with a tile count that is a multiple of 8 (the XCD-contiguous remap) and once with one that is
    not, the latter with a ragged last pixel tile and ragged filter rows."""
    import torch
    wl, s0 = _pick(gs, "cfg5_3x3")
    assert s0.direct_lds == 1
    bm, bn = s0.tile[0][0], s0.tile[1][0]
    k = tiles_m * bm - (5 if ragged else 0)
    c = 32
    found = None
    for h in range(30, 40):
        for w in range(30, 44):
            for n in range(10, 18):
                N = n * h * w
                px = _conv_tile_px(bn, N, w, tiles_m)
                total = -(-N // px) * tiles_m
                if total >= 256 and (total % 8 == 0) == whole_octets and (N % px != 0) == ragged:
                    found = found or (n, h, w, px, total)
    assert found, "no geometry with the wanted tile count"
    n, h, w, px, total = found
    p = gs.conv_problem(wl.dtype, n, c, h, w, k, 3, 3, 1, 1)
    s = gs.instance_schedule(s0.kernel_id, p)
    assert s is not None
    print(f"conv patch instance {s.kernel_id} tile {bm}x{bn}: {total} tiles of {px} pixels, n={n} c={c} h={h} w={w} k={k}", flush=True)
    I = inputs.small_ints(700, (n, c, h, w), wl.dtype, -2, 2)
    W = inputs.small_ints(701, (k, c, 3, 3), wl.dtype, -2, 2)
    dO = gs.empty_device((n, k, h, w)).fill_(float("nan"))
    gs.conv2d(p, gs.to_device(I, wl.dtype), gs.to_device(W, wl.dtype), dO, s, gs.conv_workspace(p, s))
    torch.cuda.synchronize()
    got = gs.to_host_f64(dO)
    want = ops.conv2d(I, W, wl.dtype, stride=1, pad=1)
    assert np.array_equal(got, want), f"{np.count_nonzero(got != want)} elements differ"


def test_sampled_pointwise_conv_tile_map_every_element(gs):
    """The stride-2 pointwise benchmark convolution's instance (B operand sampled while fetched) as a batched GEMM
    of 3 images x (5 x 18) tiles."""
    import torch
    wl, s0 = _pick(gs, "cfg5_1x1s2")
    bm, bn = s0.tile[0][0], s0.tile[1][0]
    k = 5 * bm - 3
    pq = 18 * bn - 16
    q = 48
    pp = -(-pq // q)
    n, c = 3, 2 * s0.tile[2][0]
    p = gs.conv_problem(wl.dtype, n, c, 2 * pp, 2 * q, k, 1, 1, 2, 0)
    s = gs.instance_schedule(s0.kernel_id, p)
    assert s is not None
    print(f"pointwise instance {s.kernel_id} tile {bm}x{bn}: n={n} c={c} h={2 * pp} w={2 * q} k={k}", flush=True)
    I = inputs.small_ints(710, (n, c, 2 * pp, 2 * q), wl.dtype, -2, 2)
    W = inputs.small_ints(711, (k, c, 1, 1), wl.dtype, -2, 2)
    dO = gs.empty_device((n, k, pp, q)).fill_(float("nan"))
    gs.conv2d(p, gs.to_device(I, wl.dtype), gs.to_device(W, wl.dtype), dO, s, gs.conv_workspace(p, s))
    torch.cuda.synchronize()
    got = gs.to_host_f64(dO)
    want = ops.conv2d(I, W, wl.dtype, stride=2, pad=0)
    assert np.array_equal(got, want), f"{np.count_nonzero(got != want)} elements differ"
