"""Pins for the operator oracle (oracle/oracle_ops.c).

The oracle is the plain definition of GEMM / BMM / Conv2d (operator table of the paper).
The paper prints no worked numeric example of an operator result, so the pins are:
hand-computed tiny cases, closed forms, identities, delta filters, independent library
routines (numpy matmul, scipy correlate2d) and an im2col formulation written only here.
Each is chosen so that a dropped term, wrong sign/index or transposed operand fails.
"""
import numpy as np
import pytest
import scipy.signal

from oracle import ops
from paper_2502_11407_amd import inputs

RNG = np.random.default_rng(1234)


def ints(shape, lo=-4, hi=4, dtype=np.float32):
    return RNG.integers(lo, hi + 1, size=shape).astype(dtype)


# ------------------------------------------------------------------ storage decoding
def test_half_decode_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    got = ops.decode(h, "f16")
    want = h.astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_half_decode_known_values():
    # sign/exponent/fraction fields of IEEE binary16 written out by hand
    cases = {0x3C00: 1.0, 0xC000: -2.0, 0x3555: 0.333251953125, 0x0001: 2.0 ** -24,
             0x0400: 2.0 ** -14, 0x7BFF: 65504.0, 0x8000: -0.0, 0x7C00: np.inf}
    for bits, val in cases.items():
        got = ops.decode(np.array([bits], dtype=np.uint16).view(np.float16), "f16")[0]
        assert got == val, hex(bits)


def test_bf16_decode_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    got = ops.decode(bits, "bf16")
    want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert ops.decode(np.array([0x3F80, 0xC040, 0x3DCD], dtype=np.uint16), "bf16").tolist() == \
        [1.0, -3.0, 0.10009765625]


def test_bf16_rounding_of_generator_is_nearest_even():
    # 1 + 2^-8 lies exactly between two bf16 values -> ties to even (1.0);
    # 1 + 3*2^-8 ties to 1 + 2^-6.
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    b = inputs.f32_to_bf16_bits(x)
    assert ops.decode(b, "bf16").tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]


# ------------------------------------------------------------------ GEMM
def test_gemm_2x2_by_hand():
    A = np.array([[1, 2], [3, 4]], dtype=np.float32)
    B = np.array([[5, 6], [7, 8]], dtype=np.float32)
    # row 0: 1*5+2*7=19, 1*6+2*8=22; row 1: 3*5+4*7=43, 3*6+4*8=50
    assert ops.gemm(A, B, "f32").tolist() == [[19, 22], [43, 50]]
    # non-symmetric check that A.B != B.A is respected: B.A = [[23,34],[31,46]]
    assert ops.gemm(B, A, "f32").tolist() == [[23, 34], [31, 46]]


def test_gemm_rectangular_by_hand():
    A = np.array([[1, 0, 2]], dtype=np.float32)            # 1x3
    B = np.array([[1, 2], [3, 4], [5, 6]], dtype=np.float32)  # 3x2
    assert ops.gemm(A, B, "f32").tolist() == [[11, 14]]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_gemm_matches_numpy_on_integers(dtype, tA, tB):
    M, N, K = 5, 7, 3
    A = ints((M, K))
    B = ints((K, N))
    As = inputs.to_storage(A.T if tA else A, dtype)
    Bs = inputs.to_storage(B.T if tB else B, dtype)
    got = ops.gemm(As, Bs, dtype, transA=tA, transB=tB)
    assert np.array_equal(got, A.astype(np.float64) @ B.astype(np.float64))


def test_gemm_alpha_beta():
    M, N, K = 4, 6, 5
    A, B, C0 = ints((M, K)), ints((K, N)), ints((M, N)).astype(np.float64)
    AB = A.astype(np.float64) @ B.astype(np.float64)
    assert np.array_equal(ops.gemm(A, B, "f32", alpha=2.0, beta=-3.0, C0=C0), 2 * AB - 3 * C0)
    assert np.array_equal(ops.gemm(A, B, "f32", alpha=0.0, beta=1.0, C0=C0), C0)
    # beta = 0 must not read C: NaNs in C0 do not propagate
    assert np.array_equal(ops.gemm(A, B, "f32", alpha=1.0, beta=0.0, C0=np.full((M, N), np.nan)), AB)


def test_gemm_identity_and_ones():
    A = ints((6, 6))
    I = np.eye(6, dtype=np.float32)
    assert np.array_equal(ops.gemm(A, I, "f32"), A)
    assert np.array_equal(ops.gemm(I, A, "f32"), A)
    ones = np.ones((4, 9), dtype=np.float16)
    assert np.array_equal(ops.gemm(ones, np.ones((9, 5), dtype=np.float16), "f16"), np.full((4, 5), 9.0))


def test_gemm_real_values_against_numpy_float64():
    w = inputs.config2_gemm_f16(size=48)
    want = w.A.astype(np.float64) @ w.B.astype(np.float64).T
    got = ops.gemm(w.A, w.B, "f16", transB=1)
    assert ops.rel_frobenius(got, want) < 1e-14


def test_gemm_leading_dimension_and_linearity():
    A, B1, B2 = ints((3, 4)), ints((4, 5)), ints((4, 5))
    lhs = ops.gemm(A, (2 * B1 - 3 * B2).astype(np.float32), "f32")
    assert np.array_equal(lhs, 2 * ops.gemm(A, B1, "f32") - 3 * ops.gemm(A, B2, "f32"))


# ------------------------------------------------------------------ BMM
def test_bmm_is_gemm_per_batch_and_at():
    nb, M, N, K = 3, 4, 5, 6
    A = inputs.small_ints(1, (nb, M, K), "f16")
    B = inputs.small_ints(2, (nb, N, K), "f16")   # stored transposed
    got = ops.bmm(A, B, "f16", transB=1)
    for b in range(nb):
        assert np.array_equal(got[b], A[b].astype(np.float64) @ B[b].astype(np.float64).T)
        assert np.array_equal(got[b], ops.gemm(A[b], B[b], "f16", transB=1))
    co = np.array([[0, 0, 0], [2, 3, 4], [1, 2, 0]])
    assert np.array_equal(ops.bmm_at(A, B, "f16", co, transB=1), got[co[:, 0], co[:, 1], co[:, 2]])


def test_bmm_alpha_beta_and_materialised_transpose():
    w = inputs.config4_bmm_scores(batch=2, seq=8, head=4)
    wt = inputs.config4_bmm_scores(batch=2, seq=8, head=4, materialised_kt=True)
    a = ops.bmm(w.A, w.B, "f16", transB=1, alpha=0.5)
    b = ops.bmm(wt.A, wt.B, "f16", transB=0, alpha=0.5)
    assert np.array_equal(a, b)
    want = 0.5 * np.einsum("bik,bjk->bij", w.A.astype(np.float64), w.B.astype(np.float64))
    assert ops.rel_frobenius(a, want) < 1e-14


# ------------------------------------------------------------------ Conv2d
def test_conv_3x3_on_4x4_by_hand():
    I = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    W = np.array([[1, 0, -1], [2, 0, -2], [1, 0, -1]], dtype=np.float32).reshape(1, 1, 3, 3)
    # cross-correlation, valid: every 3x3 window has columns differing by 2 -> (1+2+1)*(-2) = -8
    assert ops.conv2d(I, W, "f32").tolist() == [[[[-8, -8], [-8, -8]]]]
    # an asymmetric filter tells correlation from convolution: picks bottom-right of the window
    W2 = np.zeros((1, 1, 3, 3), dtype=np.float32)
    W2[0, 0, 2, 2] = 1
    assert ops.conv2d(I, W2, "f32").tolist() == [[[[10, 11], [14, 15]]]]
    # pad 1: output 4x4, corner (0,0) sees I[1][1] = 5 through tap (2,2)
    O = ops.conv2d(I, W2, "f32", pad=1)
    assert O.shape == (1, 1, 4, 4) and O[0, 0, 0, 0] == 5 and O[0, 0, 3, 3] == 0 and O[0, 0, 2, 2] == 15


@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 1), (2, 0), (2, 1), (3, 2)])
def test_conv_delta_filter_shifts_the_input(stride, pad):
    n, c, h, w, r, s = 2, 3, 7, 6, 3, 3
    I = ints((n, c, h, w))
    for (r0, s0) in [(0, 0), (1, 2), (2, 1)]:
        W = np.zeros((c, c, r, s), dtype=np.float32)
        for ch in range(c):
            W[ch, ch, r0, s0] = 1
        O = ops.conv2d(I, W, "f32", stride=stride, pad=pad)
        _, _, P, Q = O.shape
        Ipad = np.zeros((n, c, h + 2 * pad, w + 2 * pad))
        Ipad[:, :, pad:pad + h, pad:pad + w] = I
        for p in range(P):
            for q in range(Q):
                assert np.array_equal(O[:, :, p, q], Ipad[:, :, p * stride + r0, q * stride + s0])


def test_conv_all_ones_closed_form():
    c = 5
    I = np.ones((1, c, 6, 6), dtype=np.float16)
    W = np.ones((2, c, 3, 3), dtype=np.float16)
    O = ops.conv2d(I, W, "f16", pad=1)
    assert O.shape == (1, 2, 6, 6)
    assert np.all(O[:, :, 1:-1, 1:-1] == 9 * c)
    assert np.all(O[:, :, 0, 1:-1] == 6 * c) and np.all(O[:, :, 1:-1, -1] == 6 * c)
    assert O[0, 0, 0, 0] == 4 * c and O[0, 1, -1, -1] == 4 * c


def test_conv_1x1_is_a_gemm_per_image():
    n, c, h, w, k = 2, 6, 5, 4, 3
    I = inputs.small_ints(5, (n, c, h, w), "bf16")
    W = inputs.small_ints(6, (k, c, 1, 1), "bf16")
    O = ops.conv2d(I, W, "bf16")
    Wf = inputs.bf16_bits_to_f32(W).astype(np.float64).reshape(k, c)
    If = inputs.bf16_bits_to_f32(I).astype(np.float64)
    for i in range(n):
        assert np.array_equal(O[i].reshape(k, h * w), Wf @ If[i].reshape(c, h * w))


@pytest.mark.parametrize("stride,pad,r,s", [(1, 1, 3, 3), (2, 0, 1, 1), (2, 1, 3, 3), (2, 2, 5, 3)])
def test_conv_against_scipy_correlate_and_im2col(stride, pad, r, s):
    n, c, h, w, k = 2, 4, 9, 8, 3
    I = ints((n, c, h, w))
    W = ints((k, c, r, s))
    O = ops.conv2d(I, W, "f32", stride=stride, pad=pad)
    Ipad = np.zeros((n, c, h + 2 * pad, w + 2 * pad))
    Ipad[:, :, pad:pad + h, pad:pad + w] = I
    # (i) library routine: full stride-1 correlation per (image, filter, channel), then subsample
    ref = np.zeros_like(O)
    for i in range(n):
        for kk in range(k):
            acc = sum(scipy.signal.correlate2d(Ipad[i, ch], W[kk, ch].astype(np.float64), mode="valid")
                      for ch in range(c))
            ref[i, kk] = acc[::stride, ::stride]
    assert np.array_equal(O, ref)
    # (ii) im2col written here: columns = (n,p,q), rows = (c,r,s); one numpy matmul
    _, _, P, Q = O.shape
    cols = np.zeros((c * r * s, n * P * Q))
    for i in range(n):
        for p in range(P):
            for q in range(Q):
                cols[:, (i * P + p) * Q + q] = Ipad[i, :, p * stride:p * stride + r, q * stride:q * stride + s].reshape(-1)
    out = W.reshape(k, -1).astype(np.float64) @ cols
    assert np.array_equal(O, out.reshape(k, n, P, Q).transpose(1, 0, 2, 3))


def test_conv_strided_equals_subsampled_stride1():
    I, W = ints((1, 3, 11, 10)), ints((2, 3, 3, 3))
    full = ops.conv2d(I, W, "f32", stride=1, pad=1)
    assert np.array_equal(ops.conv2d(I, W, "f32", stride=2, pad=1), full[:, :, ::2, ::2])
    assert np.array_equal(ops.conv2d(I, W, "f32", stride=3, pad=1), full[:, :, ::3, ::3])


def test_conv_at_matches_full_and_output_shape_rule():
    w = inputs.config5_conv("3x3", n=2, hw=10)
    O = ops.conv2d(w.I, w.W, "f16", stride=w.stride, pad=w.pad)
    assert O.shape == (2, 64, w.p, w.q) == (2, 64, 10, 10)
    co = inputs.sample_indices(3, O.shape, 50)
    got = ops.conv2d_at(w.I, w.W, "f16", co, stride=w.stride, pad=w.pad)
    assert np.array_equal(got, O[co[:, 0], co[:, 1], co[:, 2], co[:, 3]])
    w2 = inputs.config5_conv("1x1s2", n=1, hw=8)
    assert ops.conv2d(w2.I, w2.W, "f16", stride=2, pad=0).shape == (1, 512, 4, 4)


def test_conv_real_values_against_float64_einsum():
    w = inputs.config5_conv("3x3", n=1, hw=6)
    I = np.pad(w.I.astype(np.float64), ((0, 0), (0, 0), (1, 1), (1, 1)))
    win = np.lib.stride_tricks.sliding_window_view(I, (3, 3), axis=(2, 3))  # n c p q r s
    want = np.einsum("ncpqrs,kcrs->nkpq", win, w.W.astype(np.float64))
    assert ops.rel_frobenius(ops.conv2d(w.I, w.W, "f16", pad=1), want) < 1e-14


# ------------------------------------------------------------------ error-bound sanity
def test_fp32_accumulation_error_is_far_below_the_tolerance():
    """A float32 running sum of the exact fp16 products (what the GPU's accumulate does, in
    some order) must sit near 1e-7..1e-6 of the fp64 oracle: anything near the 2e-3 limit
    would be a bug, not rounding."""
    w = inputs.config2_gemm_f16(size=256)
    want = ops.gemm(w.A, w.B, "f16", transB=1)
    acc = np.zeros((256, 256), dtype=np.float32)
    A32, B32 = w.A.astype(np.float32), w.B.astype(np.float32)
    for k in range(256):
        acc += np.outer(A32[:, k], B32[:, k])
    err = ops.rel_frobenius(acc, want)
    assert err < 5e-6


def test_seeded_inputs_are_reproducible_and_shaped():
    a = inputs.config2_gemm_f16(size=64)
    b = inputs.config2_gemm_f16(size=64)
    assert np.array_equal(a.A.view(np.uint16), b.A.view(np.uint16)) and a.B.shape == (64, 64) and a.transB == 1
    g = inputs.config3_gpt2("up", rows=16)
    assert g.A.shape == (16, 768) and g.B.shape == (768, 3072) and abs(float(g.B.astype(np.float32).std()) - 0.02) < 2e-3
    c = inputs.config5_conv("1x1s2", n=1, hw=8)
    assert c.W.shape == (512, 256, 1, 1) and c.stride == 2 and c.pad == 0
    assert abs(float(a.A.astype(np.float32).max())) <= 1.0


# ------------------------------------------------------------------ GEMV (operator table, GEMV row)
def test_gemv_hand_case_and_scalars():
    # [[1,2,3],[4,5,6]] . [1,0,-1] = [-2,-2]
    A = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)
    x = np.array([1, 0, -1], dtype=np.float32)
    assert ops.gemv(A, x, "f32").tolist() == [-2.0, -2.0]
    assert ops.gemv(A, x, "f32", alpha=3.0, beta=0.5, y0=[10.0, 20.0]).tolist() == [-1.0, 4.0]
    assert ops.gemv(A, x, "f32", alpha=0.0, beta=1.0, y0=[7.0, -9.0]).tolist() == [7.0, -9.0]
    # beta = 0 must not read y0
    assert ops.gemv(A, x, "f32", beta=0.0, y0=[np.nan, np.nan]).tolist() == [-2.0, -2.0]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_gemv_against_numpy_and_gemm(dtype):
    A = inputs.small_ints(31, (37, 53), dtype)
    x = inputs.small_ints(32, (53,), dtype)
    got = ops.gemv(A, x, dtype)
    want = ops.decode(A, dtype) @ ops.decode(x, dtype)                  # float64 library matmul
    assert np.array_equal(got, want)
    # a GEMV is the GEMM with a single column (the two oracle routines share only the decoder)
    assert np.array_equal(got, ops.gemm(A, x.reshape(53, 1), dtype)[:, 0])
    # unit vectors pick columns (a transposed A or a wrong stride would pick rows)
    for n in (0, 17, 52):
        e = np.zeros(53, dtype=np.float32)
        e[n] = 1.0
        assert np.array_equal(ops.gemv(A, inputs.to_storage(e, dtype), dtype), ops.decode(A, dtype)[:, n])


def test_gemv_real_values_close_to_longdouble():
    A = inputs.uniform_pm1(33, (64, 1000), "f16")
    x = inputs.uniform_pm1(34, (1000,), "f16")
    want = (A.astype(np.longdouble) * x.astype(np.longdouble)[None, :]).sum(axis=1)
    assert np.abs(ops.gemv(A, x, "f16") - want.astype(np.float64)).max() <= 1e-12


# ------------------------------------------------------------------ AvgPooling2d (operator table, AvgPooling2d row)
def test_avgpool_hand_case():
    I = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    # 2x2 windows at stride 2: means of {0,1,4,5}, {2,3,6,7}, {8,9,12,13}, {10,11,14,15}
    assert ops.avgpool2d(I, "f32", 2, 2).reshape(-1).tolist() == [2.5, 4.5, 10.5, 12.5]
    # 3x3 window at stride 1 on the same image: centre values 5, 6, 9, 10 (mean of a ramp = its centre)
    assert ops.avgpool2d(I, "f32", 3, 1).reshape(-1).tolist() == [5.0, 6.0, 9.0, 10.0]
    # a window that would leave the image does not exist: 4 -> floor((4-3)/2)+1 = 1
    assert ops.avgpool2d(I, "f32", 3, 2).shape == (1, 1, 1, 1)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("f,stride,h,w", [(2, 2, 8, 10), (3, 2, 9, 7), (2, 2, 7, 9), (3, 1, 6, 6), (1, 3, 7, 8)])
def test_avgpool_against_numpy_windows(dtype, f, stride, h, w):
    I = inputs.small_ints(35, (2, 3, h, w), dtype, -8, 8)
    got = ops.avgpool2d(I, dtype, f, stride)
    d = ops.decode(I, dtype)
    P, Q = (h - f) // stride + 1, (w - f) // stride + 1
    assert got.shape == (2, 3, P, Q)
    # sliding_window_view is numpy's own windowing; mean over the window axes
    win = np.lib.stride_tricks.sliding_window_view(d, (f, f), axis=(2, 3))[:, :, ::stride, ::stride]
    assert np.array_equal(got, win.sum(axis=(4, 5)) / (f * f))
    # coordinates one by one
    co = np.array([[0, 0, 0, 0], [1, 2, P - 1, Q - 1], [1, 0, P // 2, 0]], dtype=np.int64)
    assert np.array_equal(ops.avgpool2d_at(I, dtype, co, f, stride), got[co[:, 0], co[:, 1], co[:, 2], co[:, 3]])


def test_avgpool_closed_forms_and_conv_identity():
    # constant image -> the constant; delta at (y0, x0) -> 1/F^2 in exactly the windows that hold it
    I = np.full((1, 2, 9, 9), 3.0, dtype=np.float32)
    assert np.all(ops.avgpool2d(I, "f32", 3, 2) == 3.0)
    D = np.zeros((1, 1, 9, 9), dtype=np.float32)
    D[0, 0, 4, 5] = 9.0
    O = ops.avgpool2d(D, "f32", 3, 2)                          # windows start at 0,2,4,6: rows {2,4} cols {4} hold (4,5)
    want = np.zeros((1, 1, 4, 4))
    want[0, 0, 1, 2] = want[0, 0, 2, 2] = 1.0
    assert np.array_equal(O, want)
    # pooling is the convolution with a constant 1/F^2 filter per channel
    X = inputs.small_ints(36, (2, 3, 8, 8), "f32", -8, 8)
    Wt = np.zeros((3, 3, 2, 2), dtype=np.float32)
    for c in range(3):
        Wt[c, c] = 0.25
    assert np.array_equal(ops.avgpool2d(X, "f32", 2, 2), ops.conv2d(X, Wt, "f32", stride=2, pad=0))
