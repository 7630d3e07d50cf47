"""The allocation-free GEMM entry point (gensor_gemm_static_scratch: split-k counters and partial tiles in a device
array of the library itself) against gensor_gemm with a caller-owned workspace: same kernels, same summation
order, so the outputs must be identical bit for bit; and against the oracle at the stated tolerance."""
import numpy as np
import pytest

from oracle import ops
from paper_2502_11407_amd import inputs

pytestmark = pytest.mark.gpu


def _split_schedule(gs, p, split, tile):
    for idx in range(gs.num_instances()):
        s = gs.instance_schedule(idx, p)
        if s is None or (s.tile[0][0], s.tile[1][0]) != tile or (s.direct_lds and p.K % s.tile[2][0]):
            continue
        s.split_k = split
        if gs.workspace_bytes(p, s) > 0:
            return s
    raise AssertionError("no split-k instance")


def _both(gs, p, s, A, B, alpha, beta, C0):
    import torch
    dA, dB = gs.to_device(A, "f16"), gs.to_device(B, "f16")
    ref, out = gs.to_device(C0, "f32"), gs.to_device(C0, "f32")
    ws = gs.gemm_workspace(p, s)
    ws.fill_(0x5A)
    gs.gemm(p, dA, dB, ref, alpha, beta, s, workspace=ws)
    before = torch.cuda.memory_allocated()
    gs.gemm_static_scratch(p, dA, dB, out, alpha, beta, s)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return gs.to_host_f64(ref), gs.to_host_f64(out)


def test_static_scratch_gemm_equals_workspace_gemm_twice_second_smaller():
    from paper_2502_11407_amd import binding as gs
    # first call: 9 tiles of 128x128 split 8 ways over a deep k (ragged tiles); second call: a smaller problem,
    # fewer parts -- it must not see what the first left in the array
    for (M, N, K, split, tile, seed) in ((300, 330, 4096, 8, (128, 128), 1), (130, 72, 1024, 3, (64, 64), 2)):
        p = gs.gemm_problem("f16", M, N, K, 0, 1)
        s = _split_schedule(gs, p, split, tile)
        assert 0 < gs.workspace_bytes(p, s) <= gs.STATIC_SCRATCH_BYTES
        print("static scratch: ", M, N, K, "split", split, "instance", s.kernel_id, flush=True)
        A = inputs.small_ints(seed, (M, K), "f16", -2, 2)
        B = inputs.small_ints(seed + 10, (N, K), "f16", -2, 2)
        C0 = inputs.small_ints(seed + 20, (M, N), "f32", -3, 3)
        ref, out = _both(gs, p, s, A, B, 2.0, -1.0, C0)
        assert np.array_equal(out, ref)
        assert np.array_equal(out, ops.gemm(A, B, "f16", transB=1, alpha=2.0, beta=-1.0, C0=C0))      # integers: exact
        Ar, Br = inputs.uniform_pm1(seed + 30, (M, K), "f16"), inputs.uniform_pm1(seed + 40, (N, K), "f16")
        ref, out = _both(gs, p, s, Ar, Br, 1.0, 0.0, np.full((M, N), np.nan, dtype=np.float32))
        assert np.array_equal(out, ref)
        assert ops.rel_frobenius(out, ops.gemm(Ar, Br, "f16", transB=1)) <= 2e-3


def test_static_scratch_gemm_refuses_what_does_not_fit_and_constructs_when_unnamed():
    import torch
    from paper_2502_11407_amd import binding as gs
    # 16 tiles of 256x256 split 16 ways need 64 MiB of partial tiles: more than the array
    p = gs.gemm_problem("f16", 1024, 1024, 8192, 0, 1)
    s = _split_schedule(gs, p, 16, (256, 256))
    assert gs.workspace_bytes(p, s) > gs.STATIC_SCRATCH_BYTES
    dA = torch.zeros((1024, 8192), dtype=torch.float16, device="cuda")
    dC = torch.full((1024, 1024), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(gs.GensorError) as e:
        gs.gemm_static_scratch(p, dA, dA, dC, 1.0, 0.0, s)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert torch.all(dC == 7.0).item()                   # nothing was launched
    # no schedule named: the library constructs one (it may split: the array is its workspace)
    M, N, K = 256, 256, 8192
    q = gs.gemm_problem("f16", M, N, K, 0, 1)
    A, B = inputs.uniform_pm1(5, (M, K), "f16"), inputs.uniform_pm1(6, (N, K), "f16")
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    gs.gemm_static_scratch(q, gs.to_device(A, "f16"), gs.to_device(B, "f16"), out)
    torch.cuda.synchronize()
    assert ops.rel_frobenius(gs.to_host_f64(out), ops.gemm(A, B, "f16", transB=1)) <= 2e-3
