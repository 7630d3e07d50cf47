"""ctypes face of libgensor.so (include/gensor.h).  Argument marshalling only: every step
of the operators runs in the library's HIP kernels, the constructor in its C++ host code.
PyTorch is used for device memory and the current stream, nothing else.

Importing this module loads the library and raises if it has not been built
(python -m paper_2502_11407_amd.csrc.build, or __graft_entry__.build()).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgensor.so")

GENSOR_OK = 0
STATUS = {0: "OK", 1: "INVALID_ARG", 2: "UNSUPPORTED", 3: "NO_SCHEDULE", 4: "WORKSPACE", 5: "DEVICE"}
DTYPE = {"f32": 0, "f16": 1, "bf16": 2}
OP_GEMM, OP_BMM, OP_CONV2D = 0, 1, 2

EXPORTS = ["gensor_hw_mi355x", "gensor_construct", "gensor_construct_trace", "gensor_predict_us",
           "gensor_num_instances", "gensor_instance_schedule", "gensor_gemm", "gensor_bmm", "gensor_conv2d",
           "gensor_workspace_bytes", "gensor_status_string", "gensor_gemm_static_scratch", "gensor_gemv", "gensor_avgpool2d"]


class Problem(C.Structure):
    _fields_ = [("op", C.c_int32), ("in_dtype", C.c_int32), ("out_dtype", C.c_int32),
                ("transA", C.c_int32), ("transB", C.c_int32),
                ("batch", C.c_int64), ("M", C.c_int64), ("N", C.c_int64), ("K", C.c_int64),
                ("n", C.c_int64), ("c", C.c_int64), ("h", C.c_int64), ("w", C.c_int64),
                ("k", C.c_int64), ("r", C.c_int64), ("s", C.c_int64),
                ("stride", C.c_int64), ("pad", C.c_int64)]


class Schedule(C.Structure):
    _fields_ = [("version", C.c_int32), ("kernel_id", C.c_int32),
                ("tile", (C.c_int32 * 3) * 3), ("vthread", C.c_int32 * 2),
                ("stages", C.c_int32), ("unroll", C.c_int32), ("vec_bytes", C.c_int32),
                ("direct_lds", C.c_int32), ("split_k", C.c_int32), ("wg_remap", C.c_int32),
                ("predicted_us", C.c_double), ("construct_s", C.c_double),
                ("iterations", C.c_int32), ("chains", C.c_int32), ("states_scored", C.c_int32),
                ("round_units", C.c_int32), ("seed", C.c_uint64)]

    def describe(self) -> dict:
        t = [[self.tile[d][l] for l in range(3)] for d in range(3)]
        return {"kernel_id": self.kernel_id, "tile_m": t[0], "tile_n": t[1], "tile_k": t[2],
                "vthread": [self.vthread[0], self.vthread[1]], "stages": self.stages, "unroll": self.unroll,
                "vec_bytes": self.vec_bytes, "direct_lds": self.direct_lds, "wg_remap": self.wg_remap,
                "predicted_us": self.predicted_us, "construct_s": self.construct_s,
                "iterations": self.iterations, "chains": self.chains, "states_scored": self.states_scored}


class Hw(C.Structure):
    _fields_ = [("compute_units", C.c_int32), ("simds_per_cu", C.c_int32), ("wave_size", C.c_int32),
                ("max_waves_per_wg", C.c_int32), ("lds_bytes_per_cu", C.c_int32), ("regs_per_lane", C.c_int32),
                ("lds_banks", C.c_int32), ("lds_bank_bytes", C.c_int32), ("clock_ghz", C.c_double),
                ("latency_ns", C.c_double * 3), ("bandwidth_gbs", C.c_double * 3),
                ("l2_bandwidth_gbs", C.c_double), ("mfma_tflops_16bit", C.c_double),
                ("mfma_tflops_f32", C.c_double), ("launch_us", C.c_double)]


class ConstructOpts(C.Structure):
    _fields_ = [("T0", C.c_double), ("threshold", C.c_double), ("chains", C.c_int32),
                ("keep_policy", C.c_int32), ("tiling_benefit", C.c_int32), ("no_vthread", C.c_int32),
                ("no_split_k", C.c_int32), ("greedy", C.c_int32)]


class GensorError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS.get(status, status)} ({status_string(status)})")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2502_11407_amd.csrc.build` "
                          "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    P, S = C.POINTER(Problem), C.POINTER(Schedule)
    vp, i64, f32, i32 = C.c_void_p, C.c_int64, C.c_float, C.c_int32
    L.gensor_status_string.restype = C.c_char_p
    L.gensor_status_string.argtypes = [i32]
    L.gensor_num_instances.restype = i32
    L.gensor_instance_schedule.restype = i32
    L.gensor_instance_schedule.argtypes = [i32, P, S]
    L.gensor_hw_mi355x.restype = C.POINTER(Hw)
    L.gensor_construct.restype = i32
    L.gensor_construct.argtypes = [P, C.POINTER(Hw), C.POINTER(ConstructOpts), C.c_uint64, S]
    L.gensor_construct_trace.restype = i32
    L.gensor_construct_trace.argtypes = [P, C.POINTER(Hw), C.POINTER(ConstructOpts), C.c_uint64, i32,
                                         C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    L.gensor_predict_us.restype = C.c_double
    L.gensor_predict_us.argtypes = [S, P, C.POINTER(Hw)]
    L.gensor_gemm.restype = i32
    L.gensor_gemm.argtypes = [S, P, f32, vp, i64, vp, i64, f32, vp, i64, vp, C.c_size_t, vp]
    L.gensor_gemm_static_scratch.restype = i32
    L.gensor_gemm_static_scratch.argtypes = [S, P, f32, vp, i64, vp, i64, f32, vp, i64, vp]
    L.gensor_bmm.restype = i32
    L.gensor_bmm.argtypes = [S, P, f32, vp, i64, i64, vp, i64, i64, f32, vp, i64, i64, vp, C.c_size_t, vp]
    L.gensor_conv2d.restype = i32
    L.gensor_conv2d.argtypes = [S, P, vp, vp, vp, vp, C.c_size_t, vp]
    L.gensor_workspace_bytes.restype = C.c_size_t
    L.gensor_workspace_bytes.argtypes = [S, P]
    L.gensor_gemv.restype = i32
    L.gensor_gemv.argtypes = [i32, i64, i64, f32, vp, i64, vp, f32, vp, vp]
    L.gensor_avgpool2d.restype = i32
    L.gensor_avgpool2d.argtypes = [i32, i32, i64, i64, i64, i64, i64, i64, vp, vp, vp]
    return L


lib = _load()


def status_string(st: int) -> str:
    return lib.gensor_status_string(int(st)).decode()


def _check(st: int, where: str):
    if st != GENSOR_OK:
        raise GensorError(st, where)


def gemm_problem(dtype: str, M: int, N: int, K: int, transA: int = 0, transB: int = 0, batch: int = 1,
                 out_dtype: str = "f32") -> Problem:
    p = Problem()
    p.op = OP_BMM if batch > 1 else OP_GEMM
    p.in_dtype, p.out_dtype = DTYPE[dtype], DTYPE[out_dtype]
    p.transA, p.transB = transA, transB
    p.batch, p.M, p.N, p.K = batch, M, N, K
    return p


def conv_problem(dtype: str, n, c, h, w, k, r, s, stride, pad, out_dtype: str = "f32") -> Problem:
    p = Problem()
    p.op = OP_CONV2D
    p.in_dtype, p.out_dtype = DTYPE[dtype], DTYPE[out_dtype]
    p.n, p.c, p.h, p.w, p.k, p.r, p.s, p.stride, p.pad = n, c, h, w, k, r, s, stride, pad
    return p


def num_instances() -> int:
    return int(lib.gensor_num_instances())


def instance_schedule(idx: int, p: Problem) -> Optional[Schedule]:
    """Schedule describing compiled instance `idx`, or None if it does not serve `p`."""
    s = Schedule()
    st = lib.gensor_instance_schedule(idx, C.byref(p), C.byref(s))
    if st == 2:
        return None
    _check(st, "gensor_instance_schedule")
    return s


def hw_mi355x() -> Hw:
    return lib.gensor_hw_mi355x().contents


def construct(p: Problem, seed: int = 0, opts: Optional[ConstructOpts] = None, hw: Optional[Hw] = None) -> Schedule:
    s = Schedule()
    st = lib.gensor_construct(C.byref(p), C.byref(hw) if hw is not None else None,
                              C.byref(opts) if opts is not None else None, seed, C.byref(s))
    _check(st, "gensor_construct")
    return s


def construct_trace(p: Problem, seed: int = 0, opts: Optional[ConstructOpts] = None, hw: Optional[Hw] = None,
                    capacity: int = 4096):
    """One walk: returns (actions, dims, states) as int32 arrays, states of shape [steps][12]."""
    steps = C.c_int32(0)
    actions = np.zeros(capacity, dtype=np.int32)
    dims = np.zeros(capacity, dtype=np.int32)
    states = np.zeros((capacity, 12), dtype=np.int32)
    ip = C.POINTER(C.c_int32)
    st = lib.gensor_construct_trace(C.byref(p), C.byref(hw) if hw is not None else None,
                                    C.byref(opts) if opts is not None else None, seed, capacity, C.byref(steps),
                                    actions.ctypes.data_as(ip), dims.ctypes.data_as(ip), states.ctypes.data_as(ip))
    _check(st, "gensor_construct_trace")
    n = steps.value
    return actions[:n], dims[:n], states[:n]


def predict_us(s: Schedule, p: Problem, hw: Optional[Hw] = None) -> float:
    return float(lib.gensor_predict_us(C.byref(s), C.byref(p), C.byref(hw) if hw is not None else None))


def _stream_ptr(stream=None):
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(st.cuda_stream)


def _sref(s):
    return C.byref(s) if s is not None else None


def _ws(workspace):
    if workspace is None:
        return None, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def gemm(p: Problem, A, B, Cout, alpha: float = 1.0, beta: float = 0.0, schedule: Optional[Schedule] = None,
         lda: Optional[int] = None, ldb: Optional[int] = None, ldc: Optional[int] = None, stream=None, workspace=None):
    """C = alpha op(A) op(B) + beta C on device tensors (2-D, row-major with unit inner stride).
    `workspace`: device tensor of at least workspace_bytes(p, schedule) bytes for a split-k schedule (or None)."""
    ws_ptr, ws_len = _ws(workspace)
    st = lib.gensor_gemm(_sref(schedule), C.byref(p), alpha, A.data_ptr(), lda if lda is not None else A.stride(0),
                         B.data_ptr(), ldb if ldb is not None else B.stride(0), beta,
                         Cout.data_ptr(), ldc if ldc is not None else Cout.stride(0), ws_ptr, ws_len, _stream_ptr(stream))
    _check(st, "gensor_gemm")


STATIC_SCRATCH_BYTES = 32 * 1024 * 1024 + 65536


def gemm_static_scratch(p: Problem, A, B, Cout, alpha: float = 1.0, beta: float = 0.0, schedule: Optional[Schedule] = None,
                        stream=None):
    """gemm() with the split-k workspace taken from the library's own device array (nothing is allocated)."""
    st = lib.gensor_gemm_static_scratch(_sref(schedule), C.byref(p), alpha, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0),
                                        beta, Cout.data_ptr(), Cout.stride(0), _stream_ptr(stream))
    _check(st, "gensor_gemm_static_scratch")


def bmm(p: Problem, A, B, Cout, alpha: float = 1.0, beta: float = 0.0, schedule: Optional[Schedule] = None,
        stream=None, workspace=None):
    """Batched: 3-D device tensors [batch][rows][cols]."""
    ws_ptr, ws_len = _ws(workspace)
    st = lib.gensor_bmm(_sref(schedule), C.byref(p), alpha, A.data_ptr(), A.stride(1), A.stride(0),
                        B.data_ptr(), B.stride(1), B.stride(0), beta,
                        Cout.data_ptr(), Cout.stride(1), Cout.stride(0), ws_ptr, ws_len, _stream_ptr(stream))
    _check(st, "gensor_bmm")


def workspace_bytes(p: Problem, schedule: Optional[Schedule] = None) -> int:
    return int(lib.gensor_workspace_bytes(_sref(schedule), C.byref(p)))


def conv2d(p: Problem, I, W, O, schedule: Optional[Schedule] = None, workspace=None, stream=None):
    """O = conv(I, W): contiguous NCHW input, KCRS filters, NKPQ output, all on the device.
    `workspace` is a device tensor of at least workspace_bytes(p, schedule) bytes (or None)."""
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = lib.gensor_conv2d(_sref(schedule), C.byref(p), I.data_ptr(), W.data_ptr(), O.data_ptr(), ws_ptr, ws_len,
                           _stream_ptr(stream))
    _check(st, "gensor_conv2d")


# ---- device memory helpers (plumbing): stored bits <-> torch tensors
def to_device(arr: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def gemv(dtype: str, A, x, y, alpha: float = 1.0, beta: float = 0.0, lda: Optional[int] = None, stream=None):
    """y = alpha A x + beta y: A [M][N] row-major and x [N] of `dtype`, y [M] fp32, all on the device."""
    M, N = A.shape
    st = lib.gensor_gemv(DTYPE[dtype], M, N, alpha, A.data_ptr(), lda if lda is not None else A.stride(0), x.data_ptr(),
                         beta, y.data_ptr(), _stream_ptr(stream))
    _check(st, "gensor_gemv")


def avgpool2d(dtype: str, I, O, f: int, stride: int, out_dtype: str = "f32", stream=None):
    """O = f x f average pooling at `stride` of a contiguous NCHW device tensor."""
    n, c, h, w = I.shape
    st = lib.gensor_avgpool2d(DTYPE[dtype], DTYPE[out_dtype], n, c, h, w, f, stride, I.data_ptr(), O.data_ptr(),
                              _stream_ptr(stream))
    _check(st, "gensor_avgpool2d")


def gemm_workspace(p: Problem, schedule: Schedule):
    """Device buffer for gensor_gemm / gensor_bmm on `p` with a split-k `schedule`, or None if it needs none (plumbing)."""
    import torch
    n = workspace_bytes(p, schedule)
    return torch.empty(n, dtype=torch.uint8, device="cuda") if n else None


def conv_workspace(p: Problem, schedule: Optional[Schedule] = None):
    """Device buffer large enough for gensor_conv2d on `p` with `schedule` (plumbing)."""
    import torch
    return torch.empty(max(16, workspace_bytes(p, schedule)), dtype=torch.uint8, device="cuda")


def empty_device(shape, dtype: str = "f32"):
    import torch
    td = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]
    return torch.empty(shape, dtype=td, device="cuda")


def to_host_f64(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float64).cpu().numpy()
