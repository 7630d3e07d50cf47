// The two memory-bound operators of the paper's benchmark: GEMV and AvgPooling2d (operator
// table, GEMV and AvgPooling2d rows).  Neither is a contraction worth a matrix core: both
// stream their input once from HBM, so the kernels are plain coalesced vector loads, fp32
// arithmetic on the vector ALUs and one store per output.
#include <hip/hip_runtime.h>

#include "../../include/gensor.h"
#include "gemm_kernel.hpp"

namespace gensor {

// 16 bytes of stored elements -> fp32 values
template <typename T>
__device__ inline void unpack_chunk(const u32x4& v, float* f) {
  if constexpr (ElemSize<T>::value == 4) {
#pragma unroll
    for (int e = 0; e < 4; ++e) f[e] = as_f32(v[e]);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint16_t bits = (uint16_t)(v[e >> 1] >> ((e & 1) * 16));
      f[e] = to_float<T>(&bits, 0);
    }
  }
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// ---------------------------------------------------------------------------------------
// GEMV, y_i = alpha * sum_n A_in x_n + beta * y_i.  A workgroup of 4 waves owns 8 rows (two
// per wave, so every x vector read from LDS is used twice); x is staged through LDS in
// panels of PANEL elements; a lane reads 16-byte vectors of its rows, UNROLL of them in
// flight per row.  The last partial vector of a row (N not a multiple of the vector) is
// read element by element.  Needs A and x 16-byte aligned and lda a whole number of vectors.
// ---------------------------------------------------------------------------------------
constexpr int GEMV_PANEL_BYTES = 32768;

// STREAM: the rows of A are read with the non-temporal hint.  A matrix larger than the 256 MiB Infinity
// Cache only evicts itself from it (16384^2 fp16, 512 MiB: 98.7 -> 89.4 us with the hint); one that fits is
// served from it on repeated calls and loses that with the hint (16384 x 8192: 41.8 -> 45.6 us), so the
// launch sets it by the size of A.
template <bool STREAM>
__device__ inline u32x4 load_row_vector(const char* p) {
  if constexpr (STREAM) return __builtin_nontemporal_load((const u32x4*)p);
  else return *(const u32x4*)p;
}

template <typename T, bool STREAM>
__global__ __launch_bounds__(256) void gemv_vec_kernel(const char* A, int64_t lda, const char* x, float* y, int M, int N,
                                                       float alpha, float beta) {
  constexpr int ES = ElemSize<T>::value, EPC = 16 / ES, PANEL = GEMV_PANEL_BYTES / ES, UNROLL = 4;
  __shared__ __attribute__((aligned(16))) char xs[GEMV_PANEL_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row0 = blockIdx.x * 8 + wave * 2;
  const bool ok0 = row0 < M, ok1 = row0 + 1 < M;
  const char* a0 = A + (int64_t)(ok0 ? row0 : 0) * lda * ES;
  const char* a1 = A + (int64_t)(ok1 ? row0 + 1 : 0) * lda * ES;
  float acc0 = 0.f, acc1 = 0.f;
  for (int p0 = 0; p0 < N; p0 += PANEL) {
    const int pn = min(PANEL, N - p0);                 // elements of x in this panel
    const int full = pn / EPC;                         // whole vectors
    __syncthreads();                                   // the previous panel has been consumed
    // all of a thread's vectors of the panel are requested before the first is written to LDS
    constexpr int XV = GEMV_PANEL_BYTES / 16 / 256;
    u32x4 xv[XV];
#pragma unroll
    for (int i = 0; i < XV; ++i) {
      const int c = tid + i * 256;
      xv[i] = u32x4{0u, 0u, 0u, 0u};
      if (c < full) {
        xv[i] = *(const u32x4*)(x + ((int64_t)p0 + (int64_t)c * EPC) * ES);
      } else if (c < (pn + EPC - 1) / EPC) {           // ragged end of x: element by element, zero beyond N
        for (int e = 0; e < pn - full * EPC; ++e) {
          if constexpr (ES == 4) xv[i][e] = ((const uint32_t*)x)[p0 + c * EPC + e];
          else xv[i][e >> 1] |= (uint32_t)((const uint16_t*)x)[p0 + c * EPC + e] << ((e & 1) * 16);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < XV; ++i) {
      const int c = tid + i * 256;
      if (c < (pn + EPC - 1) / EPC) *(u32x4*)(xs + c * 16) = xv[i];
    }
    __syncthreads();
    int c = lane;
    for (; c + (UNROLL - 1) * 64 < full; c += UNROLL * 64) {
      u32x4 va[UNROLL], vb[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const int64_t off = ((int64_t)p0 + (int64_t)(c + u * 64) * EPC) * ES;
        va[u] = load_row_vector<STREAM>(a0 + off);
        vb[u] = load_row_vector<STREAM>(a1 + off);
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        float fx[EPC], fa[EPC], fb[EPC];
        unpack_chunk<T>(*(const u32x4*)(xs + (c + u * 64) * 16), fx);
        unpack_chunk<T>(va[u], fa);
        unpack_chunk<T>(vb[u], fb);
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
          acc0 = fmaf(fa[e], fx[e], acc0);
          acc1 = fmaf(fb[e], fx[e], acc1);
        }
      }
    }
    for (; c < full; c += 64) {
      const int64_t off = ((int64_t)p0 + (int64_t)c * EPC) * ES;
      float fx[EPC], fa[EPC], fb[EPC];
      unpack_chunk<T>(*(const u32x4*)(xs + c * 16), fx);
      unpack_chunk<T>(*(const u32x4*)(a0 + off), fa);
      unpack_chunk<T>(*(const u32x4*)(a1 + off), fb);
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        acc0 = fmaf(fa[e], fx[e], acc0);
        acc1 = fmaf(fb[e], fx[e], acc1);
      }
    }
    // ragged end of the rows: lane e takes element e of the partial vector
    const int rem = pn - full * EPC;
    if (lane < rem) {
      const int64_t i = (int64_t)p0 + (int64_t)full * EPC + lane;
      const float xv = to_float<T>(xs, full * EPC + lane);
      acc0 = fmaf(to_float<T>(a0, i), xv, acc0);
      acc1 = fmaf(to_float<T>(a1, i), xv, acc1);
    }
  }
  acc0 = wave_sum(acc0);
  acc1 = wave_sum(acc1);
  if (lane == 0) {
    if (ok0) y[row0] = alpha * acc0 + (beta != 0.f ? beta * y[row0] : 0.f);
    if (ok1) y[row0 + 1] = alpha * acc1 + (beta != 0.f ? beta * y[row0 + 1] : 0.f);
  }
}

// any alignment: one wave per row, element loads
template <typename T>
__global__ __launch_bounds__(256) void gemv_scalar_kernel(const char* A, int64_t lda, const char* x, float* y, int M, int N,
                                                          float alpha, float beta) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;                                // whole waves leave together; no barrier follows
  float acc = 0.f;
  for (int n = lane; n < N; n += 64) acc = fmaf(to_float<T>(A, (int64_t)row * lda + n), to_float<T>(x, n), acc);
  acc = wave_sum(acc);
  if (lane == 0) y[row] = alpha * acc + (beta != 0.f ? beta * y[row] : 0.f);
}

// ---------------------------------------------------------------------------------------
// AvgPooling2d, O[plane][p][q] = (1/F^2) sum_{i,j<F} I[plane][S p + i][S q + j].  The window
// is summed in fp32 and divided once by F*F.
//
// avgpool_lds_kernel: the input a workgroup needs is one contiguous span of the NCHW tensor
// (whole planes, or the rows under a run of output rows of one plane).  It is brought into
// LDS with aligned 16-byte vector loads (2-byte loads per window element would make the load
// pipeline, not HBM, the limit), and the windows are then read from LDS.
// avgpool_direct_kernel: one thread per output straight from global memory, for inputs that
// are not 16-byte aligned or whose rows do not fit the LDS span.
// ---------------------------------------------------------------------------------------
constexpr int POOL_SPAN_BYTES = 32768;
constexpr int POOL_VECS = (POOL_SPAN_BYTES + 16 + 15) / 16 / 256 + 1;     // 16-byte vectors per thread covering span + skew

template <typename T, typename OutT>
__global__ __launch_bounds__(256) void avgpool_lds_kernel(const char* in, void* out, int64_t in_bytes, int planes, int H, int W, int P,
                                                          int Q, int F, int S, int planes_per_wg, int rows_per_wg, int chunks_per_plane) {
  constexpr int ES = ElemSize<T>::value;
  extern __shared__ __attribute__((aligned(16))) char span[];      // the launch sizes it to this problem's span (+ skew)
  const int tid = threadIdx.x;
  const int group = blockIdx.x / chunks_per_plane, chunk = blockIdx.x - group * chunks_per_plane;
  const int plane0 = group * planes_per_wg;
  const int nplanes = min(planes_per_wg, planes - plane0);
  const int p0 = chunk * rows_per_wg;
  const int nrows = min(rows_per_wg, P - p0);
  // span of input elements [e0, e0 + len)
  const int64_t e0 = ((int64_t)plane0 * H + (int64_t)S * p0) * W;
  const int len = chunks_per_plane == 1 ? nplanes * H * W : ((nrows - 1) * S + F) * W;
  const int64_t b0 = e0 * ES, a0 = b0 & ~(int64_t)15;
  const int skew = (int)(b0 - a0);                            // bytes before the first element in LDS
  const int nvec = (skew + len * ES + 15) / 16;
  // all of a thread's vectors are requested before the first one is written to LDS (one memory
  // round trip per workgroup instead of one per vector); the span holds at most POOL_VECS per thread
  u32x4 d[POOL_VECS];
#pragma unroll
  for (int i = 0; i < POOL_VECS; ++i) {
    const int v = tid + i * 256;
    const int64_t addr = a0 + (int64_t)v * 16;
    d[i] = u32x4{0u, 0u, 0u, 0u};
    if (v < nvec) {
      if (addr + 16 <= in_bytes) {
        d[i] = *(const u32x4*)(in + addr);
      } else {                                                // last vector of the tensor: element by element
        for (int e = 0; e < 16 / ES; ++e) {
          if (addr + (e + 1) * ES <= in_bytes) {
            if constexpr (ES == 4) d[i][e] = *(const uint32_t*)(in + addr + e * 4);
            else d[i][e >> 1] |= (uint32_t)*(const uint16_t*)(in + addr + e * 2) << ((e & 1) * 16);
          }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < POOL_VECS; ++i) {
    const int v = tid + i * 256;
    if (v < nvec) *(u32x4*)(span + v * 16) = d[i];
  }
  __syncthreads();
  const int per_plane = nrows * Q;
  const int total = nplanes * per_plane;
  const float count = (float)(F * F);
  // thread t takes outputs t, t + 256, ...; (plane, row, column) advance incrementally
  int g = tid / per_plane, pr, q;
  {
    const int r = tid - g * per_plane;
    pr = r / Q;
    q = r - pr * Q;
  }
  const int dq = 256 % Q, dp = 256 / Q;
  for (int t = tid; t < total; t += 256) {
    const int base = (g * H + S * pr) * W + S * q;            // element offset inside the span
    float acc = 0.f;
    for (int i = 0; i < F; ++i)
      for (int j = 0; j < F; ++j) acc += to_float<T>(span + skew, base + i * W + j);
    store_out<OutT>(out, ((int64_t)(plane0 + g) * P + p0 + pr) * Q + q, acc / count);
    q += dq;
    pr += dp;
    if (q >= Q) { q -= Q; ++pr; }
    while (pr >= nrows) { pr -= nrows; ++g; }
  }
}

template <typename T, typename OutT>
__global__ __launch_bounds__(256) void avgpool_direct_kernel(const void* in, void* out, int64_t total, int H, int W, int P, int Q, int F,
                                                             int S) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int64_t t = idx / Q;
  const int q = (int)(idx - t * Q);
  const int64_t plane = t / P;
  const int p = (int)(t - plane * P);
  const int64_t base = (plane * H + (int64_t)S * p) * W + (int64_t)S * q;
  float acc = 0.f;
  for (int i = 0; i < F; ++i)
    for (int j = 0; j < F; ++j) acc += to_float<T>(in, base + (int64_t)i * W + j);
  store_out<OutT>(out, idx, acc / (float)(F * F));
}

template <typename T>
hipError_t launch_gemv(const void* A, int64_t lda, const void* x, float* y, int64_t M, int64_t N, float alpha, float beta, hipStream_t st) {
  constexpr int ES = ElemSize<T>::value, EPC = 16 / ES;
  const bool vec = ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(x)) & 15u) == 0 && lda % EPC == 0;
  const bool stream = M * lda * ES > (int64_t)256 * 1024 * 1024;      // larger than the Infinity Cache
  if (vec && stream)
    hipLaunchKernelGGL((gemv_vec_kernel<T, true>), dim3((unsigned)((M + 7) / 8)), dim3(256), 0, st, (const char*)A, lda, (const char*)x, y,
                       (int)M, (int)N, alpha, beta);
  else if (vec)
    hipLaunchKernelGGL((gemv_vec_kernel<T, false>), dim3((unsigned)((M + 7) / 8)), dim3(256), 0, st, (const char*)A, lda, (const char*)x, y,
                       (int)M, (int)N, alpha, beta);
  else
    hipLaunchKernelGGL(gemv_scalar_kernel<T>, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, (const char*)A, lda, (const char*)x, y,
                       (int)M, (int)N, alpha, beta);
  return hipGetLastError();
}

template <typename T, typename OutT>
hipError_t launch_pool(const void* in, void* out, int64_t planes, int64_t h, int64_t w, int64_t f, int64_t s, hipStream_t st) {
  constexpr int ES = ElemSize<T>::value;
  const int64_t P = (h - f) / s + 1, Q = (w - f) / s + 1;
  const int64_t plane_bytes = h * w * ES, row_bytes = w * ES;
  const bool aligned = (reinterpret_cast<uintptr_t>(in) & 15u) == 0;
  int64_t G = 0, R = 0, cpp = 0;
  if (aligned && plane_bytes <= POOL_SPAN_BYTES) {             // whole planes per workgroup
    G = POOL_SPAN_BYTES / plane_bytes;
    const int64_t cap = (8192 + P * Q - 1) / (P * Q);          // keep a workgroup to a few thousand outputs
    if (G > cap) G = cap;
    // enough workgroups to keep every CU's resident set (LDS is sized to the span) turning over several times
    const int64_t spread = planes / (256 * 8 * 4);
    if (G > spread) G = spread > 1 ? spread : 1;
    if (G > planes) G = planes;
    R = P;
    cpp = 1;
  } else if (aligned && f * row_bytes <= POOL_SPAN_BYTES) {    // runs of output rows of one plane
    G = 1;
    R = (POOL_SPAN_BYTES / row_bytes - f) / s + 1;
    if (R > P) R = P;
    cpp = (P + R - 1) / R;
  }
  const int64_t groups = G ? (planes + G - 1) / G * cpp : 0;
  if (G && groups <= INT32_MAX && planes <= INT32_MAX) {
    const int64_t span_elems = cpp == 1 ? G * h * w : ((R - 1) * s + f) * w;
    const size_t lds_bytes = (size_t)((span_elems * ES + 15 + 15) / 16 * 16 + 16);      // span + skew, whole vectors
    hipLaunchKernelGGL((avgpool_lds_kernel<T, OutT>), dim3((unsigned)groups), dim3(256), lds_bytes, st, (const char*)in, out,
                       planes * plane_bytes, (int)planes, (int)h, (int)w, (int)P, (int)Q, (int)f, (int)s, (int)G, (int)R, (int)cpp);
  } else {
    const int64_t total = planes * P * Q;
    hipLaunchKernelGGL((avgpool_direct_kernel<T, OutT>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, in, out, total, (int)h,
                       (int)w, (int)P, (int)Q, (int)f, (int)s);
  }
  return hipGetLastError();
}

}  // namespace gensor

using namespace gensor;

extern "C" gensor_status gensor_gemv(gensor_dtype in_dtype, int64_t M, int64_t N, float alpha, const void* A, int64_t lda,
                                     const void* x, float beta, float* y, void* hip_stream) {
  if (!A || !x || !y || M <= 0 || N <= 0 || lda < N) return GENSOR_ERR_INVALID_ARG;
  if (M > INT32_MAX - 8 || N > INT32_MAX - GEMV_PANEL_BYTES) return GENSOR_ERR_UNSUPPORTED;
  hipError_t e;
  switch (in_dtype) {
    case GENSOR_F32: e = launch_gemv<f32_t>(A, lda, x, y, M, N, alpha, beta, (hipStream_t)hip_stream); break;
    case GENSOR_F16: e = launch_gemv<f16_t>(A, lda, x, y, M, N, alpha, beta, (hipStream_t)hip_stream); break;
    case GENSOR_BF16: e = launch_gemv<bf16_t>(A, lda, x, y, M, N, alpha, beta, (hipStream_t)hip_stream); break;
    default: return GENSOR_ERR_INVALID_ARG;
  }
  return e == hipSuccess ? GENSOR_OK : GENSOR_ERR_DEVICE;
}

extern "C" gensor_status gensor_avgpool2d(gensor_dtype in_dtype, gensor_dtype out_dtype, int64_t n, int64_t c, int64_t h, int64_t w,
                                          int64_t f, int64_t stride, const void* input, void* output, void* hip_stream) {
  if (!input || !output || n <= 0 || c <= 0 || h <= 0 || w <= 0 || f <= 0 || stride <= 0 || f > h || f > w) return GENSOR_ERR_INVALID_ARG;
  if (in_dtype != GENSOR_F32 && in_dtype != GENSOR_F16 && in_dtype != GENSOR_BF16) return GENSOR_ERR_INVALID_ARG;
  if (out_dtype != GENSOR_F32 && out_dtype != in_dtype) return GENSOR_ERR_UNSUPPORTED;
  const int64_t P = (h - f) / stride + 1, Q = (w - f) / stride + 1;
  if (h > INT32_MAX || w > INT32_MAX || f > 4096 || (n * c * P * Q + 255) / 256 > INT32_MAX) return GENSOR_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)hip_stream;
  const int64_t planes = n * c;
  hipError_t e;
  if (in_dtype == GENSOR_F32) e = launch_pool<f32_t, f32_t>(input, output, planes, h, w, f, stride, st);
  else if (in_dtype == GENSOR_F16)
    e = out_dtype == GENSOR_F32 ? launch_pool<f16_t, f32_t>(input, output, planes, h, w, f, stride, st)
                                : launch_pool<f16_t, f16_t>(input, output, planes, h, w, f, stride, st);
  else
    e = out_dtype == GENSOR_F32 ? launch_pool<bf16_t, f32_t>(input, output, planes, h, w, f, stride, st)
                                : launch_pool<bf16_t, bf16_t>(input, output, planes, h, w, f, stride, st);
  return e == hipSuccess ? GENSOR_OK : GENSOR_ERR_DEVICE;
}
