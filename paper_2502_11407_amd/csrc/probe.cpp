// MFMA-only probe kernel: the matrix-core rate the chip sustains for given operand values.
#include <hip/hip_runtime.h>

#include "../../include/gensor.h"
#include "gemm_kernel.hpp"

namespace gensor {

template <typename T>
__global__ __launch_bounds__(256) void mfma_probe_kernel(const u32x4* operands, float* sink, int iters) {
  typedef Mfma<T, 32> MF;
  typedef typename MF::Acc Acc;
  u32x4 a[4], b[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    a[s] = operands[(threadIdx.x * 4 + s) * 2];
    b[s] = operands[(threadIdx.x * 4 + s) * 2 + 1];
  }
  Acc c[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < MF::NACC; ++v) c[i][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) MF::run(a[i % 4], b[(i / 2) % 4], c[i]);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < MF::NACC; ++v) sum += c[i][v];
  sink[blockIdx.x * 256 + threadIdx.x] = sum;
}

}  // namespace gensor

extern "C" gensor_status gensor_mfma_probe(gensor_dtype in_dtype, const void* operands, float* sink,
                                           int32_t iters, void* hip_stream) {
  using namespace gensor;
  if (!operands || !sink || iters <= 0 || (reinterpret_cast<uintptr_t>(operands) & 15u)) return GENSOR_ERR_INVALID_ARG;
  const int cus = gensor_hw_mi355x()->compute_units;
  if (in_dtype == GENSOR_F16)
    hipLaunchKernelGGL(mfma_probe_kernel<f16_t>, dim3(cus), dim3(256), 0, (hipStream_t)hip_stream, (const u32x4*)operands, sink, iters);
  else if (in_dtype == GENSOR_BF16)
    hipLaunchKernelGGL(mfma_probe_kernel<bf16_t>, dim3(cus), dim3(256), 0, (hipStream_t)hip_stream, (const u32x4*)operands, sink, iters);
  else
    return GENSOR_ERR_UNSUPPORTED;
  return hipGetLastError() == hipSuccess ? GENSOR_OK : GENSOR_ERR_DEVICE;
}
