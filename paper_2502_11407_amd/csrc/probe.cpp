// MFMA-only probe kernel: the matrix-core rate the chip sustains for given operand values.
// A measurement aid for the benchmark, built into a library of its own (libgensor_probe.so); it is
// not part of the operator library or of its header.
//
//   int gensor_probe_mfma(int in_dtype, const void* operands, float* sink, int iters, int workgroups, void* hip_stream)
//
// launches `workgroups` workgroups of 4 wavefronts, each wavefront running `iters` rounds of 8
// independent 32x32x16 MFMAs on A and B fragments loaded once from `operands` (device memory,
// 256 KiB, 16-byte aligned; the caller chooses the values).  `sink` (device, workgroups * 256
// floats) receives one value per lane so the work cannot be dropped.  in_dtype: 1 fp16, 2 bf16.
// Returns 0, 1 (bad argument), 2 (unsupported type) or 5 (launch error).  Flop count of one
// launch: workgroups * 4 * iters * 8 * 2 * 32 * 32 * 16.
#include <hip/hip_runtime.h>

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

extern "C" int gensor_probe_mfma(int in_dtype, const void* operands, float* sink, int iters, int workgroups,
                                 void* hip_stream) {
  using namespace gensor;
  if (!operands || !sink || iters <= 0 || workgroups <= 0 || (reinterpret_cast<uintptr_t>(operands) & 15u)) return 1;
  if (in_dtype == 1)
    hipLaunchKernelGGL(mfma_probe_kernel<f16_t>, dim3(workgroups), dim3(256), 0, (hipStream_t)hip_stream, (const u32x4*)operands, sink, iters);
  else if (in_dtype == 2)
    hipLaunchKernelGGL(mfma_probe_kernel<bf16_t>, dim3(workgroups), dim3(256), 0, (hipStream_t)hip_stream, (const u32x4*)operands, sink, iters);
  else
    return 2;
  return hipGetLastError() == hipSuccess ? 0 : 5;
}
