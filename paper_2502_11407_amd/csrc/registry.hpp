// Table of the ahead-of-time compiled kernel instances: the finite part of the schedule
// lattice that exists as machine code.  Each entry is one point (tiles, virtual threads,
// staging mode, vector width) for one element type and operand source.
#pragma once
#include <hip/hip_runtime.h>
#include "conv_kernel.hpp"
#include "gemm_kernel.hpp"

namespace gensor {

struct InstanceDesc {
  int id;
  int in_dtype, out_dtype;              // gensor_dtype values
  int bm, bn, bk, wm, wn, mb, vm, vn;
  int bsrc;                             // BSrc
  int vec, stages, direct;
  int lds_bytes, threads, kg;           // kg: k consumed per fragment read (lds_bytes 0: set per problem)
  int units;                            // patch-staged convolution: transpose units per thread
  hipError_t (*launch)(const KernelArgs&, hipStream_t);
};

extern const InstanceDesc g_instances[];
extern const int g_num_instances;

template <typename C>
hipError_t launch_instance(const KernelArgs& a, hipStream_t st) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)contraction_kernel<C>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const unsigned grid = (unsigned)a.tiles_m * (unsigned)a.tiles_n * (unsigned)a.batch;
  hipLaunchKernelGGL(contraction_kernel<C>, dim3(grid), dim3(C::THREADS), C::LDS_BYTES, st, a);
  return hipGetLastError();
}

// patch-staged convolution: the LDS size depends on the problem (a.cStageBytes per LDS stage
// plus, unless the filter is 1x1 or 3x3, one raw filter region of BM * R*S*BKC elements).
template <typename C>
hipError_t launch_conv_instance(const KernelArgs& a, hipStream_t st) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)conv_patch_kernel<C>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const unsigned grid = (unsigned)a.tiles_m * (unsigned)a.tiles_n;
  const int rs = a.cR * a.cS;
  const int raw_bytes = (rs == 1 || rs == 9) ? 0 : C::BM * rs * C::BKC * C::ES;   // those two reorder without it
  hipLaunchKernelGGL(conv_patch_kernel<C>, dim3(grid), dim3(C::THREADS), C::LSTAGES * a.cStageBytes + raw_bytes, st, a);
  return hipGetLastError();
}

}  // namespace gensor
