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

// patch-staged convolution: the LDS size depends on the problem (a.cStageBytes per LDS stage).
// a.A is the caller's KCRS filter tensor and a.cWorkspace receives its K,R,S,C copy.
template <typename C>
hipError_t launch_conv_instance(const KernelArgs& a0, hipStream_t st) {
  KernelArgs a = a0;
  {
    const int64_t total = (int64_t)a.M * a.cC * a.cR * a.cS;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(permute_filters<C::ES>, dim3(blocks), dim3(256), 0, st, a.A, a.cWorkspace, a.M, a.cC, a.cR * a.cS);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    a.A = a.cWorkspace;
  }
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)conv_patch_kernel<C>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const unsigned grid = (unsigned)a.tiles_m * (unsigned)a.tiles_n;
  hipLaunchKernelGGL(conv_patch_kernel<C>, dim3(grid), dim3(C::THREADS), C::LSTAGES * a.cStageBytes, st, a);
  return hipGetLastError();
}

}  // namespace gensor
