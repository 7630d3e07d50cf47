// Table of the ahead-of-time compiled kernel instances: the finite part of the schedule
// lattice that exists as machine code.  Each entry is one point (tiles, virtual threads,
// staging mode, vector width) for one element type and operand source.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

#include "conv_kernel.hpp"
#include "gemm_kernel.hpp"

namespace gensor {

struct InstanceDesc {
  int id;
  int in_dtype, out_dtype;              // gensor_dtype values
  int bm, bn, bk, wm, wn, mb, vm, vn;
  int bsrc;                             // BSrc
  int asrc;                             // ASrc
  int vec, stages, direct;
  int lds_bytes, threads, kg;           // kg: k consumed per fragment read (lds_bytes 0: set per problem)
  int units;                            // patch-staged convolution: transpose units per thread
  hipError_t (*launch)(const KernelArgs&, hipStream_t);
  hipError_t (*launch_split)(const KernelArgs&, hipStream_t);   // the same instance with split tiles; null if not compiled
};

extern const InstanceDesc g_instances[];
extern const int g_num_instances;

// The dynamic-LDS limit of a kernel is a per-device attribute: set it once on every device
// the instance is launched on (one bit per device ordinal; thread-safe, setting twice is harmless).
template <typename K>
hipError_t allow_dynamic_lds(K kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return e;
  done.fetch_or(bit, std::memory_order_release);
  return hipSuccess;
}

template <typename C, bool SPLIT = false>
hipError_t launch_instance(const KernelArgs& a, hipStream_t st) {
  static std::atomic<uint64_t> done{0};
  hipError_t e = allow_dynamic_lds(contraction_kernel<C, SPLIT>, C::LDS_BYTES, done);
  if (e != hipSuccess) return e;
  // one workgroup per whole tile and, in a split launch, a.split per tile behind them
  const unsigned tiles = (unsigned)a.tiles_m * (unsigned)a.tiles_n * (unsigned)a.batch;
  const unsigned grid = SPLIT ? (unsigned)a.whole + (tiles - (unsigned)a.whole) * (unsigned)a.split : tiles;
  hipLaunchKernelGGL((contraction_kernel<C, SPLIT>), dim3(grid), dim3(C::THREADS), C::LDS_BYTES, st, a);
  return hipGetLastError();
}

// patch-staged convolution: the LDS size depends on the problem (a.cStageBytes per LDS stage
// plus, unless the filter is 1x1 or 3x3, one raw filter region of BM * R*S*BKC elements).
template <typename C, int FMODE, bool THROUGH, bool TAIL>
hipError_t launch_conv_tail(const KernelArgs& a, hipStream_t st, int raw_bytes) {
  static std::atomic<uint64_t> done{0};
  hipError_t e = allow_dynamic_lds(conv_patch_kernel<C, FMODE, THROUGH, TAIL>, 160 * 1024, done);
  if (e != hipSuccess) return e;
  const unsigned grid = (unsigned)a.tiles_m * (unsigned)a.tiles_n;
  hipLaunchKernelGGL((conv_patch_kernel<C, FMODE, THROUGH, TAIL>), dim3(grid), dim3(C::THREADS), C::LSTAGES * a.cStageBytes + raw_bytes, st, a);
  return hipGetLastError();
}

// The element-wise fetch of the input tensor's last vector is compiled only into the launches that can need it:
// 16-bit elements and an odd row length (any other vector that runs past the end starts on a dword boundary and
// the buffer's range check returns its valid part).
template <typename C, int FMODE, bool THROUGH>
hipError_t launch_conv_route(const KernelArgs& a, hipStream_t st, int raw_bytes) {
  return ((a.cW * C::ES) & 3) != 0 ? launch_conv_tail<C, FMODE, THROUGH, true>(a, st, raw_bytes)
                                   : launch_conv_tail<C, FMODE, THROUGH, false>(a, st, raw_bytes);
}

// The output is stored write-through when the reduction is shallow (the stores are then a large share of
// the launch), write-back otherwise.
template <typename C, bool THROUGH>
hipError_t launch_conv_policy(const KernelArgs& a, hipStream_t st) {
  const int rs = a.cR * a.cS;
  if (rs == 9) return launch_conv_route<C, 2, THROUGH>(a, st, 0);       // 3x3 and 1x1 reorder their filters in registers
  if (rs == 1) return launch_conv_route<C, 1, THROUGH>(a, st, 0);
  return launch_conv_route<C, 0, THROUGH>(a, st, C::BM * rs * C::BKC * C::ES);      // the others through a raw LDS region
}

template <typename C>
hipError_t launch_conv_instance(const KernelArgs& a, hipStream_t st) {
  return a.K <= 1024 ? launch_conv_policy<C, true>(a, st) : launch_conv_policy<C, false>(a, st);
}

}  // namespace gensor
