// Host-side declarations shared by the operator entry points and the constructor.
#pragma once
#include <stdint.h>

#include "../../include/gensor.h"
#include "registry.hpp"

namespace gensor {

// GEMM view of a problem: C[M][N] += A[M][K] * B[K][N] per batch.
struct GemmView {
  int64_t M, N, K, batch;
  int64_t P, Q;          // convolution output extent
  int in_dtype, out_dtype, esize, osize;
  int bsrc;              // BSrc
  // convolution geometry (zero otherwise)
  int64_t cn, cc, ch, cw, cr, cs, cstride, cpad;
};

// LDS plan of a patch-staged convolution instance for one problem.
struct ConvPlan {
  int a_pitch, patch_rows, stage_bytes;
  int64_t in_bytes, w_bytes, out_bytes;
};
// False if instance d (a patch-staged convolution) cannot run the convolution in v.
bool conv_patch_plan(const InstanceDesc& d, const GemmView& v, ConvPlan* plan);

gensor_status gemm_view(const gensor_problem* p, GemmView* v);
void schedule_from_instance(const InstanceDesc& d, gensor_schedule* s);
bool instance_serves(const InstanceDesc& d, const GemmView& v);
const InstanceDesc* find_instance(const gensor_schedule* s, const GemmView& v);

// gensor_construct with two more inputs: whether the operands allow 16-byte vector accesses
// and whether the caller supplied the workspace that patch-staged convolutions need.
gensor_status construct_internal(const gensor_problem* p, const gensor_hw* hw, const gensor_construct_opts* opts,
                                 uint64_t seed, bool vec_ok, bool ws_ok, gensor_schedule* out);

}  // namespace gensor
