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
  int pointwise;         // convolution with a 1x1 filter and no padding, viewed as one GEMM per image
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

// A pointwise convolution (1x1 filter, no padding) is O[img] = W[k][c] * X[img][c][P*Q] with
// X the input sampled at the stride: a batched GEMM over the images with an n-contiguous B.
// allow_pointwise = false gives the general implicit-GEMM view of the same problem instead.
gensor_status gemm_view(const gensor_problem* p, GemmView* v, bool allow_pointwise = true);
void schedule_from_instance(const InstanceDesc& d, gensor_schedule* s);
bool instance_serves(const InstanceDesc& d, const GemmView& v);
const InstanceDesc* find_instance(const gensor_schedule* s, const GemmView& v);

// gensor_construct with three more inputs: whether the operands allow 16-byte vector accesses,
// whether the caller supplied the workspace that patch-staged convolutions need, and whether a
// pointwise convolution may take its batched-GEMM view.
gensor_status construct_internal(const gensor_problem* p, const gensor_hw* hw, const gensor_construct_opts* opts,
                                 uint64_t seed, bool vec_ok, bool ws_ok, bool allow_pointwise, gensor_schedule* out);

}  // namespace gensor
