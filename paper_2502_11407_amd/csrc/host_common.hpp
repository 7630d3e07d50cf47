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
  int asrc;              // ASrc: A stored [m][k] (A_KC) or [k][m] (A_MC, transA)
  int pointwise;         // convolution with a 1x1 filter and no padding, viewed as one GEMM per image
  // convolution geometry (zero otherwise)
  int64_t cn, cc, ch, cw, cr, cs, cstride, cpad;
};

// LDS plan of a patch-staged convolution instance for one problem.
struct ConvPlan {
  int a_pitch, patch_rows, stage_bytes, tile_px;
  int64_t in_bytes, w_bytes, out_bytes;
};
// Output pixels per workgroup of a patch-staged instance with a pixel tile of bn.  When output rows are
// shorter than the tile, a workgroup takes a whole number of them (its patch then has no partial rows):
// as many as fit, or fewer when that deals the tiles more evenly over `cus` compute units.  A tile's
// time is taken as 0.55 of a full tile's (MFMA work, filters, set-up: they do not shrink with the pixels)
// plus 0.45 in proportion to its pixels (patch loads, stores).
inline int64_t conv_tile_px(int64_t bn, int64_t N, int64_t Q, int64_t tiles_m, int64_t cus) {
  if (Q > bn) return bn;
  auto cost = [&](int64_t px) {
    const int64_t tiles = (N + px - 1) / px * tiles_m;
    return (double)((tiles + cus - 1) / cus) * (0.55 * (double)bn + 0.45 * (double)px);
  };
  int64_t best = bn / Q * Q;
  for (int64_t r = bn / Q - 1; r >= 1; --r)
    if (cost(r * Q) < cost(best)) best = r * Q;
  return best;
}
// False if instance d (a patch-staged convolution) cannot run the convolution in v.  round_units: the
// compute units the tiles are dealt over (0: the MI355X's).
bool conv_patch_plan(const InstanceDesc& d, const GemmView& v, ConvPlan* plan, int round_units = 0);

// A pointwise convolution (1x1 filter, no padding) is O[img] = W[k][c] * X[img][c][P*Q] with
// X the input sampled at the stride: a batched GEMM over the images with an n-contiguous B.
// VIEW_DEFAULT takes that view; with stride 2 and rows of whole 16-byte vectors the kernel
// samples the input while fetching it (B_NCS2), any other stride > 1 needs the input compacted
// into the workspace first (B_NC).  VIEW_PREPASS always compacts; VIEW_GENERAL gives the
// general implicit-GEMM view.  The three agree for every other operator.
enum ViewMode { VIEW_GENERAL = 0, VIEW_DEFAULT = 1, VIEW_PREPASS = 2 };
gensor_status gemm_view(const gensor_problem* p, GemmView* v, int mode = VIEW_DEFAULT);
void schedule_from_instance(const InstanceDesc& d, gensor_schedule* s);
bool instance_serves(const InstanceDesc& d, const GemmView& v);
const InstanceDesc* find_instance(const gensor_schedule* s, const GemmView& v);

// Workgroups and workspace of a split-k launch.
struct SplitPlan {
  int split;               // parts per split tile (1: nothing is split)
  int64_t whole;           // tiles computed by one workgroup each
  int64_t counter_bytes;   // arrival counters at the start of the workspace, padded to 256 bytes
  size_t bytes;            // counters + partial tiles
};
// round_units: the compute units a round of tiles is dealt over (gensor_schedule::round_units; 0: the MI355X's).
SplitPlan split_plan(const InstanceDesc& d, const GemmView& v, int split, int round_units);
bool split_allowed(const InstanceDesc& d, const GemmView& v, int split);

// gensor_construct with two more inputs: whether the operands allow 16-byte vector accesses
// and the view (ViewMode) a pointwise convolution is taken in.
gensor_status construct_internal(const gensor_problem* p, const gensor_hw* hw, const gensor_construct_opts* opts,
                                 uint64_t seed, bool vec_ok, int view_mode, gensor_schedule* out);

}  // namespace gensor
