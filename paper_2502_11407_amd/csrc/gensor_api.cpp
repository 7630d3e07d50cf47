// C ABI of the operators: argument validation, GEMM view of each operator, lookup of the
// kernel instance a schedule names, and the launch.  No device memory is allocated here.
#include <hip/hip_runtime.h>

#include <cstring>
#include <map>
#include <mutex>
#include <tuple>

#include "../../include/gensor.h"
#include "host_common.hpp"
#include "registry.hpp"

using namespace gensor;

extern "C" const char* gensor_status_string(gensor_status st) {
  switch (st) {
    case GENSOR_OK: return "ok";
    case GENSOR_ERR_INVALID_ARG: return "invalid argument";
    case GENSOR_ERR_UNSUPPORTED: return "unsupported combination";
    case GENSOR_ERR_NO_SCHEDULE: return "no feasible schedule / schedule does not match a compiled instance";
    case GENSOR_ERR_WORKSPACE: return "workspace too small";
    case GENSOR_ERR_DEVICE: return "HIP launch error";
  }
  return "unknown status";
}

extern "C" int32_t gensor_num_instances(void) { return g_num_instances; }

namespace gensor {

static bool valid_dtype(int d) { return d == GENSOR_F32 || d == GENSOR_F16 || d == GENSOR_BF16; }

gensor_status gemm_view(const gensor_problem* p, GemmView* v, int mode) {
  if (!p || !v) return GENSOR_ERR_INVALID_ARG;
  if (!valid_dtype(p->in_dtype) || !valid_dtype(p->out_dtype)) return GENSOR_ERR_INVALID_ARG;
  if (p->out_dtype != GENSOR_F32 && p->out_dtype != p->in_dtype) return GENSOR_ERR_UNSUPPORTED;
  std::memset(v, 0, sizeof(*v));
  v->in_dtype = p->in_dtype;
  v->out_dtype = p->out_dtype;
  v->esize = p->in_dtype == GENSOR_F32 ? 4 : 2;
  v->osize = p->out_dtype == GENSOR_F32 ? 4 : 2;
  if (p->op == GENSOR_OP_GEMM || p->op == GENSOR_OP_BMM) {
    if (p->M <= 0 || p->N <= 0 || p->K <= 0) return GENSOR_ERR_INVALID_ARG;
    if (p->op == GENSOR_OP_BMM && p->batch <= 0) return GENSOR_ERR_INVALID_ARG;
    if ((p->transA != 0 && p->transA != 1) || (p->transB != 0 && p->transB != 1)) return GENSOR_ERR_INVALID_ARG;
    v->M = p->M; v->N = p->N; v->K = p->K;
    v->batch = p->op == GENSOR_OP_BMM ? p->batch : 1;
    v->bsrc = p->transB ? B_KC : B_NC;
    v->asrc = p->transA ? A_MC : A_KC;
  } else if (p->op == GENSOR_OP_CONV2D) {
    if (p->n <= 0 || p->c <= 0 || p->h <= 0 || p->w <= 0 || p->k <= 0 || p->r <= 0 || p->s <= 0) return GENSOR_ERR_INVALID_ARG;
    if (p->stride <= 0 || p->pad < 0) return GENSOR_ERR_INVALID_ARG;
    if (p->h + 2 * p->pad < p->r || p->w + 2 * p->pad < p->s) return GENSOR_ERR_INVALID_ARG;
    v->P = (p->h + 2 * p->pad - p->r) / p->stride + 1;
    v->Q = (p->w + 2 * p->pad - p->s) / p->stride + 1;
    v->M = p->k;
    v->N = p->n * v->P * v->Q;
    v->K = p->c * p->r * p->s;
    v->batch = 1;
    v->bsrc = B_CONV;
    v->cn = p->n; v->cc = p->c; v->ch = p->h; v->cw = p->w; v->cr = p->r; v->cs = p->s;
    v->cstride = p->stride; v->cpad = p->pad;
    if (mode != VIEW_GENERAL && p->r == 1 && p->s == 1 && p->pad == 0) {
      v->pointwise = 1;
      v->N = v->P * v->Q;
      v->K = p->c;
      v->batch = p->n;
      // stride 2 on rows that are whole 16-byte vectors: sampled while fetched, no pre-pass
      v->bsrc = (mode == VIEW_DEFAULT && p->stride == 2 && p->w % (16 / v->esize) == 0) ? B_NCS2 : B_NC;
    }
  } else {
    return GENSOR_ERR_INVALID_ARG;
  }
  if (v->M > INT32_MAX || v->N > INT32_MAX || v->K > INT32_MAX || v->batch > INT32_MAX) return GENSOR_ERR_UNSUPPORTED;
  return GENSOR_OK;
}

void schedule_from_instance(const InstanceDesc& d, gensor_schedule* s) {
  std::memset(s, 0, sizeof(*s));
  s->version = GENSOR_SCHEDULE_VERSION;
  s->kernel_id = d.id;
  s->tile[GENSOR_DIM_M][0] = d.bm; s->tile[GENSOR_DIM_N][0] = d.bn; s->tile[GENSOR_DIM_K][0] = d.bk;
  s->tile[GENSOR_DIM_M][1] = d.wm; s->tile[GENSOR_DIM_N][1] = d.wn; s->tile[GENSOR_DIM_K][1] = d.kg;
  s->vthread[0] = d.vm; s->vthread[1] = d.vn;
  s->tile[GENSOR_DIM_M][2] = d.wm / d.vm; s->tile[GENSOR_DIM_N][2] = d.wn / d.vn; s->tile[GENSOR_DIM_K][2] = d.kg;
  s->stages = d.stages;
  s->unroll = d.bk / d.kg;
  s->vec_bytes = d.vec ? 16 : (d.in_dtype == GENSOR_F32 ? 4 : 2);
  s->direct_lds = d.direct;
  s->split_k = 1;
  s->wg_remap = 4;
}

bool conv_patch_plan(const InstanceDesc& d, const GemmView& v, ConvPlan* plan, int round_units) {
  const int64_t lim = 0x7fffffffll;
  const int epc = 16 / v.esize;
  const int64_t rs = v.cr * v.cs;
  if (rs > 9 || v.cc % epc != 0) return false;
  ConvPlan pl;
  pl.in_bytes = v.cn * v.cc * v.ch * v.cw * v.esize;
  pl.w_bytes = v.M * v.K * v.esize;
  pl.out_bytes = v.M * v.N * v.osize;
  if (pl.in_bytes >= lim || pl.w_bytes >= lim || pl.out_bytes >= lim) return false;
  // filter tile: [bm][rs * bkc] with a row pitch of an odd number of 16-byte chunks
  int64_t p16 = rs * d.bk * v.esize / 16;
  if (p16 % 2 == 0) ++p16;
  pl.a_pitch = (int)(p16 * 16);
  if ((int64_t)d.bm * pl.a_pitch >= (1 << 20)) return false;
  // patch rows: the most stacked padded input rows any pixel tile touches
  const int64_t hp = v.ch + 2 * v.cpad, pw = v.cw + 2 * v.cpad;
  const int64_t cus = round_units > 0 ? round_units : gensor_hw_mi355x()->compute_units;
  const int64_t px = conv_tile_px(d.bn, v.N, v.Q, (v.M + d.bm - 1) / d.bm, cus);
  pl.tile_px = (int)px;
  int64_t rows = 0;
  for (int64_t n0 = 0; n0 < v.N; n0 += px) {
    const int64_t n1 = (n0 + px < v.N ? n0 + px : v.N) - 1;
    const int64_t g0 = n0 / v.Q, g1 = n1 / v.Q;
    const int64_t r0 = (g0 / v.P) * hp + (g0 % v.P) * v.cstride;
    const int64_t r1 = (g1 / v.P) * hp + (g1 % v.P) * v.cstride + v.cr - 1;
    if (r1 - r0 + 1 > rows) rows = r1 - r0 + 1;
  }
  pl.patch_rows = (int)rows;
  const int slot = d.bk * v.esize + 16;
  const int64_t stage = (int64_t)d.bm * pl.a_pitch + rows * pw * slot;
  const int64_t raw = (rs == 1 || rs == 9) ? 0 : (int64_t)d.bm * rs * d.bk * v.esize;      // raw filter runs, one buffer
  if (d.stages * stage + raw > 160 * 1024) return false;
  pl.stage_bytes = (int)stage;
  const int64_t units = rows * ((v.cw + epc - 1) / epc) * (d.bk / epc);
  if (units > (int64_t)d.units * d.threads) return false;
  if (plan) *plan = pl;
  return true;
}

bool instance_serves(const InstanceDesc& d, const GemmView& v) {
  if (d.in_dtype != v.in_dtype || d.out_dtype != v.out_dtype || d.bsrc != v.bsrc || d.asrc != v.asrc) return false;
  if (d.units) return conv_patch_plan(d, v, nullptr);
  return true;
}

// Does instance d realise schedule s (same lattice point)?
static bool instance_matches(const InstanceDesc& d, const gensor_schedule* s) {
  return d.bm == s->tile[0][0] && d.bn == s->tile[1][0] && d.bk == s->tile[2][0] && d.wm == s->tile[0][1] &&
         d.wn == s->tile[1][1] && d.kg == s->tile[2][1] && d.vm == s->vthread[0] && d.vn == s->vthread[1] &&
         d.stages == s->stages && d.direct == s->direct_lds && (d.vec ? 16 : -1) == (s->vec_bytes == 16 ? 16 : -1);
}

const InstanceDesc* find_instance(const gensor_schedule* s, const GemmView& v) {
  if (!s || s->version != GENSOR_SCHEDULE_VERSION) return nullptr;
  if (s->kernel_id >= 0 && s->kernel_id < g_num_instances) {
    const InstanceDesc& d = g_instances[s->kernel_id];
    if (instance_serves(d, v) && instance_matches(d, s)) return &d;
  }
  for (int i = 0; i < g_num_instances; ++i)
    if (instance_serves(g_instances[i], v) && instance_matches(g_instances[i], s)) return &g_instances[i];
  return nullptr;
}

// Can the 16-byte vector path be used?  (k-contiguous operands need K and their leading
// dimension to be whole chunks; the n-contiguous operand needs N and ldb to be.)
bool vector_ok(const GemmView& v, const void* A, int64_t lda, int64_t strideA, const void* B, int64_t ldb, int64_t strideB) {
  const int epc = 16 / v.esize;
  auto al = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  if (!al(A) || lda % epc || strideA % epc || (v.asrc == A_KC ? v.K : v.M) % epc) return false;
  if (v.asrc == A_MC && v.bsrc == B_KC && v.K % epc) return false;
  if (v.bsrc == B_KC) return al(B) && ldb % epc == 0 && strideB % epc == 0;
  if (v.bsrc == B_NC || v.bsrc == B_NCS2) return al(B) && ldb % epc == 0 && strideB % epc == 0 && v.N % epc == 0;
  return al(B);  // convolution: the gather is element-wise; the patch path reads 16-byte vectors
}

}  // namespace gensor

extern "C" gensor_status gensor_instance_schedule(int32_t id, const gensor_problem* p, gensor_schedule* out) {
  if (!p || !out || id < 0 || id >= g_num_instances) return GENSOR_ERR_INVALID_ARG;
  GemmView v;
  gensor_status st = gemm_view(p, &v);
  if (st != GENSOR_OK) return st;
  if (!instance_serves(g_instances[id], v)) return GENSOR_ERR_UNSUPPORTED;
  schedule_from_instance(g_instances[id], out);
  return GENSOR_OK;
}

namespace gensor {
// Bytes of the compacted input of a strided pointwise convolution (0: the input is used as it is).
static size_t pointwise_workspace(const GemmView& v) {
  return v.pointwise && v.cstride > 1 && v.bsrc != B_NCS2 ? (size_t)(v.batch * v.K * v.N * v.esize) : 0;
}

// Split-k plan of instance d on view v with split factor `split`: the tiles that do not fill a whole
// round of compute units (all of them when there are fewer tiles than units) are computed by `split`
// workgroups each.  whole = tiles left unsplit; a plan with whole == tiles splits nothing.
SplitPlan split_plan(const InstanceDesc& d, const GemmView& v, int split, int round_units) {
  SplitPlan pl;
  const int64_t tiles = ((v.M + d.bm - 1) / d.bm) * ((v.N + d.bn - 1) / d.bn) * v.batch;
  const int64_t cus = round_units > 0 ? round_units : gensor_hw_mi355x()->compute_units;
  pl.whole = split > 1 ? tiles / cus * cus : tiles;
  pl.split = pl.whole == tiles ? 1 : split;
  const int64_t waves = d.threads / 64;
  pl.counter_bytes = pl.split > 1 ? ((tiles - pl.whole) * waves * 4 + 255) / 256 * 256 : 0;
  pl.bytes = pl.split > 1 ? (size_t)(pl.counter_bytes + (tiles - pl.whole) * pl.split * (int64_t)d.bm * d.bn * 4) : 0;
  return pl;
}

// Can the instance run a split tile?  It was compiled with the split path (operands fetched plainly, no
// gather, no sampling) and every part gets at least one k tile.
bool split_allowed(const InstanceDesc& d, const GemmView& v, int split) {
  if (split == 1) return true;
  if (split < 1 || split > 16 || !d.launch_split || (v.bsrc != B_KC && v.bsrc != B_NC)) return false;
  return (v.K + d.bk - 1) / d.bk >= split;
}

__global__ void clear_counters(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}
}  // namespace gensor

// Only a strided pointwise convolution run as a batched GEMM through the compaction pre-pass
// needs a workspace (the compacted copy of its input).
extern "C" size_t gensor_workspace_bytes(const gensor_schedule* s, const gensor_problem* p) {
  GemmView v, w;
  if (p && s && (p->op == GENSOR_OP_GEMM || p->op == GENSOR_OP_BMM)) {
    // a split-k schedule: one counter per wave of every split tile, then one fp32 tile per part
    if (s->split_k <= 1 || gemm_view(p, &v) != GENSOR_OK) return 0;
    const InstanceDesc* d = find_instance(s, v);
    return d && split_allowed(*d, v, s->split_k) ? split_plan(*d, v, s->split_k, s->round_units).bytes : 0;
  }
  if (!p || p->op != GENSOR_OP_CONV2D || gemm_view(p, &v) != GENSOR_OK || gemm_view(p, &w, VIEW_PREPASS) != GENSOR_OK) return 0;
  const size_t need_pw = pointwise_workspace(w);
  if (!s) return need_pw;                    // what any schedule the library may construct can ask for
  if (v.pointwise && find_instance(s, v)) return pointwise_workspace(v);
  if (w.pointwise && find_instance(s, w)) return need_pw;
  return 0;
}

// ------------------------------------------------------------------------------------
// schedule == NULL: construct once per (problem, alignment class) and remember it.
// ------------------------------------------------------------------------------------
namespace {
std::mutex g_memo_mutex;
std::map<std::tuple<int, int, int, int, int, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t>, gensor_schedule> g_memo;
const size_t kMemoLimit = 4096;      // shapes remembered; a full memo is emptied (a shape seen again is constructed again)

gensor_status memoised_schedule(const gensor_problem* p, bool vec_ok, int view_mode, bool no_split, gensor_schedule* out) {
  auto key = std::make_tuple((int)p->op, (int)p->in_dtype, (int)p->out_dtype, (int)p->transB + 2 * (int)p->transA,
                             (vec_ok ? 1 : 0) + (no_split ? 2 : 0) + 4 * view_mode,
                             p->op == GENSOR_OP_CONV2D ? p->n : p->batch, p->op == GENSOR_OP_CONV2D ? p->c : p->M,
                             p->op == GENSOR_OP_CONV2D ? p->h : p->N, p->op == GENSOR_OP_CONV2D ? p->w : p->K,
                             p->op == GENSOR_OP_CONV2D ? p->k : 0, p->op == GENSOR_OP_CONV2D ? p->r : 0,
                             p->op == GENSOR_OP_CONV2D ? p->s : 0,
                             p->op == GENSOR_OP_CONV2D ? p->stride : 0, p->op == GENSOR_OP_CONV2D ? p->pad : 0);
  std::lock_guard<std::mutex> lock(g_memo_mutex);
  auto it = g_memo.find(key);
  if (it != g_memo.end()) { *out = it->second; return GENSOR_OK; }
  gensor_construct_opts opts;
  std::memset(&opts, 0, sizeof(opts));
  opts.no_split_k = no_split ? 1 : 0;
  gensor_status st = construct_internal(p, nullptr, &opts, 0, vec_ok, view_mode, out);
  if (st == GENSOR_OK) {
    if (g_memo.size() >= kMemoLimit) g_memo.clear();
    g_memo[key] = *out;
  }
  return st;
}

gensor_status run(const gensor_schedule* s, const gensor_problem* p, const GemmView& v, float alpha,
                  const void* A, int64_t lda, int64_t strideA, const void* B, int64_t ldb, int64_t strideB,
                  float beta, void* C, int64_t ldc, int64_t strideC, void* workspace, size_t workspace_bytes, void* stream) {
  const bool vec_ok = vector_ok(v, A, lda, strideA, B, ldb, strideB);
  const bool ws_aligned = workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u) == 0;
  gensor_schedule local;
  const bool constructed = !s;
  const int mode = !v.pointwise ? VIEW_GENERAL : (v.cstride > 1 && v.bsrc == B_NC ? VIEW_PREPASS : VIEW_DEFAULT);
  if (!s) {
    // split-k schedules are ranked only for a caller that brought a workspace
    gensor_status st = memoised_schedule(p, vec_ok, mode, !ws_aligned, &local);
    if (st != GENSOR_OK) return st;
    s = &local;
  }
  const InstanceDesc* d = find_instance(s, v);
  if (constructed && d && s->split_k > 1 && workspace_bytes < split_plan(*d, v, s->split_k, s->round_units).bytes) {
    // the workspace is too small for the split the ranking chose: the best unsplit schedule instead
    gensor_status st = memoised_schedule(p, vec_ok, mode, true, &local);
    if (st != GENSOR_OK) return st;
    d = find_instance(s, v);
  }
  if (!d) return GENSOR_ERR_NO_SCHEDULE;
  if (d->vec && !vec_ok) return GENSOR_ERR_NO_SCHEDULE;          // schedule asks for vector accesses the operands cannot give
  if (d->direct && !d->units && v.K % d->bk != 0) return GENSOR_ERR_NO_SCHEDULE;
  if (s->split_k < 1 || !split_allowed(*d, v, s->split_k)) return GENSOR_ERR_NO_SCHEDULE;
  SplitPlan sp = split_plan(*d, v, s->split_k, s->round_units);
  if (sp.split > 1 && (!ws_aligned || workspace_bytes < sp.bytes)) return GENSOR_ERR_WORKSPACE;
  // 32-bit offsets inside one workgroup tile
  const int64_t lim = 0x7fffffffll;
  if (v.asrc == A_KC && (int64_t)(d->bm + 1) * lda * v.esize >= lim) return GENSOR_ERR_UNSUPPORTED;
  if (v.asrc == A_MC && ((int64_t)(d->bk + 1) * lda + d->bm) * v.esize >= lim) return GENSOR_ERR_UNSUPPORTED;
  // (the convolution epilogues address the output with 64-bit indices and never use ldc)
  if (v.bsrc != B_CONV && (int64_t)(d->bm + 1) * ldc * v.osize >= lim) return GENSOR_ERR_UNSUPPORTED;
  if (v.bsrc == B_KC && (int64_t)(d->bn + 1) * ldb * v.esize >= lim) return GENSOR_ERR_UNSUPPORTED;
  if ((v.bsrc == B_NC || v.bsrc == B_NCS2) && ((int64_t)(d->bk + 1) * ldb + d->bn) * v.esize >= lim) return GENSOR_ERR_UNSUPPORTED;

  KernelArgs a;
  std::memset(&a, 0, sizeof(a));
  a.A = A; a.B = B; a.C = C;
  a.M = (int32_t)v.M; a.N = (int32_t)v.N; a.K = (int32_t)v.K;
  a.lda = lda; a.ldb = ldb; a.ldc = ldc;
  a.strideA = strideA; a.strideB = strideB; a.strideC = strideC;
  a.alpha = alpha; a.beta = beta;
  a.tiles_m = (int32_t)((v.M + d->bm - 1) / d->bm);
  a.tiles_n = (int32_t)((v.N + d->bn - 1) / d->bn);
  a.batch = (int32_t)v.batch;
  a.panel = s->wg_remap > 0 ? s->wg_remap : 1;
  if (a.panel > a.tiles_m) a.panel = a.tiles_m;
  if ((int64_t)a.tiles_m * a.tiles_n * a.batch > INT32_MAX) return GENSOR_ERR_UNSUPPORTED;
  a.split = sp.split;
  a.whole = (int32_t)sp.whole;
  if (sp.split > 1) {
    a.counters = (uint32_t*)workspace;
    a.partials = (float*)((char*)workspace + sp.counter_bytes);
    const int n = (int)(sp.counter_bytes / 4);
    hipLaunchKernelGGL(clear_counters, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, a.counters, n);
    if (hipGetLastError() != hipSuccess) return GENSOR_ERR_DEVICE;
  }
  if (d->units) {
    ConvPlan pl;
    if (!conv_patch_plan(*d, v, &pl, s->round_units)) return GENSOR_ERR_NO_SCHEDULE;
    a.cTilePx = pl.tile_px;
    a.tiles_n = (int32_t)((v.N + pl.tile_px - 1) / pl.tile_px);
    if ((int64_t)a.tiles_m * a.tiles_n > INT32_MAX) return GENSOR_ERR_UNSUPPORTED;
    a.cN = (int32_t)p->n; a.cApitch = pl.a_pitch; a.cPatchRows = pl.patch_rows; a.cStageBytes = pl.stage_bytes;
    a.cInBytes = pl.in_bytes; a.cWBytes = pl.w_bytes; a.cOutBytes = pl.out_bytes;
    a.batch = 1;
  }
  if (v.bsrc == B_CONV || v.bsrc == B_NCS2) {
    a.cC = (int32_t)p->c; a.cH = (int32_t)p->h; a.cW = (int32_t)p->w; a.cR = (int32_t)p->r; a.cS = (int32_t)p->s;
    a.cP = (int32_t)v.P; a.cQ = (int32_t)v.Q; a.cStride = (int32_t)p->stride; a.cPad = (int32_t)p->pad;
  }
  hipError_t e = sp.split > 1 ? d->launch_split(a, (hipStream_t)stream) : d->launch(a, (hipStream_t)stream);
  return e == hipSuccess ? GENSOR_OK : GENSOR_ERR_DEVICE;
}
}  // namespace

extern "C" gensor_status gensor_bmm(const gensor_schedule* s, const gensor_problem* p, float alpha,
                                    const void* A, int64_t lda, int64_t strideA,
                                    const void* B, int64_t ldb, int64_t strideB,
                                    float beta, void* C, int64_t ldc, int64_t strideC,
                                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || !A || !B || !C) return GENSOR_ERR_INVALID_ARG;
  if (p->op != GENSOR_OP_GEMM && p->op != GENSOR_OP_BMM) return GENSOR_ERR_INVALID_ARG;
  GemmView v;
  gensor_status st = gemm_view(p, &v);
  if (st != GENSOR_OK) return st;
  if (lda < (v.asrc == A_KC ? v.K : v.M)) return GENSOR_ERR_INVALID_ARG;
  if (ldb < (v.bsrc == B_KC ? v.K : v.N)) return GENSOR_ERR_INVALID_ARG;
  if (ldc < v.N) return GENSOR_ERR_INVALID_ARG;
  if (strideA < 0 || strideB < 0 || strideC < 0) return GENSOR_ERR_INVALID_ARG;
  if (v.batch > 1 && strideC < v.M * ldc - (ldc - v.N)) return GENSOR_ERR_INVALID_ARG;   // outputs must not overlap
  return run(s, p, v, alpha, A, lda, strideA, B, ldb, strideB, beta, C, ldc, strideC, workspace, workspace_bytes, hip_stream);
}

extern "C" gensor_status gensor_gemm(const gensor_schedule* s, const gensor_problem* p, float alpha,
                                     const void* A, int64_t lda, const void* B, int64_t ldb,
                                     float beta, void* C, int64_t ldc,
                                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || p->op != GENSOR_OP_GEMM) return GENSOR_ERR_INVALID_ARG;
  return gensor_bmm(s, p, alpha, A, lda, 0, B, ldb, 0, beta, C, ldc, 0, workspace, workspace_bytes, hip_stream);
}

// ------------------------------------------------------------------------------------
// gensor_gemm for callers that cannot bring a workspace: the split-k counters and partial tiles
// live in a device array that is part of this library's code object.
// ------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[GENSOR_STATIC_SCRATCH_BYTES];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[64];          // per device ordinal: where that device's copy of `scratch` lives

// The address of this device's copy of the array (each device holds its own, at its own address);
// looked up once per device, with that device current.
gensor_status static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return GENSOR_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return GENSOR_ERR_DEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return GENSOR_OK;
}
}  // namespace

extern "C" gensor_status gensor_gemm_static_scratch(const gensor_schedule* s, const gensor_problem* p, float alpha,
                                                    const void* A, int64_t lda, const void* B, int64_t ldb,
                                                    float beta, void* C, int64_t ldc, void* hip_stream) {
  if (!p || p->op != GENSOR_OP_GEMM) return GENSOR_ERR_INVALID_ARG;
  if (s && gensor_workspace_bytes(s, p) > (size_t)GENSOR_STATIC_SCRATCH_BYTES) return GENSOR_ERR_WORKSPACE;
  void* ptr = nullptr;
  gensor_status st = static_scratch(&ptr);
  if (st != GENSOR_OK) return st;
  // from here on the array is a workspace like any other: the counters at its start are cleared by the
  // fill kernel in front of the operator, the partial tiles are written before they are read
  return gensor_bmm(s, p, alpha, A, lda, 0, B, ldb, 0, beta, C, ldc, 0, ptr, (size_t)GENSOR_STATIC_SCRATCH_BYTES, hip_stream);
}

extern "C" gensor_status gensor_conv2d(const gensor_schedule* s, const gensor_problem* p,
                                       const void* input, const void* weight, void* output,
                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || !input || !weight || !output || p->op != GENSOR_OP_CONV2D) return GENSOR_ERR_INVALID_ARG;
  GemmView v;
  gensor_status st = gemm_view(p, &v);
  if (st != GENSOR_OK) return st;
  if (v.pointwise) {
    // one GEMM per image: A = filters [k][c] shared by all images, B = the (sampled) input
    // [c][P*Q] of the image, C = its output [k][P*Q].  Views are tried in order of
    // preference: sampled while fetched (stride 2, no workspace), compacted by a pre-pass
    // (needs the workspace), then the general implicit GEMM.  An explicit schedule selects
    // the view whose instance it names.
    const int64_t PQ = v.N;
    for (int mode = VIEW_DEFAULT; mode <= VIEW_PREPASS; ++mode) {
      GemmView w;
      st = gemm_view(p, &w, mode);
      if (st != GENSOR_OK) return st;
      if (mode == VIEW_PREPASS && w.bsrc == v.bsrc) break;          // the same view again
      const size_t need = pointwise_workspace(w);
      const bool have = need == 0 || (workspace && (reinterpret_cast<uintptr_t>(workspace) & 15u) == 0 && workspace_bytes >= need);
      const int64_t ldb = need ? PQ : p->h * p->w;
      if (s) {
        if (!find_instance(s, w)) continue;
        if (!have) return GENSOR_ERR_WORKSPACE;
      } else {
        if (!have) continue;
        if (w.bsrc == B_NCS2 && !vector_ok(w, weight, w.K, 0, input, ldb, w.K * ldb)) continue;   // sampled instances are vector-only
      }
      const void* X = input;
      if (need) {
        const int64_t planes = p->n * p->c;
        const int epc = 16 / w.esize;
        const int64_t threads = (planes * PQ + epc - 1) / epc;
        if ((threads + 255) / 256 > INT32_MAX) return GENSOR_ERR_UNSUPPORTED;
        const unsigned blocks = (unsigned)((threads + 255) / 256);
        if (w.esize == 4)
          hipLaunchKernelGGL(subsample_input<4>, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, input, workspace, planes,
                             (int)p->h, (int)p->w, (int)w.P, (int)w.Q, (int)p->stride);
        else
          hipLaunchKernelGGL(subsample_input<2>, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, input, workspace, planes,
                             (int)p->h, (int)p->w, (int)w.P, (int)w.Q, (int)p->stride);
        if (hipGetLastError() != hipSuccess) return GENSOR_ERR_DEVICE;
        X = workspace;
      }
      return run(s, p, w, 1.0f, weight, w.K, 0, X, ldb, w.K * ldb, 0.0f, output, PQ, w.M * PQ, nullptr, 0, hip_stream);
    }
    st = gemm_view(p, &v, VIEW_GENERAL);
    if (st != GENSOR_OK) return st;
  }
  // A = filters [k][c*r*s] (k-contiguous), B = gathered input, C = output viewed per image.
  return run(s, p, v, 1.0f, weight, v.K, 0, input, 0, 0, 0.0f, output, v.N, 0, workspace, workspace_bytes, hip_stream);
}
