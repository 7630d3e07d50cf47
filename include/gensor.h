/*
 * gensor.h -- C ABI of the MI355X (gfx950) scheduled dense operators and of the
 * schedule constructor.
 *
 * The operators are the ones the paper's construction compiler schedules (operator
 * table: GEMM and Conv2d rows; batched matmul is GEMM repeated over a batch axis).
 * A *schedule* is one node of the paper's construction graph (Section IV-A): per-level
 * tile sizes D = [T_2, T_1, T_0] for every loop dimension, the virtual-thread split, and
 * the primitives derived from it (LDS caching mode, unroll, vector width).  It selects
 * one ahead-of-time compiled kernel instance.  gensor_construct() walks the graph
 * (Algorithms 1 and 2, benefit formulas Eq. 1-3) and returns the schedule that an
 * analytical MI355X cost model ranks best.
 *
 * Conventions common to every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates or frees device memory and keeps no pointer after it returns.
 *   - Operators are enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and return without synchronising.
 *   - Errors are return codes; nothing aborts and nothing is launched on error.
 *   - Matrices are dense, addressed by a leading dimension counted in elements.
 *   - Accumulation is always fp32.  alpha and beta are fp32.  beta == 0 never reads C.
 */
#ifndef GENSOR_H
#define GENSOR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GENSOR_OK = 0,
  GENSOR_ERR_INVALID_ARG = 1,  /* null pointer, non-positive extent, leading dimension too small, bad enum */
  GENSOR_ERR_UNSUPPORTED = 2,  /* legal request that no compiled kernel instance covers */
  GENSOR_ERR_NO_SCHEDULE = 3,  /* schedule does not fit the problem / fails the capacity check */
  GENSOR_ERR_WORKSPACE = 4,    /* workspace smaller than gensor_workspace_bytes() */
  GENSOR_ERR_DEVICE = 5        /* HIP reported an error on launch */
} gensor_status;

typedef enum { GENSOR_F32 = 0, GENSOR_F16 = 1, GENSOR_BF16 = 2 } gensor_dtype;
typedef enum { GENSOR_OP_GEMM = 0, GENSOR_OP_BMM = 1, GENSOR_OP_CONV2D = 2 } gensor_op;

/* The "op, tensor_shape" input of Algorithm 1. */
typedef struct {
  int32_t op;                 /* gensor_op */
  int32_t in_dtype;           /* gensor_dtype of A and B (input and filters) */
  int32_t out_dtype;          /* gensor_dtype of C (output): F32, or the same as in_dtype */
  int32_t transA;             /* GEMM/BMM: 0 = A stored [M][K], 1 = A stored [K][M] */
  int32_t transB;             /* GEMM/BMM: 0 = B stored [K][N], 1 = B stored [N][K] (column-major B) */
  int64_t batch, M, N, K;     /* GEMM: batch = 1.  C is [M][N] per batch. */
  int64_t n, c, h, w;         /* Conv2d input  I[n][c][h][w]  (NCHW) */
  int64_t k, r, s;            /* Conv2d filter W[k][c][r][s]  (KCRS) */
  int64_t stride, pad;        /* same stride and symmetric zero padding in both directions */
} gensor_problem;

enum { GENSOR_DIM_M = 0, GENSOR_DIM_N = 1, GENSOR_DIM_K = 2 };
#define GENSOR_SCHEDULE_VERSION 1

/*
 * One state of the construction graph (Section IV-A, IV-C), plain data, no pointers.
 * Loop dimensions are those of the GEMM view: m, n (spatial) and k (reduction); for
 * Conv2d m = filters k, n = (image, out row, out col), k = (channel, filter row, filter col).
 * tile[d][0] = T_2: workgroup tile staged in LDS       (BM, BN, BK)
 * tile[d][1] = T_1: wavefront tile held in registers   (WM, WN, and the MFMA k depth)
 * tile[d][2] = T_0: extent per virtual thread = tile[d][1] / vthread[d]
 * vthread[d]: virtual threads of Section IV-A / Eq. 3 on this hardware: the rows that one quarter
 *   wave reads together from the LDS tile of the m (A) or n (B) operand are interleaved over
 *   vthread[d] bank phases.  1 is the plain layout, whose reads conflict ceil(x / W) ways
 *   (x = bytes of bank address space those rows span, W = 256 bytes served per cycle); at
 *   vthread[d] = ceil(x / W) they are conflict-free, and that is the largest value on the lattice.
 */
typedef struct {
  int32_t version;            /* GENSOR_SCHEDULE_VERSION */
  int32_t kernel_id;          /* index of the compiled instance; filled by gensor_construct */
  int32_t tile[3][3];
  int32_t vthread[2];         /* V for m and n: interleave depth of that operand's LDS tile (see above) */
  int32_t stages;             /* LDS buffers: 1, 2, or a ring of 3 (two k tiles in flight) */
  int32_t unroll;             /* MFMA k-steps unrolled per LDS stage = BK / (k per fragment) */
  int32_t vec_bytes;          /* width of one global access: 16, or the element size (scalar path) */
  int32_t direct_lds;         /* 1: global->LDS loads bypass registers */
  int32_t split_k;            /* 1..16 workgroups per tile of the last, partly filled round (GEMM/BMM; see gensor_gemm) */
  int32_t wg_remap;           /* tile rows per panel in the workgroup->tile map (L2 reuse per XCD) */
  double predicted_us;        /* cost-model time of this schedule for the problem */
  double construct_s;         /* wall time gensor_construct spent */
  int32_t iterations;         /* walk steps per chain */
  int32_t chains;             /* independent walks */
  int32_t states_scored;      /* complete states handed to the cost model */
  int32_t round_units;        /* compute units a round of tiles is dealt over when split_k > 1: those of the hw the
                                 schedule was constructed for (0: gensor_hw_mi355x()->compute_units) */
  uint64_t seed;
} gensor_schedule;

/*
 * Hardware description that every benefit formula and the capacity check read
 * (Section III: peak compute, memory hierarchy, parallelism features).
 * Level 0 = HBM/global, level 1 = LDS, level 2 = registers.
 */
typedef struct {
  int32_t compute_units;        /* 256 */
  int32_t simds_per_cu;         /* 4 */
  int32_t wave_size;            /* 64 */
  int32_t max_waves_per_wg;     /* 16 */
  int32_t lds_bytes_per_cu;     /* 163840 */
  int32_t regs_per_lane;        /* 512 32-bit registers per lane (VGPR + AccVGPR) for one wave per SIMD */
  int32_t lds_banks;            /* 64 */
  int32_t lds_bank_bytes;       /* 4 */
  double clock_ghz;             /* 2.4 */
  double latency_ns[3];         /* L of Eq. 2 per level */
  double bandwidth_gbs[3];      /* B of Eq. 2 per level, whole chip */
  double l2_bandwidth_gbs;      /* aggregate L2 -> CU bandwidth (cost model only) */
  double mfma_tflops_16bit;     /* dense fp16/bf16 MFMA peak, 2516.6 */
  double mfma_tflops_f32;       /* fp32 MFMA peak, 157.3 */
  double launch_us;             /* fixed cost of one kernel launch (cost model only) */
} gensor_hw;

/* Static MI355X description; never NULL. */
const gensor_hw* gensor_hw_mi355x(void);

/* Walk parameters (inputs "T, threshold" of Algorithm 1 plus this build's knobs).
 * Zero in any field selects its default. */
typedef struct {
  double T0;                  /* initial (and per-level restart) temperature, default 2^30 */
  double threshold;           /* stop when T <= threshold, default 2^-70 (100 steps, Section IV-D) */
  int32_t chains;             /* independent seeded walks, default 16384 (about 30 ms of construction) */
  int32_t keep_policy;        /* 0: keep every complete state; 1: the paper's printed keep probability */
  int32_t tiling_benefit;     /* 0: Eq. 1 as printed; 1: footprint ratio inverted (ablation) */
  int32_t no_vthread;         /* 1: setVThread disabled (ablation) */
  int32_t no_split_k;         /* 1: only split_k = 1 is ranked (callers without a workspace) */
  int32_t greedy;             /* 1: every step takes the action of largest benefit instead of drawing one
                                 (a tree-like, single-path construction; ablation) */
} gensor_construct_opts;

/*
 * Algorithm 1 / Algorithm 2 on the host.  Pure function of (problem, hw, opts, seed).
 * hw == NULL selects gensor_hw_mi355x(); opts == NULL selects the defaults.
 * Returns GENSOR_ERR_NO_SCHEDULE if no complete state maps to a compiled instance.
 */
gensor_status gensor_construct(const gensor_problem* p, const gensor_hw* hw,
                               const gensor_construct_opts* opts, uint64_t seed,
                               gensor_schedule* out);

/*
 * Trace of ONE walk, for checking the walk against an independent implementation.
 * Writes, per step i < *steps_out: actions[i] (0 tile, 1 invTile, 2 setVThread, 3 cache),
 * dims[i] (dimension index, -1 for cache) and states[i][12] = tile[3][3], vthread[2],
 * current level after the step.  `capacity` is the room in the three arrays (steps).
 */
gensor_status gensor_construct_trace(const gensor_problem* p, const gensor_hw* hw,
                                     const gensor_construct_opts* opts, uint64_t seed,
                                     int32_t capacity, int32_t* steps_out,
                                     int32_t* actions, int32_t* dims, int32_t* states);

/* Cost-model time in microseconds of `s` on `p`; negative if `s` is infeasible. */
double gensor_predict_us(const gensor_schedule* s, const gensor_problem* p, const gensor_hw* hw);

/* Number of compiled kernel instances, and the schedule that describes instance `id`
 * for a problem of the given op / dtypes / layout (GENSOR_ERR_UNSUPPORTED if it does
 * not serve that problem). */
int32_t gensor_num_instances(void);
gensor_status gensor_instance_schedule(int32_t id, const gensor_problem* p, gensor_schedule* out);

/*
 * C = alpha * op(A) * op(B) + beta * C          (operator table, GEMM row)
 * A, B: in_dtype, C: out_dtype, row-major with leading dimensions lda, ldb, ldc in
 * elements (lda >= K, or M if transA: A is then stored [K][M]; ldb >= N, or K if transB: B stored
 * [N][K]; ldc >= N).
 * s == NULL: a schedule is constructed for `p` (seed 0) and remembered per shape.
 *
 * Split-k (s->split_k > 1).  Tiles are dealt to the compute units in rounds of
 * s->round_units.  The tiles of the last round, if it is not full (every
 * tile when there are fewer tiles than units), are each computed by split_k workgroups,
 * every one over its own range of whole k tiles (needs ceil(K / BK) >= split_k, else
 * NO_SCHEDULE); the parts of a tile leave fp32 partial tiles in `workspace` and the part
 * that finishes last adds them up (two parts: one order of addition; more: in part order,
 * so the result is reproducible) and writes C.  This is what a contraction with few output
 * tiles and a deep k needs to occupy the chip.  `workspace` is device memory, 256-byte
 * aligned, at least gensor_workspace_bytes(s, p) bytes (WORKSPACE otherwise): arrival
 * counters, which the call clears itself with a small launch of its own in front of the
 * operator, then the partial tiles.  It is scratch: nothing is kept in it between calls, and
 * two calls that overlap in time must not share it.  If the tile count is a whole number of
 * rounds nothing is split and no workspace is needed (gensor_workspace_bytes returns 0).
 * With s == NULL split-k schedules are ranked only when a workspace is passed, and one too
 * small for the ranking's choice selects the best unsplit schedule instead.
 * Schedules with split_k == 1 use no workspace (pass NULL, 0).
 */
gensor_status gensor_gemm(const gensor_schedule* s, const gensor_problem* p, float alpha,
                          const void* A, int64_t lda, const void* B, int64_t ldb,
                          float beta, void* C, int64_t ldc,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * gensor_gemm for callers that cannot allocate device memory for a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same operator, the same
 * kernels and the same results, with the split-k counters and partial tiles kept in a device array
 * of GENSOR_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the library
 * runs on holds its own copy until the process ends).  The call allocates and frees nothing.
 * A schedule whose gensor_workspace_bytes(s, p) exceeds GENSOR_STATIC_SCRATCH_BYTES is refused with
 * GENSOR_ERR_WORKSPACE and nothing is launched; with s == NULL split-k schedules are ranked and one
 * that does not fit falls back to the best unsplit schedule, as in gensor_gemm.  Every call on one
 * GPU shares that GPU's array, which keeps the last call's contents (the call clears the counters it
 * uses itself): calls that overlap in time on one GPU -- different streams, or graphs replayed
 * concurrently -- race on it and must be serialised by the caller.
 */
#define GENSOR_STATIC_SCRATCH_BYTES (32 * 1024 * 1024 + 65536)
gensor_status gensor_gemm_static_scratch(const gensor_schedule* s, const gensor_problem* p, float alpha,
                                         const void* A, int64_t lda, const void* B, int64_t ldb,
                                         float beta, void* C, int64_t ldc, void* hip_stream);

/* The same for every b < p->batch; consecutive matrices are stride{A,B,C} elements
 * apart (a stride of 0 broadcasts that operand). */
gensor_status gensor_bmm(const gensor_schedule* s, const gensor_problem* p, float alpha,
                         const void* A, int64_t lda, int64_t strideA,
                         const void* B, int64_t ldb, int64_t strideB,
                         float beta, void* C, int64_t ldc, int64_t strideC,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * O[n][k][p][q] = sum_{c,r,s} I[n][c][p*stride-pad+r][q*stride-pad+s] * W[k][c][r][s]
 * (operator table, Conv2d row: O = (I * K) downsampled by S; cross-correlation, zero
 * padding; P = floor((h + 2 pad - r)/stride) + 1, Q likewise).  All three tensors are
 * contiguous.  Computed as an implicit GEMM: no im2col buffer is materialised.
 * Schedules that cache the input patch in LDS (direct_lds = 1) and the element-gather
 * schedules use no workspace.
 * A pointwise convolution (r = s = 1, pad = 0) is one GEMM per image, O[n] = W * X[n] with
 * X[n][c][p*Q+q] = I[n][c][p*stride][q*stride]; gensor_construct and
 * gensor_instance_schedule treat it as that batched GEMM (m = k filters, n = P*Q, k = c).
 * With stride 1 the input itself is the B operand; with a larger stride the call first
 * compacts the sampled input into `workspace` (device memory, 16-byte aligned, at least
 * gensor_workspace_bytes(s, p) = n*c*P*Q elements; GENSOR_ERR_WORKSPACE otherwise; with
 * s == NULL and no such workspace the general implicit-GEMM path is used).  Stride 2 on rows
 * of whole 16-byte vectors is sampled while the operand is fetched and needs none.
 * The workspace is scratch: its contents after the call are unspecified and nothing is
 * kept in it between calls.
 */
gensor_status gensor_conv2d(const gensor_schedule* s, const gensor_problem* p,
                            const void* input, const void* weight, void* output,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of workspace the operator call on `p` with schedule `s` needs: the compacted input of a
 * strided pointwise convolution, or the counters and partial tiles of a split-k GEMM/BMM
 * (s required); 0 if none.  For a convolution s == NULL gives the most any schedule the
 * library may construct can ask for. */
size_t gensor_workspace_bytes(const gensor_schedule* s, const gensor_problem* p);

/*
 * y[i] = alpha * sum_{n<N} A[i][n] * x[n] + beta * y[i], i < M   (operator table, GEMV row).
 * A is row-major [M][lda] (lda >= N, in elements) and x has N elements, both of in_dtype on
 * the device; y is fp32 on the device and is read only if beta != 0.  Products and sums are
 * carried in fp32.  A memory-bound streaming kernel with a fixed internal schedule (no
 * gensor_schedule): 16-byte vector loads when A and x are 16-byte aligned and lda is a whole
 * number of vectors, element loads otherwise.  Enqueued on hip_stream; nothing is allocated.
 * INVALID_ARG for null pointers, non-positive extents or lda < N.
 */
gensor_status gensor_gemv(gensor_dtype in_dtype, int64_t M, int64_t N, float alpha,
                          const void* A, int64_t lda, const void* x, float beta, float* y,
                          void* hip_stream);

/*
 * O[n][c][p][q] = (1 / f^2) * sum_{i<f} sum_{j<f} I[n][c][stride*p + i][stride*q + j]
 * (operator table, AvgPooling2d row) on a contiguous NCHW input, no padding;
 * P = floor((h - f)/stride) + 1, Q likewise.  The window is summed in fp32 and divided once.
 * out_dtype is GENSOR_F32 or in_dtype (round to nearest even).  Memory-bound streaming
 * kernel, fixed internal schedule, enqueued on hip_stream, nothing allocated.
 * INVALID_ARG for null pointers, non-positive extents or f larger than the image.
 */
gensor_status gensor_avgpool2d(gensor_dtype in_dtype, gensor_dtype out_dtype,
                               int64_t n, int64_t c, int64_t h, int64_t w, int64_t f, int64_t stride,
                               const void* input, void* output, void* hip_stream);

const char* gensor_status_string(gensor_status st);

#ifdef __cplusplus
}
#endif
#endif /* GENSOR_H */
