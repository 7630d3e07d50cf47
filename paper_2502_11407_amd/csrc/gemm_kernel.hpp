// Scheduled dense-contraction kernel for gfx950 (CDNA4): one template covers GEMM, batched
// matmul and implicit-GEMM convolution.  Every template parameter is a schedule primitive
// of the construction graph (Section IV-A of the paper: per-level tiles, caching, virtual
// threads; Table I: unroll, vectorise):
//
//   BM,BN,BK   T_2  workgroup tile, staged in LDS                ("cache" primitive)
//   WM,WN      T_1  wavefront tile, fp32 accumulators in registers
//   MB         MFMA block edge (32: 32x32 blocks, 16: 16x16 blocks); fixes the MFMA k depth
//   VM,VN      virtual threads (setVThread, Eq. 3): the rows that one quarter wave reads together
//              from the LDS tile of the m (A) or n (B) operand are interleaved over V bank phases;
//              V = 1 is the plain layout, whose fragment reads conflict ceil(x / W) ways
//   STAGES     LDS buffers (1: single buffer, 2: double buffer, 3 and more: a ring that keeps STAGES-1
//              k tiles in flight; direct staging only)
//   VEC        global accesses are 16-byte vectors (true) or single elements (false)
//   DIRECT     K-contiguous operands go global->LDS without passing through registers
//
// Operand sources.  A (the m x k operand) is k-contiguous, A[m][k] (A_KC), or m-contiguous, A stored
// [k][m] (A_MC, "transA": staged and read exactly like an n-contiguous B, register-staged only).  B is
//   KC   k-contiguous,  B stored [n][k]   (column-major B / "transB")
//   NC   n-contiguous,  B stored [k][n]   (row-major B)
//   CONV n = (image, out row, out col), k = (channel, filter row, filter col): element
//        (k, n) is gathered from the NCHW input, zero outside the image; m = filter.
//
// LDS layouts.  k-contiguous tiles are [rows][BK] in 16-byte chunks; chunk c of row r sits
// at chunk c ^ ((r / rows_per_256B) % V).  The 16 rows that a quarter wave's b128 fragment read
// touches span x = 16 * min(row bytes, 256) bytes, i.e. ceil(x / (V * 256)) of them share each
// bank: with V = chunks per row the read hits 64 distinct banks.  n-contiguous tiles are
// [BK][BN + pad]; their V is the number of k rows that the pad (or, direct-staged, an XOR of the
// column bytes) spreads over different banks: 4 rows are read together by a transposing 16-bit
// read (pad 0 / 32 / 64 bytes for V = 1 / 2 / 4), 2 by a 32-bit one (pad 0 / 32).
//
// MFMA operand convention (per lane l of a 64-wide wave):
//   32x32 blocks: row/col = l % 32, holds the 16-byte chunk  2*kstep + l/32  of that row
//   16x16 blocks: row/col = l % 16, holds the 16-byte chunk  4*kstep + l/16  of that row
// For 16-bit types a chunk is 8 consecutive k and feeds one MFMA; for fp32 a chunk is 4
// consecutive k and feeds 4 MFMAs (element t of the chunk at step t).  The order in which k
// is consumed differs from memory order, identically for both operands.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <stdint.h>

namespace gensor {

// B_NCS2: n-contiguous B whose column n = p*Q + q is read at (2p)*W + 2q of a plane of H*W elements
// (= ldb): the input of a pointwise convolution with stride 2, sampled while it is fetched.
enum BSrc { B_KC = 0, B_NC = 1, B_CONV = 2, B_NCS2 = 3 };
enum ASrc { A_KC = 0, A_MC = 1 };

struct KernelArgs {
  const void* A;
  const void* B;
  void* C;
  int32_t M, N, K;                 // GEMM-view extents
  int64_t lda, ldb, ldc;           // elements
  int64_t strideA, strideB, strideC;
  float alpha, beta;
  int32_t tiles_m, tiles_n, batch;
  int32_t panel;                   // tile rows per panel in the workgroup->tile map
  // split-k: workgroups [0, whole) compute one whole tile each; the tiles behind them are computed by
  // `split` workgroups each, every one over its own range of k tiles (split == 1: whole == all tiles)
  int32_t split, whole;
  float* partials;                 // [tile - whole][split][BM * BN] fp32, lane-major inside a slot
  uint32_t* counters;              // [tile - whole][waves per workgroup], zero at launch
  // convolution geometry (B_CONV only)
  int32_t cC, cH, cW, cR, cS, cP, cQ, cStride, cPad;
  // patch-staged convolution only: images, LDS plan and tensor sizes in bytes (each < 2^31)
  int32_t cN, cApitch, cPatchRows, cStageBytes;
  int32_t cTilePx;                 // output pixels per workgroup (at most BN; whole output rows when they are shorter than BN)
  int64_t cInBytes, cWBytes, cOutBytes;
};

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define GENSOR_LDS __attribute__((address_space(3)))

struct f16_t { typedef _Float16 native; };
struct bf16_t { typedef __bf16 native; };
struct f32_t { typedef float native; };

template <typename T> struct ElemSize { static constexpr int value = 2; };
template <> struct ElemSize<f32_t> { static constexpr int value = 4; };

// ---------------------------------------------------------------- scalar conversions
template <typename T> __device__ inline float to_float(const void* p, int64_t i);
template <> __device__ inline float to_float<f32_t>(const void* p, int64_t i) { return ((const float*)p)[i]; }
template <> __device__ inline float to_float<f16_t>(const void* p, int64_t i) { return (float)((const _Float16*)p)[i]; }
template <> __device__ inline float to_float<bf16_t>(const void* p, int64_t i) {
  return __builtin_bit_cast(float, ((uint32_t)((const uint16_t*)p)[i]) << 16);
}
template <typename T> __device__ inline void store_out(void* p, int64_t i, float v);
template <> __device__ inline void store_out<f32_t>(void* p, int64_t i, float v) { ((float*)p)[i] = v; }
template <> __device__ inline void store_out<f16_t>(void* p, int64_t i, float v) { ((_Float16*)p)[i] = (_Float16)v; }
template <> __device__ inline void store_out<bf16_t>(void* p, int64_t i, float v) {
  uint32_t u = __builtin_bit_cast(uint32_t, v);                 // round to nearest even
  uint32_t r = (u & 0x7fffffffu) > 0x7f800000u ? 0x7fc0u : ((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
  ((uint16_t*)p)[i] = (uint16_t)r;
}

// ---------------------------------------------------------------- MFMA wrappers
// (the bits travel through a by-value argument: a bit cast applied directly to a vector
// element expression reads element 0 whatever the index)
__device__ inline float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ inline uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

template <typename T, int MB> struct Mfma;
template <> struct Mfma<f16_t, 32> {
  typedef f32x16 Acc;
  static constexpr int NACC = 16;
  __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mfma<f16_t, 16> {
  typedef f32x4 Acc;
  static constexpr int NACC = 4;
  __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c) {
    c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mfma<bf16_t, 32> {
  typedef f32x16 Acc;
  static constexpr int NACC = 16;
  __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mfma<bf16_t, 16> {
  typedef f32x4 Acc;
  static constexpr int NACC = 4;
  __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c) {
    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mfma<f32_t, 32> {   // true fp32 multiply-add: 32x32x2 per step, 4 steps per chunk
  typedef f32x16 Acc;
  static constexpr int NACC = 16;
  __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
      c = __builtin_amdgcn_mfma_f32_32x32x2f32(as_f32(a[t]), as_f32(b[t]), c, 0, 0, 0);
  }
};
template <> struct Mfma<f32_t, 16> {   // 16x16x4 per step
  typedef f32x4 Acc;
  static constexpr int NACC = 4;
  __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
      c = __builtin_amdgcn_mfma_f32_16x16x4f32(as_f32(a[t]), as_f32(b[t]), c, 0, 0, 0);
  }
};

// ---------------------------------------------------------------- schedule -> constants
template <typename T_, typename OutT_, int BM_, int BN_, int BK_, int WM_, int WN_, int MB_, int VM_, int VN_,
          int BSRC_, bool VEC_, int STAGES_, bool DIRECT_, int ASRC_ = A_KC>
struct Cfg {
  typedef T_ T;
  typedef OutT_ OutT;
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MB = MB_, VM = VM_, VN = VN_;
  static constexpr int BSRC = BSRC_, STAGES = STAGES_, ASRC = ASRC_;
  static constexpr bool VEC = VEC_, DIRECT = DIRECT_;
  static constexpr int ES = ElemSize<T>::value;
  static constexpr int EPC = 16 / ES;                        // elements per 16-byte chunk
  static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN, WAVES = WAVES_M * WAVES_N;
  static constexpr int THREADS = WAVES * 64;
  static constexpr int MBLK = WM / MB, NBLK = WN / MB;       // MFMA blocks per wave tile
  static constexpr int LANE_GROUPS = 64 / MB;                // 2 (32x32) or 4 (16x16)
  static constexpr int KG = LANE_GROUPS * EPC;               // k consumed per fragment read
  static constexpr int KSTEPS = BK / KG;                     // the "unroll" of the schedule
  // k-contiguous LDS tile: [rows][BK], 16-byte chunks, xor swizzle
  static constexpr int PITCH_K = BK * ES;                    // bytes per row
  static constexpr int CPR = PITCH_K / 16;                   // chunks per row
  static constexpr int RPP = (PITCH_K >= 256) ? 1 : 256 / PITCH_K;   // rows per 256-byte bank period
  // n-contiguous LDS tile: [BK][BN] + pad
  // (direct staging deposits whole 1 KB runs, so there the rows are unpadded and 32-byte
  // column segments are XOR-swizzled with the k row instead)
  static constexpr bool NC_DIRECT = DIRECT_ && BSRC_ == B_NC;
  static constexpr int V_MAX_K = CPR;                        // deepest interleave of a k-contiguous tile
  static constexpr int V_MAX_N = (ES == 2) ? 4 : 2;          // ... of an n-contiguous tile
  // the pad puts consecutive k rows 64 bytes (V = 4) or 32 bytes (V = 2) apart modulo the 256 bytes of all banks
  static constexpr int PAD_T = (VN >= 4) ? 64 : 32;
  static constexpr int PAD_N = (VN == 1) ? 0 : (PAD_T + 2 * PAD_T - (BN * ES) % (2 * PAD_T)) % (2 * PAD_T);
  static constexpr int PITCH_N = NC_DIRECT ? BN * ES : BN * ES + PAD_N;
  // m-contiguous A tile: [BK][BM] + pad, the same rule
  static constexpr int PAD_TM = (VM >= 4) ? 64 : 32;
  static constexpr int PAD_M = (VM == 1) ? 0 : (PAD_TM + 2 * PAD_TM - (BM * ES) % (2 * PAD_TM)) % (2 * PAD_TM);
  static constexpr int PITCH_M = BM * ES + PAD_M;
  static constexpr int A_BYTES = (ASRC == A_KC) ? BM * PITCH_K : BK * PITCH_M;
  static constexpr int B_BYTES = (BSRC == B_KC) ? BN * PITCH_K : BK * PITCH_N;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = STAGE_BYTES * STAGES;
  static constexpr int A_CHUNKS = (ASRC == A_KC) ? BM * CPR : BK * (BM * ES / 16);
  static constexpr int B_CHUNKS = (BSRC == B_KC) ? BN * CPR : BK * (BN * ES / 16);
  static constexpr int A_LOADS = (A_CHUNKS + THREADS - 1) / THREADS;
  static constexpr int B_LOADS = (B_CHUNKS + THREADS - 1) / THREADS;
  static_assert(BM % WM == 0 && BN % WN == 0, "wave tile must divide workgroup tile");
  static_assert(WM % MB == 0 && WN % MB == 0, "wave tiles are whole MFMA blocks");
  static_assert(VM >= 1 && (VM & (VM - 1)) == 0 && VM <= (ASRC == A_KC ? V_MAX_K : V_MAX_N), "V of the m operand: a power of two up to the chunks per row");
  static_assert(ASRC == A_KC || (!DIRECT_ && BSRC != B_CONV && BSRC != B_NCS2), "an m-contiguous A is register-staged, GEMM only");
  static_assert(VN >= 1 && (VN & (VN - 1)) == 0 && VN <= (BSRC == B_KC ? V_MAX_K : V_MAX_N), "V of the n operand");
  static_assert(BK % KG == 0, "BK must be a multiple of the fragment k extent");
  static_assert(MB == 32 || MB == 16, "MFMA block edge");
  static_assert(WAVES >= 1 && WAVES <= 16, "waves per workgroup");
  static_assert(!DIRECT || (VEC && (BSRC == B_KC || (BSRC == B_NC && BN * ES / 16 >= 16))),
                "direct-to-LDS needs vector loads; an n-contiguous B needs rows of at least 16 chunks for its swizzle");
  static_assert(!NC_DIRECT || (B_CHUNKS % THREADS == 0), "direct staging deposits whole waves");
  static_assert(BSRC != B_NCS2 || VEC, "the sampled source exists only with vector loads");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS capacity");
  static_assert(STAGES <= 2 || (DIRECT && VEC && (BSRC == B_KC || BSRC == B_NC) && KSTEPS % 2 == 0),
                "rings of three and more stages are filled by direct loads");
  static_assert(STAGES <= 2 || (A_LOADS + B_LOADS) * (STAGES - 2) <= 63, "the load counter holds 63");
};

__device__ inline int swizzled_chunk(int row, int chunk, int rpp, int v) { return chunk ^ ((row / rpp) % v); }
// Byte XOR applied inside an unpadded n-contiguous row of k row `krow`: of the four rows a
// 16-lane group of a transposing read touches, v land in different 64-byte bank groups (v = 4:
// all of them), and with v = 4 rows 8 apart (the two groups of a 16x16-block read) in
// different 32-byte halves.
__device__ inline int nc_swizzle(int krow, int v) { return ((krow & (v - 1)) << 6) ^ (v >= 4 ? (((krow >> 3) & 1) << 5) : 0); }

// ---------------------------------------------------------------- the kernel
// SPLIT: the launch has split tiles (KernelArgs::split > 1); without it the kernel knows at compile time
// that every workgroup owns a whole tile.
template <typename C, bool SPLIT = false>
__global__ __launch_bounds__(C::THREADS) void contraction_kernel(const KernelArgs args) {
  typedef typename C::T T;
  typedef Mfma<T, C::MB> MF;
  typedef typename MF::Acc Acc;
  constexpr int ES = C::ES, EPC = C::EPC, BM = C::BM, BN = C::BN, BK = C::BK, MB = C::MB;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  GENSOR_LDS char* lds = (GENSOR_LDS char*)smem;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int wave_m = wave / C::WAVES_N;
  const int wave_n = wave % C::WAVES_N;

  // ---- workgroup -> (batch, tile_m, tile_n).  Consecutive workgroup ids are dealt
  // round-robin to the 8 XCDs; give each XCD a contiguous range of tiles, and walk tiles
  // in panels of `panel` tile rows so that the tiles resident on one XCD share operand
  // slabs in that XCD's L2.
  const int tiles_per_batch = args.tiles_m * args.tiles_n;
  const int total = tiles_per_batch * args.batch;
  int wg = blockIdx.x;
  int kpart = 0, kparts = 1;                // this workgroup's share of a split tile
  if constexpr (!SPLIT) {
    if ((total & 7) == 0) wg = (wg & 7) * (total >> 3) + (wg >> 3);
  } else if (wg < args.whole) {
    if ((args.whole & 7) == 0) wg = (wg & 7) * (args.whole >> 3) + (wg >> 3);
  } else {
    // the split tiles come last in launch order; with workgroup ids dealt round-robin to the XCDs the parts
    // of one tile are neighbours on one XCD (a matter of locality only)
    kparts = args.split;
    int u = wg - args.whole;
    const int units = (total - args.whole) * kparts;
    if ((units & 7) == 0) u = (u & 7) * (units >> 3) + (u >> 3);
    wg = args.whole + u / kparts;
    kpart = u - (wg - args.whole) * kparts;
  }
  const int bidx = wg / tiles_per_batch;
  int t = wg - bidx * tiles_per_batch;
  int tile_m, tile_n;
  {
    const int panel = args.panel;
    const int per_panel = panel * args.tiles_n;
    const int pi = t / per_panel;
    const int rows_here = min(panel, args.tiles_m - pi * panel);
    const int r = t - pi * per_panel;
    tile_m = pi * panel + r % rows_here;
    tile_n = r / rows_here;
  }
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;

  // k range of this workgroup: the whole of K, or k tiles [kpart * nk / kparts, (kpart + 1) * nk / kparts) of a split
  // tile.  The operand bases move to the first k of the range and Kx is its length, so everything below
  // sees a shorter contraction.
  int Kx = args.K;
  int64_t k_first = 0;
  if (SPLIT && kparts > 1) {
    const int nk_all = (args.K + BK - 1) / BK;
    const int kt0 = kpart * nk_all / kparts, kt1 = (kpart + 1) * nk_all / kparts;
    k_first = (int64_t)kt0 * BK;
    Kx = min(args.K, kt1 * BK) - kt0 * BK;
  }
  const char* Ab = (const char*)args.A + ((int64_t)bidx * args.strideA + (C::ASRC == A_KC ? k_first : k_first * args.lda)) * ES;
  const char* Bb = (const char*)args.B + ((int64_t)bidx * args.strideB + (C::BSRC == B_KC ? k_first : k_first * args.ldb)) * ES;

  // ---- accumulators
  Acc acc[C::MBLK][C::NBLK];
#pragma unroll
  for (int i = 0; i < C::MBLK; ++i)
#pragma unroll
    for (int j = 0; j < C::NBLK; ++j)
#pragma unroll
      for (int v = 0; v < MF::NACC; ++v) acc[i][j][v] = 0.f;

  // ---- buffer resources.  Each operand is addressed through a buffer descriptor whose
  // base is this workgroup's first row (or column) at the current k tile and whose extent
  // ends with the matrix: out-of-range lanes read zero (or are dropped on store) in
  // hardware, so the loop body has no branches.  Offsets inside a tile stay below 2^31 (the
  // host checks BM * lda, BN * ldb or BK * ldb, and BM * ldc).
  constexpr uint32_t RSRC_FLAGS = 0x00020000u;
  constexpr uint32_t OOB = 0x80000000u;      // beyond every descriptor (extents are clamped below 2^31)
  auto clamp_records = [](int64_t bytes) -> uint32_t {
    return bytes <= 0 ? 0u : (bytes > 0x7fffffffll ? 0x7fffffffu : (uint32_t)bytes);
  };
  const int rows_valid = min(BM, args.M - m0);
  const int cols_valid = min(BN, args.N - n0);
  const char* a_tile = (C::ASRC == A_KC) ? Ab + (int64_t)m0 * args.lda * ES : Ab + (int64_t)m0 * ES;
  const char* b_tile = (C::BSRC == B_KC) ? Bb + (int64_t)n0 * args.ldb * ES : (C::BSRC == B_NCS2 ? Bb : Bb + (int64_t)n0 * ES);
  auto rsrc_a = [&](int k0) {
    if constexpr (C::ASRC == A_KC)
      return __builtin_amdgcn_make_buffer_rsrc((void*)(a_tile + (int64_t)k0 * ES), 0,
          clamp_records(((int64_t)(rows_valid - 1) * args.lda + (Kx - k0)) * ES), RSRC_FLAGS);
    else      // k rows beyond K fall out of range; rows of the tile beyond M read what follows them and are never stored
      return __builtin_amdgcn_make_buffer_rsrc((void*)(a_tile + (int64_t)k0 * args.lda * ES), 0,
          clamp_records(((int64_t)(Kx - k0 - 1) * args.lda + (args.M - m0)) * ES), RSRC_FLAGS);
  };
  auto rsrc_b = [&](int k0) {
    if constexpr (C::BSRC == B_KC)
      return __builtin_amdgcn_make_buffer_rsrc((void*)(b_tile + (int64_t)k0 * ES), 0,
          clamp_records(((int64_t)(cols_valid - 1) * args.ldb + (Kx - k0)) * ES), RSRC_FLAGS);
    else if constexpr (C::BSRC == B_NCS2)
      return __builtin_amdgcn_make_buffer_rsrc((void*)(b_tile + (int64_t)k0 * args.ldb * ES), 0,
          clamp_records((int64_t)(Kx - k0) * args.ldb * ES), RSRC_FLAGS);
    else
      return __builtin_amdgcn_make_buffer_rsrc((void*)(b_tile + (int64_t)k0 * args.ldb * ES), 0,
          clamp_records(((int64_t)(Kx - k0 - 1) * args.ldb + (args.N - n0)) * ES), RSRC_FLAGS);
  };

  // ---- who loads what.  A thread owns LDS chunk slots q = tid + i*THREADS of a
  // k-contiguous tile (slot q = row q/CPR, physical chunk q%CPR) and fetches the logical
  // chunk that the swizzle maps there; the same ownership serves the register-staged and
  // the direct path (a direct load deposits lane l's 16 bytes at slot base + l).
  constexpr bool SCALAR_A = !C::VEC;
  constexpr bool SCALAR_B = !C::VEC || C::BSRC == B_CONV;
  uint32_t a_voff[C::A_LOADS], a_kch[C::A_LOADS];
#pragma unroll
  for (int i = 0; i < C::A_LOADS; ++i) {
    const int q = tid + i * C::THREADS;
    if constexpr (C::ASRC == A_KC) {
      const int row = q / C::CPR, ch = swizzled_chunk(row, q % C::CPR, C::RPP, C::VM);
      a_voff[i] = (uint32_t)((row * (int)args.lda + ch * EPC) * ES);
      a_kch[i] = ch * EPC;
    } else {
      constexpr int CPRM = BM * ES / 16;
      a_voff[i] = (uint32_t)(((q / CPRM) * (int)args.lda + (q % CPRM) * EPC) * ES);
      a_kch[i] = q / CPRM;
    }
  }
  uint32_t b_voff[C::B_LOADS], b_kch[C::B_LOADS];
  uint32_t b_voff2[C::BSRC == B_NCS2 ? C::B_LOADS : 1];      // second half of a sampled chunk
#pragma unroll
  for (int i = 0; i < C::B_LOADS; ++i) {
    const int q = tid + i * C::THREADS;
    if constexpr (C::BSRC == B_KC) {
      const int row = q / C::CPR, ch = swizzled_chunk(row, q % C::CPR, C::RPP, C::VN);
      b_voff[i] = (uint32_t)((row * (int)args.ldb + ch * EPC) * ES);
      b_kch[i] = ch * EPC;
    } else if constexpr (C::BSRC == B_NCS2) {
      // chunk = EPC consecutive columns = two halves of EPC/2 columns, each inside one output
      // row (Q is a multiple of EPC/2) and so one 16-byte run of the input row it samples
      constexpr int CPRN = BN * ES / 16;
      const int krow = q / CPRN, ch = q % CPRN;
      const int nA = n0 + ch * EPC, nB = nA + EPC / 2;
      const int pA = nA / args.cQ, pB = nB / args.cQ;
      const int sA = (2 * pA) * args.cW + 2 * (nA - pA * args.cQ), sB = (2 * pB) * args.cW + 2 * (nB - pB * args.cQ);
      b_voff[i] = nA < args.N ? (uint32_t)((krow * (int)args.ldb + sA) * ES) : OOB;
      b_voff2[i] = nB < args.N ? (uint32_t)((krow * (int)args.ldb + sB) * ES) : OOB;
      b_kch[i] = krow;
    } else {
      constexpr int CPRN = BN * ES / 16;
      const int krow = q / CPRN;
      int ch = q % CPRN;
      if constexpr (C::NC_DIRECT) ch ^= nc_swizzle(krow, C::VN) >> 4;      // slot q receives the chunk the swizzle maps there
      b_voff[i] = (uint32_t)((krow * (int)args.ldb + ch * EPC) * ES);
      b_kch[i] = krow;
    }
  }

  // ---- staging registers (global -> registers -> LDS)
  u32x4 ra[C::DIRECT ? 1 : C::A_LOADS];
  u32x4 rb[C::DIRECT ? 1 : C::B_LOADS * (C::BSRC == B_NCS2 ? 2 : 1)];

  // element-wise access for the scalar path and the convolution gather
  auto a_elem_bits = [&](int row, int k) -> uint32_t {
    if (row < args.M && k < Kx) {
      int64_t idx = (C::ASRC == A_KC) ? (int64_t)row * args.lda + k : (int64_t)k * args.lda + row;
      if constexpr (ES == 4) return ((const uint32_t*)Ab)[idx];
      else return ((const uint16_t*)Ab)[idx];
    }
    return 0u;
  };
  auto b_elem_bits = [&](int k, int col) -> uint32_t {
    if (col >= args.N || k >= Kx) return 0u;
    int64_t idx;
    if constexpr (C::BSRC == B_KC) idx = (int64_t)col * args.ldb + k;
    else if constexpr (C::BSRC == B_NC) idx = (int64_t)k * args.ldb + col;
    else {
      const int rs = args.cR * args.cS;
      const int c = k / rs, rr = (k - c * rs) / args.cS, ss = k - c * rs - rr * args.cS;
      const int pq = args.cP * args.cQ;
      const int img = col / pq, p = (col - img * pq) / args.cQ, q = col - img * pq - p * args.cQ;
      const int y = p * args.cStride - args.cPad + rr, x = q * args.cStride - args.cPad + ss;
      if (y < 0 || y >= args.cH || x < 0 || x >= args.cW) return 0u;
      idx = (((int64_t)img * args.cC + c) * args.cH + y) * args.cW + x;
    }
    if constexpr (ES == 4) return ((const uint32_t*)Bb)[idx];
    else return ((const uint16_t*)Bb)[idx];
  };
  auto pack_chunk = [&](auto&& elem) -> u32x4 {   // elem(e) for e in [0, EPC)
    u32x4 v;
    if constexpr (ES == 4) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = elem(e);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = elem(2 * e) | (elem(2 * e + 1) << 16);
    }
    return v;
  };

  // ---- fetch the k tile starting at k0: into registers, or straight into LDS stage `st`.
  // In a k-contiguous row a chunk beyond K would alias the next row, so those lanes are
  // sent out of range; this can only happen in the last k tile.
  auto fetch_a = [&](int k0, int st, int part = 0, int parts = 1) {
    const bool full = Kx - k0 >= BK;
    if constexpr (SCALAR_A) {
#pragma unroll
      for (int i = 0; i < C::A_LOADS; ++i) {
        const int q = tid + i * C::THREADS;
        if (C::A_CHUNKS % C::THREADS != 0 && q >= C::A_CHUNKS) break;
        if constexpr (C::ASRC == A_KC) {
          const int row = q / C::CPR, ch = swizzled_chunk(row, q % C::CPR, C::RPP, C::VM);
          ra[i] = pack_chunk([&](int e) { return a_elem_bits(m0 + row, k0 + ch * EPC + e); });
        } else {
          constexpr int CPRM = BM * ES / 16;
          ra[i] = pack_chunk([&](int e) { return a_elem_bits(m0 + (q % CPRM) * EPC + e, k0 + q / CPRM); });
        }
      }
    } else {
      const __amdgpu_buffer_rsrc_t r = rsrc_a(k0);
#pragma unroll
      for (int i = 0; i < C::A_LOADS; ++i) {
        if (C::A_CHUNKS % C::THREADS != 0 && tid + i * C::THREADS >= C::A_CHUNKS) break;
        if (i * parts < part * C::A_LOADS || i * parts >= (part + 1) * C::A_LOADS) continue;
        // (direct staging is only launched for K a multiple of BK: every tile is full)
        const uint32_t off = (C::ASRC == A_MC || C::DIRECT || full || (int)a_kch[i] < Kx - k0) ? a_voff[i] : OOB;
        if constexpr (C::DIRECT)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (GENSOR_LDS void*)(lds + st * C::STAGE_BYTES + (i * C::THREADS + wave * 64) * 16),
                                                   16, off, 0, 0, 0);
        else
          ra[i] = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
      }
    }
  };
  auto fetch_b = [&](int k0, int st, int part = 0, int parts = 1) {
    const bool full = Kx - k0 >= BK;
    if constexpr (SCALAR_B) {
#pragma unroll
      for (int i = 0; i < C::B_LOADS; ++i) {
        const int q = tid + i * C::THREADS;
        if (C::B_CHUNKS % C::THREADS != 0 && q >= C::B_CHUNKS) break;
        if constexpr (C::BSRC == B_KC) {
          const int row = q / C::CPR, ch = swizzled_chunk(row, q % C::CPR, C::RPP, C::VN);
          rb[i] = pack_chunk([&](int e) { return b_elem_bits(k0 + ch * EPC + e, n0 + row); });
        } else {
          constexpr int CPRN = BN * ES / 16;
          const int krow = q / CPRN, ch = q % CPRN;
          rb[i] = pack_chunk([&](int e) { return b_elem_bits(k0 + krow, n0 + ch * EPC + e); });
        }
      }
    } else {
      const __amdgpu_buffer_rsrc_t r = rsrc_b(k0);
#pragma unroll
      for (int i = 0; i < C::B_LOADS; ++i) {
        if (C::B_CHUNKS % C::THREADS != 0 && tid + i * C::THREADS >= C::B_CHUNKS) break;
        if (i * parts < part * C::B_LOADS || i * parts >= (part + 1) * C::B_LOADS) continue;
        uint32_t off = b_voff[i];
        if constexpr (C::BSRC == B_KC && !C::DIRECT) off = (full || (int)b_kch[i] < Kx - k0) ? off : OOB;
        if constexpr (C::DIRECT) {
          __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (GENSOR_LDS void*)(lds + st * C::STAGE_BYTES + C::A_BYTES + (i * C::THREADS + wave * 64) * 16),
                                                   16, off, 0, 0, 0);
        } else if constexpr (C::BSRC == B_NCS2) {
          rb[2 * i] = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
          rb[2 * i + 1] = __builtin_amdgcn_raw_buffer_load_b128(r, b_voff2[i], 0, 0);
        } else {
          rb[i] = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
        }
      }
    }
  };
  // ---- registers -> LDS stage `st`
  auto commit = [&](int st) {
    if constexpr (!C::DIRECT) {
      GENSOR_LDS char* abase = lds + st * C::STAGE_BYTES;
      GENSOR_LDS char* bbase = abase + C::A_BYTES;
#pragma unroll
      for (int i = 0; i < C::A_LOADS; ++i) {
        const int q = tid + i * C::THREADS;
        if (C::A_CHUNKS % C::THREADS != 0 && q >= C::A_CHUNKS) break;
        if constexpr (C::ASRC == A_KC) {
          *(GENSOR_LDS u32x4*)(abase + q * 16) = ra[i];
        } else {
          constexpr int CPRM = BM * ES / 16;
          *(GENSOR_LDS u32x4*)(abase + (q / CPRM) * C::PITCH_M + (q % CPRM) * 16) = ra[i];
        }
      }
#pragma unroll
      for (int i = 0; i < C::B_LOADS; ++i) {
        const int q = tid + i * C::THREADS;
        if (C::B_CHUNKS % C::THREADS != 0 && q >= C::B_CHUNKS) break;
        if constexpr (C::BSRC == B_KC) {
          *(GENSOR_LDS u32x4*)(bbase + q * 16) = rb[i];
        } else if constexpr (C::BSRC == B_NCS2) {
          // keep every other element of the two 16-byte runs
          constexpr int CPRN = BN * ES / 16;
          const u32x4 v0 = rb[2 * i], v1 = rb[2 * i + 1];
          u32x4 o;
          if constexpr (ES == 4) {
            o[0] = v0[0]; o[1] = v0[2]; o[2] = v1[0]; o[3] = v1[2];
          } else {
            o[0] = __builtin_amdgcn_perm(v0[1], v0[0], 0x05040100u);
            o[1] = __builtin_amdgcn_perm(v0[3], v0[2], 0x05040100u);
            o[2] = __builtin_amdgcn_perm(v1[1], v1[0], 0x05040100u);
            o[3] = __builtin_amdgcn_perm(v1[3], v1[2], 0x05040100u);
          }
          *(GENSOR_LDS u32x4*)(bbase + (q / CPRN) * C::PITCH_N + (q % CPRN) * 16) = o;
        } else {
          constexpr int CPRN = BN * ES / 16;
          *(GENSOR_LDS u32x4*)(bbase + (q / CPRN) * C::PITCH_N + (q % CPRN) * 16) = rb[i];
        }
      }
    }
  };
  // all of this wave's direct deposits have landed (vmcnt(0); expcnt and lgkmcnt untouched)
  auto wait_deposits = [&]() {
    if constexpr (C::DIRECT) __builtin_amdgcn_s_waitcnt(0x0F70);
  };

  // ---- fragments.  fa[b] / fb[b] are two register sets so that the reads of k step s+1
  // are in flight while the MFMAs of step s issue.
  const int frow = lane % MB;          // row / column inside an MFMA block
  const int fgrp = lane / MB;          // which chunk of the k group this lane holds
  auto block_row = [&](int bi) { return wave_m * C::WM + bi * MB; };   // first row of MFMA block bi of this wave inside the BM tile
  auto block_col = [&](int bj) { return wave_n * C::WN + bj * MB; };
  // One wave per SIMD (four waves of 128x128): nothing else covers a stall, so fragments are read
  // two k steps ahead (one register set per k step of a tile) and the barrier sits in front of step 2
  // (4096^3 on all-zero operands, where the power limit does not interfere: 88.0 -> 81.4 us; 8192^3 on
  // the benchmark's operands: 971 -> 910 us, against 950 us for eight waves of 128x64).
  constexpr bool DEEP = C::DIRECT && C::STAGES == 2 && C::KSTEPS == 4 && C::MBLK * C::NBLK >= 16;
  constexpr int FSETS = DEEP ? 4 : 2;
  u32x4 fa[FSETS][C::MBLK], fb[FSETS][C::NBLK];
  // Direct staging with an n-contiguous 16-bit B: the transposing fragment reads are issued from inline assembly.
  // A compiler-issued LDS read that it cannot tell apart from the destinations of the direct loads in flight is
  // preceded by a wait for ALL of them (vmcnt(0)), which it does for the transposing-read builtin: every k tile
  // then waited out the full latency of the loads just issued for the next one.  The assembly reads are invisible
  // to the compiler's counter bookkeeping, so the kernel waits for them itself: `settle` below, in front of the
  // MFMAs that consume a register set.  LDS operations complete in issue order and the statements are volatile,
  // hence ordered: "at most N outstanding", with N no more than the number of such reads issued after the awaited
  // ones, means the awaited ones have landed.  The halves stay separate values until that wait (a copy of a pending
  // register would read stale data); the compiler's own waits only get more conservative by operations it does not see.
  constexpr bool ASM_TR = C::NC_DIRECT && ES == 2;
  u32x2 fbl[ASM_TR ? FSETS : 1][ASM_TR ? C::NBLK : 1], fbh[ASM_TR ? FSETS : 1][ASM_TR ? C::NBLK : 1];
  // Fragment of one MFMA block from a tile stored [k][rows] (an n-contiguous B or an m-contiguous A), `first` =
  // the block's first row/column inside the tile, `direct` = the tile is unpadded and XOR-swizzled.
  auto read_transposed = [&](GENSOR_LDS char* base, int pitch, int first, int ks, auto direct_tag, int v) -> u32x4 {
    constexpr bool direct = decltype(direct_tag)::value;
    if constexpr (ES == 4) {
      // fp32: element t of this lane's chunk is k = ks*KG + fgrp*4 + t
      const int col = first + frow;
      u32x4 r;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const int kr = ks * C::KG + fgrp * 4 + tt;
        const int cb = direct ? ((col * 4) ^ nc_swizzle(kr, v)) : col * 4;
        r[tt] = *(GENSOR_LDS uint32_t*)(base + kr * pitch + cb);
      }
      return r;
    } else {
      // 16-bit: two transposing reads.  In each 16-lane group, lane s fetches 4 consecutive rows/columns of
      // k row (s/4) and receives, for row/column s, the 4 consecutive k of the group's k rows.
      const int g = lane >> 4, s = lane & 15;
      int krow, col;
      if constexpr (MB == 32) {    // groups: (g%2) picks the 16-wide half, (g/2) the 8-deep k half
        krow = ks * C::KG + (g >> 1) * 8 + (s >> 2);
        col = first + (g & 1) * 16 + (s & 3) * 4;
      } else {                     // 16x16 blocks: group g holds k = 8g..8g+7
        krow = ks * C::KG + g * 8 + (s >> 2);
        col = first + (s & 3) * 4;
      }
      const int cb0 = direct ? ((col * 2) ^ nc_swizzle(krow, v)) : col * 2;
      const int cb1 = direct ? ((col * 2) ^ nc_swizzle(krow + 4, v)) : col * 2;
      GENSOR_LDS char* p = base + krow * pitch;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GENSOR_LDS s16x4*)(p + cb0));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GENSOR_LDS s16x4*)(p + 4 * pitch + cb1));
      u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
      u32x4 r = {l2[0], l2[1], h2[0], h2[1]};
      return r;
    }
  };
  auto read_frags = [&](int st, int ks, int buf) {
    GENSOR_LDS char* abase = lds + st * C::STAGE_BYTES;
    GENSOR_LDS char* bbase = abase + C::A_BYTES;
    const int ch = ks * C::LANE_GROUPS + fgrp;
#pragma unroll
    for (int bi = 0; bi < C::MBLK; ++bi) {
      if constexpr (C::ASRC == A_KC) {
        const int row = block_row(bi) + frow;
        fa[buf][bi] = *(GENSOR_LDS u32x4*)(abase + row * C::PITCH_K + swizzled_chunk(row, ch, C::RPP, C::VM) * 16);
      } else {
        fa[buf][bi] = read_transposed(abase, C::PITCH_M, block_row(bi), ks, std::false_type{}, C::VM);
      }
    }
#pragma unroll
    for (int bj = 0; bj < C::NBLK; ++bj) {
      if constexpr (C::BSRC == B_KC) {
        const int row = block_col(bj) + frow;
        fb[buf][bj] = *(GENSOR_LDS u32x4*)(bbase + row * C::PITCH_K + swizzled_chunk(row, ch, C::RPP, C::VN) * 16);
      } else if constexpr (ASM_TR) {
        const int g = lane >> 4, s = lane & 15;
        int krow, col;
        if constexpr (MB == 32) {
          krow = ks * C::KG + (g >> 1) * 8 + (s >> 2);
          col = block_col(bj) + (g & 1) * 16 + (s & 3) * 4;
        } else {
          krow = ks * C::KG + g * 8 + (s >> 2);
          col = block_col(bj) + (s & 3) * 4;
        }
        const uint32_t a0 = (uint32_t)(uintptr_t)(bbase + krow * C::PITCH_N + ((col * 2) ^ nc_swizzle(krow, C::VN)));
        const uint32_t a1 = (uint32_t)(uintptr_t)(bbase + (krow + 4) * C::PITCH_N + ((col * 2) ^ nc_swizzle(krow + 4, C::VN)));
        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(fbl[buf][bj]) : "v"(a0));
        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(fbh[buf][bj]) : "v"(a1));
      } else {
        fb[buf][bj] = read_transposed(bbase, C::PITCH_N, block_col(bj), ks, std::integral_constant<bool, C::NC_DIRECT>{}, C::VN);
      }
    }
  };
  // groups: how many later read_frags calls (each 2 * NBLK transposing reads) have been issued since the one that
  // filled register set buf -- a lower bound; 0 waits for every LDS operation
  auto settle = [&](int buf, auto groups_tag) {
    if constexpr (ASM_TR) {
      constexpr int N = decltype(groups_tag)::value * 2 * C::NBLK > 15 ? 15 : decltype(groups_tag)::value * 2 * C::NBLK;
#pragma unroll
      for (int bj = 0; bj < C::NBLK; ++bj) {
        if (bj == 0) asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(fbl[buf][bj]), "+v"(fbh[buf][bj]) : "n"(N));
        else asm volatile("" : "+v"(fbl[buf][bj]), "+v"(fbh[buf][bj]));
        const u32x4 v = {fbl[buf][bj][0], fbl[buf][bj][1], fbh[buf][bj][0], fbh[buf][bj][1]};
        fb[buf][bj] = v;
      }
    }
  };
  // Workgroup barrier of the k loop.  The transposing reads issued from assembly must have left the LDS before
  // another wave may overwrite the stage they read; the compiler does not know of them, so the wait is explicit.
  auto block_sync = [&]() {
    if constexpr (ASM_TR) __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0); the other counters untouched
    __syncthreads();
  };
  auto mma = [&](int buf, auto groups_tag) {
    settle(buf, groups_tag);
#pragma unroll
    for (int bi = 0; bi < C::MBLK; ++bi)
#pragma unroll
      for (int bj = 0; bj < C::NBLK; ++bj) {
        MF::run(fa[buf][bi], fb[buf][bj], acc[bi][bj]);
      }
  };

  // Scheduling hint for one k step: issue the fragment reads of the next step in small
  // groups in front of each MFMA of this step, so that they complete under matrix work.
  auto interleave = [&]() {
    constexpr int NM = C::MBLK * C::NBLK * (ES == 4 ? 4 : 1);
    constexpr int NR = C::MBLK * (C::ASRC == A_KC ? 1 : (ES == 4 ? 4 : 2)) + C::NBLK * (C::BSRC == B_KC ? 1 : (ES == 4 ? 4 : 2));
    constexpr int RPM = (NR + NM - 1) / NM;
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);   // LDS reads
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // the same with the global loads of this step between the MFMAs as well.  One wave per SIMD
  // (`separate`): the fragment reads in front of the first MFMAs, then one load per MFMA, so that
  // no gap between two MFMAs has to issue both a read and a load.  Two waves per SIMD measure better
  // with a load and a read per gap, loads first.
  auto interleave_vmem = [&](auto separate_tag) {
    constexpr bool separate = decltype(separate_tag)::value;
    constexpr int NM = C::MBLK * C::NBLK * (ES == 4 ? 4 : 1);
    constexpr int NR = C::MBLK * (C::ASRC == A_KC ? 1 : (ES == 4 ? 4 : 2)) + C::NBLK * (C::BSRC == B_KC ? 1 : (ES == 4 ? 4 : 2));
    constexpr int RPM = (NR + NM - 1) / NM;
    constexpr int READ_SLOTS = (NR + RPM - 1) / RPM;
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      if constexpr (separate) {
        if (i < READ_SLOTS) __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);   // LDS reads
        else __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                     // one global load
      } else {
        __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                            // one MFMA
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- main loop over k tiles.  Tile kt+1 is fetched while tile kt is multiplied; its
  // first fragments are read right after the barrier, under the MFMAs of the last k step
  // of tile kt, so that the barrier and the LDS latency are covered by matrix work.
  const int nk = (Kx + BK - 1) / BK;
  constexpr bool PIPE = (C::KSTEPS % 2 == 0) && C::STAGES == 2;
  if constexpr (C::STAGES <= 2) {
    fetch_a(0, 0);
    fetch_b(0, 0);
    commit(0);
    wait_deposits();
    __syncthreads();
  }
  if constexpr (DEEP) {
    // By the barrier in front of step 2 every wave has read (and received) steps 2 and 3 of this
    // tile, so its stage is free: the loads of tile kt+2 go out right behind the barrier, over
    // steps 2 and 3 and between their MFMAs, a whole k tile before they are needed.
    auto k_tile = [&](int kt, auto next_tag, auto fetch_tag) {
      constexpr bool has_next = decltype(next_tag)::value, has_fetch = decltype(fetch_tag)::value;
      const int cur = kt & 1, nxt = cur ^ 1;
      read_frags(cur, 2, 2);
      mma(0, std::integral_constant<int, 2>{});
      interleave();
      read_frags(cur, 3, 3);
      mma(1, std::integral_constant<int, 2>{});
      interleave();
      if constexpr (has_next) {
        wait_deposits();
        block_sync();
        read_frags(nxt, 0, 0);
        if constexpr (has_fetch) {
          fetch_a((kt + 2) * BK, cur, 0, 2);
          fetch_b((kt + 2) * BK, cur, 0, 2);
        }
      }
      mma(2, std::integral_constant<int, has_next ? 2 : 1>{});
      if constexpr (has_fetch) interleave_vmem(std::true_type{});
      else interleave();
      if constexpr (has_next) {
        read_frags(nxt, 1, 1);
        if constexpr (has_fetch) {
          fetch_a((kt + 2) * BK, cur, 1, 2);
          fetch_b((kt + 2) * BK, cur, 1, 2);
        }
      }
      mma(3, std::integral_constant<int, has_next ? 2 : 0>{});
      if constexpr (has_fetch) interleave_vmem(std::true_type{});
      else interleave();
    };
    if (nk > 1) {
      fetch_a(BK, 1);
      fetch_b(BK, 1);
    }
    read_frags(0, 0, 0);
    read_frags(0, 1, 1);
    for (int kt = 0; kt + 2 < nk; ++kt) k_tile(kt, std::true_type{}, std::true_type{});
    if (nk > 1) k_tile(nk - 2, std::true_type{}, std::false_type{});
    k_tile(nk - 1, std::false_type{}, std::false_type{});
  } else if constexpr (C::STAGES > 2) {
    // Ring of STAGES buffers: STAGES-1 k tiles are in flight, so a tile has STAGES-1 tile times to
    // arrive.  Loads complete in issue order, hence "tile kt+1 has landed" is "at most the loads
    // of the STAGES-2 younger tiles are outstanding"; near the end of k fewer tiles are in flight
    // and the wait is for all of them.  Three copies of the body (steady state, draining, last
    // tile) keep those facts compile-time.  The stage refilled at the top of tile kt is the one
    // read during tile kt-1, which every wave left before the barrier that ended that tile.
    constexpr int S = C::STAGES;
    constexpr int LPT = C::A_LOADS + C::B_LOADS;             // loads per thread and tile
    constexpr int WAIT_STEADY = 0x0F70 | ((LPT * (S - 2)) & 0xF) | (((LPT * (S - 2)) >> 4) << 14);
    // This wave's LDS reads are complete (its loads in flight are left alone), then the workgroup
    // barrier: the waits above have made the awaited deposits of every wave visible before it.
    auto ring_barrier = [&]() {
      __builtin_amdgcn_s_waitcnt(0xC07F);
      __builtin_amdgcn_s_barrier();
    };
    auto k_tile = [&](int kt, int cur, auto fetch_tag, auto more_tag) {
      constexpr bool fetch = decltype(fetch_tag)::value, more = decltype(more_tag)::value;
      const int nxt = cur + 1 == S ? 0 : cur + 1;
      if constexpr (fetch) {
        const int dst = cur == 0 ? S - 1 : cur - 1;
        fetch_a((kt + S - 1) * BK, dst);
        fetch_b((kt + S - 1) * BK, dst);
      }
#pragma unroll
      for (int ks = 0; ks < C::KSTEPS; ++ks) {
        if (ks + 1 < C::KSTEPS) {
          read_frags(cur, ks + 1, (ks + 1) & 1);
        } else if constexpr (more) {
          if constexpr (fetch) __builtin_amdgcn_s_waitcnt(WAIT_STEADY);
          else __builtin_amdgcn_s_waitcnt(0x0F70);
          ring_barrier();
          read_frags(nxt, 0, 0);
        }
        if (ks + 1 < C::KSTEPS || more) mma(ks & 1, std::integral_constant<int, 1>{});
        else mma(ks & 1, std::integral_constant<int, 0>{});
        interleave();
      }
      return nxt;
    };
#pragma unroll
    for (int t = 0; t < S - 1; ++t)
      if (t < nk) {
        fetch_a(t * BK, t);
        fetch_b(t * BK, t);
      }
    if (nk >= S - 1) __builtin_amdgcn_s_waitcnt(WAIT_STEADY);      // S-1 tiles issued: tile 0 is the oldest
    else __builtin_amdgcn_s_waitcnt(0x0F70);
    ring_barrier();
    read_frags(0, 0, 0);
    int cur = 0, kt = 0;
    for (; kt + S - 1 < nk; ++kt) cur = k_tile(kt, cur, std::true_type{}, std::true_type{});
    for (; kt + 1 < nk; ++kt) cur = k_tile(kt, cur, std::false_type{}, std::true_type{});
    k_tile(kt, cur, std::false_type{}, std::false_type{});
  } else if constexpr (PIPE) {
    // Whether a further k tile follows is a compile-time property of the loop body: the last k
    // tile is peeled.  With a run-time test the two paths would meet in front of the last k
    // step's MFMAs, where the compiler must then wait for the fragment reads issued after the
    // barrier (they are outstanding on one path only), which stalls every wave of the workgroup
    // at the same moment once per k tile.
    auto k_tile = [&](int kt, auto more_tag) {
      constexpr bool more = decltype(more_tag)::value;
      const int cur = kt & 1, nxt = cur ^ 1;
      // Wave tiles of eight and more MFMAs per k step issue the direct loads of the next tile over the
      // first two k steps, one between MFMAs, instead of in one burst at the top: with one such wave
      // per SIMD the burst is time no MFMA runs (256x256 tile of four 128x128 waves: 124 -> 116 us;
      // two 128x64 waves per SIMD gain 1 %; 64x64 wave tiles lose 1-8 % and keep the burst).
      constexpr int FS = (C::DIRECT && C::KSTEPS >= 4 && C::MBLK * C::NBLK >= 8) ? 2 : 1;
#pragma unroll
      for (int ks = 0; ks < C::KSTEPS; ++ks) {
        if constexpr (more) {
          if (ks < FS) {
            fetch_a((kt + 1) * BK, nxt, ks, FS);
            fetch_b((kt + 1) * BK, nxt, ks, FS);
          }
        }
        if (ks + 1 < C::KSTEPS) {
          read_frags(cur, ks + 1, (ks + 1) & 1);
        } else if constexpr (more) {
          commit(nxt);
          wait_deposits();
          block_sync();
          read_frags(nxt, 0, 0);
        }
        if (ks + 1 < C::KSTEPS || more) mma(ks & 1, std::integral_constant<int, 1>{});
        else mma(ks & 1, std::integral_constant<int, 0>{});
        if (FS > 1 && more && ks < FS) interleave_vmem(std::false_type{});
        else interleave();
      }
    };
    read_frags(0, 0, 0);
    for (int kt = 0; kt + 1 < nk; ++kt) k_tile(kt, std::true_type{});
    k_tile(nk - 1, std::false_type{});
  } else {
    for (int kt = 0; kt < nk; ++kt) {
      const bool more = kt + 1 < nk;
      const int cur = C::STAGES == 2 ? (kt & 1) : 0, nxt = C::STAGES == 2 ? (cur ^ 1) : 0;
      if (more) {
        if constexpr (!C::DIRECT || C::STAGES == 2) {
          fetch_a((kt + 1) * BK, nxt);
          fetch_b((kt + 1) * BK, nxt);
        }
      }
#pragma unroll
      for (int ks = 0; ks < C::KSTEPS; ++ks) {
        read_frags(cur, ks, 0);
        mma(0, std::integral_constant<int, 0>{});
      }
      if constexpr (C::STAGES == 1) {
        block_sync();                       // everyone is done reading the single buffer
        if constexpr (C::DIRECT) {
          if (more) {
            fetch_a((kt + 1) * BK, 0);
            fetch_b((kt + 1) * BK, 0);
          }
        }
      }
      if (more) commit(nxt);
      wait_deposits();
      block_sync();
    }
  }

  // ---- split tile: exchange the partial sums; one wave per (tile, wave position) goes on to the epilogue
  if (SPLIT && kparts > 1) {
    // Every wave leaves its accumulators in this workgroup's slot (16 bytes per lane and store, a wave's store
    // one contiguous KiB) and counts itself in.  The wave that finds the other parts-1 already counted adds
    // their slots to its own registers and goes on to the epilogue; the others are done.  Nothing waits.
    // Two parts: own registers plus the other slot (the sum of two terms has one order).  More: the slots are
    // summed from memory in part order, so the result does not depend on who came last.
    // The parts of a tile may run on different XCDs, whose L2s do not see each other's lines: the slot
    // stores and loads carry the device-scope cache policy (write through / fetch again), a wave counts
    // itself in only after its stores have completed, and the count is a device-scope atomic.  Nothing else
    // in the kernel pays for this (a device-scope fence would write back and invalidate the whole L2 here).
    constexpr int NV = C::MBLK * C::NBLK * MF::NACC / 4;       // 16-byte groups per lane
    constexpr int SLOT_BYTES = BM * BN * 4;
    constexpr int DEVICE_SCOPE = 16;                           // sc1: the access is coherent across the whole device
    const int64_t tile_slot = (int64_t)(wg - args.whole) * kparts;
    auto slot = [&](int o) {
      return __builtin_amdgcn_make_buffer_rsrc((void*)((char*)args.partials + (tile_slot + o) * (int64_t)SLOT_BYTES), 0,
                                               (uint32_t)SLOT_BYTES, RSRC_FLAGS);
    };
    const __amdgpu_buffer_rsrc_t own = slot(kpart);
#pragma unroll
    for (int g = 0; g < NV; ++g) {
      const int b = g / (MF::NACC / 4), q = g % (MF::NACC / 4);
      u32x4 v;
#pragma unroll
      for (int x = 0; x < 4; ++x) v[x] = as_u32(acc[b / C::NBLK][b % C::NBLK][4 * q + x]);
      __builtin_amdgcn_raw_buffer_store_b128(v, own, (uint32_t)((g * C::THREADS + tid) * 16), 0, DEVICE_SCOPE);
      if (g % 8 == 7) __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");     // compiler ordering
    __builtin_amdgcn_s_waitcnt(0x0F70);                        // vmcnt(0): this wave's slot stores have completed
    __builtin_amdgcn_sched_barrier(0);
    uint32_t before = 0;
    if (lane == 0) before = atomicAdd(args.counters + (int64_t)(wg - args.whole) * C::WAVES + wave, 1u);
    before = __builtin_amdgcn_readfirstlane(before);
    if (before != (uint32_t)(kparts - 1)) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const bool from_memory = kparts > 2;
    if (from_memory) {
#pragma unroll
      for (int i = 0; i < C::MBLK; ++i)
#pragma unroll
        for (int j = 0; j < C::NBLK; ++j)
#pragma unroll
          for (int v = 0; v < MF::NACC; ++v) acc[i][j][v] = 0.f;
    }
    for (int o = 0; o < kparts; ++o) {
      if (!from_memory && o == kpart) continue;
      const __amdgpu_buffer_rsrc_t src = slot(o);
#pragma unroll
      for (int g = 0; g < NV; ++g) {
        const int b = g / (MF::NACC / 4), q = g % (MF::NACC / 4);
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(src, (uint32_t)((g * C::THREADS + tid) * 16), 0, DEVICE_SCOPE);
#pragma unroll
        for (int x = 0; x < 4; ++x) acc[b / C::NBLK][b % C::NBLK][4 * q + x] += as_f32(v[x]);
        if (g % 8 == 7) __builtin_amdgcn_sched_barrier(0);     // eight loads in flight, not all of them: registers
      }
    }
  }

  // ---- epilogue: C = alpha * acc + beta * C through a buffer descriptor that starts at this
  // tile's first element; rows outside the matrix fall out of its range, columns beyond it are
  // sent out of range explicitly (they would alias the next row).  Lane l of a 32x32 block holds
  // column l%32 and rows 8*(v/4) + 4*(l/32) + v%4 in acc[v] (16x16: column l%16, rows 4*(l/16) + v),
  // so one element store of a wave covers two whole 128-byte row segments of C (four 64-byte
  // ones for 16x16 blocks).  Accumulating the transposed block instead, for 16-byte vector stores
  // of four columns per lane, measured slower everywhere (32 rows x 32 bytes per instruction:
  // -3 % on the 4096^3 GEMM, -9 % on 8192x3072x768, -11 % on the store-bound K = 64 shapes).
  typedef typename C::OutT OutT;
  constexpr int OS = ElemSize<OutT>::value;
  char* Cb = (char*)args.C + (int64_t)bidx * args.strideC * OS;
  const float alpha = args.alpha, beta = args.beta;
  if constexpr (C::BSRC == B_CONV) {
    // output O[img][filter][p][q]: row = filter, col = (img, p, q)
    const int pq = args.cP * args.cQ;
#pragma unroll
    for (int bi = 0; bi < C::MBLK; ++bi)
#pragma unroll
      for (int bj = 0; bj < C::NBLK; ++bj) {
        const int col = n0 + block_col(bj) + frow;
        const int img = col / pq;
        const int64_t cbase = (int64_t)img * args.M * pq + (col - img * pq);
#pragma unroll
        for (int v = 0; v < MF::NACC; ++v) {
          const int r = (MB == 32) ? 8 * (v / 4) + 4 * fgrp + (v % 4) : 4 * fgrp + v;
          const int row = m0 + block_row(bi) + r;
          if (row < args.M && col < args.N) store_out<OutT>(Cb, cbase + (int64_t)row * pq, alpha * acc[bi][bj][v]);
        }
      }
  } else {
    const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(Cb + ((int64_t)m0 * args.ldc + n0) * OS), 0,
        clamp_records(((int64_t)(rows_valid - 1) * args.ldc + cols_valid) * OS), RSRC_FLAGS);
    // C is stored with the write-through cache policy (sc1): every line goes to memory at once instead of
    // lying dirty in the L2 until it is evicted.  Measured against write-back: 10-15 % faster on the
    // store-bound shapes (96 x 1024 x 1024 x 64: 79 -> 70 us), 1-2 % on the 4096^3 and GPT-2 shapes, 0.5-2.5 %
    // slower on launches of many rounds of long tiles (8192^3, 65536 x 4096 x 1024), where a write-back L2
    // drains one tile's stores under the next tile's loop.  The policy is an immediate of the store
    // instruction; choosing it at run time (two copies of this loop behind a branch) cost every shape 1-2 %.
    constexpr int STORE_POLICY = 16;
    // One store costs an accumulator read, the scaling, one add and the store: the column part of the offset (or
    // an out-of-range one: adding a row offset below 2^31 keeps it out of range) is selected once per block column,
    // the row part is a per-lane base plus a multiple of the row pitch that is the same for the whole wave, and
    // whether C is read (beta) is decided once per block, not per element.
    const uint32_t pitch = (uint32_t)args.ldc * OS;
    auto store_block = [&](int bi, int bj, uint32_t lane_off, auto beta_tag) {
      constexpr bool with_beta = decltype(beta_tag)::value;
#pragma unroll
      for (int v = 0; v < MF::NACC; ++v) {
        const int r = (MB == 32) ? 8 * (v / 4) + (v % 4) : v;      // row inside the block, less the lane group's 4 * fgrp
        const uint32_t off = lane_off + (uint32_t)r * pitch;
        float x = alpha * acc[bi][bj][v];
        if constexpr (OS == 4) {
          if constexpr (with_beta) x += beta * as_f32(__builtin_amdgcn_raw_buffer_load_b32(rc, off, 0, 0));
          __builtin_amdgcn_raw_buffer_store_b32(as_u32(x), rc, off, 0, STORE_POLICY);
        } else {
          if constexpr (with_beta) {
            const uint16_t old = __builtin_amdgcn_raw_buffer_load_b16(rc, off, 0, 0);
            x += beta * to_float<OutT>(&old, 0);
          }
          uint16_t bits;
          store_out<OutT>(&bits, 0, x);
          __builtin_amdgcn_raw_buffer_store_b16(bits, rc, off, 0, STORE_POLICY);
        }
      }
    };
#pragma unroll
    for (int bj = 0; bj < C::NBLK; ++bj) {
      const int col = block_col(bj) + frow;
      const uint32_t col_off = col < cols_valid ? (uint32_t)(col * OS) : OOB;
#pragma unroll
      for (int bi = 0; bi < C::MBLK; ++bi) {
        const uint32_t lane_off = col_off + (uint32_t)(block_row(bi) + 4 * fgrp) * pitch;
        if (beta != 0.f) store_block(bi, bj, lane_off, std::true_type{});
        else store_block(bi, bj, lane_off, std::false_type{});
      }
    }
  }
}

}  // namespace gensor
