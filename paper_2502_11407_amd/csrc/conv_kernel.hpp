// Convolution as an implicit GEMM with the input patch cached in LDS (the "cache" primitive
// applied to the halo tile): O = (I * K) downsampled by S on NCHW input and KCRS filters,
// cross-correlation with zero padding (operator table, Conv2d row).
//
// GEMM view: m = filter, n = (image, out row, out col), k = (filter row, filter col, channel)
// with the channel innermost.  One LDS stage holds BKC channels:
//   * the filters of this workgroup's BM rows as a k-contiguous tile [BM][R*S*BKC] (row
//     pitch an odd number of 16-byte chunks, so 16 consecutive rows fall in 16 different
//     bank groups).  In the KCRS tensor the BKC channels x R*S taps of one filter are one
//     contiguous run in (channel, tap) order, fetched with 16-byte vectors and reordered to
//     (tap, channel): for 3x3 filters in registers (a thread holds the 9 vectors of one filter
//     and channel group and byte-permutes them into 9 tile vectors), for 1x1 filters the two
//     orders coincide, any other filter goes through a raw LDS region and element reads;
//   * the input patch that the workgroup's BN output pixels touch, channel-last:
//     [patch row][patch col][BKC channels + 16 bytes pad].  A patch row is a row of the
//     zero-padded images stacked on top of each other; rows and columns outside an image are
//     never written and stay zero.  Global reads run along x (16 bytes per channel), an
//     8x8 (4x4 for fp32) register transpose turns them into channel-contiguous 16-byte
//     LDS writes, so every input element is fetched once per workgroup, not once per tap.
// A workgroup's pixels are BN consecutive (image, row, col) positions, or, when an output row is shorter
// than BN, a whole number of output rows (KernelArgs::cTilePx, chosen by the host): the patch then has
// no partial rows and the tile count can be matched to the compute units; waves whose columns lie
// beyond the tile's pixels only help with the staging.
// A lane's B fragment for tap (r, s) and channel chunk c is then ONE aligned 16-byte LDS
// read at  lane_base + (r*PW + s)*SLOT + c*16 : the tap is a scalar offset, there is no
// per-tap address arithmetic and no im2col buffer.
#pragma once
#include "gemm_kernel.hpp"

namespace gensor {

template <typename T_, typename OutT_, int BM_, int BN_, int BKC_, int WM_, int WN_, int MB_, int UNITS_, int LSTAGES_>
struct ConvCfg {
  typedef T_ T;
  typedef OutT_ OutT;
  static constexpr int BM = BM_, BN = BN_, BKC = BKC_, WM = WM_, WN = WN_, MB = MB_;
  static constexpr int ES = ElemSize<T>::value;
  static constexpr int EPC = 16 / ES;
  static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN, WAVES = WAVES_M * WAVES_N;
  static constexpr int THREADS = WAVES * 64;
  static constexpr int MBLK = WM / MB, NBLK = WN / MB;
  static constexpr int LANE_GROUPS = 64 / MB;
  static constexpr int KG = LANE_GROUPS * EPC;
  static constexpr int KSTEPS_C = BKC / KG;            // MFMA k steps per tap
  static constexpr int OCT = BKC / EPC;                // 16-byte channel groups per pixel
  static constexpr int SLOT = BKC * ES + 16;           // bytes per patch pixel
  static constexpr int RS_MAX = 9;                     // taps supported by the staging registers
  static constexpr int A_VEC_MAX = (BM * BKC * RS_MAX / EPC + THREADS - 1) / THREADS;
  static constexpr int U9_MAX = (BM * (BKC / EPC) + THREADS - 1) / THREADS;   // (filter, channel group) units per thread
  static constexpr int A_REGS = A_VEC_MAX > 9 * U9_MAX ? A_VEC_MAX : 9 * U9_MAX;
  static constexpr int UNITS_MAX = UNITS_;             // patch transpose units per thread and stage
  static constexpr int LSTAGES = LSTAGES_;             // LDS buffers: 1 or 2
  static_assert(LSTAGES == 1 || LSTAGES == 2, "one or two LDS stages");
  static_assert(BKC % KG == 0 && KSTEPS_C >= 1, "channel tile must hold whole fragment k groups");
  static_assert(BM % WM == 0 && BN % WN == 0 && WM % MB == 0 && WN % MB == 0, "tiles");
};

// Input of a strided pointwise convolution, compacted: out[plane][p][q] = in[plane][p*stride][q*stride]
// for plane = (image, channel).  16 / ES consecutive outputs per thread, one 16-byte store.
template <int ES>
__global__ __launch_bounds__(256) void subsample_input(const void* in, void* out, int64_t planes, int H, int W, int P, int Q,
                                                       int stride) {
  constexpr int EPC = 16 / ES;
  const int64_t PQ = (int64_t)P * Q;
  const int64_t total = planes * PQ;
  const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * EPC;
  if (i0 >= total) return;
  int64_t plane = i0 / PQ;
  int rem = (int)(i0 - plane * PQ);
  int p = rem / Q, q = rem - p * Q;
  u32x4 v = {0u, 0u, 0u, 0u};
  const int count = (int)(total - i0 < EPC ? total - i0 : EPC);
#pragma unroll
  for (int e = 0; e < EPC; ++e) {
    if (e < count) {
      const int64_t src = (plane * H + (int64_t)p * stride) * W + (int64_t)q * stride;
      if constexpr (ES == 4) v[e] = ((const uint32_t*)in)[src];
      else v[e >> 1] |= (uint32_t)((const uint16_t*)in)[src] << ((e & 1) * 16);
      if (++q == Q) { q = 0; if (++p == P) { p = 0; ++plane; } }
    }
  }
  if (count == EPC) {
    *(u32x4*)((char*)out + i0 * ES) = v;
  } else {
    for (int e = 0; e < count; ++e) {
      if constexpr (ES == 4) ((uint32_t*)out)[i0 + e] = v[e];
      else ((uint16_t*)out)[i0 + e] = (uint16_t)(v[e >> 1] >> ((e & 1) * 16));
    }
  }
}

// FMODE, how the filters are reordered on the way into the tile, is a template parameter: with all
// three routes in one kernel the register allocation is the union of theirs (250 VGPRs, spills to
// scratch) and every convolution shape measured ran 14 % slower.
template <typename C, int FMODE, bool THROUGH, bool TAIL>
__global__ __launch_bounds__(C::THREADS) void conv_patch_kernel(const KernelArgs args) {
  typedef typename C::T T;
  typedef Mfma<T, C::MB> MF;
  typedef typename MF::Acc Acc;
  constexpr int ES = C::ES, EPC = C::EPC, BM = C::BM, BN = C::BN, BKC = C::BKC, MB = C::MB, SLOT = C::SLOT;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  GENSOR_LDS char* lds = (GENSOR_LDS char*)smem;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave / C::WAVES_N;
  const int wave_n = wave % C::WAVES_N;

  // workgroup -> (filter tile, pixel tile): contiguous tile ranges per XCD, panels of tile rows
  const int total = args.tiles_m * args.tiles_n;
  int wg = blockIdx.x;
  if ((total & 7) == 0) wg = (wg & 7) * (total >> 3) + (wg >> 3);
  int tile_m, tile_n;
  {
    const int panel = args.panel;
    const int per_panel = panel * args.tiles_n;
    const int pi = wg / per_panel;
    const int rows_here = min(panel, args.tiles_m - pi * panel);
    const int r = wg - pi * per_panel;
    tile_m = pi * panel + r % rows_here;
    tile_n = r / rows_here;
  }
  const int m0 = tile_m * BM, n0 = tile_n * args.cTilePx;
  const int n_end = min(args.N, n0 + args.cTilePx);        // columns of the tile at or beyond it belong to the next workgroup

  // geometry
  const int Cc = args.cC, H = args.cH, W = args.cW, R = args.cR, S = args.cS, P = args.cP, Q = args.cQ;
  const int stride = args.cStride, pad = args.cPad, NI = args.cN;
  const int RS = R * S, PQ = P * Q;
  const int Hp = H + 2 * pad, PW = W + 2 * pad;
  const int HW = H * W;
  const int a_pitch = args.cApitch;            // bytes per filter row in LDS
  const int patch_rows = args.cPatchRows;
  const int stage_bytes = args.cStageBytes;
  const int a_bytes = BM * a_pitch;
  const int raw_pitch = RS * BKC * ES;         // bytes of one filter's (channel, tap) run per stage; a multiple of 16
  GENSOR_LDS char* raw = lds + C::LSTAGES * stage_bytes;   // raw filter runs, one buffer after the stages
  const int g_first = n0 / Q;                  // first stacked output row of this tile
  const int R0 = (g_first / P) * Hp + (g_first % P) * stride;   // first stacked padded input row

  constexpr uint32_t RSRC_FLAGS = 0x00020000u, OOB = 0x80000000u;
  const __amdgpu_buffer_rsrc_t rs_in = __builtin_amdgcn_make_buffer_rsrc((void*)args.B, 0, (uint32_t)args.cInBytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void*)args.A, 0, (uint32_t)args.cWBytes, RSRC_FLAGS);

  Acc acc[C::MBLK][C::NBLK];
#pragma unroll
  for (int i = 0; i < C::MBLK; ++i)
#pragma unroll
    for (int j = 0; j < C::NBLK; ++j)
#pragma unroll
      for (int v = 0; v < MF::NACC; ++v) acc[i][j][v] = 0.f;

  // ---- filter staging plan.  fmode 2 (3x3): unit u of this thread is one (filter row, channel
  // group): 9 contiguous 16-byte pieces in, 9 tile vectors out, permuted in registers.
  // fmode 1 (1x1) and 0 (other): vector v of this thread is, on the way in, the v-th 16-byte
  // piece of a filter row's contiguous (channel, tap) run of this stage and, on the way out,
  // one 16-byte channel group of one tap of a filter row of the tile.
  constexpr int fmode = FMODE;                       // 2: R*S = 9, 1: R*S = 1, 0: anything else (the launcher picks)
  const int a_vec_per_row = RS * C::OCT;
  const int a_vecs = BM * a_vec_per_row;
  constexpr int a_units = BM * C::OCT;
  int a_goff[C::A_VEC_MAX];        // element offset of the piece (fmode 2: of the unit) at channel tile 0, or -1
  u32x4 a_reg[C::A_REGS];
#pragma unroll
  for (int v = 0; v < C::A_VEC_MAX; ++v) {
    const int q = tid + v * C::THREADS;
    if (fmode == 2) {
      // units are dealt from the last thread down: the patch units start at thread 0, so the
      // two kinds of loads land on different waves
      const int qu = (C::THREADS - 1 - tid) + v * C::THREADS;
      const int row = qu / C::OCT, oct = qu - row * C::OCT;
      const bool ok = v < C::U9_MAX && qu < a_units && (m0 + row) < args.M;
      a_goff[v] = ok ? ((m0 + row) * Cc + oct * EPC) * 9 : -1;
    } else {
      const int row = q / a_vec_per_row, t = q - row * a_vec_per_row;
      const bool ok = q < a_vecs && (m0 + row) < args.M;
      a_goff[v] = ok ? (m0 + row) * Cc * RS + t * EPC : -1;
    }
  }
  auto fetch_a = [&](int c0) {
    if (fmode == 2) {
#pragma unroll
      for (int u = 0; u < C::U9_MAX; ++u) {
        if ((C::THREADS - 64 - wave * 64) + u * C::THREADS >= a_units) continue;      // no lane of this wave holds a unit
        const int oct = ((C::THREADS - 1 - tid) + u * C::THREADS) % C::OCT;
        const bool ok = a_goff[u] >= 0 && c0 + oct * EPC < Cc;
        // one select per unit: an offset at or above OOB stays out of range when the piece offsets are added
        const uint32_t first = ok ? (uint32_t)((a_goff[u] + c0 * 9) * ES) : OOB;
#pragma unroll
        for (int i = 0; i < 9; ++i) a_reg[u * 9 + i] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, first + (uint32_t)(i * 16), 0, 0);
      }
    } else {
#pragma unroll
      for (int v = 0; v < C::A_VEC_MAX; ++v) {
        if (wave * 64 + v * C::THREADS >= a_vecs) continue;                            // no lane of this wave holds a piece
        // a piece starts at channel c0 + (t*EPC)/RS of the run; pieces are wholly inside or wholly
        // beyond the channels that exist (C and the channel tile are multiples of EPC)
        const int t = (tid + v * C::THREADS) % a_vec_per_row;
        const bool ok = a_goff[v] >= 0 && c0 + (t * EPC) / RS < Cc;
        a_reg[v] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, ok ? (uint32_t)((a_goff[v] + c0 * RS) * ES) : OOB, 0, 0);
      }
    }
  };
  fetch_a(0);                      // the first stage's loads go out before the rest of the set-up
  // fmode 2: element (channel c, tap rs) of a unit is element c*9 + rs of its 9 pieces
  auto commit_a9 = [&](int st) {
    GENSOR_LDS char* base = lds + st * stage_bytes;
#pragma unroll
    for (int u = 0; u < C::U9_MAX; ++u) {
      const int q = (C::THREADS - 1 - tid) + u * C::THREADS;
      if (q >= a_units) break;
      const int row = q / C::OCT, oct = q - row * C::OCT;
#pragma unroll
      for (int rs = 0; rs < 9; ++rs) {
        u32x4 o;
        if constexpr (ES == 4) {
#pragma unroll
          for (int c = 0; c < 4; ++c) o[c] = a_reg[u * 9 + (c * 9 + rs) / 4][(c * 9 + rs) % 4];
        } else {
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const int e0 = (2 * d) * 9 + rs, e1 = (2 * d + 1) * 9 + rs;      // the two elements of dword d
            const uint32_t lo = a_reg[u * 9 + e0 / 8][(e0 % 8) / 2], hi = a_reg[u * 9 + e1 / 8][(e1 % 8) / 2];
            o[d] = __builtin_amdgcn_perm(hi, lo, ((e1 & 1) ? 0x07060000u : 0x05040000u) | ((e0 & 1) ? 0x0302u : 0x0100u));
          }
        }
        *(GENSOR_LDS u32x4*)(base + row * a_pitch + (rs * C::OCT + oct) * 16) = o;
      }
    }
  };
  // fmode 1: the run is the tile row
  auto commit_a1 = [&](int st) {
    GENSOR_LDS char* base = lds + st * stage_bytes;
#pragma unroll
    for (int v = 0; v < C::A_VEC_MAX; ++v) {
      const int q = tid + v * C::THREADS;
      if (q >= a_vecs) break;
      const int row = q / a_vec_per_row, t = q - row * a_vec_per_row;
      *(GENSOR_LDS u32x4*)(base + row * a_pitch + t * 16) = a_reg[v];
    }
  };
  auto commit_raw = [&]() {
#pragma unroll
    for (int v = 0; v < C::A_VEC_MAX; ++v) {
      const int q = tid + v * C::THREADS;
      if (q >= a_vecs) break;
      *(GENSOR_LDS u32x4*)(raw + q * 16) = a_reg[v];      // row * raw_pitch + t * 16 = q * 16
    }
  };
  // fmode 0: raw (channel, tap) runs -> tile rows in (tap, channel) order
  auto permute_a = [&](int st) {
    GENSOR_LDS char* base = lds + st * stage_bytes;
#pragma unroll
    for (int v = 0; v < C::A_VEC_MAX; ++v) {
      const int q = tid + v * C::THREADS;
      if (q >= a_vecs) break;
      const int row = q / a_vec_per_row, t = q - row * a_vec_per_row;
      const int rs = t / C::OCT, oct = t - rs * C::OCT;
      GENSOR_LDS char* src = raw + row * raw_pitch + (oct * EPC * RS + rs) * ES;
      u32x4 o;
      if constexpr (ES == 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = *(GENSOR_LDS uint32_t*)(src + j * RS * 4);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          o[j] = (uint32_t)*(GENSOR_LDS uint16_t*)(src + (2 * j) * RS * 2) |
                 ((uint32_t)*(GENSOR_LDS uint16_t*)(src + (2 * j + 1) * RS * 2) << 16);
      }
      *(GENSOR_LDS u32x4*)(base + row * a_pitch + t * 16) = o;
    }
  };
  // filters of the fetched stage into tile `st`; with fmode 0 in two steps around a barrier
  auto commit_a_direct = [&](int st) {
    if (fmode == 2) commit_a9(st);
    else if (fmode == 1) commit_a1(st);
  };

  // ---- patch staging plan.  A unit is EPC channels x EPC consecutive x of one patch row.  Units are dealt
  // channel group first, then patch row, then x segment: the 16 lanes of a 16-byte LDS write then differ in
  // channel group (16 bytes) and row (the row pitch, an odd multiple of 32 bytes modulo 256 for the usual
  // widths) and fall into different banks, where lanes that differ in x segment (8 pixels = 384 bytes) share
  // them four ways (measured: 2-4 % on the 3x3 layers).
  const int w_segs = (W + EPC - 1) / EPC;
  const int units = patch_rows * w_segs * C::OCT;
  int u_goff[C::UNITS_MAX];        // element offset of (img, channel group, y, x segment) at channel tile 0, or -1
  int u_dst[C::UNITS_MAX];         // LDS byte offset of the unit's first pixel and channel group
  int u_nx[C::UNITS_MAX];          // valid x in the segment
  u32x4 u_reg[C::UNITS_MAX][C::EPC];
#pragma unroll
  for (int u = 0; u < C::UNITS_MAX; ++u) {
    const int q = tid + u * C::THREADS;
    const int oct = q % C::OCT, t = q / C::OCT;
    const int j = t % patch_rows, seg = t / patch_rows;
    const int srow = R0 + j;                       // stacked padded row
    const int img = srow / Hp, y = srow - img * Hp - pad;
    const bool ok = q < units && img < NI && y >= 0 && y < H;
    u_goff[u] = ok ? ((img * Cc + oct * EPC) * H + y) * W + seg * EPC : -1;
    u_dst[u] = (j * PW + pad + seg * EPC) * SLOT + oct * 16;
    u_nx[u] = min(EPC, W - seg * EPC);
  }
  // TAIL: a vector can run past the end of the tensor when rows are not whole vectors.  The buffer's range check
  // works dword by dword and returns the part inside, unless the vector starts off a dword boundary (16-bit
  // elements and an odd row length): only then is the kernel instantiated with the element-wise fetch of the
  // tensor's last vector (the launch decides), and every other shape runs loads without a test in front of each.
  auto fetch_patch = [&](int c0) {
#pragma unroll
    for (int u = 0; u < C::UNITS_MAX; ++u) {
      if (wave * 64 + u * C::THREADS >= units) continue;                               // no lane of this wave holds a unit
      // a channel group at or beyond C reads as zero (C is a multiple of the group size)
      const int oct = (tid + u * C::THREADS) % C::OCT;
      const bool ok = u_goff[u] >= 0 && c0 + oct * EPC < Cc;
      const uint32_t first = ok ? (uint32_t)((u_goff[u] + c0 * HW) * ES) : OOB;      // as for the filters: one select per unit
#pragma unroll
      for (int i = 0; i < EPC; ++i) {
        const uint32_t off = first + (uint32_t)(i * HW * ES);
        if (TAIL && ok && off + 16u > (uint32_t)args.cInBytes) {
          // the very last vector of the tensor: a 16-byte read would leave the buffer, which
          // drops the valid part when the start is not dword aligned; fetch element-wise
          u32x4 v = {0u, 0u, 0u, 0u};
          for (int e = 0; e < EPC; ++e) {
            const uint32_t eo = off + e * ES;
            if (eo + ES <= (uint32_t)args.cInBytes) {
              if constexpr (ES == 4) v[e] = ((const uint32_t*)args.B)[eo / 4];
              else v[e >> 1] |= (uint32_t)((const uint16_t*)args.B)[eo / 2] << ((e & 1) * 16);
            }
          }
          u_reg[u][i] = v;
        } else {
          u_reg[u][i] = __builtin_amdgcn_raw_buffer_load_b128(rs_in, off, 0, 0);
        }
      }
    }
  };
  fetch_patch(0);
  auto commit_patch = [&](int st) {
    GENSOR_LDS char* base = lds + st * stage_bytes + a_bytes;
#pragma unroll
    for (int u = 0; u < C::UNITS_MAX; ++u) {
      if (u_goff[u] < 0) continue;                 // rows outside an image stay zero
#pragma unroll
      for (int x = 0; x < EPC; ++x) {
        u32x4 o;                                   // channels i = 0..EPC-1 of pixel x
        if constexpr (ES == 4) {
#pragma unroll
          for (int i = 0; i < 4; ++i) o[i] = u_reg[u][i][x];
        } else {
          // 8x8 transpose of 16-bit elements: dword d of the output pairs channels 2d, 2d+1
#pragma unroll
          for (int d = 0; d < 4; ++d)
            o[d] = __builtin_amdgcn_perm(u_reg[u][2 * d + 1][x >> 1], u_reg[u][2 * d][x >> 1],
                                         (x & 1) ? 0x07060302u : 0x05040100u);
        }
        if (x < u_nx[u]) *(GENSOR_LDS u32x4*)(base + u_dst[u] + x * SLOT) = o;
      }
    }
  };

  // ---- fragment addressing
  const int frow = lane % MB, fgrp = lane / MB;
  auto block_row = [&](int bi) { return wave_m * C::WM + bi * MB; };
  auto block_col = [&](int bj) { return wave_n * C::WN + bj * MB; };
  int b_base[C::NBLK];             // byte offset of the lane's pixel (tap 0,0) inside the patch
#pragma unroll
  for (int bj = 0; bj < C::NBLK; ++bj) {
    int n = n0 + block_col(bj) + frow;
    n = n < n_end ? n : n_end - 1;
    const int g = n / Q, q = n - g * Q;
    const int img = g / P, p = g - img * P;
    b_base[bj] = ((img * Hp + p * stride - R0) * PW + q * stride) * SLOT;
  }
  // One tap = KSTEPS_C fragment reads per block and the MFMAs on them.  The taps run as a
  // flat loop, two per trip, with the fragments of the next tap in flight under the MFMAs
  // of this one (two register sets).
  u32x4 af[2][C::KSTEPS_C][C::MBLK], bf[2][C::KSTEPS_C][C::NBLK];
  auto compute = [&](int st) {
    GENSOR_LDS char* abase = lds + st * stage_bytes;
    GENSOR_LDS char* pbase = abase + a_bytes;
    auto read_tap = [&](int buf, int r, int s2) {
      const int tap = (r * PW + s2) * SLOT;
      const int rs = r * S + s2;
#pragma unroll
      for (int ks = 0; ks < C::KSTEPS_C; ++ks) {
        const int ch = ks * C::LANE_GROUPS + fgrp;
#pragma unroll
        for (int bi = 0; bi < C::MBLK; ++bi)
          af[buf][ks][bi] = *(GENSOR_LDS u32x4*)(abase + (block_row(bi) + frow) * a_pitch + (rs * C::OCT + ch) * 16);
#pragma unroll
        for (int bj = 0; bj < C::NBLK; ++bj) bf[buf][ks][bj] = *(GENSOR_LDS u32x4*)(pbase + b_base[bj] + tap + ch * 16);
      }
    };
    auto mma_tap = [&](int buf) {
#pragma unroll
      for (int ks = 0; ks < C::KSTEPS_C; ++ks)
#pragma unroll
        for (int bi = 0; bi < C::MBLK; ++bi)
#pragma unroll
          for (int bj = 0; bj < C::NBLK; ++bj) MF::run(af[buf][ks][bi], bf[buf][ks][bj], acc[bi][bj]);
    };
    if (n0 + wave_n * C::WN >= n_end) return;            // a wave whose columns all lie beyond the tile's pixels
    int r = 0, s2 = 0;                                  // the next tap to read
    auto advance = [&]() { if (++s2 == S) { s2 = 0; ++r; } };
    read_tap(0, 0, 0);
    advance();
    // branch-free body: two taps per trip; the last one or two taps are peeled off
    const int pairs = (RS - 1) >> 1;
    for (int i = 0; i < pairs; ++i) {
      read_tap(1, r, s2);
      advance();
      mma_tap(0);
      read_tap(0, r, s2);
      advance();
      mma_tap(1);
    }
    if (RS - 2 * pairs == 2) {
      read_tap(1, r, s2);
      mma_tap(0);
      mma_tap(1);
    } else {
      mma_tap(0);
    }
  };

  const int nstages = (Cc + BKC - 1) / BKC;
  // ---- zero the patch buffers once (under the first loads): cells outside the images are
  // never written again
  {
    const u32x4 z = {0u, 0u, 0u, 0u};
    const int patch_bytes = stage_bytes - a_bytes;
    for (int st = 0; st < C::LSTAGES; ++st)
      for (int o = tid * 16; o < patch_bytes; o += C::THREADS * 16) *(GENSOR_LDS u32x4*)(lds + st * stage_bytes + a_bytes + o) = z;
  }
  if (fmode == 0) {
    commit_raw();
    __syncthreads();
    permute_a(0);
  } else {
    __syncthreads();                   // the zero fill before the first patch writes
    commit_a_direct(0);
  }
  commit_patch(0);
  __syncthreads();
  for (int st = 0; st < nstages; ++st) {
    const bool more = st + 1 < nstages;
    const int cur = C::LSTAGES == 2 ? (st & 1) : 0, nxt = C::LSTAGES == 2 ? (cur ^ 1) : 0;
    if (more) {
      fetch_a((st + 1) * BKC);
      fetch_patch((st + 1) * BKC);
    }
    compute(cur);
    if (more) {
      if (fmode == 0) {
        commit_raw();                  // the raw region is not read by compute
        if constexpr (C::LSTAGES == 2) commit_patch(nxt);
        __syncthreads();               // raw runs visible; with one stage: everyone has finished reading it
        permute_a(nxt);
        if constexpr (C::LSTAGES == 1) commit_patch(nxt);
      } else {
        if constexpr (C::LSTAGES == 1) __syncthreads();     // everyone has finished reading the single stage
        commit_a_direct(nxt);
        commit_patch(nxt);
      }
    }
    __syncthreads();
  }

  // ---- epilogue: O[img][filter][p][q], row = filter, column = (img, p, q)
  typedef typename C::OutT OutT;
  constexpr int OS = ElemSize<OutT>::value;
  const __amdgpu_buffer_rsrc_t rs_out = __builtin_amdgcn_make_buffer_rsrc((void*)args.C, 0, (uint32_t)args.cOutBytes, RSRC_FLAGS);
  // Cache policy of the stores (an immediate of the instruction, hence a template parameter; a run-time
  // branch over two copies of the loop cost 1-4 %): write-through for a shallow reduction, where the stores
  // are a large share of the launch (64 channels x 3x3, 64 filters: 17.9 -> 15.6 us), write-back for a deep
  // one, where the L2 drains them under the next tile's work (reductions of 1152 and 2304: write-through
  // measured 1.5-2.5 % slower).
  if (n0 + wave_n * C::WN < n_end) {
    constexpr int POLICY = THROUGH ? 16 : 0;
#pragma unroll
    for (int bj = 0; bj < C::NBLK; ++bj) {
      const int col = n0 + block_col(bj) + frow;
      const int img = col / PQ;
      const int cbase = img * args.M * PQ + (col - img * PQ);
#pragma unroll
      for (int bi = 0; bi < C::MBLK; ++bi)
#pragma unroll
        for (int v = 0; v < MF::NACC; ++v) {
          const int rr = (MB == 32) ? 8 * (v / 4) + 4 * fgrp + (v % 4) : 4 * fgrp + v;
          const int row = m0 + block_row(bi) + rr;
          const uint32_t off = (row < args.M && col < n_end) ? (uint32_t)((cbase + row * PQ) * OS) : OOB;
          const float val = acc[bi][bj][v];
          if constexpr (OS == 4) {
            __builtin_amdgcn_raw_buffer_store_b32(as_u32(val), rs_out, off, 0, POLICY);
          } else {
            uint16_t bits;
            store_out<OutT>(&bits, 0, val);
            __builtin_amdgcn_raw_buffer_store_b16(bits, rs_out, off, 0, POLICY);
          }
        }
    }
  }
}

}  // namespace gensor
