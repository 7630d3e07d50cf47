// Schedule constructor: the paper's construction-graph walk (Section IV, Algorithms 1 and 2,
// benefit formulas Eq. 1-3) on the host, followed by an analytical MI355X cost model that
// ranks the complete states the walks end in and returns the best compiled instance.
//
// State (Section IV-A): tile[d] = [T_2, T_1, T_0] for d = m, n, k of the GEMM view, the
// virtual threads V for m and n (interleave depth of that operand's LDS tile), and the memory
// level being scheduled (0: T_2 / LDS, 1: T_1 / registers, 2: complete).  Actions: tile
// (double), invTile (halve), setVThread (V doubles, wrapping to 1 past the conflict-free
// depth), cache (next level).
//
// Where the paper leaves a quantity open this file takes these readings:
//   * Q and F of Eq. 1 -- level 0: Q = e M N K (1/T_m + 1/T_n) + e_out M N, F = e T_k (T_m + T_n);
//     level 1: Q = e B_m B_n B_k (1/T_m + 1/T_n), F = 4 T_m T_n + e T_k (T_m + T_n).
//   * Eq. 2 -- S is F of the current tile; L and B come from gensor_hw, B shared per CU.
//   * Eq. 3 -- W = banks * bank bytes, what the LDS serves per cycle.  x = the bytes of bank address
//     space spanned by the rows that one quarter wave reads together from the operand tile of
//     dimension d: 16 rows of min(T_2[k] e, W) bytes for a k-contiguous tile, the 4 (16-bit) or 2
//     (fp32) k rows of an n-contiguous B (or m-contiguous A) tile at W each.  ceil(x / (V W)) of those rows share a bank
//     when the tile is interleaved over V phases (V = 1: the plain layout).  setVThread doubles V
//     up to ceil(x / W), where the reads are conflict-free, then wraps to 1; the benefit is the
//     ratio of the conflict ways before and after, so the wrap has a (small) positive benefit.
//   * The cache entry is multiplied by 3 / (1 + exp(-(ln 5 / 10)(t - 10))) with
//     t = -log2(T_l); T_l is a per-level temperature that starts at T0, halves each step
//     and restarts when cache fires.  The loop's own T halves each step and ends the walk.
//   * Chain number c starts from T0 / 2^(c mod 31) (colder walks end in smaller tiles).
//   * Keep rule: every visited register-level state whose workgroup fits the wave limit is
//     kept in its completed form (policy 0), or with the printed probability (policy 1).
//   * Memory check: a transition that leaves the lattice or exceeds LDS (two stages),
//     registers per lane, or (for the last cache) waves per workgroup has probability 0.
//   * Roulette: first index whose cumulative probability exceeds u.
// Random numbers are a counter-based generator (splitmix64 finaliser), so a walk is a pure
// function of (problem, hw, opts, seed, chain).
#include <chrono>
#include <cmath>
#include <cstring>
#include <set>
#include <vector>

#include "host_common.hpp"

namespace gensor {
namespace {

enum { ACT_TILE = 0, ACT_INVTILE = 1, ACT_SETVTHREAD = 2, ACT_CACHE = 3 };
struct ActionSlot { int action, dim; };
const ActionSlot kSlots[9] = {{ACT_TILE, 0}, {ACT_TILE, 1}, {ACT_TILE, 2}, {ACT_INVTILE, 0}, {ACT_INVTILE, 1},
                              {ACT_INVTILE, 2}, {ACT_SETVTHREAD, 0}, {ACT_SETVTHREAD, 1}, {ACT_CACHE, -1}};

struct Etir {
  int tile[3][3];
  int v[2];
  int level;
  bool operator<(const Etir& o) const { return std::memcmp(this, &o, sizeof(Etir)) < 0; }
};

struct Ctx {
  GemmView view;
  gensor_hw hw;
  gensor_construct_opts opts;
  int g;          // fragment k granule: 16 elements for 16-bit inputs, 8 for fp32
  int cap[3];
};

const gensor_hw kMi355x = {
    256, 4, 64, 16, 163840, 512, 64, 4, 2.4,
    {800.0, 64.0, 4.0},
    {8000.0, 157286.4, 1258291.2},
    20000.0, 2516.6, 157.3, 2.0};

double uniform01(uint64_t seed, uint64_t chain, uint64_t step, uint64_t j) {
  uint64_t s = seed + 0x9E3779B97F4A7C15ull * (chain * 4096ull + 2ull * step + j + 1ull);
  uint64_t z = (s ^ (s >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z = z ^ (z >> 31);
  return (double)(z >> 11) * (1.0 / 9007199254740992.0);
}

int next_pow2(int64_t x) {
  int p = 1;
  while (p < x) p *= 2;
  return p;
}

void make_ctx(const GemmView& v, const gensor_hw* hw, const gensor_construct_opts* o, Ctx* c) {
  c->view = v;
  c->hw = hw ? *hw : kMi355x;
  gensor_construct_opts d = {std::ldexp(1.0, 30), std::ldexp(1.0, -70), 16384, 0, 0, 0, 0, 0};
  if (o) {
    if (o->T0 > 0) d.T0 = o->T0;
    if (o->threshold > 0) d.threshold = o->threshold;
    if (o->chains > 0) d.chains = o->chains;
    d.keep_policy = o->keep_policy;
    d.tiling_benefit = o->tiling_benefit;
    d.no_vthread = o->no_vthread;
    d.no_split_k = o->no_split_k;
    d.greedy = o->greedy;
  }
  c->opts = d;
  c->g = v.esize == 2 ? 16 : 8;
  auto clampi = [](int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); };
  c->cap[0] = clampi(next_pow2(v.M), 16, 256);
  c->cap[1] = clampi(next_pow2(v.N), 16, 256);
  c->cap[2] = clampi(next_pow2(v.K), 2 * c->g, 8 * c->g);
}

Etir initial_state(const Ctx& c) {
  Etir e;
  for (int d = 0; d < 2; ++d)
    for (int l = 0; l < 3; ++l) e.tile[d][l] = 16;
  for (int l = 0; l < 3; ++l) e.tile[2][l] = 2 * c.g;
  e.v[0] = e.v[1] = 1;
  e.level = 0;
  return e;
}

int mfma_block(const Ctx& c, const Etir& e) { return e.tile[2][1] == c.g ? 32 : 16; }

// Eq. 3: bank-conflict ways of the fragment reads of operand d (0: the m x k tile, 1: the k x n tile)
// of a workgroup tile of k depth bk whose rows are interleaved over v phases.
int conflict_ways(const GemmView& view, const gensor_hw& hw, int bk, int d, int v) {
  const int W = hw.lds_banks * hw.lds_bank_bytes;
  const bool k_contiguous = d == 0 ? view.asrc == A_KC : view.bsrc == B_KC;
  const int row_bytes = bk * view.esize;
  const int x = k_contiguous ? 16 * (row_bytes < W ? row_bytes : W) : (view.esize == 2 ? 4 : 2) * W;
  return (x + v * W - 1) / (v * W);
}
int wave_count(const Etir& e) { return (e.tile[0][0] / e.tile[0][1]) * (e.tile[1][0] / e.tile[1][1]); }

// memory footprint F and traffic Q of Eq. 1 at a level
double footprint(const Ctx& c, const Etir& e, int level) {
  const int tm = e.tile[0][level], tn = e.tile[1][level], tk = e.tile[2][level];
  if (level == 0) return (double)(c.view.esize * tk * (tm + tn));
  return (double)(4 * tm * tn + c.view.esize * tk * (tm + tn));
}
double traffic(const Ctx& c, const Etir& e, int level) {
  const double tm = e.tile[0][level], tn = e.tile[1][level];
  if (level == 0)
    return (double)c.view.esize * (double)c.view.M * (double)c.view.N * (double)c.view.K * (1.0 / tm + 1.0 / tn) +
           (double)c.view.osize * (double)c.view.M * (double)c.view.N;
  return (double)c.view.esize * (double)e.tile[0][0] * (double)e.tile[1][0] * (double)e.tile[2][0] * (1.0 / tm + 1.0 / tn);
}

// lattice membership + the memory check
bool valid(const Ctx& c, const Etir& e) {
  for (int d = 0; d < 2; ++d)
    if (e.tile[d][0] < 16 || e.tile[d][0] > c.cap[d]) return false;
  if (e.tile[2][0] < 2 * c.g || e.tile[2][0] > c.cap[2]) return false;
  if (2 * c.view.esize * e.tile[2][0] * (e.tile[0][0] + e.tile[1][0]) > c.hw.lds_bytes_per_cu) return false;
  if (e.level >= 1) {
    if ((e.tile[2][1] != c.g && e.tile[2][1] != 2 * c.g) || e.tile[2][1] > e.tile[2][0]) return false;
    const int mb = mfma_block(c, e);
    for (int d = 0; d < 2; ++d) {
      if (e.v[d] < 1 || (e.v[d] & (e.v[d] - 1)) != 0 || e.v[d] > conflict_ways(c.view, c.hw, e.tile[2][0], d, 1)) return false;
      if (e.tile[d][1] > e.tile[d][0] || e.tile[d][1] < 16 || e.tile[d][1] % mb != 0) return false;
    }
    const int regs = e.tile[0][1] * e.tile[1][1] / 64 + 2 * (e.tile[0][1] + e.tile[1][1]) * e.tile[2][1] * c.view.esize / 256;
    if (regs > c.hw.regs_per_lane) return false;
  }
  return true;
}

Etir apply_action(const Ctx& c, const Etir& e, int action, int d) {
  Etir n = e;
  switch (action) {
    case ACT_TILE: n.tile[d][e.level] *= 2; break;
    case ACT_INVTILE: n.tile[d][e.level] /= 2; break;
    case ACT_SETVTHREAD: {
      int nv = e.v[d] * 2;
      if (nv > conflict_ways(c.view, c.hw, e.tile[2][0], d, 1)) nv = 1;
      n.v[d] = nv;
      break;
    }
    case ACT_CACHE:
      n.level = e.level + 1;
      if (e.level == 0) { n.tile[0][1] = 16; n.tile[1][1] = 16; n.tile[2][1] = 2 * c.g; }
      break;
  }
  if (n.level >= 1) {
    n.tile[0][2] = n.tile[0][1] / n.v[0] > 0 ? n.tile[0][1] / n.v[0] : 1;
    n.tile[1][2] = n.tile[1][1] / n.v[1] > 0 ? n.tile[1][1] / n.v[1] : 1;
    n.tile[2][2] = n.tile[2][1];
  }
  return n;
}

double benefit_tiling(const Ctx& c, const Etir& e, const Etir& n) {       // Eq. 1
  const double q0 = traffic(c, e, e.level), q1 = traffic(c, n, e.level);
  const double f0 = footprint(c, e, e.level), f1 = footprint(c, n, e.level);
  if (c.opts.tiling_benefit == 1) return (q0 * f0) / (q1 * f1);
  return (q0 * f1) / (q1 * f0);
}
double benefit_caching(const Ctx& c, const Etir& e) {                      // Eq. 2
  const int lo = e.level, hi = e.level + 1;
  const double S = footprint(c, e, e.level);
  const double b_lo = c.hw.bandwidth_gbs[lo] / c.hw.compute_units;
  const double b_hi = c.hw.bandwidth_gbs[hi] / c.hw.compute_units;
  return (c.hw.latency_ns[lo] + S / b_lo) / (c.hw.latency_ns[hi] + S / b_hi);
}
double benefit_vthread(const Ctx& c, const Etir& e, const Etir& n, int d) {  // Eq. 3
  return (double)conflict_ways(c.view, c.hw, e.tile[2][0], d, e.v[d]) / (double)conflict_ways(c.view, c.hw, e.tile[2][0], d, n.v[d]);
}
double annealing_factor(double t) { return 3.0 / (1.0 + std::exp(-(std::log(5.0) / 10.0) * (t - 10.0))); }
double keep_probability(double T) { return 1.0 - 1.0 / (1.0 + std::exp(-0.5 * (-std::log(T) - 10.0))); }

// Algorithm 2: benefits of every (action, dim), normalised, roulette.  Returns the slot or -1.
int prog_policy(const Ctx& c, const Etir& e, double T_level, double u, double probs[9]) {
  double total = 0.0;
  for (int i = 0; i < 9; ++i) {
    const ActionSlot s = kSlots[i];
    double b = 0.0;
    if (s.action == ACT_TILE || s.action == ACT_INVTILE) {
      const Etir n = apply_action(c, e, s.action, s.dim);
      if (valid(c, n)) b = benefit_tiling(c, e, n);
    } else if (s.action == ACT_SETVTHREAD) {
      if (e.level == 1 && !c.opts.no_vthread) {
        const Etir n = apply_action(c, e, s.action, s.dim);
        if (n.v[s.dim] != e.v[s.dim] && valid(c, n)) b = benefit_vthread(c, e, n, s.dim);
      }
    } else {
      const bool ok = !(e.level == 1 && wave_count(e) > c.hw.max_waves_per_wg);
      if (ok) b = benefit_caching(c, e) * annealing_factor(-std::log2(T_level));
    }
    probs[i] = b;
    total += b;
  }
  if (total <= 0.0) {
    for (int i = 0; i < 9; ++i) probs[i] = 0.0;
    return -1;
  }
  for (int i = 0; i < 9; ++i) probs[i] = probs[i] / total;
  if (c.opts.greedy) {                       // the first action of largest probability, no draw
    int top = 0;
    for (int i = 1; i < 9; ++i)
      if (probs[i] > probs[top]) top = i;
    return top;
  }
  double acc = 0.0;
  int last = -1;
  for (int i = 0; i < 9; ++i) {
    if (probs[i] > 0.0) last = i;
    acc += probs[i];
    if (probs[i] > 0.0 && u < acc) return i;
  }
  return last;
}

struct Trace { int32_t capacity, steps; int32_t *actions, *dims, *states; };

// Algorithm 1 for one chain.  Appends kept complete states to `kept`; returns the number of steps.
int run_walk(const Ctx& c, uint64_t seed, uint64_t chain, std::vector<Etir>* kept, Trace* tr) {
  Etir e = initial_state(c);
  const double T0 = c.opts.T0 / std::ldexp(1.0, (int)(chain % 31));   // temperature ladder over the chains
  double T = T0, T_level = T0;
  int step = 0;
  while (T > c.opts.threshold && e.level < 2) {
    double probs[9];
    const int slot = prog_policy(c, e, T_level, uniform01(seed, chain, step, 0), probs);
    if (slot < 0) break;
    const Etir n = apply_action(c, e, kSlots[slot].action, kSlots[slot].dim);
    if (tr && step < tr->capacity) {
      tr->actions[step] = kSlots[slot].action;
      tr->dims[step] = kSlots[slot].dim;
      int32_t* o = tr->states + 12 * step;
      for (int d = 0; d < 3; ++d)
        for (int l = 0; l < 3; ++l) o[3 * d + l] = n.tile[d][l];
      o[9] = n.v[0]; o[10] = n.v[1]; o[11] = n.level;
    }
    // every visited register-level state that may stop here is a complete program
    if (kept && (n.level == 2 || (n.level == 1 && wave_count(n) <= c.hw.max_waves_per_wg)))
      if (c.opts.keep_policy == 0 || uniform01(seed, chain, step, 1) < keep_probability(T))
        kept->push_back(n.level == 2 ? n : apply_action(c, n, ACT_CACHE, -1));
    e = n;
    T = T / 2.0;
    T_level = kSlots[slot].action == ACT_CACHE ? T0 : T_level / 2.0;
    ++step;
  }
  if (tr) tr->steps = step < tr->capacity ? step : tr->capacity;
  return step;
}

// ---------------------------------------------------------------------------------------
// Analytical cost model: per-CU pipeline limits (MFMA issue, LDS traffic, operand feed from
// L2) scaled by how many tiles the busiest CU owns, an epilogue that streams C, bounded
// below by total HBM traffic, plus launch cost.  Microseconds; negative = infeasible.
// ---------------------------------------------------------------------------------------
// Patch-staged convolution: every workgroup runs a serial chain (first fetch, then per channel
// stage: fetch issue, taps x MFMA, transpose + LDS commit, barriers; then the stores);
// workgroups beyond the resident ones queue behind it.
double predict_patch(const GemmView& v, const gensor_hw& hw, int bm, int bn, int bk, int wm, int wn, int kg, int stages) {
  const int e = v.esize, eo = v.osize;
  const int g = e == 2 ? 16 : 8;
  const int mb = kg == g ? 32 : 16;
  const int epc = 16 / e;
  const int64_t RS = v.cr * v.cs;
  const double nst = std::ceil((double)v.cc / bk);
  const int64_t px = conv_tile_px(bn, v.N, v.Q, (v.M + bm - 1) / bm, hw.compute_units);   // the kernel's own rule
  double out_rows = px % v.Q == 0 ? (double)(px / v.Q) : std::ceil((double)(px - 1) / (double)v.Q) + 1.0;
  if (out_rows > (double)(v.cn * v.P)) out_rows = (double)(v.cn * v.P);
  const int64_t rows = ((int64_t)out_rows - 1) * v.cstride + v.cr + 2 * v.cpad;
  const int64_t pw = v.cw + 2 * v.cpad;
  const int64_t stage = (int64_t)bm * (RS * bk * e + 16) + rows * pw * (bk * e + 16);
  const int64_t lds = stages * stage + ((RS == 1 || RS == 9) ? 0 : (int64_t)bm * RS * bk * e);     // + the raw filter runs
  if (lds > hw.lds_bytes_per_cu) return -1.0;
  const int nwaves = (bm / wm) * (bn / wn);
  if (nwaves > hw.max_waves_per_wg) return -1.0;
  const int64_t units = (int64_t)std::ceil((double)(rows * (int64_t)std::ceil((double)v.cw / epc) * (bk / epc)) / (double)(nwaves * 64));
  const int64_t avec = (int64_t)std::ceil((double)(bm * RS * bk) / epc / (double)(nwaves * 64));
  const int64_t regs = wm * wn / 64 + (wm + wn) / 2 + 32 * units + 4 * avec + 48;
  if (regs > hw.regs_per_lane) return -1.0;
  int64_t occ = hw.lds_bytes_per_cu / lds;
  const int64_t by_regs = (hw.simds_per_cu * (hw.regs_per_lane / regs)) / nwaves;
  if (by_regs < occ) occ = by_regs;
  if (occ > 8) occ = 8;
  if (occ < 1) return -1.0;
  const double tiles = std::ceil((double)v.M / bm) * std::ceil((double)v.N / (double)px);
  const double cu_tiles = std::ceil(tiles / hw.compute_units);
  const double resident = (double)occ < cu_tiles ? (double)occ : cu_tiles;
  // the busiest CU runs whole groups of resident workgroups one after the other; the others even it out in part
  double rounds = tiles / (double)(hw.compute_units * occ);
  if (rounds < 1.0) rounds = 1.0;
  rounds = 0.7 * std::ceil(cu_tiles / (double)occ) + 0.3 * rounds;
  double share = resident * nwaves / hw.simds_per_cu;
  if (share < 1.0) share = 1.0;
  const double peak_simd = (e == 2 ? hw.mfma_tflops_16bit : hw.mfma_tflops_f32) * 1e6 / (double)(hw.compute_units * hw.simds_per_cu);
  const int ksteps = bk / kg;
  const double t_mfma = (double)(RS * ksteps * (wm / mb) * (wn / mb)) * (2.0 * mb * mb * kg) / peak_simd * share;
  const double lds_bw = hw.bandwidth_gbs[1] * 1e3 / hw.compute_units;
  const double t_lds = (double)(RS * ksteps * ((wm / mb) + (wn / mb))) * 1024.0 * nwaves / lds_bw * resident;
  const double l2_bw = hw.l2_bandwidth_gbs * 1e3 / hw.compute_units;
  const double t_feed = (double)(rows * v.cw * bk * e + bm * RS * bk * e) / (0.5 * l2_bw);     // 16-byte gathers: half the L2 rate; hidden by the other resident workgroups
  const double t_fixed = 0.25 * hw.latency_ns[0] * 1e-3;
  const double t_stage = t_mfma + t_lds + t_feed + t_fixed;
  const double t_pro = 0.625 * hw.latency_ns[0] * 1e-3;
  const double t_epi = (double)(bm * px * eo) / (1.5 * hw.bandwidth_gbs[0] * 1e3 / hw.compute_units);
  const double t_cu = rounds * (t_pro + nst * t_stage + t_epi);
  const double bytes_total = (double)(e * (v.cn * v.cc * v.ch * v.cw + v.M * v.K) + eo * v.M * v.N);
  const double t_hbm = bytes_total / (0.6 * hw.bandwidth_gbs[0] * 1e3);
  return (t_cu > t_hbm ? t_cu : t_hbm) + 0.3 * (t_cu > t_hbm ? t_hbm : t_cu) + hw.launch_us;
}

// split > 1: the tiles that do not fill a whole round of compute units (all of them when there are fewer tiles
// than units) are computed by `split` workgroups each, every one over 1/split of the k tiles; the parts of a
// tile exchange fp32 partial tiles through device memory (measured: about a quarter of the HBM rate) and a
// dependent launch clears their arrival counters first.  Infeasible if there is nothing to split.
double predict(const GemmView& v, const gensor_hw& hw, int bm, int bn, int bk, int wm, int wn, int kg,
               int vm, int vn, int vec, int stages, int direct, int split) {
  if (v.bsrc == B_CONV && direct) return split == 1 ? predict_patch(v, hw, bm, bn, bk, wm, wn, kg, stages) : -1.0;
  if (split < 1 || (split > 1 && v.bsrc != B_KC && v.bsrc != B_NC)) return -1.0;
  if (vm < 1 || vn < 1 || bm < 1 || bn < 1 || bk < 1 || wm < 1 || wn < 1 || kg < 1 || stages < 1) return -1.0;
  const int e = v.esize, eo = v.osize;
  const int g = e == 2 ? 16 : 8;
  const int mb = kg == g ? 32 : 16;
  const double tiles_m = std::ceil((double)v.M / bm), tiles_n = std::ceil((double)v.N / bn);
  const double tiles = tiles_m * tiles_n * (double)v.batch;
  const int nwaves = (bm / wm) * (bn / wn);
  if (nwaves > hw.max_waves_per_wg) return -1.0;
  const int lds = stages * e * bk * (bm + bn);
  if (lds > hw.lds_bytes_per_cu) return -1.0;
  const int regs = wm * wn / 64 + 2 * (wm + wn) * kg * e / 256 + (direct ? 0 : (e * bk * (bm + bn)) / (nwaves * 64 * 4)) + 32;
  if (regs > hw.regs_per_lane) return -1.0;
  int waves_per_simd = hw.regs_per_lane / regs;
  if (waves_per_simd > 8) waves_per_simd = 8;
  int occ = hw.lds_bytes_per_cu / lds;
  if ((hw.simds_per_cu * waves_per_simd) / nwaves < occ) occ = (hw.simds_per_cu * waves_per_simd) / nwaves;
  if (occ > 8) occ = 8;
  if (occ < 1) return -1.0;
  const double nk = std::ceil((double)v.K / bk);
  double whole = tiles, nk_part = nk;
  if (split > 1) {
    whole = std::floor(tiles / hw.compute_units) * hw.compute_units;
    if (whole == tiles || nk < split) return -1.0;
    nk_part = std::ceil(nk / split);
  }
  const double cu_whole = std::ceil(whole / hw.compute_units);
  const double cu_part = std::ceil((tiles - whole) * split / hw.compute_units);
  const double cu_tiles = cu_whole + cu_part;
  const double resident = occ < cu_tiles ? occ : cu_tiles;
  const double kp = nk * bk;
  // (matrix pipes sustain about 0.9 of the published rate in a tiled loop on real operands; fitted)
  const double peak = 0.9 * (e == 2 ? hw.mfma_tflops_16bit : hw.mfma_tflops_f32) * 1e6 / hw.compute_units;
  double simd_use = nwaves * resident / hw.simds_per_cu;
  if (simd_use > 1.0) simd_use = 1.0;
  const double t_mfma = 2.0 * bm * bn * kp / (peak * simd_use * (mb == 32 ? 1.0 : 0.9));
  const double lds_bw = hw.bandwidth_gbs[1] * 1e3 / hw.compute_units;
  // fragment reads of the two operand tiles, each slowed by its bank-conflict ways (Eq. 3), and the tile's deposit
  const double t_lds = e * kp * ((double)bm * (bn / wn) * conflict_ways(v, hw, bk, 0, vm) +
                                 (double)bn * (bm / wm) * conflict_ways(v, hw, bk, 1, vn) + (bm + bn)) / lds_bw;
  const double l2_bw = hw.l2_bandwidth_gbs * 1e3 / hw.compute_units;
  const double gather = (v.bsrc == B_CONV && !direct) ? 16.0 : 1.0;     // element-wise loads and their index arithmetic
  const double scalar = vec ? 1.0 : 6.0;
  const double t_feed = scalar * e * kp * (bm + gather * bn) / l2_bw;
  double par = resident * nwaves / hw.simds_per_cu;
  if (par > 4.0) par = 4.0;
  double overlap = 0.8 + 0.15 * par;
  if (direct && v.bsrc == B_KC) overlap += 0.05;      // measured: what direct staging pays for k-contiguous operands
  if (direct && v.bsrc == B_NC) overlap += 0.03;      // ... and for an n-contiguous B
  if (direct && v.bsrc == B_KC && stages == 2 && wm * wn >= 128 * 128 && bk == 4 * kg) overlap += 0.24;   // the two-steps-ahead schedule of the one-wave-per-SIMD tiles (k-contiguous operands: measured)
  double t_main = t_mfma;
  if (t_lds > t_main) t_main = t_lds;
  if (t_feed > t_main) t_main = t_feed;
  // every k tile boundary (barrier, refill of the fragment pipeline) exposes a share of the memory latency
  // (a ring of three and more stages keeps more tiles in flight)
  const double t_ktile = 0.3 * hw.latency_ns[0] * 1e-3;
  auto sync_time = [&](double tiles_k) {
    double t = tiles_k * t_ktile;
    // (a ring fills stages - 1 tiles before its first product: those boundaries are paid in full, measured as no gain
    // from the ring on a 12-tile loop and 7-13 % on 48 to 128 tiles)
    if (stages > 2 && (v.bsrc == B_KC || v.bsrc == B_NC)) {
      const double fill = tiles_k < stages - 1.0 ? tiles_k : stages - 1.0;
      t = t_ktile * (fill + (tiles_k - fill) / (stages - 1));
    }
    if (stages == 1) t = t + (tiles_k - 1.0) * 4.0 * t_ktile;          // a single buffer: each further tile waits out its own fetch
    return t;
  };
  // (a second resident workgroup works while the first waits at its k tile boundary)
  const double share = resident < 2.0 ? resident : 2.0;
  // (a twentieth of the LDS traffic time is never hidden: fragment reads that conflict cost even where the LDS is not the limit)
  // a stride-2 row of a pointwise convolution's input is fetched whole and half of it dropped: the B tile's feed is
  // paid a second time, unhidden (measured: at equal area the wider pixel tile is 12-14 % slower on such a layer)
  const double t_s2 = v.bsrc == B_NCS2 ? 2.0 * e * kp * bn / l2_bw : 0.0;
  // at equal area the taller tile is 1-3 % faster than the wider one on 10 of 13 measured pairs: priced as 1 %
  const double wide = bn > bm ? 1.01 : 1.0;
  const double t_part = wide * (t_main * (nk_part / nk) / overlap + sync_time(nk_part) / share + (0.05 * t_lds + t_s2) * (nk_part / nk));     // one part of a split tile
  t_main = wide * (t_main / overlap + sync_time(nk) / share + 0.05 * t_lds + t_s2);
  const double hbm_bw_cu = hw.bandwidth_gbs[0] * 1e3 / hw.compute_units;
  const double t_epi = bm * bn * eo / (1.2 * hbm_bw_cu);      // write-through stores
  const double t_fill = (hw.latency_ns[0] * 2.0 + hw.latency_ns[1] * 4.0) * 1e-3;
  // stores are hidden by the other waves on the SIMD, of this workgroup or of another resident one (measured on the
  // store-bound shapes: eight-wave 128x128 tiles beat four-wave ones by 8 %, four-wave 256x256 tiles trail by 20 %);
  // beyond four waves per SIMD nothing more is hidden
  double hide = resident * nwaves / hw.simds_per_cu;
  if (hide > 4.0) hide = 4.0;
  // a part writes its partial tile, and one part in `split` reads the others' and stores C
  const double t_swap = bm * bn * 4.0 / (0.8 * hbm_bw_cu);
  // the exchange is a chain of memory round trips whatever the tile size: the slot stores written through and awaited,
  // the arrival count, the other parts' slots fetched past the L2 (measured: a two-way split of the 128x128 tiles of
  // 8192x768x3072 takes 9 us longer than its halved k loop explains)
  const double t_chain = 10.0 * hw.latency_ns[0] * 1e-3;
  const double t_cu = cu_whole * (t_main + t_epi / hide) +
                      cu_part * (t_part + t_chain + t_swap + (t_swap * (split - 1) + t_epi) / split / hide) + t_fill;
  const double bytes_total = (double)v.batch * ((double)e * ((double)v.M * v.K + (double)v.K * v.N) + (double)eo * v.M * v.N);
  const double bytes_swap = split > 1 ? (tiles - whole) * (2.0 * split - 1.0) * bm * bn * 4.0 : 0.0;
  // (the store-bound shapes stream at 6.5-6.9 TB/s, measured)
  const double t_hbm = bytes_total / (0.9 * hw.bandwidth_gbs[0] * 1e3) + bytes_swap / (0.25 * hw.bandwidth_gbs[0] * 1e3);
  // soft roofline: the smaller of the two limits still costs a fraction (imperfect overlap)
  const bool prepass = v.pointwise && v.cstride > 1 && v.bsrc != B_NCS2;   // the input is compacted by a dependent launch of its own
  return (t_cu > t_hbm ? t_cu : t_hbm) + 0.2 * (t_cu > t_hbm ? t_hbm : t_cu) + hw.launch_us * (prepass ? 3.5 : 1.0) +
         (split > 1 ? hw.launch_us : 0.0);
}

double predict_instance(const GemmView& v, const gensor_hw& hw, const InstanceDesc& d, int split = 1) {
  if (split > 1 && !d.launch_split) return -1.0;
  return predict(v, hw, d.bm, d.bn, d.bk, d.wm, d.wn, d.kg, d.vm, d.vn, d.vec, d.stages, d.direct, split);
}

// split factors the ranking tries on every candidate instance
const int kSplits[] = {1, 2, 3, 4, 6, 8, 12, 16};

bool usable(const InstanceDesc& d, const GemmView& v, bool vec_ok) {
  if (!instance_serves(d, v)) return false;
  if (d.vec && !vec_ok) return false;
  if (d.direct && v.bsrc != B_CONV && v.K % d.bk != 0) return false;
  return true;
}

}  // namespace

gensor_status construct_internal(const gensor_problem* p, const gensor_hw* hw, const gensor_construct_opts* opts,
                                 uint64_t seed, bool vec_ok, int view_mode, gensor_schedule* out) {
  if (!p || !out) return GENSOR_ERR_INVALID_ARG;
  const auto t0 = std::chrono::steady_clock::now();
  GemmView v;
  gensor_status st = gemm_view(p, &v, view_mode);
  if (st != GENSOR_OK) return st;
  Ctx c;
  make_ctx(v, hw, opts, &c);

  std::vector<Etir> kept;
  int max_steps = 0;
  for (int chain = 0; chain < c.opts.chains; ++chain) {
    const int n = run_walk(c, seed, (uint64_t)chain, &kept, nullptr);
    if (n > max_steps) max_steps = n;
  }
  // rank the distinct kept states; best exact instance wins, else the instance nearest to the best state
  std::set<Etir> seen;
  const InstanceDesc* best = nullptr;
  double best_us = 0.0;
  int best_split = 1;
  int scored = 0;
  const Etir* best_state = nullptr;
  double best_state_us = 0.0;
  for (const Etir& e : kept) {
    if (!seen.insert(e).second) continue;
    ++scored;
    // a compiled instance realises the state if it sits on the same lattice point: T_2 and T_1 of m, n
    // and k, and both V.  What the walk does not decide (LDS stages, direct staging, vector width) is
    // whatever was compiled.  A patch-staged convolution instance has a k order and an LDS layout of its own
    // (channels per stage, the halo patch), so only its spatial tiles are compared.
    for (int i = 0; i < g_num_instances; ++i) {
      const InstanceDesc& d = g_instances[i];
      if (d.bm != e.tile[0][0] || d.bn != e.tile[1][0] || d.wm != e.tile[0][1] || d.wn != e.tile[1][1]) continue;
      if (!d.units && (d.bk != e.tile[2][0] || d.kg != e.tile[2][1] || d.vm != e.v[0] || d.vn != e.v[1])) continue;
      if (!usable(d, v, vec_ok)) continue;
      for (int split : kSplits) {
        if (split > 1 && c.opts.no_split_k) break;
        const double us = predict_instance(v, c.hw, d, split);
        // (equal prices: the lower instance id, whatever order the states were kept in)
        if (us > 0 && (!best || us < best_us || (us == best_us && d.id < best->id))) { best = &d; best_us = us; best_split = split; }
      }
    }
    const double us0 = predict(v, c.hw, e.tile[0][0], e.tile[1][0], e.tile[2][0], e.tile[0][1], e.tile[1][1], e.tile[2][1],
                               e.v[0], e.v[1], vec_ok ? 1 : 0, 2, 0, 1);
    if (us0 > 0 && (!best_state || us0 < best_state_us)) { best_state = &e; best_state_us = us0; }
  }
  if (!best && best_state) {
    const int target[8] = {best_state->tile[0][0], best_state->tile[1][0], best_state->tile[2][0], best_state->tile[0][1],
                           best_state->tile[1][1], best_state->tile[2][1], best_state->v[0], best_state->v[1]};
    bool have = false;
    double bd = 0.0;
    for (int i = 0; i < g_num_instances; ++i) {
      const InstanceDesc& d = g_instances[i];
      if (!usable(d, v, vec_ok)) continue;
      const double us = predict_instance(v, c.hw, d);
      if (us <= 0) continue;
      const int cand[8] = {d.bm, d.bn, d.bk, d.wm, d.wn, d.kg, d.vm, d.vn};
      double dist = 0.0;
      for (int k = 0; k < 8; ++k) dist += std::fabs(std::log2((double)cand[k]) - std::log2((double)target[k]));
      if (!have || dist < bd || (dist == bd && us < best_us)) { have = true; bd = dist; best = &d; best_us = us; }
    }
  }
  if (!best) return GENSOR_ERR_NO_SCHEDULE;
  schedule_from_instance(*best, out);
  out->split_k = best_split;
  out->round_units = c.hw.compute_units;
  out->predicted_us = best_us;
  out->iterations = max_steps;
  out->chains = c.opts.chains;
  out->states_scored = scored;
  out->seed = seed;
  out->construct_s = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  return GENSOR_OK;
}

}  // namespace gensor

using namespace gensor;

extern "C" const gensor_hw* gensor_hw_mi355x(void) { return &kMi355x; }

extern "C" gensor_status gensor_construct(const gensor_problem* p, const gensor_hw* hw, const gensor_construct_opts* opts,
                                          uint64_t seed, gensor_schedule* out) {
  // Operands are taken to be 16-byte aligned with dense leading dimensions; 16-byte vector
  // accesses are then possible exactly when the contiguous extents are whole vectors.
  GemmView v;
  gensor_status st = gemm_view(p, &v, VIEW_DEFAULT);
  if (st != GENSOR_OK) return st;
  const int epc = 16 / v.esize;
  bool vec_ok = true;
  if (v.bsrc != B_CONV) vec_ok = (v.asrc == A_KC ? v.K : v.M) % epc == 0 && (v.bsrc == B_KC ? v.K : v.N) % epc == 0;
  return construct_internal(p, hw, opts, seed, vec_ok, VIEW_DEFAULT, out);
}

extern "C" gensor_status gensor_construct_trace(const gensor_problem* p, const gensor_hw* hw,
                                                const gensor_construct_opts* opts, uint64_t seed, int32_t capacity,
                                                int32_t* steps_out, int32_t* actions, int32_t* dims, int32_t* states) {
  if (!p || !steps_out || !actions || !dims || !states || capacity <= 0) return GENSOR_ERR_INVALID_ARG;
  GemmView v;
  gensor_status st = gemm_view(p, &v);
  if (st != GENSOR_OK) return st;
  Ctx c;
  make_ctx(v, hw, opts, &c);
  Trace tr = {capacity, 0, actions, dims, states};
  run_walk(c, seed, 0, nullptr, &tr);
  *steps_out = tr.steps;
  return GENSOR_OK;
}

extern "C" double gensor_predict_us(const gensor_schedule* s, const gensor_problem* p, const gensor_hw* hw) {
  if (!s || !p) return -1.0;
  GemmView v;
  if (gemm_view(p, &v) != GENSOR_OK) return -1.0;
  const gensor_hw& h = hw ? *hw : kMi355x;
  return predict(v, h, s->tile[0][0], s->tile[1][0], s->tile[2][0], s->tile[0][1], s->tile[1][1], s->tile[2][1],
                 s->vthread[0], s->vthread[1], s->vec_bytes == 16 ? 1 : 0, s->stages, s->direct_lds, s->split_k);
}
