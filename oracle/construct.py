"""CPU oracle of the schedule constructor.  TEST INFRASTRUCTURE ONLY.

The constructor is a stochastic heuristic, so this file follows the paper's algorithm step
by step, in its notation, with the readings listed below for everything the paper leaves
open.  It shares no code with the C++ constructor; both sides implement the same published
counter-based generator (splitmix64 finaliser) so that a walk can be compared step by step.

Paper passages followed
  Section IV-A   state = ETIR: tiles per memory level, virtual threads, current level;
                 actions tile / invTile / setVThread / cache
  Section IV-B   Eq. 1 (tiling benefit), Eq. 2 (caching benefit), Eq. 3 (vThread benefit)
  Section IV-C   Algorithm 1 (annealing loop, keep rule, T <- T/2), Algorithm 2 (benefits ->
                 normalise -> roulette), the annealing multiplier on the cache entry, the
                 memory check, D = [T_L, ..., T_1, T_0]
  Section IV-D   Eq. 4: P(i,j) = Norm(Benefit) >= 0, rows sum to 1

Readings (the paper is silent or garbled here)
  dims       the GEMM view: m, n spatial, k reduction (conv: m = filters, n = image x out
             row x out col, k = channel x filter row x filter col); batch is a grid axis
  levels     L = 2: T_2 = workgroup tile in LDS, T_1 = wave tile in registers, T_0 = T_1 / V
  steps      tile doubles, invTile halves; m, n in {16..256}; k at T_2 in {2g..8g}, k at T_1
             in {g, 2g} where g = 16 elements for 16-bit types and 8 for fp32 (g selects the
             MFMA block: T_1[k] = g -> 32x32 blocks, 2g -> 16x16 blocks)
  start      every tile at its minimum (T_1[k] = 2g), V = 1, level 2 ("unscheduled")
  Q, F       level 2: Q = e M N K (1/T_m + 1/T_n) + e_out M N, F = e T_k (T_m + T_n)
             level 1: Q = e B_m B_n B_k (1/T_m + 1/T_n),       F = 4 T_m T_n + e T_k (T_m + T_n)
  Eq. 1      as printed: Q(T) F(T') / (Q(T') F(T)); option `tiling_benefit=1` inverts F
  Eq. 2      S = F of the current tile; L, B of the two levels from the hardware table, B per CU
  Eq. 3      x = 16 T_1[d] bytes (a lane reads 16 bytes per fragment), W = banks x bank bytes;
             setVThread cycles V 1 -> 2 -> 4 -> 1; benefit = ceil(x/(V W)) / ceil(x/(V' W))
  T, t       Algorithm 1 halves one temperature T per step and stops at the threshold.  The
             multiplier and the keep rule are both sigmoids centred at 10 in "-log T", so t is
             read as -log2 of a temperature.  Each memory level is annealed: the level
             temperature T_l starts at T0, halves per step and restarts at T0 when cache
             fires; t = -log2(T_l).  With the default T0 = 2^30 the multiplier is ~0.005 when
             a level is entered, 0.5 after 30 steps and 1.5 after 40, which leaves the walk
             time to mix within a level before it is pushed on (Section IV-D argues
             convergence within a level).  The loop's own T (never reset) ends the walk
             after log2(T0/threshold) = 100 steps.
  roulette   first index whose cumulative probability exceeds u, u uniform in [0,1)
  cache      one entry (no dimension); after the last level the walk stops
  check      a transition whose target breaks a capacity (LDS bytes for two stages, registers
             per lane, waves per workgroup on the last cache) or leaves the lattice gets 0
  ladder     walk number c starts from T0 / 2^(c mod 31): colder walks leave a level sooner
             and so end in smaller tiles, which small problems need (Eq. 1 is a ratio and
             does not see the problem size; only the capacity check and the caps do)
  keep       Algorithm 1 appends the state after every step.  A register-level state whose
             workgroup fits the wave limit is a complete program (stop there), so policy 0
             keeps each such visited state in its completed form; policy 1 keeps it with
             the printed probability 1 - 1/(1 + exp(-0.5 (-ln T - 10)))
  pick       kept complete states are ranked by the analytical cost model below.  A state is
             realised by every compiled instance on the same spatial tiles (T_2 and T_1 of m and
             n: the sizes Eq. 1's traffic depends on); k tile, MFMA depth, V and staging mode are
             then those of the instance.  The best such instance over all kept states wins (if
             none exists, the instance nearest to the best-ranked state)
  views      a pointwise convolution (1x1 filter, no padding) is walked and ranked as the
             batched GEMM it is (one GEMM per image, n-contiguous B); other convolutions in
             the implicit-GEMM view.  Instances that cache the input patch in LDS have a
             cost model of their own (predict_patch_us: a serial chain per workgroup)
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence, Tuple

M64 = (1 << 64) - 1
TILE, INVTILE, SETVTHREAD, CACHE = 0, 1, 2, 3
DIM_M, DIM_N, DIM_K = 0, 1, 2


# ------------------------------------------------------------------ random numbers
def uniform(seed: int, chain: int, step: int, j: int) -> float:
    """Counter-based uniform in [0,1): splitmix64 finaliser of seed + golden * counter."""
    s = (seed + 0x9E3779B97F4A7C15 * (chain * 4096 + 2 * step + j + 1)) & M64
    z = ((s ^ (s >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    z = z ^ (z >> 31)
    return (z >> 11) * (1.0 / 9007199254740992.0)


# ------------------------------------------------------------------ inputs
@dataclass
class View:
    """GEMM view of the operator (tensor_shape of Algorithm 1)."""
    M: int
    N: int
    K: int
    batch: int = 1
    e: int = 2          # bytes per input element
    e_out: int = 4
    bsrc: int = 0       # 0 k-contiguous B, 1 n-contiguous B, 2 convolution gather, 3 n-contiguous B sampled at stride 2
    conv: Optional[Tuple[int, ...]] = None   # convolution geometry (n, c, h, w, r, s, stride, pad), else None
    prepass: int = 0    # 1: a strided pointwise convolution (its input is compacted by a pre-pass kernel)


@dataclass
class Hw:
    compute_units: int = 256
    simds_per_cu: int = 4
    wave_size: int = 64
    max_waves_per_wg: int = 16
    lds_bytes_per_cu: int = 163840
    regs_per_lane: int = 512
    lds_banks: int = 64
    lds_bank_bytes: int = 4
    clock_ghz: float = 2.4
    latency_ns: Tuple[float, float, float] = (800.0, 64.0, 4.0)
    bandwidth_gbs: Tuple[float, float, float] = (8000.0, 157286.4, 1258291.2)
    l2_bandwidth_gbs: float = 20000.0
    mfma_tflops_16bit: float = 2516.6
    mfma_tflops_f32: float = 157.3
    launch_us: float = 2.0


@dataclass
class Opts:
    T0: float = 2.0 ** 30
    threshold: float = 2.0 ** -70
    chains: int = 1024
    keep_policy: int = 0
    tiling_benefit: int = 0
    no_vthread: int = 0
    no_split_k: int = 0
    greedy: int = 0


@dataclass
class State:
    """ETIR: tile[d] = [T_2, T_1, T_0] for d in (m, n, k); V for m, n; level 0 = scheduling
    T_2 (LDS), 1 = scheduling T_1 (registers), 2 = complete."""
    tile: List[List[int]]
    v: List[int]
    level: int = 0

    def copy(self) -> "State":
        return State([row[:] for row in self.tile], self.v[:], self.level)

    def flat(self) -> List[int]:
        return [x for row in self.tile for x in row] + self.v + [self.level]


def g_of(view: View) -> int:
    return 16 if view.e == 2 else 8


def next_pow2(x: int) -> int:
    p = 1
    while p < x:
        p *= 2
    return p


def caps(view: View) -> List[int]:
    g = g_of(view)
    return [max(16, min(256, next_pow2(view.M))), max(16, min(256, next_pow2(view.N))),
            max(2 * g, min(8 * g, next_pow2(view.K)))]


def initial_state(view: View) -> State:
    g = g_of(view)
    return State([[16, 16, 16], [16, 16, 16], [2 * g, 2 * g, 2 * g]], [1, 1], 0)


def mfma_block(view: View, s: State) -> int:
    return 32 if s.tile[DIM_K][1] == g_of(view) else 16


# ------------------------------------------------------------------ footprint / traffic
def F(view: View, s: State, level: int) -> float:
    tm, tn, tk = s.tile[0][level], s.tile[1][level], s.tile[2][level]
    if level == 0:
        return float(view.e * tk * (tm + tn))
    return float(4 * tm * tn + view.e * tk * (tm + tn))


def Q(view: View, s: State, level: int) -> float:
    tm, tn = s.tile[0][level], s.tile[1][level]
    if level == 0:
        return view.e * float(view.M) * float(view.N) * float(view.K) * (1.0 / tm + 1.0 / tn) \
            + view.e_out * float(view.M) * float(view.N)
    bm, bn, bk = s.tile[0][0], s.tile[1][0], s.tile[2][0]
    return view.e * float(bm) * float(bn) * float(bk) * (1.0 / tm + 1.0 / tn)


# ------------------------------------------------------------------ legality + capacity
def valid(view: View, hw: Hw, s: State) -> bool:
    g = g_of(view)
    cap = caps(view)
    for d in (0, 1):
        if not (16 <= s.tile[d][0] <= cap[d]):
            return False
    if not (2 * g <= s.tile[2][0] <= cap[2]):
        return False
    if 2 * view.e * s.tile[2][0] * (s.tile[0][0] + s.tile[1][0]) > hw.lds_bytes_per_cu:   # two LDS stages
        return False
    if s.level >= 1:
        if s.tile[2][1] not in (g, 2 * g) or s.tile[2][1] > s.tile[2][0]:
            return False
        mb = mfma_block(view, s)
        for d in (0, 1):
            if s.v[d] not in (1, 2, 4):
                return False
            if s.tile[d][1] > s.tile[d][0] or s.tile[d][1] < 16:
                return False
            if s.tile[d][1] % (mb * s.v[d]) != 0:
                return False
        regs = s.tile[0][1] * s.tile[1][1] // 64 + 2 * (s.tile[0][1] + s.tile[1][1]) * s.tile[2][1] * view.e // 256
        if regs > hw.regs_per_lane:
            return False
    return True


def waves(s: State) -> int:
    return (s.tile[0][0] // s.tile[0][1]) * (s.tile[1][0] // s.tile[1][1])


def apply_action(view: View, s: State, ac: int, d: int) -> State:
    """applyProgPolicy: the state after action `ac` on dimension `d` (no legality check)."""
    n = s.copy()
    if ac == TILE:
        n.tile[d][s.level] *= 2
    elif ac == INVTILE:
        n.tile[d][s.level] //= 2
    elif ac == SETVTHREAD:
        mb = mfma_block(view, s)
        nv = s.v[d] * 2
        if nv > 4 or s.tile[d][1] % (mb * nv) != 0:
            nv = 1
        n.v[d] = nv
    elif ac == CACHE:
        n.level = s.level + 1
        if s.level == 0:
            g = g_of(view)
            n.tile[0][1], n.tile[1][1], n.tile[2][1] = 16, 16, 2 * g
    if n.level >= 1:
        for dd in (0, 1):
            n.tile[dd][2] = n.tile[dd][1] // n.v[dd]
        n.tile[2][2] = n.tile[2][1]
    return n


# ------------------------------------------------------------------ Eq. 1-3
def benefit_tiling(view: View, s: State, n: State, opts: Opts) -> float:
    lv = s.level
    q0, q1, f0, f1 = Q(view, s, lv), Q(view, n, lv), F(view, s, lv), F(view, n, lv)
    if opts.tiling_benefit == 1:
        return (q0 * f0) / (q1 * f1)
    return (q0 * f1) / (q1 * f0)


def benefit_caching(view: View, hw: Hw, s: State) -> float:
    lo, hi = s.level, s.level + 1
    S = F(view, s, s.level)
    b_lo = hw.bandwidth_gbs[lo] / hw.compute_units
    b_hi = hw.bandwidth_gbs[hi] / hw.compute_units
    return (hw.latency_ns[lo] + S / b_lo) / (hw.latency_ns[hi] + S / b_hi)


def benefit_vthread(hw: Hw, s: State, n: State, d: int) -> float:
    x = 16.0 * s.tile[d][1]
    W = float(hw.lds_banks * hw.lds_bank_bytes)
    return math.ceil(x / (s.v[d] * W)) / math.ceil(x / (n.v[d] * W))


def annealing_factor(t: float) -> float:
    return 3.0 / (1.0 + math.exp(-(math.log(5.0) / 10.0) * (t - 10.0)))


def t_of(T_level: float) -> float:
    return -math.log2(T_level)


def keep_probability(T: float) -> float:
    return 1.0 - 1.0 / (1.0 + math.exp(-0.5 * (-math.log(T) - 10.0)))


# ------------------------------------------------------------------ Algorithm 2
ACTION_LIST = [(TILE, 0), (TILE, 1), (TILE, 2), (INVTILE, 0), (INVTILE, 1), (INVTILE, 2),
               (SETVTHREAD, 0), (SETVTHREAD, 1), (CACHE, -1)]


def get_benefits(view: View, hw: Hw, opts: Opts, s: State, T_level: float) -> List[float]:
    out = []
    for (ac, d) in ACTION_LIST:
        b = 0.0
        if ac in (TILE, INVTILE):
            n = apply_action(view, s, ac, d)
            if valid(view, hw, n):
                b = benefit_tiling(view, s, n, opts)
        elif ac == SETVTHREAD:
            if s.level == 1 and not opts.no_vthread:
                n = apply_action(view, s, ac, d)
                if n.v[d] != s.v[d] and valid(view, hw, n):
                    b = benefit_vthread(hw, s, n, d)
        else:
            ok = True
            if s.level == 1 and waves(s) > hw.max_waves_per_wg:
                ok = False
            if ok:
                b = benefit_caching(view, hw, s) * annealing_factor(t_of(T_level))
        out.append(b)
    return out


def normalize(benefits: Sequence[float]) -> List[float]:
    total = 0.0
    for b in benefits:
        total += b
    if total <= 0.0:
        return [0.0 for _ in benefits]
    return [b / total for b in benefits]


def roulette(probs: Sequence[float], u: float) -> int:
    acc = 0.0
    last = -1
    for i, p in enumerate(probs):
        if p > 0.0:
            last = i
        acc += p
        if p > 0.0 and u < acc:
            return i
    return last


def get_prog_policy(view: View, hw: Hw, opts: Opts, s: State, T_level: float, u: float) -> Tuple[int, int, List[float]]:
    probs = normalize(get_benefits(view, hw, opts, s, T_level))
    if opts.greedy and any(p > 0.0 for p in probs):
        i = max(range(len(probs)), key=lambda j: (probs[j], -j))      # first action of largest probability, no draw
    else:
        i = roulette(probs, u)
    if i < 0:
        return -1, -1, probs
    return ACTION_LIST[i][0], ACTION_LIST[i][1], probs


# ------------------------------------------------------------------ Algorithm 1
@dataclass
class Walk:
    actions: List[int] = field(default_factory=list)
    dims: List[int] = field(default_factory=list)
    states: List[List[int]] = field(default_factory=list)
    kept: List[State] = field(default_factory=list)


def walk(view: View, hw: Hw, opts: Opts, seed: int, chain: int = 0) -> Walk:
    out = Walk()
    e = initial_state(view)
    T0 = opts.T0 / 2.0 ** (chain % 31)
    T = T0
    T_level = T0
    step = 0
    while T > opts.threshold and e.level < 2:
        ac, d, _ = get_prog_policy(view, hw, opts, e, T_level, uniform(seed, chain, step, 0))
        if ac < 0:
            break
        e2 = apply_action(view, e, ac, d)
        out.actions.append(ac)
        out.dims.append(d)
        out.states.append(e2.flat())
        if e2.level == 2 or (e2.level == 1 and waves(e2) <= hw.max_waves_per_wg):
            if opts.keep_policy == 0 or uniform(seed, chain, step, 1) < keep_probability(T):
                out.kept.append(e2 if e2.level == 2 else apply_action(view, e2, CACHE, -1))
        e = e2
        T = T / 2.0
        T_level = T0 if ac == CACHE else T_level / 2.0
        step += 1
    return out


# ------------------------------------------------------------------ cost model and pick
@dataclass
class Instance:
    id: int
    bm: int
    bn: int
    bk: int
    wm: int
    wn: int
    kg: int
    vm: int
    vn: int
    vec: int
    stages: int
    direct: int
    split_ok: int = 0      # also compiled with split tiles
    split: int = 1         # split factor of a pick


def predict_patch_us(view: View, hw: Hw, bm, bn, bk, wm, wn, kg, stages) -> float:
    """Patch-staged convolution: every workgroup runs a serial chain (first fetch, then per
    channel stage: fetch issue, taps x MFMA, transpose + LDS commit, barriers; then the
    stores); workgroups beyond the resident ones queue behind it."""
    e, eo = view.e, view.e_out
    n, c, h, w, r, s, stride, pad = view.conv
    g = 16 if e == 2 else 8
    mb = 32 if kg == g else 16
    epc = 16 // e
    P = (h + 2 * pad - r) // stride + 1
    Qo = (w + 2 * pad - s) // stride + 1
    RS = r * s
    nst = math.ceil(c / bk)
    out_rows = min(math.ceil((bn - 1) / Qo) + 1, n * P)
    rows = (out_rows - 1) * stride + r + 2 * pad
    pw = w + 2 * pad
    stage = bm * (RS * bk * e + 16) + rows * pw * (bk * e + 16)
    lds = stages * stage + (0 if RS in (1, 9) else bm * RS * bk * e)        # + the raw filter runs
    if lds > hw.lds_bytes_per_cu:
        return -1.0
    nwaves = (bm // wm) * (bn // wn)
    if nwaves > hw.max_waves_per_wg:
        return -1.0
    units = math.ceil(rows * math.ceil(w / epc) * (bk // epc) / (nwaves * 64))
    avec = math.ceil(bm * RS * bk / epc / (nwaves * 64))
    regs = wm * wn // 64 + (wm + wn) // 2 + 32 * units + 4 * avec + 48
    if regs > hw.regs_per_lane:
        return -1.0
    occ = min(hw.lds_bytes_per_cu // lds, (hw.simds_per_cu * (hw.regs_per_lane // regs)) // nwaves, 8)
    if occ < 1:
        return -1.0
    tiles = math.ceil(view.M / bm) * math.ceil(view.N / bn)
    resident = min(occ, math.ceil(tiles / hw.compute_units))
    rounds = max(1.0, tiles / (hw.compute_units * occ))
    share = max(1.0, resident * nwaves / hw.simds_per_cu)
    peak_simd = (hw.mfma_tflops_16bit if e == 2 else hw.mfma_tflops_f32) * 1e6 / (hw.compute_units * hw.simds_per_cu)
    ksteps = bk // kg
    t_mfma = RS * ksteps * (wm // mb) * (wn // mb) * (2.0 * mb * mb * kg) / peak_simd * share
    lds_bw = hw.bandwidth_gbs[1] * 1e3 / hw.compute_units
    t_lds = RS * ksteps * ((wm // mb) + (wn // mb)) * 1024.0 * nwaves / lds_bw * resident
    l2_bw = hw.l2_bandwidth_gbs * 1e3 / hw.compute_units
    t_feed = (rows * w * bk * e + bm * RS * bk * e) / (0.5 * l2_bw)      # 16-byte gathers: half the L2 rate; hidden by the other resident workgroups
    t_fixed = (0.75 * hw.latency_ns[0] + 1.5 * hw.latency_ns[1]) * 1e-3     # fetch issue, commit, two barriers
    t_stage = t_mfma + t_lds + t_feed + t_fixed
    t_pro = (2.0 * hw.latency_ns[0] + 6.0 * hw.latency_ns[1]) * 1e-3        # index set-up, first fetch at full latency, zero fill
    t_epi = bm * bn * eo / (0.6 * hw.bandwidth_gbs[0] * 1e3 / hw.compute_units)
    t_cu = rounds * (t_pro + nst * t_stage + t_epi)
    bytes_total = e * (n * c * h * w + view.M * view.K) + eo * view.M * view.N
    t_hbm = bytes_total / (0.6 * hw.bandwidth_gbs[0] * 1e3)
    return max(t_cu, t_hbm) + 0.3 * min(t_cu, t_hbm) + hw.launch_us


SPLITS = (1, 2, 3, 4, 6, 8, 12, 16)      # split factors the ranking tries on every candidate instance


def predict_us(view: View, hw: Hw, bm, bn, bk, wm, wn, kg, vm, vn, vec, stages, direct, split=1) -> float:
    """Analytical time of one launch: per-CU pipeline limits (MFMA, LDS, L2 feed) scaled by
    how many tiles the busiest CU owns, an epilogue that streams C, bounded below by HBM.
    split > 1: the tiles that do not fill a whole round of compute units (all of them when there are
    fewer tiles than units) are computed by `split` workgroups each over 1/split of the k tiles; the
    parts exchange fp32 partial tiles through device memory (a quarter of the HBM rate) and a dependent
    launch clears their arrival counters first.  Infeasible if there is nothing to split."""
    if view.bsrc == 2 and direct and view.conv is not None:
        return predict_patch_us(view, hw, bm, bn, bk, wm, wn, kg, stages) if split == 1 else -1.0
    if split < 1 or (split > 1 and view.bsrc not in (0, 1)):
        return -1.0
    e, eo = view.e, view.e_out
    g = 16 if e == 2 else 8
    mb = 32 if kg == g else 16
    tiles_m = math.ceil(view.M / bm)
    tiles_n = math.ceil(view.N / bn)
    tiles = tiles_m * tiles_n * view.batch
    nwaves = (bm // wm) * (bn // wn)
    if nwaves > hw.max_waves_per_wg:
        return -1.0
    lds = stages * e * bk * (bm + bn)
    if lds > hw.lds_bytes_per_cu:
        return -1.0
    regs = wm * wn // 64 + 2 * (wm + wn) * kg * e // 256 + (0 if direct else (e * bk * (bm + bn)) // (nwaves * 64 * 4)) + 32
    if regs > hw.regs_per_lane:
        return -1.0
    waves_per_simd = min(8, hw.regs_per_lane // regs)
    occ = min(hw.lds_bytes_per_cu // lds, (hw.simds_per_cu * waves_per_simd) // nwaves, 8)
    if occ < 1:
        return -1.0
    nk = float(math.ceil(view.K / bk))
    whole, nk_part = float(tiles), nk
    if split > 1:
        whole = float(math.floor(tiles / hw.compute_units) * hw.compute_units)
        if whole == tiles or nk < split:
            return -1.0
        nk_part = float(math.ceil(nk / split))
    cu_whole = float(math.ceil(whole / hw.compute_units))
    cu_part = float(math.ceil((tiles - whole) * split / hw.compute_units))
    cu_tiles = cu_whole + cu_part
    resident = min(float(occ), cu_tiles)
    kp = nk * bk
    peak = (hw.mfma_tflops_16bit if e == 2 else hw.mfma_tflops_f32) * 1e6 / hw.compute_units   # flop/us per CU
    simd_use = min(1.0, nwaves * resident / hw.simds_per_cu)
    t_mfma = 2.0 * bm * bn * kp / (peak * simd_use * (1.0 if mb == 32 else 0.9))
    lds_bw = hw.bandwidth_gbs[1] * 1e3 / hw.compute_units                                     # bytes/us per CU
    t_lds = e * kp * (bm * (bn // wn) + bn * (bm // wm) + (bm + bn)) / lds_bw
    l2_bw = hw.l2_bandwidth_gbs * 1e3 / hw.compute_units
    gather = 16.0 if (view.bsrc == 2 and not direct) else 1.0     # element-wise loads and their index arithmetic
    scalar = 1.0 if vec else 6.0
    t_feed = scalar * e * kp * (bm + gather * bn) / l2_bw
    overlap = 0.7 + 0.1 * min(resident * nwaves / hw.simds_per_cu, 3.0)
    if direct and view.bsrc == 0:          # measured: direct staging pays for k-contiguous operands only
        overlap += 0.05
    if direct and view.bsrc == 0 and stages == 2 and wm * wn >= 128 * 128 and bk == 4 * kg:   # the two-steps-ahead schedule of the one-wave-per-SIMD tiles (k-contiguous operands: measured)
        overlap += 0.12
    # every k tile boundary (barrier, refill of the fragment pipeline) exposes a share of the memory latency
    # (a ring of three and more stages keeps more tiles in flight; measured to pay for k-contiguous operands)
    t_ktile = 0.25 * hw.latency_ns[0] * 1e-3

    def sync_time(tiles_k: float) -> float:
        t = tiles_k * t_ktile
        if stages > 2 and view.bsrc == 0:
            t = t / (stages - 1)
        if stages == 1:
            t = t + (tiles_k - 1.0) * 4.0 * t_ktile        # a single buffer: each further tile waits out its own fetch
        return t

    t_pipe = max(t_mfma, t_lds, t_feed)
    share = min(resident, 2.0)      # a second resident workgroup works while the first waits at its k tile boundary
    t_part = t_pipe * (nk_part / nk) / overlap + sync_time(nk_part) / share       # one part of a split tile
    t_main = t_pipe / overlap + sync_time(nk) / share
    hbm_bw_cu = hw.bandwidth_gbs[0] * 1e3 / hw.compute_units
    t_epi = bm * bn * eo / (1.0 * hbm_bw_cu)      # write-through stores
    t_fill = (hw.latency_ns[0] * 2.0 + hw.latency_ns[1] * 4.0) * 1e-3
    # a second resident workgroup hides the stores of the first; further ones add nothing
    hide = min(resident, 2.0)
    # a part writes its partial tile, and one part in `split` reads the others' and stores C
    t_swap = bm * bn * 4.0 / (0.8 * hbm_bw_cu)
    t_cu = cu_whole * (t_main + t_epi / hide) + cu_part * (t_part + t_swap + (t_swap * (split - 1) + t_epi) / split / hide) + t_fill
    bytes_total = view.batch * (e * (view.M * view.K + view.K * view.N) + eo * view.M * view.N)
    bytes_swap = (tiles - whole) * (2.0 * split - 1.0) * bm * bn * 4.0 if split > 1 else 0.0
    t_hbm = bytes_total / (0.6 * hw.bandwidth_gbs[0] * 1e3) + bytes_swap / (0.25 * hw.bandwidth_gbs[0] * 1e3)
    # soft roofline: the smaller of the two limits still costs a fraction (imperfect overlap)
    return (max(t_cu, t_hbm) + 0.3 * min(t_cu, t_hbm) + hw.launch_us * (3.5 if view.prepass else 1.0)
            + (hw.launch_us if split > 1 else 0.0))


def pick(view: View, hw: Hw, kept: Sequence[State], instances: Sequence[Instance], vec_ok: bool,
         no_split_k: int = 0) -> Tuple[Optional[Instance], float, int]:
    """Rank kept complete states by the cost model; return the best compiled instance."""
    best, best_us, scored = None, 0.0, 0
    seen = set()
    ranked = []
    for s in kept:
        key = tuple(s.flat())
        if key in seen:
            continue
        seen.add(key)
        bm, bn, bk = s.tile[0][0], s.tile[1][0], s.tile[2][0]
        wm, wn, kg = s.tile[0][1], s.tile[1][1], s.tile[2][1]
        scored += 1
        # every compiled instance on the same spatial tiles (T_2 and T_1 of m and n) realises the
        # state; its k tile, MFMA depth, V and staging mode are whatever was compiled
        for i in instances:
            if (i.bm, i.bn, i.wm, i.wn) != (bm, bn, wm, wn) or (i.vec and not vec_ok):
                continue
            if i.direct and view.bsrc != 2 and view.K % i.bk != 0:
                continue
            for split in SPLITS:
                if split > 1 and (no_split_k or not i.split_ok):
                    break
                us = predict_us(view, hw, i.bm, i.bn, i.bk, i.wm, i.wn, i.kg, i.vm, i.vn, i.vec, i.stages, i.direct, split)
                if us > 0 and (best is None or us < best_us):
                    best, best_us = replace(i, split=split), us
        us0 = predict_us(view, hw, bm, bn, bk, wm, wn, kg, s.v[0], s.v[1], 1 if vec_ok else 0, 2, 0)
        if us0 > 0:
            ranked.append((us0, s))
    if best is None and ranked:
        us0, s = min(ranked, key=lambda r: r[0])
        target = [s.tile[0][0], s.tile[1][0], s.tile[2][0], s.tile[0][1], s.tile[1][1], s.tile[2][1], s.v[0], s.v[1]]
        bd = None
        for i in instances:
            if (i.vec and not vec_ok) or (i.direct and view.bsrc != 2 and view.K % i.bk != 0):
                continue
            us = predict_us(view, hw, i.bm, i.bn, i.bk, i.wm, i.wn, i.kg, i.vm, i.vn, i.vec, i.stages, i.direct)
            if us <= 0:
                continue
            cand = [i.bm, i.bn, i.bk, i.wm, i.wn, i.kg, i.vm, i.vn]
            dist = sum(abs(math.log2(a) - math.log2(b)) for a, b in zip(cand, target))
            if bd is None or dist < bd or (dist == bd and us < best_us):
                bd, best, best_us = dist, i, us
    return best, best_us, scored


def construct(view: View, hw: Hw, opts: Opts, seed: int, instances: Sequence[Instance], vec_ok: bool = True):
    kept: List[State] = []
    for chain in range(opts.chains):
        kept.extend(walk(view, hw, opts, seed, chain).kept)
    return pick(view, hw, kept, instances, vec_ok, opts.no_split_k)


def transition_row(view: View, hw: Hw, opts: Opts, s: State, T_level: float) -> List[float]:
    """One row of the transition matrix P of Eq. 4 (over the 9 enumerated actions)."""
    return normalize(get_benefits(view, hw, opts, s, T_level))
