"""CPU oracle of the schedule constructor's graph walk.  TEST INFRASTRUCTURE ONLY.

The constructor is a stochastic heuristic, so this file follows the paper's algorithm step
by step, in its notation, with the readings listed below for everything the paper leaves
open.  It shares no code with the C++ constructor; both sides implement the same published
counter-based generator (splitmix64 finaliser) so that a walk can be compared step by step.
It covers what the paper defines: the state, the four actions, Eq. 1-3, Algorithms 1 and 2 and
the states they keep.  It holds no cost model: how kept states are reduced to one program is
the library's own design, pinned elsewhere (see "pick" below).

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
  Eq. 3      W = banks x bank bytes (what the LDS serves per cycle).  x = bytes of bank address space
             spanned by the rows one quarter wave reads together from the operand tile of dimension d:
             16 rows of min(T_2[k] e, W) bytes for a k-contiguous tile (A stored [m][k], B stored [n][k]),
             else the 4 (16-bit) or 2 (fp32) k rows of an n- or m-contiguous tile, W bytes each.  ceil(x/(V W))
             of those rows share a bank when the tile is interleaved over V phases.  setVThread doubles V
             up to ceil(x/W) (conflict-free) and then wraps to 1; benefit = ceil(x/(V W)) / ceil(x/(V' W))
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
  pick       how the kept states become one program is not part of the paper's algorithm and not of
             this oracle: the library ranks the compiled instances that sit on a kept state's lattice
             point with its own analytical cost model.  That model is product code; it is pinned by
             measured launch times (tests/golden/instance_times.json) and by closed-form limits, and
             the selection rule is re-derived in the tests from kept_states() below.
  views      a pointwise convolution (1x1 filter, no padding) is walked as the batched GEMM it is
             (one GEMM per image, n-contiguous B); other convolutions in the implicit-GEMM view
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
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
    asrc: int = 0       # 0 k-contiguous A (stored [m][k]), 1 m-contiguous A (stored [k][m])


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
    chains: int = 16384
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


def conflict_ways(view: View, hw: "Hw", bk: int, d: int, v: int) -> int:
    """Eq. 3's ceil(x / (V W)) for the operand tile of dimension d (0: m x k, 1: k x n)."""
    W = hw.lds_banks * hw.lds_bank_bytes
    if (view.asrc == 0) if d == DIM_M else (view.bsrc == 0):
        x = 16 * min(bk * view.e, W)
    else:
        x = (4 if view.e == 2 else 2) * W
    return -(-x // (v * W))


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
            if s.v[d] not in (1, 2, 4, 8, 16) or s.v[d] > conflict_ways(view, hw, s.tile[2][0], d, 1):
                return False
            if s.tile[d][1] > s.tile[d][0] or s.tile[d][1] < 16 or s.tile[d][1] % mb != 0:
                return False
        regs = s.tile[0][1] * s.tile[1][1] // 64 + 2 * (s.tile[0][1] + s.tile[1][1]) * s.tile[2][1] * view.e // 256
        if regs > hw.regs_per_lane:
            return False
    return True


def waves(s: State) -> int:
    return (s.tile[0][0] // s.tile[0][1]) * (s.tile[1][0] // s.tile[1][1])


def apply_action(view: View, hw: "Hw", s: State, ac: int, d: int) -> State:
    """applyProgPolicy: the state after action `ac` on dimension `d` (no legality check)."""
    n = s.copy()
    if ac == TILE:
        n.tile[d][s.level] *= 2
    elif ac == INVTILE:
        n.tile[d][s.level] //= 2
    elif ac == SETVTHREAD:
        nv = s.v[d] * 2
        if nv > conflict_ways(view, hw, s.tile[2][0], d, 1):
            nv = 1
        n.v[d] = nv
    elif ac == CACHE:
        n.level = s.level + 1
        if s.level == 0:
            g = g_of(view)
            n.tile[0][1], n.tile[1][1], n.tile[2][1] = 16, 16, 2 * g
    if n.level >= 1:
        for dd in (0, 1):
            n.tile[dd][2] = max(1, n.tile[dd][1] // n.v[dd])
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


def benefit_vthread(view: View, hw: Hw, s: State, n: State, d: int) -> float:
    bk = s.tile[2][0]
    return conflict_ways(view, hw, bk, d, s.v[d]) / conflict_ways(view, hw, bk, d, n.v[d])


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
            n = apply_action(view, hw, s, ac, d)
            if valid(view, hw, n):
                b = benefit_tiling(view, s, n, opts)
        elif ac == SETVTHREAD:
            if s.level == 1 and not opts.no_vthread:
                n = apply_action(view, hw, s, ac, d)
                if n.v[d] != s.v[d] and valid(view, hw, n):
                    b = benefit_vthread(view, hw, s, n, d)
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
        e2 = apply_action(view, hw, e, ac, d)
        out.actions.append(ac)
        out.dims.append(d)
        out.states.append(e2.flat())
        if e2.level == 2 or (e2.level == 1 and waves(e2) <= hw.max_waves_per_wg):
            if opts.keep_policy == 0 or uniform(seed, chain, step, 1) < keep_probability(T):
                out.kept.append(e2 if e2.level == 2 else apply_action(view, hw, e2, CACHE, -1))
        e = e2
        T = T / 2.0
        T_level = T0 if ac == CACHE else T_level / 2.0
        step += 1
    return out


def kept_states(view: View, hw: Hw, opts: Opts, seed: int) -> List[Tuple[int, ...]]:
    """The distinct complete states (State.flat()) that Algorithm 1's top_results holds after all walks,
    in order of first appearance."""
    seen, out = set(), []
    for chain in range(opts.chains):
        for s in walk(view, hw, opts, seed, chain).kept:
            key = tuple(s.flat())
            if key not in seen:
                seen.add(key)
                out.append(key)
    return out


def transition_row(view: View, hw: Hw, opts: Opts, s: State, T_level: float) -> List[float]:
    """One row of the transition matrix P of Eq. 4 (over the 9 enumerated actions)."""
    return normalize(get_benefits(view, hw, opts, s, T_level))
