"""Schedule constructor: pins for the oracle (oracle/construct.py) and parity of the C++
constructor (host code, runs without a GPU) against it.

Pins come from what the paper prints: the constants of the annealing multiplier and of the
keep probability (Section IV-C), special cases of Eq. 1-3, the row-stochastic transition
matrix of Eq. 4, the inverse pair tile/invTile and the level order of Section IV-D, the
loop length of Algorithm 1; plus the published splitmix64 test vector and a brute-force count
of LDS bank conflicts behind Eq. 3.  The library's pick (its own cost model over the compiled
instances on kept states) is re-derived from the oracle's walks and checked against closed-form
limits here, and against measured launch times in test_cost_model_measured.py.
"""
import itertools
import math

import pytest

from oracle import construct as oc

HW = oc.Hw()
OPTS = oc.Opts()
V4096 = oc.View(4096, 4096, 4096, 1, 2, 4, 0)


# ------------------------------------------------------------------ printed constants
def test_annealing_multiplier_printed_constants():
    assert oc.annealing_factor(0) == pytest.approx(0.5, abs=1e-12)       # 3 / (1 + 5)
    assert oc.annealing_factor(10) == pytest.approx(1.5, abs=1e-12)      # 3 / 2
    assert oc.annealing_factor(20) == pytest.approx(2.5, abs=1e-12)      # 3 / (1 + 1/5)
    assert oc.annealing_factor(200) == pytest.approx(3.0, abs=1e-9)
    assert all(oc.annealing_factor(t) < oc.annealing_factor(t + 1) for t in range(-30, 60))
    assert oc.t_of(2.0 ** 30) == -30 and oc.t_of(2.0 ** -10) == 10


def test_keep_probability_printed_constants():
    assert oc.keep_probability(1.0) == pytest.approx(1 - 1 / (1 + math.e ** 5), abs=1e-12)   # 0.9933
    assert oc.keep_probability(1.0) == pytest.approx(0.99331, abs=1e-5)
    assert oc.keep_probability(math.exp(-10)) == pytest.approx(0.5, abs=1e-12)
    assert oc.keep_probability(math.exp(-20)) == pytest.approx(0.00669, abs=1e-5)


def test_generator_matches_published_splitmix64_vector():
    # splitmix64 seeded with 0: first two outputs 0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4
    assert oc.uniform(0, 0, 0, 0) == (0xE220A8397B1DCDAF >> 11) / 2.0 ** 53
    assert oc.uniform(0, 0, 0, 1) == (0x6E789E6AA1B965F4 >> 11) / 2.0 ** 53
    us = [oc.uniform(7, c, s, j) for c in range(4) for s in range(50) for j in range(2)]
    assert all(0.0 <= u < 1.0 for u in us) and len(set(us)) == len(us)
    assert abs(sum(us) / len(us) - 0.5) < 0.06


# ------------------------------------------------------------------ Eq. 1-3
def _state(tm, tn, tk, wm=16, wn=16, wk=32, v=(1, 1), level=0):
    return oc.State([[tm, wm, wm // v[0]], [tn, wn, wn // v[1]], [tk, wk, wk]], list(v), level)


def test_eq1_special_cases():
    view = oc.View(4096, 4096, 4096, 1, 2, 0, 0)          # no output term: ratios are exact
    s = _state(64, 64, 64)
    assert oc.benefit_tiling(view, s, s, OPTS) == 1.0
    up = oc.apply_action(view, HW, s, oc.TILE, 0)
    # doubling one side of a square tile: traffic ratio (2/64)/(1/128+1/64) = 4/3, footprint ratio 3/2
    assert oc.benefit_tiling(view, s, up, OPTS) == pytest.approx(2.0, rel=1e-15)
    assert oc.benefit_tiling(view, up, s, OPTS) == pytest.approx(0.5, rel=1e-15)
    # k: traffic unchanged, footprint doubles
    upk = oc.apply_action(view, HW, s, oc.TILE, 2)
    assert oc.benefit_tiling(view, s, upk, OPTS) == pytest.approx(2.0, rel=1e-15)
    # the inverted-footprint variant is the same traffic gain divided by the footprint growth
    inv = oc.Opts(tiling_benefit=1)
    assert oc.benefit_tiling(view, s, up, inv) == pytest.approx((4 / 3) / (3 / 2), rel=1e-15)
    # with an output term the gain from a larger tile is smaller than without
    assert oc.benefit_tiling(V4096, s, up, OPTS) < 2.0


def test_eq2_special_cases():
    same = oc.Hw(latency_ns=(100.0, 100.0, 100.0), bandwidth_gbs=(1000.0, 1000.0, 1000.0))
    assert oc.benefit_caching(V4096, same, _state(64, 64, 64)) == 1.0
    s = _state(16, 16, 32)
    S = oc.F(V4096, s, 0)
    assert S == 2 * 32 * 32
    want = (800.0 + S / (8000.0 / 256)) / (64.0 + S / (157286.4 / 256))
    assert oc.benefit_caching(V4096, HW, s) == pytest.approx(want, rel=1e-15)
    # latency-bound for tiny S, bandwidth-bound for huge S
    tiny = oc.Hw(bandwidth_gbs=(1e30, 1e30, 1e30))
    assert oc.benefit_caching(V4096, tiny, s) == pytest.approx(800.0 / 64.0)


def test_eq3_special_cases():
    W = HW.lds_banks * HW.lds_bank_bytes
    kc, nc = V4096, oc.View(4096, 4096, 4096, 1, 2, 4, 1)
    # x = V * W  ->  benefit of going from the plain layout to V phases is exactly V
    for bk, V in ((32, 4), (64, 8), (128, 16)):                       # x = 16 rows * min(2 bk, 256) bytes
        s = _state(128, 128, bk, 64, 64, 16, (1, 1), 1)
        n = s.copy()
        n.v[0] = V
        assert oc.conflict_ways(kc, HW, bk, 0, 1) * W == 16 * min(2 * bk, W) == V * W
        assert oc.benefit_vthread(kc, HW, s, n, 0) == V
        assert oc.benefit_vthread(kc, HW, s, s, 0) == 1.0               # V' = V
        assert oc.benefit_vthread(kc, HW, n, s, 0) == 1.0 / V           # the wrap back to 1
    # an n-contiguous 16-bit tile: 4 k rows are read together, fp32: 2
    s = _state(128, 128, 64, 64, 64, 16, (1, 1), 1)
    n = s.copy()
    n.v[1] = 4
    assert oc.benefit_vthread(nc, HW, s, n, 1) == 4 and oc.benefit_vthread(nc, HW, s, n, 0) == 1.0
    assert oc.conflict_ways(oc.View(512, 512, 512, 1, 4, 4, 1), HW, 32, 1, 1) == 2
    # x <= W: one bank row already, nothing to gain, and no V > 1 on the lattice
    assert oc.conflict_ways(kc, HW, 8, 0, 1) == 1
    # setVThread doubles V up to the conflict-free depth, then wraps
    seq = []
    for _ in range(5):
        s = oc.apply_action(kc, HW, s, oc.SETVTHREAD, 0)
        seq.append(s.v[0])
    assert seq == [2, 4, 8, 1, 2]
    assert not oc.valid(kc, HW, _state(128, 128, 64, 64, 64, 16, (16, 1), 1))


def _lds_pass_conflicts(addr_bytes, width):
    """Most lanes of one LDS pass (256 bytes' worth of lanes) whose accesses share a 4-byte bank."""
    lanes_per_pass = 256 // width
    worst = 0
    for p0 in range(0, len(addr_bytes), lanes_per_pass):
        hits = {}
        for a in addr_bytes[p0:p0 + lanes_per_pass]:
            for b in range(a // 4, (a + width) // 4):
                hits[b % 64] = hits.get(b % 64, 0) + 1
        worst = max(worst, max(hits.values()))
    return worst


def test_eq3_reading_equals_counted_bank_conflicts_of_the_lds_layouts():
    """Brute force: lay the operand tiles out as include/gensor.h and the kernel header define them for V
    virtual threads, issue one wave's fragment read, and count how many lanes of a pass fall on the same
    bank.  The count must be Eq. 3's ceil(x / (V W)) in the reading above."""
    kc = V4096
    for e, bks in ((2, (32, 64, 128)), (4, (16, 32, 64))):
        view = oc.View(4096, 4096, 4096, 1, e, 4, 0)
        for bk in bks:
            pitch = bk * e
            cpr, rpp = pitch // 16, max(1, 256 // pitch)
            V = 1
            while V <= cpr:
                for first_row in (0, 32, 48):
                    for chunk in range(cpr):                 # a 32x32 block: lane l reads row l % 32, the same logical chunk
                        addrs = [(first_row + l) * pitch + (chunk ^ (((first_row + l) // rpp) % V)) * 16 for l in range(32)]
                        assert _lds_pass_conflicts(addrs, 16) == oc.conflict_ways(view, HW, bk, 0, V), (e, bk, V)
                V *= 2
    # n-contiguous 16-bit tile [k][BN * 2 + pad]: a transposing 8-byte read; lane group g = lane / 16 reads 4 k rows
    # (s / 4), 4 lanes of 8 bytes each per row; groups 0, 1 are the two 16-column halves of a 32-column block
    nc = oc.View(4096, 4096, 4096, 1, 2, 4, 1)
    for bn in (128, 256):
        for V, pad in ((1, 0), (2, 32), (4, 64)):
            pitch = bn * 2 + pad
            addrs = []
            for lane in range(64):
                g, s_ = lane // 16, lane % 16
                krow = (g // 2) * 8 + s_ // 4
                col = (g % 2) * 16 + (s_ % 4) * 4
                addrs.append(krow * pitch + col * 2)
            assert _lds_pass_conflicts(addrs, 8) == oc.conflict_ways(nc, HW, 64, 1, V), (bn, V)
    # fp32 [k][BN * 4 + pad]: 4-byte reads, lane l reads column l % 32 of k row 4 * (l / 32)
    nc32 = oc.View(512, 512, 512, 1, 4, 4, 1)
    for V, pad in ((1, 0), (2, 32)):
        addrs = [(4 * (l // 32)) * (64 * 4 + pad) + (l % 32) * 4 for l in range(64)]
        assert _lds_pass_conflicts(addrs, 4) == oc.conflict_ways(nc32, HW, 32, 1, V)


# ------------------------------------------------------------------ Eq. 4 and Section IV-D
def _reachable(view, level_states):
    out = []
    for s in level_states:
        for T_level in (2.0 ** 30, 1.0, 2.0 ** -20):
            out.append((s, T_level))
    return out


def _level0_states(view):
    cap = oc.caps(view)
    g = oc.g_of(view)
    tiles = [16, 32, 64, 128, 256]
    ks = [2 * g, 4 * g, 8 * g]
    for tm, tn, tk in itertools.product(tiles, tiles, ks):
        s = oc.State([[tm, 16, 16], [tn, 16, 16], [tk, 2 * g, 2 * g]], [1, 1], 0)
        if tm <= cap[0] and tn <= cap[1] and tk <= cap[2] and oc.valid(view, HW, s):
            yield s


def test_transition_rows_are_stochastic_and_infeasible_moves_are_zero():
    rows = 0
    for view in (V4096, oc.View(100, 3000, 70, 1, 4, 4, 1)):
        for s in _level0_states(view):
            for T_level in (2.0 ** 30, 1.0, 2.0 ** -20):
                p = oc.transition_row(view, HW, OPTS, s, T_level)
                assert all(x >= 0.0 for x in p) and sum(p) == pytest.approx(1.0, abs=1e-12)
                for i, (ac, d) in enumerate(oc.ACTION_LIST):
                    if ac in (oc.TILE, oc.INVTILE) and not oc.valid(view, HW, oc.apply_action(view, HW, s, ac, d)):
                        assert p[i] == 0.0
                    if ac == oc.SETVTHREAD:
                        assert p[i] == 0.0               # no virtual threads at the LDS level
                rows += 1
    assert rows > 100
    # at the register level a workgroup of too many waves cannot take the last cache
    s = _state(256, 256, 64, 16, 16, 32, (1, 1), 1)
    assert oc.waves(s) == 256
    assert oc.transition_row(V4096, HW, OPTS, s, 1.0)[8] == 0.0
    # LDS capacity: 256x256 tiles cannot take k = 128 (2 stages * 2 B * 128 * 512 = 256 KiB)
    s = _state(256, 256, 64)
    assert oc.transition_row(V4096, HW, OPTS, s, 1.0)[2] == 0.0


def test_tile_and_invtile_are_inverse_and_levels_only_advance():
    for s in _level0_states(V4096):
        for d in range(3):
            up = oc.apply_action(V4096, HW, s, oc.TILE, d)
            if oc.valid(V4096, HW, up):
                assert oc.apply_action(V4096, HW, up, oc.INVTILE, d).flat() == s.flat()
    for seed in range(20):
        w = oc.walk(V4096, HW, OPTS, seed)
        levels = [st[11] for st in w.states]
        assert levels == sorted(levels) and set(levels) <= {0, 1, 2}
        assert [a for a in w.actions].count(oc.CACHE) == levels[-1]


def test_states_of_one_level_communicate():
    """Irreducibility within a memory level: every LDS-level state is reachable from the start
    through moves of positive probability, and the start is reachable from each of them."""
    allst = {tuple(s.flat()): s for s in _level0_states(V4096)}
    start = tuple(oc.initial_state(V4096).flat())
    seen, todo = {start}, [allst[start]]
    while todo:
        s = todo.pop()
        p = oc.transition_row(V4096, HW, OPTS, s, 1.0)
        for i, (ac, d) in enumerate(oc.ACTION_LIST[:6]):
            if p[i] > 0.0:
                n = oc.apply_action(V4096, HW, s, ac, d)
                if tuple(n.flat()) not in seen:
                    seen.add(tuple(n.flat()))
                    todo.append(n)
    assert seen == set(allst)
    for s in allst.values():                           # tile has an inverse with positive probability
        p = oc.transition_row(V4096, HW, OPTS, s, 1.0)
        assert tuple(s.flat()) == start or any(p[3 + d] > 0.0 for d in range(3))


def test_walk_length_determinism_and_completion():
    limit = math.ceil(math.log2(OPTS.T0 / OPTS.threshold))
    assert limit == 100
    done = 0
    for seed in range(40):
        a = oc.walk(V4096, HW, OPTS, seed)
        b = oc.walk(V4096, HW, OPTS, seed)
        assert a.states == b.states and a.actions == b.actions
        assert len(a.actions) <= limit
        if a.states[-1][11] == 2:
            done += 1
        for k in a.kept:
            assert k.level == 2 and oc.valid(V4096, HW, k) and oc.waves(k) <= HW.max_waves_per_wg
    assert done >= 38
    short = oc.Opts(T0=1.0, threshold=2.0 ** -5)
    assert len(oc.walk(V4096, HW, short, 1).actions) <= 5


def test_cache_is_rare_when_a_level_is_entered_and_certain_later():
    s = oc.initial_state(V4096)
    early = oc.transition_row(V4096, HW, OPTS, s, OPTS.T0)[8]
    late = oc.transition_row(V4096, HW, OPTS, s, 2.0 ** -30)[8]
    assert early < 0.02 and late > 0.8


def test_paper_keep_policy_is_a_subset_of_keep_all():
    paper = oc.Opts(keep_policy=1)
    for seed in range(30):
        a = oc.walk(V4096, HW, OPTS, seed).kept
        b = oc.walk(V4096, HW, paper, seed).kept
        assert len(b) <= len(a)
        assert all(any(x.flat() == y.flat() for y in a) for x in b)


# ------------------------------------------------------------------ C++ constructor == oracle (the walk)
def _views():
    from paper_2502_11407_amd import binding as gs
    return [
        (gs.gemm_problem("f16", 4096, 4096, 4096, 0, 1), V4096),
        (gs.gemm_problem("f32", 512, 512, 512, 0, 0), oc.View(512, 512, 512, 1, 4, 4, 1)),
        (gs.gemm_problem("f16", 8192, 3072, 768, 0, 0), oc.View(8192, 3072, 768, 1, 2, 4, 1)),
        (gs.gemm_problem("bf16", 1024, 1024, 64, 0, 1, 96), oc.View(1024, 1024, 64, 96, 2, 4, 0)),
        (gs.conv_problem("f16", 32, 64, 56, 56, 64, 3, 3, 1, 1),
         oc.View(64, 32 * 56 * 56, 576, 1, 2, 4, 2, conv=(32, 64, 56, 56, 3, 3, 1, 1))),
        # pointwise convolution (1x1, no padding): one GEMM per image with an n-contiguous B
        (gs.conv_problem("f16", 32, 256, 56, 56, 512, 1, 1, 2, 0),
         oc.View(512, 28 * 28, 256, 32, 2, 4, 3, conv=(32, 256, 56, 56, 1, 1, 2, 0))),
        (gs.conv_problem("f16", 8, 64, 27, 27, 128, 1, 1, 2, 0),
         oc.View(128, 14 * 14, 64, 8, 2, 4, 1, conv=(8, 64, 27, 27, 1, 1, 2, 0), prepass=1)),
        (gs.conv_problem("f16", 32, 256, 56, 56, 512, 1, 1, 2, 1),
         oc.View(512, 32 * 29 * 29, 256, 1, 2, 4, 2, conv=(32, 256, 56, 56, 1, 1, 2, 1))),
        (gs.conv_problem("f32", 4, 24, 13, 11, 40, 3, 2, 2, 1),
         oc.View(40, 4 * 7 * 6, 24 * 6, 1, 4, 4, 2, conv=(4, 24, 13, 11, 3, 2, 2, 1))),
        (gs.gemm_problem("f16", 65536, 1024, 4, 0, 0), oc.View(65536, 1024, 4, 1, 2, 4, 1)),
        (gs.gemm_problem("f16", 77, 53, 41, 0, 0, 1, "f16"), oc.View(77, 53, 41, 1, 2, 2, 1)),
        # A stored [k][m]
        (gs.gemm_problem("f16", 2048, 1024, 512, 1, 0), oc.View(2048, 1024, 512, 1, 2, 4, 1, asrc=1)),
        (gs.gemm_problem("f32", 200, 136, 72, 1, 1), oc.View(200, 136, 72, 1, 4, 4, 0, asrc=1)),
    ]


def test_cpp_walk_equals_oracle_walk_step_by_step():
    from paper_2502_11407_amd import binding as gs
    vthread_steps = 0
    for p, view in _views():
        for seed in (0, 1, 2, 12345, 2 ** 63 + 5):
            a, d, st = gs.construct_trace(p, seed=seed)
            w = oc.walk(view, HW, OPTS, seed, 0)
            assert list(a) == w.actions and list(d) == w.dims
            assert st.tolist() == w.states
            vthread_steps += w.actions.count(oc.SETVTHREAD)
    assert vthread_steps > 50          # the comparison does exercise setVThread


def test_cpp_walk_equals_oracle_under_options():
    from paper_2502_11407_amd import binding as gs
    p, view = _views()[0]
    for (co, oo) in [(gs.ConstructOpts(0, 0, 0, 0, 1, 0), oc.Opts(tiling_benefit=1)),
                     (gs.ConstructOpts(0, 0, 0, 0, 0, 1), oc.Opts(no_vthread=1)),
                     (gs.ConstructOpts(1.0, 2.0 ** -40, 0, 0, 0, 0), oc.Opts(T0=1.0, threshold=2.0 ** -40)),
                     (gs.ConstructOpts(0, 0, 0, 0, 0, 0, 0, 1), oc.Opts(greedy=1))]:
        for seed in range(4):
            a, d, st = gs.construct_trace(p, seed=seed, opts=co)
            w = oc.walk(view, HW, oo, seed, 0)
            assert list(a) == w.actions and st.tolist() == w.states


# ------------------------------------------------------------------ the library's pick
SPLITS = (1, 2, 3, 4, 6, 8, 12, 16)


def _instances(gs, p):
    out = []
    for idx in range(gs.num_instances()):
        s = gs.instance_schedule(idx, p)
        if s is not None:
            out.append(s)
    return out


def _coords(s):
    return (s.tile[0][0], s.tile[1][0], s.tile[2][0], s.tile[0][1], s.tile[1][1], s.tile[2][1], s.vthread[0], s.vthread[1])


def _usable(p, view, s):
    """What gensor_construct assumes of the operands: aligned and dense, so vector accesses work exactly when the
    contiguous extents are whole vectors; direct staging takes whole k tiles."""
    epc = 16 // view.e
    vec_ok = view.bsrc == 2 or ((view.M if view.asrc else view.K) % epc == 0 and (view.K if view.bsrc == 0 else view.N) % epc == 0)
    if s.vec_bytes == 16 and not vec_ok:
        return False
    if s.direct_lds and view.bsrc != 2 and view.K % s.tile[2][0] != 0:
        return False
    return True


def _best_over(gs, p, view, scheds, no_split=False):
    """argmin of the library's own cost model (through the C ABI) over schedules x split factors."""
    best = None
    for s in scheds:
        for split in SPLITS:
            s.split_k = split
            if split > 1 and (no_split or p.op == 2 or gs.workspace_bytes(p, s) == 0):
                break
            us = gs.predict_us(s, p)
            if us > 0 and (best is None or us < best[0]):
                best = (us, s.kernel_id, split)
        s.split_k = 1
    return best


def test_pick_is_the_cheapest_instance_on_a_state_the_walks_kept():
    """The selection rule, re-derived from the oracle's walks: of the compiled instances that sit on the lattice
    point of a kept state (all eight coordinates; a patch-staged convolution instance: its spatial tiles), the
    one the cost model prices lowest.  So the walk, not the instance list, decides what can be picked."""
    from paper_2502_11407_amd import binding as gs
    hw = gs.hw_mi355x()
    assert (hw.compute_units, hw.lds_bytes_per_cu, hw.regs_per_lane, hw.lds_banks, hw.lds_bank_bytes) == \
        (HW.compute_units, HW.lds_bytes_per_cu, HW.regs_per_lane, HW.lds_banks, HW.lds_bank_bytes)
    assert tuple(hw.latency_ns) == HW.latency_ns and tuple(hw.bandwidth_gbs) == HW.bandwidth_gbs
    # (2048 walks on both sides: the oracle's walks are Python, the default 16384 would take a minute per case)
    variants = ((0, gs.ConstructOpts(0, 0, 2048), oc.Opts(chains=2048)), (9, gs.ConstructOpts(0, 0, 2048), oc.Opts(chains=2048)),
                (0, gs.ConstructOpts(0, 0, 2048, 0, 0, 1), oc.Opts(chains=2048, no_vthread=1)))
    for i, (p, view) in enumerate(_views()):
        insts = [s for s in _instances(gs, p) if _usable(p, view, s)]
        assert insts
        for seed, co, oo in (variants if i < 3 else variants[:1]):        # (the oracle's 4096 walks take seconds per case)
            kept = oc.kept_states(view, HW, oo, seed)
            full = {k[0:1] + k[3:4] + k[6:7] + k[1:2] + k[4:5] + k[7:8] + k[9:11] for k in kept}     # bm bn bk wm wn kg vm vn
            spatial = {c[0:2] + c[3:5] for c in full}
            patch = lambda s: p.op == 2 and s.direct_lds == 1
            cands = [s for s in insts if (_coords(s)[0:2] + _coords(s)[3:5] in spatial if patch(s) else _coords(s) in full)]
            got = gs.construct(p, seed=seed, opts=co)
            assert got.states_scored == len(kept)
            assert got.chains == 2048 and 0 < got.iterations <= 100 and got.construct_s < 10.0
            if not cands:
                continue                                   # the nearest-instance fallback is covered below
            want = _best_over(gs, p, view, cands)
            assert (got.predicted_us, got.kernel_id, got.split_k) == want, (view, seed)
            assert gs.instance_schedule(got.kernel_id, p).describe()["tile_m"] == got.describe()["tile_m"]
            if oo.no_vthread:
                assert (got.vthread[0], got.vthread[1]) == (1, 1) or patch(got)


def test_walks_do_not_miss_the_best_instance():
    """Brute force over every compiled instance that serves the problem: what the walks' pick costs under the
    cost model is within 5 % of the cheapest instance there is."""
    from paper_2502_11407_amd import binding as gs
    for p, view in _views():
        insts = [s for s in _instances(gs, p) if _usable(p, view, s)]
        best = _best_over(gs, p, view, insts)
        got = gs.construct(p, seed=0)
        assert got.predicted_us <= 1.05 * best[0], (view, got.kernel_id, best)


def test_without_setvthread_only_plain_layouts_are_reachable():
    """The ablation of the paper's Table VI: with setVThread disabled every kept state has V = 1, so the pick is
    an instance with the plain LDS layout, and the model prices it above the full walk's pick."""
    from paper_2502_11407_amd import binding as gs
    for p, view in _views()[:3]:
        full = gs.construct(p, seed=0)
        plain = gs.construct(p, seed=0, opts=gs.ConstructOpts(0, 0, 0, 0, 0, 1))
        assert (plain.vthread[0], plain.vthread[1]) == (1, 1)
        assert max(full.vthread[0], full.vthread[1]) > 1
        assert plain.kernel_id != full.kernel_id and plain.predicted_us > full.predicted_us


def _sched(gs, p, bm, bn, bk, wm, wn, kg, vm, vn, vec=1, stages=2, direct=0, split=1):
    s = gs.Schedule()
    s.version = 1
    for d, (a, b) in enumerate(((bm, wm), (bn, wn), (bk, kg))):
        s.tile[d][0], s.tile[d][1], s.tile[d][2] = a, b, b
    s.vthread[0], s.vthread[1] = vm, vn
    s.stages, s.vec_bytes, s.direct_lds, s.split_k = stages, 16 if vec else 2, direct, split
    return s


def test_cost_model_limits_and_monotonicity():
    """Closed-form pins of the library's cost model, through the C ABI: no launch is priced below its MFMA time
    or below its HBM time, capacity violations are infeasible, and each penalty term moves the price the
    right way."""
    from paper_2502_11407_amd import binding as gs
    p = gs.gemm_problem("f16", 4096, 4096, 4096, 0, 1)
    f = lambda *a, **k: gs.predict_us(_sched(gs, p, *a, **k), p)
    t_mfma = 2.0 * 4096 ** 3 / 2516.6e6
    big = f(256, 256, 64, 128, 128, 16, 8, 8, direct=1)
    assert t_mfma < big < 2.5 * t_mfma                                                   # MFMA-bound, and not absurdly above it
    assert f(32, 32, 64, 16, 16, 32, 8, 8) > f(128, 128, 64, 64, 64, 16, 8, 8) > big     # small tiles re-read operands
    assert f(128, 128, 64, 64, 64, 16, 8, 8, vec=0) > f(128, 128, 64, 64, 64, 16, 8, 8)  # element loads cost
    assert f(256, 256, 128, 128, 128, 16, 16, 16) < 0                                    # LDS capacity (two stages of 128 KiB)
    assert f(256, 256, 64, 256, 256, 16, 8, 8) < 0                                       # registers (256 x 256 accumulators per wave)
    assert f(256, 256, 64, 16, 16, 32, 8, 8) < 0                                         # 256 waves per workgroup
    assert f(128, 128, 64, 64, 64, 16, 0, 8) < 0                                         # not a state
    # Eq. 3 in the model: fewer virtual threads = more conflict ways = never cheaper, and dearer once LDS-bound
    prices = [f(128, 128, 64, 64, 64, 16, v, v) for v in (1, 2, 4, 8)]
    assert prices == sorted(prices, reverse=True) and prices[0] > 1.5 * prices[3]
    # store-bound batched matmul: the HBM time of its algorithmic bytes is a floor, and the price is near it
    q = gs.gemm_problem("f16", 1024, 1024, 64, 0, 1, 96)
    t_hbm = 96 * (2 * 2 * 1024 * 64 + 4 * 1024 * 1024) / 8000e3
    us = gs.predict_us(_sched(gs, q, 128, 128, 64, 64, 64, 16, 8, 8), q)
    assert t_hbm < us < 2.5 * t_hbm
    # split-k: nothing to split when the tiles fill whole rounds; a deep-k problem with few tiles gets cheaper
    assert f(256, 256, 64, 128, 128, 16, 8, 8, split=2) < 0
    r = gs.gemm_problem("f16", 512, 512, 32768, 0, 1)
    g = lambda split: gs.predict_us(_sched(gs, r, 128, 128, 128, 64, 64, 16, 16, 16, split=split), r)
    assert 0 < g(16) < g(4) < g(1)
    assert g(16) > 2.0 * 512 * 512 * 32768 / 2516.6e6


def test_construct_rejects_bad_problems():
    from paper_2502_11407_amd import binding as gs
    with pytest.raises(gs.GensorError) as e:
        gs.construct(gs.gemm_problem("f16", 0, 4, 4))
    assert e.value.status == 1
    with pytest.raises(gs.GensorError) as e:
        gs.construct(gs.gemm_problem("f16", 64, 64, 64, 0, 0, 1, "bf16"))      # output neither fp32 nor the input type
    assert e.value.status == 2
