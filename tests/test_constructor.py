"""Schedule constructor: pins for the oracle (oracle/construct.py) and parity of the C++
constructor (host code, runs without a GPU) against it.

Pins come from what the paper prints: the constants of the annealing multiplier and of the
keep probability (Section IV-C), special cases of Eq. 1-3, the row-stochastic transition
matrix of Eq. 4, the inverse pair tile/invTile and the level order of Section IV-D, the
loop length of Algorithm 1; plus the published splitmix64 test vector and a brute-force
search of the whole schedule lattice under the same cost model.
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
    up = oc.apply_action(view, s, oc.TILE, 0)
    # doubling one side of a square tile: traffic ratio (2/64)/(1/128+1/64) = 4/3, footprint ratio 3/2
    assert oc.benefit_tiling(view, s, up, OPTS) == pytest.approx(2.0, rel=1e-15)
    assert oc.benefit_tiling(view, up, s, OPTS) == pytest.approx(0.5, rel=1e-15)
    # k: traffic unchanged, footprint doubles
    upk = oc.apply_action(view, s, oc.TILE, 2)
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
    for V in (2, 4):
        wm = V * W // 16                                 # x = 16 * wm = W * V  ->  benefit exactly V
        s = _state(256, 256, 64, wm, 64, 16, (1, 1), 1)
        n = s.copy()
        n.v[0] = V
        assert oc.benefit_vthread(HW, s, n, 0) == V
    s = _state(256, 256, 64, 128, 64, 16, (2, 1), 1)
    assert oc.benefit_vthread(HW, s, s, 0) == 1.0
    small = _state(64, 64, 64, 16, 16, 32, (1, 1), 1)    # x = W: one bank row already, nothing to gain
    n = small.copy()
    n.v[0] = 2
    assert oc.benefit_vthread(HW, small, n, 0) == 1.0


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
                    if ac in (oc.TILE, oc.INVTILE) and not oc.valid(view, HW, oc.apply_action(view, s, ac, d)):
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
            up = oc.apply_action(V4096, s, oc.TILE, d)
            if oc.valid(V4096, HW, up):
                assert oc.apply_action(V4096, up, oc.INVTILE, d).flat() == s.flat()
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
                n = oc.apply_action(V4096, s, ac, d)
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


# ------------------------------------------------------------------ cost model + pick
def _all_complete_states(view):
    g = oc.g_of(view)
    for s0 in _level0_states(view):
        bm, bn, bk = s0.tile[0][0], s0.tile[1][0], s0.tile[2][0]
        for wm, wn, kg, vm, vn in itertools.product([16, 32, 64, 128, 256], [16, 32, 64, 128, 256], [g, 2 * g],
                                                    [1, 2, 4], [1, 2, 4]):
            s = oc.State([[bm, wm, wm // vm], [bn, wn, wn // vn], [bk, kg, kg]], [vm, vn], 2)
            if oc.valid(view, HW, s) and oc.waves(s) <= HW.max_waves_per_wg:
                yield s


def _as_instance(i, s):
    return oc.Instance(i, s.tile[0][0], s.tile[1][0], s.tile[2][0], s.tile[0][1], s.tile[1][1], s.tile[2][1],
                       s.v[0], s.v[1], 1, 2, 0)


def test_cost_model_sanity():
    f = lambda *a: oc.predict_us(V4096, HW, *a)
    assert f(256, 256, 64, 128, 128, 16, 1, 1, 1, 2, 0) > 137.44e9 / 2516.6e6          # never beats the MFMA peak
    assert f(32, 32, 64, 16, 16, 32, 1, 1, 1, 2, 0) > f(128, 128, 64, 64, 64, 16, 1, 1, 1, 2, 0)
    assert f(128, 128, 64, 64, 64, 16, 1, 1, 0, 2, 0) > f(128, 128, 64, 64, 64, 16, 1, 1, 1, 2, 0)   # scalar loads cost
    assert f(256, 256, 128, 128, 128, 16, 1, 1, 1, 2, 0) < 0                                # LDS capacity
    assert f(256, 256, 64, 256, 256, 16, 1, 1, 1, 2, 0) < 0                                 # registers
    bmm = oc.View(1024, 1024, 64, 96, 2, 4, 0)                                              # store-bound: HBM floor
    assert oc.predict_us(bmm, HW, 128, 128, 64, 64, 64, 16, 1, 1, 1, 2, 0) >= 96 * (1024 * 1024 * 4) / (8000e3)


@pytest.mark.parametrize("view", [V4096, oc.View(8192, 3072, 768, 1, 2, 4, 1), oc.View(512, 512, 512, 1, 4, 4, 1)])
def test_pick_is_close_to_the_lattice_optimum(view):
    """Brute force over every complete state of the lattice, all of them taken as available
    instances: the walk's pick must be within 15 % of the best cost-model value."""
    states = list(_all_complete_states(view))
    assert len(states) > 500
    insts = [_as_instance(i, s) for i, s in enumerate(states)]
    costs = [oc.predict_us(view, HW, i.bm, i.bn, i.bk, i.wm, i.wn, i.kg, i.vm, i.vn, 1, 2, 0) for i in insts]
    best = min(c for c in costs if c > 0)
    got, us, scored = oc.construct(view, HW, oc.Opts(chains=256), 0, insts)
    assert got is not None and scored > 50
    assert us <= 1.15 * best


# ------------------------------------------------------------------ C++ constructor == oracle
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
    ]


def _instances_for(gs, p):
    out = []
    for idx in range(gs.num_instances()):
        s = gs.instance_schedule(idx, p)
        if s is not None:
            # also compiled with split tiles: plainly fetched operands, vector loads, double buffer
            split_ok = int(p.op != 2 and s.vec_bytes == 16 and s.stages == 2)
            out.append(oc.Instance(idx, s.tile[0][0], s.tile[1][0], s.tile[2][0], s.tile[0][1], s.tile[1][1],
                                   s.tile[2][1], s.vthread[0], s.vthread[1], 1 if s.vec_bytes == 16 else 0,
                                   s.stages, s.direct_lds, split_ok))
    return out


def test_cpp_walk_equals_oracle_walk_step_by_step():
    from paper_2502_11407_amd import binding as gs
    for p, view in _views():
        for seed in (0, 1, 2, 12345, 2 ** 63 + 5):
            a, d, st = gs.construct_trace(p, seed=seed)
            w = oc.walk(view, HW, OPTS, seed, 0)
            assert list(a) == w.actions and list(d) == w.dims
            assert st.tolist() == w.states


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


def test_cpp_cost_model_and_pick_equal_oracle():
    from paper_2502_11407_amd import binding as gs
    hw = gs.hw_mi355x()
    assert (hw.compute_units, hw.lds_bytes_per_cu, hw.regs_per_lane, hw.lds_banks) == \
        (HW.compute_units, HW.lds_bytes_per_cu, HW.regs_per_lane, HW.lds_banks)
    assert tuple(hw.latency_ns) == HW.latency_ns and tuple(hw.bandwidth_gbs) == HW.bandwidth_gbs
    for p, view in _views():
        insts = _instances_for(gs, p)
        assert insts
        for i in insts:
            s = gs.instance_schedule(i.id, p)
            want = oc.predict_us(view, HW, i.bm, i.bn, i.bk, i.wm, i.wn, i.kg, i.vm, i.vn, i.vec, i.stages, i.direct)
            assert gs.predict_us(s, p) == want
            for split in (2, 3, 8):
                s.split_k = split
                assert gs.predict_us(s, p) == oc.predict_us(view, HW, i.bm, i.bn, i.bk, i.wm, i.wn, i.kg, i.vm, i.vn,
                                                            i.vec, i.stages, i.direct, split)
                # a workspace is asked for exactly where the instance exists with split tiles and the split applies
                if p.op != 2:
                    assert (gs.workspace_bytes(p, s) > 0) <= bool(i.split_ok)
        # gensor_construct assumes aligned dense operands: vector accesses iff the contiguous extents are whole vectors
        epc = 16 // view.e
        vec_ok = view.bsrc == 2 or (view.K % epc == 0 and (view.bsrc == 0 or view.N % epc == 0))
        for seed in (0, 9):
            s = gs.construct(p, seed=seed)
            got, us, scored = oc.construct(view, HW, OPTS, seed, insts, vec_ok)
            assert got is not None
            assert (s.kernel_id, s.predicted_us, s.states_scored, s.split_k) == (got.id, us, scored, got.split)
            assert s.chains == 1024 and 0 < s.iterations <= 100
            assert s.construct_s < 10.0
            # the schedule names a compiled instance that serves the problem
            assert gs.instance_schedule(s.kernel_id, p).describe()["tile_m"] == s.describe()["tile_m"]


def test_construct_rejects_bad_problems():
    from paper_2502_11407_amd import binding as gs
    with pytest.raises(gs.GensorError) as e:
        gs.construct(gs.gemm_problem("f16", 0, 4, 4))
    assert e.value.status == 1
    with pytest.raises(gs.GensorError) as e:
        gs.construct(gs.gemm_problem("f16", 64, 64, 64, 1, 0))
    assert e.value.status == 2
