"""Pins of the oracle's pipeline DAG, start times and freeze-ratio LP (Sec. 3.2;
App. "Edge Construction Rules"; Sec. 3.3) against hand-drawn schedules, brute
force and closed forms."""
import itertools

import numpy as np
import pytest

from oracle import schedule as sc

G, F = sc.GPIPE, sc.ONE_F_ONE_B


def _brute_longest(n, edges, w, target):
    """Longest weighted path into `target` by enumerating every path (tiny graphs only)."""
    succ = {}
    for i, j in edges:
        succ.setdefault(i, []).append(j)
    best = 0.0
    roots = set(range(n)) - {j for _, j in edges}

    def walk(i, acc):
        nonlocal best
        if i == target:
            best = max(best, acc)
        for j in succ.get(i, []):
            walk(j, acc + w[i])
    for r in roots:
        walk(r, 0.0)
    return best


def test_edges_of_a_hand_drawn_two_by_two_schedule():
    S = M = 2
    nid = lambda a, m, s: sc.node_id(a, m, s, M, S)
    f00, f01, f10, f11 = nid(0, 0, 0), nid(0, 0, 1), nid(0, 1, 0), nid(0, 1, 1)      # f(m, s)
    b00, b01, b10, b11 = nid(1, 0, 0), nid(1, 0, 1), nid(1, 1, 0), nid(1, 1, 1)
    src, dst = 8, 9
    common = {(src, f00), (b10, dst),                                   # rule 1
              (f00, b00), (f01, b01), (f10, b10), (f11, b11),           # rule 2: backward after its forward
              (f00, f10), (f01, f11), (b00, b10), (b01, b11),           # rule 2: microbatch order
              (f00, f01), (f10, f11), (b01, b00), (b11, b10)}           # rule 3
    gpipe = common | {(f10, b00), (f11, b01)}                           # rule 4: all forwards before any backward
    # 1F1B: stage 1 (last) alternates from the start: f0 b0 f1 b1; stage 0 warms up with one forward: f0 f1 b0 b1
    one = common | {(b01, f11), (f10, b00)}
    assert set(sc.pipeline_dag(S, M, G)) == gpipe
    assert set(sc.pipeline_dag(S, M, F)) == one
    assert sc.rank_order(1, 2, 2, F) == [(0, 0), (1, 0), (0, 1), (1, 1)]
    assert sc.rank_order(0, 2, 2, F) == [(0, 0), (0, 1), (1, 0), (1, 1)]
    assert sc.rank_order(0, 4, 4, F)[:5] == [(0, 0), (0, 1), (0, 2), (0, 3), (1, 0)]


@pytest.mark.parametrize("S,M,sched", [(2, 2, G), (2, 2, F), (3, 2, F), (2, 3, G), (3, 4, F), (4, 8, G), (4, 8, F)])
def test_every_rank_runs_each_action_once_and_the_graph_is_acyclic(S, M, sched):
    for s in range(S):
        order = sc.rank_order(s, M, S, sched)
        assert sorted(order) == [(a, m) for a in (0, 1) for m in range(M)]
        for m in range(M):
            assert order.index((0, m)) < order.index((1, m))
    E = sc.pipeline_dag(S, M, sched)
    n = 2 * M * S + 2
    P = sc.start_times(n, E, np.ones(n))             # raises on a cycle
    assert P[2 * M * S] == 0.0 and P[-1] > 0


def test_start_times_against_path_enumeration():
    rng = np.random.default_rng(4)
    for S, M, sched in [(2, 2, G), (2, 2, F), (3, 2, F), (2, 3, G), (3, 3, F)]:
        n = 2 * M * S + 2
        E = sc.pipeline_dag(S, M, sched)
        w = np.r_[rng.uniform(0.5, 2.0, n - 2), 0.0, 0.0]
        P = sc.start_times(n, E, w)
        for target in (n - 1, sc.node_id(1, 0, 0, M, S), sc.node_id(0, M - 1, S - 1, M, S)):
            assert P[target] == pytest.approx(_brute_longest(n, E, w, target), rel=1e-12)
    with pytest.raises(ValueError):
        sc.start_times(3, [(0, 1), (1, 2), (2, 0)], [1, 1, 1])


@pytest.mark.parametrize("S,M", [(2, 2), (4, 8), (3, 5)])
def test_uniform_action_times_give_the_textbook_makespans(S, M):
    # every forward takes f, every backward b: both schedules finish after (M + S - 1)(f + b)
    f, b = 1.0, 2.0
    n = 2 * M * S + 2
    w = np.r_[np.full(M * S, f), np.full(M * S, b), 0.0, 0.0]
    for sched in (G, F):
        P = sc.start_times(n, sc.pipeline_dag(S, M, sched), w)
        assert P[-1] == pytest.approx((M + S - 1) * (f + b))


def _grid_search(S, M, sched, w_min, w_max, r_max, steps):
    """Exhaustive search over freeze ratios of the backward nodes on a grid."""
    n_act = 2 * M * S
    n = n_act + 2
    E = sc.pipeline_dag(S, M, sched)
    back = [sc.node_id(1, m, s, M, S) for m in range(M) for s in range(S)]
    grid = np.linspace(0.0, 1.0, steps)
    best = None
    for combo in itertools.product(grid, repeat=len(back)):
        r = dict(zip(back, combo))
        ok = all(np.mean([r[sc.node_id(1, m, s, M, S)] for m in range(M)]) <= r_max + 1e-12 for s in range(S))
        if not ok:
            continue
        w = np.r_[w_max.copy(), 0.0, 0.0]
        for i, ri in r.items():
            w[i] = w_max[i] - ri * (w_max[i] - w_min[i])
        Pd = sc.start_times(n, E, w)[-1]
        key = (round(Pd, 9), sum(combo))
        if best is None or key < best[0]:
            best = (key, Pd, sum(combo))
    return best[1], best[2]


@pytest.mark.parametrize("sched", [G, F])
def test_lp_against_exhaustive_search_on_two_stages_two_microbatches(sched):
    S = M = 2
    rng = np.random.default_rng(10 + sched)
    n_act = 2 * M * S
    for trial in range(3):
        w_max = rng.uniform(1.0, 3.0, n_act)
        w_min = w_max.copy()
        for m in range(M):
            for s in range(S):
                i = sc.node_id(1, m, s, M, S)
                w_min[i] = w_max[i] * rng.uniform(0.4, 0.7)
        for r_max in (0.5, 1.0):
            sol = sc.freeze_ratio_lp(S, M, sched, w_min, w_max, r_max, 1e-4)
            Pd_grid, sum_grid = _grid_search(S, M, sched, w_min, w_max, r_max, steps=11)
            # the grid optimum cannot beat the LP, and comes close to it
            assert sol["P_d"] <= Pd_grid + 1e-9
            assert sol["P_d"] >= Pd_grid - 0.1 * (sol["P_d_max"] - sol["P_d"]) - 1e-9


@pytest.mark.parametrize("S,M,sched", [(2, 2, G), (4, 8, G), (4, 8, F), (3, 4, F)])
def test_lp_solution_is_consistent_and_tight(S, M, sched):
    rng = np.random.default_rng(S * 100 + M * 10 + sched)
    n_act = 2 * M * S
    w_max = rng.uniform(1.0, 2.0, n_act)
    w_min = w_max.copy()
    back = [sc.node_id(1, m, s, M, S) for m in range(M) for s in range(S)]
    w_min[back] = w_max[back] * 0.55
    prev_pd = None
    for r_max in (0.0, 0.3, 0.8, 1.0):
        sol = sc.freeze_ratio_lp(S, M, sched, w_min, w_max, r_max, 1e-4)
        r, w = sol["r"], sol["w"]
        assert np.all(r >= -1e-9) and np.all(r <= 1 + 1e-9)
        assert np.all(r[: M * S] == 0)                                        # forwards cannot be frozen
        for s in range(S):
            assert np.mean([r[sc.node_id(1, m, s, M, S)] for m in range(M)]) <= r_max + 1e-7
        # the LP's batch time is the longest path at its own durations
        n = n_act + 2
        Pd = sc.start_times(n, sc.pipeline_dag(S, M, sched), np.r_[w, 0.0, 0.0])[-1]
        assert sol["P_d"] == pytest.approx(Pd, rel=1e-7)
        assert sol["P_d"] <= sol["P_d_max"] + 1e-9
        if prev_pd is not None:
            assert sol["P_d"] <= prev_pd + 1e-7                               # a larger budget never hurts
        prev_pd = sol["P_d"]
        if r_max == 0.0:
            assert sol["P_d"] == pytest.approx(sol["P_d_max"]) and np.allclose(r, 0, atol=1e-7)
    # with the full budget the batch time is the longest path at w_min ... when lam is small enough
    full = sc.freeze_ratio_lp(S, M, sched, w_min, w_max, 1.0, 1e-6)
    n = n_act + 2
    assert full["P_d"] == pytest.approx(sc.start_times(n, sc.pipeline_dag(S, M, sched), np.r_[w_min, 0.0, 0.0])[-1], rel=1e-6)
    # and freezing is not wasted: some backward actions off the critical path stay below r = 1
    assert full["r"].sum() < M * S - 1e-6 or S == 1


def test_progressive_ratio():
    assert sc.actual_freeze_ratio(0.6, 100, 100, 200) == 0.0
    assert sc.actual_freeze_ratio(0.6, 150, 100, 200) == pytest.approx(0.3)
    assert sc.actual_freeze_ratio(0.6, 200, 100, 200) == pytest.approx(0.6)
    assert sc.actual_freeze_ratio(0.6, 5000, 100, 200) == 0.6
    assert sc.actual_freeze_ratio(0.6, 50, 100, 200) == 0.0


# ---------------------------------------------------------------------------------------------
# Interleaved 1F1B and ZBV (Sec. 4.2 "Pipeline Schedules"; edge rule 4): two stages per rank
# ---------------------------------------------------------------------------------------------
I, Z = sc.INTERLEAVED_1F1B, sc.ZBV


def test_hand_drawn_rank_orders_of_the_two_stage_per_rank_schedules():
    f = lambda m, s: (0, m, s)
    b = lambda m, s: (1, m, s)
    # 2 ranks, 4 stages, 2 microbatches.  Interleaved: rank r owns stages r and r + 2.  Rank 0 is three
    # hops from the end of the pipeline and runs all four forwards ahead; rank 1 runs two, then alternates.
    assert sc.rank_orders(2, 4, I) == [
        [f(0, 0), f(1, 0), f(0, 2), f(1, 2), b(0, 2), b(1, 2), b(0, 0), b(1, 0)],
        [f(0, 1), f(1, 1), f(0, 3), b(0, 3), f(1, 3), b(1, 3), b(0, 1), b(1, 1)]]
    # ZBV: rank r owns stages r and 3 - r (the V).  Rank 0 holds the first and the last stage: its last-stage
    # forwards are each followed at once by their backward; rank 1 holds the two middle stages.
    assert sc.rank_orders(2, 4, Z) == [
        [f(0, 0), f(1, 0), f(0, 3), b(0, 3), f(1, 3), b(1, 3), b(0, 0), b(1, 0)],
        [f(0, 1), f(0, 2), f(1, 1), f(1, 2), b(0, 2), b(0, 1), b(1, 2), b(1, 1)]]
    assert [sc.stage_rank(s, 8, I) for s in range(8)] == [0, 1, 2, 3, 0, 1, 2, 3]
    assert [sc.stage_rank(s, 8, Z) for s in range(8)] == [0, 1, 2, 3, 3, 2, 1, 0]
    # one rank: both schedules degenerate to "a microbatch's forwards, then ..." on a single device
    assert sc.rank_orders(1, 2, Z) == [[f(0, 0), f(0, 1), b(0, 1), b(0, 0)]]
    with pytest.raises(ValueError):
        sc.rank_orders(2, 3, I)                       # an odd number of stages
    with pytest.raises(ValueError):
        sc.rank_orders(5, 4, I)                       # 5 microbatches on 2 ranks: not a whole number of rounds


def _torch_rank_orders(kind, R, M):
    """The same schedules as the installed PyTorch lays them out (torch.distributed.pipelining, on
    which the training framework named in Sec. 4.2 builds): forward and input-gradient / full backward
    passes in order, idle slots and weight-gradient passes left out."""
    S = pytest.importorskip("torch.distributed.pipelining.schedules")
    if kind == I:
        o = object.__new__(S.ScheduleInterleaved1F1B)            # no process group: only the layout routine is used
        o.pp_group_size, o.n_local_stages, o._n_microbatches = R, 2, M
        o.number_of_rounds = max(1, M // R)
        o.microbatches_per_round = M // o.number_of_rounds
    else:
        o = object.__new__(S.ScheduleZBVZeroBubble)
        o.pp_group_size, o.n_local_stages, o._n_microbatches, o.num_stages = R, 2, M, 2 * R
    out = []
    for r in range(R):
        seq = []
        for act in o._calculate_single_rank_operations(r):
            if act is None:
                continue
            kind_ = str(act.computation_type)
            if kind_ == "F":
                seq.append((0, act.microbatch_index, act.stage_index))
            elif kind_ in ("B", "I"):
                seq.append((1, act.microbatch_index, act.stage_index))
        out.append(seq)
    return out


@pytest.mark.parametrize("sched", [I, Z])
def test_rank_orders_equal_the_layout_of_the_installed_pipelining_library(sched):
    checked = 0
    for R in (1, 2, 3, 4, 5):
        for M in (1, 2, 3, 4, 6, 8, 12, 16):
            if sched == I and M % max(1, M // R):
                continue
            try:
                ref = _torch_rank_orders(sched, R, M)
            except (AttributeError, TypeError):
                pytest.skip("this PyTorch lays its schedules out through another routine")
            assert sc.rank_orders(M, 2 * R, sched) == ref, (R, M)
            checked += 1
    assert checked >= 30


@pytest.mark.parametrize("S,M,sched", [(2, 1, I), (4, 2, I), (4, 4, I), (6, 3, I), (8, 8, I), (8, 4, I), (8, 3, I),
                                       (2, 1, Z), (2, 3, Z), (4, 2, Z), (4, 5, Z), (6, 4, Z), (8, 8, Z), (8, 2, Z)])
def test_every_action_once_on_its_own_rank_and_no_cycle(S, M, sched):
    orders = sc.rank_orders(M, S, sched)
    assert len(orders) == S // 2
    for r, order in enumerate(orders):
        stages = [s for s in range(S) if sc.stage_rank(s, S, sched) == r]
        assert len(stages) == 2
        assert sorted(order) == sorted((a, m, s) for a in (0, 1) for m in range(M) for s in stages)
        for s in stages:
            for m in range(M):
                assert order.index((0, m, s)) < order.index((1, m, s))            # forward before its backward
            for a in (0, 1):                                                       # microbatches in order within a stage
                ms = [m for (a_, m, s_) in order if a_ == a and s_ == s]
                assert ms == sorted(ms)
        # a microbatch's forward reaches the rank's later stage after its earlier one; its backward the other way round
        lo, hi = sorted(stages)
        for m in range(M):
            assert order.index((0, m, lo)) < order.index((0, m, hi))
            assert order.index((1, m, hi)) < order.index((1, m, lo))
    E = sc.pipeline_dag(S, M, sched)
    n = 2 * M * S + 2
    P = sc.start_times(n, E, np.ones(n))              # raises on a cycle
    assert P[n - 1] > 0


@pytest.mark.parametrize("R,M", [(2, 2), (2, 6), (3, 3), (3, 9), (4, 8), (4, 12)])
def test_interleaved_makespan_for_uniform_action_times(R, M):
    """With V chunks per rank and equal chunk times f, b the interleaved schedule's bubble is
    (R - 1)(f + b), a V-th of the non-interleaved one measured in whole-stage times: the batch
    takes V M (f + b) + (R - 1)(f + b)."""
    S, V = 2 * R, 2
    E = sc.pipeline_dag(S, M, I)
    n = 2 * M * S + 2
    for f, b in ((1.0, 1.0), (1.0, 2.0), (0.5, 1.75)):
        w = np.r_[np.full(M * S, f), np.full(M * S, b), 0.0, 0.0]
        assert sc.start_times(n, E, w)[n - 1] == pytest.approx(V * M * (f + b) + (R - 1) * (f + b))


def test_lp_on_a_two_rank_zbv_schedule_against_grid_search():
    """S = 2 stages on one rank, M = 2 (ZBV with R = 1): the LP's batch time against an exhaustive
    search over the four backward ratios on a grid."""
    S, M = 2, 2
    rs = np.random.default_rng(4)
    lo = np.r_[rs.uniform(1, 2, M * S), rs.uniform(1, 2, M * S)]
    hi = lo.copy(); hi[M * S:] += rs.uniform(0.5, 2, M * S)
    lo[:M * S] = hi[:M * S]
    sol = sc.freeze_ratio_lp(S, M, Z, lo, hi, 0.5, 1e-6)
    E = sc.pipeline_dag(S, M, Z)
    n = 2 * M * S + 2
    best = np.inf
    grid = np.linspace(0, 1, 11)
    for r in itertools.product(grid, repeat=M * S):
        r = np.array(r)
        ok = all(np.mean([r[m * S + s] for m in range(M)]) <= 0.5 + 1e-12 for s in range(S))
        if not ok:
            continue
        w = np.r_[hi[:M * S], hi[M * S:] - r * (hi[M * S:] - lo[M * S:]), 0.0, 0.0]
        best = min(best, sc.start_times(n, E, w)[n - 1])
    assert sol["P_d"] <= best + 1e-9
    assert sol["P_d"] >= best - 0.12 * np.max(hi - lo)       # the grid's resolution
