"""TEST INFRASTRUCTURE - not part of the product.

Oracle for the host-side steps that turn measured action times into freeze
ratios (TimelyFreeze Sec. 3.2: pipeline DAG, start times by longest path, the
linear program; App. "Edge Construction Rules"; Sec. 3.3: progressive ratio).
Plain Python / numpy; the LP itself is handed to scipy's solver (a library
primitive serving as a step), everything around it is written out from the
definitions.

Node numbering: action (a, m, s) with a = 0 forward / 1 backward, microbatch
m in [0, M), stage s in [0, S) has id (a M + m) S + s; the source is 2 M S,
the destination 2 M S + 1.

Pins (tests/test_oracle_schedule.py): edge sets of hand-drawn 2 x 2 schedules,
acyclicity, start times against brute-force path enumeration, the GPipe and
1F1B makespans for uniform action times in closed form, the LP against an
exhaustive grid search on 2-stage / 2-microbatch schedules, the LP's batch
time against the longest path at its own solution, monotonicity in r_max.
Interleaved 1F1B and ZBV (Sec. 4.2 "Pipeline Schedules"; edge rule 4): rank
orders written out by hand for small cases, the orders that the installed
PyTorch's torch.distributed.pipelining generates for the same schedules (the
training framework the paper names builds on it), every action exactly once
on the rank that owns its stage, forward before backward, acyclicity, and the
interleaved schedule's closed-form makespan for uniform action times.
"""
from __future__ import annotations

import itertools
import math
from typing import Sequence

import numpy as np

GPIPE, ONE_F_ONE_B, INTERLEAVED_1F1B, ZBV = 0, 1, 2, 3
STAGES_PER_RANK = 2          # of the two schedules that place several stages on a rank


def node_id(a: int, m: int, s: int, M: int, S: int) -> int:
    return (a * M + m) * S + s


def rank_order(s: int, M: int, S: int, schedule: int):
    """GPipe / 1F1B (one stage per rank): order in which the rank of stage s runs its 2 M
    actions, as (a, m) pairs."""
    if schedule == GPIPE:
        return [(0, m) for m in range(M)] + [(1, m) for m in range(M)]
    warm = min(M, S - 1 - s)                       # forwards before the first backward
    order = [(0, m) for m in range(warm)]
    for i in range(M - warm):                      # one forward, one backward
        order += [(0, warm + i), (1, i)]
    order += [(1, m) for m in range(M - warm, M)]  # the remaining backwards
    return order


def n_ranks(S: int, schedule: int) -> int:
    if schedule in (GPIPE, ONE_F_ONE_B):
        return S
    if S % STAGES_PER_RANK:
        raise ValueError("two stages per rank: the number of stages must be even")
    return S // STAGES_PER_RANK


def stage_rank(s: int, S: int, schedule: int) -> int:
    """The rank that owns stage s."""
    R = n_ranks(S, schedule)
    if schedule == INTERLEAVED_1F1B:
        return s % R                                # looped placement: stages r, r + R
    if schedule == ZBV:
        return s if s < R else 2 * R - 1 - s        # V-shaped placement: stages r, 2R - 1 - r
    return s


def _interleaved_order(r: int, M: int, R: int):
    """Interleaved 1F1B on rank r of R with V = 2 model chunks per rank (stages r and r + R):
    the rank works through V M forward and V M backward passes; pass k of either kind belongs
    to chunk (k div g) mod V counted from the first chunk for forwards and from the last for
    backwards, g = M / max(1, M div R) being the microbatches a chunk takes in a row; it runs
    (V - 1) g + 2 (R - 1 - r) forwards ahead (at most all of them), then one forward / one
    backward in turn, then the remaining backwards."""
    V = STAGES_PER_RANK
    rounds = max(1, M // R)
    if M % rounds:
        raise ValueError("the number of microbatches must be a multiple of the number of rounds")
    g = M // rounds
    total = V * M
    warm = min((V - 1) * g + 2 * (R - 1 - r), total)
    done = {}                                       # (a, stage) -> passes so far = next microbatch

    def take(a, k):
        chunk = (k // g) % V
        if a == 1:
            chunk = V - 1 - chunk
        stage = chunk * R + r
        m = done.get((a, stage), 0)
        done[(a, stage)] = m + 1
        return (a, m, stage)

    order = [take(0, k) for k in range(warm)]
    for k in range(total - warm):
        order.append(take(0, warm + k))
        order.append(take(1, k))
    order += [take(1, k) for k in range(total - warm, total)]
    return order


def _zbv_order(r: int, M: int, R: int):
    """Zero-bubble V schedule on rank r of R: chunk 0 is stage r, chunk 1 is stage 2R - 1 - r.
    The schedule separates a backward into its input-gradient and its weight-gradient pass; the
    DAG's backward node stands for both and sits where the input-gradient pass runs.  Phases:
    2 (R - r) - 1 forwards of chunk 0; r times (forward chunk 1, forward chunk 0); R - r times
    (forward chunk 1, backward chunk 1); the stable phase (forward chunk 0 while any is left,
    backward chunk 0, forward chunk 1, backward chunk 1) until chunk 1 has caught up; then the
    backwards that are left, r pairs (chunk 0, chunk 1) first and chunk 0 alone after.  The
    schedule is laid out for max(M, 2R - 1) microbatches and those past M are dropped."""
    n = max(M, 2 * R - 1)
    cnt = {(0, 0): 0, (0, 1): 0, (1, 0): 0, (1, 1): 0}      # (a, chunk) -> passes so far
    stage = (r, 2 * R - 1 - r)
    order = []

    def run(a, chunk):
        m = cnt[(a, chunk)]
        cnt[(a, chunk)] += 1
        if m < M:
            order.append((a, m, stage[chunk]))

    for _ in range(2 * (R - r) - 1):
        run(0, 0)
    for _ in range(r):
        run(0, 1); run(0, 0)
    for _ in range(R - r):
        run(0, 1); run(1, 1)
    while cnt[(0, 1)] < cnt[(0, 0)] or cnt[(0, 0)] < n:
        if cnt[(0, 0)] < n:
            run(0, 0)
        run(1, 0); run(0, 1); run(1, 1)
    for _ in range(r):
        run(1, 0); run(1, 1)
    for _ in range(R - r):
        run(1, 0)
    return order


def rank_orders(M: int, S: int, schedule: int):
    """For every rank the list of (a, m, s) in the order the rank runs them (edge rule 4)."""
    R = n_ranks(S, schedule)
    if schedule == INTERLEAVED_1F1B:
        return [_interleaved_order(r, M, R) for r in range(R)]
    if schedule == ZBV:
        return [_zbv_order(r, M, R) for r in range(R)]
    return [[(a, m, s) for a, m in rank_order(s, M, S, schedule)] for s in range(S)]


def pipeline_dag(S: int, M: int, schedule: int):
    """Edge list (set of (i, j)) of the batch's DAG: the four edge rules."""
    nid = lambda a, m, s: node_id(a, m, s, M, S)
    src, dst = 2 * M * S, 2 * M * S + 1
    E = set()
    E.add((src, nid(0, 0, 0)))                                     # rule 1
    E.add((nid(1, M - 1, 0), dst))
    for s in range(S):                                             # rule 2
        for m in range(M):
            E.add((nid(0, m, s), nid(1, m, s)))
            if m + 1 < M:
                E.add((nid(0, m, s), nid(0, m + 1, s)))
                E.add((nid(1, m, s), nid(1, m + 1, s)))
    for m in range(M):                                             # rule 3
        for s in range(S - 1):
            E.add((nid(0, m, s), nid(0, m, s + 1)))
            E.add((nid(1, m, s + 1), nid(1, m, s)))
    for order in rank_orders(M, S, schedule):                      # rule 4: each rank's own order
        for (a0, m0, s0), (a1, m1, s1) in zip(order, order[1:]):
            E.add((nid(a0, m0, s0), nid(a1, m1, s1)))
    return sorted(E)


def start_times(n_nodes: int, edges, w: Sequence[float]) -> np.ndarray:
    """P_i = max over predecessors (P_j + w_j), P = 0 for nodes without predecessors."""
    preds = [[] for _ in range(n_nodes)]
    succs = [[] for _ in range(n_nodes)]
    indeg = [0] * n_nodes
    for i, j in edges:
        preds[j].append(i)
        succs[i].append(j)
        indeg[j] += 1
    ready = [i for i in range(n_nodes) if indeg[i] == 0]
    P = np.zeros(n_nodes)
    seen = 0
    while ready:
        i = ready.pop()
        seen += 1
        for j in succs[i]:
            P[j] = max(P[j], P[i] + w[i])
            indeg[j] -= 1
            if indeg[j] == 0:
                ready.append(j)
    if seen != n_nodes:
        raise ValueError("the graph has a cycle")
    return P


def freeze_ratio_lp(S: int, M: int, schedule: int, w_min, w_max, r_max: float, lam: float):
    """min P_d - lam sum_i delta_i w_i  subject to constraints [1]-[4] of Sec. 3.2.2.

    w_min, w_max: 2 M S action durations (node numbering above).  The stage budget [4]
    averages over the freezable (backward, w_max > w_min) nodes of the stage.
    Returns dict(r, w, P, P_d, P_d_max, objective)."""
    from scipy.optimize import linprog
    n_act = 2 * M * S
    N = n_act + 2
    w_min = np.r_[np.asarray(w_min, dtype=np.float64), 0.0, 0.0]
    w_max = np.r_[np.asarray(w_max, dtype=np.float64), 0.0, 0.0]
    rng_ = w_max - w_min
    delta = np.where(rng_ > 0, 1.0 / np.where(rng_ > 0, rng_, 1.0), 0.0)
    edges = pipeline_dag(S, M, schedule)
    # variables: P_0..P_{N-1}, w_0..w_{N-1}
    c = np.zeros(2 * N)
    c[N - 1] = 1.0                                  # P_d
    c[N:] = -lam * delta
    A, b = [], []
    for i, j in edges:                              # [1]  P_i + w_i - P_j <= 0
        row = np.zeros(2 * N)
        row[i] += 1.0; row[N + i] += 1.0; row[j] -= 1.0
        A.append(row); b.append(0.0)
    for s in range(S):                              # [4]
        nodes = [node_id(a, m, s, M, S) for a in (0, 1) for m in range(M)]
        free = [i for i in nodes if rng_[i] > 0]
        if not free:
            continue
        row = np.zeros(2 * N)
        for i in free:
            row[N + i] = -delta[i]                  # sum delta (w_max - w) <= r_max n
        A.append(row); b.append(r_max * len(free) - sum(delta[i] * w_max[i] for i in free))
    bounds = [(0.0, None)] * N + [(w_min[i], w_max[i]) for i in range(N)]
    bounds[N - 2] = (0.0, 0.0)                      # [3]  P_s = 0 (w_s = 0 by its bounds)
    res = linprog(c, A_ub=np.array(A), b_ub=np.array(b), bounds=bounds, method="highs")
    if res.status != 0:
        raise RuntimeError(res.message)
    P, w = res.x[:N], res.x[N:]
    r = np.where(rng_ > 0, 1.0 - (w - w_min) * delta, 0.0)
    P_d_max = start_times(N, edges, w_max)[N - 1]
    return {"r": r[:n_act], "w": w[:n_act], "P": P, "P_d": float(P[N - 1]), "P_d_max": float(P_d_max),
            "objective": float(res.fun)}


def actual_freeze_ratio(r: float, t: int, T_m: int, T_f: int) -> float:
    """Progressive ratio of the freezing phase (Sec. 3.3): min(r, r (t - T_m) / (T_f - T_m)) for t > T_m, 0 before."""
    if t <= T_m:
        return 0.0
    return min(r, r * (t - T_m) / (T_f - T_m))
