"""Pins for the CPU oracle: what the mathematics fixes, independent of the oracle's own code.

Covered: hand-worked tables (golden fixtures), exhaustive S^L enumeration, budget
monotonicity, the exact infeasibility condition, reductions to textbook problems
(multiple-choice knapsack, layered shortest path through scipy, running sum, single
layer), an int64 DP on integer tables, and re-evaluation of every returned plan.
"""
import itertools

import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import dijkstra

from golden_io import read_example
from paper_2504_21411_amd.workloads import SplitMix64, random_tables


def bits(a):
    return np.asarray(a, np.float32).view(np.uint32)


# ----------------------------------------------------------------------------- golden tables
@pytest.mark.parametrize("name", ["worked_example_a.txt", "worked_example_b.txt"])
def test_hand_worked_example(oracle_mod, name):
    ex = read_example(name)
    full = oracle_mod.solve(ex["T"], ex["O"], ex["R"], ex["r_index"], ex["E_max"],
                            want_planes=True, want_curve=True)
    assert np.array_equal(bits(full["C"]), bits(ex["C"]))
    assert np.array_equal(full["bp"].astype(np.int64), ex["bp"])
    assert np.array_equal(bits(full["curve"]), bits(ex["C"][-1].min(axis=1)))
    for r in ex["results"]:
        got = oracle_mod.solve(ex["T"], ex["O"], ex["R"], ex["r_index"], r["E"])
        assert bits(got["best_cost"]) == bits(r["best_cost"])
        assert got["best_s"] == r["best_s"]
        assert got["mem_used"] == r["mem_used"]
        assert list(got["plan"]) == r["plan"]
    if "feasible_at_5" in ex:
        cost, nfeas, _ = oracle_mod.brute_force(ex["T"], ex["O"], ex["R"], ex["r_index"], 5)
        assert nfeas == ex["feasible_at_5"] and cost == np.float32(9.0)


def test_brute_force_matches_python_enumeration(oracle_mod):
    """The C enumerator itself against a pure-Python product loop on a few cases."""
    for seed in range(5):
        w = random_tables("t", 1, 4, 3, 10, K=2, seed=100 + seed, o_hi=5)
        T, O, R, ri = w.T[0], w.O[0], w.R, w.r_index[0]
        for E in (3, 7, 10):
            best, feas = np.float32(np.inf), 0
            for p in itertools.product(range(3), repeat=4):
                if sum(int(O[l, p[l]]) for l in range(4)) > E:
                    continue
                acc = T[0, p[0]]
                for l in range(1, 4):
                    acc = np.float32(acc + R[ri[l], p[l - 1], p[l]])
                    acc = np.float32(acc + T[l, p[l]])
                feas += 1
                best = min(best, acc)
            cost, nfeas, _ = oracle_mod.brute_force(T, O, R, ri, E)
            assert nfeas == feas and bits(cost) == bits(best)


# ------------------------------------------------------------------------- exhaustive S^L
@pytest.mark.parametrize("integer", [False, True])
def test_exhaustive_enumeration(oracle_mod, integer):
    rng = SplitMix64(77 if integer else 78)
    n_cases = 1500
    shapes = rng.randint(0, 10 ** 6, n_cases * 4).reshape(n_cases, 4)
    ties_seen = 0
    for c in range(n_cases):
        L = 1 + int(shapes[c, 0] % 6)
        S = 1 + int(shapes[c, 1] % 4)
        M = 1 + int(shapes[c, 2] % 16)
        K = 1 + int(shapes[c, 3] % 3)
        w = random_tables("t", 1, L, S, M, K=K, seed=1000 + c, o_hi=max(1, M // 2),
                          integer=integer)
        T, O, R, ri = w.T[0], w.O[0].copy(), w.R.copy(), w.r_index[0]
        if c % 5 == 0:
            O[shapes[c, 0] % L, shapes[c, 1] % S] = 0          # zero-memory strategy
        if c % 7 == 0:
            R[0, shapes[c, 2] % S, shapes[c, 3] % S] = np.inf  # forbidden transition
        if c % 11 == 0:
            O[shapes[c, 1] % L, shapes[c, 0] % S] = M + 3      # never fits
        E = int(shapes[c, 2] % (M + 1))
        got = oracle_mod.solve(T, O, R, ri, E)
        cost, nfeas, nopt = oracle_mod.brute_force(T, O, R, ri, E)
        assert bits(got["best_cost"]) == bits(cost), (c, L, S, M, E)
        if np.isinf(cost):
            assert got["best_s"] == -1 and got["mem_used"] == -1 and (got["plan"] == -1).all()
        else:
            pc, pm = oracle_mod.plan_cost(T, O, R, ri, got["plan"])
            assert bits(pc) == bits(cost) and pm == got["mem_used"] and pm <= E
            assert got["plan"][-1] == got["best_s"]
            ties_seen += nopt > 1
    if integer:
        assert ties_seen > 50      # the tie-break path really is exercised


# ------------------------------------------------------------------------------ invariants
def test_budget_monotonicity_and_infeasibility(oracle_mod):
    for seed in range(40):
        w = random_tables("t", 1, 5, 4, 24, K=2, seed=300 + seed, o_hi=9)
        T, O, R, ri = w.T[0], w.O[0], w.R, w.r_index[0]
        full = oracle_mod.solve(T, O, R, ri, 24, want_planes=True, want_curve=True)
        C = full["C"]
        # every state is non-increasing in e ("at most e bins")
        assert (C[:, 1:, :] <= C[:, :-1, :]).all()
        need = int(O.min(axis=1).sum())
        for E in range(25):
            r = oracle_mod.solve(T, O, R, ri, E)
            assert np.isinf(r["best_cost"]) == (need > E)
            # the plane of a smaller budget is a prefix of the larger one
            assert bits(r["best_cost"]) == bits(full["curve"][E])
        assert (np.diff(full["curve"][need:]) <= 0).all()


# ------------------------------------------------------------------- textbook special cases
def test_zero_transition_is_multiple_choice_knapsack(oracle_mod):
    for seed in range(20):
        w = random_tables("t", 1, 6, 5, 30, seed=500 + seed, o_hi=8, integer=True)
        T, O = w.T[0], w.O[0]
        R = np.zeros((1, 5, 5), np.float32)
        big = 10 ** 9
        dp = np.full(31, big, np.int64)
        for s in range(5):
            dp[O[0, s]:] = np.minimum(dp[O[0, s]:], int(T[0, s]))
        for l in range(1, 6):
            nd = np.full(31, big, np.int64)
            for s in range(5):
                o, t = int(O[l, s]), int(T[l, s])
                nd[o:] = np.minimum(nd[o:], dp[:31 - o] + t)
            dp = np.minimum(nd, big)
        r = oracle_mod.solve(T, O, R, np.zeros(6, np.int32), 30, want_curve=True)
        want = np.where(dp >= big, np.inf, dp).astype(np.float32)
        assert np.array_equal(bits(r["curve"]), bits(want))


def _layered_graph_shortest(T, O, R, ri, E):
    """Node (l, e_used, s); edges carry R + T; solved by scipy's Dijkstra in fp64."""
    L, S = T.shape
    nid = lambda l, e, s: 1 + (l * (E + 1) + e) * S + s
    n = 2 + L * (E + 1) * S
    rows, cols, vals = [], [], []
    for s in range(S):
        if O[0, s] <= E:
            rows.append(0); cols.append(nid(0, int(O[0, s]), s)); vals.append(float(T[0, s]) + 1e-9)
    for l in range(1, L):
        for e in range(E + 1):
            for i in range(S):
                for j in range(S):
                    e2 = e + int(O[l, j])
                    r = float(R[ri[l], i, j])
                    if e2 <= E and np.isfinite(r):
                        rows.append(nid(l - 1, e, i)); cols.append(nid(l, e2, j))
                        vals.append(r + float(T[l, j]) + 1e-9)
    for e in range(E + 1):
        for s in range(S):
            rows.append(nid(L - 1, e, s)); cols.append(n - 1); vals.append(1e-9)
    g = sp.csr_matrix((vals, (rows, cols)), shape=(n, n))
    d = dijkstra(g, directed=True, indices=0)[n - 1]
    return d


def test_state_graph_shortest_path_scipy(oracle_mod):
    """Integer tables: the fp32 DP is exact, so it must equal a library shortest path on the
    explicit (layer, memory used, strategy) graph."""
    for seed in range(12):
        w = random_tables("t", 1, 5, 3, 12, K=2, seed=700 + seed, o_hi=5, integer=True)
        T, O, R, ri = w.T[0], w.O[0], w.R, w.r_index[0]
        for E in (4, 8, 12):
            d = _layered_graph_shortest(T, O, R, ri, E)
            r = oracle_mod.solve(T, O, R, ri, E)
            if np.isinf(d):
                assert np.isinf(r["best_cost"])
            else:
                assert abs(float(r["best_cost"]) - d) < 1e-4


def test_unconstrained_budget_is_viterbi_chain(oracle_mod):
    """With E >= sum of the largest O the memory axis drops out: a plain min-plus chain."""
    for seed in range(10):
        w = random_tables("t", 1, 7, 6, 40, K=3, seed=800 + seed, o_hi=5)
        T, O, R, ri = w.T[0], w.O[0], w.R, w.r_index[0]
        E = int(O.max(axis=1).sum())
        c = T[0].copy()
        for l in range(1, 7):
            c = ((c[:, None] + R[ri[l]]).astype(np.float32).min(axis=0) + T[l]).astype(np.float32)
        r = oracle_mod.solve(T, O, R, ri, E)
        assert np.array_equal(bits(r["final_row"]), bits(c))
        assert bits(r["best_cost"]) == bits(c.min())


def test_single_strategy_is_running_sum_and_single_layer_is_min(oracle_mod):
    w = random_tables("t", 1, 9, 1, 50, seed=900, o_hi=4)
    T, O = w.T[0], w.O[0]
    R = np.full((1, 1, 1), 0.25, np.float32)
    acc = T[0, 0]
    for l in range(1, 9):
        acc = np.float32(np.float32(acc + np.float32(0.25)) + T[l, 0])
    need = int(O.sum())
    r = oracle_mod.solve(T, O, R, np.zeros(9, np.int32), need)
    assert bits(r["best_cost"]) == bits(acc) and r["mem_used"] == need
    assert np.isinf(oracle_mod.solve(T, O, R, np.zeros(9, np.int32), need - 1)["best_cost"])

    w = random_tables("t", 1, 1, 7, 20, seed=901, o_hi=20)
    T, O = w.T[0], w.O[0]
    for E in range(21):
        fit = O[0] <= E
        r = oracle_mod.solve(T, O, w.R, np.zeros(1, np.int32), E)
        if fit.any():
            want = T[0][fit].min()
            assert bits(r["best_cost"]) == bits(want)
            assert r["best_s"] == int(np.flatnonzero(fit & (T[0] == want))[0])
        else:
            assert np.isinf(r["best_cost"]) and r["best_s"] == -1


def test_tie_break_is_lowest_index_everywhere(oracle_mod):
    """All-equal tables: every argmin must be index 0, final strategy 0."""
    L, S, E = 4, 5, 8
    T = np.ones((L, S), np.float32)
    O = np.ones((L, S), np.int32)
    R = np.zeros((1, S, S), np.float32)
    r = oracle_mod.solve(T, O, R, np.zeros(L, np.int32), E, want_planes=True)
    assert (r["bp"] == 0).all() and r["best_s"] == 0 and list(r["plan"]) == [0] * L


def test_batch_wrapper_global_min(oracle_mod):
    """oracle_solve_batch: every instance equals its own single solve, the winner is the
    lowest-cost instance and, among equal costs, the one with the lowest index."""
    w = random_tables("t", 6, 4, 3, 12, K=2, seed=950, o_hi=5,
                      budget=np.array([12, 2, 9, 12, 5, 7], np.int32))
    res = oracle_mod.solve_batch(w.T, w.O, w.R, w.r_index, w.budget)
    res2 = oracle_mod.solve_batch(w.T, w.O, w.R, w.r_index, w.budget, threads=3)
    for k in ("best_cost", "best_s", "plan", "mem_used", "final_row"):
        assert np.array_equal(res[k], res2[k])
    for b in range(w.B):
        one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], int(w.budget[b]))
        assert np.float32(one["best_cost"]).view(np.uint32) == res["best_cost"][b].view(np.uint32)
        assert one["best_s"] == res["best_s"][b] and one["mem_used"] == res["mem_used"][b]
        assert np.array_equal(one["plan"], res["plan"][b])
        assert np.array_equal(one["final_row"].view(np.uint32), res["final_row"][b].view(np.uint32))
    finite = np.isfinite(res["best_cost"])
    assert not finite[1]                                     # budget 2 < 4 layers * 1 bin
    want = int(np.flatnonzero(res["best_cost"] == res["best_cost"][finite].min())[0])
    assert res["best_instance"] == want == res2["best_instance"]
    # the winner twice in the batch, behind itself: equal costs, the first copy wins
    order = np.array([1, want, 2, want, want], np.int64)
    dup = oracle_mod.solve_batch(w.T[order], w.O[order], w.R, w.r_index[order], w.budget[order])
    assert dup["best_cost"][1] == dup["best_cost"][3] == dup["best_cost"][4]
    assert dup["best_instance"] == 1
    assert oracle_mod.solve_batch(w.T[order], w.O[order], w.R, w.r_index[order],
                                  w.budget[order], threads=5)["best_instance"] == 1
    # nothing fits anywhere: no winner
    none = oracle_mod.solve_batch(w.T[:3], w.O[:3], w.R, w.r_index[:3], np.array([2, 1, 0], np.int32))
    assert none["best_instance"] == -1 and not np.isfinite(none["best_cost"]).any()
    assert (none["best_s"] == -1).all() and (none["plan"] == -1).all()
