"""CPU oracle for the strategy-search dynamic program.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product package never does.  `build()` compiles the C sources with gcc,
the functions below are thin ctypes/numpy wrappers around them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle_gsearch.so")
_SOURCES = ["gsearch_oracle.c", "brute_force.c", "pipeline_oracle.c"]
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, no FMA contraction, no fast-math)."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES if os.path.exists(os.path.join(_HERE, s))]
    if not force and os.path.exists(_LIB_PATH):
        newest = max(os.path.getmtime(s) for s in srcs)
        if os.path.getmtime(_LIB_PATH) >= newest:
            return _LIB_PATH
    cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", _LIB_PATH] + srcs + ["-lm"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.oracle_brute_force.restype = ctypes.c_int64
        _lib.oracle_enumerate.restype = ctypes.c_int32
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def solve(T, O, R, r_index, E, want_planes=False, want_curve=False):
    """One instance.  T, O: [L][S]; R: [K][S][S]; r_index: [L]; E: budget in bins.

    Returns a dict with best_cost (np.float32), best_s, final_row [S], plan [L],
    mem_used and optionally curve [E+1], C [L][E+1][S], bp [L][E+1][S].
    """
    lib = _load()
    T, O, R, r_index = _f32(T), _i32(O), _f32(R), _i32(r_index)
    L, S = T.shape
    K = R.shape[0]
    assert O.shape == (L, S) and R.shape == (K, S, S) and r_index.shape == (L,)
    best_cost = np.zeros(1, np.float32)
    best_s = np.zeros(1, np.int32)
    final_row = np.zeros(S, np.float32)
    plan = np.zeros(L, np.int32)
    mem = np.zeros(1, np.int32)
    curve = np.zeros(E + 1, np.float32) if want_curve else None
    C = np.zeros((L, E + 1, S), np.float32) if want_planes else None
    bp = np.zeros((L, E + 1, S), np.uint16) if want_planes else None
    rc = lib.oracle_solve(
        ctypes.c_int32(L), ctypes.c_int32(S), ctypes.c_int32(int(E)), ctypes.c_int32(K),
        _p(T, ctypes.c_float), _p(O, ctypes.c_int32), _p(R, ctypes.c_float),
        _p(r_index, ctypes.c_int32), _p(best_cost, ctypes.c_float), _p(best_s, ctypes.c_int32),
        _p(final_row, ctypes.c_float), _p(plan, ctypes.c_int32), _p(mem, ctypes.c_int32),
        _p(curve, ctypes.c_float), _p(C, ctypes.c_float), _p(bp, ctypes.c_uint16))
    if rc != 0:
        raise ValueError(f"oracle_solve failed with code {rc}")
    out = dict(best_cost=best_cost[0], best_s=int(best_s[0]), final_row=final_row, plan=plan,
               mem_used=int(mem[0]))
    if want_curve:
        out["curve"] = curve
    if want_planes:
        out["C"] = C
        out["bp"] = bp
    return out


def plan_cost(T, O, R, r_index, plan):
    """fp32 chain cost and memory of one plan, in the defining order."""
    lib = _load()
    T, O, R, r_index, plan = _f32(T), _i32(O), _f32(R), _i32(r_index), _i32(plan)
    L, S = T.shape
    cost = np.zeros(1, np.float32)
    mem = np.zeros(1, np.int32)
    rc = lib.oracle_plan_cost(
        ctypes.c_int32(L), ctypes.c_int32(S), ctypes.c_int32(R.shape[0]),
        _p(T, ctypes.c_float), _p(O, ctypes.c_int32), _p(R, ctypes.c_float),
        _p(r_index, ctypes.c_int32), _p(plan, ctypes.c_int32), _p(cost, ctypes.c_float),
        _p(mem, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_plan_cost failed with code {rc}")
    return cost[0], int(mem[0])


def _solve_batch_c(T, O, R, r_index, budget):
    """oracle_solve_batch on contiguous arrays: per-instance results and the batch winner."""
    lib = _load()
    B, L, S = T.shape
    res = dict(best_cost=np.zeros(B, np.float32), best_s=np.zeros(B, np.int32),
               final_row=np.zeros((B, S), np.float32), plan=np.zeros((B, L), np.int32),
               mem_used=np.zeros(B, np.int32))
    best = np.zeros(1, np.int32)
    rc = lib.oracle_solve_batch(
        ctypes.c_int32(B), ctypes.c_int32(L), ctypes.c_int32(S), ctypes.c_int32(R.shape[0]),
        _p(T, ctypes.c_float), _p(O, ctypes.c_int32), _p(R, ctypes.c_float),
        _p(r_index, ctypes.c_int32), _p(budget, ctypes.c_int32),
        _p(res["best_cost"], ctypes.c_float), _p(res["best_s"], ctypes.c_int32),
        _p(res["final_row"], ctypes.c_float), _p(res["plan"], ctypes.c_int32),
        _p(res["mem_used"], ctypes.c_int32), _p(best, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_solve_batch failed with code {rc}")
    res["best_instance"] = int(best[0])
    return res


def solve_batch(T, O, R, r_index, budget, threads=1):
    """Batch of instances.  T, O: [B][L][S]; R: [K][S][S]; r_index: [B][L]; budget: [B].

    The whole batch, including the minimum over instances, is oracle_solve_batch (C).
    threads > 1 (the benchmark's all-cores baseline) cuts the batch into contiguous slices,
    runs that same single-threaded C function on each slice side by side, and the winners of
    the slices meet in slice order under the same strict "<"; the result does not depend on
    it.
    """
    T, O, R, r_index, budget = _f32(T), _i32(O), _f32(R), _i32(r_index), _i32(budget)
    B = T.shape[0]
    assert O.shape == T.shape and r_index.shape == T.shape[:2] and budget.shape == (B,)
    if threads <= 1 or B < 2:
        return _solve_batch_c(T, O, R, r_index, budget)
    from concurrent.futures import ThreadPoolExecutor
    n = min(threads, B)
    cuts = [B * i // n for i in range(n + 1)]
    with ThreadPoolExecutor(max_workers=n) as ex:
        parts = list(ex.map(lambda i: _solve_batch_c(T[cuts[i]:cuts[i + 1]], O[cuts[i]:cuts[i + 1]],
                                                     R, r_index[cuts[i]:cuts[i + 1]],
                                                     budget[cuts[i]:cuts[i + 1]]), range(n)))
    res = {k: np.concatenate([p[k] for p in parts]) for k in
           ("best_cost", "best_s", "final_row", "plan", "mem_used")}
    best, arg = np.float32(np.inf), -1
    for i, p in enumerate(parts):
        if p["best_instance"] >= 0 and p["best_cost"][p["best_instance"]] < best:
            best, arg = p["best_cost"][p["best_instance"]], cuts[i] + p["best_instance"]
    res["best_instance"] = arg
    return res


def brute_force(T, O, R, r_index, E):
    """Exhaustive S^L enumeration.  Returns (min_cost, n_feasible, n_optimal)."""
    lib = _load()
    T, O, R, r_index = _f32(T), _i32(O), _f32(R), _i32(r_index)
    L, S = T.shape
    cost = np.zeros(1, np.float32)
    nopt = np.zeros(1, np.int64)
    n = lib.oracle_brute_force(
        ctypes.c_int32(L), ctypes.c_int32(S), ctypes.c_int32(int(E)),
        ctypes.c_int32(R.shape[0]), _p(T, ctypes.c_float), _p(O, ctypes.c_int32),
        _p(R, ctypes.c_float), _p(r_index, ctypes.c_int32), _p(cost, ctypes.c_float),
        _p(nopt, ctypes.c_int64))
    if n < 0:
        raise ValueError("oracle_brute_force: bad arguments or too many plans")
    return cost[0], int(n), int(nopt[0])


def enumerate_strategies(N, tp_max=0, sp_max=0, tpsp_max=0):
    """Descriptor table [S][5] = (tp, sp, dp, sdp, ckpt) in decision-tree order."""
    lib = _load()
    n = lib.oracle_enumerate(ctypes.c_int32(N), ctypes.c_int32(tp_max), ctypes.c_int32(sp_max),
                             ctypes.c_int32(tpsp_max), None, ctypes.c_int32(0))
    if n < 0:
        raise ValueError("oracle_enumerate: N must be a power of two")
    desc = np.zeros((n, 5), np.int32)
    lib.oracle_enumerate(ctypes.c_int32(N), ctypes.c_int32(tp_max), ctypes.c_int32(sp_max),
                         ctypes.c_int32(tpsp_max), _p(desc, ctypes.c_int32), ctypes.c_int32(n))
    return desc


def build_tables(desc, layer, hw, rmodel, M):
    """Alpha-beta cost tables.  desc [S][5]; layer [B][L][6]; hw [4]; rmodel [K][2]."""
    lib = _load()
    desc = _i32(desc)
    layer = np.ascontiguousarray(layer, dtype=np.float64)
    hw = np.ascontiguousarray(hw, dtype=np.float64)
    rmodel = np.ascontiguousarray(rmodel, dtype=np.float64)
    B, L, _ = layer.shape
    S, K = desc.shape[0], rmodel.shape[0]
    T = np.zeros((B, L, S), np.float32)
    O = np.zeros((B, L, S), np.int32)
    R = np.zeros((K, S, S), np.float32)
    rc = lib.oracle_build_tables(
        ctypes.c_int32(B), ctypes.c_int32(L), ctypes.c_int32(S), ctypes.c_int32(int(M)),
        ctypes.c_int32(K), _p(desc, ctypes.c_int32), _p(layer, ctypes.c_double),
        _p(hw, ctypes.c_double), _p(rmodel, ctypes.c_double), _p(T, ctypes.c_float),
        _p(O, ctypes.c_int32), _p(R, ctypes.c_float))
    if rc != 0:
        raise ValueError(f"oracle_build_tables failed with code {rc}")
    return T, O, R


def pipeline_reduce(stage_cost, group_offsets, group_members, group_micro):
    """Pipeline-aware outer reduction.  Returns (group_cost [G] fp32, best_group)."""
    lib = _load()
    stage_cost = _f32(stage_cost)
    group_offsets, group_members, group_micro = _i32(group_offsets), _i32(group_members), _i32(group_micro)
    G = group_micro.shape[0]
    cost = np.zeros(G, np.float32)
    best = np.zeros(1, np.int32)
    rc = lib.oracle_pipeline_reduce(
        ctypes.c_int32(stage_cost.shape[0]), ctypes.c_int32(G), _p(stage_cost, ctypes.c_float),
        _p(group_offsets, ctypes.c_int32), _p(group_members, ctypes.c_int32),
        _p(group_micro, ctypes.c_int32), _p(cost, ctypes.c_float), _p(best, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_pipeline_reduce: bad arguments")
    return cost, int(best[0])


def build_tables_profiled(desc, layer_type, profile, bw, par, M):
    """Profile-driven tables.  desc [S][5]; layer_type [B][L]; profile [Y][3]; bw [NB]; par [5]."""
    lib = _load()
    desc, layer_type = _i32(desc), _i32(layer_type)
    profile = np.ascontiguousarray(profile, dtype=np.float64)
    bw = np.ascontiguousarray(bw, dtype=np.float64)
    par = np.ascontiguousarray(par, dtype=np.float64)
    B, L = layer_type.shape
    S = desc.shape[0]
    T = np.zeros((B, L, S), np.float32)
    O = np.zeros((B, L, S), np.int32)
    rc = lib.oracle_build_tables_profiled(
        ctypes.c_int32(B), ctypes.c_int32(L), ctypes.c_int32(S), ctypes.c_int32(int(M)),
        ctypes.c_int32(profile.shape[0]), ctypes.c_int32(bw.shape[0]), _p(desc, ctypes.c_int32),
        _p(layer_type, ctypes.c_int32), _p(profile, ctypes.c_double), _p(bw, ctypes.c_double),
        _p(par, ctypes.c_double), _p(T, ctypes.c_float), _p(O, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_build_tables_profiled failed with code {rc}")
    return T, O
