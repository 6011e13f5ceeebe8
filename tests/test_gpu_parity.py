"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, bit for bit.

Costs, final rows, argmins, plans, memory use and the best instance must be identical;
with kept planes the whole C and backpointer tables are compared too.  All inputs are
seeded and synthetic.
"""
import dataclasses
import os

import numpy as np
import pytest

from golden_io import read_example
from paper_2504_21411_amd import workloads
from paper_2504_21411_amd.workloads import Workload, random_tables

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def gs():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_21411_amd import binding, runner
    binding.load_library()          # fails loudly if libgsearch.so is missing
    return binding, runner


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def assert_same(got, ref, w, what=""):
    tag = f"{w.name} {what}"
    assert got["data_status"] == 0, tag
    assert np.array_equal(bits(got["best_cost"]), bits(ref["best_cost"])), tag
    assert np.array_equal(got["best_s"], ref["best_s"]), tag
    assert np.array_equal(bits(got["final_row"]), bits(ref["final_row"])), tag
    assert int(got["best_instance"][0]) == ref["best_instance"], tag
    if "plan" in got and got["plan"].shape == ref["plan"].shape:
        assert np.array_equal(got["plan"], ref["plan"]), tag
        assert np.array_equal(got["mem_used"], ref["mem_used"]), tag


def assert_curve(oracle_mod, curve, w, what=""):
    """Best cost for every budget 0..E of every instance, and +inf beyond E."""
    for b in range(w.B):
        E = int(w.budget[b])
        one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E, want_curve=True)
        assert np.array_equal(bits(curve[b, :E + 1]), bits(one["curve"])), (w.name, what, b)
        assert np.isinf(curve[b, E + 1:]).all(), (w.name, what, b)


def oracle_batch(oracle_mod, w, T=None, O=None, R=None):
    return oracle_mod.solve_batch(w.T if T is None else T, w.O if O is None else O,
                                  w.R if R is None else R, w.r_index, w.budget, threads=THREADS)


MODES = {"bp": 0, "generic": 0x2, "nobp": 0x4, "nobp_generic": 0x6,
         "bp_push": 0x8, "bp_tile": 0x10, "nobp_push": 0xC, "nobp_tile": 0x14}

SHAPES = [
    # B, L, S,  M,   K   (S spans every register-tile size class, M spans tile tails)
    (3, 5, 1, 70, 1), (2, 6, 7, 63, 2), (4, 4, 8, 64, 1), (2, 7, 12, 65, 3),
    (3, 5, 16, 300, 1), (2, 4, 24, 1000, 2), (2, 5, 33, 257, 1), (3, 4, 44, 511, 4),
    (2, 3, 64, 320, 1), (2, 3, 65, 200, 2), (2, 3, 96, 260, 1), (1, 3, 100, 130, 1),
    (2, 3, 128, 129, 2), (5, 1, 9, 40, 1), (1, 2, 2, 1, 1),
    (2, 4, 41, 200, 1), (2, 3, 45, 130, 2),   # either side of the half-chunk variant (41..44)
    # beyond the register-tiled sizes: the LDS-streamed tile kernel (uint8 and uint16 bp)
    (2, 3, 129, 130, 2), (3, 4, 200, 150, 1), (2, 3, 256, 70, 1), (2, 3, 300, 90, 2),
    (1, 3, 601, 40, 1),
    # beyond 608 strategies the same kernel runs on 32-row tiles (tile tail at M = 75 and 100)
    (2, 3, 609, 75, 1), (1, 3, 777, 100, 2),
]


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "B%dL%dS%dM%dK%d" % s)
def test_random_tables_match_oracle(gs, oracle_mod, shape, mode):
    _, runner = gs
    B, L, S, M, K = shape
    rng = workloads.SplitMix64(hash(shape) & 0xFFFF)
    budget = rng.randint(0, M, B).astype(np.int32)
    budget[0] = M
    w = random_tables("rand", B, L, S, M, K=K, seed=sum(shape), budget=budget)
    got = runner.solve_workload(w, flags=MODES[mode])
    assert_same(got, oracle_batch(oracle_mod, w), w, mode)


@pytest.mark.parametrize("mode", ["bp_push", "bp_tile", "generic", "nobp_push", "nobp_tile"])
def test_whole_planes_and_backpointers(gs, oracle_mod, mode):
    binding, runner = gs
    w = random_tables("planes", 3, 6, 44, 333, K=2, seed=11,
                      budget=np.array([333, 100, 257], np.int32))
    w.O[0, 2, 5] = 0
    w.O[1, 3, :] = np.minimum(w.O[1, 3, :], 3)
    dw = runner.DeviceWorkload(w)
    with runner.make_context(w, flags=MODES[mode] | binding.GSEARCH_FLAG_KEEP_PLANES) as ctx:
        out = runner.run_step(ctx, dw, backtrace="all")
        C, bp = ctx.gsearch_export_planes(want_bp=not mode.startswith("nobp"))
        curve = ctx.gsearch_budget_curve()
        out = runner.to_numpy(out)
        C, curve = C.cpu().numpy(), curve.cpu().numpy()
        bp = bp.cpu().numpy() if bp is not None else None
    for b in range(w.B):
        E = int(w.budget[b])
        ref = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E, want_planes=True,
                               want_curve=True)
        assert np.array_equal(bits(C[b, :, :E + 1, :]), bits(ref["C"])), (mode, b)
        if bp is not None:
            assert np.array_equal(bp[b, :, :E + 1, :], ref["bp"].astype(np.int32)), (mode, b)
        assert np.array_equal(bits(curve[b, :E + 1]), bits(ref["curve"]))
        assert np.isinf(curve[b, E + 1:]).all()
        assert np.array_equal(out["plan"][b], ref["plan"])


@pytest.mark.parametrize("mode", ["bp_push", "bp_tile", "generic", "nobp"])
@pytest.mark.parametrize("name", ["worked_example_a.txt", "worked_example_b.txt"])
def test_hand_worked_examples_on_gpu(gs, name, mode):
    _, runner = gs
    ex = read_example(name)
    for r in ex["results"]:
        w = Workload("golden", 1, ex["L"], ex["S"], ex["E_max"], ex["K"],
                     np.array([r["E"]], np.int32), ex["r_index"][None, :].copy(), "tables",
                     T=ex["T"][None], O=ex["O"][None], R=ex["R"])
        got = runner.solve_workload(w, flags=MODES[mode])
        assert bits(got["best_cost"])[0] == bits(r["best_cost"])
        assert got["best_s"][0] == r["best_s"] and got["mem_used"][0] == r["mem_used"]
        assert list(got["plan"][0]) == r["plan"]


@pytest.mark.parametrize("mode", ["bp_push", "bp_tile", "generic", "nobp_push", "nobp_tile"])
def test_edge_cases(gs, oracle_mod, mode):
    _, runner = gs
    flags = MODES[mode]
    # ties everywhere: integer tables, many equal candidates
    w = random_tables("ties", 4, 8, 24, 200, K=2, seed=21, o_hi=6, integer=True)
    assert_same(runner.solve_workload(w, flags), oracle_batch(oracle_mod, w), w, "ties")
    # all-equal tables: every argmin must be 0
    w = random_tables("equal", 2, 5, 12, 70, seed=22)
    w.T[:] = 1.0; w.O[:] = 1; w.R[:] = 0.0
    got = runner.solve_workload(w, flags)
    assert_same(got, oracle_batch(oracle_mod, w), w, "equal")
    assert (got["plan"] == 0).all()
    # zero-memory strategies, strategies that never fit, forbidden transitions
    w = random_tables("mixed", 3, 6, 16, 90, K=2, seed=23, o_hi=20)
    w.O[:, :, 3] = 0
    w.O[:, 2, 5] = 91
    w.O[1, 4, :] = 10 ** 9
    w.R[0, 3, :] = np.inf
    w.R[1, :, 7] = np.inf
    got = runner.solve_workload(w, flags)
    ref = oracle_batch(oracle_mod, w)
    assert_same(got, ref, w, "mixed")
    assert np.isinf(ref["best_cost"][1]) and got["best_s"][1] == -1 and (got["plan"][1] == -1).all()
    # budget 0, and a batch where nothing fits
    w = random_tables("zero", 3, 4, 8, 64, seed=24, budget=np.zeros(3, np.int32))
    got = runner.solve_workload(w, flags)
    assert_same(got, oracle_batch(oracle_mod, w), w, "zero")
    assert int(got["best_instance"][0]) == -1 and np.isinf(got["best_cost"]).all()
    w.O[:] = 0
    assert_same(runner.solve_workload(w, flags), oracle_batch(oracle_mod, w), w, "zero-fit")


def test_uint16_backpointers_above_256_strategies(gs, oracle_mod):
    _, runner = gs
    w = random_tables("wide", 2, 3, 300, 90, seed=31, budget=np.array([90, 41], np.int32))
    # make high indices win so that values above 255 must survive the store
    w.T[:, :, :280] += np.float32(50.0)
    got = runner.solve_workload(w, 0)
    ref = oracle_batch(oracle_mod, w)
    assert_same(got, ref, w, "uint16")
    assert ref["plan"].max() > 255
    assert_same(runner.solve_workload(w, 0x4), ref, w, "uint16 nobp")
    # classes stated for a strategy count beyond the class kernel's sizes: the promise is
    # checked, the general kernels run
    wc, r_class = workloads.class_tables("wideclass", 2, 3, 300, 90, [6] * 50, seed=33,
                                         budget=np.array([90, 41], np.int32))
    got = runner.solve_workload(wc, 0, r_class=r_class)
    assert not got["forward_kernel"].startswith("k_dp_class") and got["data_status"] == 0
    assert_same(got, oracle_batch(oracle_mod, wc), wc, "300 strategies with classes")
    wc.R[0, 0, 7] += np.float32(1.0)
    got = runner.solve_workload(wc, 0, r_class=r_class)
    assert got["data_status"] & 0x20


def test_backtrace_instance_lists_and_capacity_errors(gs, oracle_mod):
    import torch
    binding, runner = gs
    w = random_tables("list", 6, 5, 12, 100, seed=41,
                      budget=np.array([100, 3, 50, 77, 100, 20], np.int32))
    ref = oracle_batch(oracle_mod, w)
    dw = runner.DeviceWorkload(w)
    with runner.make_context(w) as ctx:
        with pytest.raises(binding.GSearchError) as ei:
            ctx.gsearch_backtrace(None, 1)
        assert ei.value.code == binding.GSEARCH_ERR_NOT_SOLVED
        runner.run_step(ctx, dw, backtrace=None)
        ids = torch.tensor([4, -1, 0, 99, 2, 1], dtype=torch.int32, device="cuda")
        out = runner.to_numpy(ctx.gsearch_backtrace(ids))
        for q, b in enumerate([4, -1, 0, 99, 2, 1]):
            if 0 <= b < 6:
                assert np.array_equal(out["plan"][q], ref["plan"][b])
                assert out["mem_used"][q] == ref["mem_used"][b]
            else:
                assert (out["plan"][q] == -1).all() and out["mem_used"][q] == -1
        big = random_tables("big", 7, 5, 12, 100, seed=42)
        with pytest.raises(binding.GSearchError) as ei:
            runner.run_step(ctx, runner.DeviceWorkload(big))
        assert ei.value.code == binding.GSEARCH_ERR_CAPACITY
        with pytest.raises(binding.GSearchError) as ei:
            ctx.gsearch_export_planes()
        assert ei.value.code == binding.GSEARCH_ERR_UNSUPPORTED
    # a context may be reused for smaller problems; results do not depend on what ran before
    small = random_tables("small", 2, 3, 7, 40, seed=43)
    with runner.make_context(w) as ctx:
        runner.run_step(ctx, dw, backtrace="all")
        got = runner.to_numpy(runner.run_step(ctx, runner.DeviceWorkload(small), backtrace="all"))
        got["data_status"] = ctx.gsearch_data_status()
    assert_same(got, oracle_batch(oracle_mod, small), small, "reuse")


def test_bad_table_contents_are_flagged_not_fatal(gs):
    binding, runner = gs
    base = random_tables("bad", 2, 4, 12, 80, K=2, seed=51)

    def status_of(mut):
        w = random_tables("bad", 2, 4, 12, 80, K=2, seed=51)
        mut(w)
        out = runner.solve_workload(w)
        assert np.isinf(out["best_cost"]).all() and (out["best_s"] == -1).all()
        assert int(out["best_instance"][0]) == -1 and (out["plan"] == -1).all()
        return out["data_status"]

    def set_(arr, idx, v):
        arr[idx] = v
    assert runner.solve_workload(base)["data_status"] == 0
    assert status_of(lambda w: set_(w.T, (0, 1, 2), np.nan)) == binding.GSEARCH_DATA_BAD_T
    assert status_of(lambda w: set_(w.T, (1, 0, 0), -1.0)) == binding.GSEARCH_DATA_BAD_T
    assert status_of(lambda w: set_(w.T, (1, 0, 0), -0.0)) == binding.GSEARCH_DATA_BAD_T
    assert status_of(lambda w: set_(w.T, (1, 3, 11), np.inf)) == binding.GSEARCH_DATA_BAD_T
    assert status_of(lambda w: set_(w.R, (1, 2, 3), np.nan)) == binding.GSEARCH_DATA_BAD_R
    assert status_of(lambda w: set_(w.R, (0, 0, 0), -2.0)) == binding.GSEARCH_DATA_BAD_R
    assert status_of(lambda w: set_(w.O, (0, 2, 2), -5)) == binding.GSEARCH_DATA_BAD_O
    assert status_of(lambda w: set_(w.budget, 1, 81)) == binding.GSEARCH_DATA_BAD_BUDGET
    assert status_of(lambda w: set_(w.budget, 0, -1)) == binding.GSEARCH_DATA_BAD_BUDGET
    assert status_of(lambda w: set_(w.r_index, (1, 2), 2)) == binding.GSEARCH_DATA_BAD_RINDEX
    ignored = random_tables("bad", 2, 4, 12, 80, K=2, seed=51)
    ignored.r_index[0, 0] = 7                                     # entry l=0 is never read
    out = runner.solve_workload(ignored)
    assert out["data_status"] == 0
    assert np.array_equal(out["best_cost"], runner.solve_workload(base)["best_cost"])
    both = status_of(lambda w: (set_(w.T, (0, 0, 0), np.nan), set_(w.O, (0, 0, 0), -1)))
    assert both == binding.GSEARCH_DATA_BAD_T | binding.GSEARCH_DATA_BAD_O


def test_enumerator_and_table_builder_match_oracle(gs, oracle_mod):
    import torch
    binding, _ = gs
    for N, caps in [(1, (0, 0, 0)), (8, (4, 1, 0)), (8, (0, 2, 0)), (32, (8, 4, 16)),
                    (64, (0, 32, 0)), (256, (0, 0, 0)), (1 << 12, (64, 8, 0))]:
        desc, count = binding.gsearch_enumerate(N, *caps)
        ref = oracle_mod.enumerate_strategies(N, *caps)
        assert int(count.cpu()[0]) == len(ref)
        assert np.array_equal(desc.cpu().numpy(), ref)
    for cfg in (workloads.config1(), workloads.config3()):
        desc, _ = binding.gsearch_enumerate(**cfg.enum)
        dl = torch.from_numpy(cfg.layer).cuda()
        dr = torch.from_numpy(cfg.rmodel).cuda()
        T, O, R = binding.gsearch_build_tables(desc, dl, cfg.hw, dr, cfg.M)
        Tr, Or, Rr = oracle_mod.build_tables(desc.cpu().numpy(), cfg.layer, cfg.hw, cfg.rmodel, cfg.M)
        assert np.array_equal(bits(T.cpu().numpy()), bits(Tr))
        assert np.array_equal(O.cpu().numpy(), Or)
        assert np.array_equal(bits(R.cpu().numpy()), bits(Rr))
    # scales, clamping to M+1 and the one-bin floor
    rng = workloads.SplitMix64(61)
    layer = np.zeros((3, 4, 6))
    layer[..., 0] = 1000.0 + 9000.0 * rng.uniform(12).reshape(3, 4)
    layer[..., 1] = 2048.0
    layer[..., 2] = 65536.0
    layer[..., 3:] = 0.25 + rng.uniform(36).reshape(3, 4, 3)
    rm = np.array([[4096.0, 65536.0], [7000.0, 1.0e6]])
    desc, _ = binding.gsearch_enumerate(16)
    for binb in (1.0e3, 1.0e7, 1.0e12):
        hw = np.array([3.0e14, 4.0e11, binb, 0.3])
        T, O, R = binding.gsearch_build_tables(desc, torch.from_numpy(layer).cuda(), hw,
                                               torch.from_numpy(rm).cuda(), 500)
        Tr, Or, Rr = oracle_mod.build_tables(desc.cpu().numpy(), layer, hw, rm, 500)
        assert np.array_equal(bits(T.cpu().numpy()), bits(Tr))
        assert np.array_equal(O.cpu().numpy(), Or)
        assert np.array_equal(bits(R.cpu().numpy()), bits(Rr))


def test_repeated_solves_are_bit_identical(gs):
    _, runner = gs
    w = random_tables("repeat", 8, 12, 44, 700, K=2, seed=71)
    dw = runner.DeviceWorkload(w)
    with runner.make_context(w) as ctx:
        runs = [runner.to_numpy(runner.run_step(ctx, dw, backtrace="all")) for _ in range(3)]
    for r in runs[1:]:
        for k in ("best_cost", "best_s", "final_row", "plan", "mem_used", "best_instance"):
            assert np.array_equal(runs[0][k], r[k], equal_nan=True), k


# ------------------------------------------------------------------ the five configurations
def _run_config(gs, oracle_mod, i, flags, backtrace="all"):
    """Full-size configuration in the launch configuration bench.py times."""
    _, runner = gs
    w = workloads.get_config(i)
    dw = runner.DeviceWorkload(w)
    with runner.make_context(w, flags=flags) as ctx:
        got = runner.to_numpy(runner.run_step(ctx, dw, backtrace=backtrace))
        got["data_status"] = ctx.gsearch_data_status()
    if w.kind == "model":
        desc = oracle_mod.enumerate_strategies(**w.enum)
        T, O, R = oracle_mod.build_tables(desc, w.layer, w.hw, w.rmodel, w.M)
        assert np.array_equal(got["desc"], desc)
        assert np.array_equal(bits(got["T"]), bits(T)) and np.array_equal(got["O"], O)
        assert np.array_equal(bits(got["R"]), bits(R))
        ref = oracle_batch(oracle_mod, w, T, O, R)
    else:
        ref = oracle_batch(oracle_mod, w)
    assert_same(got, ref, w, f"flags={flags}")
    assert np.isfinite(ref["best_cost"]).any()
    return got, ref


@pytest.mark.parametrize("mode", ["bp", "nobp"])
@pytest.mark.parametrize("i", [0, 1, 2, 4])
def test_config_full_size(gs, oracle_mod, i, mode):
    _run_config(gs, oracle_mod, i, MODES[mode])


@pytest.mark.timeout(600)
def test_config3_large_dense_full_size(gs, oracle_mod):
    """L=128, S=96, M=16384, B=8: the oracle needs about half a minute per instance."""
    _, runner = gs
    w = workloads.get_config(3)
    desc = oracle_mod.enumerate_strategies(**w.enum)
    T, O, R = oracle_mod.build_tables(desc, w.layer, w.hw, w.rmodel, w.M)
    ref = oracle_batch(oracle_mod, w, T, O, R)
    dw = runner.DeviceWorkload(w)
    # the three launch configurations bench.py times (class kernel with and without
    # backpointers, general kernel on two instance groups) and the general min-only pass
    # (the class kernel with 64 layer fronts per launch, its default here, and with one)
    for flags, classes, kernel in ((0, True, "k_dp_class_fronts"), (0x4, True, "k_dp_class_fronts"),
                                   (0, True, "k_dp_class"), (0x4, True, "k_dp_class"),
                                   (0, False, "k_dp_wide"), (0x4, False, "k_dp_wide")):
        with runner.make_context(w, flags=flags) as ctx:
            ctx.gsearch_set_knob("fronts", -1 if kernel.endswith("fronts") else 0)
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", classes=classes))
            got["data_status"] = ctx.gsearch_data_status()
            assert ctx.gsearch_forward_kernel() == kernel
            assert ctx.gsearch_instance_groups() == (1 if classes else 2)
        assert np.array_equal(bits(got["T"]), bits(T)) and np.array_equal(got["O"], O)
        assert_same(got, ref, w, f"flags={flags} classes={classes}")
    assert np.isfinite(ref["best_cost"]).all()


def test_pipeline_aware_reduction(gs, oracle_mod):
    """Outer reduction over (pipeline degree, split, micro-batch) candidates of a reduced
    outer-search batch, then the plans of the winning candidate's stages."""
    import torch
    binding, runner = gs
    w = workloads.config4(B=704)                    # pp 1, 2 and part of pp 4
    off, mem, mic, _ = w.meta["groups"]
    w.budget[5] = 3                                  # one infeasible stage instance
    ref = oracle_batch(oracle_mod, w)
    assert np.isinf(ref["best_cost"][5])
    want_cost, want_best = oracle_mod.pipeline_reduce(ref["best_cost"], off, mem, mic)
    dw = runner.DeviceWorkload(w)
    t32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).cuda()
    with runner.make_context(w) as ctx:
        with pytest.raises(binding.GSearchError) as ei:
            ctx.gsearch_pipeline_reduce(t32(off), t32(mem), t32(mic))
        assert ei.value.code == binding.GSEARCH_ERR_NOT_SOLVED
        runner.run_step(ctx, dw, backtrace=None)
        cost, best = ctx.gsearch_pipeline_reduce(t32(off), t32(mem), t32(mic))
        cost, best = cost.cpu().numpy(), int(best.cpu()[0])
        assert np.array_equal(bits(cost), bits(want_cost)) and best == want_best
        assert np.isinf(cost).any() and np.isfinite(cost).any()
        members = t32(mem[off[best]:off[best + 1]])
        plans = runner.to_numpy(ctx.gsearch_backtrace(members))
        assert np.array_equal(plans["plan"], ref["plan"][mem[off[best]:off[best + 1]]])
        # corrupt offsets must not read outside the member list: the candidate is infeasible
        bad = off.copy(); bad[3] = 10 ** 6
        cost2, _ = ctx.gsearch_pipeline_reduce(t32(bad), t32(mem), t32(mic))
        assert np.isinf(cost2.cpu().numpy()[2:4]).all()


def test_random_shape_sweep(gs, oracle_mod):
    """Forty seeded random shapes (strategy counts around every register-tile size, ragged
    budgets, zero-memory and never-fitting strategies, forbidden transitions), each through
    the automatic kernel choice and one forced variant."""
    _, runner = gs
    rng = workloads.SplitMix64(2024)
    variants = [0x8, 0x10, 0x2, 0xC, 0x14, 0x4]
    for case in range(40):
        v = rng.randint(0, 10 ** 6, 8)
        S = [1, 2, 7, 8, 9, 15, 16, 17, 23, 24, 25, 31, 33, 47, 48, 49, 63, 64, 65, 95, 96, 97,
             127, 128, 129][int(v[0]) % 25]
        B, L, M, K = 1 + int(v[1]) % 5, 1 + int(v[2]) % 6, 1 + int(v[3]) % 700, 1 + int(v[4]) % 3
        budget = rng.randint(0, M, B).astype(np.int32)
        w = random_tables(f"sweep{case}", B, L, S, M, K=K, seed=5000 + case, budget=budget,
                          o_hi=max(1, M // max(1, L - 1)), integer=(case % 4 == 0))
        if case % 3 == 0:
            w.O[int(v[5]) % B, int(v[6]) % L, int(v[7]) % S] = 0
        if case % 5 == 0:
            w.O[:, int(v[5]) % L, int(v[6]) % S] = M + 7
        if case % 7 == 0:
            w.R[int(v[5]) % K, int(v[6]) % S, :] = np.inf
        ref = oracle_batch(oracle_mod, w)
        assert_same(runner.solve_workload(w, 0), ref, w, "auto")
        flags = variants[case % len(variants)]
        assert_same(runner.solve_workload(w, flags), ref, w, f"flags={flags:#x}")


def test_profiled_table_builder_matches_oracle_and_solves(gs, oracle_mod):
    """Tables built on the GPU from a profiler-dump-shaped file equal the oracle's bit for
    bit, and a solve on them matches the oracle's solve."""
    import torch
    binding, runner = gs
    path = os.path.join(os.path.dirname(__file__), "data", "profile_dump_example.json")
    M, B, L = 4096, 6, 20
    names, profile, bw, par = workloads.load_profile_dump(path, M)
    rng = workloads.SplitMix64(77)
    ltype = rng.randint(0, len(names) - 1, B * L).astype(np.int32).reshape(B, L)
    desc, _ = binding.gsearch_enumerate(32, 8, 4, 16)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    T, O = binding.gsearch_build_tables_profiled(desc, dev(ltype), dev(profile), dev(bw), par, M)
    Tr, Or = oracle_mod.build_tables_profiled(desc.cpu().numpy(), ltype, profile, bw, par, M)
    assert np.array_equal(bits(T.cpu().numpy()), bits(Tr)) and np.array_equal(O.cpu().numpy(), Or)
    S = desc.shape[0]
    base = random_tables("prof", B, L, S, M, K=1, seed=78)
    w = Workload("profiled", B, L, S, M, 1, np.full(B, M, np.int32), np.zeros((B, L), np.int32),
                 "tables", T=Tr, O=Or, R=base.R)
    got = runner.solve_workload(w)
    ref = oracle_batch(oracle_mod, w)
    assert_same(got, ref, w, "profiled")
    assert np.isfinite(ref["best_cost"]).all() and len(np.unique(ref["plan"])) > 1
    # a layer type outside the profile poisons the table, and the solve reports it
    bad = ltype.copy(); bad[2, 3] = 9
    T2, O2 = binding.gsearch_build_tables_profiled(desc, dev(bad), dev(profile), dev(bw), par, M)
    assert np.isinf(T2.cpu().numpy()[2, 3]).all() and (O2.cpu().numpy()[2, 3] == M + 1).all()


def test_profiling_entry_points(gs):
    binding, runner = gs
    w = random_tables("timing", 4, 6, 96, 6000, seed=91)       # 376 tiles: the LDS-streamed kernel's range
    dw = runner.DeviceWorkload(w)
    with runner.make_context(w) as ctx:
        assert ctx.gsearch_forward_kernel() == ""
        runner.run_step(ctx, dw, backtrace=None)
        with pytest.raises(binding.GSearchError) as ei:
            ctx.gsearch_forward_ms()                            # profiling was off
        assert ei.value.code == binding.GSEARCH_ERR_NOT_SOLVED
        ctx.gsearch_set_profiling(True)
        runner.run_step(ctx, dw, backtrace=None)
        assert 0.0 < ctx.gsearch_forward_ms() < 1000.0
        assert ctx.gsearch_forward_kernel() == "k_dp_wide"
    small = random_tables("timing_small", 1, 5, 12, 100, seed=92)
    with runner.make_context(small) as ctx:
        runner.run_step(ctx, runner.DeviceWorkload(small), backtrace=None)
        assert ctx.gsearch_forward_kernel() == "k_dp_small"
    with runner.make_context(w, flags=binding.GSEARCH_FLAG_FORCE_GENERIC) as ctx:
        runner.run_step(ctx, dw, backtrace=None)
        assert ctx.gsearch_forward_kernel() == "k_dp_generic"


@pytest.mark.parametrize("mode", ["bp_push", "bp_tile", "generic", "nobp_push", "nobp_tile"])
def test_instance_groups_on_parallel_streams(gs, oracle_mod, mode):
    """The batch cut into 1..8 groups (ragged sizes, more groups than instances) on the
    context's own streams: same bits as the oracle each time, also when one context
    changes the group count from solve to solve and keeps planes."""
    binding, runner = gs
    B = 7
    budget = np.array([900, 64, 511, 0, 900, 333, 700], np.int32)
    w = random_tables("groups", B, 9, 44, 900, K=3, seed=123, budget=budget)
    ref = oracle_batch(oracle_mod, w)
    dw = runner.DeviceWorkload(w)
    with runner.make_context(w, flags=MODES[mode] | binding.GSEARCH_FLAG_KEEP_PLANES) as ctx:
        for groups in (3, 1, 8, 2, 5, 0, 7):
            ctx.gsearch_set_instance_groups(groups)
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all"))
            got["data_status"] = ctx.gsearch_data_status()
            assert_same(got, ref, w, f"{mode} groups={groups}")
            assert ctx.gsearch_instance_groups() == (min(groups, B) if groups else 1)
            C, _ = ctx.gsearch_export_planes(want_bp=False)
            C = C.cpu().numpy()
            for b in (0, 3, 6):
                E = int(w.budget[b])
                one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E, want_planes=True)
                assert np.array_equal(bits(C[b, :, :E + 1, :]), bits(one["C"])), (groups, b)
        with pytest.raises(binding.GSearchError):
            ctx.gsearch_set_instance_groups(-1)


# ------------------------------------------------------------------ transition classes
CLASS_CASES = [
    # S, class sizes, K, M, coarse
    (16, [4, 4, 4, 4], 1, 200, False), (24, [1] * 24, 2, 130, False), (24, [24], 1, 90, True),
    (44, [4] * 11, 1, 300, True), (44, [2, 6, 1, 1, 9, 5, 4, 4, 4, 8], 3, 257, True),
    (64, [2] * 32, 1, 129, False), (96, [4, 4, 4, 4, 4, 4, 2] * 3 + [4, 4, 4, 2, 4], 1, 260, True),
    (100, [25, 25, 25, 25], 2, 100, True), (128, [4] * 32, 1, 70, False),
    (13, [6, 7], 1, 140, True),
    # more than 32 classes: the wide form of the class kernel (announced through r_class_bound)
    (44, [1] * 44, 1, 150, True), (64, [1] * 64, 2, 129, False), (96, [2] * 48, 1, 200, True),
    (128, [2] * 64, 1, 100, True), (100, [1] * 30 + [7] * 10, 1, 130, True),
    (128, [5, 1, 3] * 11 + [29], 3, 90, False),
    # 129..256 strategies: only the class kernel has a register-tiled form there
    (162, [4] * 36 + [2] * 9, 1, 120, True), (192, [6] * 32, 2, 100, False),
    (200, [4] * 50, 1, 90, True), (256, [4] * 64, 1, 70, True), (130, [2] * 63 + [4], 1, 80, False),
]


@pytest.mark.parametrize("fronts", [0, 3], ids=["per_front", "three_fronts_per_launch"])
@pytest.mark.parametrize("mode", ["bp", "nobp"])
@pytest.mark.parametrize("case", CLASS_CASES, ids=lambda c: "S%dnc%dK%d" % (c[0], len(c[1]), c[2]))
def test_class_kernel_matches_oracle(gs, oracle_mod, case, mode, fronts):
    """R constant on (class, class) blocks, stated through r_class: the class kernel must
    give the oracle's bits (the oracle knows nothing of classes), whole planes and
    backpointers included, also when candidates of one class round to the same sum.  Both
    forms: one launch per layer front, and several fronts per launch (which takes batches
    that are a multiple of 8)."""
    binding, runner = gs
    import torch
    S, sizes, K, M, coarse = case
    B, L = (8, 6) if fronts else (3, 6)
    budget = np.array([M, M // 3, max(0, M - 65), M // 2, 0, M - 1, M, 2 * M // 3][:B], np.int32)
    w, r_class = workloads.class_tables("classes", B, L, S, M, sizes, K=K, seed=S + len(sizes),
                                        budget=budget, coarse=coarse)
    ref = oracle_batch(oracle_mod, w)
    dw = runner.DeviceWorkload(w)
    rc = torch.from_numpy(r_class).to(dw.device)
    with runner.make_context(w, flags=MODES[mode] | binding.GSEARCH_FLAG_KEEP_PLANES) as ctx:
        ctx.gsearch_set_knob("fronts", fronts)
        out = runner.run_step(ctx, dw, backtrace="all", r_class=rc, r_class_bound=len(sizes))
        C, bp = ctx.gsearch_export_planes(want_bp=(mode == "bp"))
        got = runner.to_numpy(out)
        got["data_status"] = ctx.gsearch_data_status()
        kernel = ctx.gsearch_forward_kernel()
        C = C.cpu().numpy()
        bp = bp.cpu().numpy() if bp is not None else None
    assert kernel == (("k_dp_class_fronts" if fronts else "k_dp_class") if S >= 9 else kernel)
    assert_same(got, ref, w, f"classes {mode}")
    for b in range(B):
        E = int(w.budget[b])
        one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E, want_planes=True)
        assert np.array_equal(bits(C[b, :, :E + 1, :]), bits(one["C"])), (case, b)
        if bp is not None:
            assert np.array_equal(bp[b, :, :E + 1, :], one["bp"].astype(np.int32)), (case, b)


def test_class_kernel_with_instance_groups_and_single_layer(gs, oracle_mod):
    """Classes combined with forced instance groups (the groups share the class tables), and
    L == 1, where the promise is not even looked at."""
    binding, runner = gs
    import torch
    w, r_class = workloads.class_tables("classgroups", 5, 7, 44, 500, [4] * 11, K=2, seed=31,
                                        budget=np.array([500, 77, 300, 0, 499], np.int32),
                                        coarse=True)
    ref = oracle_batch(oracle_mod, w)
    dw = runner.DeviceWorkload(w)
    rc = torch.from_numpy(r_class).to(dw.device)
    for flags in (0, binding.GSEARCH_FLAG_NO_BACKPOINTERS, binding.GSEARCH_FLAG_KEEP_PLANES):
        with runner.make_context(w, flags=flags) as ctx:
            for groups in (2, 5, 1, 0):
                ctx.gsearch_set_instance_groups(groups)
                got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rc))
                got["data_status"] = ctx.gsearch_data_status()
                assert ctx.gsearch_forward_kernel() == "k_dp_class"
                assert ctx.gsearch_instance_groups() == (groups if groups else 1)
                assert_same(got, ref, w, f"classes groups={groups} flags={flags}")
                if flags & binding.GSEARCH_FLAG_KEEP_PLANES:
                    C, bp = ctx.gsearch_export_planes(want_bp=True)
                    C, bp = C.cpu().numpy(), bp.cpu().numpy()
                    for b in range(w.B):
                        E = int(w.budget[b])
                        one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E,
                                               want_planes=True)
                        assert np.array_equal(bits(C[b, :, :E + 1, :]), bits(one["C"])), (groups, b)
                        assert np.array_equal(bp[b, :, :E + 1, :], one["bp"].astype(np.int32))
    w1, rc1 = workloads.class_tables("classL1", 3, 1, 24, 60, [6] * 4, seed=32)
    got = runner.solve_workload(w1, r_class=np.array([0, 5, 9] + [0] * 21, np.int32))  # nonsense
    assert got["data_status"] == 0
    assert_same(got, oracle_batch(oracle_mod, w1), w1, "L=1")


def _random_partition(rng, S):
    """Random contiguous partition of S strategies into at most 64 classes."""
    nc = 1 + int(rng.randint(0, min(63, S - 1), 1)[0])
    cuts = sorted(set(int(x) for x in rng.randint(1, max(1, S - 1), nc - 1))) if nc > 1 else []
    edges = [0] + [c for c in cuts if 0 < c < S] + [S]
    edges = sorted(set(edges))
    return [b - a for a, b in zip(edges[:-1], edges[1:])]


def _class_sweep_case(runner, oracle_mod, rng, case):
    import torch
    v = rng.randint(0, 10 ** 6, 10)
    S = [9, 12, 16, 17, 24, 31, 32, 33, 44, 48, 49, 64, 65, 96, 100, 128, 129, 162, 192,
         256][int(v[0]) % 20]
    B, L, M, K = 1 + int(v[1]) % 5, 2 + int(v[2]) % 5, 1 + int(v[3]) % 600, 1 + int(v[4]) % 3
    fronts = [0, 2, 0, 64][(case // 2) % 4]        # several fronts per launch: batches of 8, 16
    if fronts:
        B = 8 * (1 + B % 2)
    sizes = _random_partition(rng, S)
    budget = rng.randint(0, M, B).astype(np.int32)
    w, r_class = workloads.class_tables(f"csweep{case}", B, L, S, M, sizes, K=K, seed=9000 + case,
                                        budget=budget, coarse=(case % 2 == 0))
    if case % 7 == 3:                              # memories with a common divisor
        for b in range(B):
            w.O[b] *= [1, 2, 3, 4, 6][(case + b) % 5]
    if case % 3 == 0:
        w.O[int(v[5]) % B, int(v[6]) % L, int(v[7]) % S] = 0
    if case % 5 == 0:
        w.O[:, int(v[5]) % L, int(v[6]) % S] = M + 7
    if case % 4 == 0:                              # a forbidden class-to-class transition
        ci, cj = int(v[8]) % len(sizes), int(v[9]) % len(sizes)
        w.R[int(v[5]) % K][np.ix_(r_class == ci, r_class == cj)] = np.inf
    ref = oracle_batch(oracle_mod, w)
    flags = 0x4 if case % 3 == 1 else 0
    dw = runner.DeviceWorkload(w)
    rc = torch.from_numpy(r_class).to(dw.device)
    with runner.make_context(w, flags=flags) as ctx:
        ctx.gsearch_set_knob("fronts", fronts)
        if case % 6 == 5 and not fronts:
            ctx.gsearch_set_instance_groups(1 + case % 3)
        got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rc,
                                              r_class_bound=len(sizes)))
        got["data_status"] = ctx.gsearch_data_status()
        want = "k_dp_class_fronts" if fronts and L >= 3 else "k_dp_class"
        assert ctx.gsearch_forward_kernel() == want, (case, S)
        curve = ctx.gsearch_budget_curve().cpu().numpy() if case % 4 == 1 else None
    assert_same(got, ref, w, f"class sweep {case} S={S} sizes={sizes} flags={flags}")
    if curve is not None:
        assert_curve(oracle_mod, curve, w, f"class sweep {case}")


def test_class_kernel_random_sweep(gs, oracle_mod):
    """Sixty seeded random class-structured workloads: strategy counts around every
    register-tile size, random partitions of 1..64 classes, several matrices, ragged budgets,
    zero-memory and never-fitting strategies, forbidden class transitions, coarse values that
    make sums collide, memories with a common divisor, both modes, forced instance groups,
    one launch per front and several fronts per launch."""
    _, runner = gs
    rng = workloads.SplitMix64(777)
    for case in range(60):
        _class_sweep_case(runner, oracle_mod, rng, case)


@pytest.mark.parametrize("mode", ["bp", "nobp", "keep"])
@pytest.mark.parametrize("shape", [(8, 20, 44, 3000), (16, 9, 96, 1500), (40, 5, 24, 700),
                                   (24, 6, 44, 900), (64, 12, 16, 260), (67, 5, 24, 300)],
                         ids=lambda t: "B%dL%dS%dM%d" % t)
def test_class_kernel_several_fronts_per_launch(gs, oracle_mod, shape, mode):
    """Several layer fronts per launch at shapes with many tiles per instance and many layers:
    an instance stays on one XCD, tiles wait for the tiles of the previous layer they read,
    and with plane slots taking turns (bp: four, two for three layers; nobp keeps every plane)
    also for those that still read the rows they overwrite.  From the second solve of a context
    on the grid has as many workgroups per front as the solves before found tiles with work.  Budgets are ragged, one instance fits nothing, memories
    are small against the tile (64 rows) in some layers and several tiles wide in others."""
    binding, runner = gs
    import torch
    B, L, S, M = shape
    sizes = [4] * (S // 4)
    rng = workloads.SplitMix64(B * 1000 + L)
    budget = rng.randint(M // 2, M, B).astype(np.int32)
    budget[0] = M
    budget[B // 2] = 3                               # fits nothing
    w, r_class = workloads.class_tables("fronts", B, L, S, M, sizes, K=2, seed=B + L + S,
                                        budget=budget, coarse=(L % 2 == 0))
    w.O[:, 1::3, :] = np.minimum(w.O[:, 1::3, :] * 9, M // 4)     # layers several tiles wide
    w.O[:, 2::3, :] = np.maximum(w.O[:, 2::3, :] // 8, 1)          # layers of a few bins
    ref = oracle_batch(oracle_mod, w)
    flags = {"bp": 0, "nobp": binding.GSEARCH_FLAG_NO_BACKPOINTERS,
             "keep": binding.GSEARCH_FLAG_KEEP_PLANES}[mode]
    dw = runner.DeviceWorkload(w)
    rc = torch.from_numpy(r_class).to(dw.device)
    with runner.make_context(w, flags=flags) as ctx:
        for rep, fronts in enumerate((64, 2, 5)):     # the flags carry over from solve to solve
            ctx.gsearch_set_knob("fronts", fronts)
            assert ctx.gsearch_get_knob("fronts") == fronts
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rc))
            got["data_status"] = ctx.gsearch_data_status()
            assert ctx.gsearch_forward_kernel() == "k_dp_class_fronts"
            assert_same(got, ref, w, f"{fronts} fronts per launch {mode} rep {rep}")
        if mode == "keep":
            C, bp = ctx.gsearch_export_planes(want_bp=True)
            C, bp = C.cpu().numpy(), bp.cpu().numpy()
            for b in (0, B - 1):
                E = int(w.budget[b])
                one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E, want_planes=True)
                assert np.array_equal(bits(C[b, :, :E + 1, :]), bits(one["C"])), b
                assert np.array_equal(bp[b, :, :E + 1, :], one["bp"].astype(np.int32)), b
        ctx.gsearch_set_knob("fronts", 0)
        got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rc))
        got["data_status"] = ctx.gsearch_data_status()
        assert ctx.gsearch_forward_kernel() == "k_dp_class"
        assert_same(got, ref, w, f"per front after several per launch {mode}")


def test_several_fronts_per_launch_on_other_streams_and_in_a_graph(gs, oracle_mod):
    """Which XCD the first workgroup of a launch lands on depends on the stream's hardware
    queue; the several-fronts form only needs an instance's workgroups to share an XCD.  Solves
    on three streams of their own, then a captured step replayed between eager solves."""
    binding, runner = gs
    import torch
    B, L, S, M = 16, 12, 44, 1200
    rng = workloads.SplitMix64(99)
    budget = rng.randint(M // 3, M, B).astype(np.int32)
    w, r_class = workloads.class_tables("streams", B, L, S, M, [4] * 11, K=2, seed=17,
                                        budget=budget, coarse=True)
    ref = oracle_batch(oracle_mod, w)
    dw = runner.DeviceWorkload(w)
    rc = torch.from_numpy(r_class).to(dw.device)
    streams = [torch.cuda.Stream() for _ in range(3)]
    with runner.make_context(w) as ctx:
        for st in streams:
            with torch.cuda.stream(st):
                got = runner.run_step(ctx, dw, backtrace="all", r_class=rc)
                st.synchronize()
                got = runner.to_numpy(got)
                got["data_status"] = ctx.gsearch_data_status()
                assert ctx.gsearch_forward_kernel() == "k_dp_class_fronts"
                assert_same(got, ref, w, "own stream")
        st = streams[1]
        with torch.cuda.stream(st):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=st):
                captured = runner.run_step(ctx, dw, backtrace="all",
                                           r_class=rc)
            for _ in range(3):
                graph.replay()
                got = runner.to_numpy(captured)
                got["data_status"] = ctx.gsearch_data_status()
                assert_same(got, ref, w, "replay")


def most_tiles_with_work(w):
    """Most 64-row tiles with work of any instance and layer front: between the least memory of
    the layers before the front and the budget less the least memory of the layers from it on
    (memories as given: for tables without a common divisor)."""
    mo = np.minimum(w.O.min(axis=2).astype(np.int64), w.M + 1)
    low = np.cumsum(mo, axis=1)
    top = w.budget.astype(np.int64)[:, None] - np.cumsum(mo[:, ::-1], axis=1)[:, ::-1]
    active = np.where(top[:, 1:] >= 0, (top[:, 1:] >> 6) - (low[:, :-1] >> 6) + 1, 0)
    return int(active.max())


@pytest.mark.parametrize("mode", ["bp", "nobp"])
@pytest.mark.parametrize("shape", [(8, 11, 44, 3000), (16, 7, 96, 1500), (67, 5, 24, 2000),
                                   (264, 4, 16, 2000)],
                         ids=lambda t: "B%dL%dS%dM%d" % t)
def test_a_front_with_more_tiles_than_workgroups_is_redone_the_plain_way(gs, oracle_mod, shape,
                                                                        mode):
    """The several-fronts form sizes its grid by the tiles with work that the fronts of earlier
    solves of the context had.  When a solve needs more (here: the knob asks for eight
    workgroups per front, and then a context that has only seen tight budgets is given loose
    ones), the fast launches leave at once and one slow launch does the forward pass with the
    same results; the solve after it has a grid that fits.  264 instances: more workgroups
    than are surely resident together, so an instance gets one."""
    binding, runner = gs
    import torch
    B, L, S, M = shape
    sizes = [4] * (S // 4)
    rng = workloads.SplitMix64(B * 77 + L)
    loose = rng.randint(3 * M // 4, M, B).astype(np.int32)
    loose[0] = M
    tight = np.maximum(loose // 6, 70).astype(np.int32)
    flags = {"bp": 0, "nobp": binding.GSEARCH_FLAG_NO_BACKPOINTERS}[mode]
    cases = {}
    for name, budget in (("loose", loose), ("tight", tight)):
        w, r_class = workloads.class_tables("plain", B, L, S, M, sizes, K=2, seed=B + L + S,
                                            budget=budget, coarse=(L % 2 == 0))
        w.O[:, 1::2, :] = np.maximum(w.O[:, 1::2, :] // 6, 1)     # leaves slack: many tiles with work
        cases[name] = (w, r_class, oracle_batch(oracle_mod, w))
    assert np.gcd.reduce(cases["loose"][0].O.ravel()) == 1
    need_loose, need_tight = (most_tiles_with_work(cases[n][0]) for n in ("loose", "tight"))
    # (what the test is about: eight workgroups are too few for the loose budgets, and so is
    # the grid that the tight budgets leave behind)
    grid_after_tight = need_tight + max(4, need_tight // 16)
    assert need_loose > 8 and need_loose > grid_after_tight, (need_loose, need_tight)
    w0 = cases["loose"][0]
    with runner.make_context(w0, flags=flags) as ctx:
        def solve(name, what):
            w, r_class, ref = cases[name]
            dw = runner.DeviceWorkload(w)
            rc = torch.from_numpy(r_class).to(dw.device)
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rc))
            got["data_status"] = ctx.gsearch_data_status()
            assert ctx.gsearch_forward_kernel() == "k_dp_class_fronts"
            assert_same(got, ref, w, f"{what} {mode}")
        ctx.gsearch_set_knob("front_tiles", 1)          # eight workgroups per instance and front
        solve("loose", "eight workgroups per front")
        solve("loose", "eight workgroups per front, again")
        ctx.gsearch_set_knob("front_tiles", 0)
        for rep in range(3):                              # the context learns the tight need
            solve("tight", f"tight budgets {rep}")
        solve("loose", "loose budgets after tight ones")  # more tiles than the grid has
        solve("loose", "loose budgets, second solve")
        solve("tight", "tight again")


def test_a_captured_solve_stays_right_when_its_inputs_come_to_need_a_larger_grid(gs, oracle_mod):
    """A captured solve keeps the grid it was captured with.  Captured after solves with tight
    budgets, then replayed on loose budgets written into the same device buffers: the fronts
    need more workgroups than the graph's launches have, and every replay still gives the
    loose budgets' results (the slow launch is part of the graph)."""
    binding, runner = gs
    import torch
    B, L, S, M = 8, 9, 44, 3000
    sizes = [4] * (S // 4)
    rng = workloads.SplitMix64(4242)
    loose = rng.randint(3 * M // 4, M, B).astype(np.int32)
    tight = np.maximum(loose // 6, 70).astype(np.int32)
    made = {}
    for name, budget in (("loose", loose), ("tight", tight)):
        w, r_class = workloads.class_tables("graph", B, L, S, M, sizes, K=2, seed=5, budget=budget)
        w.O[:, 1::2, :] = np.maximum(w.O[:, 1::2, :] // 6, 1)
        made[name] = (w, r_class, oracle_batch(oracle_mod, w))
    w_t, r_class, ref_t = made["tight"]
    w_l, _, ref_l = made["loose"]
    assert np.array_equal(w_t.O, w_l.O) and np.array_equal(w_t.T, w_l.T)   # only the budgets differ
    need_t, need_l = most_tiles_with_work(w_t), most_tiles_with_work(w_l)
    assert np.gcd.reduce(w_l.O.ravel()) == 1 and need_l > need_t + max(4, need_t // 16)
    dw = runner.DeviceWorkload(w_t)
    rc = torch.from_numpy(r_class).to(dw.device)
    st = torch.cuda.Stream()
    with runner.make_context(w_t) as ctx, torch.cuda.stream(st):
        for _ in range(3):
            got = runner.run_step(ctx, dw, backtrace="all", r_class=rc)
            st.synchronize()
        got = runner.to_numpy(got)
        got["data_status"] = ctx.gsearch_data_status()
        assert_same(got, ref_t, w_t, "tight, eager")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            captured = runner.run_step(ctx, dw, backtrace="all", r_class=rc)
        graph.replay()
        got = runner.to_numpy(captured)
        got["data_status"] = ctx.gsearch_data_status()
        assert_same(got, ref_t, w_t, "tight, replay")
        dw.budget.copy_(torch.from_numpy(loose).to(dw.device))
        for rep in range(2):
            graph.replay()
            got = runner.to_numpy(captured)
            got["data_status"] = ctx.gsearch_data_status()
            assert_same(got, ref_l, w_l, f"loose, replay {rep}")


def test_a_wait_that_gives_up_ends_the_solve_with_the_internal_status(gs, oracle_mod):
    """The error path of the several-fronts form, forced from the host: with the completion
    flags held back and a spin limit of a few polls every wait gives up, every kernel still
    ends normally, the status word says so, every instance is reported as infeasible, and the
    next solve on the same context is right again."""
    binding, runner = gs
    import torch
    B, L, S, M = 8, 8, 24, 700
    w, r_class = workloads.class_tables("giveup", B, L, S, M, [4] * 6, K=1, seed=12,
                                        budget=np.arange(M - 7, M + 1, dtype=np.int32))
    ref = oracle_batch(oracle_mod, w)
    dw = runner.DeviceWorkload(w)
    rc = torch.from_numpy(r_class).to(dw.device)
    with runner.make_context(w) as ctx:
        ctx.gsearch_set_knob("spin_limit", 4)
        ctx.gsearch_set_knob("hold_flags", 1)
        got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rc))
        assert ctx.gsearch_forward_kernel() == "k_dp_class_fronts"
        assert ctx.gsearch_data_status() == binding.GSEARCH_DATA_INTERNAL
        assert np.isinf(got["best_cost"]).all() and int(got["best_instance"][0]) == -1
        assert (got["plan"] == -1).all()
        ctx.gsearch_set_knob("spin_limit", 0)
        ctx.gsearch_set_knob("hold_flags", 0)
        got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rc))
        got["data_status"] = ctx.gsearch_data_status()
        assert_same(got, ref, w, "after a solve that gave up")


def test_solve_counter_wraps_without_mistaking_old_flags_for_new(gs, oracle_mod):
    """The flags of the several-fronts form hold the number of the solve that set them; the
    counter wraps at 2^29, and the flags are cleared then.  Walk a context across the wrap
    (flags of solves 2^29 - 2 and 2^29 - 1, then 1, 2, 3 again, whose flags the earlier solves
    of this test had set as well)."""
    binding, runner = gs
    import torch
    B, L, S, M = 8, 10, 24, 900
    w, r_class = workloads.class_tables("wrap", B, L, S, M, [4] * 6, K=1, seed=5,
                                        budget=np.arange(M - 7, M + 1, dtype=np.int32))
    other = dataclasses.replace(w, budget=(w.budget // 2).astype(np.int32))
    ref, ref_other = oracle_batch(oracle_mod, w), oracle_batch(oracle_mod, other)
    dw, dwo = runner.DeviceWorkload(w), runner.DeviceWorkload(other)
    rc = torch.from_numpy(r_class).to(dw.device)
    with runner.make_context(w) as ctx:
        for start in (0, (1 << 29) - 3):
            ctx.gsearch_set_solve_counter(start)
            for rep in range(6):
                which, d, r = (w, dw, ref) if rep % 2 == 0 else (other, dwo, ref_other)
                got = runner.to_numpy(runner.run_step(ctx, d, backtrace="all", r_class=rc))
                got["data_status"] = ctx.gsearch_data_status()
                assert ctx.gsearch_forward_kernel() == "k_dp_class_fronts"
                assert_same(got, r, which, f"counter from {start}, solve {rep}")


@pytest.mark.parametrize("mode", ["bp", "nobp", "bp_push", "bp_tile", "nobp_tile", "generic",
                                  "class_bp", "class_nobp", "class_fronts"])
def test_rows_that_no_plan_can_use_are_skipped_exactly(gs, oracle_mod, mode):
    """Every strategy of every layer needs a good share of the budget, so most rows of the
    early layers cannot be completed to a plan within the budget and the forward kernels
    leave them out (unless the planes are kept for export).  What the results are read from
    must not change: costs, final rows, plans of every instance, the budget curve; twice on
    one context, the second time after a solve with kept-planes semantics off and other
    budgets has left other values in the planes."""
    binding, runner = gs
    import torch
    B, L, S, M = 8, 9, 24, 1800
    budget = np.array([M, M - 1, 1300, 1230, 700, 1500, 1264, 1799], np.int32)
    if mode.startswith("class"):
        sizes = [4] * (S // 4)
        w, r_class = workloads.class_tables("topcut", B, L, S, M, sizes, K=2, seed=91,
                                            budget=budget, coarse=True)
    else:
        w, r_class = random_tables("topcut", B, L, S, M, K=2, seed=91, budget=budget), None
    # layer minima between 64 and 200 bins: the budgets of the last two instances fit no
    # plan or only the leanest ones, and the rows cut off span many 64-row tiles
    rng = workloads.SplitMix64(5)
    floor = 64 + rng.randint(0, 136, L)
    w.O[:] = np.minimum(w.O % 90 + floor[None, :, None], M + 1).astype(w.O.dtype)
    ref = oracle_batch(oracle_mod, w)
    assert np.isfinite(ref["best_cost"][:4]).all() and not np.isfinite(ref["best_cost"][4])
    flags = {"class_bp": 0, "class_nobp": 0x4, "class_fronts": 0}.get(mode, MODES.get(mode, 0))
    dw = runner.DeviceWorkload(w)
    kw = {}
    if r_class is not None:
        kw = dict(r_class=torch.from_numpy(r_class).to(dw.device), r_class_bound=S // 4)
    other = dataclasses.replace(w, budget=(w.budget[::-1] // 2).astype(np.int32))
    dother = runner.DeviceWorkload(other)
    with runner.make_context(w, flags=flags) as ctx:
        ctx.gsearch_set_knob("fronts", 4 if mode == "class_fronts" else 0)
        for rep in range(2):
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", **kw))
            got["data_status"] = ctx.gsearch_data_status()
            curve = ctx.gsearch_budget_curve().cpu().numpy()
            assert_same(got, ref, w, f"{mode} rep {rep}")
            assert_curve(oracle_mod, curve, w, f"{mode} rep {rep}")
            if r_class is not None:
                assert ctx.gsearch_forward_kernel().startswith("k_dp_class")
            runner.run_step(ctx, dother, backtrace="all", **kw)


def test_rounding_tie_inside_a_class_keeps_the_lowest_index(gs, oracle_mod):
    """Two strategies of one class, the SECOND has the smaller previous cost, and the class
    transition value is large enough that both sums round to the same fp32 value: the
    lowest-index rule then picks the first, which a class minimum alone would miss."""
    _, runner = gs
    S, L, M = 16, 2, 70
    ulp = np.float32(2.0 ** -13)
    T = np.full((1, L, S), 2000.0, np.float32)
    T[0, 0, 0] = np.float32(1024.0) + ulp      # class 0, index 0: larger cost
    T[0, 0, 1] = np.float32(1024.0)            # class 0, index 1: smaller cost
    O = np.ones((1, L, S), np.int32)
    r_class = np.repeat(np.arange(4, dtype=np.int32), 4)
    Rc = np.full((4, 4), 4096.0, np.float32)
    R = np.ascontiguousarray(Rc[r_class][:, r_class])[None]
    w = Workload("tie", 1, L, S, M, 1, np.array([M], np.int32), np.zeros((1, L), np.int32),
                 "tables", T=T, O=O, R=R)
    assert np.float32(T[0, 0, 0] + np.float32(4096.0)) == np.float32(T[0, 0, 1] + np.float32(4096.0))
    ref = oracle_mod.solve(T[0], O[0], R, w.r_index[0], M, want_planes=True)
    assert (ref["bp"][1, 2:, :] == 0).all()                   # the oracle takes index 0
    got = runner.solve_workload(w, r_class=r_class)
    assert got["forward_kernel"].startswith("k_dp_class") and got["data_status"] == 0
    assert np.array_equal(got["plan"][0], ref["plan"]) and got["plan"][0][0] == 0


def test_bad_transition_classes_are_flagged(gs):
    binding, runner = gs
    w, r_class = workloads.class_tables("badclass", 2, 4, 24, 100, [4] * 6, seed=5)
    ok = runner.solve_workload(w, r_class=r_class)
    assert ok["data_status"] == 0 and np.isfinite(ok["best_cost"]).all()
    cases = {}
    c = r_class.copy(); c[5] = 3                      # not contiguous / not ascending by <= 1
    cases["order"] = (w, c)
    c = r_class.copy(); c[0] = 1
    cases["start"] = (w, c)
    c = r_class.copy(); c[3] = -2
    cases["negative"] = (w, c)
    w40, _ = workloads.class_tables("many", 2, 3, 40, 60, [1] * 40, seed=6)
    cases["more_than_announced"] = (w40, np.arange(40, dtype=np.int32), 32)
    w80, _ = workloads.class_tables("toomany", 2, 3, 80, 60, [1] * 80, seed=7)
    cases["too_many"] = (w80, np.arange(80, dtype=np.int32), 80)
    import copy
    w2 = copy.deepcopy(w); w2.R = w.R.copy(); w2.R[0, 1, 9] += np.float32(0.5)   # row differs inside class 0
    cases["row"] = (w2, r_class)
    w3 = copy.deepcopy(w); w3.R = w.R.copy(); w3.R[0, 9, 2] += np.float32(0.5)   # column differs
    cases["column"] = (w3, r_class)
    ok40 = runner.solve_workload(w40, r_class=np.arange(40, dtype=np.int32))   # announced: fine
    assert ok40["data_status"] == 0 and ok40["forward_kernel"].startswith("k_dp_class")
    # the bound is an upper bound: larger than the count (even absurdly) is fine, and a
    # negative one means "not announced"
    for bound in (64, 10 ** 6, -5):
        got = runner.solve_workload(w, r_class=r_class, r_class_bound=bound)
        assert got["data_status"] == 0 and got["forward_kernel"].startswith("k_dp_class"), bound
        assert np.array_equal(bits(got["best_cost"]), bits(ok["best_cost"])), bound
        assert np.array_equal(got["plan"], ok["plan"]), bound
    got = runner.solve_workload(w40, r_class=np.arange(40, dtype=np.int32), r_class_bound=10 ** 6)
    assert got["data_status"] == 0 and np.array_equal(got["plan"], ok40["plan"])
    for name, case in cases.items():
        ww, cc = case[0], case[1]
        got = runner.solve_workload(ww, r_class=cc, r_class_bound=case[2] if len(case) > 2 else None)
        assert got["data_status"] & binding.GSEARCH_DATA_BAD_RCLASS, name
        assert np.isinf(got["best_cost"]).all() and (got["best_s"] == -1).all(), name
        assert int(got["best_instance"][0]) == -1, name
    # forced kernels ignore the classes but the promise is still checked
    got = runner.solve_workload(w2, flags=MODES["bp_tile"], r_class=r_class)
    assert got["data_status"] & binding.GSEARCH_DATA_BAD_RCLASS
    got = runner.solve_workload(w, flags=MODES["bp_push"], r_class=r_class)
    assert got["data_status"] == 0 and got["forward_kernel"] == "k_dp_push"


def test_layout_classes_of_enumerated_strategies(gs, oracle_mod):
    binding, _ = gs
    for enum in (dict(N=32, tp_max=8, sp_max=4, tpsp_max=16), dict(N=64, sp_max=32), dict(N=8)):
        desc, _ = binding.gsearch_enumerate(**enum)
        r_class, count = binding.gsearch_layout_classes(desc)
        d = oracle_mod.enumerate_strategies(**enum)
        change = np.any(d[1:, :3] != d[:-1, :3], axis=1)
        want = np.concatenate([[0], np.cumsum(change)]).astype(np.int32)
        assert np.array_equal(r_class.cpu().numpy(), want)
        assert int(count.cpu()[0]) == want[-1] + 1


@pytest.mark.timeout(600)
@pytest.mark.parametrize("i", [1, 3])
def test_model_configs_without_classes_use_the_general_kernels(gs, oracle_mod, i):
    """The model workloads hand their layout classes to the solve by default; withheld, the
    general kernels must give the same bits."""
    _, runner = gs
    w = workloads.get_config(i) if i == 1 else workloads.config3()
    if i == 3:
        w.B, w.layer, w.budget, w.r_index = 2, w.layer[[0, 7]], w.budget[[0, 7]], w.r_index[[0, 7]]
    desc = oracle_mod.enumerate_strategies(**w.enum)
    T, O, R = oracle_mod.build_tables(desc, w.layer, w.hw, w.rmodel, w.M)
    ref = oracle_batch(oracle_mod, w, T, O, R)
    a = runner.solve_workload(w, classes=True)
    b = runner.solve_workload(w, classes=False)
    assert a["forward_kernel"].startswith("k_dp_class") and b["forward_kernel"] in ("k_dp_tile", "k_dp_wide")
    assert_same(a, ref, w, "classes")
    assert_same(b, ref, w, "general")


def test_a_whole_step_can_be_captured_in_a_hip_graph_and_replayed(gs, oracle_mod):
    """A solve issues only kernel launches and event fork/joins (the status word is cleared
    by a kernel, not a memset), so a whole step - two instance groups on parallel streams
    included - can be captured and replayed.  Every replay, with eager solves of another
    workload on the same context in between, must give the oracle's bits."""
    binding, runner = gs
    import torch
    w = random_tables("graph", 6, 9, 44, 900, K=2, seed=321,
                      budget=np.array([900, 450, 899, 64, 700, 333], np.int32))
    other = random_tables("graph_other", 6, 9, 44, 900, K=2, seed=322)
    ref, ref_other = oracle_batch(oracle_mod, w), oracle_batch(oracle_mod, other)
    dw, dwo = runner.DeviceWorkload(w), runner.DeviceWorkload(other)
    st = torch.cuda.Stream()
    with runner.make_context(w) as ctx, torch.cuda.stream(st):
        ctx.gsearch_set_instance_groups(2)
        runner.run_step(ctx, dw, backtrace="all")                 # warm-up outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            captured = runner.run_step(ctx, dw, backtrace="all")
        for _ in range(3):
            eager = runner.to_numpy(runner.run_step(ctx, dwo, backtrace="all"))
            eager["data_status"] = ctx.gsearch_data_status()
            assert_same(eager, ref_other, other, "eager between replays")
            graph.replay()
            got = runner.to_numpy(captured)
            got["data_status"] = ctx.gsearch_data_status()
            assert_same(got, ref, w, "graph replay")


def test_strategy_sets_with_more_than_32_layouts(gs, oracle_mod):
    """128 devices without caps: 128 strategies in 36 layout classes, which the runner
    announces, so the wide form of the class kernel runs; the same classes handed over
    without the announcement are flagged, not silently wrong.  256 devices: 162 strategies in
    45 classes, beyond the general kernels' register-tiled sizes but not the class kernel's.
    1024 devices: 242 strategies in
    66 classes, more than a solve can exploit: the runner withholds them and the general
    kernels run."""
    binding, runner = gs
    import torch
    w = workloads._model_workload("n128", 2, 5, 700, dict(N=128), [8192.0], [4096.0], 262144.0,
                                  80.0e9, seed=77, S=128)
    desc = oracle_mod.enumerate_strategies(**w.enum)
    assert len(desc) == 128
    T, O, R = oracle_mod.build_tables(desc, w.layer, w.hw, w.rmodel, w.M)
    ref = oracle_batch(oracle_mod, w, T, O, R)
    dw = runner.DeviceWorkload(w)
    assert dw.n_class == 36
    for flags in (0, binding.GSEARCH_FLAG_NO_BACKPOINTERS):
        with runner.make_context(w, flags=flags) as ctx:
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all"))
            got["data_status"] = ctx.gsearch_data_status()
            assert ctx.gsearch_forward_kernel().startswith("k_dp_class")
            assert_same(got, ref, w, f"36 classes, wide class kernel, flags={flags}")
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", classes=False))
            got["data_status"] = ctx.gsearch_data_status()
            assert not ctx.gsearch_forward_kernel().startswith("k_dp_class")
            assert_same(got, ref, w, f"36 classes withheld, flags={flags}")
            r_class, _ = binding.gsearch_layout_classes(torch.from_numpy(desc).to(dw.device))
            runner.run_step(ctx, dw, backtrace=None, r_class=r_class)       # bound not announced
            assert ctx.gsearch_data_status() & binding.GSEARCH_DATA_BAD_RCLASS
    w = workloads._model_workload("n256", 2, 4, 400, dict(N=256), [8192.0], [4096.0], 262144.0,
                                  80.0e9, seed=79, S=162)
    desc = oracle_mod.enumerate_strategies(**w.enum)
    T, O, R = oracle_mod.build_tables(desc, w.layer, w.hw, w.rmodel, w.M)
    dw = runner.DeviceWorkload(w)
    assert len(desc) == 162 and dw.n_class == 45
    with runner.make_context(w) as ctx:
        got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all"))
        got["data_status"] = ctx.gsearch_data_status()
        assert ctx.gsearch_forward_kernel().startswith("k_dp_class")
        assert_same(got, oracle_batch(oracle_mod, w, T, O, R), w, "256 devices, 45 classes")
    w = workloads._model_workload("n1024", 1, 3, 300, dict(N=1024), [8192.0], [4096.0], 262144.0,
                                  80.0e9, seed=78, S=242)
    desc = oracle_mod.enumerate_strategies(**w.enum)
    T, O, R = oracle_mod.build_tables(desc, w.layer, w.hw, w.rmodel, w.M)
    dw = runner.DeviceWorkload(w)
    assert len(desc) == 242 and dw.n_class == 66 > binding.GSEARCH_MAX_CLASSES
    with runner.make_context(w) as ctx:
        got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all"))
        got["data_status"] = ctx.gsearch_data_status()
        assert not ctx.gsearch_forward_kernel().startswith("k_dp_class") and "r_class" not in got
        assert_same(got, oracle_batch(oracle_mod, w, T, O, R), w, "66 classes, general kernels")


@pytest.mark.parametrize("mode", ["bp", "nobp"])
def test_one_context_solves_different_workloads_in_turn(gs, oracle_mod, mode):
    """A context is a workspace, not a cache: problems of different shapes, budgets and class
    structure solved one after the other in the same context (whose planes then hold whatever
    the previous solve left, including rows the next solve never writes) each match the
    oracle, whole planes included."""
    binding, runner = gs
    import torch
    big, rc_big = workloads.class_tables("reuse_big", 4, 7, 96, 900, [4] * 24, K=2, seed=501,
                                         budget=np.array([900, 850, 400, 899], np.int32),
                                         coarse=True)
    small, rc_small = workloads.class_tables("reuse_small", 3, 5, 44, 300, [4] * 11, K=1, seed=502,
                                             budget=np.array([120, 300, 7], np.int32))
    plain = random_tables("reuse_plain", 2, 6, 24, 500, K=2, seed=503)
    cases = [(big, rc_big), (small, rc_small), (plain, None), (small, rc_small), (big, rc_big)]
    refs = {id(w): oracle_batch(oracle_mod, w) for w, _ in cases}
    flags = MODES[mode] | binding.GSEARCH_FLAG_KEEP_PLANES
    with binding.GSearch(4, 7, 96, 900, 2, flags=flags) as ctx:
        for n, (w, rc) in enumerate(cases):
            dw = runner.DeviceWorkload(w)
            r_class = None if rc is None else torch.from_numpy(rc).to(dw.device)
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=r_class))
            got["data_status"] = ctx.gsearch_data_status()
            C, _ = ctx.gsearch_export_planes(want_bp=False)
            C = C.cpu().numpy()
            assert_same(got, refs[id(w)], w, f"solve {n} ({w.name}, {mode})")
            for b in range(w.B):
                E = int(w.budget[b])
                one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E, want_planes=True)
                assert np.array_equal(bits(C[b, :, :E + 1, :]), bits(one["C"])), (n, w.name, b)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("case", [(256, [4] * 64, 16384), (162, [4] * 36 + [2] * 9, 20000),
                                  (96, [2] * 48, 33000)],
                         ids=lambda c: "S%dnc%dM%d" % (c[0], len(c[1]), c[2]))
def test_wide_class_kernel_at_large_budgets(gs, oracle_mod, case):
    """The wide form and the 192/256-strategy forms of the class kernel with tens of thousands
    of budget rows (row pitches and per-class strides of the size the benchmark uses, several
    hundred tiles, a ragged last tile), both modes, against the oracle."""
    binding, runner = gs
    import torch
    S, sizes, M = case
    B, L = 2, 3
    budget = np.array([M, M - 4097], np.int32)
    w, r_class = workloads.class_tables("widebig", B, L, S, M, sizes, K=1, seed=S + M,
                                        budget=budget, coarse=True)
    ref = oracle_batch(oracle_mod, w)
    dw = runner.DeviceWorkload(w)
    rc = torch.from_numpy(r_class).to(dw.device)
    for mode in ("bp", "nobp"):
        with runner.make_context(w, flags=MODES[mode]) as ctx:
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rc,
                                                  r_class_bound=len(sizes)))
            got["data_status"] = ctx.gsearch_data_status()
            assert ctx.gsearch_forward_kernel().startswith("k_dp_class")
            curve = ctx.gsearch_budget_curve().cpu().numpy()
        assert_same(got, ref, w, f"{case[0]} strategies, {len(sizes)} classes, M={M}, {mode}")
        for b in range(B):
            E = int(w.budget[b])
            one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E, want_curve=True)
            assert np.array_equal(bits(curve[b, :E + 1]), bits(one["curve"])), (case, mode, b)
            assert np.isinf(curve[b, E + 1:]).all()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("mode", ["bp", "nobp", "bp_tile", "nobp_push", "generic"])
def test_several_hundred_thousand_budget_rows(gs, oracle_mod, mode):
    """Long planes: 300 001 budget rows (4688 tiles, row pitch above 2^18, plane offsets in
    the tens of millions of elements), ragged budgets and strategies that use thousands of
    bins, every general kernel; and the largest strategy count (1024) on a short plane."""
    _, runner = gs
    M = 300000
    w = random_tables("longplane", 2, 3, 12, M, K=2, seed=91, o_hi=9000,
                      budget=np.array([M, M - 70001], np.int32))
    assert_same(runner.solve_workload(w, MODES[mode]), oracle_batch(oracle_mod, w), w,
                f"M={M} {mode}")
    if mode in ("bp", "nobp"):
        w = random_tables("maxS", 1, 3, 1024, 40, seed=92, o_hi=8)
        assert_same(runner.solve_workload(w, MODES[mode]), oracle_batch(oracle_mod, w), w,
                    f"S=1024 {mode}")


@pytest.mark.parametrize("B", [9, 37, 257])
def test_class_kernel_batch_sizes_that_are_not_a_multiple_of_eight(gs, oracle_mod, B):
    """For such batches the class kernel numbers its workgroups in eight contiguous runs of
    the instance-major tile list (one per XCD): every (instance, tile) must still be computed
    exactly once, whatever the division of the list comes to."""
    binding, runner = gs
    import torch
    rng = workloads.SplitMix64(4000 + B)
    M = 333
    budget = rng.randint(0, M, B).astype(np.int32)
    budget[0] = M
    w, r_class = workloads.class_tables("oddbatch", B, 4, 44, M, [4] * 11, K=2, seed=600 + B,
                                        budget=budget, coarse=True)
    ref = oracle_batch(oracle_mod, w)
    dw = runner.DeviceWorkload(w)
    rc = torch.from_numpy(r_class).to(dw.device)
    for mode in ("bp", "nobp"):
        with runner.make_context(w, flags=MODES[mode]) as ctx:
            got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rc))
            got["data_status"] = ctx.gsearch_data_status()
            assert ctx.gsearch_forward_kernel().startswith("k_dp_class")
        assert_same(got, ref, w, f"B={B} {mode}")


def _coarse_memories(w, units, seed):
    """Multiply every instance's memories by its unit, then plant what must not disturb the
    unit (a zero, entries beyond the budget that are no multiple of it) - and, for the last
    instance, one entry that fits and is no multiple, which must bring its unit back to 1."""
    rng = workloads.SplitMix64(seed)
    v = rng.randint(0, 10 ** 6, 6 * w.B).reshape(w.B, 6)
    for b in range(w.B):
        w.O[b] *= int(units[b])
        w.O[b, v[b, 0] % w.L, v[b, 1] % w.S] = 0
        w.O[b, v[b, 2] % w.L, v[b, 3] % w.S] = int(w.budget[b]) + 1      # never fits
        w.O[b, v[b, 4] % w.L, v[b, 5] % w.S] = w.M + 5                   # nor does this
    b = w.B - 1
    w.O[b, 0, 0] = 1 if w.budget[b] >= 1 else 0
    return w


@pytest.mark.parametrize("mode", ["bp", "nobp", "bp_push", "bp_tile", "nobp_push", "generic",
                                  "class", "class_nobp"])
def test_instances_are_solved_in_their_own_bin_unit(gs, oracle_mod, mode):
    """Memories with a common divisor: the library divides it out per instance (fewer plane
    rows), which must change nothing that is reported: costs, plans, memory in the caller's
    bins, whole planes, backpointers and the budget curve, against the oracle on the
    original tables.  Budgets that are no multiple of the unit, units that differ from
    instance to instance, entries that never fit and are no multiple, zero memories."""
    binding, runner = gs
    import torch
    units = np.array([4, 1, 3, 7, 2, 16, 5, 6], np.int32)
    B, L, S, M = len(units), 6, 44, 700
    budget = np.array([700, 650, 333, 699, 1, 640, 14, 500], np.int32)
    rc = None
    if mode.startswith("class"):
        w, rc = workloads.class_tables("unit", B, L, S, M, [4] * 11, K=2, seed=61, budget=budget)
        w.O = np.minimum(w.O, 20)
        flags = binding.GSEARCH_FLAG_NO_BACKPOINTERS if mode == "class_nobp" else 0
    else:
        w = random_tables("unit", B, L, S, M, K=2, seed=61, budget=budget, o_hi=20)
        flags = MODES[mode]
    w = _coarse_memories(w, units, 62)
    ref = oracle_batch(oracle_mod, w)
    assert np.isfinite(ref["best_cost"]).sum() >= 5       # the budgets bind, but not all fail
    for extra in (0, binding.GSEARCH_FLAG_NO_BIN_UNIT):
        got = runner.solve_workload(w, flags | extra, r_class=rc)
        assert_same(got, ref, w, f"{mode} flags {flags | extra:#x}")
        if rc is not None:
            assert got["forward_kernel"].startswith("k_dp_class")
    # whole planes, backpointers and curve in the caller's bins
    dw = runner.DeviceWorkload(w)
    rct = None if rc is None else torch.from_numpy(rc).to(dw.device)
    with runner.make_context(w, flags=flags | binding.GSEARCH_FLAG_KEEP_PLANES) as ctx:
        out = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all", r_class=rct,
                                              r_class_bound=0 if rc is None else 11))
        C, bp = ctx.gsearch_export_planes(want_bp="nobp" not in mode)
        curve = ctx.gsearch_budget_curve().cpu().numpy()
        C = C.cpu().numpy()
        bp = bp.cpu().numpy() if bp is not None else None
    for b in range(B):
        E = int(w.budget[b])
        one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E, want_planes=True,
                               want_curve=True)
        assert np.array_equal(bits(C[b, :, :E + 1, :]), bits(one["C"])), (mode, b)
        assert np.isinf(C[b, :, E + 1:, :]).all()
        if bp is not None:
            assert np.array_equal(bp[b, :, :E + 1, :], one["bp"].astype(np.int32)), (mode, b)
        assert np.array_equal(bits(curve[b, :E + 1]), bits(one["curve"])), (mode, b)
        assert np.isinf(curve[b, E + 1:]).all()
        assert np.array_equal(out["plan"][b], one["plan"]) and out["mem_used"][b] == one["mem_used"]


def test_a_common_divisor_of_the_memories_shortens_the_forward_pass(gs, oracle_mod):
    """The point of the bin unit: with every memory a multiple of 8 the planes have an eighth
    of the rows.  Checked through the results (identical to the oracle's on the original
    tables, with the rescaling on and off); the forward times of both are printed, not
    asserted (measured on an idle box: 0.19 of the time without the rescaling)."""
    binding, runner = gs
    w = random_tables("unit8", 32, 12, 64, 16000, seed=63, o_hi=150)
    w.O *= 8
    ref = oracle_batch(oracle_mod, w)
    dw = runner.DeviceWorkload(w)
    ms = {}
    for flags in (0, binding.GSEARCH_FLAG_NO_BIN_UNIT):
        with runner.make_context(w, flags=flags) as ctx:
            ctx.gsearch_set_profiling(True)
            for _ in range(3):
                out = runner.run_step(ctx, dw, backtrace="all")
            ms[flags] = ctx.gsearch_forward_ms()
            got = runner.to_numpy(out)
            got["data_status"] = ctx.gsearch_data_status()
        assert_same(got, ref, w, f"flags {flags:#x}")
    print(f"forward ms with the bin unit {ms[0]:.3f}, without "
          f"{ms[binding.GSEARCH_FLAG_NO_BIN_UNIT]:.3f}")


@pytest.mark.parametrize("case", [
    # B, L, S, M, K: where the one-launch kernel takes over (its tables fit LDS) ...
    (3, 9, 12, 100, 2), (2, 24, 12, 255, 1), (5, 6, 8, 256, 3), (2, 7, 24, 63, 2),
    (4, 5, 16, 127, 1), (2, 12, 4, 1000, 1), (1, 30, 2, 1023, 2), (70, 4, 6, 90, 1),
    # ... and a transition pool too large to stage (220 matrices of 8 x 8 padded entries),
    # which the per-layer kernels take instead
    (2, 6, 7, 80, 220),
], ids=lambda c: "B%dL%dS%dM%dK%d" % c)
def test_one_launch_kernel_for_small_instances(gs, oracle_mod, case):
    """The latency path: every layer front of an instance in one launch, planes in LDS.
    Costs, plans, whole planes, backpointers and the budget curve against the oracle, with
    and without backpointers, ragged budgets, a zero-memory and a never-fitting strategy."""
    binding, runner = gs
    B, L, S, M, K = case
    rng = workloads.SplitMix64(sum(case))
    budget = rng.randint(0, M, B).astype(np.int32)
    budget[0] = M
    w = random_tables("onelaunch", B, L, S, M, K=K, seed=sum(case) + 5, budget=budget,
                      o_hi=max(1, (2 * M) // L))
    w.O[0, L // 2, S // 2] = 0
    w.O[B - 1, 0, S - 1] = M + 3
    ref = oracle_batch(oracle_mod, w)
    for mode in ("bp", "nobp"):
        got = runner.solve_workload(w, MODES[mode])
        assert (got["forward_kernel"] == "k_dp_small") == (K < 220), (case, mode)
        assert_same(got, ref, w, mode)
    dw = runner.DeviceWorkload(w)
    with runner.make_context(w, flags=binding.GSEARCH_FLAG_KEEP_PLANES) as ctx:
        out = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all"))
        assert (ctx.gsearch_forward_kernel() == "k_dp_small") == (K < 220)
        C, bp = ctx.gsearch_export_planes(want_bp=True)
        curve = ctx.gsearch_budget_curve().cpu().numpy()
        C, bp = C.cpu().numpy(), bp.cpu().numpy()
    for b in range(B):
        E = int(w.budget[b])
        one = oracle_mod.solve(w.T[b], w.O[b], w.R, w.r_index[b], E, want_planes=True,
                               want_curve=True)
        assert np.array_equal(bits(C[b, :, :E + 1, :]), bits(one["C"])), (case, b)
        assert np.array_equal(bp[b, :, :E + 1, :], one["bp"].astype(np.int32)), (case, b)
        assert np.array_equal(bits(curve[b, :E + 1]), bits(one["curve"])), (case, b)
        assert np.array_equal(out["plan"][b], one["plan"]), (case, b)


def test_general_kernels_random_sweep(gs, oracle_mod):
    """Two hundred seeded random table workloads through the general kernels: strategy counts
    on both sides of every tile size, 1..9 instances, 1..7 layers, up to 1500 bins, several
    matrices, ragged budgets, integer tables (ties), zero-memory and never-fitting
    strategies, a forbidden source strategy, memories with a common divisor, forced instance
    groups; the default choice and one forced kernel or mode per case."""
    _, runner = gs
    rng = workloads.SplitMix64(4242)
    variants = [0x8, 0x10, 0x2, 0xC, 0x14, 0x4, 0x6]
    sizes = [1, 2, 7, 8, 9, 15, 16, 17, 23, 24, 25, 31, 33, 41, 44, 45, 47, 48, 49, 63, 64, 65,
             95, 96, 97, 127, 128, 129, 200]
    for case in range(200):
        v = rng.randint(0, 10 ** 6, 9)
        S = sizes[int(v[0]) % len(sizes)]
        B, L, M, K = 1 + int(v[1]) % 9, 1 + int(v[2]) % 7, 1 + int(v[3]) % 1500, 1 + int(v[4]) % 4
        budget = rng.randint(0, M, B).astype(np.int32)
        w = random_tables(f"sweep{case}", B, L, S, M, K=K, seed=60000 + case, budget=budget,
                          o_hi=max(1, M // max(1, L - 1)), integer=(case % 4 == 0))
        if case % 3 == 0:
            w.O[int(v[5]) % B, int(v[6]) % L, int(v[7]) % S] = 0
        if case % 3 == 1:
            for b in range(B):
                w.O[b] *= [1, 2, 3, 4, 6][(case + b) % 5]
        if case % 5 == 0:
            w.O[:, int(v[5]) % L, int(v[6]) % S] = M + 7
        if case % 7 == 0:
            w.R[int(v[5]) % K, int(v[6]) % S, :] = np.inf
        ref = oracle_batch(oracle_mod, w)
        dw = runner.DeviceWorkload(w)
        for flags in (0, variants[case % len(variants)]):
            with runner.make_context(w, flags=flags) as ctx:
                g = int(v[8]) % 4
                if g:
                    ctx.gsearch_set_instance_groups(g)
                got = runner.to_numpy(runner.run_step(ctx, dw, backtrace="all"))
                got["data_status"] = ctx.gsearch_data_status()
                curve = ctx.gsearch_budget_curve().cpu().numpy() if case % 4 == 1 else None
            assert_same(got, ref, w, f"sweep {case} S={S} flags={flags:#x} groups={g}")
            if curve is not None:
                assert_curve(oracle_mod, curve, w, f"sweep {case} flags={flags:#x}")
