"""Pins for the oracle's strategy enumerator and alpha-beta table builder.

The paper names both steps but prints no formula, so the table model is this build's own
reading ("parity unpinned" against the paper).  What is pinned here is the arithmetic:
closed-form counts for the enumerator, and for the tables exact rational evaluation on
power-of-two inputs, where every fp64 operation of the builder is exact.
"""
from fractions import Fraction

import numpy as np
import pytest

from paper_2504_21411_amd import workloads


@pytest.mark.parametrize("k", range(0, 8))
def test_enumerator_closed_form_uncapped(oracle_mod, k):
    N = 1 << k
    d = oracle_mod.enumerate_strategies(N)
    assert len(d) == 2 * (k + 1) ** 2
    assert (d[:, 0] * d[:, 1] * d[:, 2] == N).all()
    assert len({tuple(r) for r in d.tolist()}) == len(d)
    assert not ((d[:, 3] == 1) & (d[:, 2] == 1)).any()        # nothing to shard over
    key = [(r[1], r[0], r[3], r[4]) for r in d.tolist()]
    assert key == sorted(key)                                  # tree order, ckpt fastest
    assert set(d[:, 3].tolist()) <= {0, 1} and set(d[:, 4].tolist()) <= {0, 1}


def test_enumerator_caps_give_the_benchmark_shapes(oracle_mod):
    assert len(oracle_mod.enumerate_strategies(8, tp_max=4, sp_max=1)) == 12
    assert len(oracle_mod.enumerate_strategies(32, tp_max=8, sp_max=4, tpsp_max=16)) == 44
    assert len(oracle_mod.enumerate_strategies(64, sp_max=32)) == 96
    assert len(oracle_mod.enumerate_strategies(8, sp_max=2)) == 24
    d = oracle_mod.enumerate_strategies(32, tp_max=8, sp_max=4, tpsp_max=16)
    assert d[:, 0].max() == 8 and d[:, 1].max() == 4 and (d[:, 0] * d[:, 1]).max() == 16
    for i, cfg in enumerate(workloads.CONFIGS):
        w = cfg() if i != 4 else workloads.config4(B=64)
        assert len(oracle_mod.enumerate_strategies(**w.enum)) == w.S
    with pytest.raises(ValueError):
        oracle_mod.enumerate_strategies(12)


def _exact_tables(desc, h, q, n, F, BW, binb, keep, M):
    """Rational evaluation of the same model, no rounding anywhere."""
    T, O = [], []
    for tp, spd, dp, sdp, ckpt in desc.tolist():
        t = Fraction(n, dp * spd)
        P = 12 * h * h
        flops = 3 * (24 * t * h * h + 4 * t * q * h)
        if ckpt:
            flops = flops * 4 / 3
        comm = Fraction(0)
        if tp > 1:
            comm += 16 * t * h * Fraction(tp - 1, tp)
        if dp > 1:
            comm += 4 * Fraction(P, tp) * Fraction(dp - 1, dp) * (Fraction(3, 2) if sdp else 1)
        if spd > 1:
            comm += 8 * t * h * Fraction(spd - 1, spd)
        T.append(1000 * (flops / (tp * F) + comm / BW))
        mem = Fraction(16 * P, tp * (dp if sdp else 1)) + 68 * t * h / tp * (keep if ckpt else 1)
        bins = -((-mem) // binb)
        O.append(min(max(1, int(bins)), M + 1))
    return T, O


def test_table_builder_exact_on_power_of_two_inputs(oracle_mod):
    desc = oracle_mod.enumerate_strategies(16)
    h, q, n = 4096, 2048, 1 << 18
    F, BW, binb, keep, M = 1 << 47, 1 << 37, 1 << 24, Fraction(1, 4), 4096
    layer = np.array([[[h, q, n, 1.0, 1.0, 1.0]]], np.float64)
    hw = np.array([F, BW, binb, 0.25], np.float64)
    rmodel = np.array([[h, n]], np.float64)
    T, O, R = oracle_mod.build_tables(desc, layer, hw, rmodel, M)
    Tx, Ox = _exact_tables(desc, h, q, n, F, BW, binb, keep, M)
    # a bin size that divides none of the memories: the count of bins must round UP (a true
    # quotient with denominator 3 is at least 1/3 away from an integer, far beyond the
    # rounding of one fp64 division)
    odd_bin = 3 << 22
    _, O3, _ = oracle_mod.build_tables(desc, layer, np.array([F, BW, odd_bin, 0.25]), rmodel, M)
    _, Ox3 = _exact_tables(desc, h, q, n, F, BW, odd_bin, keep, M)
    assert O3[0, 0].tolist() == Ox3 and Ox3 != Ox
    for s, d in enumerate(desc.tolist()):
        want = np.float32(float(Tx[s]))
        if d[4] == 0:
            assert T[0, 0, s] == want, (s, d)                 # every step exact -> same bits
        else:
            assert abs(float(T[0, 0, s]) - float(want)) <= float(np.spacing(want))
        assert O[0, 0, s] == Ox[s], (s, d)
    # transition table: zero iff the (tp, sp, dp) layout agrees, value as defined otherwise
    for i, a in enumerate(desc.tolist()):
        for j, c in enumerate(desc.tolist()):
            if a[:3] == c[:3]:
                assert R[0, i, j] == 0.0
            else:
                gi, gj = a[2] * a[1], c[2] * c[1]
                w = Fraction(1) if a[0] == c[0] else Fraction(1, 2)
                x = 1000 * 2 * h * Fraction(n, gj) * (1 - w * Fraction(min(gi, gj), max(gi, gj))) / BW
                assert R[0, i, j] == np.float32(float(x)), (i, j)
    assert (R >= 0).all() and not np.array_equal(R[0], R[0].T)


def test_table_builder_scales_and_clamps(oracle_mod):
    desc = oracle_mod.enumerate_strategies(8)
    base = np.array([[[4096.0, 4096.0, 2.0 ** 18, 1.0, 1.0, 1.0]]], np.float64)
    hw = np.array([1.0e14, 1.0e11, 2.0 ** 24, 0.2], np.float64)
    rm = np.array([[4096.0, 2.0 ** 18]], np.float64)
    T1, O1, _ = oracle_mod.build_tables(desc, base, hw, rm, 1 << 20)
    half = base.copy(); half[..., 3] = 0.5
    T2, O2, _ = oracle_mod.build_tables(desc, half, hw, rm, 1 << 20)
    assert np.array_equal(T2, (T1 * np.float32(0.5)).astype(np.float32))   # power-of-two scale
    assert np.array_equal(O1, O2)
    # recomputation: more time, less memory; sharding: less memory
    d = desc.tolist()
    for s in range(0, len(d), 2):
        assert d[s][:4] == d[s + 1][:4] and d[s][4] == 0 and d[s + 1][4] == 1
        assert T1[0, 0, s + 1] > T1[0, 0, s] and O1[0, 0, s + 1] <= O1[0, 0, s]
    # clamp to M + 1 ("never fits") and floor of one bin
    T3, O3, _ = oracle_mod.build_tables(desc, base, hw, rm, 4)
    assert O3.max() == 5 and O3.min() >= 1
    huge = hw.copy(); huge[2] = 1.0e30
    _, O4, _ = oracle_mod.build_tables(desc, base, huge, rm, 4)
    assert (O4 == 1).all()


def test_workload_generators_are_deterministic_and_shaped():
    a, b = workloads.config0(), workloads.config0()
    assert np.array_equal(a.T, b.T) and np.array_equal(a.O, b.O) and np.array_equal(a.R, b.R)
    assert a.relaxations() == 23 * 257 * 144
    assert (np.diagonal(a.R[0]) == 0).all() and (a.T >= 1).all() and (a.T < 10).all()
    assert (a.T[0, 0] == a.T[0, 5]).all()                       # identical layers
    w1, w3 = workloads.config1(), workloads.config3()
    assert w1.layer.shape == (64, 48, 6) and w3.layer.shape == (8, 128, 6)
    assert w1.relaxations() == 64 * 47 * 2049 * 44 * 44
    assert w3.relaxations() == 8 * 127 * 16385 * 96 * 96
    assert set(w3.layer[:, 0, 1].tolist()) == {8192.0, 32768.0}
    w2 = workloads.config2()
    assert w2.T.shape == (256, 32, 44) and w2.K == 4 and w2.r_index.max() == 3
    assert w2.relaxations() == 256 * 31 * 4097 * 44 * 44
    w4 = workloads.config4()
    assert w4.B == 2048 and w4.T.shape == (2048, 32, 24)
    assert w4.budget.min() >= 1024 and w4.budget.max() < 2048
    r = workloads.SplitMix64(5)
    u = r.uniform(1000)
    assert u.min() >= 0 and u.max() < 1 and u.dtype == np.float32
    # SplitMix64 reference value: first output for seed 0 is the published test vector
    assert int(workloads.SplitMix64(0).u64(1)[0]) == 0xE220A8397B1DCDAF


def test_profiled_table_builder_exact_on_power_of_two_inputs(oracle_mod):
    """Profile-driven builder ("parity unpinned" against the paper, which gives no formula):
    with power-of-two inputs every fp64 step is exact, so the result must equal a rational
    evaluation of the stated formula."""
    desc = oracle_mod.enumerate_strategies(16)
    fwd, param, act = Fraction(3, 2), 1 << 28, 1 << 17
    tokens, overlap, binb, keep, sf, M = 1 << 17, Fraction(1, 4), 1 << 24, Fraction(1, 4), 8, 1 << 14
    bw = [1, 1 << 38, 1 << 37, 1 << 36, 1 << 35]
    T, O = oracle_mod.build_tables_profiled(
        desc, [[0]], [[float(fwd), param, act]], [float(x) for x in bw],
        [tokens, float(overlap), binb, float(keep), sf], M)
    for s, (tp, sp, dp, sdp, ckpt) in enumerate(desc.tolist()):
        t = Fraction(tokens, dp * sp)
        comp = 3 * fwd * t / 1000 / tp * (Fraction(4, 3) if ckpt else 1)
        lg = lambda v: v.bit_length() - 1
        tpc = 1000 * 4 * act * t * Fraction(tp - 1, tp) / bw[lg(tp)] if tp > 1 else 0
        dpc = (1000 * 2 * Fraction(param, tp) * Fraction(dp - 1, dp) * (Fraction(3, 2) if sdp else 1)
               / bw[lg(dp)]) if dp > 1 else 0
        spc = 1000 * 2 * act * t * Fraction(sp - 1, sp) / bw[lg(sp)] if sp > 1 else 0
        want = comp + tpc + (1 - overlap) * dpc + spc
        # t/1000 and the 4/3 factor round, so allow a few ulps of fp32; the rest is exact
        assert abs(float(T[0, 0, s]) - float(want)) <= 4 * float(np.spacing(np.float32(float(want))))
        mem = Fraction(sf * param, tp * (dp if sdp else 1)) + Fraction(act, 1) * t / tp * (keep if ckpt else 1)
        assert O[0, 0, s] == min(max(1, int(-((-mem) // binb))), M + 1)
    # a bin size that divides few of the memories: the count of bins rounds up
    odd_bin = 3 << 22
    _, O3 = oracle_mod.build_tables_profiled(
        desc, [[0]], [[float(fwd), param, act]], [float(x) for x in bw],
        [tokens, float(overlap), odd_bin, float(keep), sf], M)
    ragged = 0
    for s, (tp, sp, dp, sdp, ckpt) in enumerate(desc.tolist()):
        mem = (Fraction(sf * param, tp * (dp if sdp else 1))
               + Fraction(act, 1) * Fraction(tokens, dp * sp) / tp * (keep if ckpt else 1))
        ragged += mem % odd_bin != 0
        assert O3[0, 0, s] == min(max(1, int(-((-mem) // odd_bin))), M + 1)
    assert ragged >= 10
    # more overlap can only hide data-parallel communication
    T2, _ = oracle_mod.build_tables_profiled(
        desc, [[0]], [[float(fwd), param, act]], [float(x) for x in bw],
        [tokens, 1.0, binb, float(keep), sf], M)
    assert (T2 <= T).all() and (T2 < T)[0, 0, desc[:, 2] > 1].all()
    assert np.array_equal(T2[0, 0, desc[:, 2] == 1], T[0, 0, desc[:, 2] == 1])


def test_profile_dump_reader():
    import os
    path = os.path.join(os.path.dirname(__file__), "data", "profile_dump_example.json")
    names, profile, bw, par = workloads.load_profile_dump(path, 4096)
    assert names == ["decoder", "encoder"] and profile.shape == (2, 3)
    assert len(bw) == 6 and bw[1] == 3.0e11 and bw[5] == 2.5e10
    assert par[2] == 68719476736 / 4096 and par[1] == 0.5
