"""Pins for the oracle's pipeline-aware outer reduction.

The paper gives no formula for combining pipeline stages ("parity unpinned" against it);
what is pinned is the arithmetic of the stated reading: closed forms on exactly
representable inputs, an independent fp64 evaluation, infeasibility and tie rules.
"""
import numpy as np

from paper_2504_21411_amd import workloads


def test_hand_values_and_rules(oracle_mod):
    t = np.array([1.0, 2.0, 4.0, np.inf, 8.0, 0.5], np.float32)
    off = np.array([0, 1, 3, 5, 6, 8, 9], np.int32)
    mem = np.array([0, 1, 2, 2, 3, 4, 5, 0, 7], np.int32)
    mic = np.array([4, 3, 1, 1, 2, 5], np.int32)
    cost, best = oracle_mod.pipeline_reduce(t, off, mem, mic)
    # g0: 1 + 3*1 = 4; g1: (2+4) + 2*4 = 14; g2: member 3 infeasible; g3: 8 + 0*8 = 8;
    # g4: (0.5 + 1) + 1*1 = 2.5; g5: member id 7 is not an instance
    assert cost.tolist() == [4.0, 14.0, np.inf, 8.0, 2.5, np.inf]
    assert best == 4
    # single stage: t + (m-1) t = m t exactly for powers of two
    cost, _ = oracle_mod.pipeline_reduce(np.array([0.25], np.float32), [0, 1], [0], [64])
    assert cost[0] == 16.0
    # ties go to the lowest candidate; nothing feasible gives -1
    cost, best = oracle_mod.pipeline_reduce(np.array([3.0, 3.0], np.float32), [0, 1, 2], [0, 1], [2, 2])
    assert best == 0 and cost[0] == cost[1] == 6.0
    _, best = oracle_mod.pipeline_reduce(np.array([np.inf], np.float32), [0, 1], [0], [1])
    assert best == -1


def test_against_independent_evaluation(oracle_mod):
    rng = workloads.SplitMix64(5)
    B, G = 200, 60
    # multiples of 1/8 below 64: every sum and product here is exact in fp32 and fp64
    t = (rng.randint(1, 511, B) / 8.0).astype(np.float32)
    t[rng.randint(0, B - 1, 10)] = np.inf
    sizes = rng.randint(1, 16, G)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    mem = rng.randint(0, B - 1, int(off[-1])).astype(np.int32)
    mic = rng.randint(1, 64, G).astype(np.int32)
    cost, best = oracle_mod.pipeline_reduce(t, off, mem, mic)
    want = np.empty(G)
    for g in range(G):
        v = t[mem[off[g]:off[g + 1]]].astype(np.float64)
        want[g] = np.inf if np.isinf(v).any() else v.sum() + (mic[g] - 1) * v.max()
    assert np.array_equal(cost.astype(np.float64), want)
    finite = np.isfinite(want)
    assert best == int(np.flatnonzero(want == want[finite].min())[0])


def test_workload_groups_are_complete_candidates():
    w = workloads.config4()
    off, mem, mic, key = w.meta["groups"]
    assert len(mic) == 512 and off[-1] == len(mem) == 1728
    for g in range(len(mic)):
        ids = mem[off[g]:off[g + 1]]
        assert len(ids) == key[g][0]
        assert (w.meta["pp"][ids] == key[g][0]).all() and (w.meta["split"][ids] == key[g][1]).all()
        assert (w.meta["micro"][ids] == mic[g]).all()
        assert list(w.meta["stage"][ids]) == list(range(key[g][0]))
