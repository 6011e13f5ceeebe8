"""Seeded synthetic workloads for the strategy-search DP (inputs only, numpy only).

This module holds no arithmetic of the method itself: it draws numbers from a
counter-based SplitMix64 stream and shapes them into the problem's inputs.  Both the
HIP path and the CPU oracle are fed from here; neither is imported here.

Two kinds of workload come out:
  * "tables": T, O, R are drawn directly (random-table configurations);
  * "model":  per-layer scalars (hidden size, sequence length, tokens, scales) plus
    enumerator caps and hardware constants; the cost tables are then produced by the
    table builder under test (HIP kernel or oracle), not here.

The paper evaluates on real clusters and models and publishes no search workload, so
these five shapes stand in for it (single decoder stack, batched decoder stacks,
heterogeneous encoder-decoder, large dense model, full outer pipeline search).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


class SplitMix64:
    """Counter-based SplitMix64: draw n is a pure function of (seed, n)."""

    def __init__(self, seed: int):
        self.seed = np.uint64(seed & 0xFFFFFFFFFFFFFFFF)
        self.pos = 0

    def u64(self, n: int) -> np.ndarray:
        idx = np.arange(self.pos + 1, self.pos + n + 1, dtype=np.uint64)
        self.pos += n
        with np.errstate(over="ignore"):
            z = self.seed + idx * _GOLDEN
            z = (z ^ (z >> np.uint64(30))) * _M1
            z = (z ^ (z >> np.uint64(27))) * _M2
            z = z ^ (z >> np.uint64(31))
        return z

    def uniform(self, n: int) -> np.ndarray:
        """fp32 in [0, 1): top 24 bits times 2^-24 (exact)."""
        return ((self.u64(n) >> np.uint64(40)).astype(np.float32)) * np.float32(2.0 ** -24)

    def uniform_range(self, lo: float, hi: float, n: int) -> np.ndarray:
        u = self.uniform(n)
        return (np.float32(lo) + u * np.float32(hi - lo)).astype(np.float32)

    def randint(self, lo: int, hi: int, n: int) -> np.ndarray:
        """Integers in [lo, hi] inclusive."""
        span = np.uint64(hi - lo + 1)
        return (self.u64(n) % span).astype(np.int64) + lo

    def normal(self, n: int) -> np.ndarray:
        """fp64 standard normal by Box-Muller on two 53-bit uniforms."""
        a = ((self.u64(n) >> np.uint64(11)).astype(np.float64) + 0.5) * 2.0 ** -53
        b = ((self.u64(n) >> np.uint64(11)).astype(np.float64) + 0.5) * 2.0 ** -53
        return np.sqrt(-2.0 * np.log(a)) * np.cos(2.0 * np.pi * b)


@dataclass
class Workload:
    name: str
    B: int
    L: int
    S: int
    M: int
    K: int
    budget: np.ndarray            # [B] int32
    r_index: np.ndarray           # [B][L] int32
    kind: str                     # "tables" or "model"
    T: Optional[np.ndarray] = None        # [B][L][S] fp32
    O: Optional[np.ndarray] = None        # [B][L][S] int32
    R: Optional[np.ndarray] = None        # [K][S][S] fp32
    enum: Optional[dict] = None           # N, tp_max, sp_max, tpsp_max
    layer: Optional[np.ndarray] = None    # [B][L][6] fp64
    hw: Optional[np.ndarray] = None       # [4] fp64
    rmodel: Optional[np.ndarray] = None   # [K][2] fp64
    meta: dict = field(default_factory=dict)

    def relaxations(self) -> int:
        """Nominal min-plus update count: sum_b (L-1) (E_b+1) S^2."""
        return int((self.L - 1) * self.S * self.S * int((self.budget.astype(np.int64) + 1).sum()))

    def states(self) -> int:
        return int(self.L * self.S * int((self.budget.astype(np.int64) + 1).sum()))


def _transition(rng: SplitMix64, K: int, S: int, hi: float = 2.0) -> np.ndarray:
    R = rng.uniform_range(0.0, hi, K * S * S).reshape(K, S, S)
    for k in range(K):
        np.fill_diagonal(R[k], np.float32(0.0))
    return R


def random_tables(name, B, L, S, M, K=1, seed=0, o_hi=None, budget=None, identical_layers=False,
                  integer=False) -> Workload:
    """Generic random-table workload (also used by the edge-case tests)."""
    rng = SplitMix64(seed)
    o_hi = o_hi if o_hi is not None else max(1, (2 * M) // max(L, 1))
    rows = 1 if identical_layers else L
    if integer:
        T = rng.randint(1, 9, B * rows * S).astype(np.float32).reshape(B, rows, S)
    else:
        T = rng.uniform_range(1.0, 10.0, B * rows * S).reshape(B, rows, S)
    O = rng.randint(1, o_hi, B * rows * S).astype(np.int32).reshape(B, rows, S)
    if identical_layers:
        T = np.repeat(T, L, axis=1)
        O = np.repeat(O, L, axis=1)
    if integer:
        R = rng.randint(0, 3, K * S * S).astype(np.float32).reshape(K, S, S)
    else:
        R = _transition(rng, K, S)
    r_index = (rng.randint(0, K - 1, B * L).astype(np.int32).reshape(B, L)
               if K > 1 else np.zeros((B, L), np.int32))
    if budget is None:
        budget = np.full(B, M, np.int32)
    return Workload(name, B, L, S, M, K, np.asarray(budget, np.int32), r_index, "tables",
                    T=np.ascontiguousarray(T), O=np.ascontiguousarray(O), R=R)


def class_tables(name, B, L, S, M, sizes, K=1, seed=0, budget=None, coarse=False):
    """Random tables whose transition matrices depend on the strategies only through
    contiguous classes of the given sizes (sum(sizes) == S).  Returns (workload, r_class).

    coarse=True draws T from 1024 + k * 2^-13 (k in 0..7, neighbouring fp32 values) and the
    class transition values from {0, 4096, 8192}: adding 4096 or more drops the low bits of
    the sum, so different candidates of a class often ROUND to the same sum; that is the
    case in which the member with the smallest previous cost is not the lowest-index
    argmin."""
    sizes = [int(x) for x in sizes]
    assert sum(sizes) == S and all(x >= 1 for x in sizes)
    w = random_tables(name, B, L, S, M, K=K, seed=seed, budget=budget)
    rng = SplitMix64(seed + 7919)
    r_class = np.repeat(np.arange(len(sizes), dtype=np.int32), sizes)
    nc = len(sizes)
    if coarse:
        w.T = (np.float32(1024.0) + rng.randint(0, 7, w.T.size).astype(np.float32)
               * np.float32(2.0 ** -13)).reshape(w.T.shape).astype(np.float32)
        Rc = (rng.randint(0, 2, K * nc * nc).astype(np.float32) * np.float32(4096.0))
    else:
        Rc = rng.uniform_range(0.0, 2.0, K * nc * nc)
    Rc = Rc.reshape(K, nc, nc).astype(np.float32)
    for k in range(K):
        np.fill_diagonal(Rc[k], 0.0)
    w.R = np.ascontiguousarray(Rc[:, r_class][:, :, r_class])
    return w, r_class


# --------------------------------------------------------------------------------------
# The five benchmark configurations (zero-based numbering).
# --------------------------------------------------------------------------------------

def config0() -> Workload:
    """Single instance, 24 identical decoder layers, S=12, M=256, seed 0."""
    w = random_tables("cfg0_single_decoder", 1, 24, 12, 256, K=1, seed=0, o_hi=20,
                      identical_layers=True)
    w.enum = dict(N=8, tp_max=4, sp_max=1, tpsp_max=0)
    return w


def _model_workload(name, B, L, M, enum, hidden_choices, seqs, tokens_per_step, device_bytes,
                    seed, sigma=0.1, S=None) -> Workload:
    rng = SplitMix64(seed)
    pick = rng.randint(0, len(hidden_choices) - 1, B * L).reshape(B, L)
    base = np.asarray(hidden_choices, np.float64)[pick]
    hidden = base * np.exp(sigma * rng.normal(B * L).reshape(B, L))
    layer = np.zeros((B, L, 6), np.float64)
    seq = np.asarray([seqs[b % len(seqs)] if len(seqs) < B else seqs[b] for b in range(B)],
                     np.float64)
    layer[:, :, 0] = hidden
    layer[:, :, 1] = seq[:, None]
    layer[:, :, 2] = float(tokens_per_step)
    layer[:, :, 3] = 1.0      # time scale
    layer[:, :, 4] = 1.0      # model-state scale
    layer[:, :, 5] = 1.0      # activation scale
    hw = np.asarray([1.0e14, 1.0e11, device_bytes / M, 0.2], np.float64)
    rmodel = np.asarray([[float(np.mean(hidden_choices)), float(tokens_per_step)]],
                        np.float64)
    return Workload(name, B, L, S, M, 1, np.full(B, M, np.int32), np.zeros((B, L), np.int32),
                    "model", enum=enum, layer=layer, hw=hw, rmodel=rmodel)


def config1() -> Workload:
    """64 instances, L=48, S=44 (32 devices), M=2048, alpha-beta tables, seed 1."""
    return _model_workload("cfg1_batch_decoder", 64, 48, 2048,
                           dict(N=32, tp_max=8, sp_max=4, tpsp_max=16),
                           [4096.0, 5120.0], [4096.0], 262144.0, 64.0e9, seed=1, S=44)


def config2() -> Workload:
    """256 instances, 32 layers of two alternating types, S=44, M=4096, K=4, seed 2."""
    B, L, S, M, K = 256, 32, 44, 4096, 4
    rng = SplitMix64(2)
    T = rng.uniform_range(1.0, 10.0, B * L * S).reshape(B, L, S)
    O = rng.randint(1, (2 * M) // L, B * L * S).astype(np.int32).reshape(B, L, S)
    # layer type 0 = encoder, 1 = decoder; even instances alternate layer by layer,
    # odd instances alternate in pairs, so all four (type, type) transition matrices occur
    ltype = np.zeros((B, L), np.int32)
    ltype[0::2] = (np.arange(L) % 2)[None, :]
    ltype[1::2] = ((np.arange(L) // 2) % 2)[None, :]
    enc = ltype == 0
    T = np.where(enc[:, :, None], (T * np.float32(0.7)).astype(np.float32), T).astype(np.float32)
    O = np.where(enc[:, :, None], np.maximum(1, np.rint(O * 0.7)), O).astype(np.int32)
    R = _transition(rng, K, S)
    r_index = np.zeros((B, L), np.int32)
    r_index[:, 1:] = 2 * ltype[:, :-1] + ltype[:, 1:]
    return Workload("cfg2_hetero_encdec", B, L, S, M, K, np.full(B, M, np.int32), r_index,
                    "tables", T=np.ascontiguousarray(T), O=np.ascontiguousarray(O), R=R,
                    enum=dict(N=32, tp_max=8, sp_max=4, tpsp_max=16),
                    meta=dict(layer_type=ltype))


def config3() -> Workload:
    """8 instances, L=128, S=96 (64 devices), M=16384, hidden 16384, seq 8192/32768, seed 3."""
    seqs = [8192.0] * 4 + [32768.0] * 4
    return _model_workload("cfg3_large_dense", 8, 128, 16384,
                           dict(N=64, tp_max=0, sp_max=32, tpsp_max=0),
                           [16384.0], seqs, 131072.0, 288.0e9, seed=3, S=96)


def pipeline_instances(limit=2048, pps=(1, 2, 4, 8, 16), splits_per_pp=3, max_micro=64):
    """Canonical outer enumeration: pp, then stage-split id, then stage, then micro-batches.

    Returns int32 arrays (pp, split, stage, micro), truncated to `limit` rows.
    """
    rows = []
    for pp in pps:
        for split in range(1 if pp == 1 else splits_per_pp):
            for stage in range(pp):
                for m in range(1, max_micro + 1):
                    rows.append((pp, split, stage, m))
                    if len(rows) == limit:
                        a = np.asarray(rows, np.int32)
                        return a[:, 0], a[:, 1], a[:, 2], a[:, 3]
    a = np.asarray(rows, np.int32)
    return a[:, 0], a[:, 1], a[:, 2], a[:, 3]


def pipeline_groups(pp, split, stage, micro):
    """Complete candidates (pp, split, micro) of an instance list, as CSR.

    A candidate is complete when all its pp stages are present; members are listed in
    stage order.  Returns int32 arrays (offsets [G+1], members, micro [G]) plus the
    (pp, split) of every group.
    """
    index = {}
    for b in range(len(pp)):
        index[(int(pp[b]), int(split[b]), int(micro[b]), int(stage[b]))] = b
    offsets, members, gm, gkey = [0], [], [], []
    seen = set()
    for b in range(len(pp)):
        key = (int(pp[b]), int(split[b]), int(micro[b]))
        if key in seen:
            continue
        seen.add(key)
        ids = [index.get(key + (st,)) for st in range(key[0])]
        if any(i is None for i in ids):
            continue
        members.extend(ids)
        offsets.append(len(members))
        gm.append(key[2])
        gkey.append(key[:2])
    return (np.asarray(offsets, np.int32), np.asarray(members, np.int32),
            np.asarray(gm, np.int32), np.asarray(gkey, np.int32))


def config4(B=2048) -> Workload:
    """Full outer search: B pipeline-stage instances, L=32, S=24, M=2048, seed 4."""
    L, S, M = 32, 24, 2048
    pp, split, stage, micro = pipeline_instances(limit=B)
    B = len(pp)
    rng = SplitMix64(4)
    budget = np.floor(rng.uniform_range(0.5, 1.0, B).astype(np.float64) * M).astype(np.int32)
    # one base table per (pp, split, stage); the 64 micro-batch counts rescale it
    key = (pp.astype(np.int64) * 64 + split) * 64 + stage
    uniq, inv = np.unique(key, return_inverse=True)
    G = len(uniq)
    Tb = rng.uniform_range(1.0, 10.0, G * L * S).reshape(G, L, S)
    state = rng.randint(1, 32, G * L * S).astype(np.int64).reshape(G, L, S)
    act = rng.randint(1, 64, G * L * S).astype(np.int64).reshape(G, L, S)
    T = (Tb[inv] * (np.float32(1.0) / micro.astype(np.float32))[:, None, None]).astype(np.float32)
    inflight = np.minimum(pp - stage, micro).astype(np.float64) / micro.astype(np.float64)
    O = state[inv] + np.maximum(1, np.rint(act[inv] * inflight[:, None, None])).astype(np.int64)
    R = _transition(rng, 1, S)
    return Workload("cfg4_outer_search", B, L, S, M, 1, budget, np.zeros((B, L), np.int32),
                    "tables", T=np.ascontiguousarray(T), O=np.ascontiguousarray(O.astype(np.int32)),
                    R=R, enum=dict(N=8, tp_max=0, sp_max=2, tpsp_max=0),
                    meta=dict(pp=pp, split=split, stage=stage, micro=micro,
                              groups=pipeline_groups(pp, split, stage, micro)))


def load_profile_dump(path, M):
    """Read a profiler-dump-shaped JSON file into the arrays the profiled table builder takes.

    Returns (type_names, profile fp64 [Y][3], bandwidth fp64 [NB], par fp64 [5]) with
    par = (tokens, overlap, bin_bytes, ckpt_keep, state_factor), bin_bytes = device_bytes / M.
    Only reshapes the file's numbers; no cost-model arithmetic happens here.
    """
    import json
    with open(path) as fh:
        d = json.load(fh)
    names = sorted(d["layer_types"])
    profile = np.asarray([[d["layer_types"][n]["fwd_ms_per_ktoken"],
                           d["layer_types"][n]["param_bytes"],
                           d["layer_types"][n]["act_bytes_per_token"]] for n in names], np.float64)
    sizes = {int(k): float(v) for k, v in d["allreduce_bandwidth_bytes_per_s"].items()}
    nb = max(sizes).bit_length()
    bw = np.full(nb, min(sizes.values()), np.float64)
    for g in range(1, nb):
        if (1 << g) in sizes:
            bw[g] = sizes[1 << g]
    par = np.asarray([d["tokens_per_step"], d["overlap"], d["device_bytes"] / M, d["ckpt_keep"],
                      d["state_factor"]], np.float64)
    return names, profile, bw, par


CONFIGS = [config0, config1, config2, config3, config4]


def get_config(i: int) -> Workload:
    return CONFIGS[i]()
