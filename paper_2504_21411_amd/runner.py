"""Drives the whole hot path for one workload through the C-ABI binding.

enumerate strategies -> build cost tables (model workloads) -> batched DP -> final
reductions -> backtrace.  Everything runs in libgsearch; this file only moves arrays
between numpy and the GPU and orders the calls.
"""
from __future__ import annotations

import numpy as np

from . import binding
from .workloads import Workload


class DeviceWorkload:
    """A workload's inputs resident in HBM (uploaded once, reused by every step)."""

    def __init__(self, w: Workload, device="cuda"):
        import torch
        self.w = w
        self.device = torch.device(device)
        t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(self.device, dtype=dt)
        self.r_index = t(w.r_index, torch.int32)
        self.budget = t(w.budget, torch.int32)
        if w.kind == "tables":
            self.T, self.O, self.R = t(w.T, torch.float32), t(w.O, torch.int32), t(w.R, torch.float32)
            self.layer = self.rmodel = None
        else:
            self.T = self.O = self.R = None
            self.layer = t(w.layer, torch.float64)
            self.rmodel = t(w.rmodel, torch.float64)
        self.desc = None
        # Set-up, once per workload: how many layout classes the strategy set has.  A solve
        # can exploit at most GSEARCH_MAX_CLASSES of them and would flag a longer list, so
        # run_step hands the classes over only when they fit, and announces their number
        # (above 32 the solve needs the wide form of the class kernel).
        self.n_class = None
        if w.kind == "model":
            desc, _ = binding.gsearch_enumerate(device=self.device, **w.enum)
            _, count = binding.gsearch_layout_classes(desc)
            self.n_class = int(count.cpu()[0])


def make_context(w: Workload, flags=0, device=0) -> binding.GSearch:
    return binding.GSearch(w.B, w.L, w.S, w.M, w.K, flags=flags, device=device)


def run_step(ctx: binding.GSearch, dw: DeviceWorkload, backtrace="best", stream=None,
             classes=True, r_class=None, r_class_bound=0):
    """One pass of the hot path.  Returns device tensors; nothing is synchronised here.

    Model workloads build R from the strategy layouts, so the layout classes of the
    enumerated strategies are handed to the solve (classes=False withholds them).  Table
    workloads pass r_class only when the caller supplies one."""
    w = dw.w
    out = {}
    if w.kind == "model":
        desc, count = binding.gsearch_enumerate(device=dw.device, stream=stream, **w.enum)
        T, O, R = binding.gsearch_build_tables(desc, dw.layer, w.hw, dw.rmodel, w.M, stream=stream)
        out.update(desc=desc, count=count, T=T, O=O, R=R)
        if classes and r_class is None and dw.n_class <= binding.GSEARCH_MAX_CLASSES:
            r_class, n_class = binding.gsearch_layout_classes(desc, stream=stream)
            r_class_bound = dw.n_class
            out.update(r_class=r_class, n_class=n_class)
    else:
        T, O, R = dw.T, dw.O, dw.R
    res = ctx.gsearch_solve_batch(T, O, R, dw.r_index, dw.budget, w.M, stream=stream,
                                  r_class=r_class if classes else None,
                                  r_class_bound=r_class_bound)
    out.update(res)
    if backtrace == "best":
        out.update(ctx.gsearch_backtrace(res["best_instance"], 1, stream=stream))
    elif backtrace == "all":
        out.update(ctx.gsearch_backtrace(None, w.B, stream=stream))
    return out


def to_numpy(out: dict) -> dict:
    import torch
    torch.cuda.synchronize()
    return {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}


def solve_workload(w: Workload, flags=0, backtrace="all", classes=True, r_class=None,
                   r_class_bound=None) -> dict:
    """Convenience: upload, run one step, download everything as numpy.  r_class: optional
    numpy int32 [S] for table workloads (its class count is announced unless r_class_bound
    says otherwise)."""
    import torch
    dw = DeviceWorkload(w)
    if r_class is not None:
        if r_class_bound is None:
            r_class_bound = int(np.max(r_class)) + 1
        r_class = torch.from_numpy(np.ascontiguousarray(r_class, np.int32)).to(dw.device)
    with make_context(w, flags=flags) as ctx:
        out = to_numpy(run_step(ctx, dw, backtrace=backtrace, classes=classes, r_class=r_class,
                                r_class_bound=r_class_bound or 0))
        out["data_status"] = ctx.gsearch_data_status()
        out["forward_kernel"] = ctx.gsearch_forward_kernel()
    return out
