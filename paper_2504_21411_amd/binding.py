"""ctypes binding of libgsearch.so: same entry-point names as include/gsearch.h.

Argument marshalling only.  torch is used for device memory and the stream handle; every
step of the search runs in the HIP library.  There is no CPU fallback: if the library
is missing or cannot be loaded, importing callers get a RuntimeError.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgsearch.so")

GSEARCH_OK = 0
GSEARCH_ERR_INVALID_ARG = -1
GSEARCH_ERR_CAPACITY = -2
GSEARCH_ERR_NO_DEVICE = -3
GSEARCH_ERR_HIP = -4
GSEARCH_ERR_NOT_SOLVED = -5
GSEARCH_ERR_NO_MEMORY = -6
GSEARCH_ERR_UNSUPPORTED = -7

GSEARCH_FLAG_KEEP_PLANES = 0x1
GSEARCH_FLAG_FORCE_GENERIC = 0x2
GSEARCH_FLAG_NO_BACKPOINTERS = 0x4
GSEARCH_FLAG_FORCE_PUSH = 0x8
GSEARCH_FLAG_FORCE_TILE = 0x10
GSEARCH_FLAG_NO_BIN_UNIT = 0x20

GSEARCH_DATA_BAD_T = 0x1
GSEARCH_DATA_BAD_R = 0x2
GSEARCH_DATA_BAD_O = 0x4
GSEARCH_DATA_BAD_BUDGET = 0x8
GSEARCH_DATA_BAD_RINDEX = 0x10
GSEARCH_DATA_BAD_RCLASS = 0x20
GSEARCH_DATA_INTERNAL = 0x40
GSEARCH_MAX_CLASSES = 64
GSEARCH_DEFAULT_CLASSES = 32
GSEARCH_MAX_S = 1024
GSEARCH_NOALLOC_SCRATCH_BYTES = 16 << 20

EXPORTS = [
    "gsearch_workspace_bytes", "gsearch_create", "gsearch_destroy", "gsearch_solve_batch",
    "gsearch_backtrace", "gsearch_data_status", "gsearch_budget_curve", "gsearch_export_planes",
    "gsearch_enumerate_count", "gsearch_enumerate", "gsearch_build_tables", "gsearch_strerror",
    "gsearch_set_profiling", "gsearch_forward_ms", "gsearch_forward_kernel",
    "gsearch_pipeline_reduce", "gsearch_build_tables_profiled", "gsearch_set_instance_groups",
    "gsearch_instance_groups", "gsearch_layout_classes", "gsearch_solve_batch_noalloc",
    "gsearch_knob_name", "gsearch_set_knob", "gsearch_get_knob", "gsearch_lds_calibration",
    "gsearch_set_solve_counter", "gsearch_knob_initial",
]


class gsearch_config(ctypes.Structure):
    _fields_ = [("device", ctypes.c_int32), ("max_B", ctypes.c_int32), ("max_L", ctypes.c_int32),
                ("max_S", ctypes.c_int32), ("max_M", ctypes.c_int32), ("max_K", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]


class gsearch_problem(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("L", ctypes.c_int32), ("S", ctypes.c_int32),
                ("M", ctypes.c_int32), ("K", ctypes.c_int32), ("T", ctypes.c_void_p),
                ("O", ctypes.c_void_p), ("R", ctypes.c_void_p), ("r_index", ctypes.c_void_p),
                ("budget", ctypes.c_void_p), ("r_class", ctypes.c_void_p),
                ("r_class_bound", ctypes.c_int32)]


class gsearch_result(ctypes.Structure):
    _fields_ = [("best_cost", ctypes.c_void_p), ("best_s", ctypes.c_void_p),
                ("final_row", ctypes.c_void_p), ("best_instance", ctypes.c_void_p)]


class gsearch_hw_model(ctypes.Structure):
    _fields_ = [("flops_per_s", ctypes.c_double), ("bytes_per_s", ctypes.c_double),
                ("bin_bytes", ctypes.c_double), ("ckpt_keep", ctypes.c_double)]


class gsearch_profile_params(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_double), ("overlap", ctypes.c_double),
                ("bin_bytes", ctypes.c_double), ("ckpt_keep", ctypes.c_double),
                ("state_factor", ctypes.c_double)]


class GSearchError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libgsearch.so from the package directory (raises if it is not built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2504_21411_amd.build` "
            "(there is no fallback path)")
    # PyTorch ships its own HIP runtime and owns the device memory this library works on:
    # import it first, so that libgsearch.so binds to the runtime PyTorch has loaded instead
    # of bringing a second one into the process (whose calls would see no usable device).
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    lib.gsearch_workspace_bytes.restype = ctypes.c_size_t
    lib.gsearch_workspace_bytes.argtypes = [ctypes.POINTER(gsearch_config)]
    lib.gsearch_create.restype = ctypes.c_int
    lib.gsearch_create.argtypes = [ctypes.POINTER(gsearch_config), ctypes.POINTER(vp)]
    lib.gsearch_destroy.restype = ctypes.c_int
    lib.gsearch_destroy.argtypes = [vp]
    lib.gsearch_solve_batch.restype = ctypes.c_int
    lib.gsearch_solve_batch.argtypes = [vp, ctypes.POINTER(gsearch_problem),
                                        ctypes.POINTER(gsearch_result), vp]
    lib.gsearch_solve_batch_noalloc.restype = ctypes.c_int
    lib.gsearch_solve_batch_noalloc.argtypes = [i32, ctypes.POINTER(gsearch_problem),
                                                ctypes.POINTER(gsearch_result), vp, vp, vp, vp]
    lib.gsearch_backtrace.restype = ctypes.c_int
    lib.gsearch_backtrace.argtypes = [vp, vp, i32, vp, vp, vp]
    lib.gsearch_data_status.restype = ctypes.c_int
    lib.gsearch_data_status.argtypes = [vp, vp, ctypes.POINTER(i32)]
    lib.gsearch_set_profiling.restype = ctypes.c_int
    lib.gsearch_set_profiling.argtypes = [vp, ctypes.c_int]
    lib.gsearch_set_instance_groups.restype = ctypes.c_int
    lib.gsearch_set_instance_groups.argtypes = [vp, ctypes.c_int]
    lib.gsearch_lds_calibration.restype = ctypes.c_int
    lib.gsearch_lds_calibration.argtypes = [i32, i32, vp, vp]
    lib.gsearch_knob_name.restype = ctypes.c_char_p
    lib.gsearch_knob_name.argtypes = [ctypes.c_int]
    lib.gsearch_set_solve_counter.restype = ctypes.c_int
    lib.gsearch_set_solve_counter.argtypes = [vp, ctypes.c_uint32, vp]
    lib.gsearch_knob_initial.restype = ctypes.c_int
    lib.gsearch_knob_initial.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_int)]
    lib.gsearch_set_knob.restype = ctypes.c_int
    lib.gsearch_set_knob.argtypes = [vp, ctypes.c_char_p, ctypes.c_int]
    lib.gsearch_get_knob.restype = ctypes.c_int
    lib.gsearch_get_knob.argtypes = [vp, ctypes.c_char_p, ctypes.POINTER(ctypes.c_int)]
    lib.gsearch_instance_groups.restype = ctypes.c_int
    lib.gsearch_instance_groups.argtypes = [vp]
    lib.gsearch_layout_classes.restype = ctypes.c_int
    lib.gsearch_layout_classes.argtypes = [vp, i32, vp, vp, vp]
    lib.gsearch_forward_ms.restype = ctypes.c_int
    lib.gsearch_forward_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    lib.gsearch_forward_kernel.restype = ctypes.c_char_p
    lib.gsearch_forward_kernel.argtypes = [vp]
    lib.gsearch_pipeline_reduce.restype = ctypes.c_int
    lib.gsearch_pipeline_reduce.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp]
    lib.gsearch_budget_curve.restype = ctypes.c_int
    lib.gsearch_budget_curve.argtypes = [vp, vp, vp]
    lib.gsearch_export_planes.restype = ctypes.c_int
    lib.gsearch_export_planes.argtypes = [vp, vp, vp, vp]
    lib.gsearch_enumerate_count.restype = i32
    lib.gsearch_enumerate_count.argtypes = [i32, i32, i32, i32]
    lib.gsearch_enumerate.restype = ctypes.c_int
    lib.gsearch_enumerate.argtypes = [i32, i32, i32, i32, vp, i32, vp, vp]
    lib.gsearch_build_tables.restype = ctypes.c_int
    lib.gsearch_build_tables.argtypes = [i32, i32, i32, i32, i32, vp, vp,
                                         ctypes.POINTER(gsearch_hw_model), vp, vp, vp, vp, vp]
    lib.gsearch_build_tables_profiled.restype = ctypes.c_int
    lib.gsearch_build_tables_profiled.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp,
                                                  ctypes.POINTER(gsearch_profile_params), vp, vp,
                                                  vp]
    lib.gsearch_strerror.restype = ctypes.c_char_p
    lib.gsearch_strerror.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().gsearch_strerror(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != GSEARCH_OK:
        raise GSearchError(code, where)


def _ptr(t, dtype=None, name="tensor") -> Optional[int]:
    """Device pointer of a contiguous torch tensor (None passes NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def gsearch_lds_calibration(mode: int, iters: int, device="cuda", stream=None) -> int:
    """One launch of LDS traffic of known size; returns the bytes it moves through LDS."""
    import torch
    sink = torch.empty(1024 * 256, dtype=torch.float32, device=device)
    _check(load_library().gsearch_lds_calibration(int(mode), int(iters), _ptr(sink),
                                                  _stream(stream)), "gsearch_lds_calibration")
    return 1024 * 256 * int(iters) * (16 if mode == 1 else 4)


def gsearch_knob_initial(name: str) -> int:
    """Value a new context would start the knob with (default or GSEARCH_<NAME>); host only."""
    v = ctypes.c_int(0)
    _check(load_library().gsearch_knob_initial(name.encode(), ctypes.byref(v)),
           "gsearch_knob_initial")
    return int(v.value)


def gsearch_knob_names() -> list:
    lib, names, i = load_library(), [], 0
    while True:
        n = lib.gsearch_knob_name(i)
        if n is None:
            return names
        names.append(n.decode())
        i += 1


def gsearch_workspace_bytes(max_B, max_L, max_S, max_M, max_K=1, flags=0, device=0) -> int:
    cfg = gsearch_config(device, max_B, max_L, max_S, max_M, max_K, flags)
    return int(load_library().gsearch_workspace_bytes(ctypes.byref(cfg)))


def gsearch_enumerate_count(N, tp_max=0, sp_max=0, tpsp_max=0) -> int:
    n = int(load_library().gsearch_enumerate_count(N, tp_max, sp_max, tpsp_max))
    if n < 0:
        raise GSearchError(n, "gsearch_enumerate_count")
    return n


def gsearch_enumerate(N, tp_max=0, sp_max=0, tpsp_max=0, device="cuda", stream=None):
    """Device enumeration; returns (desc int32 [S][5] on the GPU, count tensor [1])."""
    import torch
    n = gsearch_enumerate_count(N, tp_max, sp_max, tpsp_max)
    desc = torch.empty((n, 5), dtype=torch.int32, device=device)
    count = torch.empty(1, dtype=torch.int32, device=device)
    _check(load_library().gsearch_enumerate(N, tp_max, sp_max, tpsp_max, _ptr(desc), n,
                                            _ptr(count), _stream(stream)), "gsearch_enumerate")
    return desc, count


def gsearch_layout_classes(desc, stream=None):
    """desc int32 [S][5] on the GPU -> (r_class int32 [S], count int32 [1]) on the GPU."""
    import torch
    S = desc.shape[0]
    r_class = torch.empty(S, dtype=torch.int32, device=desc.device)
    count = torch.empty(1, dtype=torch.int32, device=desc.device)
    _check(load_library().gsearch_layout_classes(_ptr(desc, torch.int32, "desc"), S,
                                                 _ptr(r_class), _ptr(count), _stream(stream)),
           "gsearch_layout_classes")
    return r_class, count


def gsearch_build_tables(desc, layer, hw, rmodel, M, stream=None):
    """desc int32 [S][5], layer fp64 [B][L][6], rmodel fp64 [K][2] on the GPU; hw 4 floats.

    Returns device tensors T [B][L][S] fp32, O [B][L][S] int32, R [K][S][S] fp32.
    """
    import torch
    B, L, _ = layer.shape
    S, K = desc.shape[0], rmodel.shape[0]
    dev = layer.device
    T = torch.empty((B, L, S), dtype=torch.float32, device=dev)
    O = torch.empty((B, L, S), dtype=torch.int32, device=dev)
    R = torch.empty((K, S, S), dtype=torch.float32, device=dev)
    hwm = gsearch_hw_model(*[float(x) for x in hw])
    _check(load_library().gsearch_build_tables(
        B, L, S, int(M), K, _ptr(desc, torch.int32, "desc"), _ptr(layer, torch.float64, "layer"),
        ctypes.byref(hwm), _ptr(rmodel, torch.float64, "rmodel"), _ptr(T), _ptr(O), _ptr(R),
        _stream(stream)), "gsearch_build_tables")
    return T, O, R


def gsearch_build_tables_profiled(desc, layer_type, profile, bandwidth, par, M, stream=None):
    """desc int32 [S][5], layer_type int32 [B][L], profile fp64 [Y][3], bandwidth fp64 [NB] on
    the GPU; par = (tokens, overlap, bin_bytes, ckpt_keep, state_factor).
    Returns device tensors T [B][L][S] fp32 and O [B][L][S] int32."""
    import torch
    B, L = layer_type.shape
    S = desc.shape[0]
    dev = layer_type.device
    T = torch.empty((B, L, S), dtype=torch.float32, device=dev)
    O = torch.empty((B, L, S), dtype=torch.int32, device=dev)
    pp = gsearch_profile_params(*[float(x) for x in par])
    _check(load_library().gsearch_build_tables_profiled(
        B, L, S, int(M), int(profile.shape[0]), int(bandwidth.numel()),
        _ptr(desc, torch.int32, "desc"), _ptr(layer_type, torch.int32, "layer_type"),
        _ptr(profile, torch.float64, "profile"), _ptr(bandwidth, torch.float64, "bandwidth"),
        ctypes.byref(pp), _ptr(T), _ptr(O), _stream(stream)), "gsearch_build_tables_profiled")
    return T, O


def gsearch_solve_batch_noalloc(T, O, R, r_index, budget, M, r_class=None, r_class_bound=0,
                                stream=None, out=None):
    """Solve and backtrace of every instance on the library's fixed scratch array (no context,
    no allocation inside the library).  Tensors as for GSearch.gsearch_solve_batch; `out` may
    bring the output tensors (best_cost, best_s, final_row, best_instance, plan, mem_used,
    data_status), otherwise they are made here, on the caller's side of the boundary."""
    import torch
    B, L, S = T.shape
    K = R.shape[0]
    if tuple(O.shape) != (B, L, S) or tuple(R.shape) != (K, S, S) or \
            tuple(r_index.shape) != (B, L) or tuple(budget.shape) != (B,) or \
            (r_class is not None and tuple(r_class.shape) != (S,)):
        raise ValueError("table shapes do not agree")
    dev = T.device
    if out is None:
        out = dict(best_cost=torch.empty(B, dtype=torch.float32, device=dev),
                   best_s=torch.empty(B, dtype=torch.int32, device=dev),
                   final_row=torch.empty((B, S), dtype=torch.float32, device=dev),
                   best_instance=torch.empty(1, dtype=torch.int32, device=dev),
                   plan=torch.empty((B, L), dtype=torch.int32, device=dev),
                   mem_used=torch.empty(B, dtype=torch.int32, device=dev),
                   data_status=torch.empty(1, dtype=torch.int32, device=dev))
    prob = gsearch_problem(B, L, S, int(M), K, _ptr(T, torch.float32, "T"),
                           _ptr(O, torch.int32, "O"), _ptr(R, torch.float32, "R"),
                           _ptr(r_index, torch.int32, "r_index"),
                           _ptr(budget, torch.int32, "budget"),
                           _ptr(r_class, torch.int32, "r_class"), int(r_class_bound))
    res = gsearch_result(_ptr(out["best_cost"]), _ptr(out["best_s"]),
                         _ptr(out.get("final_row")), _ptr(out["best_instance"]))
    _check(load_library().gsearch_solve_batch_noalloc(
        dev.index or 0, ctypes.byref(prob), ctypes.byref(res), _ptr(out.get("plan")),
        _ptr(out.get("mem_used")), _ptr(out.get("data_status")), _stream(stream)),
        "gsearch_solve_batch_noalloc")
    return out


class GSearch:
    """Owner of one gsearch_ctx.  Methods carry the C entry-point names."""

    def __init__(self, max_B, max_L, max_S, max_M, max_K=1, flags=0, device=0):
        self._lib = load_library()
        self._ctx = ctypes.c_void_p()
        self.cfg = gsearch_config(device, max_B, max_L, max_S, max_M, max_K, flags)
        _check(self._lib.gsearch_create(ctypes.byref(self.cfg), ctypes.byref(self._ctx)),
               "gsearch_create")
        self._shape = None

    def gsearch_destroy(self):
        if self._ctx:
            ctx, self._ctx = self._ctx, ctypes.c_void_p()
            _check(self._lib.gsearch_destroy(ctx), "gsearch_destroy")

    close = gsearch_destroy

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.gsearch_destroy()

    def __del__(self):
        try:
            self.gsearch_destroy()
        except Exception:
            pass

    def gsearch_solve_batch(self, T, O, R, r_index, budget, M, want_final_row=True, stream=None,
                            out=None, r_class=None, r_class_bound=0):
        """T fp32 [B][L][S], O int32 [B][L][S], R fp32 [K][S][S], r_index int32 [B][L],
        budget int32 [B], optional r_class int32 [S], all on the GPU; r_class_bound: host
        upper bound on the number of classes (needed above 32).  Returns a dict of device
        tensors (asynchronous)."""
        import torch
        B, L, S = T.shape
        K = R.shape[0]
        if tuple(O.shape) != (B, L, S) or tuple(R.shape) != (K, S, S) or \
                tuple(r_index.shape) != (B, L) or tuple(budget.shape) != (B,) or \
                (r_class is not None and tuple(r_class.shape) != (S,)):
            raise ValueError("table shapes do not agree")
        dev = T.device
        if out is None:
            out = dict(best_cost=torch.empty(B, dtype=torch.float32, device=dev),
                       best_s=torch.empty(B, dtype=torch.int32, device=dev),
                       final_row=(torch.empty((B, S), dtype=torch.float32, device=dev)
                                  if want_final_row else None),
                       best_instance=torch.empty(1, dtype=torch.int32, device=dev))
        prob = gsearch_problem(B, L, S, int(M), K, _ptr(T, torch.float32, "T"),
                               _ptr(O, torch.int32, "O"), _ptr(R, torch.float32, "R"),
                               _ptr(r_index, torch.int32, "r_index"),
                               _ptr(budget, torch.int32, "budget"),
                               _ptr(r_class, torch.int32, "r_class"), int(r_class_bound))
        res = gsearch_result(_ptr(out["best_cost"]), _ptr(out["best_s"]),
                             _ptr(out.get("final_row")), _ptr(out["best_instance"]))
        _check(self._lib.gsearch_solve_batch(self._ctx, ctypes.byref(prob), ctypes.byref(res),
                                             _stream(stream)), "gsearch_solve_batch")
        self._shape = (B, L, S, int(M), K)
        return out

    def gsearch_backtrace(self, instances=None, n=None, stream=None, out=None):
        """Plans of the last solve: instances is an int32 device tensor of ids or None (all)."""
        import torch
        if self._shape is None:
            raise GSearchError(GSEARCH_ERR_NOT_SOLVED, "gsearch_backtrace")
        B, L = self._shape[0], self._shape[1]
        if n is None:
            n = B if instances is None else int(instances.numel())
        dev = instances.device if instances is not None else torch.device("cuda", self.cfg.device)
        if out is None:
            out = dict(plan=torch.empty((n, L), dtype=torch.int32, device=dev),
                       mem_used=torch.empty(n, dtype=torch.int32, device=dev))
        _check(self._lib.gsearch_backtrace(self._ctx, _ptr(instances, torch.int32, "instances"), n,
                                           _ptr(out["plan"]), _ptr(out["mem_used"]),
                                           _stream(stream)), "gsearch_backtrace")
        return out

    def gsearch_data_status(self, stream=None) -> int:
        bits = ctypes.c_int32(0)
        _check(self._lib.gsearch_data_status(self._ctx, _stream(stream), ctypes.byref(bits)),
               "gsearch_data_status")
        return int(bits.value)

    def gsearch_set_profiling(self, enable: bool):
        _check(self._lib.gsearch_set_profiling(self._ctx, int(bool(enable))),
               "gsearch_set_profiling")

    def gsearch_set_instance_groups(self, groups: int):
        _check(self._lib.gsearch_set_instance_groups(self._ctx, int(groups)),
               "gsearch_set_instance_groups")

    def gsearch_set_knob(self, name: str, value: int):
        _check(self._lib.gsearch_set_knob(self._ctx, name.encode(), int(value)), "gsearch_set_knob")

    def gsearch_set_solve_counter(self, value: int, stream=None):
        _check(self._lib.gsearch_set_solve_counter(self._ctx, int(value), _stream(stream)),
               "gsearch_set_solve_counter")

    def gsearch_get_knob(self, name: str) -> int:
        v = ctypes.c_int(0)
        _check(self._lib.gsearch_get_knob(self._ctx, name.encode(), ctypes.byref(v)),
               "gsearch_get_knob")
        return int(v.value)

    def gsearch_instance_groups(self) -> int:
        return int(self._lib.gsearch_instance_groups(self._ctx))

    def gsearch_forward_ms(self) -> float:
        ms = ctypes.c_float(0.0)
        _check(self._lib.gsearch_forward_ms(self._ctx, ctypes.byref(ms)), "gsearch_forward_ms")
        return float(ms.value)

    def gsearch_forward_kernel(self) -> str:
        return self._lib.gsearch_forward_kernel(self._ctx).decode()

    def gsearch_pipeline_reduce(self, group_offsets, group_members, group_micro, stream=None):
        """int32 device tensors (CSR offsets [G+1], member ids, micro-batch counts [G]).
        Returns (group_cost fp32 [G], best_group int32 [1]) on the GPU."""
        import torch
        G = int(group_micro.numel())
        dev = group_micro.device
        cost = torch.empty(G, dtype=torch.float32, device=dev)
        best = torch.empty(1, dtype=torch.int32, device=dev)
        _check(self._lib.gsearch_pipeline_reduce(
            self._ctx, G, _ptr(group_offsets, torch.int32, "group_offsets"),
            _ptr(group_members, torch.int32, "group_members"), int(group_members.numel()),
            _ptr(group_micro, torch.int32, "group_micro"), _ptr(cost), _ptr(best),
            _stream(stream)), "gsearch_pipeline_reduce")
        return cost, best

    def gsearch_budget_curve(self, stream=None):
        import torch
        B, _, _, M, _ = self._shape
        curve = torch.empty((B, M + 1), dtype=torch.float32,
                            device=torch.device("cuda", self.cfg.device))
        _check(self._lib.gsearch_budget_curve(self._ctx, _ptr(curve), _stream(stream)),
               "gsearch_budget_curve")
        return curve

    def gsearch_export_planes(self, want_bp=True, stream=None):
        import torch
        B, L, S, M, _ = self._shape
        dev = torch.device("cuda", self.cfg.device)
        C = torch.empty((B, L, M + 1, S), dtype=torch.float32, device=dev)
        bp = torch.empty((B, L, M + 1, S), dtype=torch.int32, device=dev) if want_bp else None
        _check(self._lib.gsearch_export_planes(self._ctx, _ptr(C), _ptr(bp), _stream(stream)),
               "gsearch_export_planes")
        return C, bp
