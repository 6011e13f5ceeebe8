"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes its workspace, counts strategies, and reports a missing device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2504_21411_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2504_21411_amd import build
        build.build()
    return binding.load_library()


def _has_gpu():
    import torch
    return torch.cuda.is_available()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "gsearch.h")).read()
    declared = set(re.findall(r"\b(gsearch_[a-z_]+)\s*\(", header))
    declared -= {"gsearch_ctx"}
    assert {"gsearch_create", "gsearch_solve_batch", "gsearch_backtrace",
            "gsearch_destroy"} <= declared
    from paper_2504_21411_amd import binding
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror_and_codes(lib):
    from paper_2504_21411_amd import binding
    assert binding.strerror(0) == "ok"
    seen = {binding.strerror(c) for c in range(-7, 1)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert binding.strerror(-99) == "unknown status"


def test_workspace_bytes_is_host_arithmetic(lib):
    from paper_2504_21411_amd import binding as b
    assert b.gsearch_workspace_bytes(0, 1, 1, 1) == 0
    assert b.gsearch_workspace_bytes(1, 1, 2000, 1) == 0          # S above the library limit
    small = b.gsearch_workspace_bytes(1, 24, 12, 256)
    # at least two plane slots + 23 uint8 backpointer planes of 12 x 320 elements, plus tables
    assert small >= 2 * 12 * 320 * 4 + 23 * 12 * 320
    assert small < 1 << 20
    keep = b.gsearch_workspace_bytes(1, 24, 12, 256, flags=b.GSEARCH_FLAG_KEEP_PLANES)
    assert keep > small
    nobp = b.gsearch_workspace_bytes(8, 128, 96, 16384, flags=b.GSEARCH_FLAG_NO_BACKPOINTERS)
    withbp = b.gsearch_workspace_bytes(8, 128, 96, 16384)
    # (with backpointers: four plane slots that take turns, 50 MB each, and 1.07 GB of
    # backpointers)
    assert 6.0e9 < nobp < 7.0e9 and 1.7e9 < withbp < 1.9e9
    big16 = b.gsearch_workspace_bytes(1, 40, 257, 1000)
    big8 = b.gsearch_workspace_bytes(1, 40, 256, 1000)
    assert big16 > big8 * 1.5                                      # uint16 backpointers


def test_enumerate_count_matches_oracle(lib, oracle_mod):
    from paper_2504_21411_amd import binding as b
    for k in range(0, 9):
        for caps in [(0, 0, 0), (8, 4, 16), (4, 1, 0), (0, 2, 0), (0, 32, 0), (2, 2, 2)]:
            n = b.gsearch_enumerate_count(1 << k, *caps)
            assert n == len(oracle_mod.enumerate_strategies(1 << k, *caps))
    with pytest.raises(b.GSearchError):
        b.gsearch_enumerate_count(12)


def test_create_reports_argument_errors_and_missing_device(lib):
    from paper_2504_21411_amd import binding as b
    ctx = ctypes.c_void_p()
    assert lib.gsearch_create(None, ctypes.byref(ctx)) == b.GSEARCH_ERR_INVALID_ARG
    bad = b.gsearch_config(0, 0, 1, 1, 1, 1, 0)
    assert lib.gsearch_create(ctypes.byref(bad), ctypes.byref(ctx)) == b.GSEARCH_ERR_INVALID_ARG
    badflag = b.gsearch_config(0, 1, 1, 1, 1, 1, 0x80)
    assert lib.gsearch_create(ctypes.byref(badflag), ctypes.byref(ctx)) == b.GSEARCH_ERR_INVALID_ARG
    ok = b.gsearch_config(0, 1, 2, 2, 4, 1, 0)
    assert lib.gsearch_create(ctypes.byref(ok), None) == b.GSEARCH_ERR_INVALID_ARG
    if not _has_gpu():
        assert lib.gsearch_create(ctypes.byref(ok), ctypes.byref(ctx)) == b.GSEARCH_ERR_NO_DEVICE
        assert not ctx.value
        with pytest.raises(b.GSearchError) as ei:
            b.GSearch(1, 2, 2, 4)
        assert ei.value.code == b.GSEARCH_ERR_NO_DEVICE
    assert lib.gsearch_destroy(None) == b.GSEARCH_OK
    assert lib.gsearch_solve_batch(None, None, None, None) == b.GSEARCH_ERR_INVALID_ARG
    assert lib.gsearch_backtrace(None, None, 1, None, None, None) == b.GSEARCH_ERR_INVALID_ARG
    assert lib.gsearch_build_tables(0, 1, 1, 1, 1, None, None, None, None, None, None, None,
                                    None) == b.GSEARCH_ERR_INVALID_ARG


def test_new_entry_points_reject_bad_arguments_without_a_gpu(lib):
    from paper_2504_21411_amd import binding as b
    assert lib.gsearch_set_instance_groups(None, 2) == b.GSEARCH_ERR_INVALID_ARG
    assert lib.gsearch_instance_groups(None) == 0
    assert lib.gsearch_layout_classes(None, 4, None, None, None) == b.GSEARCH_ERR_INVALID_ARG
    dummy = ctypes.c_void_p(64)       # never dereferenced: the size check comes first
    assert lib.gsearch_layout_classes(dummy, 0, dummy, None, None) == b.GSEARCH_ERR_INVALID_ARG
    assert lib.gsearch_layout_classes(dummy, 1025, dummy, None, None) == b.GSEARCH_ERR_INVALID_ARG
    assert lib.gsearch_forward_kernel(None) == b""
    # tuning knobs: the names are host data; setting needs a context
    names = b.gsearch_knob_names()
    assert names == ["kernel", "small", "jsplit", "waves_per_block", "row_groups", "streams", "fronts", "spin_limit", "hold_flags", "front_tiles"]
    assert lib.gsearch_knob_name(-1) is None and lib.gsearch_knob_name(len(names)) is None
    assert lib.gsearch_set_knob(None, b"fronts", 1) == b.GSEARCH_ERR_INVALID_ARG
    v = ctypes.c_int(0)
    assert lib.gsearch_get_knob(None, b"fronts", ctypes.byref(v)) == b.GSEARCH_ERR_INVALID_ARG
    assert lib.gsearch_set_solve_counter(None, 5, None) == b.GSEARCH_ERR_INVALID_ARG


def test_knobs_take_their_initial_values_from_the_environment(lib, monkeypatch):
    """GSEARCH_<NAME> is read when a context is created and nowhere else; what a new context
    would start with can be asked without a GPU.  Numbers in [-1, 64] count, anything else is
    ignored."""
    from paper_2504_21411_amd import binding as b
    for name in b.gsearch_knob_names():
        monkeypatch.delenv("GSEARCH_" + name.upper(), raising=False)
    defaults = {name: b.gsearch_knob_initial(name) for name in b.gsearch_knob_names()}
    assert defaults["fronts"] == -1 and defaults["small"] == -1 and defaults["jsplit"] == 0
    assert defaults["spin_limit"] == 0 and defaults["hold_flags"] == 0
    monkeypatch.setenv("GSEARCH_FRONTS", "5")
    monkeypatch.setenv("GSEARCH_JSPLIT", "8")
    monkeypatch.setenv("GSEARCH_STREAMS", "-1")
    assert b.gsearch_knob_initial("fronts") == 5 and b.gsearch_knob_initial("jsplit") == 8
    assert b.gsearch_knob_initial("streams") == -1
    for bad in ("65", "-2", "4x", "", "3 ", "1e1", "0x10"):
        monkeypatch.setenv("GSEARCH_FRONTS", bad)
        assert b.gsearch_knob_initial("fronts") == defaults["fronts"], bad
    monkeypatch.setenv("GSEARCH_FRONTS", "0")
    assert b.gsearch_knob_initial("fronts") == 0
    assert b.gsearch_knob_initial("kernel") == defaults["kernel"]      # others untouched
    with pytest.raises(b.GSearchError):
        b.gsearch_knob_initial("no_such_knob")
    # the entry point on the fixed array checks its arguments before it touches a device
    assert lib.gsearch_solve_batch_noalloc(0, None, None, None, None, None, None) == \
        b.GSEARCH_ERR_INVALID_ARG
    prob = b.gsearch_problem(0, 1, 1, 1, 1, None, None, None, None, None, None, 0)
    res = b.gsearch_result(None, None, None, None)
    assert lib.gsearch_solve_batch_noalloc(0, ctypes.byref(prob), ctypes.byref(res), None, None,
                                           None, None) == b.GSEARCH_ERR_INVALID_ARG
    prob = b.gsearch_problem(8, 128, 96, 16384, 1, None, None, None, None, None, None, 0)
    assert lib.gsearch_solve_batch_noalloc(0, ctypes.byref(prob), ctypes.byref(res), None, None,
                                           None, None) == b.GSEARCH_ERR_CAPACITY
    assert lib.gsearch_solve_batch_noalloc(-1, ctypes.byref(prob), ctypes.byref(res), None, None,
                                           None, None) == b.GSEARCH_ERR_INVALID_ARG
    # the problem struct carries the optional class promise as its last two fields
    assert [f[0] for f in b.gsearch_problem._fields_][-2:] == ["r_class", "r_class_bound"]
    header = open(os.path.join(ROOT, "include", "gsearch.h")).read()
    assert "const int32_t *r_class;" in header and "int32_t r_class_bound;" in header
    assert b.GSEARCH_DEFAULT_CLASSES == int(re.search(r"#define GSEARCH_DEFAULT_CLASSES (\d+)",
                                                      header).group(1))
    assert b.GSEARCH_MAX_CLASSES == int(re.search(r"#define GSEARCH_MAX_CLASSES (\d+)", header).group(1))
    assert b.GSEARCH_DATA_BAD_RCLASS == int(re.search(r"#define GSEARCH_DATA_BAD_RCLASS (0x[0-9a-f]+)",
                                                     header).group(1), 16)


def test_binding_constants_equal_the_header():
    """Every flag, data-status bit, limit and status code of the binding is the header's."""
    from paper_2504_21411_amd import binding as b
    header = open(os.path.join(ROOT, "include", "gsearch.h")).read()
    defines = {m.group(1): int(m.group(2), 0) for m in
               re.finditer(r"#define (GSEARCH_[A-Z0-9_]+) (0x[0-9a-fA-F]+|\d+)u?\b", header)}
    enums = {m.group(1): int(m.group(2)) for m in
             re.finditer(r"(GSEARCH_(?:OK|ERR_[A-Z_]+)) = (-?\d+)", header)}
    assert len(defines) >= 15 and len(enums) >= 7
    for name, value in {**defines, **enums}.items():
        assert getattr(b, name) == value, name
    for name in dir(b):
        if name.startswith("GSEARCH_") and isinstance(getattr(b, name), int):
            assert name in defines or name in enums, f"{name} is not in the header"
    # a context refuses flag bits it does not know (before touching any device)
    assert b.gsearch_workspace_bytes(1, 2, 2, 2, flags=0x40) == 0
    assert b.gsearch_workspace_bytes(1, 2, 2, 2, flags=b.GSEARCH_FLAG_NO_BIN_UNIT) > 0


def test_workspace_covers_class_tables_and_plane_slack(lib):
    """More strategies never shrink the workspace; small S still reserves the 32 backpointer
    columns of the class kernel and the slack block behind the planes."""
    from paper_2504_21411_amd import binding as b
    sizes = [b.gsearch_workspace_bytes(4, 10, S, 1000) for S in (9, 16, 24, 33, 44, 96)]
    assert sizes == sorted(sizes)
    pitch = 1024                                   # round_up(1001, 64)
    assert sizes[0] >= 2 * 4 * 9 * pitch * 4 + 16 * pitch * 4 + 9 * 4 * 32 * pitch


def test_product_package_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_21411_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "liboracle" not in text, f
