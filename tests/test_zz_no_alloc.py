"""gsearch_solve_batch_noalloc (workspace in the library's fixed device array) against
gsearch_solve_batch + gsearch_backtrace on a context, bit for bit, through the C ABI.

Calls follow each other on one stream with shrinking and changing shapes, so every call
finds the previous call's data in the array, including at the place of the words it needs
cleared.
"""
import numpy as np
import pytest

from paper_2504_21411_amd import workloads

pytestmark = pytest.mark.gpu


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def cases():
    w1, rc1 = workloads.class_tables("na_classes", 4, 10, 44, 700, [4] * 11, seed=31, coarse=True,
                                     budget=np.array([700, 333, 65, 512], np.int32))
    w2 = workloads.random_tables("na_small", 2, 6, 12, 100, K=2, seed=32,
                                 budget=np.array([100, 37], np.int32))
    w3, rc3 = workloads.class_tables("na_classes_small", 3, 5, 24, 130, [2] * 12, seed=33,
                                     budget=np.array([130, 64, 9], np.int32))
    w4 = workloads.random_tables("na_mid", 3, 7, 44, 300, K=3, seed=34,
                                 budget=np.array([300, 2, 129], np.int32))
    return [(w1, rc1), (w2, None), (w3, rc3), (w4, None), (w2, None)]


def test_noalloc_entry_point_matches_the_context_path():
    import torch
    assert torch.cuda.is_available(), "needs the MI355X"
    from paper_2504_21411_amd import binding, runner
    binding.load_library()
    dev = torch.device("cuda", 0)
    for w, r_class in cases():
        print("case", w.name, w.B, w.L, w.S, w.M, flush=True)
        want = runner.solve_workload(w, r_class=r_class)
        assert want["data_status"] == 0
        dw = runner.DeviceWorkload(w)
        rc = None if r_class is None else torch.from_numpy(np.ascontiguousarray(r_class, np.int32)).to(dev)
        out = binding.gsearch_solve_batch_noalloc(
            dw.T, dw.O, dw.R, dw.r_index, dw.budget, w.M, r_class=rc,
            r_class_bound=0 if r_class is None else int(r_class.max()) + 1)
        torch.cuda.synchronize()
        got = {k: v.cpu().numpy() for k, v in out.items()}
        assert int(got["data_status"][0]) == 0, w.name
        for k in ("best_cost", "final_row"):
            assert np.array_equal(bits(got[k]), bits(want[k])), (w.name, k)
        for k in ("best_s", "plan", "mem_used", "best_instance"):
            assert np.array_equal(got[k], want[k]), (w.name, k)


def test_noalloc_entry_point_reports_bad_tables_and_rejects_large_shapes():
    import torch
    from paper_2504_21411_amd import binding, runner
    binding.load_library()
    w = workloads.random_tables("na_bad", 2, 4, 8, 50, seed=35)
    w.T[1, 2, 3] = -1.0
    dw = runner.DeviceWorkload(w)
    out = binding.gsearch_solve_batch_noalloc(dw.T, dw.O, dw.R, dw.r_index, dw.budget, w.M)
    torch.cuda.synchronize()
    assert int(out["data_status"].cpu()[0]) == binding.GSEARCH_DATA_BAD_T
    assert int(out["best_instance"].cpu()[0]) == -1
    # a clean call afterwards starts from a cleared status word
    w.T[1, 2, 3] = 1.0
    dw = runner.DeviceWorkload(w)
    out = binding.gsearch_solve_batch_noalloc(dw.T, dw.O, dw.R, dw.r_index, dw.budget, w.M)
    torch.cuda.synchronize()
    assert int(out["data_status"].cpu()[0]) == 0
    want = runner.solve_workload(w)
    assert np.array_equal(out["plan"].cpu().numpy(), want["plan"])
    # beyond the fixed array: refused before anything is launched
    big = workloads.random_tables("na_big", 16, 32, 44, 4096, seed=36)
    assert binding.gsearch_workspace_bytes(16, 32, 44, 4096) > binding.GSEARCH_NOALLOC_SCRATCH_BYTES
    dwb = runner.DeviceWorkload(big)
    with pytest.raises(binding.GSearchError) as e:
        binding.gsearch_solve_batch_noalloc(dwb.T, dwb.O, dwb.R, dwb.r_index, dwb.budget, big.M)
    assert e.value.code == binding.GSEARCH_ERR_CAPACITY
