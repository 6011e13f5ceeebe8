"""Reader for the small text fixtures under tests/golden/ (key, then numbers)."""
import os

import numpy as np

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_example(name):
    vals, results = {}, []
    with open(os.path.join(HERE, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *rest = line.split()
            nums = [float(x) for x in rest]
            if key == "result":
                results.append(nums)
            else:
                vals[key] = nums
    L, S, K = int(vals["L"][0]), int(vals["S"][0]), int(vals["K"][0])
    E = int(vals["E_max"][0])
    ex = dict(L=L, S=S, K=K, E_max=E,
              T=np.asarray(vals["T"], np.float32).reshape(L, S),
              O=np.asarray(vals["O"], np.int32).reshape(L, S),
              R=np.asarray(vals["R"], np.float32).reshape(K, S, S),
              r_index=np.asarray(vals["r_index"], np.int32),
              C=np.stack([np.asarray(vals[f"C{l}"], np.float32).reshape(E + 1, S)
                          for l in range(L)]),
              bp=np.stack([np.zeros((E + 1, S), np.int64)] +
                          [np.asarray(vals[f"bp{l}"], np.int64).reshape(E + 1, S)
                           for l in range(1, L)]),
              results=[dict(E=int(r[0]), best_cost=np.float32(r[1]), best_s=int(r[2]),
                            mem_used=int(r[3]), plan=[int(x) for x in r[4:]])
                       for r in results])
    if "feasible_at_5" in vals:
        ex["feasible_at_5"] = int(vals["feasible_at_5"][0])
    return ex
