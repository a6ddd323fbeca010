"""Tune the delta threshold of each synthetic workload to its target delta-matrix sparsity.

Calls only the CPU oracle's delta scan (Sec. II-C Eq. 2-3) on the seeded inputs and
writes paper_2507_19608_amd/workload_thetas.json.  Bisection on [0, 4], at most 40
halvings, stops when the pooled S_m is within 0.1 % of the target; the threshold is
kept as a binary32 value and stored as a hex float.

Run:  python -m oracle.tune_theta
"""
import json
import os

import numpy as np

from paper_2507_19608_amd import workloads as wl
from . import delta_oracle as orc

OUT = os.path.join(os.path.dirname(os.path.abspath(wl.__file__)), "workload_thetas.json")


def pooled_sm(K, theta):
    B, H, n, d = K.shape
    nnz = 0
    for b in range(B):
        for h in range(H):
            m, _, _, _ = orc.delta_scan(K[b, h], theta)
            nnz += int(m.sum())
    return 1.0 - nnz / float(B * H * n * d), nnz


def tune(w):
    K = wl.generate(w, ("K",))["K"]
    lo, hi = np.float32(0.0), np.float32(4.0)
    best = None
    for _ in range(40):
        mid = np.float32((lo + hi) / np.float32(2))
        sm, nnz = pooled_sm(K, mid)
        best = (mid, sm, nnz)
        if abs(sm - w.target_sparsity) < 1e-3:
            break
        if sm < w.target_sparsity:
            lo = mid
        else:
            hi = mid
    return best


def main():
    table = {}
    todo = [wl.C2, wl.C3, wl.C4] + [w for w in wl.C5_SWEEP if w.target_sparsity is not None]
    for w in todo:
        theta, sm, nnz = tune(w)
        table[w.key()] = {"theta_hex": float(theta).hex(), "theta": float(theta), "s_m": sm, "nnz": nnz,
                          "rows": w.total_len}
        print(w.key(), table[w.key()], flush=True)
    with open(OUT, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)


if __name__ == "__main__":
    main()
