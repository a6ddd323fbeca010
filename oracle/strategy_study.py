"""CPU-only study of the three delta-matrix construction strategies of Sec. III-A (prefilling stage analysis).

TEST INFRASTRUCTURE / ANALYSIS ONLY: this script uses the CPU oracle's delta scan (Sec. II-C Eq. 2-3) and
plain numpy; nothing here is part of the GPU product path.

  (1) top-down query deltas     delta rows of Q from the first row down, keys unchanged
  (2) bottom-up query deltas    delta rows of Q from the last row up, keys unchanged
  (3) top-down key deltas       delta rows of K from the first row down, queries unchanged (the adopted one)

By Eq. 4 summed up (the deltas of a reference telescope), every strategy replaces one operand of Q K^T by
its held reference: S1 = Q_hat K^T, S2 = Q_hat' K^T, S3 = Q K_hat^T.  No exact window is applied: the
study isolates what the construction alone preserves after causal masking.  Thresholds are tuned per
strategy to the same delta-matrix sparsity, so the comparison is at equal compute.

Run:  python -m oracle.strategy_study        (prints a table; a few seconds)
"""
import math

import numpy as np

from paper_2507_19608_amd import workloads as wl
from . import delta_oracle as orc


def reference_rows(X, theta, bottom_up=False):
    """Held reference of every row of X [n, d] when the rows are scanned in the given direction."""
    Y = X[::-1] if bottom_up else X
    mask, _, Xhat, _ = orc.delta_scan(np.ascontiguousarray(Y), theta)
    if bottom_up:
        Xhat, mask = Xhat[::-1], mask[::-1]
    return np.ascontiguousarray(Xhat), mask


def tune_theta(X, target, bottom_up=False):
    lo, hi = np.float32(0.0), np.float32(8.0)
    mid = hi
    for _ in range(40):
        mid = np.float32((lo + hi) / np.float32(2))
        _, mask = reference_rows(X, mid, bottom_up)
        s = 1.0 - mask.mean()
        if abs(s - target) < 2e-3:
            break
        if s < target:
            lo = mid
        else:
            hi = mid
    return float(mid)


def causal_softmax_out(S, V):
    n = S.shape[0]
    S = np.where(np.tril(np.ones((n, n), dtype=bool)), S, -np.inf)
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    return P @ V, P


def study(Q, K, V, sparsity):
    """Per strategy: exact causal scores, mean / max score error over the causal entries (scaled scores),
    mean / max output error against dense causal attention, total-variation distance of the probabilities."""
    n, d = Q.shape
    scale = 1.0 / math.sqrt(d)
    tri = np.tril(np.ones((n, n), dtype=bool))
    S = (Q @ K.T) * scale
    O, P = causal_softmax_out(S, V)
    rows = {}
    for name, which, bottom_up in (("(1) top-down query", "q", False), ("(2) bottom-up query", "q", True),
                                   ("(3) top-down key", "k", False)):
        X = Q if which == "q" else K
        theta = tune_theta(X, sparsity, bottom_up)
        Xhat, mask = reference_rows(X, theta, bottom_up)
        Sa = ((Xhat @ K.T) if which == "q" else (Q @ Xhat.T)) * scale
        Oa, Pa = causal_softmax_out(Sa, V)
        err = np.abs(Sa - S)[tri]
        rows[name] = dict(theta=theta, sparsity=1.0 - mask.mean(), exact=int((err == 0).sum()),
                          score_mean=float(err.mean()), score_max=float(err.max()),
                          out_mean=float(np.abs(Oa - O).mean()), out_max=float(np.abs(Oa - O).max()),
                          tv=float(0.5 * np.abs(Pa - P).sum(axis=1).mean()))
    return rows


def inputs(seed, n, d, sink):
    """One head of the synthetic AR(1)+jump streams; `sink` > 0 turns key 0 into an attention sink: a key
    aligned with the mean query direction, so that the first column carries a large share of every row's mass."""
    Q = wl.ar1_jump(seed, "Q", [0], 1, n, d, 0.05, False)[0, 0]
    K = wl.ar1_jump(seed, "K", [0], 1, n, d, 0.05, False)[0, 0]
    V = wl.ar1_jump(seed, "V", [0], 1, n, d, 0.05, False)[0, 0]
    if sink > 0:
        K = K.copy()
        Q = Q + 0.5                                                  # a common query component of 0.5 per channel
        K[0] = sink * np.ones(d)
    return (wl.round_to_dtype(x, "bf16") for x in (Q, K, V))


def main():
    n, d, sparsity = 512, 64, 0.60
    for sink in (0.0, 1.0):
        print(f"\nn = {n}, d = {d}, delta-matrix sparsity {sparsity:.2f}, "
              f"{'with an attention sink at key 0' if sink else 'no attention sink'}; mean over 4 seeds")
        acc = {}
        for seed in (11, 12, 13, 14):
            Q, K, V = inputs(seed, n, d, sink)
            for name, r in study(Q, K, V, sparsity).items():
                a = acc.setdefault(name, {k: 0.0 for k in r})
                for k, v in r.items():
                    a[k] += v / 4.0
        print(f"{'strategy':22s} {'theta':>7s} {'exact':>6s} {'|dS| mean':>10s} {'|dS| max':>9s} {'|dO| mean':>10s} "
              f"{'|dO| max':>9s} {'TV(P)':>7s}")
        for name, a in acc.items():
            print(f"{name:22s} {a['theta']:7.3f} {a['exact']:6.0f} {a['score_mean']:10.4f} {a['score_max']:9.3f} "
                  f"{a['out_mean']:10.5f} {a['out_max']:9.4f} {a['tv']:7.4f}")


if __name__ == "__main__":
    main()
