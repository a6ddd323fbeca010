"""Python face of the fp64 CPU oracle (oracle/delta_oracle.c).

TEST INFRASTRUCTURE ONLY.  The product package never imports this module and
this module never imports the product's kernels or binding.  Inputs are numpy
float64 arrays holding the exactly-widened bf16 / fp32 input values.

What is computed, in the paper's order:
  * delta_scan      Sec. II-C Eq. 2-3 on the key matrix, top row first
                    (Sec. III-A strategy 3); basis row kept whole.
  * prefill         Sec. III-B prefill hybrid attention: exact scores in the
                    squares of side W on the diagonal, Eq. 4 recursion
                    elsewhere, then Eq. 1 softmax and PV.
  * DecodeState     Sec. III-C workflow: cache of dK, the last W_d raw keys,
                    V; one decode step extends the delta matrix by a row and
                    attends with a sliding exact window of W_d keys.
  * sparsity        Eq. 6.
  * window_from_gamma  Eq. 5.
Grouped-query attention: one delta matrix per KV head, shared by the
Hq/Hkv query heads that read it (query head h reads KV head h // (Hq/Hkv)).
"""
import ctypes
import math
import os

import numpy as np

from . import build_oracle

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = build_oracle.build(force=False)
        lib = ctypes.CDLL(path)
        i64, dbl, f32, ptr = ctypes.c_int64, ctypes.c_double, ctypes.c_float, ctypes.c_void_p
        lib.oracle_delta_scan.argtypes = [ptr, i64, i64, f32, ptr, ptr, ptr, ptr, ptr]
        lib.oracle_delta_scan.restype = None
        lib.oracle_hybrid_rows.argtypes = [ptr, ptr, ptr, ptr, i64, i64, ctypes.c_int, dbl, i64, i64, i64, ptr]
        lib.oracle_hybrid_rows.restype = None
        lib.oracle_hybrid_scores.argtypes = [ptr, ptr, ptr, i64, i64, i64, ctypes.c_int, dbl, i64, i64, i64,
                                             ptr, ptr]
        lib.oracle_hybrid_scores.restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _c(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def delta_scan(K, theta, state=None):
    """K [n, d] -> (mask uint8 [n, d], dK [n, d], Khat [n, d], knife_edge_count).

    state: None for the start of a sequence (row 0 is the basis), else the [d]
    reference vector held before K[0]."""
    lib = _load()
    K, Kp = _c(K)
    n, d = K.shape
    mask = np.zeros((n, d), dtype=np.uint8)
    dK = np.zeros((n, d), dtype=np.float64)
    Khat = np.zeros((n, d), dtype=np.float64)
    knife = ctypes.c_int64(0)
    if state is not None:
        state, sp = _c(state)
        assert state.shape == (d,)
    else:
        sp = None
    lib.oracle_delta_scan(Kp, n, d, ctypes.c_float(np.float32(theta)), sp,
                          mask.ctypes.data_as(ctypes.c_void_p), dK.ctypes.data_as(ctypes.c_void_p),
                          Khat.ctypes.data_as(ctypes.c_void_p), ctypes.byref(knife))
    return mask, dK, Khat, int(knife.value)


def hybrid_rows(Q, K, V, dK, W, mode=0, scale=None, q_off=0, rows=None):
    """Outputs O[len(rows), d] of one query head for a contiguous row range."""
    lib = _load()
    Q, Qp = _c(Q)
    K, Kp = _c(K)
    V, Vp = _c(V)
    dK, dp = _c(dK)
    d = Q.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    r0, r1 = (0, Q.shape[0]) if rows is None else rows
    assert 0 <= r0 <= r1 <= Q.shape[0] and r1 - 1 + q_off < K.shape[0] or r0 == r1
    O = np.zeros((r1 - r0, d), dtype=np.float64)
    lib.oracle_hybrid_rows(Qp, Kp, Vp, dp, d, int(W), int(mode), float(scale), int(q_off), int(r0), int(r1),
                           O.ctypes.data_as(ctypes.c_void_p))
    return O


def hybrid_scores(Q, K, dK, W, mode=0, scale=None, q_off=0, rows=None):
    """Scaled hybrid score rows S[len(rows), nk] (-inf above the causal edge) and the
    uint8 map of which entries are exact (inside the window)."""
    lib = _load()
    Q, Qp = _c(Q)
    K, Kp = _c(K)
    dK, dp = _c(dK)
    nk, d = K.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    r0, r1 = (0, Q.shape[0]) if rows is None else rows
    S = np.zeros((r1 - r0, nk), dtype=np.float64)
    ex = np.zeros((r1 - r0, nk), dtype=np.uint8)
    lib.oracle_hybrid_scores(Qp, Kp, dp, nk, d, int(W), int(mode), float(scale), int(q_off), int(r0), int(r1),
                             S.ctypes.data_as(ctypes.c_void_p), ex.ctypes.data_as(ctypes.c_void_p))
    return S, ex


def sparsity(nnz_total, rows, d, n_units, window):
    """Eq. 6.  S_m is the fraction of zeroed entries of the delta matrices (all rows,
    the basis row included, pooled over n_units KV heads of `rows` rows each);
    S_c = S_m * (1 - W/n) with W clipped to n."""
    total = float(rows) * d * n_units
    s_m = 1.0 - float(nnz_total) / total
    w = min(int(window), int(rows))
    return s_m, s_m * (1.0 - w / float(rows))


def window_from_gamma(n, gamma, w_max):
    """Eq. 5: W = min(floor(gamma * n), W_max); clamped to at least 1 so that the
    attention of a short prompt still has a window."""
    return max(1, min(int(math.floor(gamma * n)), int(w_max)))


def prefill(Q, K, V, theta, window, scale=None, rows=None, q_heads=None, window_mode=0):
    """Whole-layer prefill.  Q [B, Hq, n, d], K/V [B, Hkv, n, d] (float64).
    window_mode 0: exact squares of side `window` on the diagonal (Sec. III-B prefill stage);
    1: exact band of the `window` newest keys per row (the decode stage's rule, row by row).

    Returns dict(O [B, Hq, r, d], mask [B, Hkv, n, d] uint8, nnz [B, Hkv] int64,
    s_m, s_c, knife).  rows=(r0, r1) restricts the output rows; q_heads restricts
    the query heads computed (others left zero)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, Hq, n, d = Q.shape
    Hkv = K.shape[1]
    g = Hq // Hkv
    assert Hq == g * Hkv
    r0, r1 = (0, n) if rows is None else rows
    O = np.zeros((B, Hq, r1 - r0, d))
    mask = np.zeros((B, Hkv, n, d), dtype=np.uint8)
    nnz = np.zeros((B, Hkv), dtype=np.int64)
    knife = 0
    for b in range(B):
        for hk in range(Hkv):
            m, dK, _, ke = delta_scan(K[b, hk], theta)
            mask[b, hk] = m
            nnz[b, hk] = int(m.sum())
            knife += ke
            for h in range(hk * g, (hk + 1) * g):
                if q_heads is not None and h not in q_heads:
                    continue
                O[b, h] = hybrid_rows(Q[b, h], K[b, hk], V[b, hk], dK, window, int(window_mode), scale, 0, (r0, r1))
    s_m, s_c = sparsity(int(nnz.sum()), n, d, B * Hkv, window)
    return dict(O=O, mask=mask, nnz=nnz, s_m=s_m, s_c=s_c, knife=knife)


class DecodeState:
    """The decode-time cache of Sec. III-C for a batch: the delta matrix built so far,
    the raw keys (only the last W_d are ever read), V, and the reference vector."""

    def __init__(self, theta, decode_window, scale=None):
        self.theta = float(np.float32(theta))
        self.W = int(decode_window)
        self.scale = scale
        self.K = None      # [B, Hkv, t, d] raw keys
        self.V = None
        self.dK = None
        self.mask = None   # uint8
        self.khat = None   # [B, Hkv, d]
        self.knife = 0

    @property
    def length(self):
        return 0 if self.K is None else self.K.shape[2]

    def append(self, K_new, V_new):
        """Extend the cache by rows K_new/V_new [B, Hkv, m, d] (prefill hand-off with
        m = n, or one decode token with m = 1).  Returns the mask rows [B, Hkv, m, d]."""
        K_new = np.asarray(K_new, dtype=np.float64)
        V_new = np.asarray(V_new, dtype=np.float64)
        B, Hkv, m, d = K_new.shape
        mask = np.zeros((B, Hkv, m, d), dtype=np.uint8)
        dK = np.zeros((B, Hkv, m, d))
        khat = np.zeros((B, Hkv, d))
        for b in range(B):
            for hk in range(Hkv):
                st = None if self.K is None else self.khat[b, hk]
                mk, dk, kh, ke = delta_scan(K_new[b, hk], self.theta, st)
                mask[b, hk], dK[b, hk], khat[b, hk] = mk, dk, kh[-1]
                self.knife += ke
        if self.K is None:
            self.K, self.V, self.dK, self.mask = K_new.copy(), V_new.copy(), dK, mask
        else:
            self.K = np.concatenate([self.K, K_new], axis=2)
            self.V = np.concatenate([self.V, V_new], axis=2)
            self.dK = np.concatenate([self.dK, dK], axis=2)
            self.mask = np.concatenate([self.mask, mask], axis=2)
        self.khat = khat
        return mask

    def step(self, q, k, v):
        """One decode step: q [B, Hq, d], k/v [B, Hkv, d].  Returns (o [B, Hq, d],
        mask_row [B, Hkv, d]).  The W_d most recent keys, the new one included, get
        exact scores; older keys get the Eq. 4 recursion over the cached deltas."""
        q = np.asarray(q, dtype=np.float64)
        mask_row = self.append(np.asarray(k)[:, :, None, :], np.asarray(v)[:, :, None, :])[:, :, 0, :]
        B, Hq, d = q.shape
        Hkv = self.K.shape[1]
        g = Hq // Hkv
        t = self.length - 1
        o = np.zeros((B, Hq, d))
        for b in range(B):
            for h in range(Hq):
                hk = h // g
                o[b, h] = hybrid_rows(q[b, h][None, :], self.K[b, hk], self.V[b, hk], self.dK[b, hk],
                                      self.W, 1, self.scale, t, (0, 1))[0]
        return o, mask_row

    def nnz(self):
        return self.mask.reshape(self.mask.shape[0], self.mask.shape[1], -1).sum(axis=2).astype(np.int64)
