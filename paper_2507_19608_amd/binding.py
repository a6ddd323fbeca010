"""Thin ctypes binding of libdelta_attn.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch is used for device
memory and the current stream.  There is no CPU fallback: if the library is missing
or no GPU is present, calls raise.
"""
import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdelta_attn.so")

DA_OK = 0
DA_F32, DA_BF16 = 0, 1
DA_SCORE_GATHER, DA_SCORE_REBASE = 0, 1
DA_WINDOW_BLOCK, DA_WINDOW_SLIDING = 0, 1

EXPORTS = [
    "delta_attn_version", "delta_attn_status_string", "delta_attn_last_error",
    "delta_attn_stage_timing_enable", "delta_attn_stage_timing_read", "delta_attn_window_from_gamma",
    "delta_attn_prefill_workspace_bytes", "delta_attn_delta_scan_workspace_bytes", "delta_attn_delta_scan", "delta_attn_prefill",
    "delta_attn_prefill_noalloc",
    "delta_attn_prefill_append_workspace_bytes", "delta_attn_prefill_append", "delta_attn_cache_create", "delta_attn_cache_destroy", "delta_attn_cache_reset",
    "delta_attn_cache_set_launch_plan", "delta_attn_cache_length", "delta_attn_cache_nnz", "delta_attn_cache_mask", "delta_attn_decode",
    "delta_attn_sparsity",
]


class PrefillParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("seq_len", ctypes.c_int32), ("window", ctypes.c_int32),
                ("theta", ctypes.c_float), ("scale", ctypes.c_float), ("dtype", ctypes.c_int32),
                ("score_mode", ctypes.c_int32), ("window_mode", ctypes.c_int32)]


class DeltaAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = lib().delta_attn_last_error().decode() if status in (3, 5) else ""
        super().__init__(f"{where}: {status_string(status)} (da_status {status}) {detail}")


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2507_19608_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_double
        pp = ctypes.POINTER(PrefillParams)
        L.delta_attn_version.restype = ctypes.c_char_p
        L.delta_attn_status_string.restype = ctypes.c_char_p
        L.delta_attn_status_string.argtypes = [ctypes.c_int]
        L.delta_attn_last_error.restype = ctypes.c_char_p
        L.delta_attn_stage_timing_enable.restype = None
        L.delta_attn_stage_timing_enable.argtypes = [i32]
        L.delta_attn_stage_timing_read.restype = i32
        L.delta_attn_stage_timing_read.argtypes = [ctypes.POINTER(dbl), ctypes.POINTER(i32)]
        L.delta_attn_window_from_gamma.restype = i32
        L.delta_attn_window_from_gamma.argtypes = [i32, dbl, i32]
        L.delta_attn_prefill_workspace_bytes.restype = ctypes.c_size_t
        L.delta_attn_prefill_workspace_bytes.argtypes = [pp]
        L.delta_attn_delta_scan.restype = ctypes.c_int
        L.delta_attn_delta_scan_workspace_bytes.restype = ctypes.c_size_t
        L.delta_attn_delta_scan_workspace_bytes.argtypes = [pp]
        L.delta_attn_delta_scan.argtypes = [pp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.delta_attn_prefill.restype = ctypes.c_int
        L.delta_attn_prefill.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.delta_attn_prefill_noalloc.restype = ctypes.c_int
        L.delta_attn_prefill_noalloc.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
        L.delta_attn_prefill_append_workspace_bytes.restype = ctypes.c_size_t
        L.delta_attn_prefill_append_workspace_bytes.argtypes = [pp, vp]
        L.delta_attn_prefill_append.restype = ctypes.c_int
        L.delta_attn_prefill_append.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.delta_attn_cache_create.restype = ctypes.c_int
        L.delta_attn_cache_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32, i32, i32, i32, f32, f32, i32]
        L.delta_attn_cache_destroy.restype = ctypes.c_int
        L.delta_attn_cache_destroy.argtypes = [vp]
        L.delta_attn_cache_reset.restype = ctypes.c_int
        L.delta_attn_cache_reset.argtypes = [vp, vp]
        L.delta_attn_cache_set_launch_plan.restype = ctypes.c_int
        L.delta_attn_cache_set_launch_plan.argtypes = [vp, i32, i32]
        L.delta_attn_cache_length.restype = i64
        L.delta_attn_cache_length.argtypes = [vp]
        L.delta_attn_cache_nnz.restype = vp
        L.delta_attn_cache_nnz.argtypes = [vp]
        L.delta_attn_cache_mask.restype = vp
        L.delta_attn_cache_mask.argtypes = [vp]
        L.delta_attn_decode.restype = ctypes.c_int
        L.delta_attn_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        L.delta_attn_sparsity.restype = ctypes.c_int
        L.delta_attn_sparsity.argtypes = [vp, i32, i32, i64, i32, i32, vp, ctypes.POINTER(dbl), ctypes.POINTER(dbl)]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().delta_attn_status_string(status).decode()


def version() -> str:
    return lib().delta_attn_version().decode()


def delta_attn_window_from_gamma(n: int, gamma: float, w_max: int) -> int:
    return int(lib().delta_attn_window_from_gamma(n, gamma, w_max))


STAGES = ("scan", "emit", "attn", "cache_fill", "append", "chunk", "combine")


def delta_attn_stage_timing_enable(on: bool):
    lib().delta_attn_stage_timing_enable(1 if on else 0)


def delta_attn_stage_timing_read():
    """{stage: (total_ms, launches)} since the previous read; synchronise the device first."""
    ms = (ctypes.c_double * len(STAGES))()
    calls = (ctypes.c_int32 * len(STAGES))()
    lib().delta_attn_stage_timing_read(ms, calls)
    return {name: (ms[i], calls[i]) for i, name in enumerate(STAGES)}


def _check(st: int, where: str):
    if st != DA_OK:
        raise DeltaAttnError(st, where)


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("delta_attn needs a GPU: there is no CPU path")
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return DA_F32
    if t.dtype == torch.bfloat16:
        return DA_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream() -> int:
    return _torch().cuda.current_stream().cuda_stream


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dev(t, name):
    if not (t.is_cuda and t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous device tensor")
    return t


def make_params(Q, K, window: int, theta: float, scale: float = 0.0, score_mode: int = DA_SCORE_GATHER,
                window_mode: int = DA_WINDOW_BLOCK):
    B, Hq, n, d = Q.shape
    return PrefillParams(B, Hq, K.shape[1], d, n, int(window), float(theta), float(scale), _dtype_code(Q),
                         int(score_mode), int(window_mode))


def delta_attn_prefill_workspace_bytes(params: PrefillParams) -> int:
    return int(lib().delta_attn_prefill_workspace_bytes(ctypes.byref(params)))


class Cache:
    """Owner of a da_cache handle."""

    def __init__(self, batch, n_q_heads, n_kv_heads, head_dim, max_seq, decode_window, theta, dtype, scale=0.0):
        torch = _torch()
        code = DA_F32 if dtype == torch.float32 else DA_BF16 if dtype == torch.bfloat16 else -1
        h = ctypes.c_void_p()
        _check(lib().delta_attn_cache_create(ctypes.byref(h), batch, n_q_heads, n_kv_heads, head_dim, max_seq,
                                             decode_window, float(theta), float(scale), code),
               "delta_attn_cache_create")
        self.handle = h
        self.shape = (batch, n_q_heads, n_kv_heads, head_dim, max_seq)
        self.dtype = dtype

    def __len__(self):
        return int(lib().delta_attn_cache_length(self.handle))

    def reset(self):
        _check(lib().delta_attn_cache_reset(self.handle, _stream()), "delta_attn_cache_reset")

    def set_launch_plan(self, merge_in_kernel: int = -1, wave_slots: int = 0):
        _check(lib().delta_attn_cache_set_launch_plan(self.handle, int(merge_in_kernel), int(wave_slots)),
               "delta_attn_cache_set_launch_plan")

    def nnz(self):
        """[B, Hkv] int64 copy of the per-unit nnz counters."""
        torch = _torch()
        B, _, Hkv, _, _ = self.shape
        out = torch.empty(B * Hkv, dtype=torch.int64, device="cuda")
        src = lib().delta_attn_cache_nnz(self.handle)
        torch.cuda.current_stream().synchronize()
        _hip_copy(out.data_ptr(), src, B * Hkv * 8)
        return out.view(B, Hkv)

    def mask_rows(self, length=None):
        """[B, Hkv, length, d/32] int32 copy of the cached mask bits."""
        torch = _torch()
        B, _, Hkv, d, max_seq = self.shape
        full = torch.empty(B * Hkv * max_seq * (d // 32), dtype=torch.int32, device="cuda")
        src = lib().delta_attn_cache_mask(self.handle)
        torch.cuda.current_stream().synchronize()
        _hip_copy(full.data_ptr(), src, full.numel() * 4)
        n = len(self) if length is None else length
        return full.view(B, Hkv, max_seq, d // 32)[:, :, :n]

    def close(self):
        if self.handle is not None:
            lib().delta_attn_cache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


_hip = None


def _hip_copy(dst: int, src: int, nbytes: int):
    """Device-to-device copy through the HIP runtime (plumbing for the cache accessors)."""
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
        _hip.hipMemcpy.restype = ctypes.c_int
    rc = _hip.hipMemcpy(dst, src, nbytes, 3)   # hipMemcpyDeviceToDevice
    if rc != 0:
        raise RuntimeError(f"hipMemcpy failed with {rc}")


def delta_attn_delta_scan(K, theta: float, want_khat: bool = False):
    """K [B, Hkv, n, d] -> (mask_bits int32 [B, Hkv, n, d/32], nnz int64 [B, Hkv], k_hat or None)."""
    torch = _torch()
    _dev(K, "K")
    B, Hkv, n, d = K.shape
    p = PrefillParams(B, Hkv, Hkv, d, n, 1, float(theta), 0.0, _dtype_code(K), DA_SCORE_GATHER)
    mask = torch.empty((B, Hkv, n, d // 32), dtype=torch.int32, device=K.device)
    nnz = torch.empty((B, Hkv), dtype=torch.int64, device=K.device)
    khat = torch.empty_like(K) if want_khat else None
    ws = torch.empty(max(int(lib().delta_attn_delta_scan_workspace_bytes(ctypes.byref(p))), 1), dtype=torch.uint8,
                     device=K.device)
    _check(lib().delta_attn_delta_scan(ctypes.byref(p), K.data_ptr(), mask.data_ptr(), nnz.data_ptr(), _ptr(khat),
                                       ws.data_ptr(), ws.numel(), _stream()), "delta_attn_delta_scan")
    return mask, nnz, khat


def delta_attn_prefill(Q, K, V, theta: float, window: int, scale: float = 0.0, score_mode: int = DA_SCORE_GATHER,
                       cache: Optional[Cache] = None, workspace=None, out=None, window_mode: int = DA_WINDOW_BLOCK):
    """Returns (O, mask_bits int32 [B, Hkv, n, d/32], nnz int64 [B, Hkv]).  Buffers may be passed in
    (workspace: uint8 tensor, out: (O, mask_bits, nnz)) so a timing loop allocates nothing."""
    torch = _torch()
    for t, name in ((Q, "Q"), (K, "K"), (V, "V")):
        _dev(t, name)
    if K.shape != V.shape or Q.shape[0] != K.shape[0] or Q.shape[2:] != K.shape[2:] or Q.dtype != K.dtype \
            or K.dtype != V.dtype:
        raise ValueError("Q/K/V shapes or dtypes disagree")
    p = make_params(Q, K, window, theta, scale, score_mode, window_mode)
    need = delta_attn_prefill_workspace_bytes(p)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=Q.device)
    B, Hkv, n, d = K.shape
    if out is None:
        O = torch.empty_like(Q)
        mask = torch.empty((B, Hkv, n, d // 32), dtype=torch.int32, device=Q.device)
        nnz = torch.empty((B, Hkv), dtype=torch.int64, device=Q.device)
    else:
        O, mask, nnz = out
    st = lib().delta_attn_prefill(ctypes.byref(p), Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                  mask.data_ptr(), nnz.data_ptr(), None if cache is None else cache.handle,
                                  workspace.data_ptr(), workspace.numel(), _stream())
    _check(st, "delta_attn_prefill")
    return O, mask, nnz


NOALLOC_SCRATCH_BYTES = 32 << 20


def delta_attn_prefill_noalloc(Q, K, V, theta: float, window: int, out, scale: float = 0.0,
                               score_mode: int = DA_SCORE_GATHER, window_mode: int = DA_WINDOW_BLOCK):
    """delta_attn_prefill on the library's built-in scratch: the call allocates nothing, so `out` = (O, mask_bits int32
    [B, Hkv, n, d/32], nnz int64 [B, Hkv]) must be passed in.  Returns `out`."""
    for t, name in ((Q, "Q"), (K, "K"), (V, "V")) + tuple(zip(out, ("O", "mask_bits", "nnz"))):
        _dev(t, name)
    if K.shape != V.shape or Q.shape[0] != K.shape[0] or Q.shape[2:] != K.shape[2:] or Q.dtype != K.dtype \
            or K.dtype != V.dtype:
        raise ValueError("Q/K/V shapes or dtypes disagree")
    p = make_params(Q, K, window, theta, scale, score_mode, window_mode)
    O, mask, nnz = out
    st = lib().delta_attn_prefill_noalloc(ctypes.byref(p), Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                          mask.data_ptr(), nnz.data_ptr(), _stream())
    _check(st, "delta_attn_prefill_noalloc")
    return out


def delta_attn_prefill_append(cache: Cache, Q, K, V, theta: float, window: int, scale: float = 0.0,
                              score_mode: int = DA_SCORE_GATHER, window_mode: int = DA_WINDOW_BLOCK):
    """Chunked prefill: the rows of Q, K, V continue the sequence the cache holds.  Returns
    (O, mask_bits int32 [B, Hkv, m, d/32], nnz int64 [B, Hkv]) of the new rows; the cache is extended."""
    torch = _torch()
    for t, name in ((Q, "Q"), (K, "K"), (V, "V")):
        _dev(t, name)
    if K.shape != V.shape or Q.shape[0] != K.shape[0] or Q.shape[2:] != K.shape[2:] or Q.dtype != K.dtype \
            or K.dtype != V.dtype:
        raise ValueError("Q/K/V shapes or dtypes disagree")
    p = make_params(Q, K, window, theta, scale, score_mode, window_mode)
    need = int(lib().delta_attn_prefill_append_workspace_bytes(ctypes.byref(p), cache.handle))
    if need == 0:
        # let the call itself say why
        need = 1
    workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    B, Hkv, m, d = K.shape
    O = torch.empty_like(Q)
    mask = torch.empty((B, Hkv, m, d // 32), dtype=torch.int32, device=Q.device)
    nnz = torch.empty((B, Hkv), dtype=torch.int64, device=Q.device)
    st = lib().delta_attn_prefill_append(ctypes.byref(p), Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                         mask.data_ptr(), nnz.data_ptr(), cache.handle, workspace.data_ptr(),
                                         workspace.numel(), _stream())
    _check(st, "delta_attn_prefill_append")
    return O, mask, nnz


def delta_attn_decode(cache: Cache, q_new, k_new, v_new, out=None, mask_row=None):
    """One decode step.  q_new [B, Hq, d], k_new/v_new [B, Hkv, d].  Returns (o, mask_row)."""
    torch = _torch()
    for t, name in ((q_new, "q_new"), (k_new, "k_new"), (v_new, "v_new")):
        _dev(t, name)
    B, Hq, Hkv, d, _ = cache.shape
    if tuple(q_new.shape) != (B, Hq, d) or tuple(k_new.shape) != (B, Hkv, d) or tuple(v_new.shape) != (B, Hkv, d) \
            or q_new.dtype != cache.dtype or k_new.dtype != cache.dtype or v_new.dtype != cache.dtype:
        raise ValueError("decode tensors do not match the cache")
    if out is None:
        out = torch.empty_like(q_new)
    if mask_row is None:
        mask_row = torch.empty((B, Hkv, d // 32), dtype=torch.int32, device=q_new.device)
    st = lib().delta_attn_decode(cache.handle, q_new.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), out.data_ptr(),
                                 mask_row.data_ptr(), _stream())
    _check(st, "delta_attn_decode")
    return out, mask_row


def delta_attn_sparsity(nnz, rows: int, head_dim: int, window: int):
    """Eq. 6 from the device nnz counters [B, Hkv]; synchronises the stream.  Returns (s_m, s_c)."""
    _dev(nnz, "nnz")
    B, Hkv = nnz.shape
    s_m, s_c = ctypes.c_double(), ctypes.c_double()
    st = lib().delta_attn_sparsity(nnz.data_ptr(), B, Hkv, rows, head_dim, window, _stream(), ctypes.byref(s_m),
                                   ctypes.byref(s_c))
    _check(st, "delta_attn_sparsity")
    return s_m.value, s_c.value
