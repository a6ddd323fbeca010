"""The C-ABI library loads and exports every symbol include/delta_attn.h declares; host-only
entry points and argument checks behave as documented.  No GPU compute here."""
import ctypes
import os
import re

import pytest

from paper_2507_19608_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "delta_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(delta_attn_\w+)\s*\(", text)))


# the boundary: the calls the method needs (prefill, decode, delta scan, sparsity, Eq. 5 window, cache life cycle,
# workspace sizes, status / error text) plus the documented extensions (chunked prefill, launch plan, stage timing for
# benchmarks, the entry point that allocates nothing)
BOUNDARY = sorted([
    "delta_attn_version", "delta_attn_status_string", "delta_attn_last_error",
    "delta_attn_window_from_gamma", "delta_attn_sparsity",
    "delta_attn_prefill_workspace_bytes", "delta_attn_prefill", "delta_attn_prefill_noalloc",
    "delta_attn_delta_scan_workspace_bytes", "delta_attn_delta_scan",
    "delta_attn_prefill_append_workspace_bytes", "delta_attn_prefill_append",
    "delta_attn_cache_create", "delta_attn_cache_destroy", "delta_attn_cache_reset", "delta_attn_cache_length",
    "delta_attn_cache_nnz", "delta_attn_cache_mask", "delta_attn_cache_set_launch_plan", "delta_attn_decode",
    "delta_attn_stage_timing_enable", "delta_attn_stage_timing_read",
])


def exported_symbols():
    """Dynamic symbols of the built library that carry the boundary's prefix (read with nm)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", binding.LIB_PATH], capture_output=True, text=True, check=True)
    return sorted({ln.split()[-1] for ln in out.stdout.splitlines() if ln.split()[-1].startswith("delta_attn_")})


def test_header_symbols_are_exported():
    names = declared_symbols()
    assert names == BOUNDARY
    L = binding.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names
    assert exported_symbols() == names          # nothing beyond the header leaves the library (no probes, no tools)


def test_host_only_entry_points():
    assert "gfx950" in binding.version()
    assert binding.status_string(0) == "ok"
    assert "workspace" in binding.status_string(3)
    # Eq. 5
    assert binding.delta_attn_window_from_gamma(100, 0.25, 1000) == 25
    assert binding.delta_attn_window_from_gamma(10, 0.25, 1000) == 2
    assert binding.delta_attn_window_from_gamma(1000, 0.05, 32) == 32
    assert binding.delta_attn_window_from_gamma(10, 0.05, 32) == 1


def _params(**kw):
    base = dict(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, seq_len=128, window=16, theta=0.1, scale=0.0,
                dtype=1, score_mode=0)
    base.update(kw)
    return binding.PrefillParams(**base)


def test_workspace_size_and_argument_checks():
    L = binding.lib()
    p = _params()
    need = binding.delta_attn_prefill_workspace_bytes(p)
    rows = 2 * 128
    assert need >= rows * 64 * 2 + rows * 64 * 8 + rows * 4
    for bad in (dict(n_q_heads=3), dict(window=0), dict(theta=-1.0), dict(theta=float("nan")), dict(seq_len=0),
                dict(head_dim=48), dict(head_dim=512), dict(dtype=7), dict(score_mode=5), dict(window_mode=2)):
        assert binding.delta_attn_prefill_workspace_bytes(_params(**bad)) == 0, bad
    # invalid arguments are rejected before anything touches the GPU
    st = L.delta_attn_prefill(ctypes.byref(_params(n_q_heads=3)), 1, 1, 1, 1, 1, 1, None, 1, 1 << 40, None)
    assert st == 1
    st = L.delta_attn_prefill(ctypes.byref(_params(head_dim=48)), 1, 1, 1, 1, 1, 1, None, 1, 1 << 40, None)
    assert st == 2
    st = L.delta_attn_prefill(ctypes.byref(p), None, 1, 1, 1, 1, 1, None, 1, 1 << 40, None)
    assert st == 1
    st = L.delta_attn_prefill(ctypes.byref(p), 1, 1, 1, 1, 1, 1, None, 256, need - 1, None)
    assert st == 3
    st = L.delta_attn_prefill(ctypes.byref(p), 1, 1, 1, 1, 1, 1, None, 256 + 64, need, None)   # not 256-byte aligned
    assert st == 3
    # the entry point that allocates nothing: same argument checks; a prompt beyond its built-in scratch is refused
    # with both sizes in the error text, before anything is enqueued
    assert L.delta_attn_prefill_noalloc(ctypes.byref(_params(n_q_heads=3)), 1, 1, 1, 1, 1, 1, None) == 1
    assert L.delta_attn_prefill_noalloc(ctypes.byref(p), None, 1, 1, 1, 1, 1, None) == 1
    big = _params(batch=4, n_q_heads=20, n_kv_heads=5, head_dim=128, seq_len=8192, window=512)
    assert binding.delta_attn_prefill_workspace_bytes(big) > binding.NOALLOC_SCRATCH_BYTES
    assert L.delta_attn_prefill_noalloc(ctypes.byref(big), 1, 1, 1, 1, 1, 1, None) == 3
    text = L.delta_attn_last_error().decode()
    assert str(binding.delta_attn_prefill_workspace_bytes(big)) in text and str(binding.NOALLOC_SCRATCH_BYTES) in text
    header = open(os.path.join(ROOT, "include", "delta_attn.h")).read()
    assert "#define DA_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)" in header and binding.NOALLOC_SCRATCH_BYTES == 32 << 20
    assert L.delta_attn_decode(None, 1, 1, 1, 1, None, None) == 1
    assert L.delta_attn_cache_length(None) == -1
    h = ctypes.c_void_p()
    assert L.delta_attn_cache_create(ctypes.byref(h), 1, 3, 2, 64, 128, 4, 0.1, 0.0, 1) == 1
    assert L.delta_attn_cache_create(ctypes.byref(h), 1, 4, 2, 48, 128, 4, 0.1, 0.0, 1) == 2


def test_binding_refuses_to_run_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        binding.delta_attn_prefill(torch.zeros(1, 1, 8, 32), torch.zeros(1, 1, 8, 32), torch.zeros(1, 1, 8, 32), 0.1, 4)
