"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import numpy as np
import torch

from paper_2507_19608_amd import workloads as wl

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float64 array already on dtype's grid -> device tensor of that dtype (exact)."""
    return torch.from_numpy(np.ascontiguousarray(x)).to(TORCH_DTYPE[dtype]).cuda().contiguous()


def unpack_mask(bits: torch.Tensor, d: int) -> np.ndarray:
    """int32 words [..., d/32] -> uint8 [..., d] with bit (c % 32) of word c / 32 at channel c."""
    w = bits.cpu().numpy().view(np.uint32)
    sh = np.arange(32, dtype=np.uint32)
    out = ((w[..., None] >> sh) & 1).astype(np.uint8)
    return out.reshape(*w.shape[:-1], d)


def rand_walk(seed, B, H, n, d, dtype="bf16", step=0.15, clip=None):
    """Random-walk rows (temporally correlated like real keys).  `clip` bounds the magnitude: value
    tensors are kept below 4 so that rounding the output to bf16 (half an ulp = 2^-8 relative)
    stays well inside the absolute 2e-2 tolerance."""
    rng = np.random.default_rng(seed)
    x = np.cumsum(step * rng.standard_normal((B, H, n, d)), axis=2) + rng.standard_normal((B, H, 1, d))
    if clip is not None:
        x = np.clip(x, -clip, clip)
    return wl.round_to_dtype(x, dtype)


def check_output(o_gpu: torch.Tensor, o_ref: np.ndarray, dtype: str):
    """Tolerances of the benchmark spec: bf16 inputs -> max abs error <= 2e-2;
    fp32 inputs -> max abs error <= 1e-4 * max |reference| (relative to the tensor's scale)."""
    got = o_gpu.double().cpu().numpy()
    assert np.isfinite(got).all()
    err = np.abs(got - o_ref).max() if got.size else 0.0
    if dtype == "bf16":
        assert err <= 2e-2, f"max abs err {err}"
    else:
        ref = np.abs(o_ref).max()
        assert err <= 1e-4 * max(ref, 1e-30), f"max abs err {err} vs ref scale {ref}"
    return err
