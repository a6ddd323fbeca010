"""CPU pins of tests/dense_form.py, the second reference that the full-size GPU tests use.

dense_form evaluates the closed form of the method (outside scores q . k_hat(j), Eq. 4 telescoped; inside scores
q . k_j; Eq. 1 on top) with library tensor operations.  Here its three functions run on CPU tensors and are held
against the fp64 oracle (oracle/, which follows Eq. 2-4 step by step and is itself pinned by test_oracle_pins.py)
at small sizes: both window modes, grouped-query heads, ragged sizes, decode steps across the window edge.
No GPU and none of the HIP path is involved.
"""
import numpy as np
import pytest
import torch

import dense_form as df
from paper_2507_19608_amd import workloads as wl
from oracle import delta_oracle as orc


def _walk(seed, B, H, n, d, dtype="bf16", step=0.15):
    rng = np.random.default_rng(seed)
    x = np.cumsum(step * rng.standard_normal((B, H, n, d)), axis=2) + rng.standard_normal((B, H, 1, d))
    return wl.round_to_dtype(x, dtype)


def _t(x, dtype):
    return torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16 if dtype == "bf16" else torch.float32)


@pytest.mark.parametrize("dtype,theta", [("bf16", 0.0), ("bf16", 0.11), ("bf16", 0.4), ("f32", 0.07), ("bf16", float("inf"))])
def test_reference_keys_equal_the_oracles_scan(dtype, theta):
    """Eq. 2-3: masks and reference keys of every unit equal the oracle's, bit for bit (binary32 decision, strict >)."""
    B, Hkv, n, d = 2, 3, 150, 32
    K = _walk(1, B, Hkv, n, d, dtype)
    khat, mask = df.reference_keys(_t(K, dtype), theta)
    assert khat.dtype == torch.float64 and mask.dtype == torch.bool
    for b in range(B):
        for h in range(Hkv):
            m, _, kh, _ = orc.delta_scan(K[b, h], theta)
            assert (mask[b, h].numpy() == m.astype(bool)).all()
            assert (khat[b, h].numpy() == kh).all()


def test_reference_keys_strict_inequality_and_basis_row():
    """A difference equal to theta does not fire; the first row is kept whole even where it is below theta."""
    K = torch.tensor([[[[0.25], [0.75], [1.25], [1.25 + 2 ** -7]]]], dtype=torch.bfloat16)
    khat, mask = df.reference_keys(K, 0.5)
    assert mask.ravel().tolist() == [True, False, True, False]
    assert khat.ravel().tolist() == [0.25, 0.25, 1.25, 1.25]


def test_unpack_bits_bit_order():
    """Bit (c % 32) of word c / 32 is channel c; the sign bit of an int32 word is channel 31."""
    bits = torch.tensor([[1, 2], [-2 ** 31, 5]], dtype=torch.int32)
    got = df.unpack_bits(bits, 64)
    want = torch.zeros(2, 64, dtype=torch.bool)
    want[0, 0] = want[0, 33] = want[1, 31] = want[1, 32] = want[1, 34] = True
    assert torch.equal(got, want)


@pytest.mark.parametrize("sliding", [False, True])
@pytest.mark.parametrize("n,d,W,B,Hq,Hkv,theta", [(70, 32, 8, 2, 4, 2, 0.2), (45, 64, 7, 1, 6, 2, 0.1),
                                                  (33, 32, 1, 1, 2, 2, 0.3), (40, 32, 100, 1, 2, 1, 0.2)])
def test_prefill_reference_equals_the_oracle(sliding, n, d, W, B, Hq, Hkv, theta):
    """prefill_worst_error's reference is the oracle's output: feeding it the oracle's own output must give an error
    at rounding level (the oracle sums Eq. 4 column by column, dense_form takes q . k_hat: telescoping), and an output
    that is off by 1e-3 in one element must be seen.  Square windows and bands, grouped-query heads, a ragged last
    square, W = 1, a window that covers the prompt."""
    Q, K, V = _walk(2, B, Hq, n, d), _walk(3, B, Hkv, n, d), _walk(4, B, Hkv, n, d)
    ref = orc.prefill(Q, K, V, theta, W, window_mode=int(sliding))
    Qt, Kt, Vt = _t(Q, "bf16"), _t(K, "bf16"), _t(V, "bf16")
    khat, mask = df.reference_keys(Kt, theta)
    assert (mask.numpy().astype(np.uint8) == ref["mask"]).all()
    O = torch.from_numpy(ref["O"])
    assert df.prefill_worst_error(Qt, Kt, Vt, khat, W, sliding, [O], row_block=16) <= 1e-12
    bad = O.clone()
    bad[B - 1, Hq - 1, n - 1, d - 1] += 1e-3
    err = df.prefill_worst_error(Qt, Kt, Vt, khat, W, sliding, [O, bad], row_block=16)
    assert 0.999e-3 <= err <= 1.001e-3
    # the other window shape is a different function (unless the window covers everything)
    if W < n and W > 1:
        assert df.prefill_worst_error(Qt, Kt, Vt, khat, W, not sliding, [O], row_block=16) > 1e-6


@pytest.mark.parametrize("d,Hq,Hkv,Wd,theta", [(32, 4, 2, 5, 0.2), (64, 6, 2, 1, 0.1), (32, 2, 2, 64, 0.3)])
def test_decode_reference_equals_the_oracles_decode_workflow(d, Hq, Hkv, Wd, theta):
    """decode_reference at position t against oracle.DecodeState stepping through the same sequence (Sec. III-C):
    from an empty cache, across the step where keys first leave the decode window."""
    B, L = 2, 24
    Q, K, V = _walk(5, B, Hq, L, d), _walk(6, B, Hkv, L, d), _walk(7, B, Hkv, L, d)
    Qt, Kt, Vt = _t(Q, "bf16"), _t(K, "bf16"), _t(V, "bf16")
    khat, _ = df.reference_keys(Kt, theta)
    st = orc.DecodeState(theta, Wd)
    for t in range(L):
        o_ref, _ = st.step(Q[:, :, t], K[:, :, t], V[:, :, t])
        got = df.decode_reference(Qt[:, :, t], Kt.double(), Vt.double(), khat, t, Wd)
        assert np.abs(got.numpy() - o_ref).max() <= 1e-12, t
