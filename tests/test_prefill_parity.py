"""GPU parity: delta_attn_prefill / delta_attn_delta_scan (through the C ABI) against the fp64
oracle on the same seeded inputs.  Masks and nnz bit-exact; outputs within the stated tolerance."""
import numpy as np
import pytest
import torch

from paper_2507_19608_amd import binding as da
from paper_2507_19608_amd import workloads as wl
from oracle import delta_oracle as orc
from util import check_output, rand_walk, to_dev, unpack_mask

pytestmark = pytest.mark.gpu

MODES = [da.DA_SCORE_GATHER, da.DA_SCORE_REBASE]


def run_case(Q, K, V, theta, W, dtype, mode, rows=None, q_heads=None, scale=0.0, window_mode=0):
    d = Q.shape[-1]
    Og, maskg, nnzg = da.delta_attn_prefill(to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype), theta, W,
                                            scale=scale, score_mode=mode, window_mode=window_mode)
    torch.cuda.synchronize()
    ref = orc.prefill(Q, K, V, theta, W, scale=None if scale == 0.0 else scale, rows=rows, q_heads=q_heads,
                      window_mode=window_mode)
    assert ref["knife"] == 0
    assert (unpack_mask(maskg, d) == ref["mask"]).all()
    assert (nnzg.cpu().numpy() == ref["nnz"]).all()
    s_m, s_c = da.delta_attn_sparsity(nnzg, K.shape[2], d, W)
    assert s_m == ref["s_m"] and s_c == pytest.approx(ref["s_c"], abs=1e-15)
    r0, r1 = (0, Q.shape[2]) if rows is None else rows
    heads = range(Q.shape[1]) if q_heads is None else q_heads
    errs = [check_output(Og[:, h, r0:r1], ref["O"][:, h], dtype) for h in heads]
    return max(errs)


@pytest.mark.parametrize("mode", MODES)
def test_c1_fp32_single_head(mode):
    x = wl.generate(wl.C1)
    w = wl.C1
    run_case(x["Q"], x["K"], x["V"], wl.theta_for(w), w.window, w.dtype, mode)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n,d,W,B,Hq,Hkv,theta", [
    (333, 64, 32, 2, 4, 2, 0.2),     # several tiles, ragged tail, windows smaller than a tile
    (200, 128, 64, 1, 4, 1, 0.15),
    (257, 32, 7, 1, 2, 2, 0.3),      # odd window, tile spans many squares
    (130, 96, 1, 1, 3, 1, 0.25),     # W = 1 (the paper's illustration), head_dim 96
    (190, 64, 128, 1, 8, 2, 0.2),    # truncated last square
    (64, 256, 16, 1, 1, 1, 0.2),     # largest head_dim
])
def test_small_shapes_bf16(mode, n, d, W, B, Hq, Hkv, theta):
    Q = rand_walk(1, B, Hq, n, d)
    K = rand_walk(2, B, Hkv, n, d)
    V = rand_walk(3, B, Hkv, n, d, clip=3.5)
    run_case(Q, K, V, theta, W, "bf16", mode)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n,d,W,B,Hq,Hkv,theta,dtype", [
    (333, 64, 48, 2, 4, 2, 0.2, "bf16"),     # band narrower than a row tile, ragged tail
    (200, 128, 5, 1, 4, 1, 0.15, "bf16"),    # the paper's small windows
    (300, 64, 64, 1, 8, 1, 0.2, "bf16"),     # band = one key block
    (260, 128, 1, 1, 2, 2, 0.25, "bf16"),    # W = 1: only the diagonal is exact
    (150, 64, 1000, 1, 2, 1, 0.3, "bf16"),   # band covers everything: dense attention
    (130, 96, 10, 1, 3, 1, 0.25, "bf16"),    # vector-ALU kernel
    (120, 32, 7, 1, 1, 1, 0.05, "f32"),
])
def test_sliding_window_prefill(mode, n, d, W, B, Hq, Hkv, theta, dtype):
    """The band reading of the prefill window (DA_WINDOW_SLIDING) against the oracle's."""
    step = 0.05 if dtype == "f32" else 0.15
    Q = rand_walk(51, B, Hq, n, d, dtype)
    K = rand_walk(52, B, Hkv, n, d, dtype, step)
    V = rand_walk(53, B, Hkv, n, d, dtype, clip=3.5)
    run_case(Q, K, V, theta, W, dtype, mode, window_mode=da.DA_WINDOW_SLIDING)


@pytest.mark.parametrize("mode", MODES)
def test_sliding_prefill_rows_equal_decode_steps(mode):
    """Two separate GPU paths, one definition: row t of a sliding-window prefill is the decode step at
    position t with decode_window W (Sec. III-B decode stage); both within tolerance of the oracle,
    hence within twice the tolerance of each other, at every position."""
    B, Hq, Hkv, n, d, W, theta = 1, 4, 1, 230, 64, 64, 0.2
    Q, K, V = rand_walk(61, B, Hq, n, d), rand_walk(62, B, Hkv, n, d), rand_walk(63, B, Hkv, n, d, clip=3.5)
    Qd, Kd, Vd = (to_dev(x, "bf16") for x in (Q, K, V))
    O, _, _ = da.delta_attn_prefill(Qd, Kd, Vd, theta, W, score_mode=mode, window_mode=da.DA_WINDOW_SLIDING)
    cache = da.Cache(B, Hq, Hkv, d, n, W, theta, torch.bfloat16)
    for t in range(n):
        o, _ = da.delta_attn_decode(cache, Qd[:, :, t].contiguous(), Kd[:, :, t].contiguous(), Vd[:, :, t].contiguous())
        assert (o.float() - O[:, :, t].float()).abs().max().item() <= 4e-2, t
    cache.close()


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n,d,W,theta", [(300, 64, 32, 0.1), (150, 128, 50, 0.05)])
def test_small_shapes_fp32(mode, n, d, W, theta):
    Q = rand_walk(4, 1, 2, n, d, "f32")
    K = rand_walk(5, 1, 1, n, d, "f32", step=0.05)
    V = rand_walk(6, 1, 1, n, d, "f32", clip=3.5)
    run_case(Q, K, V, theta, W, "f32", mode, scale=0.2)


@pytest.mark.parametrize("mode", MODES)
def test_degenerate_cases(mode):
    B, Hq, Hkv, n, d = 1, 2, 1, 150, 64
    Q, K, V = rand_walk(7, B, Hq, n, d), rand_walk(8, B, Hkv, n, d), rand_walk(9, B, Hkv, n, d, clip=3.5)
    run_case(Q, K, V, 0.0, 16, "bf16", mode)                 # theta = 0: dense attention
    run_case(Q, K, V, 0.3, n, "bf16", mode)                  # window covers the sequence
    run_case(Q, K, V, 0.3, 100000, "bf16", mode)
    run_case(Q, K, V, float("inf"), 16, "bf16", mode)        # nothing fires after the basis
    Kc = np.tile(K[:, :, :1], (1, 1, n, 1))                   # constant keys
    run_case(Q, Kc, V, 0.2, 16, "bf16", mode)
    Kall = wl.round_to_dtype(np.cumsum(np.ones((B, Hkv, n, d)), axis=2) * 0.015, "bf16")  # every entry fires
    run_case(wl.round_to_dtype(Q * 0.05, "bf16"), Kall, V, 0.005, 16, "bf16", mode)
    run_case(Q[:, :, :1], K[:, :, :1], V[:, :, :1], 0.2, 4, "bf16", mode)   # a single token


@pytest.mark.parametrize("mode", MODES)
def test_c2_llama_shape_full(mode):
    w = wl.C2
    x = wl.generate(w)
    run_case(x["Q"], x["K"], x["V"], wl.theta_for(w), w.window, w.dtype, mode)


_generated = {}


def _inputs(w):
    """Inputs of a workload, kept for the other parametrisations of the same test (one workload at a time)."""
    if w not in _generated:
        _generated.clear()
        _generated[w] = wl.generate(w)
    return _generated[w]


def _sampled(w, mode, row_ranges, heads, window_mode=0):
    x = _inputs(w)
    d = w.head_dim
    Qd, Kd, Vd = (to_dev(x[k], w.dtype) for k in "QKV")
    theta = wl.theta_for(w)
    Og, maskg, nnzg = da.delta_attn_prefill(Qd, Kd, Vd, theta, w.window, score_mode=mode, window_mode=window_mode)
    torch.cuda.synchronize()
    first = True
    for rows in row_ranges:
        ref = orc.prefill(x["Q"], x["K"], x["V"], theta, w.window, rows=rows, q_heads=heads, window_mode=window_mode)
        if first:   # masks of every unit, all rows
            assert (unpack_mask(maskg, d) == ref["mask"]).all()
            assert (nnzg.cpu().numpy() == ref["nnz"]).all()
            s_m, _ = da.delta_attn_sparsity(nnzg, w.seq_len, d, w.window)
            assert s_m == ref["s_m"]
            first = False
        for h in heads:
            check_output(Og[:, h, rows[0]:rows[1]], ref["O"][:, h], w.dtype)


@pytest.mark.parametrize("mode", MODES)
def test_c3_bitnet_shape_sampled(mode):
    _sampled(wl.C3, mode, [(0, 40), (2030, 2070), (4064, 4096)], [0, 7, 19])


@pytest.mark.parametrize("mode", MODES)
def test_c3_sliding_window_sampled(mode):
    _sampled(wl.C3, mode, [(200, 230), (2040, 2060), (4070, 4096)], [1, 18], window_mode=da.DA_WINDOW_SLIDING)


def test_mid_size_launch_cut_in_two_sampled():
    """4 x 4096 tokens of C5's head shape with the window of Eq. 5 (W = 204: tiles straddle window squares): 1280 row
    tiles, five per compute unit - few enough that the gather launch gives every tile two work groups, each on half of
    its gather blocks, and merges them in a second launch.  Masks and nnz of every unit, sampled output rows."""
    import dataclasses
    w = dataclasses.replace(wl.C5, seq_len=4096, window=da.delta_attn_window_from_gamma(4096, 0.05, 512),
                            theta=wl.theta_for(wl.C5), target_sparsity=None)
    assert w.window == 204
    _sampled(w, da.DA_SCORE_GATHER, [(1000, 1020), (2600, 2615), (4076, 4096)], [2, 17])


@pytest.mark.parametrize("mode", MODES)
def test_c5_long_context_sampled(mode):
    _sampled(wl.C5, mode, [(500, 530), (4090, 4110), (8170, 8192)], [3, 16])


def test_c5_every_output_element():
    """The benchmark's launch at full size, every output element (the sampled rows above are checked against the
    oracle): the same bits on a second run; finite; inside the per-channel range of the value rows its query row may mix (Eq. 1: a weighted mean
    with weights that sum to one, whatever the approximate scores are), up to the rounding of the output; and the
    two score modes, each within 2e-2 of the oracle, within 4e-2 of each other everywhere."""
    w = wl.C5
    x = _inputs(w)
    Qd, Kd, Vd = (to_dev(x[k], w.dtype) for k in "QKV")
    theta = wl.theta_for(w)
    outs = []
    for mode in MODES:
        O, bits, nnz = da.delta_attn_prefill(Qd, Kd, Vd, theta, w.window, score_mode=mode)
        O2, bits2, nnz2 = da.delta_attn_prefill(Qd, Kd, Vd, theta, w.window, score_mode=mode)
        assert torch.equal(O, O2) and torch.equal(bits, bits2) and torch.equal(nnz, nnz2)   # bitwise reproducible
        outs.append(O)
    torch.cuda.synchronize()
    g = w.n_q_heads // w.n_kv_heads
    Vf = Vd.float()
    lo = torch.cummin(Vf, dim=2).values.repeat_interleave(g, dim=1)
    hi = torch.cummax(Vf, dim=2).values.repeat_interleave(g, dim=1)
    tol = 2.0 ** -8 * Vf.abs().max().item()                  # bf16 rounding of an output of that size
    for O in outs:
        Of = O.float()
        assert torch.isfinite(Of).all()
        assert (Of >= lo - tol).all() and (Of <= hi + tol).all()
    assert (outs[0].float() - outs[1].float()).abs().max().item() <= 4e-2


@pytest.mark.parametrize("how", ["one call", "sliding window", "four pieces onto a cache", "theta 0",
                                 "80 % sparsity, 20 % jumps"])
def test_c5_every_output_element_against_the_dense_form(how):
    """Every output element of the benchmark's launch against the closed form the oracle is pinned to: outside a
    row's window (square, or band) the Eq. 4 score is q . k_hat(j) (the deltas up to column j sum to the held key),
    inside it q . k_j; Eq. 1 on top.  Evaluated head by head with library matrix products in fp64 on the device
    (tests/dense_form.py, pinned to the oracle on the CPU).  The reference keys and the delta mask are worked out from
    the inputs alone (Eq. 2-3 written out with tensor operations); the masks and nnz that the library returns, in
    either score mode, must equal them bit for bit, and two units of them are also held against the oracle's scan.
    Tolerance as for the oracle.
    Also for the prompt fed in four pieces through the chunked entry point, as `bench.py --chunks 4` times it, and
    at the two ends of the sparsity sweep (every delta kept: the longest entry lists; 80 % zeroed with bursts)."""
    import dense_form as df
    w = wl.c5(0.0, 0.05) if how == "theta 0" else wl.c5(0.80, 0.20) if how.startswith("80") else wl.C5
    x = _inputs(w)
    Qd, Kd, Vd = (to_dev(x[k], w.dtype) for k in "QKV")
    theta, n, d, W = wl.theta_for(w), w.seq_len, w.head_dim, w.window
    sliding = how == "sliding window"
    if how == "four pieces onto a cache":
        outs = []
        for mode in MODES:
            cache = da.Cache(w.batch, w.n_q_heads, w.n_kv_heads, d, n, W, theta, torch.bfloat16)
            parts = [da.delta_attn_prefill_append(cache, Qd[:, :, a:a + n // 4].contiguous(),
                                                  Kd[:, :, a:a + n // 4].contiguous(),
                                                  Vd[:, :, a:a + n // 4].contiguous(), theta, W, score_mode=mode)
                     for a in range(0, n, n // 4)]
            outs.append(tuple(torch.cat([p[k] for p in parts], dim=2) for k in range(2)) + (cache.nnz().clone(),))
            cache.close()
    else:
        outs = [da.delta_attn_prefill(Qd, Kd, Vd, theta, W, score_mode=mode,
                                      window_mode=da.DA_WINDOW_SLIDING if sliding else da.DA_WINDOW_BLOCK)
                for mode in MODES]
    torch.cuda.synchronize()
    khat, mask = df.reference_keys(Kd, theta)                # from the inputs, not from the library's output
    for b, hk in ((0, 0), (w.batch - 1, w.n_kv_heads - 1)):
        m, _, kh, knife = orc.delta_scan(x["K"][b, hk], theta)
        assert knife == 0
        assert (mask[b, hk].cpu().numpy() == m.astype(bool)).all() and (khat[b, hk].cpu().numpy() == kh).all()
    for O, bits, nnz in outs:
        assert (df.unpack_bits(bits, d) == mask).all()
        assert (nnz == mask.sum(dim=(2, 3))).all()
    worst = df.prefill_worst_error(Qd, Kd, Vd, khat, W, sliding, [o[0] for o in outs])
    assert worst <= 2e-2, worst


@pytest.mark.parametrize("dtype,d,n,W", [("f32", 64, 1536, 96), ("f32", 256, 700, 33), ("bf16", 96, 2048, 128),
                                         ("bf16", 32, 3000, 7)])
def test_generic_kernel_every_output_element_against_the_dense_form(dtype, d, n, W):
    """The vector-ALU kernel (fp32 inputs; head sizes other than 64 / 128) at sizes of a few thousand rows, every
    output element of both score modes and both window modes against the same closed form in fp64."""
    import dense_form as df
    B, Hq, Hkv, theta = 2, 6, 2, 0.12
    Q, K, V = rand_walk(71, B, Hq, n, d, dtype), rand_walk(72, B, Hkv, n, d, dtype), rand_walk(73, B, Hkv, n, d, dtype, clip=3.5)
    Qd, Kd, Vd = to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype)
    rows = torch.arange(n, device="cuda")
    causal = rows[None, :] <= rows[:, None]
    sh = torch.arange(32, device="cuda", dtype=torch.int32)
    for window_mode in (da.DA_WINDOW_BLOCK, da.DA_WINDOW_SLIDING):
        outs = [da.delta_attn_prefill(Qd, Kd, Vd, theta, W, score_mode=mode, window_mode=window_mode) for mode in MODES]
        torch.cuda.synchronize()
        _, mask = df.reference_keys(Kd, theta)               # from the inputs; the library's masks must equal it
        for _, bits, _ in outs:
            assert (df.unpack_bits(bits, d) == mask).all()
        assert (mask.cpu().numpy() == np.stack([[orc.delta_scan(K[b, h], theta)[0] for h in range(Hkv)]
                                                for b in range(B)]).astype(bool)).all()
        inside = (rows[:, None] - rows[None, :] < W) if window_mode == da.DA_WINDOW_SLIDING \
            else (rows[:, None] // W == rows[None, :] // W)
        for b in range(B):
            for h in range(Hq):
                hk = h // (Hq // Hkv)
                Kx, Vx, Qx = Kd[b, hk].double(), Vd[b, hk].double(), Qd[b, h].double()
                last = torch.where(mask[b, hk], rows[:, None], torch.zeros_like(rows[:, None])).cummax(dim=0).values
                S = torch.where(inside, Qx @ Kx.T, Qx @ torch.gather(Kx, 0, last).T) / d ** 0.5
                ref = torch.softmax(S.masked_fill(~causal, float("-inf")), dim=-1) @ Vx
                for O, _, _ in outs:
                    check_output(O[b, h], ref.cpu().numpy(), dtype)


@pytest.mark.parametrize("seed", range(12))
def test_random_mid_size_shapes_against_the_dense_form(seed):
    """Seeded random shapes of 700-4100 rows (head sizes 64 / 128, group sizes 1-8, windows 1-1024, both window
    modes, one call or 2-5 ragged pieces through the chunked entry point): masks equal Eq. 2-3 written out with
    tensor operations, every output element of both score modes within tolerance of the dense form."""
    import random
    import dense_form as df
    rng = random.Random(1000 + seed)
    d, Hkv, g, B = rng.choice([64, 128]), rng.choice([1, 2, 3]), rng.choice([1, 2, 3, 4, 6, 8]), rng.choice([1, 2])
    n = rng.choice([700, 1024, 1500, 2048, 2500, 3000, 4096]) + rng.choice([0, 0, 1, 31, 33])
    W = rng.choice([1, 5, 32, 64, 100, 128, 256, 300, 512, 1024])
    theta, wm, pieces = rng.choice([0.0, 0.05, 0.11, 0.2, 0.5]), rng.choice([0, 1]), rng.choice([1, 1, 2, 3, 5])
    Hq = Hkv * g
    Qd, Kd, Vd = (to_dev(rand_walk(5000 + 3 * seed + k, B, H, n, d, clip=c), "bf16")
                  for k, (H, c) in enumerate(((Hq, None), (Hkv, None), (Hkv, 3.5))))
    outs = []
    for mode in MODES:
        if pieces == 1:
            O, bits, _ = da.delta_attn_prefill(Qd, Kd, Vd, theta, W, score_mode=mode, window_mode=wm)
        else:
            cache = da.Cache(B, Hq, Hkv, d, n, max(64, min(W, n)), theta, torch.bfloat16)
            cuts = sorted(set([0, n] + [rng.randrange(1, n) for _ in range(pieces - 1)]))
            parts = [da.delta_attn_prefill_append(cache, Qd[:, :, a:b].contiguous(), Kd[:, :, a:b].contiguous(),
                                                  Vd[:, :, a:b].contiguous(), theta, W, score_mode=mode, window_mode=wm)
                     for a, b in zip(cuts[:-1], cuts[1:])]
            O, bits = (torch.cat([p[k] for p in parts], dim=2) for k in range(2))
            cache.close()
        outs.append(O)
        khat, mask = df.reference_keys(Kd, theta)
        assert (df.unpack_bits(bits, d) == mask).all()
    assert df.prefill_worst_error(Qd, Kd, Vd, khat, W, wm == 1, outs) <= 2e-2


@pytest.mark.parametrize("window_mode,pieces", [(da.DA_WINDOW_BLOCK, 1), (da.DA_WINDOW_SLIDING, 1),
                                                (da.DA_WINDOW_BLOCK, 8), (da.DA_WINDOW_SLIDING, 5)])
def test_64k_tokens_every_output_element_against_the_dense_form(window_mode, pieces):
    """The 65536-token prompt of the test below, every output element of both score modes against the same closed
    form, 2048 query rows at a time (reference keys and mask from the inputs; the library's masks must equal them, and
    they equal the oracle's scan) - in one call, and fed in equal pieces through the chunked entry point (the last
    pieces continue a cache of more than 50 000 rows)."""
    w = wl.Workload("L64K", 1, 4, 1, 128, 65536, 512, "bf16", seed=64, theta=0.11)
    x = _inputs(w)
    Qd, Kd, Vd = (to_dev(x[k], w.dtype) for k in "QKV")
    n, d, W = w.seq_len, w.head_dim, w.window
    if pieces == 1:
        outs = [da.delta_attn_prefill(Qd, Kd, Vd, w.theta, W, score_mode=mode, window_mode=window_mode)
                for mode in MODES]
    else:
        outs = []
        cuts = [n * k // pieces for k in range(pieces + 1)]
        for mode in MODES:
            cache = da.Cache(1, 4, 1, d, n, W, w.theta, torch.bfloat16)
            parts = [da.delta_attn_prefill_append(cache, Qd[:, :, a:b].contiguous(), Kd[:, :, a:b].contiguous(),
                                                  Vd[:, :, a:b].contiguous(), w.theta, W, score_mode=mode,
                                                  window_mode=window_mode) for a, b in zip(cuts[:-1], cuts[1:])]
            outs.append(tuple(torch.cat([p[k] for p in parts], dim=2) for k in range(2)) + (None,))
            cache.close()
    torch.cuda.synchronize()
    import dense_form as df
    khat, mask = df.reference_keys(Kd, w.theta)              # from the inputs; the library's masks must equal it
    m, _, kh, knife = orc.delta_scan(x["K"][0, 0], w.theta)
    assert knife == 0 and (mask[0, 0].cpu().numpy() == m.astype(bool)).all() and (khat[0, 0].cpu().numpy() == kh).all()
    for _, bits, _ in outs:
        assert (df.unpack_bits(bits, d) == mask).all()
    worst = df.prefill_worst_error(Qd, Kd, Vd, khat, W, window_mode == da.DA_WINDOW_SLIDING, [o[0] for o in outs])
    assert worst <= 2e-2, worst


def test_two_to_the_31_query_elements():
    """Maximum sizes: batch 4, 32 / 8 heads of 128, 131072 tokens - Q and O hold 2^31 elements each (4 GiB), so element
    offsets leave 32 bits and byte offsets 33; the running Eq. 4 score of a late row is a sum over 130 000 columns.
    Inputs are drawn on the device (random walks like the workloads'); the masks of three units and 1024-row blocks at
    the start, middle and end of three heads (the last head of the last batch entry among them) are compared with
    the oracle's Eq. 2-3 and the dense form in fp64, in both score modes."""
    import dense_form as df
    B, Hq, Hkv, n, d, W, theta = 4, 32, 8, 131072, 128, 512, 0.11
    gen = torch.Generator(device="cuda").manual_seed(31)

    def walk(H, clip=None):
        x = torch.cumsum(0.15 * torch.randn(B, H, n, d, device="cuda", generator=gen), dim=2)
        x += torch.randn(B, H, 1, d, device="cuda", generator=gen)
        return (x.clamp(-clip, clip) if clip else x).to(torch.bfloat16)

    Qd, Kd, Vd = walk(Hq), walk(Hkv), walk(Hkv, 3.5)
    assert Qd.numel() == 2 ** 31
    rows = torch.arange(n, device="cuda")
    heads = ((B - 1, Hq - 1), (0, 0), (2, 17))
    scans = {}                                                # Eq. 2-3 of the three units, from the oracle
    for b, h in heads:
        m, _, kh, knife = orc.delta_scan(Kd[b, h // (Hq // Hkv)].double().cpu().numpy(), theta)
        assert knife == 0
        scans[b, h] = (torch.from_numpy(m).cuda().bool(), torch.from_numpy(kh).cuda())
    for mode in MODES:
        O, bits, _ = da.delta_attn_prefill(Qd, Kd, Vd, theta, W, score_mode=mode)
        for b, h in heads:
            hk = h // (Hq // Hkv)
            mask, khat = scans[b, h]
            assert (df.unpack_bits(bits[b, hk], d) == mask).all()
            for r0 in (0, n // 2 - 512, n - 1024):
                r1 = r0 + 1024
                i, j = rows[r0:r1, None], rows[None, :r1]
                K, V, H = Kd[b, hk, :r1].double(), Vd[b, hk, :r1].double(), khat[:r1]
                Q = Qd[b, h, r0:r1].double()
                S = torch.where(i // W == j // W, Q @ K.T, Q @ H.T) / d ** 0.5
                ref = torch.softmax(S.masked_fill(j > i, float("-inf")), dim=-1) @ V
                assert (O[b, h, r0:r1].double() - ref).abs().max().item() <= 2e-2
        del O, bits


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("window_mode", [da.DA_WINDOW_BLOCK, da.DA_WINDOW_SLIDING])
def test_64k_tokens_sampled(mode, window_mode):
    """A prompt of 65536 tokens (one KV head, four query heads, C5's head size and window): the running
    Eq. 4 score of a late row is a sum over 65 000 columns, the softmax runs over as many keys."""
    w = wl.Workload("L64K", 1, 4, 1, 128, 65536, 512, "bf16", seed=64, theta=0.11)
    _sampled(w, mode, [(0, 8), (32760, 32776), (65528, 65536)], [0, 3], window_mode=window_mode)


@pytest.mark.parametrize("dtype,n,d", [("bf16", 8192, 128), ("bf16", 30000, 64), ("f32", 5000, 96), ("bf16", 1000, 256)])
def test_delta_scan_every_reference_key(dtype, n, d):
    """delta_attn_delta_scan with its k_hat output at sizes of many time chunks: masks, nnz and every reference key
    (Eq. 3) equal Eq. 2-3 written out row by row with tensor operations (binary32 decision), for thresholds from
    dense to frozen; two units also against the oracle."""
    import dense_form as df
    B, Hkv = 3, 4
    Kd = to_dev(rand_walk(11, B, Hkv, n, d, dtype), dtype)
    for theta in (0.0, 0.05, 0.2, 3.0):
        bits, nnz, khat = da.delta_attn_delta_scan(Kd, theta, want_khat=True)
        ref_khat, ref_mask = df.reference_keys(Kd, theta)
        assert (df.unpack_bits(bits, d) == ref_mask).all()
        assert (nnz == ref_mask.sum(dim=(2, 3))).all()
        assert (khat.double() == ref_khat).all()
        for b, hk in ((0, 0), (B - 1, Hkv - 1)):
            m, _, kh, _ = orc.delta_scan(Kd[b, hk].double().cpu().numpy(), theta)
            assert (ref_mask[b, hk].cpu().numpy() == m).all() and (ref_khat[b, hk].cpu().numpy() == kh).all()


_sweep_inputs = {}


@pytest.mark.parametrize("w", wl.C5_SWEEP, ids=lambda w: w.key())
def test_c5_sweep_point_masks_sparsity_and_outputs(w):
    """Config 5 is a family: threshold in {0, theta_40, theta_60, theta_80} x jump rate in {1, 5, 20} %.  At every one
    of the 12 points, at full size and in both score modes: the delta masks and nnz of all 20 (batch, KV head) units
    equal the oracle's Eq. 2-3 scan bit for bit, S_m equals the oracle's, and three row ranges (start, middle, end
    of the prompt; the middle one straddles a window square's edge) of two query heads match the oracle's outputs
    within the bf16 tolerance."""
    key = (w.seed, w.p_jump)                                  # the inputs depend on the jump rate, not on the threshold
    if key not in _sweep_inputs:
        _sweep_inputs.clear()
        _sweep_inputs[key] = wl.generate(w)
    x = _sweep_inputs[key]
    theta, d = wl.theta_for(w), w.head_dim
    Qd, Kd, Vd = (to_dev(x[k], w.dtype) for k in "QKV")
    heads, row_ranges = [2, 17], [(0, 24), (4084, 4108), (8176, 8192)]
    refs = [orc.prefill(x["Q"], x["K"], x["V"], theta, w.window, rows=rows, q_heads=heads) for rows in row_ranges]
    assert refs[0]["knife"] == 0
    for mode in MODES:
        Og, maskg, nnzg = da.delta_attn_prefill(Qd, Kd, Vd, theta, w.window, score_mode=mode)
        torch.cuda.synchronize()
        assert (unpack_mask(maskg, d) == refs[0]["mask"]).all()          # all 20 units, all 8192 rows
        assert (nnzg.cpu().numpy() == refs[0]["nnz"]).all()
        s_m, s_c = da.delta_attn_sparsity(nnzg, w.seq_len, d, w.window)
        assert s_m == refs[0]["s_m"] and s_c == pytest.approx(refs[0]["s_c"], abs=1e-15)
        if w.target_sparsity:
            assert abs(s_m - w.target_sparsity) < 0.015
        for rows, ref in zip(row_ranges, refs):
            for h in heads:
                check_output(Og[:, h, rows[0]:rows[1]], ref["O"][:, h], w.dtype)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n,d,W,Hq,Hkv", [(700, 128, 64, 4, 1), (450, 64, 32, 4, 2)])
def test_values_up_to_eight(mode, n, d, W, Hq, Hkv):
    """Value rows that are not clipped to |v| < 4 (the other random cases clip them so that the bf16 rounding of the
    output alone, half an ulp = 2^-9 relative to the next power of two below |o|, stays well inside 2e-2).  Here |v|
    reaches 8 and outputs pass 4, where half an ulp is 2^-6 = 0.0156: the absolute 2e-2 is kept for |o| <= 4 and scaled
    with the output's bf16 grid above it - per element, |error| <= 2e-2 * max(1, |o| / 4) - which is the same
    5e-3 relative bound that 2e-2 is at |o| = 4."""
    Q, K = rand_walk(101, 2, Hq, n, d), rand_walk(102, 2, Hkv, n, d)
    V = rand_walk(103, 2, Hkv, n, d, step=0.5, clip=8.0)
    assert np.abs(V).max() == 8.0
    theta = 0.15
    Og, maskg, nnzg = da.delta_attn_prefill(to_dev(Q, "bf16"), to_dev(K, "bf16"), to_dev(V, "bf16"), theta, W,
                                            score_mode=mode)
    torch.cuda.synchronize()
    ref = orc.prefill(Q, K, V, theta, W)
    assert (unpack_mask(maskg, d) == ref["mask"]).all() and (nnzg.cpu().numpy() == ref["nnz"]).all()
    got = Og.double().cpu().numpy()
    assert np.abs(ref["O"]).max() > 4.5                       # the case does reach past the clipped range
    tol = 2e-2 * np.maximum(1.0, np.abs(ref["O"]) / 4.0)
    assert (np.abs(got - ref["O"]) <= tol).all(), float((np.abs(got - ref["O"]) / tol).max())


@pytest.mark.parametrize("n,d", [(5000, 96), (4097, 64), (130, 32), (63, 128), (1, 64)])
def test_delta_scan_time_chunks_adversarial(n, d):
    """The scan is cut into time chunks that start from a guessed state and are repaired afterwards;
    these inputs make the repair walk long: keys that never fire, a slow drift that fires every few
    rows at different phases per channel, and a mix with isolated jumps."""
    rng = np.random.default_rng(n + d)
    const = np.tile(rng.standard_normal((1, 1, 1, d)), (1, 1, n, 1))
    drift = const + 0.03125 * np.arange(n)[None, None, :, None] * (1 + (np.arange(d) % 5))[None, None, None, :] / 4
    jumps = const + np.cumsum((rng.random((1, 1, n, d)) < 0.01) * rng.standard_normal((1, 1, n, d)), axis=2)
    saw = const + 0.01 * (np.arange(n)[None, None, :, None] % 97)
    for name, K, dtype, theta in [("const", const, "bf16", 0.1), ("drift", drift, "f32", 0.1),
                                  ("jumps", jumps, "bf16", 0.3), ("saw", saw, "f32", 0.25),
                                  ("drift_bf16", drift, "bf16", 0.1)]:
        K = wl.round_to_dtype(K, dtype)
        maskg, nnzg, khat = da.delta_attn_delta_scan(to_dev(K, dtype), theta, want_khat=True)
        m, _, Kh, knife = orc.delta_scan(K[0, 0], theta)
        # (fp32 inputs may sit on a binary32 rounding edge; the decision is defined in binary32)
        assert knife == 0 or dtype == "f32", name
        assert (unpack_mask(maskg, d)[0, 0] == m).all(), name
        assert int(nnzg[0, 0]) == int(m.sum()), name
        assert (khat.double().cpu().numpy()[0, 0] == Kh).all(), name


def test_binding_rejects_bad_arguments():
    Q = torch.zeros(1, 4, 64, 64, dtype=torch.bfloat16, device="cuda")
    K = torch.zeros(1, 2, 64, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_prefill(Q, K, K, -1.0, 8)
    assert e.value.status == 1
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_prefill(Q, K, K, 0.1, 8, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 3
    with pytest.raises(ValueError):
        da.delta_attn_prefill(Q, K.float(), K.float(), 0.1, 8)


def test_reruns_are_bit_identical_and_modes_agree():
    """No float atomics anywhere in the output path: two runs give the same bits.  The two score modes
    evaluate the same real-number function (Eq. 4 vs its telescoped form) and agree to rounding."""
    w = wl.C2
    x = wl.generate(w, batch_ids=[0])
    Qd, Kd, Vd = (to_dev(x[k][:, :, :1024], w.dtype) for k in "QKV")
    theta = wl.theta_for(w)
    outs = {}
    for mode in MODES:
        a = da.delta_attn_prefill(Qd, Kd, Vd, theta, w.window, score_mode=mode)
        b = da.delta_attn_prefill(Qd, Kd, Vd, theta, w.window, score_mode=mode)
        torch.cuda.synchronize()
        for t1, t2 in zip(a, b):
            assert torch.equal(t1, t2)
        outs[mode] = a
    assert torch.equal(outs[MODES[0]][1], outs[MODES[1]][1]) and torch.equal(outs[MODES[0]][2], outs[MODES[1]][2])
    assert (outs[MODES[0]][0].float() - outs[MODES[1]][0].float()).abs().max().item() <= 2e-2


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("d,n,dtype", [(64, 300, "bf16"), (128, 200, "bf16"), (64, 150, "f32")])
def test_subnormal_keys(mode, d, n, dtype):
    """Keys that are small multiples of the smallest bf16 subnormal (2^-133), thresholds of that size: the
    binary32 threshold decision keeps subnormals (no flush to zero), so the masks still match bit for bit."""
    rng = np.random.default_rng(5)
    walk = np.cumsum(rng.integers(-1, 2, size=(1, 2, n, d)), axis=2).astype(np.float64)
    K = wl.round_to_dtype(walk * 2.0 ** -133, dtype)
    Q, V = rand_walk(1, 1, 4, n, d, dtype), rand_walk(2, 1, 2, n, d, dtype, clip=3.5)
    for theta in (0.0, 2.0 ** -133, 3 * 2.0 ** -133):
        run_case(Q, K, V, theta, 16, dtype, mode)


@pytest.mark.parametrize("mode", MODES)
def test_large_scores(mode):
    """Queries eight times larger than usual: scaled scores of several hundred, a softmax that is all but one-hot."""
    n, d = 400, 64
    Q = wl.round_to_dtype(rand_walk(3, 1, 4, n, d) * 8.0, "bf16")
    K, V = rand_walk(4, 1, 2, n, d), rand_walk(5, 1, 2, n, d, clip=3.5)
    for wm in (da.DA_WINDOW_BLOCK, da.DA_WINDOW_SLIDING):
        run_case(Q, K, V, 0.1, 32, "bf16", mode, window_mode=wm)


def test_all_work_goes_to_the_callers_stream():
    """Prefill with cache hand-off, chunked prefill and decode steps issued on a side stream, with inputs that are
    produced on that stream right before: a launch or copy that went to another stream would read them too early.
    Results must equal those of the default stream bit for bit."""
    g = torch.Generator(device="cpu").manual_seed(77)
    B, Hq, Hkv, n, d, W, theta = 2, 8, 2, 700, 64, 64, 0.1
    host = [torch.cumsum(0.15 * torch.randn(B, h, n + 8, d, generator=g), 2).clamp(-3.5, 3.5).to(torch.bfloat16)
            for h in (Hq, Hkv, Hkv)]

    def run(stream):
        with torch.cuda.stream(stream):
            # big fill first, so that the copies below are still in flight when the library is called
            junk = torch.empty(1 << 28, dtype=torch.uint8, device="cuda").fill_(1)
            Q, K, V = (x.cuda(non_blocking=False).clone() for x in host)
            cache = da.Cache(B, Hq, Hkv, d, n + 8, 64, theta, torch.bfloat16)
            outs = list(da.delta_attn_prefill(Q[:, :, :400].contiguous(), K[:, :, :400].contiguous(),
                                              V[:, :, :400].contiguous(), theta, W, cache=cache))
            outs += list(da.delta_attn_prefill_append(cache, Q[:, :, 400:n].contiguous(), K[:, :, 400:n].contiguous(),
                                                      V[:, :, 400:n].contiguous(), theta, W))
            for t in range(n, n + 8):
                outs += list(da.delta_attn_decode(cache, Q[:, :, t].contiguous(), K[:, :, t].contiguous(),
                                                  V[:, :, t].contiguous()))
            outs.append(cache.nnz().clone())
        torch.cuda.synchronize()
        cache.close()
        del junk
        return outs

    ref = run(torch.cuda.default_stream())
    got = run(torch.cuda.Stream())
    assert len(ref) == len(got)
    for a, b in zip(ref, got):
        assert torch.equal(a, b)


def test_generic_kernel_matches_on_matrix_core_shapes():
    """The vector-ALU kernel (fp32 inputs, unusual head dims) and the matrix-core kernel implement the
    same path; run both on a bf16 d = 64 case through the fp32 route by widening the inputs."""
    Q, K, V = rand_walk(21, 1, 4, 200, 64), rand_walk(22, 1, 2, 200, 64), rand_walk(23, 1, 2, 200, 64, clip=3.5)
    theta, W = 0.2, 32
    O16, m16, n16 = da.delta_attn_prefill(to_dev(Q, "bf16"), to_dev(K, "bf16"), to_dev(V, "bf16"), theta, W)
    O32, m32, n32 = da.delta_attn_prefill(to_dev(Q, "f32"), to_dev(K, "f32"), to_dev(V, "f32"), theta, W)
    torch.cuda.synchronize()
    assert torch.equal(m16, m32) and torch.equal(n16, n32)     # same keys -> same binary32 decisions
    assert (O16.float() - O32).abs().max().item() <= 2e-2


@pytest.mark.parametrize("mode", MODES)
def test_prefill_replays_from_a_captured_graph(mode):
    """The prefill entry point allocates nothing and records no memset, so a caller may capture it into a HIP graph
    (short prompts are launch-bound: six launches per call).  Replays - with eager work and synchronisations between
    them - must reproduce the eager result bit for bit."""
    B, Hq, Hkv, n, d, W, theta = 2, 4, 2, 200, 64, 16, 0.2
    Q, K, V = rand_walk(81, B, Hq, n, d), rand_walk(82, B, Hkv, n, d), rand_walk(83, B, Hkv, n, d, clip=3.5)
    Qd, Kd, Vd = (to_dev(x, "bf16") for x in (Q, K, V))
    p = da.make_params(Qd, Kd, W, theta, 0.0, mode)
    ws = torch.empty(da.delta_attn_prefill_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    out = (torch.empty_like(Qd), torch.empty((B, Hkv, n, d // 32), dtype=torch.int32, device="cuda"),
           torch.empty((B, Hkv), dtype=torch.int64, device="cuda"))
    eager = [t.clone() for t in da.delta_attn_prefill(Qd, Kd, Vd, theta, W, score_mode=mode, workspace=ws, out=out)]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        da.delta_attn_prefill(Qd, Kd, Vd, theta, W, score_mode=mode, workspace=ws, out=out)
    for rep in range(3):
        for t in out:
            t.zero_()
        ws.random_(0, 255)                      # scratch contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(out, eager):
            assert torch.equal(got, want), rep
    ref = orc.prefill(Q, K, V, theta, W)
    for h in range(Hq):
        check_output(out[0][:, h], ref["O"][:, h], "bf16")


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n,d,W,dtype", [(1, 64, 4, "bf16"), (2, 128, 1, "bf16"), (33, 64, 40, "bf16"),
                                         (1, 32, 1, "f32"), (31, 96, 5, "bf16")])
def test_tiny_sequences(mode, n, d, W, dtype):
    """Sequences shorter than a key block or a row tile: one token (the basis row attends to itself), two, 33."""
    Q, K, V = rand_walk(91, 1, 2, n, d, dtype), rand_walk(92, 1, 1, n, d, dtype), rand_walk(93, 1, 1, n, d, dtype, clip=3.5)
    run_case(Q, K, V, 0.2, W, dtype, mode)
    run_case(Q, K, V, 0.2, W, dtype, mode, window_mode=da.DA_WINDOW_SLIDING)


@pytest.mark.parametrize("window_mode", [da.DA_WINDOW_BLOCK, da.DA_WINDOW_SLIDING])
@pytest.mark.parametrize("d,Hq,Hkv,n,W,p_jump,theta", [(128, 4, 1, 900, 64, 0.3, 0.12), (64, 8, 2, 700, 32, 0.5, 0.2),
                                                       (128, 2, 2, 600, 96, 0.15, 0.0), (64, 2, 1, 500, 32, 1.0, 0.3)])
def test_rebased_full_columns(window_mode, d, Hq, Hkv, n, W, p_jump, theta):
    """Key streams with many whole-vector jumps (and theta = 0, where every column is full): in blocks with several
    full columns the gather kernel does not gather those columns but re-bases the running Eq. 4 score there from
    q . k_hat(j) on the matrix cores - exact by the telescoped sum - so masks, nnz and outputs must still match the
    oracle, which adds up Eq. 4 column by column."""
    rng = np.random.default_rng(int(1000 * p_jump) + d)
    Q, V = rand_walk(111, 2, Hq, n, d), rand_walk(113, 2, Hkv, n, d, clip=3.5)
    K = rand_walk(112, 2, Hkv, n, d, step=0.05)
    jump = rng.random((2, Hkv, n, 1)) < p_jump
    K = wl.round_to_dtype(np.where(jump, rng.standard_normal((2, Hkv, n, d)), K), "bf16")
    run_case(Q, K, V, theta, W, "bf16", da.DA_SCORE_GATHER, window_mode=window_mode)


@pytest.mark.parametrize("window_mode", [da.DA_WINDOW_BLOCK, da.DA_WINDOW_SLIDING])
@pytest.mark.parametrize("B,Hq,Hkv,n,d,W,theta", [
    (1, 4, 2, 1777, 64, 100, 0.15),     # 28 tiles of 128 rows x 2 heads: cut up to 4 ways, ragged last tile and block
    (1, 2, 1, 2500, 128, 32, 0.2),      # 10 tiles of 256 rows: up to 8 parts per tile, short first tiles uncut
    (2, 8, 2, 1100, 128, 300, 0.1),     # windows wider than a part: late tiles have few gather blocks, early ones none
    (1, 1, 1, 3000, 64, 64, 0.0),       # one head; every column full, so parts also re-base columns inside them
])
def test_small_launches_cut_along_the_keys(window_mode, B, Hq, Hkv, n, d, W, theta):
    """A gather-mode launch with too few row tiles to fill the chip gives every long tile several work groups, each on
    a range of its key blocks (a part that does not start at key 0 starts its running Eq. 4 score from q . k_hat of
    the column before, exact by the telescoped sum), and a second launch merges their partial softmax results.  The
    outputs are still those of the oracle's column-by-column recursion, for every row; masks and nnz bit-exact."""
    Q, K, V = rand_walk(131, B, Hq, n, d), rand_walk(132, B, Hkv, n, d), rand_walk(133, B, Hkv, n, d, clip=3.5)
    run_case(Q, K, V, theta, W, "bf16", da.DA_SCORE_GATHER, window_mode=window_mode)


def test_rebase_is_skipped_for_keys_beyond_fp16():
    """The re-base tile is taken in fp16; a block whose reference keys do not fit (|k| >= 2^15) keeps gathering its
    full columns in binary32.  Keys of 5e4 in part of the prompt, every column full (theta = 0): results still match."""
    n, d = 400, 64
    Q, V = wl.round_to_dtype(rand_walk(121, 1, 2, n, d) * 2.0 ** -14, "bf16"), rand_walk(123, 1, 1, n, d, clip=3.5)
    K = rand_walk(122, 1, 1, n, d)
    K[:, :, 100:230] *= 5e4 / np.abs(K[:, :, 100:230]).max()
    K = wl.round_to_dtype(K, "bf16")
    assert np.abs(K).max() >= 2.0 ** 15
    run_case(Q, K, V, 0.0, 32, "bf16", da.DA_SCORE_GATHER)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("window_mode", [da.DA_WINDOW_BLOCK, da.DA_WINDOW_SLIDING])
@pytest.mark.parametrize("n,d", [(64, 128), (128, 128), (256, 128), (512, 128), (100, 64), (512, 64), (257, 128)])
def test_short_prompts_with_the_window_of_eq5(mode, window_mode, n, d):
    """The paper's own regime: prompts of tens to hundreds of tokens with the window of Eq. 5 (gamma = 0.05: W = 3 .. 25).
    Prompts whose keys fit in LDS (n * head_dim <= 32768) take the fused launch - scan, compaction, V re-order and
    attention in one kernel, every work group preparing its unit itself - the others a launch per stage; both must
    match the oracle in masks, nnz, sparsity and every output element."""
    W = da.delta_attn_window_from_gamma(n, 0.05, 512)
    assert W == orc.window_from_gamma(n, 0.05, 512) and 3 <= W <= 25
    Q, K, V = rand_walk(131, 2, 8, n, d), rand_walk(132, 2, 2, n, d), rand_walk(133, 2, 2, n, d, clip=3.5)
    run_case(Q, K, V, 0.12, W, "bf16", mode, window_mode=window_mode)
