"""GPU parity of the decode path (cache hand-off from prefill + delta_attn_decode) against the
oracle's decode workflow.  Mask rows / nnz bit-exact, outputs within tolerance at every step."""
import numpy as np
import pytest
import torch

from paper_2507_19608_amd import binding as da
from paper_2507_19608_amd import workloads as wl
from oracle import delta_oracle as orc
from util import check_output, rand_walk, to_dev, unpack_mask

pytestmark = pytest.mark.gpu


def run_decode(Q, K, V, n, steps, theta, Wd, dtype, W_prefill=16, check_every=1, scale=0.0, plan=None):
    """Prefill n rows into a cache, then `steps` decode steps; compares every check_every-th step."""
    B, Hq, _, d = Q.shape
    Hkv = K.shape[1]
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    cache = da.Cache(B, Hq, Hkv, d, n + steps, Wd, theta, tdt, scale=scale)
    if plan is not None:
        cache.set_launch_plan(*plan)
    st = orc.DecodeState(theta, Wd, scale=None if scale == 0.0 else scale)
    Qd, Kd, Vd = (to_dev(x, dtype) for x in (Q, K, V))
    if n > 0:
        _, maskg, nnzg = da.delta_attn_prefill(Qd[:, :, :n].contiguous(), Kd[:, :, :n].contiguous(),
                                               Vd[:, :, :n].contiguous(), theta, W_prefill, scale=scale, cache=cache)
        mref = st.append(K[:, :, :n], V[:, :, :n])
        assert (unpack_mask(maskg, d) == mref).all()
        assert len(cache) == n
    for t in range(n, n + steps):
        o, mrow = da.delta_attn_decode(cache, Qd[:, :, t].contiguous(), Kd[:, :, t].contiguous(),
                                       Vd[:, :, t].contiguous())
        if (t - n) % check_every == 0 or t == n + steps - 1:
            o_ref, m_ref = st.step(Q[:, :, t], K[:, :, t], V[:, :, t])
            assert (unpack_mask(mrow, d) == m_ref).all(), t
            check_output(o, o_ref, dtype)
        else:
            st.append(K[:, :, t:t + 1], V[:, :, t:t + 1])
    torch.cuda.synchronize()
    assert len(cache) == n + steps
    assert (cache.nnz().cpu().numpy() == st.nnz()).all()
    assert (unpack_mask(cache.mask_rows(), d) == st.mask).all()
    assert st.knife == 0
    # Sec. III-C: the incrementally built delta matrix equals one scan over the whole sequence
    maskw, nnzw, _ = da.delta_attn_delta_scan(Kd[:, :, :n + steps].contiguous(), theta)
    assert (unpack_mask(maskw, d) == st.mask).all()
    assert (nnzw.cpu().numpy() == st.nnz()).all()
    s_m, s_c = da.delta_attn_sparsity(cache.nnz(), n + steps, d, Wd)
    ref = orc.sparsity(int(st.nnz().sum()), n + steps, d, B * Hkv, Wd)
    assert s_m == ref[0] and s_c == pytest.approx(ref[1], abs=1e-15)
    cache.close()


@pytest.mark.parametrize("n,steps,d,Wd,B,Hq,Hkv,theta,dtype", [
    (70, 70, 64, 5, 2, 4, 2, 0.2, "bf16"),      # crosses chunk boundaries at 64 and 128
    (100, 40, 128, 4, 1, 4, 1, 0.15, "bf16"),   # the paper's W_d = 4
    (33, 20, 32, 1, 1, 2, 2, 0.3, "bf16"),      # W_d = 1: only the new key is exact
    (64, 66, 96, 70, 1, 3, 1, 0.25, "bf16"),    # window wider than a chunk
    (50, 30, 64, 8, 1, 2, 1, 0.05, "f32"),
])
def test_decode_small(n, steps, d, Wd, B, Hq, Hkv, theta, dtype):
    L = n + steps
    step = 0.05 if dtype == "f32" else 0.15
    Q, K, V = rand_walk(11, B, Hq, L, d, dtype), rand_walk(12, B, Hkv, L, d, dtype, step), rand_walk(13, B, Hkv, L, d, dtype, clip=3.5)
    run_decode(Q, K, V, n, steps, theta, Wd, dtype, scale=0.0 if dtype == "bf16" else 0.15)


@pytest.mark.parametrize("n,steps,d,Wd,B,Hq,Hkv,theta", [
    (70, 130, 64, 64, 2, 4, 2, 0.2),      # window = one chunk: a chunk is sealed one step before its first row leaves
    (200, 70, 128, 70, 1, 8, 1, 0.15),    # head_dim 128, 8 query heads per KV head
    (0, 140, 64, 64, 1, 2, 1, 0.25),      # from an empty cache through two seals
    (128, 65, 64, 100, 1, 32, 1, 0.1),    # prefill ends on a chunk boundary; 32 heads share the KV head
    (191, 3, 128, 128, 1, 2, 2, 0.3),     # the prefill leaves an unsealed chunk one row short of full
    (10, 12, 64, 96, 2, 4, 2, 0.2),       # a cache shorter than a chunk: the decode window is cut to its 22 rows
    (0, 40, 128, 1000, 1, 4, 1, 0.1),     # the same at head_dim 128, from an empty cache
])
def test_decode_column_run_layout(n, steps, d, Wd, B, Hq, Hkv, theta):
    """bf16 caches with head_dim 64 / 128 and a decode window of at least one chunk keep the compact
    cache as per-channel runs sealed chunk by chunk; same oracle, same tolerances."""
    L = n + steps
    Q, K, V = rand_walk(31, B, Hq, L, d), rand_walk(32, B, Hkv, L, d), rand_walk(33, B, Hkv, L, d, clip=3.5)
    run_decode(Q, K, V, n, steps, theta, Wd, "bf16")


@pytest.mark.parametrize("plan", [(1, 0), (0, 2), (0, 5), (1, 1)])
@pytest.mark.parametrize("n,steps,d,Hq,Hkv", [(300, 70, 64, 4, 2), (0, 200, 64, 8, 1), (260, 130, 128, 4, 1)])
def test_decode_launch_plans(plan, n, steps, d, Hq, Hkv):
    """Every way of laying a step out over the GPU gives the same result: one work group per unit whose
    waves merge on chip (with idle waves while the cache is short), or single-wave work groups that walk
    several chunks each (2 or 5 wave slots for 2 units force up to all chunks into one wave) + merge launch."""
    B, L = 2, n + steps
    Q, K, V = rand_walk(41, B, Hq, L, d), rand_walk(42, B, Hkv, L, d), rand_walk(43, B, Hkv, L, d, clip=3.5)
    run_decode(Q, K, V, n, steps, 0.2, 64, "bf16", check_every=7, plan=plan)


def test_decode_from_empty_cache_and_dense_limits():
    B, Hq, Hkv, L, d = 1, 2, 1, 40, 64
    Q, K, V = rand_walk(14, B, Hq, L, d), rand_walk(15, B, Hkv, L, d), rand_walk(16, B, Hkv, L, d, clip=3.5)
    run_decode(Q, K, V, 0, 40, 0.2, 6, "bf16")            # first decoded token is the basis row
    run_decode(Q, K, V, 10, 30, 0.0, 3, "bf16")           # theta = 0: dense attention
    run_decode(Q, K, V, 10, 30, 0.4, 1000, "bf16")        # window covers everything
    run_decode(Q, K, V, 10, 30, float("inf"), 3, "bf16")  # history frozen at the basis key
    L = 200
    Q, K, V = rand_walk(14, B, Hq, L, d), rand_walk(15, B, Hkv, L, d), rand_walk(16, B, Hkv, L, d, clip=3.5)
    run_decode(Q, K, V, 100, 100, 0.0, 64, "bf16")           # the same limits in the column-run layout
    run_decode(Q, K, V, 100, 100, float("inf"), 64, "bf16")


def test_cache_state_errors():
    cache = da.Cache(1, 2, 1, 64, 4, 2, 0.1, torch.bfloat16)
    z = lambda h: torch.zeros(1, h, 64, dtype=torch.bfloat16, device="cuda")
    for _ in range(4):
        da.delta_attn_decode(cache, z(2), z(1), z(1))
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_decode(cache, z(2), z(1), z(1))
    assert e.value.status == 4                                # cache full
    with pytest.raises(da.DeltaAttnError):
        cache.set_launch_plan(2, 0)
    with pytest.raises(da.DeltaAttnError):
        cache.set_launch_plan(0, -1)
    Q = torch.zeros(1, 2, 4, 64, dtype=torch.bfloat16, device="cuda")
    K = torch.zeros(1, 1, 4, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_prefill(Q, K, K, 0.1, 2, cache=cache)   # not empty
    assert e.value.status == 4
    cache.reset()
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_prefill(Q, K, K, 0.2, 2, cache=cache)   # theta differs from the cache's
    assert e.value.status == 4
    da.delta_attn_prefill(Q, K, K, 0.1, 2, cache=cache)
    assert len(cache) == 4
    cache.close()


def test_c4_decode_llama_shape_sampled_batch():
    """Config 4 at full size on the GPU (batch 32, 2048 cached + 256 steps); the oracle follows
    three batch entries (streams are independent per batch entry)."""
    w = wl.C4
    ids = [0, 17, 31]
    x = wl.generate(w)
    theta = wl.theta_for(w)
    B, Hq, Hkv, d, n, steps = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.seq_len, w.decode_steps
    Qd, Kd, Vd = (to_dev(x[k], w.dtype) for k in "QKV")
    cache = da.Cache(B, Hq, Hkv, d, n + steps, w.window, theta, torch.bfloat16)
    da.delta_attn_prefill(Qd[:, :, :n].contiguous(), Kd[:, :, :n].contiguous(), Vd[:, :, :n].contiguous(), theta,
                          w.window, cache=cache)
    st = orc.DecodeState(theta, w.window)
    xs = {k: x[k][ids] for k in "QKV"}
    st.append(xs["K"][:, :, :n], xs["V"][:, :, :n])
    # every output element of every batch entry and step (the oracle follows three entries): finite, and inside
    # the per-channel range of the value rows cached so far (Eq. 1: weights that sum to one), up to output rounding
    Vf = Vd.float()
    lo_all = torch.cummin(Vf, dim=2).values.repeat_interleave(Hq // Hkv, dim=1)
    hi_all = torch.cummax(Vf, dim=2).values.repeat_interleave(Hq // Hkv, dim=1)
    tol = 2.0 ** -8 * Vf.abs().max().item()
    for t in range(n, n + steps):
        o, mrow = da.delta_attn_decode(cache, Qd[:, :, t].contiguous(), Kd[:, :, t].contiguous(),
                                       Vd[:, :, t].contiguous())
        of = o.float()
        assert torch.isfinite(of).all()
        assert (of >= lo_all[:, :, t] - tol).all() and (of <= hi_all[:, :, t] + tol).all()
        if (t - n) % 37 == 0 or t == n + steps - 1:
            o_ref, m_ref = st.step(xs["Q"][:, :, t], xs["K"][:, :, t], xs["V"][:, :, t])
            assert (unpack_mask(mrow, d)[ids] == m_ref).all()
            check_output(o[ids], o_ref, w.dtype)
        else:
            st.append(xs["K"][:, :, t:t + 1], xs["V"][:, :, t:t + 1])
    assert (cache.nnz().cpu().numpy()[ids] == st.nnz()).all()
    s_m, _ = da.delta_attn_sparsity(cache.nnz(), n + steps, d, w.window)
    assert abs(s_m - 0.57) < 0.01
    cache.close()


@pytest.mark.parametrize("shape", ["C4", "head_dim 128", "fp32 cache", "head_dim 96", "window 40"])
def test_c4_every_output_element_against_the_dense_form(shape):
    """Config 4 at full size, every output element of every step and batch entry against the closed form the oracle
    is pinned to - q . k_hat(j) for keys left of the decode window, q . k_j inside it, Eq. 1 on top - in fp64 with
    library products on the device.  k_hat comes from Eq. 2-3 written out with tensor operations over all units at
    once (binary32 decision, as the oracle takes it).  Tolerance as for the oracle.  Also at batch 32 with config 3's
    heads (20 / 5 of 128 channels: a pair of waves per chunk), 130 steps that cross two chunk seals; and for the
    row-layout caches of the generic kernels (fp32; a head size other than 64 / 128; a decode window below 64)."""
    w = {"C4": wl.C4,
         "head_dim 128": wl.Workload("D128", 32, 20, 5, 128, 2048, 128, "bf16", seed=44, decode_steps=130, theta=0.11),
         "fp32 cache": wl.Workload("DF32", 4, 8, 2, 64, 1200, 128, "f32", seed=45, decode_steps=70, theta=0.11),
         "head_dim 96": wl.Workload("D96", 4, 6, 2, 96, 1000, 100, "bf16", seed=46, decode_steps=70, theta=0.11),
         "window 40": wl.Workload("DW40", 4, 8, 2, 64, 1000, 40, "bf16", seed=47, decode_steps=70, theta=0.11)}[shape]
    x = wl.generate(w)
    theta = wl.theta_for(w)
    B, Hq, Hkv, d, n, steps = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.seq_len, w.decode_steps
    g = Hq // Hkv
    Qd, Kd, Vd = (to_dev(x[k], w.dtype) for k in "QKV")
    cache = da.Cache(B, Hq, Hkv, d, n + steps, w.window, theta, Qd.dtype)
    da.delta_attn_prefill(Qd[:, :, :n].contiguous(), Kd[:, :, :n].contiguous(), Vd[:, :, :n].contiguous(), theta,
                          w.window, cache=cache)
    K64, V64 = Kd.double(), Vd.double()
    Khat64 = torch.empty_like(K64)
    held = Kd[:, :, 0].float()
    Khat64[:, :, 0] = held.double()
    th32 = torch.tensor(theta, dtype=torch.float32, device="cuda")
    for t in range(1, n + steps):
        kt = Kd[:, :, t].float()
        held = torch.where((kt - held).abs() > th32, kt, held)
        Khat64[:, :, t] = held.double()
    worst = 0.0
    for t in range(n, n + steps):
        o, _ = da.delta_attn_decode(cache, Qd[:, :, t].contiguous(), Kd[:, :, t].contiguous(),
                                    Vd[:, :, t].contiguous())
        q = Qd[:, :, t].double().reshape(B, Hkv, g, d)
        s_hist = torch.einsum("bkgd,bktd->bkgt", q, Khat64[:, :, :t + 1])
        s_win = torch.einsum("bkgd,bktd->bkgt", q, K64[:, :, :t + 1])
        in_window = torch.arange(t + 1, device="cuda") > t - w.window
        p = torch.softmax(torch.where(in_window, s_win, s_hist) / d ** 0.5, dim=-1)
        ref = torch.einsum("bkgt,bktd->bkgd", p, V64[:, :, :t + 1]).reshape(B, Hq, d)
        assert torch.isfinite(o.float()).all()
        worst = max(worst, (o.double() - ref).abs().max().item())
    cache.close()
    assert worst <= (2e-2 if w.dtype == "bf16" else 1e-4 * V64.abs().max().item()), worst


@pytest.mark.parametrize("seed", range(8))
def test_random_decode_runs_against_the_dense_form(seed):
    """Seeded random decode runs (batch 1-24, group sizes up to 32, prompts of 0-3000 rows through the prefill or in
    two pieces through the chunked entry point, 3-200 steps, decode windows 64-512, every launch plan): every output
    element of every step within tolerance of the dense form."""
    import random
    import dense_form as df
    rng = random.Random(2000 + seed)
    d, Hkv, g = rng.choice([64, 128]), rng.choice([1, 2, 4, 8]), rng.choice([1, 2, 4, 5, 8, 16, 32])
    B, n0 = rng.choice([1, 2, 8, 24]), rng.choice([0, 1, 63, 64, 200, 700, 1500, 2047, 2048, 3000])
    steps, Wd, theta = rng.choice([3, 65, 70, 130, 200]), rng.choice([64, 100, 128, 256, 512]), rng.choice([0.0, 0.05, 0.11, 0.3])
    plan = rng.choice([None, None, (1, 0), (0, 0), (0, 5), (-1, 64)])
    Hq, L = Hkv * g, n0 + steps
    if B * Hq * L * d > 4e8:
        B = 1
    Qd, Kd, Vd = (to_dev(rand_walk(7000 + 3 * seed + k, B, H, L, d, clip=c), "bf16")
                  for k, (H, c) in enumerate(((Hq, None), (Hkv, None), (Hkv, 3.5))))
    cache = da.Cache(B, Hq, Hkv, d, L, Wd, theta, torch.bfloat16)
    if plan is not None:
        cache.set_launch_plan(*plan)
    if n0 > 0:
        Wp = rng.choice([16, 64, min(Wd, 128)])
        cuts = [0, n0] if (rng.random() < 0.5 or n0 < 3) else [0, rng.randrange(1, n0), n0]
        for a, b in zip(cuts[:-1], cuts[1:]):
            args = (Qd[:, :, a:b].contiguous(), Kd[:, :, a:b].contiguous(), Vd[:, :, a:b].contiguous(), theta, Wp)
            if len(cuts) == 2:
                da.delta_attn_prefill(*args, score_mode=da.DA_SCORE_REBASE, cache=cache)
            else:
                da.delta_attn_prefill_append(cache, *args, score_mode=da.DA_SCORE_REBASE)
    khat, _ = df.reference_keys(Kd, theta)
    K64, V64 = Kd.double(), Vd.double()
    worst = 0.0
    for t in range(n0, L):
        o, _ = da.delta_attn_decode(cache, Qd[:, :, t].contiguous(), Kd[:, :, t].contiguous(), Vd[:, :, t].contiguous())
        worst = max(worst, (o.double() - df.decode_reference(Qd[:, :, t], K64, V64, khat, t, Wd)).abs().max().item())
    cache.close()
    assert worst <= 2e-2, worst


@pytest.mark.parametrize("d,dtype,Wd", [(64, "bf16", 64), (128, "bf16", 100), (64, "f32", 16), (96, "bf16", 32)])
def test_decode_awkward_numbers(d, dtype, Wd):
    """Both cache layouts on inputs at the edges of the number range: keys that are small multiples of the smallest
    bf16 subnormal with thresholds of that size (masks must still match bit for bit: no flush to zero in the
    binary32 decision), and queries eight times larger than usual (scaled scores of several hundred, a softmax that
    is all but one-hot)."""
    rng = np.random.default_rng(9)
    n, steps = 150, 80
    L = n + steps
    tiny = wl.round_to_dtype(np.cumsum(rng.integers(-1, 2, size=(1, 2, L, d)), axis=2).astype(np.float64) * 2.0 ** -133, dtype)
    Q, V = rand_walk(1, 1, 4, L, d, dtype), rand_walk(2, 1, 2, L, d, dtype, clip=3.5)
    for theta in (0.0, 2.0 ** -133, 3 * 2.0 ** -133):
        run_decode(Q, tiny, V, n, steps, theta, Wd, dtype, W_prefill=16, check_every=7)
    big = wl.round_to_dtype(rand_walk(3, 1, 4, L, d, dtype) * 8.0, dtype)
    run_decode(big, rand_walk(4, 1, 2, L, d, dtype), V, n, steps, 0.1, Wd, dtype, W_prefill=16, check_every=7)


def test_decode_on_a_cache_beyond_4_gib():
    """Maximum sizes: batch 16, 32 / 8 heads of 128, 131072 cached tokens - the cache's V array alone is 4 GiB, its
    offsets leave 32 bits - filled by one prefill (telescoped mode), then three decode steps; three batch entries
    (first, middle, last) are compared with the dense form in fp64, with k_hat from the oracle's Eq. 2-3."""
    import dense_form as df
    B, Hq, Hkv, n, d, Wd, theta, steps = 16, 32, 8, 131072, 128, 128, 0.11, 3
    L = n + steps
    gen = torch.Generator(device="cuda").manual_seed(32)

    def walk(H, clip=None):
        x = torch.cumsum(0.15 * torch.randn(B, H, L, d, device="cuda", generator=gen), dim=2)
        x += torch.randn(B, H, 1, d, device="cuda", generator=gen)
        return (x.clamp(-clip, clip) if clip else x).to(torch.bfloat16)

    Kd, Vd, Qd = walk(Hkv), walk(Hkv, 3.5), walk(Hq)
    assert B * Hkv * L * d * 2 > 2 ** 32
    cache = da.Cache(B, Hq, Hkv, d, L, Wd, theta, torch.bfloat16)
    da.delta_attn_prefill(Qd[:, :, :n].contiguous(), Kd[:, :, :n].contiguous(), Vd[:, :, :n].contiguous(), theta, 512,
                          score_mode=da.DA_SCORE_REBASE, cache=cache)
    ids = (0, 7, B - 1)
    khat = {b: torch.stack([torch.from_numpy(orc.delta_scan(Kd[b, hk].double().cpu().numpy(), theta)[2])
                            for hk in range(Hkv)]).cuda() for b in ids}
    for t in range(n, L):
        o, _ = da.delta_attn_decode(cache, Qd[:, :, t].contiguous(), Kd[:, :, t].contiguous(), Vd[:, :, t].contiguous())
        for b in ids:
            ref = df.decode_reference(Qd[b:b + 1, :, t], Kd[b:b + 1].double(), Vd[b:b + 1].double(), khat[b][None], t, Wd)
            assert (o[b:b + 1].double() - ref).abs().max().item() <= 2e-2
    cache.close()


@pytest.mark.parametrize("d,Hq,Hkv", [(128, 4, 1), (64, 8, 2)])
def test_decode_after_a_32k_token_prompt(d, Hq, Hkv):
    """A long history: 32 768 cached tokens (512 sealed chunks per unit), then 70 steps, which cross a chunk seal."""
    w = wl.Workload("L32K", 1, Hq, Hkv, d, 32768, 128, "bf16", seed=32, decode_steps=70, theta=0.11)
    x = wl.generate(w)
    run_decode(x["Q"], x["K"], x["V"], w.seq_len, w.decode_steps, 0.11, w.window, "bf16", W_prefill=512, check_every=23)


@pytest.mark.parametrize("score_mode", [da.DA_SCORE_GATHER, da.DA_SCORE_REBASE])
@pytest.mark.parametrize("window_mode", [da.DA_WINDOW_BLOCK, da.DA_WINDOW_SLIDING])
@pytest.mark.parametrize("d,Hq,Hkv,W,Wd,chunks", [
    (64, 4, 2, 48, 64, (100, 37, 64, 91)),      # unaligned pieces: old partial chunks get completed and sealed
    (128, 4, 1, 20, 70, (64, 130, 1, 70)),      # a piece of one row; pieces that start on chunk boundaries
    (64, 8, 1, 64, 64, (10, 300)),              # a short first piece, then several chunks at once
    (128, 1, 1, 16, 96, (10, 1)),               # a cache of 23 rows: shorter than a chunk
    (64, 4, 2, 128, 128, (1, 64)),              # window above the cache's length
    (128, 4, 1, 64, 128, (256, 256, 128)),      # pieces and window squares on row-tile boundaries: the kernel
    (64, 16, 2, 128, 128, (128, 64, 64, 192)),  # instantiation without a K_hat tile, entered with a row offset
])
def test_chunked_prefill_then_decode(score_mode, window_mode, d, Hq, Hkv, W, Wd, chunks):
    """Prefill in pieces onto a growing cache (Sec. III-C): every piece must equal the same rows of one prefill
    over the whole prefix (window squares anchored at position 0), the masks must equal one scan, and decode
    must continue from the cache as if it had been filled in one go."""
    B, steps, theta = 2, 12, 0.2
    L = sum(chunks) + steps
    Q, K, V = rand_walk(71, B, Hq, L, d), rand_walk(72, B, Hkv, L, d), rand_walk(73, B, Hkv, L, d, clip=3.5)
    Qd, Kd, Vd = (to_dev(x, "bf16") for x in (Q, K, V))
    cache = da.Cache(B, Hq, Hkv, d, L, Wd, theta, torch.bfloat16)
    t0 = 0
    for m in chunks:
        sl = slice(t0, t0 + m)
        O, maskg, nnzg = da.delta_attn_prefill_append(cache, Qd[:, :, sl].contiguous(), Kd[:, :, sl].contiguous(),
                                                      Vd[:, :, sl].contiguous(), theta, W, score_mode=score_mode,
                                                      window_mode=window_mode)
        ref = orc.prefill(Q[:, :, :t0 + m], K[:, :, :t0 + m], V[:, :, :t0 + m], theta, W, rows=(t0, t0 + m),
                          window_mode=window_mode)
        assert ref["knife"] == 0
        assert (unpack_mask(maskg, d) == ref["mask"][:, :, t0:]).all()
        assert (nnzg.cpu().numpy() == ref["mask"][:, :, t0:].sum(axis=(2, 3))).all()
        for h in range(Hq):
            check_output(O[:, h], ref["O"][:, h], "bf16")
        t0 += m
        assert len(cache) == t0
        assert (cache.nnz().cpu().numpy() == ref["nnz"]).all()
    st = orc.DecodeState(theta, Wd)
    st.append(K[:, :, :t0], V[:, :, :t0])
    assert (unpack_mask(cache.mask_rows(), d) == st.mask).all()
    for t in range(t0, t0 + steps):
        o, mrow = da.delta_attn_decode(cache, Qd[:, :, t].contiguous(), Kd[:, :, t].contiguous(), Vd[:, :, t].contiguous())
        o_ref, m_ref = st.step(Q[:, :, t], K[:, :, t], V[:, :, t])
        assert (unpack_mask(mrow, d) == m_ref).all()
        check_output(o, o_ref, "bf16")
    assert (cache.nnz().cpu().numpy() == st.nnz()).all()
    cache.close()


@pytest.mark.parametrize("d,Hq,Hkv", [(64, 4, 2), (128, 4, 1)])
def test_chunked_prefill_between_decode_steps_resets_and_score_modes(d, Hq, Hkv):
    """The cache keeps the sequence as plain arrays between pieces and only adds a piece's rows; whatever else moves
    the cache on (decode steps, a reset, a one-shot prefill into it) must make the next piece rebuild them, and a
    piece in gather mode must find the entry lists of columns that earlier telescoped pieces did not write.  Every
    piece against the same rows of the oracle's prefill over the whole prefix, the final cache through decode."""
    B, W, Wd, theta = 2, 40, 96, 0.2
    G, R = da.DA_SCORE_GATHER, da.DA_SCORE_REBASE
    # (kind, rows, score mode): pieces that start inside a block of 32 columns and inside a chunk of 64 rows
    plan = [("piece", 75, G), ("piece", 50, R), ("piece", 45, G), ("decode", 7, None), ("piece", 90, R),
            ("piece", 33, G), ("decode", 1, None), ("piece", 64, G)]
    L = sum(r for _, r, _ in plan) + 6
    Q, K, V = rand_walk(81, B, Hq, L, d), rand_walk(82, B, Hkv, L, d), rand_walk(83, B, Hkv, L, d, clip=3.5)
    Qd, Kd, Vd = (to_dev(x, "bf16") for x in (Q, K, V))
    cache = da.Cache(B, Hq, Hkv, d, L, Wd, theta, torch.bfloat16)

    def run(plan, t0):
        for kind, rows, mode in plan:
            if kind == "decode":
                for t in range(t0, t0 + rows):
                    da.delta_attn_decode(cache, Qd[:, :, t].contiguous(), Kd[:, :, t].contiguous(), Vd[:, :, t].contiguous())
                t0 += rows
                continue
            sl = slice(t0, t0 + rows)
            O, maskg, nnzg = da.delta_attn_prefill_append(cache, Qd[:, :, sl].contiguous(), Kd[:, :, sl].contiguous(),
                                                          Vd[:, :, sl].contiguous(), theta, W, score_mode=mode)
            ref = orc.prefill(Q[:, :, :t0 + rows], K[:, :, :t0 + rows], V[:, :, :t0 + rows], theta, W, rows=(t0, t0 + rows))
            assert ref["knife"] == 0
            assert (unpack_mask(maskg, d) == ref["mask"][:, :, t0:]).all(), (t0, rows)
            for h in range(Hq):
                check_output(O[:, h], ref["O"][:, h], "bf16")
            t0 += rows
            assert len(cache) == t0
            assert (cache.nnz().cpu().numpy() == ref["nnz"]).all()
        return t0

    t0 = run(plan, 0)
    # the same cache again from empty: pieces straight after a reset, then after a one-shot prefill into the cache
    cache.reset()
    t0 = run([("piece", 40, G), ("piece", 30, G)], 0)
    cache.reset()
    da.delta_attn_prefill(Qd[:, :, :100].contiguous(), Kd[:, :, :100].contiguous(), Vd[:, :, :100].contiguous(), theta, W,
                          cache=cache)
    t0 = run([("piece", 70, G), ("piece", 70, R), ("piece", 31, G)], 100)
    st = orc.DecodeState(theta, Wd)
    st.append(K[:, :, :t0], V[:, :, :t0])
    assert (unpack_mask(cache.mask_rows(), d) == st.mask).all()
    for t in range(t0, t0 + 6):
        o, mrow = da.delta_attn_decode(cache, Qd[:, :, t].contiguous(), Kd[:, :, t].contiguous(), Vd[:, :, t].contiguous())
        o_ref, m_ref = st.step(Q[:, :, t], K[:, :, t], V[:, :, t])
        assert (unpack_mask(mrow, d) == m_ref).all()
        check_output(o, o_ref, "bf16")
    cache.close()


def test_chunked_prefill_argument_checks():
    z = lambda h, m, d=64: torch.zeros(1, h, m, d, dtype=torch.bfloat16, device="cuda")
    small = da.Cache(1, 2, 1, 64, 300, 8, 0.1, torch.bfloat16)          # decode window below one chunk: row layout
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_prefill_append(small, z(2, 10), z(1, 10), z(1, 10), 0.1, 4)
    assert e.value.status == 2
    small.close()
    cache = da.Cache(1, 2, 1, 64, 100, 64, 0.1, torch.bfloat16)
    da.delta_attn_prefill_append(cache, z(2, 70), z(1, 70), z(1, 70), 0.1, 16)
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_prefill_append(cache, z(2, 31), z(1, 31), z(1, 31), 0.1, 16)   # 101 rows > max_seq
    assert e.value.status == 4
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_prefill_append(cache, z(2, 10), z(1, 10), z(1, 10), 0.1, 65)   # window wider than the ring
    assert e.value.status == 2
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_prefill_append(cache, z(2, 10), z(1, 10), z(1, 10), 0.2, 16)   # theta differs
    assert e.value.status == 4
    assert len(cache) == 70
    cache.close()
