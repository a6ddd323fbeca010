"""delta_attn_prefill_noalloc (the entry point for callers that cannot allocate: its scratch is a buffer built into
the library's device image) against delta_attn_prefill on the same inputs: same kernels, so masks and nnz must be
bit-identical and so must the outputs - except where delta_attn_prefill cuts a small launch along the keys and the
built-in buffer has no room for the parts' results: the two then differ in rounding order, each inside the output
tolerance of the oracle, against which both calls are held as well.  Two calls in a row share the one buffer - the
second, smaller prompt must not see anything of the first."""
import numpy as np
import pytest
import torch

from paper_2507_19608_amd import binding as da
from oracle import delta_oracle as orc
from util import check_output, rand_walk, to_dev, unpack_mask

pytestmark = pytest.mark.gpu


def _outs(Q, K):
    B, Hkv, n, d = K.shape
    return (torch.empty_like(Q), torch.empty((B, Hkv, n, d // 32), dtype=torch.int32, device="cuda"),
            torch.empty((B, Hkv), dtype=torch.int64, device="cuda"))


@pytest.mark.parametrize("mode", [da.DA_SCORE_GATHER, da.DA_SCORE_REBASE])
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 96)])
def test_noalloc_equals_prefill_on_two_calls_in_a_row(mode, dtype, d):
    theta = 0.15
    shapes = [(2, 8, 2, 1500, 64), (1, 4, 1, 333, 16)]           # (B, Hq, Hkv, n, W): the second call is the smaller one
    if dtype == "f32":
        shapes = [(1, 4, 2, 400, 32), (1, 2, 1, 130, 8)]
    for k, (B, Hq, Hkv, n, W) in enumerate(shapes):
        Q, K, V = (rand_walk(200 + 10 * k + i, B, H, n, d, dtype, clip=c)
                   for i, (H, c) in enumerate(((Hq, None), (Hkv, None), (Hkv, 3.5))))
        Qd, Kd, Vd = (to_dev(x, dtype) for x in (Q, K, V))
        want = da.delta_attn_prefill(Qd, Kd, Vd, theta, W, score_mode=mode)
        out = _outs(Qd, Kd)
        for t in out:
            t.fill_(-1)
        allocs = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
        got = da.delta_attn_prefill_noalloc(Qd, Kd, Vd, theta, W, out, score_mode=mode)
        # no allocation request reached torch's allocator during the call either (the binding marshals only)
        assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == allocs
        torch.cuda.synchronize()
        assert torch.equal(got[1], want[1]) and torch.equal(got[2], want[2]), (k, dtype, d)
        if k == 1 or dtype == "f32":                             # one work group per tile in both: the same arithmetic
            assert torch.equal(got[0], want[0]), (k, dtype, d)
        check_output(got[0], want[0].double().cpu().numpy(), dtype)
        ref = orc.prefill(Q, K, V, theta, W)                     # and the results are the oracle's
        assert (unpack_mask(got[1], d) == ref["mask"]).all() and (got[2].cpu().numpy() == ref["nnz"]).all()
        for h in range(Hq):
            check_output(got[0][:, h], ref["O"][:, h], dtype)


def test_noalloc_rejects_a_prompt_beyond_its_scratch():
    Q = torch.zeros(4, 20, 8192, 128, dtype=torch.bfloat16, device="cuda")
    K = torch.zeros(4, 5, 8192, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(da.DeltaAttnError) as e:
        da.delta_attn_prefill_noalloc(Q, K, K, 0.1, 512, _outs(Q, K))
    assert e.value.status == 3 and str(da.NOALLOC_SCRATCH_BYTES) in str(e.value)


@pytest.mark.parametrize("n,d", [(200, 64), (1500, 128)])
def test_noalloc_replays_from_a_captured_graph(n, d):
    """The callers it is for: captured into a HIP graph (after one eager call that did the one-time set-up), replayed
    with eager work and synchronisations in between; every replay must reproduce the eager call bit for bit (and
    delta_attn_prefill's masks and nnz; its outputs to the tolerance, see above).
    200 tokens take the fused single launch, 1500 the launch-per-stage path (whose counters are cleared by a fill
    kernel, not by a memset node)."""
    B, Hq, Hkv, W, theta = 2, 4, 2, 32, 0.15
    Qd, Kd, Vd = (to_dev(rand_walk(300 + i, B, H, n, d, clip=c), "bf16")
                  for i, (H, c) in enumerate(((Hq, None), (Hkv, None), (Hkv, 3.5))))
    want = da.delta_attn_prefill(Qd, Kd, Vd, theta, W)
    out = _outs(Qd, Kd)
    da.delta_attn_prefill_noalloc(Qd, Kd, Vd, theta, W, out)     # eager first call: symbol look-up, LDS limits
    torch.cuda.synchronize()
    eager = [t.clone() for t in out]
    assert torch.equal(eager[1], want[1]) and torch.equal(eager[2], want[2])
    check_output(eager[0], want[0].double().cpu().numpy(), "bf16")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        da.delta_attn_prefill_noalloc(Qd, Kd, Vd, theta, W, out)
    for rep in range(3):
        for t in out:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for g, w_ in zip(out, eager):
            assert torch.equal(g, w_), rep
