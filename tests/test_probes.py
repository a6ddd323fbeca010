"""The measurement aids of the C ABI (streaming read, arithmetic-rate loops): they must run, leave their
inputs alone and reject bad arguments; their rates are reported by bench.py, not asserted here."""
import pytest
import torch

from paper_2507_19608_amd import binding as da

pytestmark = pytest.mark.gpu


def test_stream_read_and_rate_probes():
    buf = torch.arange(1 << 18, dtype=torch.int32, device="cuda")          # 1 MiB
    keep = buf.clone()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    da.delta_attn_stream_read(buf, sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, keep) and int(sink[0]) == 0
    with pytest.raises(da.DeltaAttnError):
        da.delta_attn_stream_read(buf[:100], sink)                          # 400 bytes: not a multiple of 1024
    fsink = torch.zeros(1, dtype=torch.float32, device="cuda")
    for kind, per_round in ((0, 4.0 * 2 * 32 * 32 * 16), (1, 16.0 * 64 * 2), (2, 16.0 * 64 * 2), (3, 16.0 * 64 * 2)):
        flop = da.delta_attn_rate_probe(kind, 4, 16, fsink)
        assert flop == 4 * 4 * 16 * per_round                               # work groups x waves x rounds
    torch.cuda.synchronize()
    assert float(fsink[0]) == 0.0
    with pytest.raises(da.DeltaAttnError):
        da.delta_attn_rate_probe(4, 4, 16, fsink)
