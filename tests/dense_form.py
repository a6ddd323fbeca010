"""The closed form that the oracle is pinned to (tests/test_oracle_pins.py: outside scores equal q . k_hat), evaluated
in fp64 with library tensor operations on the device: a second reference that is fast enough to check every output
element at full size.  Eq. 2-3 written out row by row over all units at once (binary32 decision); scores q . k_hat(j)
outside a row's window and q . k_j inside it; Eq. 1 on top.  Test infrastructure only: it shares nothing with the HIP
path, and the GPU tests that use it also compare masks, or sampled rows, with the fp64 CPU oracle."""
import torch


def reference_keys(Kd: torch.Tensor, theta: float):
    """K [B, Hkv, L, d] on the device -> (k_hat fp64 [B, Hkv, L, d], mask bool): Eq. 2-3, row 0 the basis."""
    held = Kd[:, :, 0].float()
    khat = torch.empty_like(Kd, dtype=torch.float64)
    mask = torch.ones_like(Kd, dtype=torch.bool)
    khat[:, :, 0] = held.double()
    th32 = torch.tensor(theta, dtype=torch.float32, device=Kd.device)
    for t in range(1, Kd.shape[2]):
        kt = Kd[:, :, t].float()
        fire = (kt - held).abs() > th32
        held = torch.where(fire, kt, held)
        khat[:, :, t] = held.double()
        mask[:, :, t] = fire
    return khat, mask


def unpack_bits(bits: torch.Tensor, d: int) -> torch.Tensor:
    """int32 words [..., d/32] -> bool [..., d]."""
    sh = torch.arange(32, device=bits.device, dtype=torch.int32)
    return ((bits.unsqueeze(-1) >> sh) & 1).reshape(*bits.shape[:-1], d).bool()


def prefill_worst_error(Qd, Kd, Vd, khat, W, sliding, outputs, row_block=2048):
    """max |O - reference| over every element of every tensor in `outputs` ([B, Hq, n, d] each)."""
    B, Hq, n, d = Qd.shape
    g = Hq // Kd.shape[1]
    rows = torch.arange(n, device=Qd.device)
    worst = 0.0
    for b in range(B):
        for h in range(Hq):
            K, V, H = Kd[b, h // g].double(), Vd[b, h // g].double(), khat[b, h // g]
            for r0 in range(0, n, row_block):
                r1 = min(n, r0 + row_block)
                i, j = rows[r0:r1, None], rows[None, :r1]
                inside = (i - j < W) if sliding else (i // W == j // W)
                Q = Qd[b, h, r0:r1].double()
                S = torch.where(inside, Q @ K[:r1].T, Q @ H[:r1].T) / d ** 0.5
                ref = torch.softmax(S.masked_fill(j > i, float("-inf")), dim=-1) @ V[:r1]
                for O in outputs:
                    worst = max(worst, (O[b, h, r0:r1].double() - ref).abs().max().item())
    return worst


def decode_reference(q, K64, V64, khat, t, Wd):
    """One decode step at position t: q [B, Hq, d]; K64, V64, khat fp64 [B, Hkv, L, d] -> fp64 [B, Hq, d]."""
    B, Hq, d = q.shape
    Hkv = K64.shape[1]
    qq = q.double().reshape(B, Hkv, Hq // Hkv, d)
    s_hist = torch.einsum("bkgd,bktd->bkgt", qq, khat[:, :, :t + 1])
    s_win = torch.einsum("bkgd,bktd->bkgt", qq, K64[:, :, :t + 1])
    in_window = torch.arange(t + 1, device=q.device) > t - Wd
    p = torch.softmax(torch.where(in_window, s_win, s_hist) / d ** 0.5, dim=-1)
    return torch.einsum("bkgt,bktd->bkgd", p, V64[:, :, :t + 1]).reshape(B, Hq, d)
