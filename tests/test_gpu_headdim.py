"""GPU parity for head dimensions other than the two the kernels are built for (64, 128):
every multiple of 8 up to 128 runs in the next larger kernel with the missing columns read
as zeros.  Outputs sit in NaN-poisoned, padded allocations, so a stray load shows up as NaN
and a stray store as a changed pad."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import workloads as wl
from parity_util import check_bf16, check_grad, check_lse, to_dev, to_f64

pytestmark = pytest.mark.gpu

# (B,Hq,Hkv,Sq,Sk,D,causal)
CASES = [
    (1, 2, 2, 128, 128, 32, True), (2, 4, 2, 65, 65, 32, False), (1, 2, 2, 300, 300, 96, True),
    (1, 4, 1, 200, 513, 96, True), (1, 2, 2, 257, 257, 80, False), (1, 2, 1, 129, 129, 8, True),
    (1, 2, 2, 96, 96, 120, True), (1, 2, 2, 70, 70, 40, False), (2, 8, 2, 1, 300, 96, True),
    (1, 2, 2, 64, 3000, 32, True),
]


def padded(x, pad, fill=float("nan")):
    """Device tensor [B,H,S,D] living in a [B,H,S,D+pad] allocation filled with `fill`."""
    B, H, S, D = x.shape
    buf = torch.full((B, H, S, D + pad), fill, dtype=torch.bfloat16, device="cuda")
    buf[..., :D] = to_dev(x)
    return buf, buf[..., :D]


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", CASES)
def test_headdim_parity_in_padded_poisoned_buffers(B, Hq, Hkv, Sq, Sk, D, causal):
    print("case headdim", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=1700 + D + Sq)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    pad = 8  # rows stay 16-byte aligned; the pad columns hold NaN
    (_, Q), (_, K), (_, V), (_, dO) = (padded(x[k], pad) for k in ("Q", "K", "V", "dO"))
    obuf = torch.full((B, Hq, Sq, D + pad), float("nan"), dtype=torch.bfloat16, device="cuda")
    O, LSE = attn.attn_fwd_rect(Q, K, V, x["scale"], causal, O=obuf[..., :D])
    gq = torch.full_like(obuf, float("nan"))
    gk = torch.full((B, Hkv, Sk, D + pad), float("nan"), dtype=torch.bfloat16, device="cuda")
    gv = torch.full_like(gk, float("nan"))
    dQ, dK, dV = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], causal,
                                    dQ=gq[..., :D], dK=gk[..., :D], dV=gv[..., :D])
    torch.cuda.synchronize()
    for buf in (obuf, gq, gk, gv):      # nothing was stored past column D
        assert torch.isnan(buf[..., D:]).all()
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)
    for name, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        if min(Sq, Sk) < 32 or D < 32:
            check_bf16(name, to_f64(g), r, floor_gate=False)
        else:
            check_grad(name, to_f64(g), r)


def test_headdim_96_equals_zero_padded_128_bitwise():
    """D = 96 and the same data zero-padded to D = 128 with the same scale run the same
    instructions on the same numbers."""
    B, H, S, D = 1, 2, 200, 96
    print("case headdim_pad128", flush=True)
    x = wl.random_rect_inputs(B, H, H, S, S, D, seed=1801)
    t = {k: to_dev(x[k]) for k in ("Q", "K", "V", "dO")}
    z = {k: torch.zeros((B, H, S, 128), dtype=torch.bfloat16, device="cuda") for k in t}
    for k in t:
        z[k][..., :D] = t[k]
    O1, L1 = attn.attn_fwd_rect(t["Q"], t["K"], t["V"], x["scale"], True)
    g1 = attn.attn_bwd_rect(t["Q"], t["K"], t["V"], O1, t["dO"], L1, x["scale"], True)
    O2, L2 = attn.attn_fwd_rect(z["Q"], z["K"], z["V"], x["scale"], True)
    g2 = attn.attn_bwd_rect(z["Q"], z["K"], z["V"], O2, z["dO"], L2, x["scale"], True)
    torch.cuda.synchronize()
    assert torch.equal(L1, L2)
    assert torch.equal(O1.view(torch.int16), O2[..., :D].contiguous().view(torch.int16))
    for a, b in zip(g1, g2):
        assert torch.equal(a.view(torch.int16), b[..., :D].contiguous().view(torch.int16))
        assert (b[..., D:] == 0).all()
