"""GPU parity for head dimensions above 128: D = 256 has kernels of its own (one wave per SIMD,
double-buffered tiles), and every multiple of 8 in between runs in them with the missing
columns read as zeros.  Outputs sit in NaN-poisoned, padded allocations, so a stray load shows
up as NaN and a stray store as a changed pad."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import workloads as wl
from parity_util import check_bf16, check_grad, check_lse, to_dev, to_f64

pytestmark = pytest.mark.gpu

# (B,Hq,Hkv,Sq,Sk,D,causal): several tiles and a ragged tail in both directions, grouped-query
# heads, more keys than rows, one row (decoding), a single short tile
CASES = [
    (1, 2, 2, 256, 256, 256, True), (1, 2, 2, 256, 256, 256, False),
    (2, 3, 3, 333, 333, 256, True), (1, 2, 2, 130, 130, 256, False),
    (1, 4, 2, 200, 200, 192, True), (1, 2, 1, 129, 513, 136, True),
    (1, 2, 2, 65, 65, 160, False), (1, 8, 2, 1, 300, 256, True),
    (1, 2, 2, 17, 17, 256, True), (1, 1, 1, 700, 700, 224, True),
]


def padded(x, pad, fill=float("nan")):
    B, H, S, D = x.shape
    buf = torch.full((B, H, S, D + pad), fill, dtype=torch.bfloat16, device="cuda")
    buf[..., :D] = to_dev(x)
    return buf, buf[..., :D]


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", CASES)
def test_wide_headdim_parity_in_padded_poisoned_buffers(B, Hq, Hkv, Sq, Sk, D, causal):
    print("case headdim_wide", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=2600 + D + Sq)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    pad = 8
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
        if min(Sq, Sk) < 32:
            check_bf16(name, to_f64(g), r, floor_gate=False)
        else:
            check_grad(name, to_f64(g), r)


def test_wide_headdim_192_equals_zero_padded_256_bitwise():
    """D = 192 and the same data zero-padded to D = 256 with the same scale run the same
    instructions on the same numbers."""
    B, H, S, D = 1, 2, 200, 192
    print("case headdim_pad256", flush=True)
    x = wl.random_rect_inputs(B, H, H, S, S, D, seed=2801)
    t = {k: to_dev(x[k]) for k in ("Q", "K", "V", "dO")}
    z = {k: torch.zeros((B, H, S, 256), dtype=torch.bfloat16, device="cuda") for k in t}
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


def test_wide_headdim_large_scores_move_the_reference_max():
    """Scores of several hundred: the lazily moved reference max of the D = 256 forward must
    track them (its rescaling path runs again and again); LSE within 1e-5 + 1e-5 |LSE|."""
    print("case headdim_wide_large_scores", flush=True)
    B, H, S, D = 1, 2, 500, 256
    x = wl.random_inputs(B, H, S, D, seed=2901, sigma=6.0)
    for causal in (True, False):
        Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
        assert Lref.max() > 100
        O, LSE = attn.attn_fwd(to_dev(x["Q"]), to_dev(x["K"]), to_dev(x["V"]), x["scale"], causal)
        torch.cuda.synchronize()
        got = to_f64(LSE)
        assert np.isfinite(got).all() and (np.abs(got - Lref) <= 1e-5 + 1e-5 * np.abs(Lref)).all()
        d = np.abs(to_f64(O) - Oref)
        assert d.max() <= 2e-2 * max(1.0, np.abs(Oref).max()) and np.isfinite(d).all()
