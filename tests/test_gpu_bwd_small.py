"""GPU parity for the fused backward of short heads (one work-group per head computes dQ, dK
and dV in one launch): at most 128 query rows and keys at D = 128, at most 256 at D = 64, with
one or several query heads per K/V head.  Shapes sit on both sides of every boundary of that form (block counts,
the four- and the eight-wave kernel, lengths that differ, padded head dimensions); each is
compared with the fp64 oracle and, where the lengths are equal, with the two-kernel backward called stage by
stage."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import binding, workloads as wl
from parity_util import check_bf16, check_grad, to_dev, to_f64

pytestmark = pytest.mark.gpu

# (B,H,Sq,Sk,D,causal)
CASES = [
    (2, 3, 1, 1, 64, True), (2, 2, 1, 100, 64, False), (1, 4, 33, 97, 64, True),
    (2, 2, 128, 128, 64, True), (1, 3, 129, 129, 64, True), (1, 2, 256, 256, 64, False),
    (1, 2, 256, 256, 64, True), (2, 2, 200, 77, 64, False), (1, 2, 77, 200, 64, True),
    (1, 2, 255, 130, 40, False), (1, 3, 65, 65, 64, False), (3, 2, 96, 96, 128, True),
    (1, 2, 128, 128, 128, False), (1, 2, 31, 128, 96, True), (1, 2, 100, 64, 120, False),
    (1, 2, 17, 17, 8, True),
]


@pytest.mark.parametrize("B,H,Sq,Sk,D,causal", CASES)
def test_fused_small_backward(B, H, Sq, Sk, D, causal):
    print("case bwd_small", B, H, Sq, Sk, D, causal, flush=True)
    x = wl.random_rect_inputs(B, H, H, Sq, Sk, D, seed=3100 + 7 * Sq + Sk + D)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd_rect(Q, K, V, x["scale"], causal)
    nan = lambda t: torch.full_like(t, float("nan"))
    ws = torch.empty(attn.attn_bwd_rect_workspace_bytes(B, H, H, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    ws.fill_(0x7F)
    dQ, dK, dV = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], causal,
                                    dQ=nan(Q), dK=nan(K), dV=nan(V), workspace=ws)
    torch.cuda.synchronize()
    if Sq == Sk:
        # the same gradients from the two-kernel path, called stage by stage (the stage-wise entry
        # point exists for the square form only)
        ws2 = torch.empty_like(ws)
        ws2.fill_(0x7F)
        two = (nan(Q), nan(K), nan(V))
        for st in (binding.STAGE_DELTA, binding.STAGE_DKDV, binding.STAGE_DQ):
            attn.attn_bwd(Q, K, V, O, dO, LSE, x["scale"], causal, dQ=two[0], dK=two[1], dV=two[2],
                          workspace=ws2, stages=st)
        torch.cuda.synchronize()
        n = B * H * 2 * Sq   # both paths leave the row statistics in the workspace
        assert torch.allclose(ws.view(torch.float32)[:n], ws2.view(torch.float32)[:n], rtol=1e-5, atol=1e-5)
        for nm, f, s in zip(("dQ", "dK", "dV"), (dQ, dK, dV), two):
            d = (f.double() - s.double()).abs()
            tol = 2.0 ** -7 * torch.maximum(f.double().abs(),
                                            torch.tensor(2.0 ** -6, device="cuda", dtype=torch.float64))
            assert bool((d <= tol).all()), (nm, d.max().item())
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    for nm, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        if min(Sq, Sk) < 32 or D < 32:
            check_bf16(nm, to_f64(g), r, floor_gate=False)
        else:
            check_grad(nm, to_f64(g), r)


# (B,Hq,Hkv,Sq,Sk,D,causal): several query heads read one K/V head; the work-group of that K/V
# head walks them and sums their dK and dV.  The fused form takes grouped heads from 256 K/V
# heads (B * Hkv) on; the last two cases sit just below and take the two-kernel path.
GQA_CASES = [
    (128, 4, 2, 64, 64, 64, True), (256, 8, 1, 100, 100, 64, False), (128, 6, 2, 33, 97, 64, True),
    (64, 8, 4, 256, 256, 64, True), (86, 6, 3, 200, 130, 48, False), (256, 4, 1, 128, 128, 128, True),
    (128, 8, 2, 77, 128, 128, False), (128, 4, 2, 1, 50, 128, True), (86, 6, 3, 129, 255, 64, True),
    (85, 6, 3, 64, 64, 64, True), (255, 2, 1, 96, 96, 128, False),
]


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", GQA_CASES)
def test_fused_small_backward_grouped_heads(B, Hq, Hkv, Sq, Sk, D, causal):
    print("case bwd_small gqa", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=3300 + 7 * Sq + Sk + D + Hq)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd_rect(Q, K, V, x["scale"], causal)
    nan = lambda t: torch.full_like(t, float("nan"))
    dQ, dK, dV = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], causal, dQ=nan(Q), dK=nan(K), dV=nan(V))
    torch.cuda.synchronize()
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    for nm, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        if min(Sq, Sk) < 32:
            check_bf16(nm, to_f64(g), r, floor_gate=False)
        else:
            check_grad(nm, to_f64(g), r)
