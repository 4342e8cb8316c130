"""GPU parity for grouped-query heads (Hq = G * Hkv) through attn_fwd_gqa / attn_bwd_gqa,
against the fp64 oracle, element by element; plus consistency with the multi-head entry
points on explicitly repeated K/V."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import workloads as wl
from parity_util import check_bf16, check_grad, check_lse, to_dev, to_f64

pytestmark = pytest.mark.gpu

# (B,Hq,Hkv,S,D,causal): multi-query, several group sizes, ragged lengths, both head dims,
# lengths below and above the dK/dV kernel's 128-key blocks and its 5-slot ring
CASES = [
    (1, 4, 2, 128, 64, False), (1, 4, 2, 128, 64, True),
    (2, 6, 2, 65, 64, True), (1, 8, 1, 33, 128, False),
    (1, 8, 1, 300, 64, True), (2, 4, 1, 257, 128, True),
    (1, 6, 3, 513, 128, False), (1, 12, 4, 160, 64, True),
    (1, 2, 2, 96, 128, True), (1, 3, 1, 1, 64, False),
]


def run(x, causal):
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd_gqa(Q, K, V, x["scale"], causal)
    dQ, dK, dV = attn.attn_bwd_gqa(Q, K, V, O, dO, LSE, x["scale"], causal)
    torch.cuda.synchronize()
    return O, LSE, dQ, dK, dV


@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal", CASES)
def test_gqa_parity(B, Hq, Hkv, S, D, causal):
    print("case gqa_parity", B, Hq, Hkv, S, D, causal, flush=True)
    x = wl.random_gqa_inputs(B, Hq, Hkv, S, D, seed=800 + S + Hq)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    O, LSE, dQ, dK, dV = run(x, causal)
    assert dK.shape == (B, Hkv, S, D) and dV.shape == (B, Hkv, S, D)
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)
    for name, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        if S < 32 and name != "dV":
            # few outputs, and delta formed from the bf16 O dominates dS (see test_gpu_bwd);
            # for S = 1 the exact dQ and dK are zero
            check_bf16(name, to_f64(g), r, floor_gate=False)
        else:
            # unit-variance inputs and sums over a group of query heads give gradients of
            # magnitude 2-10: the scale-aware reading applies (see test_gpu_bwd)
            check_grad(name, to_f64(g), r)


def test_gqa_forward_and_dq_bitwise_equal_multihead_on_repeated_kv():
    """Query head h of the grouped call and of the multi-head call on repeat_interleave'd K/V
    run the same instructions on the same data: O, LSE and dQ must agree bit for bit."""
    B, Hq, Hkv, S, D, causal = 2, 8, 2, 200, 128, True
    print("case gqa_bitwise", B, Hq, Hkv, S, D, flush=True)
    x = wl.random_gqa_inputs(B, Hq, Hkv, S, D, seed=901)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    G = Hq // Hkv
    Kr, Vr = K.repeat_interleave(G, dim=1).contiguous(), V.repeat_interleave(G, dim=1).contiguous()
    O, LSE = attn.attn_fwd_gqa(Q, K, V, x["scale"], causal)
    Om, Lm = attn.attn_fwd(Q, Kr, Vr, x["scale"], causal)
    dQ, dK, dV = attn.attn_bwd_gqa(Q, K, V, O, dO, LSE, x["scale"], causal)
    dQm, dKm, dVm = attn.attn_bwd(Q, Kr, Vr, Om, dO, Lm, x["scale"], causal)
    torch.cuda.synchronize()
    assert torch.equal(O.view(torch.int16), Om.view(torch.int16))
    assert torch.equal(LSE, Lm)
    assert torch.equal(dQ.view(torch.int16), dQm.view(torch.int16))
    # dK/dV: the grouped kernel sums the group in fp32 before rounding once; the multi-head
    # results are rounded per head, so only closeness can be asked of their sum
    s = dKm.float().view(B, Hkv, G, S, D).sum(2)
    assert (dK.float() - s).abs().max().item() <= 0.05 * max(1.0, s.abs().max().item())


def test_gqa_strided_kv_and_poisoned_outputs():
    """K/V taken as a [B,S,Hkv,D] slab (different strides from Q), outputs pre-filled with NaN."""
    B, Hq, Hkv, S, D, causal = 1, 4, 2, 150, 64, True
    print("case gqa_strided", B, Hq, Hkv, S, D, flush=True)
    x = wl.random_gqa_inputs(B, Hq, Hkv, S, D, seed=902)
    Q, dO = to_dev(x["Q"]), to_dev(x["dO"])
    Kc, Vc = to_dev(x["K"]), to_dev(x["V"])
    K = Kc.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)   # [B,Hkv,S,D] view of BSHD storage
    V = Vc.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    O = torch.full_like(Q, float("nan"))
    LSE = torch.full((B, Hq, S), float("nan"), device="cuda")
    attn.attn_fwd_gqa(Q, K, V, x["scale"], causal, O=O, LSE=LSE)
    dQ = torch.full_like(Q, float("nan"))
    dK = torch.full_like(K, float("nan"))
    dV = torch.full_like(V, float("nan"))
    attn.attn_bwd_gqa(Q, K, V, O, dO, LSE, x["scale"], causal, dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)
    for name, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        check_grad(name, to_f64(g.contiguous()), r)


def test_gqa_full_size_sampled_groups():
    """The grouped comparison shape at full size; the oracle checks two sampled K/V heads
    with their groups (the kernels treat every K/V head independently)."""
    w = wl.GQA_WORKLOADS["gqa_cmp"]
    print("case gqa_full", w, flush=True)
    G = w.Hq // w.Hkv
    x = wl.make_gqa_inputs(w)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd_gqa(Q, K, V, x["scale"], w.causal)
    dQ, dK, dV = attn.attn_bwd_gqa(Q, K, V, O, dO, LSE, x["scale"], w.causal)
    torch.cuda.synchronize()
    for kv in (3, w.B * w.Hkv - 2):
        xs = wl.make_gqa_inputs(w, kv_heads=[kv])
        Oref, Lref = oracle.attn_fwd(xs["Q"], xs["K"], xs["V"], xs["scale"], w.causal)
        ref = oracle.attn_bwd(xs["Q"], xs["K"], xs["V"], xs["dO"], xs["scale"], w.causal)
        b, hk = kv // w.Hkv, kv % w.Hkv
        qs = slice(hk * G, hk * G + G)
        check_bf16("O", to_f64(O[b:b + 1, qs]), Oref)
        check_lse(to_f64(LSE[b:b + 1, qs]), Lref)
        check_grad("dQ", to_f64(dQ[b:b + 1, qs]), ref[0])
        check_grad("dK", to_f64(dK[b:b + 1, hk:hk + 1]), ref[1])
        check_grad("dV", to_f64(dV[b:b + 1, hk:hk + 1]), ref[2])
