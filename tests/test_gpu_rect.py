"""GPU parity for rectangular attention (Sq query rows against Sk keys, causal mask aligned
bottom-right) through attn_fwd_rect / attn_bwd_rect, against the fp64 oracle element by
element: decoding (Sq = 1), chunked prefill, more rows than keys, with and without the
forward's split over the keys; plus consistency with the square entry points."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import workloads as wl
from parity_util import bf16_round, check_bf16, check_grad, check_lse, f16_round, to_dev, to_f64

pytestmark = pytest.mark.gpu

# (B,Hq,Hkv,Sq,Sk,D,causal): decode rows, ragged chunks crossing the 64-key tiles and the
# 128-key / 256-row blocks, Sk < Sq without a mask, both head dims, grouped heads
CASES = [
    (2, 8, 2, 1, 300, 64, True), (1, 4, 4, 1, 1, 128, True), (1, 4, 1, 1, 77, 128, False),
    (2, 4, 2, 100, 356, 128, True), (1, 2, 2, 33, 64, 64, True), (1, 2, 1, 257, 300, 64, True),
    (1, 4, 4, 150, 77, 64, False), (1, 2, 2, 64, 1000, 128, False), (1, 3, 3, 300, 513, 128, True),
    (1, 2, 2, 7, 2049, 64, True), (1, 1, 1, 129, 129, 128, True),
    # a few new rows per sequence with grouped heads: the G x Sq rows of a K/V head run as one
    # packed head (mask by position r % Sq); 16, 30 and 32 rows; ragged last key tile
    (2, 8, 2, 4, 3000, 128, True), (1, 12, 2, 5, 1025, 64, True), (1, 16, 2, 4, 777, 128, False),
    (1, 8, 4, 3, 5, 128, True), (2, 4, 2, 16, 4100, 128, True),
    # ... up to one query tile of 128 packed rows (64, 128 and 108 rows: the last wave partly
    # filled; D = 256; 48 rows at D = 64 and 64 rows at D = 96)
    (1, 16, 2, 8, 3000, 128, True), (2, 8, 1, 16, 2100, 128, True), (1, 24, 2, 9, 1000, 128, True),
    (1, 32, 4, 6, 1500, 256, True), (1, 12, 2, 8, 700, 64, True), (1, 16, 2, 8, 900, 96, False),
]


def run(x, causal, split=True):
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd_rect(Q, K, V, x["scale"], causal, split=split)
    dQ, dK, dV = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], causal)
    torch.cuda.synchronize()
    return O, LSE, dQ, dK, dV


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", CASES)
def test_rect_parity(B, Hq, Hkv, Sq, Sk, D, causal):
    print("case rect_parity", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=1200 + Sq + Sk)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    O, LSE, dQ, dK, dV = run(x, causal)
    assert O.shape == (B, Hq, Sq, D) and dK.shape == (B, Hkv, Sk, D) and dV.shape == dK.shape
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)
    for name, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        if min(Sq, Sk) < 32:
            # few terms per output: delta formed from the bf16 O dominates dS (see
            # test_gpu_bwd); with one key the exact dQ and dK are zero
            check_bf16(name, to_f64(g), r, floor_gate=False)
        else:
            check_grad(name, to_f64(g), r)


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", [
    (1, 4, 2, 1, 4096, 128, True), (2, 2, 2, 16, 2100, 64, True), (1, 2, 1, 200, 3000, 128, True),
    (1, 8, 8, 1, 1024, 64, False), (1, 2, 2, 300, 1500, 128, False),
    # many splits (the merge walks a row's splits in several steps): 125, 63, and 32 at D = 256
    (1, 8, 2, 1, 40000, 128, True), (1, 4, 4, 1, 20000, 64, False), (1, 2, 2, 64, 8192, 256, False),
    # a single row (the merge's work-group holds two rows at D = 64: one of them is past the end),
    # and four splits at D = 256
    (1, 1, 1, 1, 3000, 64, False), (1, 2, 2, 64, 1024, 256, True),
    # packed grouped heads with several new rows: the last split starts inside the last Sq keys
    # (rows that see none of its keys), many splits, D = 256
    (1, 8, 2, 4, 8193, 128, True), (1, 4, 1, 8, 40000, 128, True), (1, 8, 2, 3, 5000, 256, True)])
def test_rect_forward_split_matches_unsplit_and_oracle(B, Hq, Hkv, Sq, Sk, D, causal):
    """Shapes for which the library's plan splits the keys: the merged result must match the
    oracle, and the one-kernel result (no workspace) as well."""
    print("case rect_split", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    assert attn.attn_fwd_rect_workspace_bytes(B, Hq, Hkv, Sq, Sk, D) > 0, "plan does not split"
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=1300 + Sq + Sk)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    Q, K, V = (to_dev(x[k]) for k in ("Q", "K", "V"))
    for split in (True, False):
        O = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        LSE = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
        attn.attn_fwd_rect(Q, K, V, x["scale"], causal, O=O, LSE=LSE, split=split)
        torch.cuda.synchronize()
        check_bf16("O split=%s" % split, to_f64(O), Oref)
        check_lse(to_f64(LSE), Lref)


def test_rect_square_is_bitwise_the_gqa_call():
    """Sq = Sk through the rectangular entry points runs the same kernels on the same data
    as the grouped-query entry points."""
    B, Hq, Hkv, S, D, causal = 2, 4, 2, 200, 128, True
    print("case rect_square", B, Hq, Hkv, S, D, flush=True)
    x = wl.random_gqa_inputs(B, Hq, Hkv, S, D, seed=1401)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O1, L1 = attn.attn_fwd_gqa(Q, K, V, x["scale"], causal)
    g1 = attn.attn_bwd_gqa(Q, K, V, O1, dO, L1, x["scale"], causal)
    O2, L2 = attn.attn_fwd_rect(Q, K, V, x["scale"], causal)
    g2 = attn.attn_bwd_rect(Q, K, V, O2, dO, L2, x["scale"], causal)
    torch.cuda.synchronize()
    assert torch.equal(O1.view(torch.int16), O2.view(torch.int16)) and torch.equal(L1, L2)
    for a, b in zip(g1, g2):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_rect_causal_tail_of_square_problem():
    """The rectangular causal result equals the last Sq rows of the square causal problem on
    the same keys (the property that pins the oracle's mask), here on the GPU path: O, LSE
    and dQ of those rows bit for bit (same tiles, same order), dK/dV to rounding."""
    B, H, Sq, Sk, D = 1, 2, 256, 768, 128
    print("case rect_tail", B, H, Sq, Sk, D, flush=True)
    x = wl.random_rect_inputs(B, H, H, Sq, Sk, D, seed=1402)
    Qs = np.zeros((B, H, Sk, D), np.uint16); Qs[:, :, Sk - Sq:] = x["Q"]
    Gs = np.zeros((B, H, Sk, D), np.uint16); Gs[:, :, Sk - Sq:] = x["dO"]
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, L = attn.attn_fwd_rect(Q, K, V, x["scale"], True, split=False)
    dQ, dK, dV = attn.attn_bwd_rect(Q, K, V, O, dO, L, x["scale"], True)
    Os, Ls = attn.attn_fwd(to_dev(Qs), K, V, x["scale"], True)
    dQs, dKs, dVs = attn.attn_bwd(to_dev(Qs), K, V, Os, to_dev(Gs), Ls, x["scale"], True)
    torch.cuda.synchronize()
    assert torch.equal(O.view(torch.int16), Os[:, :, Sk - Sq:].contiguous().view(torch.int16))
    assert torch.equal(L, Ls[:, :, Sk - Sq:])
    assert torch.equal(dQ.view(torch.int16), dQs[:, :, Sk - Sq:].contiguous().view(torch.int16))
    np.testing.assert_allclose(to_f64(dK), to_f64(dKs), rtol=0, atol=2e-2)
    np.testing.assert_allclose(to_f64(dV), to_f64(dVs), rtol=0, atol=2e-2)


def test_rect_strided_cache_and_poisoned_outputs():
    """K/V taken as the first Sk rows of a longer cache allocation (row stride and head stride
    of the cache), outputs pre-filled with NaN: every output element is written, nothing
    beyond Sk is read into the result."""
    B, Hq, Hkv, Sq, Sk, cap, D = 2, 4, 2, 5, 333, 512, 64
    print("case rect_strided", B, Hq, Hkv, Sq, Sk, D, flush=True)
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=1403)
    cacheK = torch.full((B, Hkv, cap, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    cacheV = torch.full((B, Hkv, cap, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    cacheK[:, :, :Sk] = to_dev(x["K"]); cacheV[:, :, :Sk] = to_dev(x["V"])
    K, V = cacheK[:, :, :Sk], cacheV[:, :, :Sk]
    Q, dO = to_dev(x["Q"]), to_dev(x["dO"])
    O, LSE = attn.attn_fwd_rect(Q, K, V, x["scale"], True)
    dK = torch.full_like(cacheK, float("nan"))[:, :, :Sk]
    dV = torch.full_like(cacheV, float("nan"))[:, :, :Sk]
    dQ, dK, dV = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], True, dK=dK, dV=dV)
    torch.cuda.synchronize()
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], True)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], True)
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)
    for name, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        check_bf16(name, to_f64(g), r, floor_gate=False)


def test_rect_full_size_sampled_heads():
    """The bench shapes at full size, in the launch configuration bench.py times: sampled K/V
    heads (with their query groups) against the oracle."""
    for name, heads in (("decode_cmp", [0, 37, 63]), ("spec_decode", [1, 62]), ("prefill_chunk", [5])):
        w = wl.RECT_WORKLOADS[name]
        print("case rect_full", name, flush=True)
        full = wl.make_rect_inputs(w)
        Q, K, V, dO = (to_dev(full[k]) for k in ("Q", "K", "V", "dO"))
        O, LSE = attn.attn_fwd_rect(Q, K, V, full["scale"], w.causal)
        dQ, dK, dV = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, full["scale"], w.causal)
        torch.cuda.synchronize()
        G = w.Hq // w.Hkv
        for kvh in heads:
            sub = wl.make_rect_inputs(w, kv_heads=[kvh])
            b, hk = kvh // w.Hkv, kvh % w.Hkv
            qs = slice(hk * G, hk * G + G)
            assert np.array_equal(sub["K"][0, 0], full["K"][b, hk])
            Oref, Lref = oracle.attn_fwd(sub["Q"], sub["K"], sub["V"], sub["scale"], w.causal)
            ref = oracle.attn_bwd(sub["Q"], sub["K"], sub["V"], sub["dO"], sub["scale"], w.causal)
            check_bf16("O", to_f64(O[b, qs]), Oref[0])
            check_lse(to_f64(LSE[b, qs]), Lref[0])
            if w.Sq >= 32:
                check_grad("dQ", to_f64(dQ[b, qs]), ref[0][0])
                check_grad("dK", to_f64(dK[b, hk]), ref[1][0, 0])
                check_grad("dV", to_f64(dV[b, hk]), ref[2][0, 0])
            else:
                check_bf16("dQ", to_f64(dQ[b, qs]), ref[0][0], floor_gate=False)
                check_bf16("dK", to_f64(dK[b, hk]), ref[1][0, 0], floor_gate=False)
                check_bf16("dV", to_f64(dV[b, hk]), ref[2][0, 0], floor_gate=False)


@pytest.mark.parametrize("B,Hq,Hkv,Sk,D,f16", [
    (16, 16, 16, 4099, 128, False),    # every head its own K/V: the masked kernel
    (8, 32, 8, 16389, 128, False),     # grouped heads packed into one head of 4 rows: no mask
    (32, 16, 16, 4200, 64, True),      # D = 64, fp16
])
def test_decode_with_more_keys_and_values_than_the_last_level_cache(B, Hq, Hkv, Sk, D, f16):
    """Decoding against more K and V than the last-level cache holds (every byte then really comes
    from HBM, through the decoding launches' non-temporal transfers): sampled heads against the
    oracle, with the planned split and in one kernel."""
    print("case decode_large", B, Hq, Hkv, Sk, D, f16, flush=True)
    assert B * Hkv * Sk * D * 4 > 256 << 20
    dt = torch.float16 if f16 else torch.bfloat16
    g = torch.Generator(device="cuda"); g.manual_seed(1500 + Sk)
    Q = torch.randn((B, Hq, 1, D), device="cuda", generator=g).to(dt)
    K = torch.randn((B, Hkv, Sk, D), device="cuda", generator=g).to(dt)
    V = torch.randn((B, Hkv, Sk, D), device="cuda", generator=g).to(dt)
    scale = wl.default_scale(D)
    # (the first two shapes split their keys, the third has a work-group per head and does not)
    assert (attn.attn_fwd_rect_workspace_bytes(B, Hq, Hkv, 1, Sk, D) > 0) == (B * Hkv < 512)
    O, LSE = attn.attn_fwd_rect(Q, K, V, scale, True)
    O1, LSE1 = attn.attn_fwd_rect(Q, K, V, scale, True, split=False)
    torch.cuda.synchronize()
    G = Hq // Hkv
    bits = (lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16))
    for b, hk in ((0, 0), (B // 2, Hkv - 1), (B - 1, Hkv // 2)):
        qs = slice(hk * G, hk * G + G)
        q, k, v = bits(Q[b:b + 1, qs]), bits(K[b:b + 1, hk:hk + 1]), bits(V[b:b + 1, hk:hk + 1])
        Oref, Lref = oracle.attn_fwd(q, k, v, scale, True, dtype="f16" if f16 else "bf16")
        for name, o, l in (("split", O, LSE), ("one kernel", O1, LSE1)):
            check_bf16("O " + name, to_f64(o[b:b + 1, qs]), Oref, rnd=f16_round if f16 else bf16_round)
            check_lse(to_f64(l[b:b + 1, qs]), Lref)


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", [
    (8, 32, 32, 300, 300, 128, True),     # 256 heads x 2 key blocks of 192: ragged second block
    (4, 64, 64, 200, 450, 96, True),      # rectangular, head dimension below the kernel's 128
    (16, 64, 16, 130, 385, 128, False),   # grouped heads: 256 K/V heads x 3 blocks, group loop
    (2, 128, 128, 64, 1000, 72, True),    # few rows against many keys
])
def test_backward_with_192_key_work_groups(B, Hq, Hkv, Sq, Sk, D, causal):
    """At D > 64 launches of at least 512 dK/dV work-groups use work-groups of six producer and
    six consumer waves that own 192 keys; these shapes reach that path with ragged last blocks,
    padded head dimensions, grouped heads and rectangular problems."""
    assert (B * Hkv) * ((Sk + 191) // 192) >= 512
    test_rect_parity(B, Hq, Hkv, Sq, Sk, D, causal)


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", [
    (1, 8, 2, 300, 2000, 128, True), (2, 4, 4, 512, 1100, 64, False), (1, 4, 4, 1030, 1030, 128, True),
    (1, 2, 1, 257, 4100, 128, True), (1, 2, 2, 700, 3000, 64, True), (1, 32, 8, 512, 4096, 128, True)])
def test_rect_backward_with_dq_split_over_the_keys(B, Hq, Hkv, Sq, Sk, D, causal):
    """Few query tiles against many keys: the plan splits the dQ kernel over the keys (the
    workspace then holds fp32 partial results next to the row statistics).  The merged dQ must
    match the oracle, and the unsplit dQ (a workspace that only holds the statistics) to the
    rounding of the output; dK and dV do not depend on the plan at all."""
    print("case rect_dq_split", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    full = attn.attn_bwd_rect_workspace_bytes(B, Hq, Hkv, Sq, Sk, D)
    stats = (8 * B * Hq * Sq + 255) // 256 * 256
    assert full > stats, "plan does not split"
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=1400 + Sq + Sk)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd_rect(Q, K, V, x["scale"], causal)
    ws = torch.full((full,), 0x7F, dtype=torch.uint8, device="cuda")   # poisoned: nothing may be relied on
    dQ, dK, dV = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], causal, workspace=ws)
    dQ1, dK1, dV1 = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], causal, workspace=ws[:stats])
    torch.cuda.synchronize()
    for name, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        check_grad(name, to_f64(g), r)
    check_grad("unsplit dQ", to_f64(dQ1), ref[0])
    assert torch.equal(dK.view(torch.int16), dK1.view(torch.int16))
    assert torch.equal(dV.view(torch.int16), dV1.view(torch.int16))
    # the two dQ differ only by the order of fp32 additions: rarely, and then by one bf16 step
    # (or, where the terms cancel, by the fp32 rounding of the partial sums)
    a, b = to_f64(dQ), to_f64(dQ1)
    assert (a != b).mean() < 0.05
    assert (np.abs(a - b) <= np.abs(b) * 2.0 ** -7 + 1e-4 * np.abs(b).max()).all()
    # and a second call on the same workspace gives the same bits (nothing is accumulated)
    dQ2, _, _ = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], causal, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(dQ.view(torch.int16), dQ2.view(torch.int16))


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", [
    (2, 8, 2, 4, 3000, 128, True), (1, 12, 2, 5, 1025, 64, True), (1, 16, 2, 8, 2000, 128, True),
    (1, 8, 2, 4, 700, 256, True)])
def test_packed_rows_of_grouped_heads_in_bshd_tensors(B, Hq, Hkv, Sq, Sk, D, causal):
    """A few new rows per sequence with Q and O stored [B,S,H,D]: the rows of a query head are
    not contiguous to the next head's, so a packed row is addressed by (head, position) (at
    D = 256 the problem runs unpacked).  Forward with the planned split and in one kernel."""
    print("case packed_bshd", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=1600 + Sq + Sk)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    Q = to_dev(x["Q"]).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)   # BSHD memory
    assert Q.stride() == (Sq * Hq * D, D, Hq * D, 1)
    K, V = to_dev(x["K"]), to_dev(x["V"])
    for split in (True, False):
        O = torch.full((B, Sq, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda").permute(0, 2, 1, 3)
        LSE = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
        attn.attn_fwd_rect(Q, K, V, x["scale"], causal, O=O, LSE=LSE, split=split)
        torch.cuda.synchronize()
        check_bf16("O split=%s" % split, to_f64(O), Oref)
        check_lse(to_f64(LSE), Lref)
