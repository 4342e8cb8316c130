"""Rotary embedding fused into the attention calls (attn_fwd_rope / attn_bwd_rope) against the
composed fp64 oracle, and bit for bit against the unfused GPU sequence rotary kernel ->
attention kernel."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import binding, rowops, workloads as wl
from parity_util import check_bf16, check_grad, check_lse, to_dev, to_f64

pytestmark = pytest.mark.gpu


def tables(S, D, base=10000.0):
    inv = base ** (-np.arange(0, D, 2, dtype=np.float64) / D)
    ang = np.arange(S, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


CASES = [  # B, Hq, Hkv, Sq, Sk, D, causal
    (1, 2, 2, 128, 128, 64, False),
    (2, 4, 2, 300, 300, 128, True),
    (1, 8, 2, 77, 1000, 128, True),      # rectangular: the rows are the last 77 positions
    (2, 8, 8, 513, 513, 64, True),
    (1, 8, 2, 3, 4096, 128, True),       # few rows against a long cache: forward split over the keys
    (1, 2, 1, 641, 641, 128, False),
    (2, 8, 2, 1, 3000, 128, True),       # decoding: the query heads of a K/V head share the last position
    (1, 8, 8, 1, 513, 64, True), (1, 4, 2, 20, 700, 64, True),
    (2, 3, 3, 100, 100, 128, True), (1, 4, 4, 200, 256, 64, True),   # short heads: the fused one-launch backward
    (64, 8, 4, 60, 90, 64, True),         # ... and its grouped-head form (256 K/V heads)
    (2, 16, 2, 8, 2500, 128, True), (1, 12, 2, 5, 1100, 64, True),   # a few new rows, grouped heads: packed rows, each at its position
]


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", CASES)
def test_rope_fwd_bwd_against_the_oracle_and_the_unfused_sequence(B, Hq, Hkv, Sq, Sk, D, causal):
    print("case rope", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=1300 + Sq + D)
    cos, sin = tables(Sk, D)
    K_rot_bits = oracle.rope_rotate_queries(x["K"], cos, sin, Sk)   # keys: positions 0..Sk-1
    Oref, Lref, Qr_ref = oracle.attn_fwd_rope(x["Q"], K_rot_bits, x["V"], cos, sin, x["scale"], causal)
    gref = oracle.attn_bwd_rope(Qr_ref, K_rot_bits, x["V"], x["dO"], cos, sin, x["scale"], causal)

    Q, K_rot, V, dO = (to_dev(b) for b in (x["Q"], K_rot_bits, x["V"], x["dO"]))
    c, s = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    O, LSE, Q_rot = attn.attn_fwd_rope(Q, K_rot, V, c, s, x["scale"], causal)
    dQ, dK, dV = attn.attn_bwd_rope(Q_rot, K_rot, V, O, dO, LSE, c, s, x["scale"], causal)
    torch.cuda.synchronize()
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)
    # the rotated rows: both sides decide the bf16 value in fp32 with the same fused
    # multiply-adds, so they must agree bit for bit
    assert np.array_equal(Q_rot.cpu().view(torch.int16).numpy().view(np.uint16), Qr_ref)
    for name, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), gref):
        check_grad(name, to_f64(g), r)

    # unfused: the rotary kernel on Q, then the plain rectangular forward -- the same bits
    pos0 = Sk - Sq
    Q_rot2 = rowops.rotary_fwd(Q, c[pos0:pos0 + Sq].contiguous(), s[pos0:pos0 + Sq].contiguous())
    O2, LSE2 = attn.attn_fwd_rect(Q_rot2, K_rot, V, x["scale"], causal)
    torch.cuda.synchronize()
    assert torch.equal(Q_rot.view(torch.int16), Q_rot2.view(torch.int16))
    assert torch.equal(O.view(torch.int16), O2.view(torch.int16))
    assert torch.equal(LSE, LSE2)
    # and the backward's dK, dV (which never see the rotation) equal the plain backward's
    dQ2, dK2, dV2 = attn.attn_bwd_rect(Q_rot, K_rot, V, O, dO, LSE, x["scale"], causal)
    torch.cuda.synchronize()
    assert torch.equal(dK.view(torch.int16), dK2.view(torch.int16))
    assert torch.equal(dV.view(torch.int16), dV2.view(torch.int16))


def test_rope_forward_without_storing_the_rotated_rows():
    B, H, S, D = 1, 2, 200, 128
    x = wl.random_rect_inputs(B, H, H, S, S, D, seed=77)
    cos, sin = tables(S, D)
    Q, K, V = (to_dev(x[k]) for k in ("Q", "K", "V"))
    c, s = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    O1, L1, Qr = attn.attn_fwd_rope(Q, K, V, c, s, x["scale"], True)
    O2, L2, none = attn.attn_fwd_rope(Q, K, V, c, s, x["scale"], True, want_q_rot=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(O1.view(torch.int16), O2.view(torch.int16)) and torch.equal(L1, L2)


def test_rope_entry_points_reject_what_they_cannot_do():
    """Head dimensions other than 64 / 128 and Sk < Sq: ATTN_ERR_SHAPE, decided on the host."""
    fake = ctypes.c_void_p(0x10000)
    for Sq, Sk, D in ((16, 16, 96), (16, 16, 32), (32, 16, 64)):
        p = binding.make_rect_params(1, 2, 2, Sq, Sk, D, 0.125, False)
        rc = binding.lib().attn_fwd_rope(fake, fake, fake, fake, fake, fake, fake, None, None, 0,
                                         ctypes.byref(p), None)
        assert rc == binding.ATTN_ERR_SHAPE, (Sq, Sk, D, rc)
        rc = binding.lib().attn_bwd_rope(fake, fake, fake, fake, fake, fake, fake, fake, fake, fake,
                                         fake, fake, 1 << 20, ctypes.byref(p), None)
        assert rc == binding.ATTN_ERR_SHAPE, (Sq, Sk, D, rc)
    p = binding.make_rect_params(1, 2, 2, 16, 16, 64, 0.125, False)
    rc = binding.lib().attn_fwd_rope(fake, fake, fake, None, fake, fake, fake, None, None, 0,
                                     ctypes.byref(p), None)
    assert rc == binding.ATTN_ERR_NULL
