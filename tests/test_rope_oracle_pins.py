"""Pins of the rotary + attention composition in oracle/attn_oracle.py (CPU only).

The fused entry points are defined as the sequence rotary -> (bf16) -> attention.  These tests
tie the composition to things fixed outside it: the unit rotation, exact quarter turns against
torch fp64 autograd, the relative-position property of the rotary embedding, and the position
of the query rows of a rectangular problem."""
import numpy as np
import pytest
import torch

import oracle
from oracle import rowops_oracle as ro
from paper_2601_16238_amd import workloads as wl


def tables(S, D, base=10000.0, shift=0):
    inv = base ** (-np.arange(0, D, 2, dtype=np.float64) / D)
    ang = (np.arange(S, dtype=np.float64) + shift)[:, None] * inv[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def f64(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def test_unit_rotation_is_plain_attention():
    x = wl.random_rect_inputs(2, 4, 2, 9, 13, 16, seed=5)
    one, zero = np.ones((13, 8), np.float32), np.zeros((13, 8), np.float32)
    for causal in (False, True):
        O, LSE, Qr = oracle.attn_fwd_rope(x["Q"], x["K"], x["V"], one, zero, x["scale"], causal)
        O0, LSE0 = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
        assert np.array_equal(Qr, x["Q"]) and np.array_equal(O, O0) and np.array_equal(LSE, LSE0)
        g = oracle.attn_bwd_rope(Qr, x["K"], x["V"], x["dO"], one, zero, x["scale"], causal)
        g0 = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
        for a, b in zip(g, g0):
            assert np.array_equal(a, b)


@pytest.mark.parametrize("causal", [False, True])
def test_quarter_turns_against_torch_autograd(causal):
    """Angles that are multiples of 90 degrees make the rotated rows exact in bf16 (signed
    copies), so the composition has no rounding of its own and must agree with torch's fp64
    softmax attention on explicitly rotated queries, and with autograd THROUGH the rotation."""
    B, Hq, Hkv, Sq, Sk, D = 1, 4, 2, 6, 9, 8
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=11)
    rng = np.random.Generator(np.random.PCG64(3))
    turns = rng.integers(0, 4, size=(Sk, D // 2))
    cos = np.array([1, 0, -1, 0], np.float32)[turns]
    sin = np.array([0, 1, 0, -1], np.float32)[turns]
    O, LSE, Qr = oracle.attn_fwd_rope(x["Q"], x["K"], x["V"], cos, sin, x["scale"], causal)
    dQ, dK, dV = oracle.attn_bwd_rope(Qr, x["K"], x["V"], x["dO"], cos, sin, x["scale"], causal)
    q = torch.tensor(f64(x["Q"]), requires_grad=True)
    k = torch.tensor(f64(x["K"]), requires_grad=True)
    v = torch.tensor(f64(x["V"]), requires_grad=True)
    c = torch.tensor(cos[Sk - Sq:].astype(np.float64)); s = torch.tensor(sin[Sk - Sq:].astype(np.float64))
    h = D // 2
    qr = torch.cat([q[..., :h] * c - q[..., h:] * s, q[..., h:] * c + q[..., :h] * s], dim=-1)
    kk = k.repeat_interleave(Hq // Hkv, dim=1); vv = v.repeat_interleave(Hq // Hkv, dim=1)
    sc = float(np.float32(x["scale"]))
    scores = sc * qr @ kk.transpose(-1, -2)
    if causal:
        i = torch.arange(Sq)[:, None]; j = torch.arange(Sk)[None, :]
        scores = scores.masked_fill(j > i + Sk - Sq, float("-inf"))
    o = torch.softmax(scores, dim=-1) @ vv
    (o * torch.tensor(f64(x["dO"]))).sum().backward()
    np.testing.assert_allclose(O, o.detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(LSE, torch.logsumexp(scores, dim=-1).detach().numpy(), rtol=1e-12)
    np.testing.assert_allclose(dQ, q.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, k.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, v.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_scores_depend_on_relative_positions_only():
    """Rotating queries and keys with all positions shifted by a constant leaves the attention
    unchanged (the defining property of the rotary embedding), up to the bf16 rounding of the
    rotated rows.  A query row placed at the wrong position (the Sk - Sq offset dropped) would
    change O by order one."""
    B, H, Sq, Sk, D = 1, 2, 5, 12, 32
    x = wl.random_rect_inputs(B, H, H, Sq, Sk, D, seed=21)
    outs = []
    for shift in (0, 37):
        cos, sin = tables(Sk, D, shift=shift)
        K_rot = oracle.rope_rotate_queries(x["K"], cos, sin, Sk)   # keys: positions 0 .. Sk-1
        outs.append(oracle.attn_fwd_rope(x["Q"], K_rot, x["V"], cos, sin, x["scale"], True)[0])
    assert np.abs(outs[0] - outs[1]).max() < 2e-2
    cos, sin = tables(Sk, D)
    K_rot = oracle.rope_rotate_queries(x["K"], cos, sin, Sk)
    wrong = oracle.attn_fwd(ro_bits(x["Q"], cos[:Sq], sin[:Sq]), K_rot, x["V"], x["scale"], True)[0]
    assert np.abs(outs[0] - wrong).max() > 0.1


def ro_bits(Q, cos, sin):
    y = ro.rotary_fwd(Q, np.ascontiguousarray(cos), np.ascontiguousarray(sin))
    return wl.f32_to_bf16_bits(y.astype(np.float32))


def test_rectangular_rows_sit_at_the_last_positions():
    """The rows of a rectangular causal problem are the LAST Sq positions: its result equals the
    tail rows of the square problem on the same keys, exactly (same arithmetic per row)."""
    B, H, Sk, D, Sq = 1, 2, 11, 16, 4
    x = wl.random_rect_inputs(B, H, H, Sk, Sk, D, seed=31)
    cos, sin = tables(Sk, D)
    K_rot = oracle.rope_rotate_queries(x["K"], cos, sin, Sk)
    Of, Lf, Qf = oracle.attn_fwd_rope(x["Q"], K_rot, x["V"], cos, sin, x["scale"], True)
    Qt = np.ascontiguousarray(x["Q"][:, :, Sk - Sq:])
    Ot, Lt, Qrt = oracle.attn_fwd_rope(Qt, K_rot, x["V"], cos, sin, x["scale"], True)
    assert np.array_equal(Ot, Of[:, :, Sk - Sq:]) and np.array_equal(Lt, Lf[:, :, Sk - Sq:])
    assert np.array_equal(Qrt, Qf[:, :, Sk - Sq:])
    dOt = np.ascontiguousarray(x["dO"][:, :, Sk - Sq:])
    dOz = x["dO"].copy(); dOz[:, :, :Sk - Sq] = 0
    gt = oracle.attn_bwd_rope(Qrt, K_rot, x["V"], dOt, cos, sin, x["scale"], True)
    gf = oracle.attn_bwd_rope(Qf, K_rot, x["V"], dOz, cos, sin, x["scale"], True)
    np.testing.assert_allclose(gt[0], gf[0][:, :, Sk - Sq:], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(gt[1], gf[1], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(gt[2], gf[2], rtol=1e-12, atol=1e-14)


def test_gradient_of_unrotated_queries_by_finite_differences():
    """dQ of the composition against central differences of sum(O * dO) taken in fp64 through
    rotation and attention (torch used as plain fp64 arithmetic), for generic angles.  The
    oracle's own intermediate rounding of the rotated rows to bf16 limits the agreement to a
    few 1e-3 relative; a missing or transposed back-rotation would be off by order one."""
    B, H, S, D = 1, 2, 7, 8
    x = wl.random_rect_inputs(B, H, H, S, S, D, seed=41)
    cos, sin = tables(S, D)
    K_rot = oracle.rope_rotate_queries(x["K"], cos, sin, S)
    _, _, Qr = oracle.attn_fwd_rope(x["Q"], K_rot, x["V"], cos, sin, x["scale"], True)
    dQ = oracle.attn_bwd_rope(Qr, K_rot, x["V"], x["dO"], cos, sin, x["scale"], True)[0]
    k = torch.tensor(f64(K_rot)); v = torch.tensor(f64(x["V"])); g = torch.tensor(f64(x["dO"]))
    c = torch.tensor(cos.astype(np.float64)); s = torch.tensor(sin.astype(np.float64))
    sc, h = float(np.float32(x["scale"])), D // 2

    def loss(q):
        qr = torch.cat([q[..., :h] * c - q[..., h:] * s, q[..., h:] * c + q[..., :h] * s], dim=-1)
        scores = sc * qr @ k.transpose(-1, -2)
        i = torch.arange(S)[:, None]; j = torch.arange(S)[None, :]
        scores = scores.masked_fill(j > i, float("-inf"))
        return ((torch.softmax(scores, dim=-1) @ v) * g).sum().item()

    q0 = torch.tensor(f64(x["Q"]))
    fd = np.zeros_like(dQ)
    eps = 1e-5
    for idx in np.ndindex(*dQ.shape):
        qp, qm = q0.clone(), q0.clone()
        qp[idx] += eps; qm[idx] -= eps
        fd[idx] = (loss(qp) - loss(qm)) / (2 * eps)
    assert np.abs(dQ - fd).max() <= 1e-2 * max(1.0, np.abs(fd).max())
    assert np.abs(dQ - fd).mean() <= 2e-3 * max(1.0, np.abs(fd).mean() * 10)


def test_rotated_rows_agree_with_the_fp64_rotary_oracle():
    """The composition rounds the rotated rows to bf16 from fp32 arithmetic (the kernels'
    precision); against the fp64 rotary oracle rounded to bf16 at most a few elements per
    million may land on the neighbouring bf16 value, and never further."""
    B, H, S, D = 2, 8, 1024, 128
    x = wl.random_inputs(B, H, S, D, seed=51)
    cos, sin = tables(S, D)
    got = wl.bf16_bits_to_f32(oracle.rope_rotate_queries(x["Q"], cos, sin, S)).astype(np.float64)
    y64 = ro.rotary_fwd(x["Q"], cos, sin)
    # round the exact value directly to bf16 (ties to even), not through fp32
    m, e = np.frexp(y64)
    ref = np.ldexp(np.rint(np.ldexp(m, 8)), e - 8)
    diff = np.abs(got - ref)
    assert (diff > 0).mean() < 1e-4
    # (one bf16 step, or -- where the two products cancel -- the fp32 rounding of the products)
    assert (diff <= np.abs(ref) * 2.0 ** -7 + 2.0 ** -20).all()
    assert np.abs(got - y64).max() <= np.abs(y64).max() * 2.0 ** -8
