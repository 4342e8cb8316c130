"""Pins for the fp64 oracles of the row-wise kernels (RMSNorm fwd, LayerNorm fwd+bwd, rotary
fwd): closed forms, invariants, finite differences and torch's fp64 routines -- nothing here
comes from the oracle itself or from the GPU path.  The paper prints no values for these
operators (latencies only), so parity with printed values is unpinned."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_16238_amd import workloads as wl

ro = oracle.rowops


def bits(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def f64(b):
    return wl.bf16_bits_to_f32(b).astype(np.float64)


def rnd(shape, seed, sigma=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    return bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma))


def params(cols, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal(cols).astype(np.float32) * 0.5 + 1.0,
            rng.standard_normal(cols).astype(np.float32) * 0.3)


SHAPES = [(1, 8), (3, 16), (5, 40), (2, 1024), (7, 264)]


@pytest.mark.parametrize("rows,cols", SHAPES)
def test_rmsnorm_against_torch_fp64_and_unit_rms(rows, cols):
    x = rnd((rows, cols), 11 + cols)
    w, _ = params(cols, 12)
    eps = 1e-6
    y = ro.rmsnorm_fwd(x, w, eps)
    xt = torch.tensor(f64(x))
    want = xt * torch.rsqrt(xt.pow(2).mean(-1, keepdim=True) + float(np.float32(eps))) * torch.tensor(w, dtype=torch.float64)
    np.testing.assert_allclose(y, want.numpy(), rtol=1e-13, atol=1e-13)
    # with w = 1 and eps = 0 every output row has root-mean-square exactly 1
    y1 = ro.rmsnorm_fwd(x, np.ones(cols, np.float32), 0.0)
    np.testing.assert_allclose(np.sqrt((y1 ** 2).mean(-1)), 1.0, rtol=1e-13)


def test_rmsnorm_scale_invariance_and_weight_position():
    """eps = 0: scaling a row by a power of two (exact in bf16) leaves y unchanged; the weight
    multiplies column-wise (a one-hot weight selects one column)."""
    x = rnd((4, 32), 21)
    w, _ = params(32, 22)
    y = ro.rmsnorm_fwd(x, w, 0.0)
    y4 = ro.rmsnorm_fwd(bits(f64(x) * 4.0), w, 0.0)
    np.testing.assert_allclose(y4, y, rtol=1e-14, atol=0)
    onehot = np.zeros(32, np.float32); onehot[5] = 2.0
    y5 = ro.rmsnorm_fwd(x, onehot, 0.0)
    assert (np.delete(y5, 5, axis=1) == 0).all()
    np.testing.assert_allclose(y5[:, 5], 2.0 * f64(x)[:, 5] / np.sqrt((f64(x) ** 2).mean(-1)), rtol=1e-14)
    # eps enters under the root, added to the MEAN of squares: constant rows x = c give c/sqrt(c^2+eps)
    xc = bits(np.full((1, 8), 0.5, np.float32))
    np.testing.assert_allclose(ro.rmsnorm_fwd(xc, np.ones(8, np.float32), 0.75), 0.5 / np.sqrt(0.25 + 0.75), rtol=1e-14)


@pytest.mark.parametrize("rows,cols", SHAPES[1:])
def test_layernorm_forward_against_torch_fp64_and_moments(rows, cols):
    x = rnd((rows, cols), 31 + cols, sigma=2.0)
    w, b = params(cols, 32)
    eps = 1e-5
    y, mean, rstd = ro.layernorm_fwd(x, w, b, eps)
    xt = torch.tensor(f64(x))
    want = torch.nn.functional.layer_norm(xt, (cols,), torch.tensor(w, dtype=torch.float64),
                                          torch.tensor(b, dtype=torch.float64), float(np.float32(eps)))
    np.testing.assert_allclose(y, want.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(mean, f64(x).mean(-1), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(rstd, 1.0 / np.sqrt(f64(x).var(-1) + float(np.float32(eps))), rtol=1e-13)
    # w = 1, b = 0, eps = 0: rows have mean 0 and (biased) variance exactly 1
    y1, _, _ = ro.layernorm_fwd(x, np.ones(cols, np.float32), np.zeros(cols, np.float32), 0.0)
    np.testing.assert_allclose(y1.mean(-1), 0.0, atol=1e-13)
    np.testing.assert_allclose((y1 ** 2).mean(-1), 1.0, rtol=1e-12)


def test_layernorm_shift_invariance_and_bias():
    x = rnd((3, 16), 41)
    w, b = params(16, 42)
    y, _, _ = ro.layernorm_fwd(x, w, b, 1e-5)
    xs = bits(f64(x) + 8.0)          # exact in bf16? not in general: compare against its own widening
    ys, means, _ = ro.layernorm_fwd(xs, w, b, 1e-5)
    y_again, _, _ = ro.layernorm_fwd(bits(f64(xs) - 0.0), w, b, 1e-5)
    np.testing.assert_array_equal(ys, y_again)
    # exact shift: integers are exact in bf16 up to 256
    xi = bits(np.arange(16, dtype=np.float32)[None, :].repeat(2, 0))
    xj = bits(np.arange(16, dtype=np.float32)[None, :].repeat(2, 0) + 64.0)
    yi, mi, ri = ro.layernorm_fwd(xi, w, b, 1e-5)
    yj, mj, rj = ro.layernorm_fwd(xj, w, b, 1e-5)
    np.testing.assert_allclose(yi, yj, rtol=0, atol=1e-13)
    np.testing.assert_allclose(mj - mi, 64.0, rtol=0, atol=1e-13)
    np.testing.assert_allclose(ri, rj, rtol=1e-14)
    # the bias is added after the scaling: with w = 0 the output is the bias
    y0, _, _ = ro.layernorm_fwd(x, np.zeros(16, np.float32), b, 1e-5)
    np.testing.assert_allclose(y0, np.broadcast_to(b.astype(np.float64), y0.shape), rtol=0, atol=0)


@pytest.mark.parametrize("rows,cols", [(3, 16), (5, 40), (4, 264)])
def test_layernorm_backward_against_torch_autograd_and_identities(rows, cols):
    x = rnd((rows, cols), 51 + cols, sigma=1.5)
    dy = rnd((rows, cols), 52 + cols)
    w, b = params(cols, 53)
    eps = 1e-5
    dx, dw, db = ro.layernorm_bwd(dy, x, w, eps)
    xt = torch.tensor(f64(x), requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    bt = torch.tensor(b, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.layer_norm(xt, (cols,), wt, bt, float(np.float32(eps)))
    gx, gw, gb = torch.autograd.grad(yt, (xt, wt, bt), grad_outputs=torch.tensor(f64(dy)))
    np.testing.assert_allclose(dx, gx.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dw, gw.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(db, gb.numpy(), rtol=1e-12, atol=1e-12)
    # structure of the Jacobian: dx rows sum to zero and, for eps = 0 (then sum xhat^2 = cols),
    # are orthogonal to the centred row
    np.testing.assert_allclose(dx.sum(-1), 0.0, atol=1e-12)
    dx0, _, _ = ro.layernorm_bwd(dy, x, w, 0.0)
    xh = (f64(x) - f64(x).mean(-1, keepdims=True))
    np.testing.assert_allclose((dx0 * xh).sum(-1), 0.0, atol=1e-11)
    np.testing.assert_allclose(db, f64(dy).sum(0), rtol=1e-13)


def test_layernorm_backward_finite_differences():
    rows, cols = 2, 8
    x = rnd((rows, cols), 61)
    dy = rnd((rows, cols), 62)
    w, b = params(cols, 63)
    eps = 1e-3
    dx, dw, _ = ro.layernorm_bwd(dy, x, w, eps)

    def loss(xv, wv):   # sum(y * dy) in double, written out with numpy
        mu = xv.mean(-1, keepdims=True)
        var = ((xv - mu) ** 2).mean(-1, keepdims=True)
        y = (xv - mu) / np.sqrt(var + float(np.float32(eps))) * wv + b.astype(np.float64)
        return float((y * f64(dy)).sum())

    x0, w0, h = f64(x), w.astype(np.float64), 1e-6
    for idx in [(0, 0), (1, 3), (0, 7)]:
        xp, xm = x0.copy(), x0.copy(); xp[idx] += h; xm[idx] -= h
        assert abs((loss(xp, w0) - loss(xm, w0)) / (2 * h) - dx[idx]) < 1e-7
    for j in (0, 5):
        wp, wm = w0.copy(), w0.copy(); wp[j] += h; wm[j] -= h
        assert abs((loss(x0, wp) - loss(x0, wm)) / (2 * h) - dw[j]) < 1e-7


def rope_tables(S, D, base=10000.0):
    inv = base ** (-np.arange(0, D, 2, dtype=np.float64) / D)
    ang = np.arange(S, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


@pytest.mark.parametrize("B,H,S,D", [(1, 1, 1, 2), (2, 3, 7, 8), (1, 2, 33, 64), (1, 1, 5, 128)])
def test_rotary_is_complex_multiplication_on_half_split_pairs(B, H, S, D):
    x = rnd((B, H, S, D), 71 + D)
    cos, sin = rope_tables(S, D)
    y = ro.rotary_fwd(x, cos, sin)
    xv = f64(x)
    z = (xv[..., :D // 2] + 1j * xv[..., D // 2:]) * (cos.astype(np.float64) + 1j * sin.astype(np.float64))
    np.testing.assert_allclose(y[..., :D // 2], z.real, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(y[..., D // 2:], z.imag, rtol=1e-14, atol=1e-15)
    # position 0 has angle 0: identity
    np.testing.assert_array_equal(y[:, :, 0], xv[:, :, 0])


def test_rotary_preserves_pair_norms_and_inverts_with_negated_sine():
    B, H, S, D = 1, 2, 9, 16
    x = rnd((B, H, S, D), 81)
    ang = np.random.Generator(np.random.PCG64(82)).uniform(-3, 3, size=(S, D // 2))
    # exact unit pairs in float32 are rare; use the tables as given and compare norms with
    # the factor cos^2 + sin^2 of the (rounded) table entries
    cos, sin = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    y = ro.rotary_fwd(x, cos, sin)
    xv = f64(x)
    n_in = xv[..., :D // 2] ** 2 + xv[..., D // 2:] ** 2
    n_out = y[..., :D // 2] ** 2 + y[..., D // 2:] ** 2
    fac = cos.astype(np.float64) ** 2 + sin.astype(np.float64) ** 2
    np.testing.assert_allclose(n_out, n_in * fac, rtol=1e-13, atol=1e-15)
    # a quarter turn (cos 0, sin 1) maps (a, b) to (-b, a): fixes the sign convention
    q = ro.rotary_fwd(x, np.zeros((S, D // 2), np.float32), np.ones((S, D // 2), np.float32))
    np.testing.assert_array_equal(q[..., :D // 2], -xv[..., D // 2:])
    np.testing.assert_array_equal(q[..., D // 2:], xv[..., :D // 2])
    # the table is indexed by the POSITION within the sequence, the same for every batch and head
    c2, s2 = rope_tables(S, D)
    y2 = ro.rotary_fwd(x, c2, s2)
    y_single = ro.rotary_fwd(x[:, 1:2], c2, s2)
    np.testing.assert_array_equal(y2[:, 1:2], y_single)
