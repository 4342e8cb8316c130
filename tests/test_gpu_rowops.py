"""GPU parity for the row-wise kernels (RMSNorm fwd, LayerNorm fwd+bwd, rotary fwd) against
their fp64 oracles, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_16238_amd import rowops
from paper_2601_16238_amd import workloads as wl
from parity_util import bf16_round, to_dev, to_f64

pytestmark = pytest.mark.gpu
ro = oracle.rowops


def inputs(rows, cols, seed, sigma=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    x = wl.f32_to_bf16_bits(rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(sigma) + np.float32(0.25))
    dy = wl.f32_to_bf16_bits(rng.standard_normal((rows, cols), dtype=np.float32))
    w = (rng.standard_normal(cols).astype(np.float32) * 0.5 + 1.0)
    b = rng.standard_normal(cols).astype(np.float32) * 0.3
    return x, dy, w, b


def close_bf16(name, got, ref):
    """bf16 output: within 3x (max) / 2x (mean) of the error that rounding the exact result
    to bf16 makes (fp32 arithmetic adds a little to that floor)."""
    assert np.isfinite(got).all(), name
    e = np.abs(got - ref); f = np.abs(bf16_round(ref) - ref)
    assert e.max() <= 3.0 * f.max() + 1e-6 and e.mean() <= 2.0 * f.mean() + 1e-8, \
        "%s: max %.3e mean %.3e (floor %.3e / %.3e)" % (name, e.max(), e.mean(), f.max(), f.mean())


# rows x cols: the paper's benchmark width, ragged widths for every vectors-per-thread variant
# (1, 2, 4, 8), a single row, the maximum width
SHAPES = [(64, 8192), (5, 8), (3, 264), (7, 2048), (4, 2056), (9, 4096), (2, 5000), (3, 16384), (1, 1024), (1030, 512)]
# more than 512 rows: the LayerNorm backward pairs two rows per work-group (odd counts leave the last
# pair half empty; 16384 columns keep one row per work-group)
LN_SHAPES = SHAPES + [(1027, 2056), (513, 4104), (1539, 8192), (515, 16384)]


@pytest.mark.parametrize("rows,cols", SHAPES)
def test_rmsnorm_fwd(rows, cols):
    print("case rmsnorm", rows, cols, flush=True)
    x, _, w, _ = inputs(rows, cols, 2000 + cols)
    y = rowops.rmsnorm_fwd(to_dev(x), torch.from_numpy(w).cuda(), 1e-6)
    torch.cuda.synchronize()
    close_bf16("y", to_f64(y), ro.rmsnorm_fwd(x, w, 1e-6))


@pytest.mark.parametrize("rows,cols", LN_SHAPES)
def test_layernorm_fwd_bwd(rows, cols):
    print("case layernorm", rows, cols, flush=True)
    x, dy, w, b = inputs(rows, cols, 2100 + cols, sigma=2.0)
    eps = 1e-5
    xd, dyd, wd, bd = to_dev(x), to_dev(dy), torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda()
    y, mean, rstd = rowops.layernorm_fwd(xd, wd, bd, eps)
    dx, dw, db = rowops.layernorm_bwd(dyd, xd, wd, mean, rstd)
    torch.cuda.synchronize()
    yr, mr, rr = ro.layernorm_fwd(x, w, b, eps)
    dxr, dwr, dbr = ro.layernorm_bwd(dy, x, w, eps)
    close_bf16("y", to_f64(y), yr)
    np.testing.assert_allclose(to_f64(mean), mr, rtol=0, atol=2e-6)
    np.testing.assert_allclose(to_f64(rstd), rr, rtol=2e-6, atol=0)
    close_bf16("dx", to_f64(dx), dxr)
    # fp32 column sums over the rows: error grows like sqrt(rows) * 2^-24 * |terms|
    tol = 4e-6 * np.sqrt(rows) * max(1.0, float(np.abs(dwr).max())) + 1e-6
    np.testing.assert_allclose(to_f64(dw), dwr, rtol=0, atol=tol)
    np.testing.assert_allclose(to_f64(db), dbr, rtol=0, atol=tol)


# one row team per work-group, and two (more than 512 rows of 8192 columns)
@pytest.mark.parametrize("rows,cols,pitch", [(600, 1024, 1032), (1301, 8192, 8200)])
def test_layernorm_bwd_is_deterministic_and_handles_strided_rows(rows, cols, pitch):
    print("case layernorm_strided", rows, cols, pitch, flush=True)
    x, dy, w, b = inputs(rows, cols, 2201)
    wd, bd = torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda()

    def pitched(bits):
        buf = torch.full((rows, pitch), float("nan"), dtype=torch.bfloat16, device="cuda")
        buf[:, :cols] = to_dev(bits)
        return buf[:, :cols]

    xd, dyd = pitched(x), pitched(dy)
    ybuf = torch.full((rows, pitch), float("nan"), dtype=torch.bfloat16, device="cuda")
    y, mean, rstd = rowops.layernorm_fwd(xd, wd, bd, 1e-5, y=ybuf[:, :cols])
    r1 = rowops.layernorm_bwd(dyd, xd, wd, mean, rstd)
    r2 = rowops.layernorm_bwd(dyd, xd, wd, mean, rstd)
    torch.cuda.synchronize()
    assert torch.isnan(ybuf[:, cols:]).all()
    for a, c in zip(r1, r2):
        assert torch.equal(a, c)
    close_bf16("y", to_f64(y), ro.layernorm_fwd(x, w, b, 1e-5)[0])
    close_bf16("dx", to_f64(r1[0]), ro.layernorm_bwd(dy, x, w, 1e-5)[0])


def rope_tables(S, D, base=10000.0):
    inv = base ** (-np.arange(0, D, 2, dtype=np.float64) / D)
    ang = np.arange(S, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


@pytest.mark.parametrize("B,H,S,D", [(4, 8, 2048, 128), (1, 1, 1, 16), (2, 3, 65, 64), (1, 2, 33, 32), (1, 2, 7, 256)])
def test_rotary_fwd(B, H, S, D):
    print("case rotary", B, H, S, D, flush=True)
    rng = np.random.Generator(np.random.PCG64(2300 + D))
    x = wl.f32_to_bf16_bits(rng.standard_normal((B, H, S, D), dtype=np.float32))
    cos, sin = rope_tables(S, D)
    y = rowops.rotary_fwd(to_dev(x), torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda())
    torch.cuda.synchronize()
    close_bf16("y", to_f64(y), ro.rotary_fwd(x, cos, sin))


def test_rotary_strided_layout_and_in_place():
    """[B,S,H,D] storage viewed as [B,H,S,D], rotated in place."""
    B, H, S, D = 2, 4, 50, 64
    print("case rotary_inplace", flush=True)
    rng = np.random.Generator(np.random.PCG64(2401))
    x = wl.f32_to_bf16_bits(rng.standard_normal((B, H, S, D), dtype=np.float32))
    cos, sin = rope_tables(S, D)
    bshd = to_dev(x).permute(0, 2, 1, 3).contiguous()   # memory order B,S,H,D
    view = bshd.permute(0, 2, 1, 3)                      # logical B,H,S,D
    rowops.rotary_fwd(view, torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda(), y=view)
    torch.cuda.synchronize()
    close_bf16("y", to_f64(view), ro.rotary_fwd(x, cos, sin))
