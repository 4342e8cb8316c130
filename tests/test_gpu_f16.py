"""GPU parity for the IEEE fp16 variant (attn_fwd_rect_f16 / attn_bwd_rect_f16) against the
fp64 oracle reading the same fp16 bit patterns, element by element."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import workloads as wl
from parity_util import check_bf16, check_lse, f16_round, to_dev_f16, to_f64

pytestmark = pytest.mark.gpu

# (B,Hq,Hkv,Sq,Sk,D,causal): square and rectangular, both head dims, ragged, grouped, decode
CASES = [
    (1, 2, 2, 128, 128, 64, False), (1, 2, 2, 128, 128, 64, True), (2, 4, 2, 65, 65, 64, True),
    (1, 2, 2, 300, 300, 128, True), (1, 4, 1, 513, 513, 128, False), (1, 2, 2, 33, 64, 64, True),
    (2, 4, 2, 100, 356, 128, True), (2, 8, 2, 1, 300, 64, True), (1, 4, 4, 150, 77, 64, False),
    (1, 1, 1, 1, 1, 128, True), (1, 2, 2, 1024, 1024, 128, True),
    (1, 2, 2, 300, 300, 256, True), (1, 4, 2, 130, 200, 192, False),   # the kernels for D > 128
]


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", CASES)
def test_f16_parity(B, Hq, Hkv, Sq, Sk, D, causal):
    """fp16 outputs carry 11 significant bits, so besides the stated bf16 tolerance the
    tighter gate applies: error within 4x (max) / 6x (mean) of what rounding the exact
    result to fp16 makes, plus the share of delta = rowsum(dO o O) formed from the fp16 O."""
    print("case f16_parity", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    x = wl.random_rect_inputs_f16(B, Hq, Hkv, Sq, Sk, D, seed=1500 + Sq + Sk)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal, dtype="f16")
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal, dtype="f16")
    Q, K, V, dO = (to_dev_f16(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd_rect(Q, K, V, x["scale"], causal)
    dQ, dK, dV = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], causal)
    torch.cuda.synchronize()
    assert O.dtype == torch.float16 and dK.dtype == torch.float16
    check_bf16("O", to_f64(O), Oref, rnd=f16_round)
    check_lse(to_f64(LSE), Lref)
    for name, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        got = to_f64(g)
        check_bf16(name, got, r, floor_gate=False)           # the stated tolerance
        # and relative to the attainable: P and dS are rounded to fp16 (2^-11) before the
        # second product of each stage, so errors scale with the magnitude of the result
        scale = max(1.0, float(np.abs(r).max()))
        emax = float(np.abs(got - r).max())
        assert emax <= 4e-3 * scale, "%s: max %.3e vs scale %.3g" % (name, emax, scale)


def test_f16_and_bf16_agree_on_values_both_formats_hold():
    """Inputs exact in both formats: the two builds of the kernels see the same numbers; the
    fp16 result must be at least as close to the oracle as the bf16 one is, up to noise."""
    B, H, S, D = 1, 2, 256, 128
    print("case f16_vs_bf16", B, H, S, D, flush=True)
    rng = np.random.Generator(np.random.PCG64(1601))
    vals = {k: (rng.integers(-127, 128, size=(B, H, S, D)) / 64.0).astype(np.float32)
            for k in ("Q", "K", "V", "dO")}
    sc = wl.default_scale(D)
    hb = {k: wl.f32_to_f16_bits(v) for k, v in vals.items()}
    bb = {k: wl.f32_to_bf16_bits(v) for k, v in vals.items()}
    Oref, Lref = oracle.attn_fwd(hb["Q"], hb["K"], hb["V"], sc, True, dtype="f16")
    th = {k: to_dev_f16(v) for k, v in hb.items()}
    tb = {k: torch.from_numpy(v.view(np.int16)).cuda().view(torch.bfloat16) for k, v in bb.items()}
    Oh, Lh = attn.attn_fwd_rect(th["Q"], th["K"], th["V"], sc, True)
    Ob, Lb = attn.attn_fwd_rect(tb["Q"], tb["K"], tb["V"], sc, True)
    torch.cuda.synchronize()
    eh = float(np.abs(to_f64(Oh) - Oref).max()); eb = float(np.abs(to_f64(Ob) - Oref).max())
    print("max err fp16 %.3e bf16 %.3e" % (eh, eb), flush=True)
    assert eh <= eb + 1e-6
    check_lse(to_f64(Lh), Lref)
    check_lse(to_f64(Lb), Lref)
