"""Seeded synthetic attention workloads (shapes of the paper's attention call sites).

This module holds no attention arithmetic: it only draws Gaussian tensors from a seed,
applies the per-workload scaling, and rounds to bf16 bit patterns.  Both the GPU tests /
bench and the CPU checker read the bytes produced here, so neither side's result depends
on how they were drawn.

The shapes stand in for: the CIFAR-10 ViT and Shakespeare miniGPT training runs (paper,
end-to-end training section -- only "depth 6" / "6 layers" are given there, the head
counts and lengths are this build's), and the SDPA/FlashAttention microbenchmark (paper,
microbenchmark table, attention rows: (B,Hq,Hkv,S,D) = (32,10,10,2048,128), bf16, causal).
No dataset or trained weight is used anywhere.
"""
from collections import namedtuple

import numpy as np

Workload = namedtuple("Workload", "name B H S D causal sigma outlier_frac outlier_gain seed note")

# name -> Workload.  sigma multiplies all four tensors before rounding; outliers scale a
# fraction of the rows of Q and (independently) of K.
WORKLOADS = {w.name: w for w in [
    Workload("tiny", 1, 2, 128, 64, False, 1.0, 0.0, 1.0, 1001, "tiny non-causal"),
    Workload("vit_cifar", 128, 6, 65, 64, False, 1.0, 0.0, 1.0, 1002,
             "CIFAR-ViT-shaped, 64 patches + cls token"),
    Workload("minigpt", 8, 8, 1024, 64, True, 0.5, 0.0, 1.0, 1003, "miniGPT-shaped causal"),
    Workload("sdpa_cmp", 4, 32, 4096, 128, False, 1.0, 0.0, 1.0, 1004,
             "SDPA/FlashAttention comparison shape, non-causal"),
    Workload("sdpa_cmp_causal", 4, 32, 4096, 128, True, 1.0, 0.0, 1.0, 1004,
             "SDPA/FlashAttention comparison shape, causal (same tensors as sdpa_cmp)"),
    Workload("long_causal", 1, 16, 16384, 128, True, 1.0, 0.01, 8.0, 1005,
             "long-sequence causal, 1% of Q/K rows x8"),
    Workload("paper_table", 32, 10, 2048, 128, True, 1.0, 0.0, 1.0, 1006,
             "the microbenchmark table's own shape (context only)"),
    Workload("headdim256", 4, 16, 4096, 256, True, 1.0, 0.0, 1.0, 1007,
             "head dimension 256 (the kernels with one wave per SIMD), causal"),
]}


def f32_to_bf16_bits(x):
    """Round float32 -> bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b):
    """Widen bf16 bit patterns (uint16) exactly to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def default_scale(D):
    """The fp32 value of 1/sqrt(D) that both sides receive."""
    return float(np.float32(1.0) / np.sqrt(np.float32(D)))


def make_inputs(w, heads=None):
    """Draw Q, K, V, dO for workload `w` (a Workload or its name).

    Returns a dict of uint16 arrays [B,H,S,D] (bf16 bit patterns) plus 'scale' (python
    float holding an fp32 value) and 'causal'.  Draw order: Q, K, V, dO, then the outlier
    row choices for Q and K.  `heads` (an iterable of flat b*H+h indices) returns only
    those heads, as a [1,len(heads),S,D] array drawn identically to the full tensor.
    """
    if isinstance(w, str):
        w = WORKLOADS[w]
    rng = np.random.Generator(np.random.PCG64(w.seed))
    BH = w.B * w.H
    out = {}
    for name in ("Q", "K", "V", "dO"):
        x = rng.standard_normal((BH, w.S, w.D), dtype=np.float32)
        if w.sigma != 1.0:
            x *= np.float32(w.sigma)
        out[name] = x
    if w.outlier_frac > 0.0:
        n_rows = BH * w.S
        n_out = int(round(w.outlier_frac * n_rows))
        for name in ("Q", "K"):
            rows = rng.permutation(n_rows)[:n_out]
            flat = out[name].reshape(n_rows, w.D)
            flat[rows] *= np.float32(w.outlier_gain)
    for name in ("Q", "K", "V", "dO"):
        x = out[name]
        if heads is not None:
            x = x[np.asarray(list(heads), dtype=np.int64)]
            out[name] = f32_to_bf16_bits(x).reshape(1, x.shape[0], w.S, w.D)
        else:
            out[name] = f32_to_bf16_bits(x).reshape(w.B, w.H, w.S, w.D)
    out["scale"] = default_scale(w.D)
    out["causal"] = bool(w.causal)
    return out


def random_inputs(B, H, S, D, seed, sigma=1.0):
    """Free-form seeded bf16 N(0, sigma^2) tensors for the small parity / edge cases."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name in ("Q", "K", "V", "dO"):
        x = rng.standard_normal((B, H, S, D), dtype=np.float32) * np.float32(sigma)
        out[name] = f32_to_bf16_bits(x)
    out["scale"] = default_scale(D)
    return out


# ---- grouped-query heads (the microbenchmark table's shape tuple carries Hq and Hkv) ---------
GqaWorkload = namedtuple("GqaWorkload", "name B Hq Hkv S D causal sigma seed note")

GQA_WORKLOADS = {w.name: w for w in [
    GqaWorkload("gqa_cmp", 4, 32, 8, 4096, 128, True, 1.0, 1007,
                "the comparison shape with 4 query heads per K/V head, causal"),
    GqaWorkload("mqa_small", 2, 8, 1, 300, 64, True, 1.0, 1008, "multi-query, ragged length"),
]}


def random_gqa_inputs(B, Hq, Hkv, S, D, seed, sigma=1.0):
    """Seeded bf16 N(0, sigma^2) tensors: Q, dO [B,Hq,S,D]; K, V [B,Hkv,S,D]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name, heads in (("Q", Hq), ("K", Hkv), ("V", Hkv), ("dO", Hq)):
        x = rng.standard_normal((B, heads, S, D), dtype=np.float32) * np.float32(sigma)
        out[name] = f32_to_bf16_bits(x)
    out["scale"] = default_scale(D)
    return out


def make_gqa_inputs(w, kv_heads=None):
    """Draw Q, K, V, dO for grouped-query workload `w` (a GqaWorkload or its name), draw order
    Q, K, V, dO.  `kv_heads` (flat b*Hkv+hkv indices) returns only those K/V heads and the
    query heads of their groups, as [1,n*G,S,D] and [1,n,S,D] arrays drawn identically."""
    if isinstance(w, str):
        w = GQA_WORKLOADS[w]
    rng = np.random.Generator(np.random.PCG64(w.seed))
    G = w.Hq // w.Hkv
    out = {}
    for name, heads in (("Q", w.Hq), ("K", w.Hkv), ("V", w.Hkv), ("dO", w.Hq)):
        x = rng.standard_normal((w.B * heads, w.S, w.D), dtype=np.float32)
        if w.sigma != 1.0:
            x *= np.float32(w.sigma)
        if kv_heads is not None:
            kv = np.asarray(list(kv_heads), dtype=np.int64)
            if heads == w.Hkv:
                sel = kv
            else:  # the G query heads of K/V head (b, hkv) are b*Hq + hkv*G + 0..G-1
                b, hk = kv // w.Hkv, kv % w.Hkv
                sel = ((b * w.Hq + hk * G)[:, None] + np.arange(G)[None, :]).reshape(-1)
            x = x[sel]
            out[name] = f32_to_bf16_bits(x).reshape(1, x.shape[0], w.S, w.D)
        else:
            out[name] = f32_to_bf16_bits(x).reshape(w.B, heads, w.S, w.D)
    out["scale"] = default_scale(w.D)
    out["causal"] = bool(w.causal)
    return out


def fwd_flops(B, H, S, D, causal):
    """Benchmark FLOP convention: 4*B*H*S^2*D forward, halved under a causal mask."""
    f = 4.0 * B * H * S * S * D
    return f / 2 if causal else f


def bwd_flops(B, H, S, D, causal):
    """Backward is counted as 2.5x forward (five GEMMs against two)."""
    return 2.5 * fwd_flops(B, H, S, D, causal)


def fwd_bytes(B, H, S, D):
    """Algorithmic HBM bytes forward: read Q,K,V, write O (bf16) and LSE (fp32)."""
    return 4 * B * H * S * D * 2 + B * H * S * 4


def bwd_bytes(B, H, S, D):
    """Algorithmic HBM bytes backward: read Q,K,V,O,dO, write dQ,dK,dV, read LSE."""
    return 8 * B * H * S * D * 2 + B * H * S * 4


# ---- rectangular problems: Sq query rows against Sk cached keys (decoding, chunked prefill) ----
RectWorkload = namedtuple("RectWorkload", "name B Hq Hkv Sq Sk D causal sigma seed note")

RECT_WORKLOADS = {w.name: w for w in [
    RectWorkload("decode_cmp", 8, 32, 8, 1, 8192, 128, True, 1.0, 1009,
                 "one new token per sequence against an 8K cache, grouped-query heads"),
    RectWorkload("prefill_chunk", 1, 32, 8, 512, 4096, 128, True, 1.0, 1010,
                 "small-batch chunked prefill: 512 new rows after 3584 cached ones"),
    RectWorkload("spec_decode", 8, 32, 8, 4, 8192, 128, True, 1.0, 1013,
                 "four new tokens per sequence (speculative decoding) against an 8K cache, grouped-query heads"),
    RectWorkload("decode_small", 2, 8, 2, 1, 300, 64, True, 1.0, 1011, "parity-size decode"),
    RectWorkload("cross_small", 1, 4, 4, 150, 77, 64, False, 1.0, 1012,
                 "more rows than keys, no mask"),
]}


def random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed, sigma=1.0):
    """Seeded bf16 N(0, sigma^2) tensors: Q, dO [B,Hq,Sq,D]; K, V [B,Hkv,Sk,D]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name, heads, rows in (("Q", Hq, Sq), ("K", Hkv, Sk), ("V", Hkv, Sk), ("dO", Hq, Sq)):
        x = rng.standard_normal((B, heads, rows, D), dtype=np.float32) * np.float32(sigma)
        out[name] = f32_to_bf16_bits(x)
    out["scale"] = default_scale(D)
    return out


def make_rect_inputs(w, kv_heads=None):
    """Draw Q, K, V, dO for rectangular workload `w` (a RectWorkload or its name), draw order
    Q, K, V, dO.  `kv_heads` (flat b*Hkv+hkv indices) returns only those K/V heads and the
    query heads of their groups, as [1,n*G,Sq,D] and [1,n,Sk,D] arrays drawn identically."""
    if isinstance(w, str):
        w = RECT_WORKLOADS[w]
    rng = np.random.Generator(np.random.PCG64(w.seed))
    G = w.Hq // w.Hkv
    out = {}
    for name, heads, rows in (("Q", w.Hq, w.Sq), ("K", w.Hkv, w.Sk), ("V", w.Hkv, w.Sk),
                              ("dO", w.Hq, w.Sq)):
        x = rng.standard_normal((w.B * heads, rows, w.D), dtype=np.float32)
        if w.sigma != 1.0:
            x *= np.float32(w.sigma)
        if kv_heads is not None:
            kv = np.asarray(list(kv_heads), dtype=np.int64)
            if heads == w.Hq:
                idx = (kv[:, None] // w.Hkv * w.Hq + kv[:, None] % w.Hkv * G +
                       np.arange(G)[None, :]).reshape(-1)
            else:
                idx = kv
            out[name] = f32_to_bf16_bits(x[idx])[None]
        else:
            out[name] = f32_to_bf16_bits(x).reshape(w.B, heads, rows, w.D)
    out["scale"] = default_scale(w.D)
    out["causal"] = bool(w.causal)
    return out


# ---- IEEE fp16 inputs (the second 16-bit input type) ------------------------------------------

def f32_to_f16_bits(x):
    """Round float32 -> IEEE fp16 (round-to-nearest-even), returned as uint16 bit patterns."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(b):
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


def random_rect_inputs_f16(B, Hq, Hkv, Sq, Sk, D, seed, sigma=1.0):
    """As random_rect_inputs (same draws), rounded to fp16 instead of bf16."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name, heads, rows in (("Q", Hq, Sq), ("K", Hkv, Sk), ("V", Hkv, Sk), ("dO", Hq, Sq)):
        x = rng.standard_normal((B, heads, rows, D), dtype=np.float32) * np.float32(sigma)
        out[name] = f32_to_f16_bits(x)
    out["scale"] = default_scale(D)
    return out
