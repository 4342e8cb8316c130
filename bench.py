#!/usr/bin/env python3
"""Attention benchmark: one "step" = attn_fwd + attn_bwd over one synthetic batch.

Prints ONE JSON line.  `value` is fwd+bwd TFLOP/s under the usual attention-benchmark FLOP
convention (4*B*H*S^2*D forward, halved if causal; backward 2.5x forward), inputs resident
in HBM before the timed region.  Timing follows the paper's protocol for its fused-attention
microbenchmark: seeded inputs, warm-up, synchronise around the timed region, mean latency.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (published)
PEAK_HBM_GBS = 8000.0
CALIB_COPY_BYTES = 256 * 1024 * 1024   # --calib-copy reads this many bytes and writes as many
# HBM traffic per launch of the row-wise kernels, from the two rocprofv3 --pmc passes summarised in
# profiles/rowops_hbm_traffic_pmc.txt: FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 (KiB); for the
# backward: rows kernel + column kernel.
MEASURED_TRAFFIC_BYTES = {
    ("rowops", "rmsnorm_fwd"): int((32927.1 * 2.0 + 65536.0) * 1024),
    ("rowops", "layernorm_fwd"): int((33062.6 * 2.0 + 65792.4) * 1024),
    ("rowops", "layernorm_bwd"): int(((65853.2 + 8210.1) * 2.0 + 81920.0 + 64.0) * 1024),
    ("rowops", "rotary_fwd"): int((8741.5 * 2.0 + 16384.0) * 1024),
}


def measured_traffic_bytes(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` (read + written, scaled counter readings)
    from the committed rocprofv3 summary of that workload, profiles/<workload>_kernel_trace_and_
    hbm_traffic.txt; None if there is none.  The summaries are regenerated with the kernels, so
    the figure cannot outlive the code it was measured on unnoticed."""
    path = os.path.join(ROOT, "profiles", "%s_kernel_trace_and_hbm_traffic.txt" % workload)
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    start = next((i for i, ln in enumerate(lines) if ln.startswith("HBM traffic counters")), None)
    if start is None:
        return None
    for ln in lines[start:]:
        f = ln.split()
        if len(f) == 5 and f[0].startswith(kernel + "<"):
            return int((float(f[3]) + float(f[4])) * 1024 * 1024)
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="long_causal",
                    help="one of paper_2601_16238_amd.workloads.WORKLOADS, GQA_WORKLOADS or RECT_WORKLOADS, "
                         "'rowops' (the row-wise kernels) or 'rope' (rotary fused into the forward against "
                         "rotary-then-forward)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all", action="store_true",
                    help="also time every other workload (reported under 'other_workloads')")
    ap.add_argument("--calib-copy", action="store_true",
                    help="before the timed region, run one plain device copy of 256 MiB (the "
                         "known-size kernel that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings "
                         "are scaled by)")
    return ap.parse_args()


def time_calls(torch, fn, n):
    """Mean milliseconds per call of fn over n back-to-back calls, by events on the current
    stream (the stream the library launches on)."""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def graph_ms(torch, fn, n):
    """Milliseconds per call of fn when n calls are recorded into one HIP graph and replayed
    (events around the replay on the replaying stream): the device time of kernels that take
    less than issuing a launch from Python costs.  The library's calls only enqueue kernels."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        fn()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(n):
                fn()
    torch.cuda.synchronize()
    graph.replay()
    return time_calls(torch, graph.replay, 3) / n


def measure(torch, attn, wl, w, steps, warmup):
    import numpy as np
    from paper_2601_16238_amd import binding
    gqa = hasattr(w, "Hq")   # grouped-query workload: K, V, dK, dV have Hkv heads
    H, Hkv = (w.Hq, w.Hkv) if gqa else (w.H, w.H)
    x = wl.make_gqa_inputs(w) if gqa else wl.make_inputs(w)

    def dev(b):
        return torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16)

    Q, K, V, dO = (dev(x[k]) for k in ("Q", "K", "V", "dO"))
    del x
    scale, causal = wl.default_scale(w.D), w.causal
    O = torch.empty_like(Q)
    LSE = torch.empty((w.B, H, w.S), dtype=torch.float32, device="cuda")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(K)
    ws = torch.empty(attn.attn_bwd_gqa_workspace_bytes(w.B, H, Hkv, w.S, w.D), dtype=torch.uint8,
                     device="cuda")
    fwd_call, bwd_call = (attn.attn_fwd_gqa, attn.attn_bwd_gqa) if gqa else (attn.attn_fwd, attn.attn_bwd)

    def fwd():
        fwd_call(Q, K, V, scale, causal, O=O, LSE=LSE)

    def bwd(stages=None):
        bwd_call(Q, K, V, O, dO, LSE, scale, causal, dQ=dQ, dK=dK, dV=dV, workspace=ws,
                 stages=stages)

    def step():
        fwd()
        bwd()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms_step = time_calls(torch, step, steps)
    wall = time.perf_counter() - t0
    n = max(3, steps // 2)

    def stage_ms(fn):
        # the shorter of two loops: these figures pick the kernel the roofline is quoted for, and
        # one disturbed loop (seen once: a 1.3 ms stage read 4.5 ms next to an undisturbed step)
        # would pick the wrong one
        return min(time_calls(torch, fn, n), time_calls(torch, fn, n))

    ms = {"fwd": stage_ms(fwd), "bwd": stage_ms(bwd),
          "bwd_delta": stage_ms(lambda: bwd(binding.STAGE_DELTA)),
          "bwd_dkdv": stage_ms(lambda: bwd(binding.STAGE_DKDV)),
          "bwd_dq": stage_ms(lambda: bwd(binding.STAGE_DQ))}
    if w.B * H * w.S * w.D * 2 <= (16 << 20):
        # small shapes: a call takes less than issuing it from Python costs
        ms["fwd_graph_replay"] = graph_ms(torch, fwd, 20)
        ms["bwd_graph_replay"] = graph_ms(torch, bwd, 20)
    f_fwd = wl.fwd_flops(w.B, H, w.S, w.D, causal)
    f_bwd = wl.bwd_flops(w.B, H, w.S, w.D, causal)
    # algorithmic bytes: Q-shaped tensors have H heads, K/V-shaped ones Hkv
    t_q, t_kv, lse_b = w.B * H * w.S * w.D * 2, w.B * Hkv * w.S * w.D * 2, w.B * H * w.S * 4
    b_fwd, b_bwd = 2 * t_q + 2 * t_kv + lse_b, 4 * t_q + 4 * t_kv + lse_b
    res = {
        "ms_per_step": ms_step, "ms": ms, "wall_s": wall,
        "tflops_fwdbwd": (f_fwd + f_bwd) / (ms_step * 1e-3) / 1e12,
        "tflops_fwd": f_fwd / (ms["fwd"] * 1e-3) / 1e12,
        "tflops_bwd": f_bwd / (ms["bwd"] * 1e-3) / 1e12,
        "gbs_fwd": b_fwd / (ms["fwd"] * 1e-3) / 1e9,
        "gbs_bwd": b_bwd / (ms["bwd"] * 1e-3) / 1e9,
    }
    if "fwd_graph_replay" in ms:   # small shapes: the device-time figures
        res["gbs_fwd_graph_replay"] = b_fwd / (ms["fwd_graph_replay"] * 1e-3) / 1e9
        res["gbs_bwd_graph_replay"] = b_bwd / (ms["bwd_graph_replay"] * 1e-3) / 1e9
        res["tflops_fwdbwd_graph_replay"] = (f_fwd + f_bwd) / (
            (ms["fwd_graph_replay"] + ms["bwd_graph_replay"]) * 1e-3) / 1e12
    # Algorithmic FLOPs per launch of each MFMA kernel (GEMM = 2*N_s*D flops, N_s = S^2 or
    # S^2/2): forward 2 GEMMs; dK/dV kernel 4 (S, dP, dV, dK); dQ kernel 1 (dQ -- its
    # recomputed S and dP are overhead, not algorithmic work).
    gemm = f_fwd / 2.0
    kern = {"attn_fwd_kernel": (2 * gemm, ms["fwd"]), "attn_bwd_dkdv_kernel": (4 * gemm, ms["bwd_dkdv"]),
            "attn_bwd_dq_kernel": (1 * gemm, ms["bwd_dq"])}
    if (not gqa or w.B * Hkv >= 256) and w.S <= (256 if w.D <= 64 else 128 if w.D <= 128 else 0):
        # short heads: the full backward call is ONE fused kernel (5 algorithmic GEMMs); the
        # stage-wise timings above still show the two-kernel path that it replaces
        kern["attn_bwd_small_kernel"] = (5 * gemm, ms.get("bwd_graph_replay", ms["bwd"]))
    res["kernels"] = {k: {"ms": t, "achieved_tflops": f / (t * 1e-3) / 1e12,
                          "frac": f / (t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
                      for k, (f, t) in kern.items()}
    return res


def measure_mfma_peak(torch, attn):
    """What the matrix pipes of this GPU sustain on nothing but bf16 32x32x16 MFMAs (the
    library's measurement kernel: 1024 work-groups of 8 waves, ~30 ms per launch), to print
    beside the nominal peak every fraction here is quoted against: once with operands that
    toggle like real data (the figure the fractions 'of measured peak' use) and once with
    constant operands (less power, higher clock)."""
    wgs, iters = 1024, 16384
    sink = torch.empty(wgs * 512, dtype=torch.float32, device="cuda")
    out = {"kernel": "MFMA-only loop, 2 waves per SIMD, 4 independent accumulator chains"}
    for key, rnd in (("constant_operands", False), ("random_operands", True)):
        flop = attn.attn_probe_mfma_bf16(wgs, iters, sink, random_operands=rnd)   # warm-up launch
        ms = time_calls(torch, lambda: attn.attn_probe_mfma_bf16(wgs, iters, sink, random_operands=rnd), 3)
        out[key] = {"tflops": flop / (ms * 1e-3) / 1e12, "ms_per_launch": ms,
                    "frac_of_nominal": flop / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    out["tflops"] = out["random_operands"]["tflops"]
    return out


def measure_cold(torch, attn, wl, w, steps):
    """Cold-cache timing of a small workload: every call works on its own set of tensors, and
    the sets together exceed the 256 MiB last-level cache several times over, so no call finds
    its inputs cached.  (Each call is still issued from Python, which costs some microseconds
    that the smallest shapes cannot hide.)"""
    g = torch.Generator(device="cuda"); g.manual_seed(w.seed)
    per_set = 9 * w.B * w.H * w.S * w.D * 2
    nsets = int(max(4, min(4096, (1 << 30) // per_set)))
    mk = lambda: torch.randn((nsets, w.B, w.H, w.S, w.D), device="cuda", generator=g).to(torch.bfloat16)
    Q, K, V, dO = mk(), mk(), mk(), mk()
    O, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
    LSE = torch.empty((nsets, w.B, w.H, w.S), dtype=torch.float32, device="cuda")
    ws = torch.empty(attn.attn_bwd_workspace_bytes(w.B, w.H, w.S, w.D), dtype=torch.uint8, device="cuda")
    scale = wl.default_scale(w.D)
    state = {"i": 0}

    def fwd():
        i = state["i"] = (state["i"] + 1) % nsets
        attn.attn_fwd(Q[i], K[i], V[i], scale, w.causal, O=O[i], LSE=LSE[i])

    def bwd():
        i = state["i"] = (state["i"] + 1) % nsets
        attn.attn_bwd(Q[i], K[i], V[i], O[i], dO[i], LSE[i], scale, w.causal, dQ=dQ[i], dK=dK[i],
                      dV=dV[i], workspace=ws)

    for _ in range(nsets):   # every O and LSE the backward will read is a forward result
        fwd()
    n = max(steps, min(nsets, 200))
    return {"sets": nsets, "bytes_per_set": per_set, "fwd_ms": time_calls(torch, fwd, n),
            "bwd_ms": time_calls(torch, bwd, n)}


def per_tensor_bytes(w):
    return w.B * (w.Hq if hasattr(w, "Hq") else w.H) * w.S * w.D * 2


def visible_pairs(Sq, Sk, causal):
    """(query, key) pairs under the mask; causal is aligned bottom-right (needs Sk >= Sq)."""
    return Sq * (Sk - Sq) + Sq * (Sq + 1) // 2 if causal else Sq * Sk


def measure_rect(torch, attn, wl, w, steps, warmup):
    """Rectangular workloads (Sq rows against Sk cached keys): forward with the library's
    split plan, forward in one kernel, and backward.  FLOPs count the visible (query, key)
    pairs exactly: 4*D per pair forward, 10*D backward."""
    import numpy as np
    x = wl.make_rect_inputs(w)

    def dev(b):
        return torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16)

    Q, K, V, dO = (dev(x[k]) for k in ("Q", "K", "V", "dO"))
    del x
    scale, causal = wl.default_scale(w.D), w.causal
    O = torch.empty_like(Q)
    LSE = torch.empty((w.B, w.Hq, w.Sq), dtype=torch.float32, device="cuda")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(K)
    shape = (w.B, w.Hq, w.Hkv, w.Sq, w.Sk, w.D)
    fws_bytes = attn.attn_fwd_rect_workspace_bytes(*shape)
    fws = torch.empty(max(fws_bytes, 256), dtype=torch.uint8, device="cuda")
    bws = torch.empty(attn.attn_bwd_rect_workspace_bytes(*shape), dtype=torch.uint8, device="cuda")

    def fwd():
        attn.attn_fwd_rect(Q, K, V, scale, causal, O=O, LSE=LSE, workspace=fws)

    def fwd_one_kernel():
        attn.attn_fwd_rect(Q, K, V, scale, causal, O=O, LSE=LSE, split=False)

    def bwd():
        attn.attn_bwd_rect(Q, K, V, O, dO, LSE, scale, causal, dQ=dQ, dK=dK, dV=dV, workspace=bws)

    def step():
        fwd()
        bwd()

    for _ in range(warmup):
        step()
        fwd_one_kernel()
    ms = {"step": time_calls(torch, step, steps), "fwd": time_calls(torch, fwd, steps),
          "fwd_one_kernel": time_calls(torch, fwd_one_kernel, steps),
          "bwd": time_calls(torch, bwd, steps)}
    if w.Sq <= 32:
        # Decoding re-reads nothing: a model's next call reads another layer's cache.  The loop
        # above reads the same K and V again and again, and what of them fits the 256 MB last-level
        # cache comes from there; this one rotates over copies that together exceed 768 MiB.
        kv_bytes = 2 * K.numel() * K.element_size()
        sets = [(K, V)] + [(K.clone(), V.clone()) for _ in range(max(1, -(-(768 << 20) // kv_bytes) - 1))]

        def fwd_rotating():
            for Kc, Vc in sets:
                attn.attn_fwd_rect(Q, Kc, Vc, scale, causal, O=O, LSE=LSE, workspace=fws)

        fwd_rotating()
        ms["fwd_cache_cold"] = time_calls(torch, fwd_rotating, max(2, steps // 2)) / len(sets)
        del sets
    pairs = w.B * w.Hq * visible_pairs(w.Sq, w.Sk, causal)
    f_fwd, f_bwd = 4.0 * pairs * w.D, 10.0 * pairs * w.D
    t_q, t_kv = w.B * w.Hq * w.Sq * w.D * 2, w.B * w.Hkv * w.Sk * w.D * 2
    lse_b = w.B * w.Hq * w.Sq * 4
    b_fwd, b_bwd = 2 * t_q + 2 * t_kv + lse_b, 4 * t_q + 4 * t_kv + lse_b
    return {"ms": ms, "splits": fws_bytes // max(1, w.B * w.Hq * w.Sq * (w.D + 1) * 4),
            "tflops_fwd": f_fwd / (ms["fwd"] * 1e-3) / 1e12,
            "tflops_fwdbwd": (f_fwd + f_bwd) / (ms["step"] * 1e-3) / 1e12,
            "gbs_fwd": b_fwd / (ms["fwd"] * 1e-3) / 1e9, "gbs_bwd": b_bwd / (ms["bwd"] * 1e-3) / 1e9,
            "gbs_fwd_cache_cold": b_fwd / (ms["fwd_cache_cold"] * 1e-3) / 1e9 if "fwd_cache_cold" in ms else None,
            "bytes_fwd": b_fwd, "flops_fwd": f_fwd, "flops_bwd": f_bwd}


def rect_main(torch, attn, wl, w, a):
    """The JSON line for a rectangular workload given as --workload."""
    r = measure_rect(torch, attn, wl, w, a.steps, a.warmup)
    hbm_bound = w.Sq < 64   # a handful of rows per K/V row read: the stream of K and V bounds it
    # (decoding: the figure with the cache cold -- K and V really from HBM -- is the one quoted)
    gbs = r["gbs_fwd_cache_cold"] or r["gbs_fwd"]
    roof = ({"kernel": "attn_fwd_wide_kernel (+ merge)", "bound": "hbm", "achieved": gbs,
             "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "traffic": None}
            if hbm_bound else
            {"kernel": "attn_fwd_kernel (+ merge)", "bound": "mfma", "achieved": r["tflops_fwd"],
             "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": r["tflops_fwd"] / PEAK_BF16_TFLOPS,
             "traffic": None})
    if hbm_bound:
        # what work-groups that only read stream from HBM on this machine (512 MiB, more than the
        # last-level cache holds; plain loads with the non-temporal hint, and the direct transfers
        # in the decoding kernel's shape), beside the nominal peak the fraction is quoted against
        buf = torch.ones(512 << 18, dtype=torch.int32, device="cuda")
        chk = torch.empty(512, dtype=torch.int32, device="cuda")
        probe = {}
        for key, direct in (("loads", False), ("direct_transfers", True)):
            fn = lambda: attn.attn_probe_stream(buf, 512, chk, direct=direct, nontemporal=True)
            fn()
            probe[key + "_gbs"] = buf.numel() * 4 / (time_calls(torch, fn, 10) * 1e-3) / 1e9
        del buf
        roof["measured_stream_gbs"] = probe
        roof["frac_of_measured_stream"] = gbs / max(probe.values())
    out = {
        "metric": "attention fwd+bwd TFLOP/s (FLOPs = 4*D fwd + 10*D bwd per visible query-key pair)",
        "value": r["tflops_fwdbwd"], "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": r["ms"]["step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %s" % (w.name, " ".join(
            "%s=%s" % (k, getattr(w, k)) for k in ("B", "Hq", "Hkv", "Sq", "Sk", "D", "causal"))),
                   "seed": w.seed},
        "ms": r["ms"], "key_splits": r["splits"],
        "tflops": {"fwd": r["tflops_fwd"], "fwd_bwd": r["tflops_fwdbwd"]},
        "algorithmic_gbs": {"fwd": r["gbs_fwd"], "fwd_cache_cold": r["gbs_fwd_cache_cold"],
                            "bwd": r["gbs_bwd"], "hbm_peak": PEAK_HBM_GBS},
        "roofline": roof,
    }
    if not a.no_cpu_baseline:
        import oracle
        G = w.Hq // w.Hkv
        n_heads = w.B * w.Hkv

        def run(heads):
            x = wl.make_rect_inputs(w, kv_heads=range(heads))
            t0 = time.perf_counter()
            oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], w.causal)
            oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], w.causal)
            return time.perf_counter() - t0

        heads, dt = 1, run(1)
        more = int(min(n_heads, 15.0 // max(dt, 1e-3)))
        if more > 1:
            heads, dt = more, run(more)
        flops = heads * G * 14.0 * w.D * visible_pairs(w.Sq, w.Sk, w.causal)
        out["cpu_baseline"] = {"value": flops / dt / 1e12, "unit": "TFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle", "seconds": dt,
                               "sample": "fwd+bwd of the first %d of %d K/V heads (with their query "
                                         "groups) of %s (fp64)" % (heads, n_heads, w.name),
                               "nproc": os.cpu_count()}
    print(json.dumps(out))


def measure_rowops(torch, steps, warmup):
    """The row-wise kernels on the shapes of the paper's kernel table: (4096, 8192) bf16 for the
    norms, (4, 8, 2048, 128) for rotary.  Algorithmic bytes: every activation read once and
    written once (parameters, statistics and tables are negligible)."""
    from paper_2601_16238_amd import rowops
    rows, cols = 4096, 8192
    g = torch.Generator(device="cuda"); g.manual_seed(1013)
    x = torch.randn((rows, cols), device="cuda", generator=g).to(torch.bfloat16)
    dy = torch.randn((rows, cols), device="cuda", generator=g).to(torch.bfloat16)
    w = torch.randn(cols, device="cuda", generator=g) * 0.5 + 1.0
    b = torch.randn(cols, device="cuda", generator=g) * 0.3
    y, dx = torch.empty_like(x), torch.empty_like(x)
    mean, rstd = (torch.empty(rows, dtype=torch.float32, device="cuda") for _ in range(2))
    dw, db = (torch.empty(cols, dtype=torch.float32, device="cuda") for _ in range(2))
    ws = torch.empty(rowops.layernorm_bwd_workspace_bytes(rows, cols), dtype=torch.uint8, device="cuda")
    B, H, S, D = 4, 8, 2048, 128
    xr = torch.randn((B, H, S, D), device="cuda", generator=g).to(torch.bfloat16)
    yr = torch.empty_like(xr)
    ang = torch.arange(S, device="cuda", dtype=torch.float32)[:, None] * \
        (10000.0 ** (-torch.arange(0, D, 2, device="cuda", dtype=torch.float32) / D))[None, :]
    cos, sin = torch.cos(ang).contiguous(), torch.sin(ang).contiguous()
    act = rows * cols * 2
    cases = {
        "rmsnorm_fwd": (lambda: rowops.rmsnorm_fwd(x, w, 1e-6, y=y), 2 * act),
        "layernorm_fwd": (lambda: rowops.layernorm_fwd(x, w, b, 1e-5, y=y, mean=mean, rstd=rstd), 2 * act),
        "layernorm_bwd": (lambda: rowops.layernorm_bwd(dy, x, w, mean, rstd, dx=dx, dw=dw, db=db,
                                                       workspace=ws), 3 * act),
        "rotary_fwd": (lambda: rowops.rotary_fwd(xr, cos, sin, y=yr), 2 * xr.numel() * 2),
    }
    out = {}
    n = max(steps, 20)
    for name, (fn, nbytes) in cases.items():
        for _ in range(warmup):
            fn()
        ms_eager = time_calls(torch, fn, n)
        # These kernels take 5-50 us, less than issuing a launch from Python costs: the figure
        # that says something about the kernel is taken from n launches recorded into one HIP
        # graph and replayed (events around the replay on the replaying stream).
        ms = graph_ms(torch, fn, n)
        out[name] = {"ms": ms, "ms_eager_python_launch": ms_eager, "algorithmic_bytes": nbytes,
                     "gbs": nbytes / (ms * 1e-3) / 1e9,
                     "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
    out["layernorm_fwd_bwd_ms"] = out["layernorm_fwd"]["ms"] + out["layernorm_bwd"]["ms"]
    out["shapes"] = {"norms": [rows, cols], "rotary": [B, H, S, D]}
    return out


def measure_rope(torch, attn, steps, warmup):
    """Rotary embedding fused into the forward's Q load against the two-kernel sequence (rotary
    kernel on Q, then the forward), on the paper's rotary shape (4, 8, 2048, 128) with a causal
    mask and on the long-sequence shape; K is rotated beforehand in both (it is rotated where it
    is written).  Small shape by graph replay (device time)."""
    from paper_2601_16238_amd import rowops
    out = {}
    for name, (B, H, S, D) in (("paper_rotary_shape", (4, 8, 2048, 128)), ("long_causal_shape", (1, 16, 16384, 128))):
        g = torch.Generator(device="cuda"); g.manual_seed(1015)
        Q, K, V = (torch.randn((B, H, S, D), device="cuda", generator=g).to(torch.bfloat16) for _ in range(3))
        ang = torch.arange(S, device="cuda", dtype=torch.float32)[:, None] * \
            (10000.0 ** (-torch.arange(0, D, 2, device="cuda", dtype=torch.float32) / D))[None, :]
        cos, sin = torch.cos(ang).contiguous(), torch.sin(ang).contiguous()
        K_rot = rowops.rotary_fwd(K, cos, sin)
        O, Qr = torch.empty_like(Q), torch.empty_like(Q)
        LSE = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
        sc = 1.0 / float(D) ** 0.5

        def fused():
            attn.attn_fwd_rope(Q, K_rot, V, cos, sin, sc, True, O=O, LSE=LSE, Q_rot=Qr, split=False)

        def unfused():
            rowops.rotary_fwd(Q, cos, sin, y=Qr)
            attn.attn_fwd_rect(Qr, K_rot, V, sc, True, O=O, LSE=LSE, split=False)

        def plain():
            attn.attn_fwd_rect(Qr, K_rot, V, sc, True, O=O, LSE=LSE, split=False)

        for _ in range(warmup):
            fused(); unfused()
        timer = (lambda f: graph_ms(torch, f, 20)) if S <= 4096 else (lambda f: time_calls(torch, f, max(steps, 10)))
        out[name] = {"shape": [B, H, S, D], "fused_ms": timer(fused), "rotary_then_forward_ms": timer(unfused),
                     "forward_alone_ms": timer(plain)}
    # decoding: one new row per sequence against a rotated cache (the decode_cmp shape); the
    # forward splits the keys, so both forms get the workspace
    B, Hq, Hkv, Sk, D = 8, 32, 8, 8192, 128
    g = torch.Generator(device="cuda"); g.manual_seed(1016)
    Q = torch.randn((B, Hq, 1, D), device="cuda", generator=g).to(torch.bfloat16)
    K, V = (torch.randn((B, Hkv, Sk, D), device="cuda", generator=g).to(torch.bfloat16) for _ in range(2))
    ang = torch.arange(Sk, device="cuda", dtype=torch.float32)[:, None] * \
        (10000.0 ** (-torch.arange(0, D, 2, device="cuda", dtype=torch.float32) / D))[None, :]
    cos, sin = torch.cos(ang).contiguous(), torch.sin(ang).contiguous()
    last_c, last_s = cos[Sk - 1:].contiguous(), sin[Sk - 1:].contiguous()
    O, Qr = torch.empty_like(Q), torch.empty_like(Q)
    LSE = torch.empty((B, Hq, 1), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(256, attn.attn_fwd_rect_workspace_bytes(B, Hq, Hkv, 1, Sk, D, True)),
                     dtype=torch.uint8, device="cuda")
    sc = 1.0 / float(D) ** 0.5

    def fused_d():
        attn.attn_fwd_rope(Q, K, V, cos, sin, sc, True, O=O, LSE=LSE, Q_rot=Qr)   # allocates its workspace

    def unfused_d():
        rowops.rotary_fwd(Q, last_c, last_s, y=Qr)
        attn.attn_fwd_rect(Qr, K, V, sc, True, O=O, LSE=LSE, workspace=ws)

    for _ in range(warmup):
        fused_d(); unfused_d()
    out["decode_shape"] = {"shape": [B, Hq, Hkv, 1, Sk, D], "fused_ms": graph_ms(torch, fused_d, 20),
                           "rotary_then_forward_ms": graph_ms(torch, unfused_d, 20)}
    return out


def rowops_main(torch, a):
    """The JSON line for --workload rowops."""
    r = measure_rowops(torch, a.steps, a.warmup)
    names = ("rmsnorm_fwd", "layernorm_fwd", "layernorm_bwd", "rotary_fwd")
    total_b = sum(r[k]["algorithmic_bytes"] for k in names)
    total_ms = sum(r[k]["ms"] for k in names)
    dom = max(names, key=lambda k: r[k]["ms"])
    out = {
        "metric": "row-wise kernels (RMSNorm fwd, LayerNorm fwd+bwd, rotary fwd): algorithmic GB/s",
        "value": total_b / (total_ms * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": total_ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "rowops: norms (4096, 8192), rotary (4, 8, 2048, 128), the paper's table shapes"},
        "kernels": r,
        "roofline": {"kernel": dom, "bound": "hbm", "achieved": r[dom]["gbs"], "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": r[dom]["frac_hbm_peak"],
                     "traffic": MEASURED_TRAFFIC_BYTES.get(("rowops", dom))},
    }
    if not a.no_cpu_baseline:
        import numpy as np
        import oracle
        rows, cols = 512, 8192
        rng = np.random.Generator(np.random.PCG64(1013))
        from paper_2601_16238_amd import workloads as wl
        xb = wl.f32_to_bf16_bits(rng.standard_normal((rows, cols), dtype=np.float32))
        w = np.ones(cols, np.float32)
        t0 = time.perf_counter()
        oracle.rowops.rmsnorm_fwd(xb, w, 1e-6)
        oracle.rowops.layernorm_fwd(xb, w, w, 1e-5)
        oracle.rowops.layernorm_bwd(xb, xb, w, 1e-5)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 7 * rows * cols * 2 / dt / 1e9, "unit": "GB/s",
                               "cores": oracle.num_threads(), "kind": "oracle", "seconds": dt,
                               "sample": "RMSNorm fwd, LayerNorm fwd and bwd on 512 of the 4096 rows (fp64)"}
    print(json.dumps(out))


def cpu_baseline(wl, w):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload: forward +
    backward of whole heads at full sequence length -- one head first, then as many as fit
    in roughly 15 s of CPU work (the reported figure is from that second run)."""
    import oracle

    gqa = hasattr(w, "Hq")   # grouped-query: a "head" of the sample is a K/V head with its group
    n_heads = w.B * (w.Hkv if gqa else w.H)
    per_head = (w.Hq // w.Hkv) if gqa else 1

    def run(heads):
        x = wl.make_gqa_inputs(w, kv_heads=range(heads)) if gqa else wl.make_inputs(w, heads=range(heads))
        t0 = time.perf_counter()
        oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], w.causal)
        oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], w.causal)
        return time.perf_counter() - t0

    heads, dt = 1, run(1)
    more = int(min(n_heads, 15.0 // max(dt, 1e-3)))
    if more > 1:
        heads, dt = more, run(more)
    flops = heads * per_head * 3.5 * wl.fwd_flops(1, 1, w.S, w.D, w.causal)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": dt,
            "sample": "fwd+bwd of the first %d of %d %sheads of %s at full S=%d (fp64, convention FLOPs)"
                      % (heads, n_heads, "K/V " if gqa else "", w.name, w.S)}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build is single-GPU (attention shards over batch*heads with no "
              "exchange; nothing here uses a second GPU). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2601_16238_amd as attn
    from paper_2601_16238_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    attn.lib()  # fail loudly if the HIP library is not built
    if a.calib_copy:
        src = torch.empty(CALIB_COPY_BYTES // 2, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if a.workload == "rowops":
        rowops_main(torch, a)
        return
    if a.workload == "rope":
        print(json.dumps({"rope_fused_forward": measure_rope(torch, attn, a.steps, a.warmup)}))
        return
    if a.workload in wl.RECT_WORKLOADS:
        rect_main(torch, attn, wl, wl.RECT_WORKLOADS[a.workload], a)
        return
    w = wl.WORKLOADS[a.workload] if a.workload in wl.WORKLOADS else wl.GQA_WORKLOADS[a.workload]
    r = measure(torch, attn, wl, w, a.steps, a.warmup)
    dom = max(r["kernels"], key=lambda k: r["kernels"][k]["ms"])
    out = {
        "metric": "attention fwd+bwd TFLOP/s (FLOPs = 4*B*H*S^2*D fwd, /2 causal, bwd = 2.5x fwd)",
        "value": r["tflops_fwdbwd"], "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %s" % (w.name, " ".join(
            "%s=%s" % (k, getattr(w, k)) for k in w._fields if k in ("B", "H", "Hq", "Hkv", "S", "D", "causal"))),
                   "seed": w.seed},
        "frac_of_bf16_peak": {"fwd": r["tflops_fwd"] / PEAK_BF16_TFLOPS,
                              "fwd_bwd": r["tflops_fwdbwd"] / PEAK_BF16_TFLOPS,
                              "peak_tflops": PEAK_BF16_TFLOPS},
        "tflops": {"fwd": r["tflops_fwd"], "bwd": r["tflops_bwd"], "fwd_bwd": r["tflops_fwdbwd"]},
        "ms": r["ms"],
        "algorithmic_gbs": {"fwd": r["gbs_fwd"], "bwd": r["gbs_bwd"], "hbm_peak": PEAK_HBM_GBS},
        "roofline": {"kernel": dom, "bound": "mfma", "achieved": r["kernels"][dom]["achieved_tflops"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": r["kernels"][dom]["frac"],
                     "traffic": measured_traffic_bytes(w.name, dom)},
        "roofline_all": r["kernels"],
    }
    probe = measure_mfma_peak(torch, attn)
    out["mfma_probe"] = probe
    out["roofline"]["frac_of_measured_peak"] = out["roofline"]["achieved"] / probe["tflops"]
    out["frac_of_measured_mfma_peak"] = {"fwd": r["tflops_fwd"] / probe["tflops"],
                                         "fwd_bwd": r["tflops_fwdbwd"] / probe["tflops"]}
    if a.all:
        others = {}
        for name, ow in list(wl.WORKLOADS.items()) + list(wl.GQA_WORKLOADS.items()):
            if name == w.name:
                continue
            o = measure(torch, attn, wl, ow, max(5, a.steps // 2), a.warmup)
            others[name] = {"shape": {k: getattr(ow, k) for k in ow._fields if k in
                                      ("B", "H", "Hq", "Hkv", "S", "D", "causal")},
                            "ms": o["ms"], "tflops_fwd": o["tflops_fwd"], "tflops_fwdbwd": o["tflops_fwdbwd"],
                            "frac_fwd": o["tflops_fwd"] / PEAK_BF16_TFLOPS,
                            "frac_fwdbwd": o["tflops_fwdbwd"] / PEAK_BF16_TFLOPS,
                            "gbs_fwd": o["gbs_fwd"], "gbs_bwd": o["gbs_bwd"]}
            for k in ("gbs_fwd_graph_replay", "gbs_bwd_graph_replay", "tflops_fwdbwd_graph_replay"):
                if k in o:
                    others[name][k] = o[k]
            if per_tensor_bytes(ow) <= (16 << 20) and not hasattr(ow, "Hq"):
                others[name]["cold"] = measure_cold(torch, attn, wl, ow, max(5, a.steps // 2))
            torch.cuda.empty_cache()
        out["other_workloads"] = others
        rect = {}
        for name, ow in wl.RECT_WORKLOADS.items():
            o = measure_rect(torch, attn, wl, ow, max(5, a.steps // 2), a.warmup)
            rect[name] = {"shape": {k: getattr(ow, k) for k in ("B", "Hq", "Hkv", "Sq", "Sk", "D", "causal")},
                          "ms": o["ms"], "key_splits": o["splits"], "tflops_fwd": o["tflops_fwd"],
                          "tflops_fwdbwd": o["tflops_fwdbwd"], "gbs_fwd": o["gbs_fwd"],
                          "gbs_fwd_cache_cold": o["gbs_fwd_cache_cold"], "gbs_bwd": o["gbs_bwd"]}
            torch.cuda.empty_cache()
        out["rect_workloads"] = rect
        out["row_kernels"] = measure_rowops(torch, a.steps, a.warmup)
        out["rope_fused_forward"] = measure_rope(torch, attn, a.steps, a.warmup)
        # the fp16 build of the kernels on the main shape (through the rectangular entry points)
        g = torch.Generator(device="cuda"); g.manual_seed(w.seed)
        H = w.Hq if hasattr(w, "Hq") else w.H
        q16, k16, v16, do16 = (torch.randn((w.B, H, w.S, w.D), device="cuda", generator=g)
                               .to(torch.float16) for _ in range(4))
        sc = wl.default_scale(w.D)
        o16, l16 = attn.attn_fwd_rect(q16, k16, v16, sc, w.causal)
        bufs = [torch.empty_like(q16) for _ in range(3)]
        ws16 = torch.empty(attn.attn_bwd_rect_workspace_bytes(w.B, H, H, w.S, w.S, w.D),
                           dtype=torch.uint8, device="cuda")
        f16_fwd = time_calls(torch, lambda: attn.attn_fwd_rect(q16, k16, v16, sc, w.causal, O=o16, LSE=l16), 10)
        f16_bwd = time_calls(torch, lambda: attn.attn_bwd_rect(q16, k16, v16, o16, do16, l16, sc, w.causal,
                                                                dQ=bufs[0], dK=bufs[1], dV=bufs[2],
                                                                workspace=ws16), 10)
        ff = wl.fwd_flops(w.B, H, w.S, w.D, w.causal)
        out["f16_same_shape"] = {"ms": {"fwd": f16_fwd, "bwd": f16_bwd},
                                 "tflops_fwd": ff / (f16_fwd * 1e-3) / 1e12,
                                 "tflops_fwdbwd": 3.5 * ff / ((f16_fwd + f16_bwd) * 1e-3) / 1e12}
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, w)
        out["cpu_baseline"]["nproc"] = os.cpu_count()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
