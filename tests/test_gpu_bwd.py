"""GPU parity: attn_bwd through the C ABI against the fp64 oracle, element by element.

End-to-end reading: the GPU backward consumes the GPU forward's bf16 O and fp32 LSE; the
oracle backward always uses its own fp64 O and LSE.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import workloads as wl
from parity_util import check_bf16, check_grad, to_dev, to_f64

pytestmark = pytest.mark.gpu

SMALL = [
    (1, 2, 128, 64, False), (1, 2, 128, 64, True),
    (2, 3, 65, 64, False), (2, 3, 65, 64, True),
    (1, 1, 1, 64, False), (1, 1, 1, 128, True),
    (1, 2, 31, 128, False), (1, 2, 33, 64, True), (1, 2, 96, 128, True),
    (1, 2, 300, 64, True), (1, 2, 300, 64, False),
    (2, 2, 257, 128, True), (2, 2, 257, 128, False),
    (1, 2, 1000, 128, True), (1, 1, 777, 128, False), (1, 3, 513, 64, True),
]


def run_gpu(x, causal):
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd(Q, K, V, x["scale"], causal)
    dQ, dK, dV = attn.attn_bwd(Q, K, V, O, dO, LSE, x["scale"], causal)
    torch.cuda.synchronize()
    return to_f64(dQ), to_f64(dK), to_f64(dV)


@pytest.mark.parametrize("B,H,S,D,causal", SMALL)
def test_bwd_small(B, H, S, D, causal):
    print("case bwd_small", B, H, S, D, causal, flush=True)
    x = wl.random_inputs(B, H, S, D, seed=200 + S)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    got = run_gpu(x, causal)
    for name, g, r in zip(("dQ", "dK", "dV"), got, ref):
        check_bf16(name, g, r)


# Sequence lengths around the tile sizes of the kernels: 32-row slots / sub-tiles, 64-row tiles,
# 128-key blocks of the dK/dV kernel, 256-query blocks of the dQ kernel, and lengths short
# enough that the streaming ring never fills.
SWEEP_S = [2, 32, 34, 63, 64, 95, 127, 129, 160, 161, 192, 255, 256, 259, 383, 385, 641]


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("causal", [False, True])
def test_bwd_length_sweep(D, causal):
    for S in SWEEP_S:
        print("case bwd_length_sweep", S, D, causal, flush=True)
        x = wl.random_inputs(1, 2, S, D, seed=700 + S)
        ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
        got = run_gpu(x, causal)
        for name, g, r in zip(("dQ", "dK", "dV"), got, ref):
            if S < 32:
                # probabilities near 1/2 make dS = P (dP - delta) feel the bf16 rounding of the
                # forward's O (through delta) far above the rounding floor of the few outputs;
                # the literal tolerances still hold
                check_bf16("S=%d %s" % (S, name), g, r, floor_gate=False)
            else:
                # unit-variance inputs (the paper-shaped workloads use smaller ones) give
                # gradients of magnitude 2-5, where one bf16 ulp is already 1.6e-2 to 3.1e-2:
                # the scale-aware reading with its gate relative to the rounding floor applies
                check_grad("S=%d %s" % (S, name), g, r)


@pytest.mark.parametrize("name", ["tiny", "vit_cifar", "minigpt"])
def test_bwd_workload_full(name):
    print("case bwd_workload_full", name, flush=True)
    x = wl.make_inputs(name)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], x["causal"])
    got = run_gpu(x, x["causal"])
    for nm, g, r in zip(("dQ", "dK", "dV"), got, ref):
        check_bf16(nm, g, r)
