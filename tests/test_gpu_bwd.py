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
from parity_util import check_bf16, to_dev, to_f64

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


@pytest.mark.parametrize("name", ["tiny", "vit_cifar", "minigpt"])
def test_bwd_workload_full(name):
    print("case bwd_workload_full", name, flush=True)
    x = wl.make_inputs(name)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], x["causal"])
    got = run_gpu(x, x["causal"])
    for nm, g, r in zip(("dQ", "dK", "dV"), got, ref):
        check_bf16(nm, g, r)
