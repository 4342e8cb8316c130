"""GPU parity: attn_fwd through the C ABI against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import workloads as wl
from parity_util import check_bf16, check_lse, to_dev, to_f64

pytestmark = pytest.mark.gpu

# (B,H,S,D,causal): several tiles, ragged tails, single row, every work-group width.
SMALL = [
    (1, 2, 128, 64, False), (1, 2, 128, 64, True),
    (2, 3, 65, 64, False), (2, 3, 65, 64, True),
    (1, 1, 1, 64, False), (1, 1, 1, 128, True),
    (1, 2, 31, 128, False), (1, 2, 33, 64, True), (1, 2, 96, 128, True),
    (1, 2, 300, 64, True), (1, 2, 300, 64, False),
    (2, 2, 257, 128, True), (2, 2, 257, 128, False),
    (1, 2, 1000, 128, True), (1, 1, 777, 128, False), (1, 3, 513, 64, True),
]


@pytest.mark.parametrize("B,H,S,D,causal", SMALL)
def test_fwd_small(B, H, S, D, causal):
    print("case fwd_small", B, H, S, D, causal, flush=True)
    x = wl.random_inputs(B, H, S, D, seed=100 + S)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    O, LSE = attn.attn_fwd(to_dev(x["Q"]), to_dev(x["K"]), to_dev(x["V"]), x["scale"], causal)
    torch.cuda.synchronize()
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)


# Sequence lengths around the tile sizes: 32-key sub-tiles, 64-key tiles, 256-query blocks.
SWEEP_S = [2, 32, 34, 63, 64, 95, 127, 129, 160, 161, 192, 255, 256, 259, 383, 385, 641]


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("causal", [False, True])
def test_fwd_length_sweep(D, causal):
    for S in SWEEP_S:
        print("case fwd_length_sweep", S, D, causal, flush=True)
        x = wl.random_inputs(1, 2, S, D, seed=600 + S)
        Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
        O, LSE = attn.attn_fwd(to_dev(x["Q"]), to_dev(x["K"]), to_dev(x["V"]), x["scale"], causal)
        torch.cuda.synchronize()
        check_bf16("S=%d O" % S, to_f64(O), Oref)
        check_lse(to_f64(LSE), Lref)


@pytest.mark.parametrize("name", ["tiny", "vit_cifar", "minigpt"])
def test_fwd_workload_full(name):
    print("case fwd_workload_full", name, flush=True)
    x = wl.make_inputs(name)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], x["causal"])
    O, LSE = attn.attn_fwd(to_dev(x["Q"]), to_dev(x["K"]), to_dev(x["V"]), x["scale"], x["causal"])
    torch.cuda.synchronize()
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)
