"""The backward entry point that allocates nothing (static scratch inside the library) against
attn_bwd_rect, which takes the same scratch as a workspace argument (here of the same size):
same kernels and the same plan, so the results must agree bit for bit -- on two calls in a row, the second on a smaller problem (the
scratch keeps the first call's contents), and beyond the scratch's size the call must refuse."""
import ctypes

import pytest
import torch

import paper_2601_16238_amd as attn
from paper_2601_16238_amd import binding, workloads as wl
from parity_util import to_dev

pytestmark = pytest.mark.gpu


def run_pair(B, Hq, Hkv, Sq, Sk, D, causal, seed):
    x = wl.random_rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=seed)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd_rect(Q, K, V, x["scale"], causal)
    # (a workspace of the static scratch's size: the same plan for the dQ kernel)
    ws = torch.empty(binding.NOALLOC_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    ref = attn.attn_bwd_rect(Q, K, V, O, dO, LSE, x["scale"], causal, workspace=ws)
    got = tuple(torch.full_like(t, float("nan")) for t in ref)
    binding.attn_bwd_rect_noalloc(Q, K, V, O, dO, LSE, x["scale"], causal, *got)
    torch.cuda.synchronize()
    for name, g, r in zip(("dQ", "dK", "dV"), got, ref):
        assert torch.isfinite(g.float()).all(), name
        assert torch.equal(g.view(torch.int16), r.view(torch.int16)), name


def test_noalloc_backward_equals_the_workspace_form_on_two_calls_in_a_row():
    print("case noalloc 1: B=2 Hq=8 Hkv=2 Sq=Sk=1500 D=128 causal", flush=True)
    run_pair(2, 8, 2, 1500, 1500, 128, True, seed=901)
    print("case noalloc 2 (smaller, same scratch): B=1 Hq=4 Hkv=4 Sq=77 Sk=300 D=64", flush=True)
    run_pair(1, 4, 4, 77, 300, 64, False, seed=902)
    print("case noalloc 3: B=1 Hq=2 Hkv=1 Sq=Sk=640 D=96 causal", flush=True)
    run_pair(1, 2, 1, 640, 640, 96, True, seed=903)


def test_noalloc_backward_refuses_problems_beyond_its_scratch():
    """More query rows than the static scratch holds statistics for: ATTN_ERR_WORKSPACE, decided
    on the host from the shape alone (the pointers are never dereferenced)."""
    rows = binding.NOALLOC_SCRATCH_BYTES // 8
    B, H, D = 1, 8, 64
    S = rows // H + 256
    p = binding.make_rect_params(B, H, H, S, S, D, 0.125, False)
    fake = ctypes.c_void_p(0x10000)  # aligned, non-NULL, never used
    rc = binding.lib().attn_bwd_rect_noalloc(fake, fake, fake, fake, fake, fake, fake, fake, fake,
                                             ctypes.byref(p), None)
    assert rc == binding.ATTN_ERR_WORKSPACE, rc
    # one row fewer than the limit would be accepted by the size check (not launched here)
    assert 8 * B * H * (rows // H) <= binding.NOALLOC_SCRATCH_BYTES
