"""The autograd wrapper: gradients that torch.autograd routes through the fused operator
equal the oracle's, also when the upstream gradient arrives in another layout."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import workloads as wl

pytestmark = pytest.mark.gpu


def dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def host(t):
    return t.detach().to(torch.float64).cpu().numpy()


@pytest.mark.parametrize("causal", [False, True])
def test_gradients_through_autograd_match_the_oracle(causal):
    w = wl.RectWorkload("autograd_case", 2, 4, 2, 70, 133, 64, causal, 1.0, 4242, "test")
    x = wl.make_rect_inputs(w)
    print("case", w, flush=True)
    q, k, v = (dev(x[n]).requires_grad_(True) for n in ("Q", "K", "V"))
    out = attn.fused_attention(q, k, v, causal=causal, scale=x["scale"])
    # the upstream gradient in a different memory order than the output
    dO = dev(x["dO"]).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert dO.stride() != out.stride()
    out.backward(dO)
    torch.cuda.synchronize()
    Oref, _ = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    gref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    for name, got, ref in (("O", out, Oref), ("dQ", q.grad, gref[0]), ("dK", k.grad, gref[1]),
                           ("dV", v.grad, gref[2])):
        d = np.abs(host(got) - ref)
        assert d.max() <= 2e-2 and d.mean() <= 2e-3, (name, d.max(), d.mean())


def test_default_scale_and_non_dense_inputs():
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    big = torch.randn((1, 2, 40, 72), device="cuda", generator=g).to(torch.bfloat16)
    q = big[..., 4:68]          # D = 64 view at an offset of 8 bytes: not 16-byte aligned
    k, v = (torch.randn((1, 2, 40, 64), device="cuda", generator=g).to(torch.bfloat16) for _ in range(2))
    out = attn.fused_attention(q, k, v)
    ref, _ = attn.attn_fwd_rect(q.contiguous(), k, v, 64 ** -0.5, False)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


def test_cpu_tensors_are_refused():
    t = torch.zeros((1, 1, 8, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        attn.fused_attention(t, t, t)
