"""GPU regression guards for the bug classes the paper's debugging table lists for its
attention kernel: buffers reused across iterations without initialisation, launch
configurations, and call-interface (stride) handling."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_16238_amd as attn
from paper_2601_16238_amd import workloads as wl
from parity_util import check_bf16, check_grad, check_lse, to_dev, to_f64

pytestmark = pytest.mark.gpu


def poison(*ts):
    for t in ts:
        if t.dtype == torch.uint8:
            t.fill_(0x7F)
        else:
            t.fill_(float("nan"))


@pytest.mark.parametrize("B,H,S,D,causal", [(2, 2, 300, 64, True), (1, 2, 257, 128, False)])
def test_poisoned_outputs_and_workspace_repeat_bit_identical(B, H, S, D, causal):
    """Outputs and workspace are filled with NaN / garbage before every call; twelve
    consecutive fwd+bwd calls on the same buffers must give bit-identical, finite results
    (no atomics, nothing accumulated into caller buffers)."""
    print("case poison_repeat", B, H, S, D, causal, flush=True)
    x = wl.random_inputs(B, H, S, D, seed=300 + S)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O = torch.empty_like(Q)
    LSE = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
    ws = torch.empty(attn.attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")
    first = None
    for it in range(12):
        poison(O, LSE, dQ, dK, dV, ws)
        attn.attn_fwd(Q, K, V, x["scale"], causal, O=O, LSE=LSE)
        attn.attn_bwd(Q, K, V, O, dO, LSE, x["scale"], causal, dQ=dQ, dK=dK, dV=dV, workspace=ws)
        torch.cuda.synchronize()
        cur = [t.clone() for t in (O, LSE, dQ, dK, dV)]
        for t in cur:
            assert torch.isfinite(t.float()).all(), "iteration %d produced non-finite values" % it
        if first is None:
            first = cur
        else:
            for a, b in zip(first, cur):
                assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), "iteration %d differs" % it
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    for nm, t, r in zip(("dQ", "dK", "dV"), first[2:], ref):
        check_bf16(nm, to_f64(t), r)


@pytest.mark.parametrize("B,H,S,D,causal", [(2, 3, 200, 64, True), (1, 3, 333, 128, True), (1, 2, 300, 256, False)])
def test_bshd_strides_and_side_stream(B, H, S, D, causal):
    """[B,S,H,D] storage viewed as [B,H,S,D] (stride_h = D, stride_s = H*D), launched on a
    non-default stream.  (The second shape runs the eight-wave kernels, the third the D = 256
    ones: their rows enter and leave through LDS in whole-row transfers, strided here.)"""
    print("case bshd_strides", B, H, S, D, causal, flush=True)
    x = wl.random_inputs(B, H, S, D, seed=41)

    def bshd(bits):
        t = to_dev(bits)                                   # [B,H,S,D] contiguous
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)  # same values, BSHD memory

    Q, K, V, dO = (bshd(x[k]) for k in ("Q", "K", "V", "dO"))
    assert Q.stride() == (S * H * D, D, H * D, 1)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        O, LSE = attn.attn_fwd(Q, K, V, x["scale"], causal, stream=st)
        dQ, dK, dV = attn.attn_bwd(Q, K, V, O, dO, LSE, x["scale"], causal, stream=st)
    st.synchronize()
    assert O.stride() == Q.stride() and dK.stride() == Q.stride()
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)
    for nm, t, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        check_bf16(nm, to_f64(t), r)


def test_explicit_stream_without_stream_context():
    """stream= given while torch's current stream is another one: outputs and workspaces that
    the binding allocates itself must belong to the stream the kernels run on.  While the side
    stream works, the current stream allocates and overwrites buffers of the workspace's size;
    if the workspace had been handed back to the current stream's pool, one of them would land
    on it."""
    print("case explicit_stream", flush=True)
    B, H, S, D, causal = 2, 4, 1500, 128, True
    x = wl.random_inputs(B, H, S, D, seed=47)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    results = []
    for _ in range(5):
        O, LSE = attn.attn_fwd(Q, K, V, x["scale"], causal, stream=st)
        dQ, dK, dV = attn.attn_bwd(Q, K, V, O, dO, LSE, x["scale"], causal, stream=st)
        # work of the current stream that would reuse a block freed to its pool
        junk = [torch.full((attn.attn_bwd_workspace_bytes(B, H, S, D) // 4,), float("nan"),
                           device="cuda") for _ in range(4)]
        results.append((O, LSE, dQ, dK, dV))
        del junk
    st.synchronize()
    torch.cuda.synchronize()
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    for O, LSE, dQ, dK, dV in results:
        check_bf16("O", to_f64(O), Oref)
        check_lse(to_f64(LSE), Lref)
        for nm, t, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
            check_grad(nm, to_f64(t), r)


def test_isolated_backward_from_oracle_O_and_LSE():
    """Backward fed with bf16(O_oracle) and fp32(LSE_oracle) instead of the GPU forward's
    outputs: isolates the backward kernels from the forward."""
    print("case isolated_bwd", flush=True)
    B, H, S, D, causal = 1, 2, 333, 128, True
    x = wl.random_inputs(B, H, S, D, seed=42)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    ref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O = torch.from_numpy(Oref).to(torch.bfloat16).cuda()
    LSE = torch.from_numpy(Lref).to(torch.float32).cuda()
    dQ, dK, dV = attn.attn_bwd(Q, K, V, O, dO, LSE, x["scale"], causal)
    torch.cuda.synchronize()
    for nm, t, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        check_bf16(nm, to_f64(t), r)


def test_large_scores_do_not_overflow():
    """Scores of several hundred (outlier rows of the long-sequence workload): the running
    max must track them; compare with the oracle at 1e-5 + 1e-5*|LSE|."""
    print("case large_scores", flush=True)
    B, H, S, D = 1, 2, 500, 128
    x = wl.random_inputs(B, H, S, D, seed=43, sigma=8.0)
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], True)
    assert Lref.max() > 100
    O, LSE = attn.attn_fwd(to_dev(x["Q"]), to_dev(x["K"]), to_dev(x["V"]), x["scale"], True)
    torch.cuda.synchronize()
    got = to_f64(LSE)
    assert np.isfinite(got).all() and (np.abs(got - Lref) <= 1e-5 + 1e-5 * np.abs(Lref)).all()
    d = np.abs(to_f64(O) - Oref)
    assert d.max() <= 2e-2 * max(1.0, np.abs(Oref).max()) and np.isfinite(d).all()


@pytest.mark.parametrize("B,H,S,D,causal", [(5, 8, 600, 64, True), (3, 8, 520, 64, False),
                                            (1, 24, 300, 128, True), (9, 8, 130, 64, True)])
def test_work_group_order_covers_every_head_and_tile(B, H, S, D, causal):
    """The work-groups walk the heads of an XCD in small groups; with B*H = 40, 24 or 72 the
    heads per XCD (5, 3, 9) are no multiple of the group size, so the last group is a smaller
    one.  Every (head, tile) must still be computed exactly once: outputs are poisoned first
    and all of them are compared with the oracle."""
    print("case tile_order", B, H, S, D, causal, flush=True)
    x = wl.random_inputs(B, H, S, D, seed=900 + B * H)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O = torch.empty_like(Q)
    LSE = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
    ws = torch.empty(attn.attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")
    poison(O, LSE, dQ, dK, dV, ws)
    attn.attn_fwd(Q, K, V, x["scale"], causal, O=O, LSE=LSE)
    attn.attn_bwd(Q, K, V, O, dO, LSE, x["scale"], causal, dQ=dQ, dK=dK, dV=dV, workspace=ws)
    torch.cuda.synchronize()
    Oref, Lref = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    gref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    check_bf16("O", to_f64(O), Oref)
    check_lse(to_f64(LSE), Lref)
    for nm, t, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), gref):
        check_bf16(nm, to_f64(t), r)


@pytest.mark.parametrize("B,H,S,D,causal", [(2, 3, 333, 128, True), (1, 8, 96, 64, False)])
def test_stage_wise_backward_equals_the_full_call(B, H, S, D, causal):
    """attn_bwd forms the row statistics inside the dQ kernel; called stage by stage (separate
    statistics kernel, then dK/dV and dQ reading them from the workspace) the gradients must be
    the same.  The statistics of the two paths may differ in the last bit (other summation
    order), so dK/dV of the stage-wise path are compared within one bf16 ulp; dQ from the
    separately computed statistics likewise."""
    from paper_2601_16238_amd import binding
    print("case stage_wise", B, H, S, D, causal, flush=True)
    x = wl.random_inputs(B, H, S, D, seed=1300 + S)
    Q, K, V, dO = (to_dev(x[k]) for k in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd(Q, K, V, x["scale"], causal)
    ws = torch.empty(attn.attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")
    full = attn.attn_bwd(Q, K, V, O, dO, LSE, x["scale"], causal, workspace=ws)
    torch.cuda.synchronize()
    stats_full = ws.clone()
    outs = [torch.full_like(Q, float("nan")) for _ in range(3)]
    ws.fill_(0x7F)
    for st in (binding.STAGE_DELTA, binding.STAGE_DKDV, binding.STAGE_DQ):
        attn.attn_bwd(Q, K, V, O, dO, LSE, x["scale"], causal, dQ=outs[0], dK=outs[1], dV=outs[2],
                      workspace=ws, stages=st)
    torch.cuda.synchronize()
    a, b = stats_full.view(torch.float32), ws.view(torch.float32)
    n = B * H * 2 * S
    assert torch.allclose(a[:n], b[:n], rtol=1e-5, atol=1e-5)
    for nm, f, s in zip(("dQ", "dK", "dV"), full, outs):
        d = (f.double() - s.double()).abs()
        tol = 2.0 ** -7 * torch.maximum(f.double().abs(), torch.tensor(2.0 ** -6, device="cuda", dtype=torch.float64))
        assert bool((d <= tol).all()), (nm, d.max().item())
    gref = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    for nm, t, r in zip(("dQ", "dK", "dV"), outs, gref):
        check_bf16(nm, to_f64(t), r)
