"""Pins for the CPU fp64 oracle: everything here is fixed by mathematics or by an
independent library routine, never by the oracle itself and never by the GPU path.

The paper prints no numeric attention values (its microbenchmark table has latencies
only), so there is no golden file from the paper; the pins are closed forms, invariants,
finite differences and torch's fp64 autograd on small inputs.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_16238_amd import workloads as wl


def rnd(B, H, S, D, seed, sigma=1.0):
    return wl.random_inputs(B, H, S, D, seed, sigma)


def f64(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def bits(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


SHAPES = [(1, 1, 1, 8), (1, 2, 5, 8), (2, 1, 7, 16), (1, 1, 33, 64), (1, 2, 65, 64)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", SHAPES)
def test_rows_of_P_sum_to_one_and_mask_is_zero(shape, causal):
    x = rnd(*shape, seed=11)
    P = oracle.attn_probs(x["Q"], x["K"], x["V"], x["scale"], causal)
    assert np.all(P >= 0)
    np.testing.assert_allclose(P.sum(-1), 1.0, rtol=0, atol=1e-12)
    if causal:
        S = shape[2]
        upper = np.triu(np.ones((S, S), bool), k=1)
        assert np.all(P[..., upper] == 0.0)
        # the diagonal is allowed: it carries probability
        assert np.all(P[..., np.arange(S), np.arange(S)] > 0)


@pytest.mark.parametrize("causal", [False, True])
def test_uniform_V_gives_O_equal_V(causal):
    x = rnd(1, 2, 37, 16, seed=12)
    v = f64(bits(np.random.default_rng(0).standard_normal(16)))
    V = np.broadcast_to(bits(v), x["V"].shape).copy()
    O, _ = oracle.attn_fwd(x["Q"], x["K"], V, x["scale"], causal)
    np.testing.assert_allclose(O, np.broadcast_to(v, O.shape), rtol=0, atol=1e-13)


def test_causal_row0_is_V0_and_LSE_is_s00():
    x = rnd(2, 2, 19, 16, seed=13)
    O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], True)
    np.testing.assert_allclose(O[:, :, 0, :], f64(x["V"])[:, :, 0, :], rtol=0, atol=1e-14)
    s00 = np.float64(np.float32(x["scale"])) * (f64(x["Q"])[:, :, 0] * f64(x["K"])[:, :, 0]).sum(-1)
    np.testing.assert_allclose(LSE[:, :, 0], s00, rtol=0, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("S", [1, 7, 65])
def test_zero_Q_closed_form_natural_log(S, causal):
    """Q = 0 => P uniform over the allowed keys: LSE_i = ln n_i (natural log), O_i = mean
    of the allowed V rows, dV_j = sum_{i: j allowed} dO_i / n_i, dK = 0."""
    x = rnd(1, 2, S, 8, seed=14)
    Q0 = np.zeros_like(x["Q"])
    O, LSE = oracle.attn_fwd(Q0, x["K"], x["V"], x["scale"], causal)
    n = np.arange(1, S + 1, dtype=np.float64) if causal else np.full(S, float(S))
    np.testing.assert_allclose(LSE, np.broadcast_to(np.log(n), LSE.shape), rtol=0, atol=1e-13)
    V, dO = f64(x["V"]), f64(x["dO"])
    if causal:
        Oref = np.cumsum(V, axis=2) / n[None, None, :, None]
        # dV_j = sum_{i>=j} dO_i / (i+1): reversed cumulative sum
        w = dO / n[None, None, :, None]
        dVref = np.flip(np.cumsum(np.flip(w, 2), axis=2), 2)
    else:
        Oref = np.broadcast_to(V.mean(2, keepdims=True), V.shape)
        dVref = np.broadcast_to(dO.sum(2, keepdims=True) / S, V.shape)
    np.testing.assert_allclose(O, Oref, rtol=0, atol=1e-13)
    dQ, dK, dV = oracle.attn_bwd(Q0, x["K"], x["V"], x["dO"], x["scale"], causal)
    np.testing.assert_allclose(dV, dVref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dK, 0.0, rtol=0, atol=1e-13)


def test_single_key_degenerate():
    x = rnd(2, 3, 1, 16, seed=15)
    for causal in (False, True):
        O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
        np.testing.assert_array_equal(O, f64(x["V"]))
        s = np.float64(np.float32(x["scale"])) * (f64(x["Q"]) * f64(x["K"])).sum(-1)
        np.testing.assert_allclose(LSE, s, rtol=0, atol=1e-13)
        dQ, dK, dV = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
        np.testing.assert_array_equal(dV, f64(x["dO"]))
        np.testing.assert_allclose(dQ, 0.0, atol=1e-14)
        np.testing.assert_allclose(dK, 0.0, atol=1e-14)


@pytest.mark.parametrize("causal", [False, True])
def test_dS_rows_sum_to_zero(causal):
    x = rnd(1, 2, 23, 16, seed=16)
    dS = oracle.attn_dscores(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    np.testing.assert_allclose(dS.sum(-1), 0.0, rtol=0, atol=1e-12)
    if causal:
        upper = np.triu(np.ones((23, 23), bool), k=1)
        assert np.all(dS[..., upper] == 0.0)


@pytest.mark.parametrize("causal", [False, True])
def test_key_shift_invariance(causal):
    """K_j -> K_j + c for all j leaves P (hence O, dV) unchanged and moves LSE_i by
    scale * q_i . c.  c is chosen so that K + c is still exactly representable in bf16."""
    rng = np.random.default_rng(17)
    B, H, S, D = 1, 2, 21, 16
    # small integers / 8 are exact in bf16 and so are their sums here
    K = rng.integers(-8, 9, (B, H, S, D)) / 8.0
    c = rng.integers(-8, 9, (D,)) / 8.0
    Q = rng.integers(-8, 9, (B, H, S, D)) / 8.0
    x = rnd(B, H, S, D, seed=17)
    Qb, Kb, K2b = bits(Q), bits(K), bits(K + c)
    assert np.array_equal(f64(K2b), K + c)
    O1, L1 = oracle.attn_fwd(Qb, Kb, x["V"], x["scale"], causal)
    O2, L2 = oracle.attn_fwd(Qb, K2b, x["V"], x["scale"], causal)
    np.testing.assert_allclose(O1, O2, rtol=0, atol=1e-12)
    shift = np.float64(np.float32(x["scale"])) * (Q @ c)
    np.testing.assert_allclose(L2 - L1, shift, rtol=0, atol=1e-12)
    g1 = oracle.attn_bwd(Qb, Kb, x["V"], x["dO"], x["scale"], causal)
    g2 = oracle.attn_bwd(Qb, K2b, x["V"], x["dO"], x["scale"], causal)
    np.testing.assert_allclose(g1[2], g2[2], rtol=0, atol=1e-12)   # dV
    np.testing.assert_allclose(g1[1], g2[1], rtol=0, atol=1e-12)   # dK (depends on P, Q only)


def test_key_permutation_equivariance_noncausal():
    x = rnd(1, 2, 29, 16, seed=18)
    perm = np.random.default_rng(18).permutation(29)
    Kp, Vp = x["K"][:, :, perm], x["V"][:, :, perm]
    O1, L1 = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], False)
    O2, L2 = oracle.attn_fwd(x["Q"], Kp, Vp, x["scale"], False)
    np.testing.assert_allclose(O1, O2, rtol=0, atol=1e-13)
    np.testing.assert_allclose(L1, L2, rtol=0, atol=1e-13)
    g1 = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], False)
    g2 = oracle.attn_bwd(x["Q"], Kp, Vp, x["dO"], x["scale"], False)
    np.testing.assert_allclose(g1[0], g2[0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(g1[1][:, :, perm], g2[1], rtol=0, atol=1e-13)
    np.testing.assert_allclose(g1[2][:, :, perm], g2[2], rtol=0, atol=1e-13)


def _loss_f64(Q, K, V, dO, scale, causal):
    """L = sum(O * dO) with O from an independent numpy einsum softmax (used only for the
    finite-difference quotient, on perturbed fp64 inputs the bf16 oracle cannot take)."""
    s = np.einsum("bhid,bhjd->bhij", Q, K) * scale
    if causal:
        S = Q.shape[2]
        s = np.where(np.tril(np.ones((S, S), bool)), s, -np.inf)
    s = s - s.max(-1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(-1, keepdims=True)
    return float((np.einsum("bhij,bhjd->bhid", p, V) * dO).sum())


@pytest.mark.parametrize("causal", [False, True])
def test_gradients_match_central_finite_differences(causal):
    """d/dx sum(O*dO) by central differences in fp64, every entry of Q, K and V.
    The loss helper is first tied to the oracle's own forward at the unperturbed point."""
    B, H, S, D = 1, 2, 6, 4
    x = rnd(B, H, S, D, seed=19)
    scale = np.float64(np.float32(0.37))
    Q, K, V, dO = (f64(x[k]) for k in ("Q", "K", "V", "dO"))
    O, _ = oracle.attn_fwd(x["Q"], x["K"], x["V"], 0.37, causal)
    assert abs((O * dO).sum() - _loss_f64(Q, K, V, dO, scale, causal)) < 1e-12
    grads = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], 0.37, causal)
    h = 1e-5
    for name, g in zip(("Q", "K", "V"), grads):
        arrs = {"Q": Q.copy(), "K": K.copy(), "V": V.copy()}
        a = arrs[name]
        fd = np.empty_like(a)
        it = np.nditer(a, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = a[idx]
            a[idx] = old + h
            lp = _loss_f64(arrs["Q"], arrs["K"], arrs["V"], dO, scale, causal)
            a[idx] = old - h
            lm = _loss_f64(arrs["Q"], arrs["K"], arrs["V"], dO, scale, causal)
            a[idx] = old
            fd[idx] = (lp - lm) / (2 * h)
        err = np.abs(fd - g).max() / max(1e-30, np.abs(g).max())
        assert err < 1e-6, (name, err)


TORCH_CASES = [(1, 2, 128, 64, False), (2, 3, 65, 64, False), (1, 2, 65, 64, True),
               (2, 2, 100, 128, True), (1, 1, 33, 128, False), (1, 1, 1, 64, True)]


@pytest.mark.parametrize("B,H,S,D,causal", TORCH_CASES)
def test_against_torch_fp64_autograd(B, H, S, D, causal):
    """Independent library routine: torch.softmax(Q K^T * scale + mask) V in CPU fp64 and
    torch.autograd for the gradients, plus torch.logsumexp for the LSE."""
    x = rnd(B, H, S, D, seed=20 + S)
    scale32 = np.float32(x["scale"])
    t = {k: torch.tensor(f64(x[k]), dtype=torch.float64, requires_grad=(k != "dO"))
         for k in ("Q", "K", "V", "dO")}
    s = (t["Q"] @ t["K"].transpose(-1, -2)) * float(scale32)
    if causal:
        mask = torch.ones(S, S, dtype=torch.bool).tril()
        s = s.masked_fill(~mask, float("-inf"))
    lse_t = torch.logsumexp(s, dim=-1)
    o_t = torch.softmax(s, dim=-1) @ t["V"]
    gq, gk, gv = torch.autograd.grad(o_t, (t["Q"], t["K"], t["V"]), grad_outputs=t["dO"])
    O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    dQ, dK, dV = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    np.testing.assert_allclose(O, o_t.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE, lse_t.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dQ, gq.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dK, gk.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dV, gv.numpy(), rtol=0, atol=1e-11)


def test_scale_is_applied_before_softmax_and_in_both_input_gradients():
    """Doubling scale must equal doubling Q (exactly representable), for O, LSE, dK, dV;
    and dQ halves (chain rule) -- catches a dropped or doubled scale factor."""
    x = rnd(1, 2, 17, 16, seed=21)
    Q2 = bits(2.0 * f64(x["Q"]))
    a = oracle.attn_fwd(x["Q"], x["K"], x["V"], 0.5, True)
    b = oracle.attn_fwd(Q2, x["K"], x["V"], 0.25, True)
    np.testing.assert_allclose(a[0], b[0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(a[1], b[1], rtol=0, atol=1e-13)
    ga = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], 0.5, True)
    gb = oracle.attn_bwd(Q2, x["K"], x["V"], x["dO"], 0.25, True)
    np.testing.assert_allclose(ga[0], 2.0 * gb[0], rtol=0, atol=1e-12)
    np.testing.assert_allclose(ga[1], gb[1], rtol=0, atol=1e-12)
    np.testing.assert_allclose(ga[2], gb[2], rtol=0, atol=1e-12)


def test_stability_with_large_scores():
    """Scores in the hundreds (the long-sequence workload's outlier rows) must not
    overflow: compare with torch.logsumexp on the same fp64 scores."""
    x = rnd(1, 1, 40, 32, seed=22, sigma=6.0)
    O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], 1.0, False)
    assert np.isfinite(O).all() and np.isfinite(LSE).all() and LSE.max() > 300
    s = torch.tensor(f64(x["Q"])[0, 0] @ f64(x["K"])[0, 0].T)
    np.testing.assert_allclose(LSE[0, 0], torch.logsumexp(s, -1).numpy(), rtol=1e-14, atol=1e-11)


# ---- grouped-query heads (the paper's benchmark shape is written (B,Hq,Hkv,S,D)) ----------
# K/V head of query head h is h // (Hq // Hkv); dK, dV of a K/V head sum over its group.

def gqa_inputs(B, Hq, Hkv, S, D, seed):
    x = rnd(B, Hq, S, D, seed)
    kv = rnd(B, Hkv, S, D, seed + 1000)
    x["K"], x["V"] = kv["K"], kv["V"]
    return x


GQA_CASES = [(1, 4, 2, 33, 16, False), (2, 6, 2, 20, 8, True), (1, 8, 1, 17, 16, True),
             (1, 4, 1, 65, 64, False), (1, 3, 3, 9, 8, True)]


@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal", GQA_CASES)
def test_gqa_equals_multihead_on_repeated_kv(B, Hq, Hkv, S, D, causal):
    """Reduction to the multi-head case pinned above: repeating every K/V head G times gives
    the same O, LSE and dQ, and the K/V gradients are the sums over each group."""
    x = gqa_inputs(B, Hq, Hkv, S, D, seed=40 + S)
    G = Hq // Hkv
    Kr, Vr = np.repeat(x["K"], G, axis=1), np.repeat(x["V"], G, axis=1)
    O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    dQ, dK, dV = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    Om, Lm = oracle.attn_fwd(x["Q"], Kr, Vr, x["scale"], causal)
    dQm, dKm, dVm = oracle.attn_bwd(x["Q"], Kr, Vr, x["dO"], x["scale"], causal)
    assert dK.shape == (B, Hkv, S, D) and dV.shape == (B, Hkv, S, D)
    np.testing.assert_allclose(O, Om, rtol=0, atol=1e-14)
    np.testing.assert_allclose(LSE, Lm, rtol=0, atol=1e-14)
    np.testing.assert_allclose(dQ, dQm, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dK, dKm.reshape(B, Hkv, G, S, D).sum(2), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dV, dVm.reshape(B, Hkv, G, S, D).sum(2), rtol=0, atol=1e-12)


@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal", GQA_CASES[:3])
def test_gqa_against_torch_fp64_autograd(B, Hq, Hkv, S, D, causal):
    """Independent library route: repeat_interleave of the K/V heads inside the autograd graph,
    so torch itself sums the group's gradients."""
    x = gqa_inputs(B, Hq, Hkv, S, D, seed=50 + S)
    G = Hq // Hkv
    t = {k: torch.tensor(f64(x[k]), dtype=torch.float64, requires_grad=(k != "dO"))
         for k in ("Q", "K", "V", "dO")}
    Kt, Vt = t["K"].repeat_interleave(G, dim=1), t["V"].repeat_interleave(G, dim=1)
    s = (t["Q"] @ Kt.transpose(-1, -2)) * float(np.float32(x["scale"]))
    if causal:
        s = s.masked_fill(~torch.ones(S, S, dtype=torch.bool).tril(), float("-inf"))
    o_t = torch.softmax(s, dim=-1) @ Vt
    gq, gk, gv = torch.autograd.grad(o_t, (t["Q"], t["K"], t["V"]), grad_outputs=t["dO"])
    O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    dQ, dK, dV = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    np.testing.assert_allclose(O, o_t.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE, torch.logsumexp(s, dim=-1).detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dQ, gq.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dK, gk.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dV, gv.numpy(), rtol=0, atol=1e-11)


def test_gqa_head_mapping_is_blocked_not_interleaved():
    """Query heads 0..G-1 read K/V head 0, G..2G-1 read head 1, ...: with V constant per K/V
    head, O of a query head equals the constant of head h // G (and not h % Hkv)."""
    B, Hq, Hkv, S, D = 1, 6, 3, 11, 8
    x = gqa_inputs(B, Hq, Hkv, S, D, seed=61)
    consts = np.array([1.0, -2.0, 0.5])
    V = bits(np.broadcast_to(consts[None, :, None, None], (B, Hkv, S, D)).copy())
    O, _ = oracle.attn_fwd(x["Q"], x["K"], V, x["scale"], False)
    for h in range(Hq):
        np.testing.assert_allclose(O[0, h], consts[h // (Hq // Hkv)], rtol=0, atol=1e-13)


def test_gqa_rejects_non_dividing_head_counts():
    x = gqa_inputs(1, 4, 3, 5, 8, seed=62)
    with pytest.raises(ValueError):
        oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], False)


# ---- rectangular attention: Sq query rows against Sk keys, causal mask aligned bottom-right --
# (decoding / chunked prefill against a longer key-value cache).  Row i sees keys 0..i+Sk-Sq.

def rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed):
    x = rnd(B, Hq, Sq, D, seed)
    kv = rnd(B, Hkv, Sk, D, seed + 2000)
    x["K"], x["V"] = kv["K"], kv["V"]
    return x


RECT_CASES = [(1, 2, 2, 1, 9, 8), (2, 2, 1, 3, 17, 16), (1, 4, 2, 5, 5, 8), (1, 1, 1, 7, 40, 16),
              (1, 2, 2, 33, 65, 64)]


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D", RECT_CASES)
def test_rect_causal_is_the_tail_of_square_causal(B, Hq, Hkv, Sq, Sk, D):
    """Reduction to the square case pinned above.  Put the Sq query rows at the END of a
    square problem of length Sk (any rows in front, here zeros, with zero upstream gradient):
    the tail of O, LSE and dQ is the rectangular result, and since the front rows carry no
    gradient, dK and dV are the rectangular ones as well."""
    x = rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=70 + Sq)
    Qs = np.zeros((B, Hq, Sk, D), np.uint16); Qs[:, :, Sk - Sq:] = x["Q"]
    Gs = np.zeros((B, Hq, Sk, D), np.uint16); Gs[:, :, Sk - Sq:] = x["dO"]
    O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], True)
    dQ, dK, dV = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], True)
    Os, Ls = oracle.attn_fwd(Qs, x["K"], x["V"], x["scale"], True)
    dQs, dKs, dVs = oracle.attn_bwd(Qs, x["K"], x["V"], Gs, x["scale"], True)
    assert O.shape == (B, Hq, Sq, D) and dK.shape == (B, Hkv, Sk, D)
    np.testing.assert_allclose(O, Os[:, :, Sk - Sq:], rtol=0, atol=1e-14)
    np.testing.assert_allclose(LSE, Ls[:, :, Sk - Sq:], rtol=0, atol=1e-14)
    np.testing.assert_allclose(dQ, dQs[:, :, Sk - Sq:], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dK, dKs, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dV, dVs, rtol=0, atol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D", RECT_CASES[:4] + [(1, 2, 1, 6, 3, 8)])
def test_rect_against_torch_fp64_autograd(B, Hq, Hkv, Sq, Sk, D, causal):
    """Independent library route with an explicit boolean mask key <= row + Sk - Sq."""
    if causal and Sk < Sq:
        pytest.skip("rows without keys: rejected, see test_rect_rejects_causal_with_fewer_keys")
    x = rect_inputs(B, Hq, Hkv, Sq, Sk, D, seed=80 + Sk)
    G = Hq // Hkv
    t = {k: torch.tensor(f64(x[k]), dtype=torch.float64, requires_grad=(k != "dO"))
         for k in ("Q", "K", "V", "dO")}
    Kt, Vt = t["K"].repeat_interleave(G, dim=1), t["V"].repeat_interleave(G, dim=1)
    s = (t["Q"] @ Kt.transpose(-1, -2)) * float(np.float32(x["scale"]))
    if causal:
        keep = torch.arange(Sk)[None, :] <= torch.arange(Sq)[:, None] + (Sk - Sq)
        s = s.masked_fill(~keep, float("-inf"))
    o_t = torch.softmax(s, dim=-1) @ Vt
    gq, gk, gv = torch.autograd.grad(o_t, (t["Q"], t["K"], t["V"]), grad_outputs=t["dO"])
    O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
    dQ, dK, dV = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], causal)
    np.testing.assert_allclose(O, o_t.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE, torch.logsumexp(s, dim=-1).detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dQ, gq.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dK, gk.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dV, gv.numpy(), rtol=0, atol=1e-11)


def test_rect_decode_row_closed_form_and_mask_shape():
    """One query row (decoding): causal and non-causal coincide (the last row sees every key),
    O is the softmax-weighted mean of V written out with numpy.  With Sq = 3, Sk = 5 the
    causal probability matrix has exactly the bottom-right staircase of zeros."""
    x = rect_inputs(1, 1, 1, 1, 13, 8, seed=91)
    q, K, V = f64(x["Q"])[0, 0, 0], f64(x["K"])[0, 0], f64(x["V"])[0, 0]
    s = (K @ q) * float(np.float32(x["scale"]))
    p = np.exp(s - s.max()); p /= p.sum()
    for causal in (False, True):
        O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], causal)
        np.testing.assert_allclose(O[0, 0, 0], p @ V, rtol=0, atol=1e-14)
        np.testing.assert_allclose(LSE[0, 0, 0], s.max() + np.log(np.exp(s - s.max()).sum()),
                                   rtol=0, atol=1e-13)
    y = rect_inputs(1, 1, 1, 3, 5, 8, seed=92)
    P = oracle.attn_probs(y["Q"], y["K"], y["V"], y["scale"], True)[0, 0]
    assert P.shape == (3, 5)
    assert ((P > 0) == np.array([[1, 1, 1, 0, 0], [1, 1, 1, 1, 0], [1, 1, 1, 1, 1]], bool)).all()
    np.testing.assert_allclose(P.sum(-1), 1.0, rtol=0, atol=1e-14)
    dS = oracle.attn_dscores(y["Q"], y["K"], y["V"], y["dO"], y["scale"], True)[0, 0]
    assert (dS[P == 0] == 0).all()
    np.testing.assert_allclose(dS.sum(-1), 0.0, rtol=0, atol=1e-13)


def test_rect_rejects_causal_with_fewer_keys():
    x = rect_inputs(1, 1, 1, 6, 3, 8, seed=93)
    oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], False)      # fine without the mask
    with pytest.raises(RuntimeError):
        oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], True)
    with pytest.raises(RuntimeError):
        oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], True)


# ---- fp16 inputs: only the widening of the inputs differs ---------------------------------------

def test_f16_widening_matches_numpy_for_every_bit_pattern():
    """The oracle's own half -> double conversion against numpy's float16 (an independent
    implementation), for all 65536 patterns: zeros, subnormals, normals, infinities, NaNs."""
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = h.view(np.float16).astype(np.float64)
    got = np.array([oracle.f16_to_f64(int(v)) for v in h])
    nan = np.isnan(want)
    assert (np.isnan(got) == nan).all()
    assert (got[~nan] == want[~nan]).all()
    assert (np.signbit(got[~nan]) == np.signbit(want[~nan])).all()


@pytest.mark.parametrize("causal", [False, True])
def test_f16_path_equals_bf16_path_on_values_both_formats_hold(causal):
    """Inputs with at most 8 significant bits and small exponents are exact in bf16 AND in
    fp16, so both readings must give the same result to the last bit; this ties the fp16 path
    to the bf16 one that everything above pins."""
    B, Hq, Hkv, Sq, Sk, D = 1, 4, 2, 9, 21, 16
    rng = np.random.Generator(np.random.PCG64(97))
    vals = {}
    for name, heads, rows in (("Q", Hq, Sq), ("K", Hkv, Sk), ("V", Hkv, Sk), ("dO", Hq, Sq)):
        vals[name] = (rng.integers(-127, 128, size=(B, heads, rows, D)) / 64.0).astype(np.float32)
    as_bf = {k: bits(v) for k, v in vals.items()}
    as_h = {k: wl.f32_to_f16_bits(v) for k, v in vals.items()}
    for k in vals:     # the premise: both encodings hold the values exactly
        assert (f64(as_bf[k]) == vals[k]).all() and (wl.f16_bits_to_f32(as_h[k]) == vals[k]).all()
    sc = wl.default_scale(D)
    a = oracle.attn_fwd(as_bf["Q"], as_bf["K"], as_bf["V"], sc, causal)
    b = oracle.attn_fwd(as_h["Q"], as_h["K"], as_h["V"], sc, causal, dtype="f16")
    ga = oracle.attn_bwd(as_bf["Q"], as_bf["K"], as_bf["V"], as_bf["dO"], sc, causal)
    gb = oracle.attn_bwd(as_h["Q"], as_h["K"], as_h["V"], as_h["dO"], sc, causal, dtype="f16")
    for x, y in zip(a + ga, b + gb):
        assert np.array_equal(x, y)


def test_f16_against_torch_fp64_on_fp16_inputs():
    """fp16 inputs that are NOT representable in bf16 (11 significant bits), against torch."""
    x = wl.random_rect_inputs_f16(1, 2, 1, 5, 12, 8, seed=98)
    assert (bits(wl.f16_bits_to_f32(x["Q"])) != 0).any()
    assert not np.array_equal(f64(bits(wl.f16_bits_to_f32(x["Q"]))),
                              wl.f16_bits_to_f32(x["Q"]).astype(np.float64))
    t = {k: torch.tensor(wl.f16_bits_to_f32(x[k]).astype(np.float64), requires_grad=(k != "dO"))
         for k in ("Q", "K", "V", "dO")}
    Kt, Vt = t["K"].repeat_interleave(2, dim=1), t["V"].repeat_interleave(2, dim=1)
    s = (t["Q"] @ Kt.transpose(-1, -2)) * float(np.float32(x["scale"]))
    o_t = torch.softmax(s, dim=-1) @ Vt
    gq, gk, gv = torch.autograd.grad(o_t, (t["Q"], t["K"], t["V"]), grad_outputs=t["dO"])
    O, LSE = oracle.attn_fwd(x["Q"], x["K"], x["V"], x["scale"], False, dtype="f16")
    dQ, dK, dV = oracle.attn_bwd(x["Q"], x["K"], x["V"], x["dO"], x["scale"], False, dtype="f16")
    np.testing.assert_allclose(O, o_t.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE, torch.logsumexp(s, dim=-1).detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dQ, gq.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dK, gk.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dV, gv.numpy(), rtol=0, atol=1e-11)
