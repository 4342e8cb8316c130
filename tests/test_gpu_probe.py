"""The MFMA-only measurement kernel really executes the work its flop count claims: with
operands that are small integers times 2^-10 every product and partial sum is exact in fp32,
so the grand total of a wave's accumulators has a closed form."""
import numpy as np
import pytest
import torch

import paper_2601_16238_amd as attn

pytestmark = pytest.mark.gpu


def test_probe_total_matches_the_closed_form_and_the_flop_count():
    wgs, iters = 3, 5
    sink = torch.full((wgs * 512,), -1.0, dtype=torch.float32, device="cuda")
    flop = attn.attn_probe_mfma_bf16(wgs, iters, sink)
    torch.cuda.synchronize()
    assert flop == wgs * 8 * iters * 16 * 32768.0
    got = sink.cpu().numpy().astype(np.float64).reshape(wgs * 8, 64)
    # operand layout of the 32x32x16 MFMA: lane l holds A[l % 32][8 * (l // 32) + i] and
    # B[8 * (l // 32) + i][l % 32], i = 0..7
    lanes = np.arange(64)
    A = np.zeros((32, 16)); B = np.zeros((16, 32))
    for i in range(8):
        A[lanes % 32, 8 * (lanes // 32) + i] = (1 + ((lanes + i) & 15)) / 1024.0
        B[8 * (lanes // 32) + i, lanes % 32] = (1 + ((lanes * 3 + i) & 15)) / 1024.0
    total = (A @ B).sum() * iters * 16        # 16 MFMAs per iteration, all accumulated
    np.testing.assert_allclose(got.sum(axis=1), total, rtol=1e-6)
    assert np.array_equal(got[0], got[-1])    # every wave does the same work


def test_probe_with_random_operands_matches_numpy():
    wgs, iters = 2, 3
    sink = torch.empty(wgs * 512, dtype=torch.float32, device="cuda")
    flop = attn.attn_probe_mfma_bf16(wgs, iters, sink, random_operands=True)
    torch.cuda.synchronize()
    assert flop == wgs * 8 * iters * 16 * 32768.0
    got = sink.cpu().numpy().astype(np.float64).reshape(wgs * 8, 64)
    lanes = np.arange(64, dtype=np.uint64)
    A = np.zeros((4, 32, 16)); B = np.zeros((4, 16, 32))
    M = np.uint64(0xFFFFFFFF)
    for s in range(4):
        for i in range(8):
            x = ((lanes * np.uint64(64) + np.uint64(s * 8 + i)) * np.uint64(2654435761)) & M
            x ^= x >> np.uint64(15); x = (x * np.uint64(2246822519)) & M; x ^= x >> np.uint64(13)
            ua = (0x3F000000 | ((x & np.uint64(0x7F)) << np.uint64(16)) | ((x & np.uint64(0x80)) << np.uint64(24))) & M
            ub = (0x3F000000 | ((x & np.uint64(0x7F00)) << np.uint64(8)) | ((x & np.uint64(0x8000)) << np.uint64(16))) & M
            fa = ua.astype(np.uint32).view(np.float32).astype(np.float64)
            fb = ub.astype(np.uint32).view(np.float32).astype(np.float64)
            assert np.all((np.abs(fa) >= 0.5) & (np.abs(fa) < 1.0))
            li = lanes.astype(np.int64)
            A[s, li % 32, 8 * (li // 32) + i] = fa
            B[s, 8 * (li // 32) + i, li % 32] = fb
    total = iters * sum((A[(s + j) & 3] @ B[s]).sum() for s in range(4) for j in range(4))
    np.testing.assert_allclose(got.sum(axis=1), total, rtol=0, atol=2e-3)
    assert np.array_equal(got[0], got[-1])


def test_probe_rejects_a_small_sink():
    sink = torch.empty(511, dtype=torch.float32, device="cuda")
    with pytest.raises(attn.AttnError):
        attn.attn_probe_mfma_bf16(1, 1, sink)


def test_atomic_probe_adds_what_it_counts_and_reports_its_rate():
    """Every element of the accumulator must hold the number of key blocks that see its row's
    slot, and the byte count must equal the sum of those tiles; the rate is printed (it is the
    measurement behind the choice of a two-kernel backward without atomics)."""
    BH, S = 16, 16384
    acc = torch.zeros(BH * S * 128, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for key_block, causal in ((128, True), (192, True), (256, True), (192, False)):
        acc.zero_()
        torch.cuda.synchronize()
        e0.record()
        nbytes = attn.attn_probe_atomic_f32(BH, S, key_block, causal, acc)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        nkb = (S + key_block - 1) // key_block
        slot = np.arange(S // 32)
        first = (np.arange(nkb) * key_block) // 32 if causal else np.zeros(nkb, dtype=np.int64)
        expect = (first[None, :] <= slot[:, None]).sum(axis=1)          # per slot
        assert nbytes == float(expect.sum()) * BH * 32 * 128 * 4
        got = acc.view(BH, S // 32, 32 * 128)
        ref = torch.from_numpy(expect.astype(np.float32)).cuda()[None, :, None]
        assert torch.equal(got, ref.expand_as(got))
        print("atomic adds, %d heads x %d rows, key blocks of %d, causal=%s: %.2f GB in %.3f ms = %.2f TB/s"
              % (BH, S, key_block, causal, nbytes / 1e9, ms, nbytes / ms / 1e9), flush=True)


def test_atomic_probe_rejects_bad_shapes():
    acc = torch.zeros(8 * 64 * 128, dtype=torch.float32, device="cuda")
    for args in ((7, 64, 32), (8, 65, 32), (8, 64, 48), (8, 64, 128), (16, 64, 32)):
        with pytest.raises(attn.AttnError):
            attn.attn_probe_atomic_f32(*args, False, acc)


def test_stream_probe_reads_every_byte_and_reports_its_rate():
    """The per-work-group XOR of both forms must equal the XOR of the words of the work-group's
    share (so every byte was read, none twice); the rates over 256 MiB and 512 MiB are printed
    (they are the ceiling the decoding forward is compared with)."""
    print("case stream_probe checksum", flush=True)
    words = torch.randint(-2**31, 2**31 - 1, (8 << 18,), dtype=torch.int32, device="cuda")   # 8 MiB
    host = words.cpu().numpy().view(np.uint32)
    for wgs in (64, 256):
        per = host.size // wgs
        out = torch.empty(wgs, dtype=torch.int32, device="cuda")
        for nt in (False, True):
            out.fill_(0)
            attn.attn_probe_stream(words, wgs, out, direct=False, nontemporal=nt)
            torch.cuda.synchronize()
            expect = np.bitwise_xor.reduce(host.reshape(wgs, per), axis=1)
            assert np.array_equal(out.cpu().numpy().view(np.uint32), expect)
            out.fill_(0)
            attn.attn_probe_stream(words, wgs, out, direct=True, nontemporal=nt)
            torch.cuda.synchronize()
            halves = host.reshape(2, wgs, per // 2)
            expect = np.bitwise_xor.reduce(halves[0], axis=1) ^ np.bitwise_xor.reduce(halves[1], axis=1)
            assert np.array_equal(out.cpu().numpy().view(np.uint32), expect)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for mib in (256, 512):
        print("case stream_probe rate", mib, flush=True)
        buf = torch.ones(mib << 18, dtype=torch.int32, device="cuda")
        out = torch.empty(512, dtype=torch.int32, device="cuda")
        for direct, nt in ((False, False), (False, True), (True, False), (True, True)):
            for _ in range(3):
                attn.attn_probe_stream(buf, 512, out, direct=direct, nontemporal=nt)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(10):
                nbytes = attn.attn_probe_stream(buf, 512, out, direct=direct, nontemporal=nt)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 10
            assert nbytes == mib << 20 and nbytes / ms / 1e9 > 1.0       # TB/s; a sanity floor only
            print("read-only streaming, %d MiB, 512 work-groups, %s%s: %.1f us = %.2f TB/s"
                  % (mib, "direct transfers to LDS" if direct else "plain loads",
                     ", non-temporal" if nt else "", ms * 1e3, nbytes / ms / 1e9), flush=True)
        del buf
