"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and
argument validation returns the documented status codes without touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2601_16238_amd as attn
from paper_2601_16238_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "attn.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(attn_\w+)\s*\(", src)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_functions()
    assert "attn_fwd" in names and "attn_bwd" in names and "attn_bwd_workspace_bytes" in names
    L = attn.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert sorted(binding.EXPORTS) == names


def test_version_and_status_strings():
    assert attn.attn_version() == 1005
    seen = set()
    for code in range(0, -8, -1):
        s = attn.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert attn.status_string(-99) == "unknown status"


def test_params_contiguous_and_workspace_size():
    p = attn.make_params(4, 32, 4096, 128, 0.0883, True)
    assert (p.stride_s, p.stride_h, p.stride_b) == (128, 4096 * 128, 32 * 4096 * 128)
    assert attn.attn_bwd_workspace_bytes(4, 32, 4096, 128) == 2 * 4 * 32 * 4096 * 4
    assert attn.attn_bwd_workspace_bytes(1, 1, 1, 64) == 256          # rounded up
    assert attn.attn_bwd_workspace_bytes(1, 1, 1, 100) == 0           # invalid D


FAKE = 0x1000  # a non-NULL, 16-byte aligned address; never dereferenced on the host


def call_fwd(p, Q=FAKE, K=FAKE, V=FAKE, O=FAKE, LSE=FAKE):
    return attn.lib().attn_fwd(Q, K, V, O, LSE, ctypes.byref(p) if p is not None else None, None)


def call_bwd(p, ws=FAKE, ws_bytes=1 << 40, ptr=FAKE, stages=None):
    args = [ptr] * 9 + [ws, ws_bytes, ctypes.byref(p), None]
    if stages is None:
        return attn.lib().attn_bwd(*args)
    return attn.lib().attn_bwd_stages(*args, stages)


@pytest.mark.parametrize("mutate,code", [
    (lambda p: setattr(p, "B", 0), binding.ATTN_ERR_SHAPE),
    (lambda p: setattr(p, "S", 0), binding.ATTN_ERR_SHAPE),
    (lambda p: setattr(p, "D", 100), binding.ATTN_ERR_SHAPE),
    (lambda p: setattr(p, "stride_s", 60), binding.ATTN_ERR_STRIDE),
    (lambda p: setattr(p, "stride_h", 132), binding.ATTN_ERR_STRIDE),
    (lambda p: setattr(p, "scale", 0.0), binding.ATTN_ERR_SCALE),
    (lambda p: setattr(p, "scale", -1.0), binding.ATTN_ERR_SCALE),
    (lambda p: setattr(p, "scale", float("nan")), binding.ATTN_ERR_SCALE),
    (lambda p: setattr(p, "scale", float("inf")), binding.ATTN_ERR_SCALE),
])
def test_bad_params_rejected_before_any_launch(mutate, code):
    p = attn.make_params(1, 2, 128, 64, 0.125, False)
    mutate(p)
    assert call_fwd(p) == code
    assert call_bwd(p) == code


def test_null_alignment_and_workspace_errors():
    p = attn.make_params(1, 2, 128, 64, 0.125, False)
    assert call_fwd(p, Q=None) == binding.ATTN_ERR_NULL
    assert call_fwd(p, LSE=None) == binding.ATTN_ERR_NULL
    assert call_fwd(None) == binding.ATTN_ERR_NULL
    assert call_fwd(p, K=FAKE + 8) == binding.ATTN_ERR_ALIGN
    assert call_fwd(p, LSE=FAKE + 2) == binding.ATTN_ERR_ALIGN
    assert call_bwd(p, ptr=None) == binding.ATTN_ERR_NULL
    assert call_bwd(p, ptr=FAKE + 2) == binding.ATTN_ERR_ALIGN
    assert call_bwd(p, ws=None) == binding.ATTN_ERR_WORKSPACE
    assert call_bwd(p, ws=FAKE + 16) == binding.ATTN_ERR_WORKSPACE
    assert call_bwd(p, ws_bytes=1023) == binding.ATTN_ERR_WORKSPACE
    assert call_bwd(p, stages=0) == binding.ATTN_ERR_SHAPE
    assert call_bwd(p, stages=8) == binding.ATTN_ERR_SHAPE


def test_row_count_overflow_is_a_shape_error():
    p = attn.make_params(1 << 15, 1 << 10, 1 << 10, 64, 0.125, False)
    assert call_fwd(p) == binding.ATTN_ERR_SHAPE


def test_workloads_are_seeded_and_shaped():
    from paper_2601_16238_amd import workloads as wl
    import numpy as np
    a = wl.make_inputs("tiny")
    b = wl.make_inputs("tiny")
    assert a["Q"].shape == (1, 2, 128, 64) and a["Q"].dtype == np.uint16
    for k in ("Q", "K", "V", "dO"):
        assert np.array_equal(a[k], b[k])
    sub = wl.make_inputs("vit_cifar", heads=[0, 5, 767])
    full = wl.make_inputs("vit_cifar")
    assert sub["K"].shape == (1, 3, 65, 64)
    assert np.array_equal(sub["K"][0, 1], full["K"].reshape(768, 65, 64)[5])
    x = wl.bf16_bits_to_f32(wl.make_inputs("minigpt")["V"])
    assert abs(float(x.std()) - 0.5) < 0.01
    # bf16 rounding: nearest-even on the 16 dropped bits
    f = np.array([1.0, 1.00390625, 1.01171875, -3.0e38], np.float32)
    assert list(wl.f32_to_bf16_bits(f)) == [0x3F80, 0x3F80, 0x3F82, 0xFF62]


# ---- grouped-query entry points ----------------------------------------------------------

def call_fwd_gqa(p, ptr=FAKE):
    return attn.lib().attn_fwd_gqa(ptr, ptr, ptr, ptr, ptr, ctypes.byref(p), None)


def call_bwd_gqa(p, ws=FAKE, ws_bytes=1 << 40, stages=None):
    args = [FAKE] * 9 + [ws, ws_bytes, ctypes.byref(p), None]
    if stages is None:
        return attn.lib().attn_bwd_gqa(*args)
    return attn.lib().attn_bwd_gqa_stages(*args, stages)


def test_gqa_params_contiguous_and_workspace_size():
    p = attn.make_gqa_params(4, 32, 8, 4096, 128, 0.0883, True)
    assert (p.q_stride_s, p.q_stride_h, p.q_stride_b) == (128, 4096 * 128, 32 * 4096 * 128)
    assert (p.kv_stride_s, p.kv_stride_h, p.kv_stride_b) == (128, 4096 * 128, 8 * 4096 * 128)
    # the workspace is per QUERY row
    assert attn.attn_bwd_gqa_workspace_bytes(4, 32, 8, 4096, 128) == 2 * 4 * 32 * 4096 * 4
    assert attn.attn_bwd_gqa_workspace_bytes(1, 6, 4, 16, 64) == 0     # 4 does not divide 6


@pytest.mark.parametrize("mutate,code", [
    (lambda p: setattr(p, "Hkv", 3), binding.ATTN_ERR_SHAPE),           # 3 does not divide 8
    (lambda p: setattr(p, "Hkv", 0), binding.ATTN_ERR_SHAPE),
    (lambda p: setattr(p, "Hkv", 16), binding.ATTN_ERR_SHAPE),          # more K/V than query heads
    (lambda p: setattr(p, "D", 264), binding.ATTN_ERR_SHAPE),           # above the widest kernel
    (lambda p: setattr(p, "kv_stride_s", 60), binding.ATTN_ERR_STRIDE),
    (lambda p: setattr(p, "kv_stride_h", 132), binding.ATTN_ERR_STRIDE),
    (lambda p: setattr(p, "q_stride_b", 4), binding.ATTN_ERR_STRIDE),
    (lambda p: setattr(p, "kv_stride_s", 1 << 24), binding.ATTN_ERR_STRIDE),  # 32-bit row offsets
    (lambda p: setattr(p, "scale", 0.0), binding.ATTN_ERR_SCALE),
])
def test_gqa_bad_params_rejected_before_any_launch(mutate, code):
    p = attn.make_gqa_params(1, 8, 2, 128, 64, 0.125, False)
    mutate(p)
    assert call_fwd_gqa(p) == code
    assert call_bwd_gqa(p) == code


def test_gqa_null_workspace_and_stage_errors():
    p = attn.make_gqa_params(1, 8, 2, 128, 64, 0.125, False)
    assert call_fwd_gqa(p, ptr=None) == binding.ATTN_ERR_NULL
    assert call_fwd_gqa(p, ptr=FAKE + 8) == binding.ATTN_ERR_ALIGN
    assert call_bwd_gqa(p, ws=None) == binding.ATTN_ERR_WORKSPACE
    assert call_bwd_gqa(p, ws_bytes=8 * 128 * 8 - 1) == binding.ATTN_ERR_WORKSPACE
    assert call_bwd_gqa(p, stages=0) == binding.ATTN_ERR_SHAPE
    assert call_bwd_gqa(p, stages=16) == binding.ATTN_ERR_SHAPE


def test_gqa_workloads_are_seeded_and_group_selection_matches():
    from paper_2601_16238_amd import workloads as wl
    import numpy as np
    w = wl.GQA_WORKLOADS["mqa_small"]
    a, b = wl.make_gqa_inputs(w), wl.make_gqa_inputs(w)
    assert a["Q"].shape == (w.B, w.Hq, w.S, w.D) and a["K"].shape == (w.B, w.Hkv, w.S, w.D)
    for k in ("Q", "K", "V", "dO"):
        assert np.array_equal(a[k], b[k])
    sub = wl.make_gqa_inputs(w, kv_heads=[1])            # batch 1's only K/V head and its group
    assert sub["Q"].shape == (1, w.Hq, w.S, w.D) and sub["K"].shape == (1, 1, w.S, w.D)
    assert np.array_equal(sub["K"][0, 0], a["K"][1, 0])
    assert np.array_equal(sub["Q"][0], a["Q"][1])


# ---- rectangular entry points ----------------------------------------------------------------

def call_fwd_rect(p, ptr=FAKE, ws=None, ws_bytes=0):
    return attn.lib().attn_fwd_rect(ptr, ptr, ptr, ptr, ptr, ws, ws_bytes, ctypes.byref(p), None)


def call_bwd_rect(p, ws=FAKE, ws_bytes=1 << 40):
    return attn.lib().attn_bwd_rect(*([FAKE] * 9 + [ws, ws_bytes, ctypes.byref(p), None]))


def test_rect_params_contiguous_and_workspace_sizes():
    p = attn.make_rect_params(2, 8, 2, 5, 300, 64, 0.125, True)
    assert (p.q_stride_s, p.q_stride_h, p.q_stride_b) == (64, 5 * 64, 8 * 5 * 64)
    assert (p.kv_stride_s, p.kv_stride_h, p.kv_stride_b) == (64, 300 * 64, 2 * 300 * 64)
    # backward: two fp32 per QUERY row, rounded up to 256 bytes
    assert attn.attn_bwd_rect_workspace_bytes(2, 8, 2, 5, 300, 64) == 768
    assert attn.attn_bwd_rect_workspace_bytes(4, 32, 8, 4096, 4096, 128) == \
        attn.attn_bwd_gqa_workspace_bytes(4, 32, 8, 4096, 128)
    # forward: nothing to split when the launch fills the chip or the keys are few ...
    assert attn.attn_fwd_rect_workspace_bytes(4, 32, 8, 4096, 4096, 128) == 0
    assert attn.attn_fwd_rect_workspace_bytes(2, 8, 2, 1, 300, 64) == 0
    # ... otherwise (D+1) fp32 per split and query row; decoding 8 sequences of 32 heads
    # against 8192 keys: the 4 query heads of a group are packed into one head of 4 rows (64
    # work-groups), which splits 8 ways: two work-groups per compute unit, 16 tiles each
    assert attn.attn_fwd_rect_workspace_bytes(8, 32, 8, 1, 8192, 128) == 8 * 256 * 129 * 4
    # a sixteenth of the keys: 2 ways with one work-group per compute unit would leave 4 tiles per
    # split, which is the floor (no finer split for a second work-group per unit)
    assert attn.attn_fwd_rect_workspace_bytes(8, 32, 8, 1, 512, 128) == 2 * 256 * 129 * 4
    assert attn.attn_fwd_rect_workspace_bytes(1, 6, 4, 1, 8192, 64) == 0      # invalid heads


@pytest.mark.parametrize("mutate,code", [
    (lambda p: setattr(p, "Sq", 0), binding.ATTN_ERR_SHAPE),
    (lambda p: setattr(p, "Sk", 0), binding.ATTN_ERR_SHAPE),
    (lambda p: (setattr(p, "Sk", 8), setattr(p, "causal", 1)), binding.ATTN_ERR_SHAPE),  # Sk < Sq
    (lambda p: setattr(p, "Hkv", 3), binding.ATTN_ERR_SHAPE),
    (lambda p: setattr(p, "D", 100), binding.ATTN_ERR_SHAPE),
    (lambda p: setattr(p, "kv_stride_s", 60), binding.ATTN_ERR_STRIDE),
    (lambda p: setattr(p, "q_stride_h", 4), binding.ATTN_ERR_STRIDE),
    (lambda p: setattr(p, "scale", float("nan")), binding.ATTN_ERR_SCALE),
])
def test_rect_bad_params_rejected_before_any_launch(mutate, code):
    p = attn.make_rect_params(1, 8, 2, 16, 128, 64, 0.125, False)
    mutate(p)
    assert call_fwd_rect(p) == code
    assert call_bwd_rect(p) == code


def test_rect_fewer_keys_than_rows_is_fine_without_a_mask():
    p = attn.make_rect_params(1, 8, 2, 16, 8, 64, 0.125, False)
    assert call_fwd_rect(p, ptr=None) == binding.ATTN_ERR_NULL     # got past the shape check
    p.causal = 1
    assert call_fwd_rect(p, ptr=None) == binding.ATTN_ERR_NULL     # NULL is checked first
    assert call_fwd_rect(p) == binding.ATTN_ERR_SHAPE


def test_rect_workspace_errors():
    p = attn.make_rect_params(8, 32, 8, 1, 8192, 128, 0.0883, True)   # the plan splits
    need = 4 * 256 * 129 * 4
    assert call_fwd_rect(p, ws=FAKE + 16, ws_bytes=need) == binding.ATTN_ERR_WORKSPACE
    assert call_fwd_rect(p, ws=FAKE, ws_bytes=need - 1) == binding.ATTN_ERR_WORKSPACE
    assert call_fwd_rect(p, ptr=FAKE + 8, ws=FAKE, ws_bytes=need) == binding.ATTN_ERR_ALIGN
    assert call_bwd_rect(p, ws=None) == binding.ATTN_ERR_WORKSPACE
    assert call_bwd_rect(p, ws_bytes=8 * 32 * 8 - 1) == binding.ATTN_ERR_WORKSPACE


def test_rect_workloads_are_seeded_and_group_selection_matches():
    from paper_2601_16238_amd import workloads as wl
    import numpy as np
    w = wl.RECT_WORKLOADS["decode_small"]
    a, b = wl.make_rect_inputs(w), wl.make_rect_inputs(w)
    assert a["Q"].shape == (w.B, w.Hq, w.Sq, w.D) and a["K"].shape == (w.B, w.Hkv, w.Sk, w.D)
    for k in ("Q", "K", "V", "dO"):
        assert np.array_equal(a[k], b[k])
    sub = wl.make_rect_inputs(w, kv_heads=[3])            # batch 1, K/V head 1 and its group
    G = w.Hq // w.Hkv
    assert sub["Q"].shape == (1, G, w.Sq, w.D) and sub["K"].shape == (1, 1, w.Sk, w.D)
    assert np.array_equal(sub["K"][0, 0], a["K"][1, 1])
    assert np.array_equal(sub["dO"][0], a["dO"][1, G:2 * G])


def test_f16_entry_points_validate_like_the_bf16_ones():
    p = attn.make_rect_params(1, 8, 2, 16, 128, 64, 0.125, True)
    L = attn.lib()
    assert L.attn_fwd_rect_f16(FAKE, FAKE, FAKE, FAKE, None, None, 0, ctypes.byref(p), None) == \
        binding.ATTN_ERR_NULL
    assert L.attn_fwd_rect_f16(FAKE, FAKE + 2, FAKE, FAKE, FAKE, None, 0, ctypes.byref(p), None) == \
        binding.ATTN_ERR_ALIGN
    assert L.attn_bwd_rect_f16(*([FAKE] * 9 + [None, 0, ctypes.byref(p), None])) == \
        binding.ATTN_ERR_WORKSPACE
    p.D = 100
    assert L.attn_fwd_rect_f16(FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, ctypes.byref(p), None) == \
        binding.ATTN_ERR_SHAPE


def test_stream_probe_validates_its_arguments():
    L = attn.lib()
    MB = 1 << 20
    assert L.attn_probe_stream(None, 8 * MB, 64, 0, FAKE, None) == binding.ATTN_ERR_NULL
    assert L.attn_probe_stream(FAKE, 8 * MB, 64, 0, None, None) == binding.ATTN_ERR_NULL
    assert L.attn_probe_stream(FAKE, 8 * MB, 0, 0, FAKE, None) == binding.ATTN_ERR_SHAPE
    assert L.attn_probe_stream(FAKE, 8 * MB + 4096, 64, 1, FAKE, None) == binding.ATTN_ERR_SHAPE   # not whole 32 KB steps
    assert L.attn_probe_stream(FAKE, 0, 64, 1, FAKE, None) == binding.ATTN_ERR_SHAPE
    assert L.attn_probe_stream(FAKE + 8, 8 * MB, 64, 0, FAKE, None) == binding.ATTN_ERR_ALIGN
    assert L.attn_probe_stream(FAKE, 8 * MB, 64, 1, FAKE + 2, None) == binding.ATTN_ERR_ALIGN


def test_mfma_probe_validates_its_arguments():
    L = attn.lib()
    assert L.attn_probe_mfma_bf16(4, 10, 0, None, 4 * 512, None, None) == binding.ATTN_ERR_NULL
    assert L.attn_probe_mfma_bf16(0, 10, 0, FAKE, 4 * 512, None, None) == binding.ATTN_ERR_SHAPE
    assert L.attn_probe_mfma_bf16(4, 0, 1, FAKE, 4 * 512, None, None) == binding.ATTN_ERR_SHAPE
    assert L.attn_probe_mfma_bf16(4, 10, 1, FAKE, 4 * 512 - 1, None, None) == binding.ATTN_ERR_WORKSPACE
    assert L.attn_probe_mfma_bf16(4, 10, 0, FAKE + 2, 4 * 512, None, None) == binding.ATTN_ERR_ALIGN


# ---- row-wise entry points (include/rowops.h) ---------------------------------------------------

def test_every_rowops_symbol_is_exported_and_bound():
    from paper_2601_16238_amd import rowops
    src = open(os.path.join(ROOT, "include", "rowops.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = sorted(set(re.findall(r"\b(rowops_\w+)\s*\(", src)))
    assert len(names) == 5 and sorted(rowops.EXPORTS) == names
    for n in names:
        assert getattr(attn.lib(), n) is not None


def test_rowops_validation_without_a_gpu():
    from paper_2601_16238_amd import rowops
    L = rowops._lib()
    ok_args = dict(rows=16, cols=256, xs=256, ys=256)
    call = lambda x=FAKE, w=FAKE, y=FAKE, rows=16, cols=256, xs=256, ys=256: \
        L.rowops_rmsnorm_fwd(x, w, y, rows, cols, xs, ys, 1e-6, None)
    assert call(x=None) == binding.ATTN_ERR_NULL
    assert call(cols=12) == binding.ATTN_ERR_SHAPE            # not a multiple of 8
    assert call(cols=16392, xs=16392, ys=16392) == binding.ATTN_ERR_SHAPE   # above the row budget
    assert call(rows=0) == binding.ATTN_ERR_SHAPE
    assert call(xs=128) == binding.ATTN_ERR_STRIDE            # row stride below cols
    assert call(ys=260) == binding.ATTN_ERR_STRIDE            # not a multiple of 8
    assert call(w=FAKE + 4) == binding.ATTN_ERR_ALIGN
    # one pair of fp32 rows per work-group; above 512 rows: 256 two-team groups, 512 at <= 2048 columns,
    # 256 one-team groups at 16384 columns; never more groups than rows
    assert rowops.layernorm_bwd_workspace_bytes(4096, 8192) == 256 * 2 * 8192 * 4
    assert rowops.layernorm_bwd_workspace_bytes(400, 8192) == 400 * 2 * 8192 * 4
    assert rowops.layernorm_bwd_workspace_bytes(4096, 2048) == 512 * 2 * 2048 * 4
    assert rowops.layernorm_bwd_workspace_bytes(4096, 4096) == 256 * 2 * 4096 * 4
    assert rowops.layernorm_bwd_workspace_bytes(4096, 16384) == 256 * 2 * 16384 * 4
    assert rowops.layernorm_bwd_workspace_bytes(3, 64) == 3 * 2 * 64 * 4
    assert rowops.layernorm_bwd_workspace_bytes(3, 60) == 0
    bwd = lambda ws=FAKE, nbytes=1 << 30: L.rowops_layernorm_bwd(
        FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ws, nbytes, 16, 256, 256, 256, 256, None)
    assert bwd(ws=None) == binding.ATTN_ERR_WORKSPACE
    assert bwd(nbytes=16 * 2 * 256 * 4 - 1) == binding.ATTN_ERR_WORKSPACE
    rot = lambda D=128, ss=128: L.rowops_rotary_fwd(FAKE, FAKE, FAKE, FAKE, 2, 4, 64, D,
                                                   4 * 64 * 128, 64 * 128, ss, 4 * 64 * 128, 64 * 128, 128, None)
    assert rot(D=24) == binding.ATTN_ERR_SHAPE                # halves must be multiples of 8
    assert rot(ss=64) == binding.ATTN_ERR_STRIDE
