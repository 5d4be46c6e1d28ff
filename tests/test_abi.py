"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

from paper_2503_18893_amd import binding as xb
from paper_2503_18893_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_entry_points():
    text = open(os.path.join(ROOT, "include", "xkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"XKV_API[^;(]*?\b(xkv_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_calls():
    names = declared_entry_points()
    for must in ("xkv_sr_decode", "xkv_sr_decode_tail", "xkv_dense_decode", "xkv_score", "xkv_topk", "xkv_gather_attend",
                 "xkv_workspace_bytes", "xkv_reconstruct", "xkv_factorize", "xkv_factorize_workspace_bytes"):
        assert must in names
    assert sorted(xb.ENTRY_POINTS) == names      # the binding wraps exactly what the header declares


def test_library_exports_every_declared_symbol():
    lib = xb.load()
    for name in declared_entry_points():
        assert getattr(lib, name) is not None, name


def test_status_strings_and_version():
    assert xb.status_string(0) == "XKV_OK"
    assert xb.status_string(-1) == "XKV_ERR_INVALID_ARG"
    assert xb.status_string(-2) == "XKV_ERR_UNSUPPORTED"
    assert xb.status_string(-3) == "XKV_ERR_WORKSPACE"
    assert xb.status_string(-4) == "XKV_ERR_HIP"
    assert xb.xkv_version() >= 100


def test_workspace_query_and_shape_validation():
    good = xb.Shape.of(synth.LLAMA_GROUP)
    assert xb.xkv_workspace_bytes(good) > 0
    bad = [dict(k=0), dict(k=good.L + 1), dict(H_q=30), dict(L=0), dict(r_k=0), dict(batch=-1), dict(scale=-1.0),
           dict(scale=float("nan")), dict(dtype_code=7), dict(G=0)]
    for kw in bad:
        c = good.c()
        for name, val in kw.items():
            setattr(c, "dtype" if name == "dtype_code" else name, val)
        n = ctypes.c_size_t(0)
        st = xb.load().xkv_workspace_bytes(ctypes.byref(c), ctypes.byref(n))
        assert st == xb.XKV_ERR_INVALID_ARG, kw
    for kw in (dict(d_h=512), dict(H_q=8 * 32)):       # shapes no kernel handles
        c = good.c()
        for name, val in kw.items():
            setattr(c, name, val)
        n = ctypes.c_size_t(0)
        assert xb.load().xkv_workspace_bytes(ctypes.byref(c), ctypes.byref(n)) == xb.XKV_ERR_UNSUPPORTED, kw
    assert xb.load().xkv_workspace_bytes(None, ctypes.byref(ctypes.c_size_t(0))) == xb.XKV_ERR_INVALID_ARG
    assert xb.load().xkv_workspace_bytes(ctypes.byref(good.c()), None) == xb.XKV_ERR_INVALID_ARG


def test_calls_reject_null_pointers_before_touching_the_gpu():
    lib = xb.load()
    c = xb.Shape.of(synth.TINY).c()
    null = ctypes.c_void_p(0)
    assert lib.xkv_topk(ctypes.byref(c), null, null, null, 0, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_sr_decode(ctypes.byref(c), 0, null, null, null, null, null, null, null, null, null, 0,
                             null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_reconstruct(ctypes.byref(c), 0, null, null, 4, null, null) == xb.XKV_ERR_INVALID_ARG
    one = ctypes.c_void_p(256)  # never dereferenced: the calls below fail on the host
    assert lib.xkv_sr_decode_tail(ctypes.byref(c), 0, one, one, one, one, one, null, null, -1, one, null, null, one,
                                  1 << 30, null) == xb.XKV_ERR_INVALID_ARG      # negative tail length
    assert lib.xkv_sr_decode_tail(ctypes.byref(c), 0, one, one, one, one, one, null, one, 5, one, null, null, one,
                                  1 << 30, null) == xb.XKV_ERR_INVALID_ARG      # tail tokens without their keys


def test_factorize_validates_on_the_host():
    lib = xb.load()
    good = xb.Shape.of(synth.LLAMA_GROUP)
    c, null, one = good.c(), ctypes.c_void_p(0), ctypes.c_void_p(256)
    assert xb.xkv_factorize_workspace_bytes(good, 512) > good.L * good.G * good.H_kv * good.d_h * 2   # holds a copy of X
    n = ctypes.c_size_t(0)
    assert lib.xkv_factorize(ctypes.byref(c), null, 512, 8, 0, one, one, one, 1 << 40, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_factorize(ctypes.byref(c), one, 512, 0, 0, one, one, one, 1 << 40, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_factorize(ctypes.byref(c), one, 0, 8, 0, one, one, one, 1 << 40, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_factorize(ctypes.byref(c), one, 2048, 8, 0, one, one, one, 1 << 40, null) == xb.XKV_ERR_UNSUPPORTED
    assert lib.xkv_factorize(ctypes.byref(c), one, 512, 8, 0, one, one, one, 1024, null) == xb.XKV_ERR_WORKSPACE
    assert lib.xkv_factorize_workspace_bytes(ctypes.byref(c), 2048, ctypes.byref(n)) == xb.XKV_ERR_UNSUPPORTED
    c96 = xb.Shape(G=2, H_kv=2, H_q=2, d_h=96, r_k=8, r_v=8, L=100, k=1, batch=1).c()
    assert lib.xkv_factorize_workspace_bytes(ctypes.byref(c96), 8, ctypes.byref(n)) == xb.XKV_ERR_UNSUPPORTED


def test_landmark_calls_validate_on_the_host():
    lib = xb.load()
    good = xb.Shape.of(synth.LLAMA_GROUP)
    c, null, one = good.c(), ctypes.c_void_p(0), ctypes.c_void_p(256)
    n = ctypes.c_size_t(0)
    assert xb.xkv_landmark_workspace_bytes(good, 8, 4) > xb.xkv_workspace_bytes(good)
    assert lib.xkv_landmark_workspace_bytes(ctypes.byref(c), 0, 0, ctypes.byref(n)) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_landmark_workspace_bytes(ctypes.byref(c), 8, -1, ctypes.byref(n)) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_landmark_workspace_bytes(ctypes.byref(c), 8, good.L, ctypes.byref(n)) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_landmarks(ctypes.byref(c), null, 8, 0, one, null, null, null, 0, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_landmarks(ctypes.byref(c), one, 8, 2, one, null, null, one, 1 << 40, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_landmarks(ctypes.byref(c), one, 8, 2, one, null, one, one, 16, null) == xb.XKV_ERR_WORKSPACE
    args = [ctypes.byref(c), 0, one, one, one, one, one, one, null, 8, 0, ctypes.c_float(0.0), null, null, 0, one, null, null,
            null, one]
    assert lib.xkv_sr_decode_landmark(*args, 16, null) == xb.XKV_ERR_WORKSPACE
    args[7] = null                                            # no landmarks
    assert lib.xkv_sr_decode_landmark(*args, 1 << 40, null) == xb.XKV_ERR_INVALID_ARG
    args[7], args[10] = one, 3                                # outliers announced but not given
    assert lib.xkv_sr_decode_landmark(*args, 1 << 40, null) == xb.XKV_ERR_INVALID_ARG
    args[10], args[14] = 0, 5                                 # tail tokens without their keys
    assert lib.xkv_sr_decode_landmark(*args, 1 << 40, null) == xb.XKV_ERR_INVALID_ARG


def test_absorbed_calls_validate_on_the_host():
    lib = xb.load()
    good = xb.Shape.of(synth.LLAMA_FULL)
    c, null, one, al = good.c(), ctypes.c_void_p(0), ctypes.c_void_p(256), ctypes.c_void_p(4096)
    n = ctypes.c_size_t(0)
    need = xb.xkv_absorbed_workspace_bytes(good)
    heads = good.batch * good.H_kv * good.L * xb.head_pitch(good) * 4          # the head scores live in the workspace
    assert need >= xb.xkv_workspace_bytes(good) + heads
    assert xb.head_pitch(xb.Shape.of(synth.QWEN)) == 8 and xb.head_pitch(good) == 4
    ragged = xb.Shape.of(synth.LLAMA_FULL.with_(r_v=508)).c()                   # rows of A^V not whole 16-byte pieces
    assert lib.xkv_absorbed_workspace_bytes(ctypes.byref(ragged), ctypes.byref(n)) == xb.XKV_ERR_UNSUPPORTED
    assert lib.xkv_absorbed_workspace_bytes(ctypes.byref(c), None) == xb.XKV_ERR_INVALID_ARG
    big = 1 << 40
    assert lib.xkv_head_scores(ctypes.byref(c), 0, one, one, one, null, null, al, big, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_head_scores(ctypes.byref(c), 0, one, one, one, null, ctypes.c_void_p(260), al, big, null) \
        == xb.XKV_ERR_INVALID_ARG                                               # misaligned head scores
    assert lib.xkv_head_scores(ctypes.byref(c), 9, one, one, one, null, al, al, big, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_attend_absorbed(ctypes.byref(c), 0, al, one, al, null, one, al, big, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_attend_absorbed(ctypes.byref(c), 0, ctypes.c_void_p(264), one, al, one, one, al, big, null) \
        == xb.XKV_ERR_INVALID_ARG                                               # misaligned A^V
    assert lib.xkv_attend_absorbed(ctypes.byref(c), 0, al, one, al, one, one, al, need - 1, null) == xb.XKV_ERR_WORKSPACE
    assert lib.xkv_sr_decode_absorbed(ctypes.byref(c), 0, al, al, one, one, one, null, null, 0, null, null, null, al, big,
                                      null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_sr_decode_absorbed(ctypes.byref(c), 0, al, al, one, one, one, null, null, 5, one, null, null, al, big,
                                      null) == xb.XKV_ERR_INVALID_ARG          # a tail length without tail tensors
    assert lib.xkv_sr_decode_absorbed(ctypes.byref(c), 0, al, al, one, one, one, null, null, 0, one, null, null, al,
                                      xb.xkv_workspace_bytes(good), null) == xb.XKV_ERR_WORKSPACE


def test_quantised_calls_validate_on_the_host():
    lib = xb.load()
    good = xb.Shape.of(synth.LLAMA_FULL)
    c, null, one, al = good.c(), ctypes.c_void_p(0), ctypes.c_void_p(256), ctypes.c_void_p(4096)
    n = ctypes.c_size_t(0)
    assert xb.xkv_quantized_row_bytes(512) == 320 and xb.xkv_quantized_row_bytes(384) == 240     # 5r/8
    assert lib.xkv_quantized_row_bytes(512, 3, ctypes.byref(n)) == xb.XKV_OK and n.value == 256    # 3-bit rows: r/2
    assert lib.xkv_quantized_row_bytes(512, 2, ctypes.byref(n)) == xb.XKV_ERR_UNSUPPORTED          # 2-bit rows: not built
    assert xb.xkv_quantized_row_bytes(96) == 64 and xb.xkv_quantized_row_bytes(576) == 368      # padded to 16 bytes
    assert lib.xkv_quantized_row_bytes(100, 4, ctypes.byref(n)) == xb.XKV_ERR_UNSUPPORTED          # r % 32 != 0
    assert lib.xkv_quantized_row_bytes(512, 4, None) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_quantize_rows(al, 0, 512, 4, al, null) == xb.XKV_OK                             # nothing to do
    assert lib.xkv_quantize_rows(null, 5, 512, 4, al, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_quantize_rows(ctypes.c_void_p(260), 5, 512, 4, al, null) == xb.XKV_ERR_INVALID_ARG   # misaligned
    assert lib.xkv_quantize_rows(al, -1, 512, 4, al, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_quantize_rows(al, 5, 500, 4, al, null) == xb.XKV_ERR_UNSUPPORTED
    big = 1 << 40
    odd = xb.Shape.of(synth.LLAMA_FULL.with_(r_k=448)).c()                                         # r_k not a multiple of 128
    assert lib.xkv_head_scores_q4(ctypes.byref(odd), 0, al, al, al, null, al, al, big, null) == xb.XKV_ERR_UNSUPPORTED
    assert lib.xkv_head_scores_q4(ctypes.byref(c), 0, null, al, al, null, al, al, big, null) == xb.XKV_ERR_INVALID_ARG
    f32 = xb.Shape.of(synth.LLAMA_FULL.with_(dtype="f32")).c()
    assert lib.xkv_attend_absorbed_q4(ctypes.byref(f32), 0, al, one, al, one, one, al, big, null) == xb.XKV_ERR_UNSUPPORTED
    assert lib.xkv_sr_decode_absorbed_q4(ctypes.byref(f32), 0, al, al, al, al, al, null, null, 0, one, null, null, al,
                                         big, null) == xb.XKV_ERR_UNSUPPORTED
    assert lib.xkv_sr_decode_absorbed_q4(ctypes.byref(c), 0, al, al, al, al, al, null, null, 0, one, null, null, al, 64,
                                         null) == xb.XKV_ERR_WORKSPACE


def test_binding_has_no_cpu_fallback(monkeypatch):
    monkeypatch.setattr(xb, "_lib", None)
    monkeypatch.setattr(xb, "LIB_PATH", os.path.join(ROOT, "does_not_exist.so"))
    with pytest.raises(RuntimeError):
        xb.load()


def test_packed_and_static_calls_validate_on_the_host():
    """The calls on B_l re-ordered once per prompt, and the call on the library's own scratch: rejected on the host,
    before any launch, for missing operands, shapes the matrix-core kernel does not take, and plans beyond the
    static scratch."""
    lib = xb.load()
    good = xb.Shape.of(synth.LLAMA_GROUP)
    c, null, one, al = good.c(), ctypes.c_void_p(0), ctypes.c_void_p(256), ctypes.c_void_p(4096)
    n = ctypes.c_size_t(0)
    big = 1 << 40
    # size of the packed copy: about B_k and B_v themselves (ranks padded to whole pairs of 128-rank groups)
    plain = 2 * good.batch * good.G * good.r_k * good.H_kv * good.d_h * 2
    assert plain <= xb.xkv_packed_b_bytes(good) <= 2 * plain
    assert lib.xkv_packed_b_bytes(ctypes.byref(c), None) == xb.XKV_ERR_INVALID_ARG
    f32 = xb.Shape.of(synth.TINY).c()                                            # fp32: no matrix-core kernel
    assert lib.xkv_packed_b_bytes(ctypes.byref(f32), ctypes.byref(n)) == xb.XKV_ERR_UNSUPPORTED
    assert lib.xkv_pack_b(ctypes.byref(c), null, al, al, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_pack_b(ctypes.byref(c), al, al, null, null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_pack_b(ctypes.byref(f32), al, al, al, null) == xb.XKV_ERR_UNSUPPORTED
    # the packed steps: no packed copy, no workspace, a workspace too small
    assert lib.xkv_sr_decode_packed(ctypes.byref(c), 0, al, al, al, null, al, al, null, null, al, big,
                                    null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_sr_decode_packed(ctypes.byref(c), 0, al, al, al, al, al, al, null, null, al, 16,
                                    null) == xb.XKV_ERR_WORKSPACE
    assert lib.xkv_sr_decode_packed(ctypes.byref(c), 0, al, al, al, ctypes.c_void_p(4100), al, al, null, null, al, big,
                                    null) == xb.XKV_ERR_UNSUPPORTED             # misaligned packed copy
    assert lib.xkv_sr_decode_tail_packed(ctypes.byref(c), 0, al, al, al, null, al, null, null, 0, al, null, null, al, big,
                                         null) == xb.XKV_ERR_INVALID_ARG
    assert lib.xkv_sr_decode_tail_packed(ctypes.byref(c), 0, al, al, al, al, al, null, al, 7, al, null, null, al, big,
                                         null) == xb.XKV_ERR_INVALID_ARG         # tail tokens without their keys
    args = [ctypes.byref(c), 0, al, al, 0, al, null, al, al, null, 8, 0, ctypes.c_float(0.0), null, null, 0, al, null,
            null, null, al]
    assert lib.xkv_sr_decode_landmark_packed(*args, big, null) == xb.XKV_ERR_INVALID_ARG     # no packed copy
    args[6], args[4] = al, 5
    assert lib.xkv_sr_decode_landmark_packed(*args, big, null) == xb.XKV_ERR_UNSUPPORTED     # 5-bit rows
    args[4] = 0
    assert lib.xkv_sr_decode_landmark_packed(*args, 16, null) == xb.XKV_ERR_WORKSPACE
    # the static scratch: configuration 3's plan is larger than the array
    full = xb.Shape.of(synth.LLAMA_FULL)
    assert xb.xkv_workspace_bytes(full) > xb.STATIC_SCRATCH_BYTES >= xb.xkv_workspace_bytes(good)
    assert lib.xkv_sr_decode_static(ctypes.byref(full.c()), 0, al, al, al, al, al, al, null, null,
                                    null) == xb.XKV_ERR_WORKSPACE
    assert lib.xkv_sr_decode_static(ctypes.byref(c), 0, al, al, al, al, null, al, null, null,
                                    null) == xb.XKV_ERR_INVALID_ARG
