"""Thin Python binding of libxkv's C ABI: argument marshalling only.

Every function has the name and argument order of its C entry point (include/xkv.h) and takes
torch tensors for device memory; the stream is torch's current stream unless one is given.
There is no CPU fallback: if the HIP library is not built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libxkv.so")

XKV_OK, XKV_ERR_INVALID_ARG, XKV_ERR_UNSUPPORTED, XKV_ERR_WORKSPACE, XKV_ERR_HIP = 0, -1, -2, -3, -4
XKV_F32, XKV_BF16 = 0, 1
DTYPES = {"f32": XKV_F32, "bf16": XKV_BF16}

ENTRY_POINTS = ("xkv_workspace_bytes", "xkv_sr_decode", "xkv_sr_decode_static", "xkv_packed_b_bytes", "xkv_pack_b",
                "xkv_sr_decode_packed", "xkv_sr_decode_tail", "xkv_dense_decode", "xkv_score",
                "xkv_topk", "xkv_gather_attend", "xkv_reconstruct", "xkv_factorize_workspace_bytes", "xkv_factorize",
                "xkv_factorize_svd",
                "xkv_landmark_workspace_bytes", "xkv_landmarks", "xkv_sr_decode_landmark", "xkv_gather_attend_ex",
                "xkv_absorbed_workspace_bytes", "xkv_head_scores", "xkv_attend_absorbed", "xkv_sr_decode_absorbed",
                "xkv_quantized_row_bytes", "xkv_quantize_rows", "xkv_attend_absorbed_q4", "xkv_head_scores_q4",
                "xkv_sr_decode_absorbed_q4", "xkv_gather_attend_q", "xkv_sr_decode_landmark_q", "xkv_sr_decode_q4",
                "xkv_sr_decode_landmark_packed", "xkv_sr_decode_tail_packed",
                "xkv_profile_kernel", "xkv_status_string", "xkv_version")


class XkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where} failed: {status_string(status)} ({status})")


class xkv_shape(ctypes.Structure):
    _fields_ = [("G", ctypes.c_int32), ("H_kv", ctypes.c_int32), ("H_q", ctypes.c_int32), ("d_h", ctypes.c_int32),
                ("r_k", ctypes.c_int32), ("r_v", ctypes.c_int32), ("L", ctypes.c_int32), ("k", ctypes.c_int32),
                ("batch", ctypes.c_int32), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float)]


@dataclass(frozen=True)
class Shape:
    G: int
    H_kv: int
    H_q: int
    d_h: int
    r_k: int
    r_v: int
    L: int
    k: int
    batch: int
    dtype: str = "bf16"
    scale: float = 0.0

    def c(self) -> xkv_shape:
        return xkv_shape(self.G, self.H_kv, self.H_q, self.d_h, self.r_k, self.r_v, self.L, self.k, self.batch,
                         DTYPES[self.dtype], self.scale)

    @staticmethod
    def of(w, **kw) -> "Shape":
        """From a synth.Workload (or anything with the same field names)."""
        f = dict(G=w.G, H_kv=w.H_kv, H_q=w.H_q, d_h=w.d_h, r_k=w.r_k, r_v=w.r_v, L=w.L, k=w.k, batch=w.batch,
                 dtype=w.dtype)
        f.update(kw)
        return Shape(**f)


_lib = None


def load() -> ctypes.CDLL:
    """Load libxkv.so (built in-tree by build.build_library()).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2503_18893_amd.build` "
                               "(or __graft_entry__.build()); there is no fallback path")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        sp = ctypes.POINTER(xkv_shape)
        lib.xkv_workspace_bytes.argtypes = [sp, ctypes.POINTER(sz)]
        lib.xkv_sr_decode.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_packed_b_bytes.argtypes = [sp, ctypes.POINTER(sz)]
        lib.xkv_pack_b.argtypes = [sp, vp, vp, vp, vp]
        lib.xkv_sr_decode_packed.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_sr_decode_static.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.xkv_sr_decode_tail.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz, vp]
        lib.xkv_sr_decode_tail_packed.argtypes = lib.xkv_sr_decode_tail.argtypes
        lib.xkv_dense_decode.argtypes = [sp, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_score.argtypes = [sp, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_topk.argtypes = [sp, vp, vp, vp, sz, vp]
        lib.xkv_gather_attend.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_reconstruct.argtypes = [sp, i32, vp, vp, i32, vp, vp]
        lib.xkv_factorize_workspace_bytes.argtypes = [sp, i32, ctypes.POINTER(sz)]
        lib.xkv_factorize.argtypes = [sp, vp, i32, i32, ctypes.c_uint32, vp, vp, vp, sz, vp]
        lib.xkv_factorize_svd.argtypes = [sp, vp, i32, i32, i32, ctypes.c_uint32, vp, vp, vp, vp, sz, vp]
        lib.xkv_landmark_workspace_bytes.argtypes = [sp, i32, i32, ctypes.POINTER(sz)]
        lib.xkv_landmarks.argtypes = [sp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
        lib.xkv_sr_decode_landmark.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, i32, i32, ctypes.c_float, vp, vp, i32,
                                               vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_gather_attend_ex.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
        lib.xkv_absorbed_workspace_bytes.argtypes = [sp, ctypes.POINTER(sz)]
        lib.xkv_head_scores.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_attend_absorbed.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_sr_decode_absorbed.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz, vp]
        lib.xkv_quantized_row_bytes.argtypes = [i32, i32, ctypes.POINTER(sz)]
        lib.xkv_quantize_rows.argtypes = [vp, ctypes.c_int64, i32, i32, vp, vp]
        lib.xkv_attend_absorbed_q4.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_head_scores_q4.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_sr_decode_absorbed_q4.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz, vp]
        lib.xkv_gather_attend_q.argtypes = [sp, i32, vp, vp, i32, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
        lib.xkv_sr_decode_landmark_q.argtypes = [sp, i32, vp, vp, i32, vp, vp, vp, vp, vp, i32, i32, ctypes.c_float, vp, vp,
                                                 i32, vp, vp, vp, vp, vp, sz, vp]
        lib.xkv_sr_decode_q4.argtypes = [sp, i32, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, i32, vp, vp, vp, vp, sz, vp]
        lib.xkv_sr_decode_landmark_packed.argtypes = lib.xkv_sr_decode_landmark_q.argtypes
        lib.xkv_profile_kernel.argtypes = [i32, vp, vp]
        lib.xkv_status_string.argtypes = [ctypes.c_int]
        lib.xkv_status_string.restype = ctypes.c_char_p
        lib.xkv_version.restype = i32
        for name in ENTRY_POINTS:
            if name not in ("xkv_status_string", "xkv_version"):   # every other call returns an xkv_status
                getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().xkv_status_string(int(status)).decode()


def xkv_version() -> int:
    return int(load().xkv_version())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(int(stream))


def _check(status: int, where: str):
    if status != XKV_OK:
        raise XkvError(status, where)


def xkv_workspace_bytes(shape: Shape) -> int:
    n = ctypes.c_size_t(0)
    _check(load().xkv_workspace_bytes(ctypes.byref(shape.c()), ctypes.byref(n)), "xkv_workspace_bytes")
    return int(n.value)


def alloc_workspace(shape: Shape, device="cuda"):
    """A torch byte tensor large enough for any entry point at this shape (256-byte aligned by torch)."""
    import torch
    return torch.empty(max(xkv_workspace_bytes(shape), 256), dtype=torch.uint8, device=device)


def xkv_sr_decode(shape, layer_in_group, A_k, A_v, B_k, B_v, q, out, idx_out, score_out, workspace, stream=None):
    _check(load().xkv_sr_decode(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), _ptr(B_k), _ptr(B_v),
                                _ptr(q), _ptr(out), _ptr(idx_out), _ptr(score_out), _ptr(workspace),
                                workspace.numel(), _stream(stream)), "xkv_sr_decode")


def xkv_packed_b_bytes(shape: Shape) -> int:
    n = ctypes.c_size_t(0)
    _check(load().xkv_packed_b_bytes(ctypes.byref(shape.c()), ctypes.byref(n)), "xkv_packed_b_bytes")
    return int(n.value)


def xkv_pack_b(shape, B_k, B_v, packed_out, stream=None):
    _check(load().xkv_pack_b(ctypes.byref(shape.c()), _ptr(B_k), _ptr(B_v), _ptr(packed_out), _stream(stream)),
           "xkv_pack_b")


def xkv_sr_decode_packed(shape, layer_in_group, A_k, A_v, B_k, B_packed, q, out, idx_out, score_out, workspace,
                         stream=None):
    _check(load().xkv_sr_decode_packed(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), _ptr(B_k),
                                       _ptr(B_packed), _ptr(q), _ptr(out), _ptr(idx_out), _ptr(score_out),
                                       _ptr(workspace), workspace.numel(), _stream(stream)), "xkv_sr_decode_packed")


STATIC_SCRATCH_BYTES = 40 << 20


def xkv_sr_decode_tail_packed(shape, layer_in_group, A_k, A_v, B_k, B_packed, q, K_tail, V_tail, T, out, idx_out, score_out,
                              workspace, stream=None):
    _check(load().xkv_sr_decode_tail_packed(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), _ptr(B_k),
                                            _ptr(B_packed), _ptr(q), _ptr(K_tail), _ptr(V_tail), int(T), _ptr(out),
                                            _ptr(idx_out), _ptr(score_out), _ptr(workspace), workspace.numel(),
                                            _stream(stream)), "xkv_sr_decode_tail_packed")


def xkv_sr_decode_static(shape, layer_in_group, A_k, A_v, B_k, B_v, q, out, idx_out, score_out, stream=None):
    _check(load().xkv_sr_decode_static(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), _ptr(B_k),
                                       _ptr(B_v), _ptr(q), _ptr(out), _ptr(idx_out), _ptr(score_out), _stream(stream)),
           "xkv_sr_decode_static")


def xkv_sr_decode_tail(shape, layer_in_group, A_k, A_v, B_k, B_v, q, K_tail, V_tail, T, out, idx_out, score_out,
                       workspace, stream=None):
    _check(load().xkv_sr_decode_tail(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), _ptr(B_k),
                                     _ptr(B_v), _ptr(q), _ptr(K_tail), _ptr(V_tail), int(T), _ptr(out), _ptr(idx_out),
                                     _ptr(score_out), _ptr(workspace), workspace.numel(), _stream(stream)),
           "xkv_sr_decode_tail")


def xkv_dense_decode(shape, K, V, q, out, workspace, stream=None):
    _check(load().xkv_dense_decode(ctypes.byref(shape.c()), _ptr(K), _ptr(V), _ptr(q), _ptr(out), _ptr(workspace),
                                   workspace.numel(), _stream(stream)), "xkv_dense_decode")


def xkv_score(shape, layer_in_group, A_k, B_k, q, score_out, workspace, stream=None):
    _check(load().xkv_score(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(B_k), _ptr(q), _ptr(score_out),
                            _ptr(workspace), workspace.numel(), _stream(stream)), "xkv_score")


def xkv_topk(shape, score, idx_out, workspace, stream=None):
    _check(load().xkv_topk(ctypes.byref(shape.c()), _ptr(score), _ptr(idx_out), _ptr(workspace), workspace.numel(),
                           _stream(stream)), "xkv_topk")


def xkv_gather_attend(shape, layer_in_group, A_k, A_v, B_k, B_v, q, idx, out, workspace, stream=None):
    _check(load().xkv_gather_attend(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), _ptr(B_k),
                                    _ptr(B_v), _ptr(q), _ptr(idx), _ptr(out), _ptr(workspace), workspace.numel(),
                                    _stream(stream)), "xkv_gather_attend")


def xkv_reconstruct(shape, layer_in_group, A, B, r, X_out, stream=None):
    _check(load().xkv_reconstruct(ctypes.byref(shape.c()), layer_in_group, _ptr(A), _ptr(B), r, _ptr(X_out),
                                  _stream(stream)), "xkv_reconstruct")


def xkv_factorize_workspace_bytes(shape: Shape, r: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load().xkv_factorize_workspace_bytes(ctypes.byref(shape.c()), r, ctypes.byref(n)),
           "xkv_factorize_workspace_bytes")
    return int(n.value)


def xkv_factorize(shape, X, r, iters, seed, A_out, B_out, workspace, stream=None):
    _check(load().xkv_factorize(ctypes.byref(shape.c()), _ptr(X), r, iters, seed, _ptr(A_out), _ptr(B_out),
                                _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "xkv_factorize")


def xkv_factorize_svd(shape, X, r, r_out, iters, seed, A_out, B_out, sigma_out, workspace, stream=None):
    _check(load().xkv_factorize_svd(ctypes.byref(shape.c()), _ptr(X), r, r_out, iters, seed, _ptr(A_out), _ptr(B_out),
                                    _ptr(sigma_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream(stream)), "xkv_factorize_svd")


def xkv_landmark_workspace_bytes(shape: Shape, c: int, o: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load().xkv_landmark_workspace_bytes(ctypes.byref(shape.c()), c, o, ctypes.byref(n)),
           "xkv_landmark_workspace_bytes")
    return int(n.value)


def xkv_landmarks(shape, K_rope, c, o, landmarks_out, neg_min_cos_out, outliers_out, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().xkv_landmarks(ctypes.byref(shape.c()), _ptr(K_rope), c, o, _ptr(landmarks_out), _ptr(neg_min_cos_out),
                                _ptr(outliers_out), _ptr(workspace), nbytes, _stream(stream)), "xkv_landmarks")


def xkv_gather_attend_ex(shape, layer_in_group, A_k, A_v, B_k, B_v, q, idx, counts, rope_theta, out, workspace,
                         stream=None):
    _check(load().xkv_gather_attend_ex(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), _ptr(B_k),
                                       _ptr(B_v), _ptr(q), _ptr(idx), _ptr(counts), float(rope_theta), _ptr(out),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "xkv_gather_attend_ex")


def xkv_sr_decode_landmark(shape, layer_in_group, A_k, A_v, B_k, B_v, q, landmarks, outliers, c, o, out, rows_out,
                           count_out, score_out, workspace, stream=None, rope_theta=0.0, K_tail=None, V_tail=None, T=0):
    _check(load().xkv_sr_decode_landmark(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), _ptr(B_k),
                                         _ptr(B_v), _ptr(q), _ptr(landmarks), _ptr(outliers), c, o, float(rope_theta),
                                         _ptr(K_tail), _ptr(V_tail), T, _ptr(out),
                                         _ptr(rows_out), _ptr(count_out), _ptr(score_out), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "xkv_sr_decode_landmark")


def head_pitch(shape) -> int:
    """Row length of the per-head score array: query heads per KV head rounded up to a power of two."""
    n_rep = shape.H_q // shape.H_kv
    return 1 << max(0, (n_rep - 1).bit_length())


def xkv_absorbed_workspace_bytes(shape) -> int:
    n = ctypes.c_size_t(0)
    _check(load().xkv_absorbed_workspace_bytes(ctypes.byref(shape.c()), ctypes.byref(n)), "xkv_absorbed_workspace_bytes")
    return int(n.value)


def xkv_head_scores(shape, layer_in_group, A_k, B_k, q, score_out, heads_out, workspace, stream=None):
    _check(load().xkv_head_scores(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(B_k), _ptr(q), _ptr(score_out),
                                  _ptr(heads_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                  _stream(stream)), "xkv_head_scores")


def xkv_attend_absorbed(shape, layer_in_group, A_v, B_v, head_scores, idx, out, workspace, stream=None):
    _check(load().xkv_attend_absorbed(ctypes.byref(shape.c()), layer_in_group, _ptr(A_v), _ptr(B_v), _ptr(head_scores),
                                      _ptr(idx), _ptr(out), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream)),
           "xkv_attend_absorbed")


def xkv_quantized_row_bytes(r: int, bits: int = 4) -> int:
    n = ctypes.c_size_t(0)
    _check(load().xkv_quantized_row_bytes(r, bits, ctypes.byref(n)), "xkv_quantized_row_bytes")
    return int(n.value)


def xkv_quantize_rows(X, rows, r, out, bits=4, stream=None):
    _check(load().xkv_quantize_rows(_ptr(X), int(rows), int(r), int(bits), _ptr(out), _stream(stream)),
           "xkv_quantize_rows")


def xkv_attend_absorbed_q4(shape, layer_in_group, Aq_v, B_v, head_scores, idx, out, workspace, stream=None):
    _check(load().xkv_attend_absorbed_q4(ctypes.byref(shape.c()), layer_in_group, _ptr(Aq_v), _ptr(B_v),
                                         _ptr(head_scores), _ptr(idx), _ptr(out), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "xkv_attend_absorbed_q4")


def xkv_head_scores_q4(shape, layer_in_group, Aq_k, B_k, q, score_out, heads_out, workspace, stream=None):
    _check(load().xkv_head_scores_q4(ctypes.byref(shape.c()), layer_in_group, _ptr(Aq_k), _ptr(B_k), _ptr(q),
                                     _ptr(score_out), _ptr(heads_out), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)), "xkv_head_scores_q4")


def xkv_sr_decode_absorbed_q4(shape, layer_in_group, Aq_k, Aq_v, B_k, B_v, q, out, idx_out, score_out, workspace,
                              stream=None, K_tail=None, V_tail=None, T=0):
    _check(load().xkv_sr_decode_absorbed_q4(ctypes.byref(shape.c()), layer_in_group, _ptr(Aq_k), _ptr(Aq_v), _ptr(B_k),
                                            _ptr(B_v), _ptr(q), _ptr(K_tail), _ptr(V_tail), int(T), _ptr(out),
                                            _ptr(idx_out), _ptr(score_out), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream)),
           "xkv_sr_decode_absorbed_q4")


def xkv_sr_decode_absorbed(shape, layer_in_group, A_k, A_v, B_k, B_v, q, out, idx_out, score_out, workspace,
                           stream=None, K_tail=None, V_tail=None, T=0):
    _check(load().xkv_sr_decode_absorbed(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), _ptr(B_k),
                                         _ptr(B_v), _ptr(q), _ptr(K_tail), _ptr(V_tail), int(T), _ptr(out),
                                         _ptr(idx_out), _ptr(score_out), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "xkv_sr_decode_absorbed")


def xkv_gather_attend_q(shape, layer_in_group, Aq_k, Aq_v, bits, B_k, B_v, q, idx, counts, rope_theta, out, workspace,
                        stream=None):
    _check(load().xkv_gather_attend_q(ctypes.byref(shape.c()), layer_in_group, _ptr(Aq_k), _ptr(Aq_v), int(bits),
                                      _ptr(B_k), _ptr(B_v), _ptr(q), _ptr(idx), _ptr(counts), float(rope_theta),
                                      _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)), "xkv_gather_attend_q")


def xkv_sr_decode_landmark_q(shape, layer_in_group, Aq_k, Aq_v, bits, B_k, B_v, q, landmarks, outliers, c, o, out,
                             rows_out, count_out, score_out, workspace, stream=None, rope_theta=0.0, K_tail=None,
                             V_tail=None, T=0):
    _check(load().xkv_sr_decode_landmark_q(ctypes.byref(shape.c()), layer_in_group, _ptr(Aq_k), _ptr(Aq_v), int(bits),
                                           _ptr(B_k), _ptr(B_v), _ptr(q), _ptr(landmarks), _ptr(outliers), c, o,
                                           float(rope_theta), _ptr(K_tail), _ptr(V_tail), T, _ptr(out), _ptr(rows_out),
                                           _ptr(count_out), _ptr(score_out), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream(stream)),
           "xkv_sr_decode_landmark_q")


def xkv_sr_decode_landmark_packed(shape, layer_in_group, A_k, A_v, bits, B_k, B_packed, q, landmarks, outliers, c, o, out,
                                  rows_out, count_out, score_out, workspace, stream=None, rope_theta=0.0, K_tail=None,
                                  V_tail=None, T=0):
    _check(load().xkv_sr_decode_landmark_packed(ctypes.byref(shape.c()), layer_in_group, _ptr(A_k), _ptr(A_v), int(bits),
                                                _ptr(B_k), _ptr(B_packed), _ptr(q), _ptr(landmarks), _ptr(outliers), c,
                                                o, float(rope_theta), _ptr(K_tail), _ptr(V_tail), T, _ptr(out),
                                                _ptr(rows_out), _ptr(count_out), _ptr(score_out), _ptr(workspace),
                                                workspace.numel() * workspace.element_size(), _stream(stream)),
           "xkv_sr_decode_landmark_packed")


def xkv_sr_decode_q4(shape, layer_in_group, Aq_k, Aq_v, B_k, B_v, q, out, idx_out, score_out, workspace, stream=None,
                     rope_theta=0.0, K_tail=None, V_tail=None, T=0):
    _check(load().xkv_sr_decode_q4(ctypes.byref(shape.c()), layer_in_group, _ptr(Aq_k), _ptr(Aq_v), _ptr(B_k), _ptr(B_v),
                                   _ptr(q), float(rope_theta), _ptr(K_tail), _ptr(V_tail), int(T), _ptr(out),
                                   _ptr(idx_out), _ptr(score_out), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)), "xkv_sr_decode_q4")


STAGE_SCORE, STAGE_GATHER_ATTEND, STAGE_DENSE, STAGE_FACTORIZE_GRAM, STAGE_ABSORB_ROWS = 0, 1, 2, 3, 4


def xkv_profile_kernel(stage, start_event=None, stop_event=None):
    """start_event / stop_event: hipEvent_t handles as integers (e.g. torch.cuda.Event(...).cuda_event), or None."""
    a = ctypes.c_void_p(int(start_event)) if start_event else None
    b = ctypes.c_void_p(int(stop_event)) if stop_event else None
    _check(load().xkv_profile_kernel(stage, a, b), "xkv_profile_kernel")
