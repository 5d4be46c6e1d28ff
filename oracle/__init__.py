"""CPU oracle for xKV Selective-Reconstruction decode (test infrastructure).

Thin ctypes wrapper around ``xkv_oracle.c`` (plain C, double precision).  Only
``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg
may import this package; the GPU library never does and shares no code with it.

Inputs may be float64, float32 or bf16 (given as ``uint16`` bit patterns); they
are widened to float64 exactly before the C code sees them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "xkv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fvisibility=hidden", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_compression_ratio.restype = ctypes.c_double
        _lib.oracle_compression_ratio.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                  ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    return _lib


def widen(x) -> np.ndarray:
    """Exact widening to float64: float arrays as they are, uint16 taken as bf16 bits."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        x = (x.astype(np.uint32) << 16).view(np.float32)
    return np.ascontiguousarray(x, dtype=np.float64)


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def default_scale(d_h: int) -> float:
    return 1.0 / float(np.sqrt(np.float64(d_h)))


def project(B_k, q, H_kv):
    """p[H_q][r_k] = B^K_{l,rho(h)} q_h (step 1)."""
    B_k, q = widen(B_k), widen(q)
    r_k, d = B_k.shape
    H_q, d_h = q.shape
    assert d == H_kv * d_h and H_q % H_kv == 0
    p = np.empty((H_q, r_k), np.float64)
    _load().oracle_project(_dp(B_k), _dp(q), r_k, H_kv, H_q, d_h, _dp(p))
    return p


def scores(A_k, p, scale):
    """s[H_q][L] = scale * A^K p_h (step 2)."""
    A_k, p = widen(A_k), widen(p)
    L, r_k = A_k.shape
    H_q = p.shape[0]
    assert p.shape[1] == r_k
    s = np.empty((H_q, L), np.float64)
    _load().oracle_scores(_dp(A_k), _dp(p), L, r_k, H_q, ctypes.c_double(scale), _dp(s))
    return s


def pool(s, H_kv):
    """S[H_kv][L] = max over the query heads of each KV head (step 3)."""
    s = widen(s)
    H_q, L = s.shape
    assert H_q % H_kv == 0
    S = np.empty((H_kv, L), np.float64)
    _load().oracle_pool(_dp(s), L, H_kv, H_q, _dp(S))
    return S


def pooled_scores(A_k, B_k, q, H_kv, scale=None):
    """Steps 1-3: pooled fp64 scores S[H_kv][L]."""
    q = widen(q)
    scale = default_scale(q.shape[1]) if scale is None else scale
    return pool(scores(A_k, project(B_k, q, H_kv), scale), H_kv)


def select(S_row, k):
    """Step 4 on one fp32 score row: the k selected indices, ascending."""
    S_row = np.ascontiguousarray(S_row, dtype=np.float32)
    assert S_row.ndim == 1
    idx = np.empty((k,), np.int32)
    rc = _load().oracle_select(_fp(S_row), S_row.shape[0], k, _ip(idx))
    if rc != 0:
        raise ValueError(f"oracle_select failed ({rc})")
    return idx


def reconstruct(A, B):
    """Dense reconstruction X^ = A B."""
    A, B = widen(A), widen(B)
    L, r = A.shape
    assert B.shape[0] == r
    d = B.shape[1]
    X = np.empty((L, d), np.float64)
    _load().oracle_reconstruct(_dp(A), _dp(B), L, r, d, _dp(X))
    return X


def gather_attend(A_k, A_v, B_k, B_v, q, idx, scale=None):
    """Steps 5-6 for given index sets idx[H_kv][k]: out[H_q][d_h]."""
    A_k, A_v, B_k, B_v, q = map(widen, (A_k, A_v, B_k, B_v, q))
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    L, r_k = A_k.shape
    r_v = A_v.shape[1]
    H_q, d_h = q.shape
    H_kv, k = idx.shape
    assert B_k.shape == (r_k, H_kv * d_h) and B_v.shape == (r_v, H_kv * d_h) and A_v.shape[0] == L
    scale = default_scale(d_h) if scale is None else scale
    out = np.empty((H_q, d_h), np.float64)
    rc = _load().oracle_gather_attend(_dp(A_k), _dp(A_v), _dp(B_k), _dp(B_v), _dp(q), _ip(idx),
                                      L, r_k, r_v, H_kv, H_q, d_h, k, ctypes.c_double(scale), _dp(out))
    if rc != 0:
        raise ValueError(f"oracle_gather_attend failed ({rc})")
    return out


def head_scores(A_k, B_k, q, H_kv, scale=None):
    """Steps 1-2 without the pooling: s[H_q][L] = scale * A^K (B^K_{rho(h)} q_h), the per-head logits of every token."""
    q = widen(q)
    scale = default_scale(q.shape[1]) if scale is None else scale
    return scores(A_k, project(B_k, q, H_kv), scale)


def gather_attend_absorbed(A_k, A_v, B_k, B_v, q, idx, scale=None):
    """Steps 5-6 in the form that never builds K^ or V^ (associativity of Eq. 3, valid as long as nothing such as a
    rotation sits between the factors and the query): the logits of the selected tokens are entries of the head
    scores, logits = s[h][I_g]; the weighted sum runs over rows of A^V and B^V is applied once at the end,
    o_h = ((w^T A^V[I_g]) B^V_g).  Written out in numpy; equals gather_attend."""
    A_k, A_v, B_k, B_v, q = map(widen, (A_k, A_v, B_k, B_v, q))
    idx = np.asarray(idx)
    H_q, d_h = q.shape
    H_kv = idx.shape[0]
    n_rep = H_q // H_kv
    s = head_scores(A_k, B_k, q, H_kv, scale)
    out = np.empty((H_q, d_h), np.float64)
    for g in range(H_kv):
        rows_v = A_v[idx[g]]
        for h in range(g * n_rep, (g + 1) * n_rep):
            z = s[h][idx[g]]
            wgt = np.exp(z - z.max())
            u = (wgt / wgt.sum()) @ rows_v
            out[h] = u @ B_v[:, g * d_h:(g + 1) * d_h]
    return out


def dense(K, V, q, H_kv, scale=None):
    """Textbook decode attention, K and V as [L][H_kv*d_h]: out[H_q][d_h]."""
    K, V, q = widen(K), widen(V), widen(q)
    L, d = K.shape
    H_q, d_h = q.shape
    assert d == H_kv * d_h and V.shape == K.shape
    scale = default_scale(d_h) if scale is None else scale
    out = np.empty((H_q, d_h), np.float64)
    rc = _load().oracle_dense(_dp(K), _dp(V), _dp(q), L, H_kv, H_q, d_h, ctypes.c_double(scale), _dp(out))
    if rc != 0:
        raise ValueError(f"oracle_dense failed ({rc})")
    return out


def sr_decode(A_k, A_v, B_k, B_v, q, H_kv, k, scale=None):
    """Whole SR step (steps 1-6).  Returns (out[H_q][d_h], idx[H_kv][k], S32[H_kv][L])."""
    A_k, A_v, B_k, B_v, q = map(widen, (A_k, A_v, B_k, B_v, q))
    L, r_k = A_k.shape
    r_v = A_v.shape[1]
    H_q, d_h = q.shape
    scale = default_scale(d_h) if scale is None else scale
    out = np.empty((H_q, d_h), np.float64)
    idx = np.empty((H_kv, k), np.int32)
    S32 = np.empty((H_kv, L), np.float32)
    rc = _load().oracle_sr_decode(_dp(A_k), _dp(A_v), _dp(B_k), _dp(B_v), _dp(q), L, r_k, r_v, H_kv, H_q, d_h,
                                  k, ctypes.c_double(scale), _dp(out), _ip(idx), _fp(S32))
    if rc != 0:
        raise ValueError(f"oracle_sr_decode failed ({rc})")
    return out, idx, S32


def gather_attend_tail(A_k, A_v, B_k, B_v, q, idx, K_tail, V_tail, scale=None):
    """Steps 5-6 for given index sets idx[H_kv][k] over a context whose T most recent tokens are uncompressed:
    attention over the k reconstructed rows of each KV head (Eq. 3) together with all T tail rows, one softmax over
    the union.  K_tail, V_tail: [H_kv][T][d_h].  Written out in numpy on purpose (no blocking, no running maxima).
    """
    A_k, A_v, B_k, B_v, q = map(widen, (A_k, A_v, B_k, B_v, q))
    K_tail, V_tail = widen(K_tail), widen(V_tail)
    idx = np.asarray(idx)
    H_q, d_h = q.shape
    H_kv = idx.shape[0]
    n_rep = H_q // H_kv
    scale = default_scale(d_h) if scale is None else scale
    out = np.empty((H_q, d_h), np.float64)
    for g in range(H_kv):
        cols = slice(g * d_h, (g + 1) * d_h)
        K_all = np.concatenate([A_k[idx[g]] @ B_k[:, cols], K_tail[g]], axis=0)   # Eq. 3 rows, then the tail
        V_all = np.concatenate([A_v[idx[g]] @ B_v[:, cols], V_tail[g]], axis=0)
        for h in range(g * n_rep, (g + 1) * n_rep):
            z = scale * (K_all @ q[h])
            wgt = np.exp(z - z.max())
            out[h] = (wgt / wgt.sum()) @ V_all
    return out


def sr_decode_tail(A_k, A_v, B_k, B_v, q, H_kv, k, K_tail, V_tail, scale=None):
    """SR step over a context whose most recent T tokens are still uncompressed (Sec. 4, "Implementation
    details": newly generated tokens are kept uncompressed; Sec. 7, long-generation scenario).

    The L compressed tokens are scored, pooled and selected exactly as in sr_decode (steps 1-4); attention then
    runs over the selected rows and the tail (gather_attend_tail).  Returns (out[H_q][d_h], idx[H_kv][k]).
    """
    q64 = widen(q)
    scale = default_scale(q64.shape[1]) if scale is None else scale
    S32 = pooled_scores(A_k, B_k, q, H_kv, scale).astype(np.float32)   # the selection is taken in fp32 (step 4)
    idx = np.stack([select(S32[g], k) for g in range(H_kv)]).astype(np.int32)
    return gather_attend_tail(A_k, A_v, B_k, B_v, q, idx, K_tail, V_tail, scale), idx


def landmarks(K_rope, c, o=0):
    """Landmark construction at prefill (App. B.1, Alg. 1).  K_rope [H_kv][L][d_h] -> (Lm [H_kv][n_c][d_h],
    m [H_kv][n_c], outliers [H_kv][o]).

    Chunk j holds tokens j c .. min(j c + c, L) - 1; its landmark is the mean of its keys (a shorter last chunk
    is averaged over the tokens it has); m is the smallest cosine between a key of the chunk and the landmark
    (0 when either vector is zero); the outliers of a head are its o chunks with the smallest m, i.e.
    ArgTopK(-m, o), decided on the fp32 values of -m with ties towards the smaller chunk index (the order of the
    top-k step of Alg. 2), returned ascending.
    """
    K = widen(K_rope)
    H_kv, L, d_h = K.shape
    n_c = -(-L // c)
    Lm = np.empty((H_kv, n_c, d_h), np.float64)
    m = np.empty((H_kv, n_c), np.float64)
    for g in range(H_kv):
        for j in range(n_c):
            chunk = K[g, j * c:min(j * c + c, L)]
            mean = chunk.sum(axis=0) / chunk.shape[0]
            Lm[g, j] = mean
            worst = np.inf
            for x in chunk:
                den = np.sqrt(x @ x) * np.sqrt(mean @ mean)
                worst = min(worst, (x @ mean) / den if den > 0.0 else 0.0)
            m[g, j] = worst
    if o > 0:
        outliers = np.stack([select((-m[g]).astype(np.float32), o) for g in range(H_kv)]).astype(np.int32)
    else:
        outliers = np.zeros((H_kv, 0), np.int32)
    return Lm, m, outliers


def chunk_scores(Lm, q, scale=None):
    """Alg. 2, scoring and pooling: P[h][j] = scale <q_h, Lm[rho(h)][j]>, S[g][j] = max over the heads of g."""
    Lm, q = widen(Lm), widen(q)
    H_kv, n_c, d_h = Lm.shape
    H_q = q.shape[0]
    n_rep = H_q // H_kv
    scale = default_scale(d_h) if scale is None else scale
    S = np.empty((H_kv, n_c), np.float64)
    for g in range(H_kv):
        P = scale * (Lm[g] @ q[g * n_rep:(g + 1) * n_rep].T)   # [n_c][n_rep]
        S[g] = P.max(axis=1)
    return S


def chunk_budget(k, c, n_c):
    """k_ch = ceil(k / c) (Alg. 2), never more than there are chunks."""
    return min(-(-k // c), n_c)


def expand_chunks(chunks, outliers, c, L):
    """Union of the selected chunks with the static outliers (Alg. 2), expanded to token rows, ascending."""
    rows = []
    for j in sorted(set(int(x) for x in chunks) | set(int(x) for x in outliers)):
        rows.extend(range(j * c, min(j * c + c, L)))
    return np.asarray(rows, np.int32)


def select_rows_by_landmarks(Lm, outliers, q, k, c, L, scale=None):
    """Alg. 2 for one layer and decode step: per KV head the token rows to reconstruct (list of ascending int32
    arrays of different lengths), and the pooled chunk scores as the fp32 values the top-k saw."""
    S32 = chunk_scores(Lm, q, scale).astype(np.float32)
    H_kv, n_c = S32.shape
    k_ch = chunk_budget(k, c, n_c)
    rows = [expand_chunks(select(S32[g], k_ch), outliers[g], c, L) for g in range(H_kv)]
    return rows, S32


def rope(X, positions, theta):
    """Rotary position embedding of rows X [n][d_h] at the given integer positions (the reconstructed keys are
    pre-RoPE, Sec. 4 and App. C.6 "Setup"; the rotation is re-applied to the rows that are reconstructed).
    Convention of the Llama / Qwen2 reference implementations: channel j < d_h/2 is paired with channel j + d_h/2,
    the pair is rotated by the angle position * theta^(-2j/d_h):
      out[j] = x[j] cos - x[j + d_h/2] sin,   out[j + d_h/2] = x[j + d_h/2] cos + x[j] sin."""
    X = widen(X)
    n, d_h = X.shape
    half = d_h // 2
    assert d_h == 2 * half
    inv_freq = float(theta) ** (-np.arange(half, dtype=np.float64) * 2.0 / d_h)
    ang = np.asarray(positions, np.float64)[:, None] * inv_freq[None, :]
    cs, sn = np.cos(ang), np.sin(ang)
    out = np.empty_like(X)
    out[:, :half] = X[:, :half] * cs - X[:, half:] * sn
    out[:, half:] = X[:, half:] * cs + X[:, :half] * sn
    return out


def gather_attend_rows(A_k, A_v, B_k, B_v, q, rows, scale=None, rope_theta=None, K_tail=None, V_tail=None):
    """Steps 5-6 (Eq. 3 and softmax attention) for per-head row lists of different lengths: out[H_q][d_h].
    With rope_theta, every reconstructed key row is rotated to its position (= its row number) before it meets
    the (already rotated) query; values are not rotated.  With K_tail, V_tail [H_kv][T][d_h], the uncompressed
    most recent tokens (Sec. 4: newly generated tokens are kept uncompressed; their keys are stored as the model
    produced them, rotated) join the same softmax.  Written out in numpy."""
    A_k, A_v, B_k, B_v, q = map(widen, (A_k, A_v, B_k, B_v, q))
    if K_tail is not None:
        K_tail, V_tail = widen(K_tail), widen(V_tail)
    H_q, d_h = q.shape
    H_kv = len(rows)
    n_rep = H_q // H_kv
    scale = default_scale(d_h) if scale is None else scale
    out = np.empty((H_q, d_h), np.float64)
    for g in range(H_kv):
        cols = slice(g * d_h, (g + 1) * d_h)
        K_sel = A_k[rows[g]] @ B_k[:, cols]
        if rope_theta is not None:
            K_sel = rope(K_sel, rows[g], rope_theta)
        V_sel = A_v[rows[g]] @ B_v[:, cols]
        if K_tail is not None:
            K_sel = np.concatenate([K_sel, K_tail[g]], axis=0)
            V_sel = np.concatenate([V_sel, V_tail[g]], axis=0)
        for h in range(g * n_rep, (g + 1) * n_rep):
            z = scale * (K_sel @ q[h])
            wgt = np.exp(z - z.max())
            out[h] = (wgt / wgt.sum()) @ V_sel
    return out


def sr_decode_landmark(A_k, A_v, B_k, B_v, q, Lm, outliers, k, c, scale=None, rope_theta=None, K_tail=None,
                       V_tail=None):
    """SR step with the paper's own selector (App. B.1): chunks are scored against their landmarks, the top
    ceil(k / c) chunks per KV head plus the static outliers are expanded to rows, those rows are reconstructed
    (Eq. 3), with rope_theta rotated to their positions, and attended over together with the uncompressed tail
    if there is one.  Returns (out[H_q][d_h], rows, S32[H_kv][n_c])."""
    L = widen(A_k).shape[0]
    rows, S32 = select_rows_by_landmarks(Lm, outliers, q, k, c, L, scale)
    return gather_attend_rows(A_k, A_v, B_k, B_v, q, rows, scale, rope_theta, K_tail, V_tail), rows, S32


def factorize(X_cat, r):
    """Eq. 1: (A[L][r], B[r][n], sigma[n]) with A = U Sigma, B = V_r^T."""
    X = widen(X_cat)
    L, n = X.shape
    A = np.empty((L, r), np.float64)
    B = np.empty((r, n), np.float64)
    sigma = np.empty((n,), np.float64)
    rc = _load().oracle_factorize(_dp(X), L, n, r, _dp(A), _dp(B), _dp(sigma))
    if rc != 0:
        raise ValueError(f"oracle_factorize failed ({rc})")
    return A, B, sigma


_RATIO = {"C_K": 0, "C_V": 1, "xKV": 2, "xK-SR-gpu": 3, "xK-SR-total": 4, "xKV-SR": 5}


def compression_ratio(which, N, W, d, L, r_k, r_v=0, c=0):
    """Closed-form compression ratios of App. C.6."""
    return float(_load().oracle_compression_ratio(_RATIO[which], N, W, d, float(L), r_k, r_v, c))


# ---------------------------------------------------------------------------------------------
# Round-to-nearest quantisation of the token basis A (App. "Integrate with Quantization": a plain RTN
# quantiser applied to the compressed cache; 4 bits -> 25.6x, 3 bits -> 32x on top of xKV's 8x).  The paper
# gives no format.  The reading taken here is the one its two ratios fix: 25.6 / 8 = 16 / 5 and 32 / 8 = 16 / 4,
# i.e. one extra bit per element of side information = two 16-bit numbers per group of 32 elements
# (asymmetric quantisation: a step and an offset per group).  Groups are 32 consecutive ranks of one token's
# row.  Where floating point decides an integer (the code), the arithmetic is fp32, the same on both sides.
# ---------------------------------------------------------------------------------------------
Q_GROUP = 32


def _bf16_rne(x32: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bf16 (ties to even), returned as fp32.  Finite inputs."""
    u = np.ascontiguousarray(x32, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def quantize_rows(X, bits=4):
    """RTN quantisation of X [rows][r] (r a multiple of 32) in groups of 32 along a row.

    Per group: lo = min, step = bf16((max - lo) / (2^bits - 1)) (1 if that is 0), inv = 1 / step,
    code = clip(rint((x - lo) * inv), 0, 2^bits - 1); every operation is a single fp32 operation.  lo is stored as
    bf16 (exact when X is bf16).  Returns codes uint8 [rows][r], step and lo as fp32 [rows][r / 32]."""
    X = np.asarray(X)
    if X.dtype == np.uint16:
        X = (X.astype(np.uint32) << 16).view(np.float32)
    X = np.ascontiguousarray(X, np.float32)
    rows, r = X.shape
    assert r % Q_GROUP == 0 and 2 <= bits <= 8
    g = X.reshape(rows, r // Q_GROUP, Q_GROUP)
    qmax = np.float32((1 << bits) - 1)
    lo = _bf16_rne(g.min(axis=2))
    step = _bf16_rne((g.max(axis=2) - lo) / qmax)
    step = np.where(step > 0, step, np.float32(1.0)).astype(np.float32)
    inv = (np.float32(1.0) / step).astype(np.float32)
    t = ((g - lo[:, :, None]).astype(np.float32) * inv[:, :, None]).astype(np.float32)
    codes = np.clip(np.rint(t), 0, qmax).astype(np.uint8)
    return codes.reshape(rows, r), step, lo


def dequantize_rows(codes, step, lo):
    """x^ = step * code + lo in float64: the values every later stage of the path sees."""
    rows, r = codes.shape
    c = codes.reshape(rows, r // Q_GROUP, Q_GROUP).astype(np.float64)
    return (c * step.astype(np.float64)[:, :, None] + lo.astype(np.float64)[:, :, None]).reshape(rows, r)


def pack_q4(codes, step, lo):
    """Byte layout of a 4-bit row as the library stores it: r/8 little-endian 32-bit words of codes -- word j holds
    ranks 8j .. 8j+7, rank 8j + 2i in bits [4i, 4i+4) and rank 8j + 2i + 1 in bits [16 + 4i, 16 + 4i + 4), i = 0..3,
    so that two adjacent ranks sit 16 bits apart like a packed pair of 16-bit numbers -- then per group (step, lo) as
    two bf16 numbers: 5r/8 bytes, then zero bytes up to the next multiple of 16 (none when r is a multiple of 128)."""
    rows, r = codes.shape
    assert codes.max(initial=0) < 16
    c = codes.reshape(rows, r // 8, 4, 2).astype(np.uint32)          # [word][i][even / odd rank]
    sh = (4 * np.arange(4, dtype=np.uint32))[None, None, :]
    words = ((c[:, :, :, 0] << sh) | (c[:, :, :, 1] << (sh + 16))).sum(axis=2).astype('<u4')
    nib = np.ascontiguousarray(words).view(np.uint8).reshape(rows, r // 2)
    par = np.empty((rows, r // Q_GROUP, 2), np.uint16)
    par[:, :, 0] = (np.ascontiguousarray(step, np.float32).view(np.uint32) >> 16).astype(np.uint16)
    par[:, :, 1] = (np.ascontiguousarray(lo, np.float32).view(np.uint32) >> 16).astype(np.uint16)
    row = np.concatenate([nib, par.reshape(rows, -1).view(np.uint8)], axis=1)
    pad = (-row.shape[1]) % 16
    return np.concatenate([row, np.zeros((rows, pad), np.uint8)], axis=1) if pad else row


def unpack_q4(packed, r):
    """Inverse of pack_q4: (codes, step, lo)."""
    packed = np.ascontiguousarray(packed, np.uint8)
    rows = packed.shape[0]
    words = np.ascontiguousarray(packed[:, :r // 2]).view('<u4').reshape(rows, r // 8)
    codes = np.empty((rows, r // 8, 4, 2), np.uint8)
    for i in range(4):
        codes[:, :, i, 0] = (words >> (4 * i)) & 15
        codes[:, :, i, 1] = (words >> (16 + 4 * i)) & 15
    codes = codes.reshape(rows, r)
    par = np.ascontiguousarray(packed[:, r // 2:r // 2 + r // 8]).view(np.uint16).reshape(rows, r // Q_GROUP, 2)
    step = (par[:, :, 0].astype(np.uint32) << 16).view(np.float32)
    lo = (par[:, :, 1].astype(np.uint32) << 16).view(np.float32)
    return codes, np.ascontiguousarray(step), np.ascontiguousarray(lo)


def pack_q3(codes, step, lo):
    """Byte layout of a 3-bit row as the library stores it: one 16-byte piece per group of 32 ranks.  The first 12
    bytes are 96 bits of codes, read as one little-endian number: unit u (ranks 8u .. 8u+7 of the group) occupies bits
    [24u, 24u + 24); inside a unit rank 8u + 2i sits at bits [3i, 3i + 3) and rank 8u + 2i + 1 at bits
    [12 + 3i, 12 + 3i + 3), i = 0..3.  The last 4 bytes are (step, lo) as two bf16 numbers.  r/2 bytes per row."""
    rows, r = codes.shape
    assert codes.max(initial=0) < 8
    n_g = r // Q_GROUP
    c = codes.reshape(rows, n_g, 4, 4, 2).astype(object)              # [group][unit][i][even / odd rank]
    big = np.zeros((rows, n_g), dtype=object)
    for u in range(4):
        for i in range(4):
            big = big + (c[:, :, u, i, 0] << (24 * u + 3 * i)) + (c[:, :, u, i, 1] << (24 * u + 12 + 3 * i))
    out = np.zeros((rows, n_g, 16), np.uint8)
    for byte in range(12):
        out[:, :, byte] = ((big >> (8 * byte)) & 0xFF).astype(np.uint8)
    par = np.empty((rows, n_g, 2), np.uint16)
    par[:, :, 0] = (np.ascontiguousarray(step, np.float32).view(np.uint32) >> 16).astype(np.uint16)
    par[:, :, 1] = (np.ascontiguousarray(lo, np.float32).view(np.uint32) >> 16).astype(np.uint16)
    out[:, :, 12:16] = par.reshape(rows, n_g, 2).view(np.uint8).reshape(rows, n_g, 4)
    return out.reshape(rows, n_g * 16)


def unpack_q3(packed, r):
    """Inverse of pack_q3: (codes, step, lo)."""
    packed = np.ascontiguousarray(packed, np.uint8)
    rows = packed.shape[0]
    n_g = r // Q_GROUP
    pieces = packed.reshape(rows, n_g, 16)
    big = np.zeros((rows, n_g), dtype=object)
    for byte in range(12):
        big = big + (pieces[:, :, byte].astype(object) << (8 * byte))
    codes = np.empty((rows, n_g, 4, 4, 2), np.uint8)
    for u in range(4):
        for i in range(4):
            codes[:, :, u, i, 0] = ((big >> (24 * u + 3 * i)) & 7).astype(np.uint8)
            codes[:, :, u, i, 1] = ((big >> (24 * u + 12 + 3 * i)) & 7).astype(np.uint8)
    par = np.ascontiguousarray(pieces[:, :, 12:16]).view(np.uint16).reshape(rows, n_g, 2)
    step = (par[:, :, 0].astype(np.uint32) << 16).view(np.float32)
    lo = (par[:, :, 1].astype(np.uint32) << 16).view(np.float32)
    return codes.reshape(rows, r), np.ascontiguousarray(step), np.ascontiguousarray(lo)


def quantized_bits_per_element(bits):
    """Storage per element of a quantised row: the code plus two 16-bit numbers per group of 32."""
    return bits + 2 * 16 / Q_GROUP
