"""Pins for the CPU oracle: it is checked here against things that are not itself.

Every check uses numpy / scipy / torch library routines, brute force, closed forms or
values the paper prints; none re-types an oracle loop.  A dropped term, a wrong sign
or index, a transposed operand or a wrong head mapping in the oracle fails at least
one of these.
"""
import os

import numpy as np
import pytest
import scipy.special

import oracle
from paper_2503_18893_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_case(seed=0, L=96, H_kv=2, H_q=6, d_h=8, r_k=5, r_v=7, batch=1, G=1):
    rng = np.random.default_rng(seed)
    d = H_kv * d_h
    return dict(
        A_k=rng.standard_normal((L, r_k)), A_v=rng.standard_normal((L, r_v)),
        B_k=rng.standard_normal((r_k, d)), B_v=rng.standard_normal((r_v, d)),
        q=rng.standard_normal((H_q, d_h)), H_kv=H_kv, H_q=H_q, d_h=d_h, L=L, r_k=r_k, r_v=r_v)


def np_softmax_attention(K, V, q, H_kv, scale):
    """Textbook attention with numpy/scipy: K,V [L][H_kv*d_h], q [H_q][d_h]."""
    H_q, d_h = q.shape
    n_rep = H_q // H_kv
    out = np.empty((H_q, d_h))
    for h in range(H_q):
        g = h // n_rep
        Kg, Vg = K[:, g * d_h:(g + 1) * d_h], V[:, g * d_h:(g + 1) * d_h]
        w = scipy.special.softmax(scale * (Kg @ q[h]))
        out[h] = w @ Vg
    return out


def brute_topk(row_f32, k):
    """k largest under (fp32 value desc with -0 < +0, index asc), by a full lexsort."""
    row = np.asarray(row_f32, dtype=np.float32)
    bits = row.view(np.uint32).astype(np.uint64)
    key = np.where(bits & 0x80000000, (~bits) & 0xFFFFFFFF, bits | 0x80000000)
    order = np.lexsort((np.arange(row.size), -key.astype(np.int64)))
    return np.sort(order[:k]).astype(np.int32)


# ----------------------------------------------------------------- steps 1-3
def test_scores_equal_query_dot_reconstructed_keys():
    """s[h,t] = scale * q_h . (A^K B^K_l)[t, head rho(h)]  (Eq. 3 + associativity)."""
    c = small_case(1)
    scale = 0.37
    p = oracle.project(c["B_k"], c["q"], c["H_kv"])
    s = oracle.scores(c["A_k"], p, scale)
    Khat = c["A_k"] @ c["B_k"]                       # numpy matmul, not the oracle
    n_rep = c["H_q"] // c["H_kv"]
    for h in range(c["H_q"]):
        g = h // n_rep
        ref = scale * Khat[:, g * c["d_h"]:(g + 1) * c["d_h"]] @ c["q"][h]
        np.testing.assert_allclose(s[h], ref, rtol=1e-12, atol=1e-12)


def test_project_uses_the_right_head_block():
    """A query of head h must see only columns rho(h)*d_h.. of B: zeroing other blocks changes nothing."""
    c = small_case(2, H_kv=3, H_q=6)
    p = oracle.project(c["B_k"], c["q"], c["H_kv"])
    for h in range(c["H_q"]):
        g = h // 2
        Bz = np.zeros_like(c["B_k"])
        Bz[:, g * c["d_h"]:(g + 1) * c["d_h"]] = c["B_k"][:, g * c["d_h"]:(g + 1) * c["d_h"]]
        np.testing.assert_allclose(oracle.project(Bz, c["q"], c["H_kv"])[h], p[h], rtol=0, atol=0)
        np.testing.assert_allclose(p[h], c["B_k"][:, g * c["d_h"]:(g + 1) * c["d_h"]] @ c["q"][h], rtol=1e-13)


def test_pool_is_max_over_the_group():
    rng = np.random.default_rng(3)
    s = rng.standard_normal((12, 50))
    S = oracle.pool(s, 4)
    np.testing.assert_array_equal(S, s.reshape(4, 3, 50).max(axis=1))
    np.testing.assert_array_equal(oracle.pool(s, 12), s)          # H_q == H_kv: no pooling


# ----------------------------------------------------------------- step 4
@pytest.mark.parametrize("case", ["random", "ties", "all_equal", "signed_zero", "denormal", "sorted",
                                  "reverse", "negative"])
def test_select_matches_brute_force(case):
    rng = np.random.default_rng(4)
    L = 257
    if case == "random":
        row = rng.standard_normal(L)
    elif case == "ties":
        row = rng.integers(0, 5, L).astype(np.float64)
    elif case == "all_equal":
        row = np.full(L, 1.25)
    elif case == "signed_zero":
        row = np.where(rng.random(L) < 0.5, 0.0, -0.0)
    elif case == "denormal":
        row = rng.standard_normal(L) * 1e-42
    elif case == "sorted":
        row = np.arange(L, dtype=np.float64)
    elif case == "reverse":
        row = -np.arange(L, dtype=np.float64)
    else:
        row = -np.abs(rng.standard_normal(L)) - 1.0
    row = row.astype(np.float32)
    for k in (1, 2, 31, 64, L - 1, L):
        got = oracle.select(row, k)
        np.testing.assert_array_equal(got, brute_topk(row, k))
        assert len(set(got.tolist())) == k


def test_select_order_invariants():
    """min selected >= max unselected; ties broken towards the smaller index; -0.0 < +0.0."""
    row = np.array([0.5, 2.0, 2.0, -1.0, 2.0, 0.0, -0.0, 3.0], np.float32)
    np.testing.assert_array_equal(oracle.select(row, 1), [7])
    np.testing.assert_array_equal(oracle.select(row, 3), [1, 2, 7])      # of three 2.0s the first two
    np.testing.assert_array_equal(oracle.select(row, 6), [0, 1, 2, 4, 5, 7])  # +0.0 (idx 5) beats -0.0 (idx 6)
    rng = np.random.default_rng(5)
    row = rng.standard_normal(1000).astype(np.float32)
    sel = oracle.select(row, 100)
    mask = np.zeros(1000, bool)
    mask[sel] = True
    assert row[mask].min() >= row[~mask].max()
    # permutation equivariance (distinct values): selecting on a permuted row selects the permuted set
    perm = rng.permutation(1000)
    sel_p = oracle.select(row[perm], 100)
    np.testing.assert_array_equal(np.sort(perm[sel_p]), sel)


# ----------------------------------------------------------------- steps 5-6
def test_gather_attend_matches_sliced_dense_reconstruction():
    """Eq. 3: A[S] B_{l,g} are rows S of (A B_l)[:, head g]; then textbook softmax."""
    c = small_case(6)
    rng = np.random.default_rng(6)
    k = 17
    idx = np.stack([rng.choice(c["L"], k, replace=False) for _ in range(c["H_kv"])]).astype(np.int32)
    scale = 0.9
    got = oracle.gather_attend(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], idx, scale)
    Khat, Vhat = c["A_k"] @ c["B_k"], c["A_v"] @ c["B_v"]
    n_rep, d_h = c["H_q"] // c["H_kv"], c["d_h"]
    for h in range(c["H_q"]):
        g = h // n_rep
        Ks, Vs = Khat[idx[g], g * d_h:(g + 1) * d_h], Vhat[idx[g], g * d_h:(g + 1) * d_h]
        w = scipy.special.softmax(scale * Ks @ c["q"][h])
        np.testing.assert_allclose(got[h], w @ Vs, rtol=1e-11, atol=1e-12)
        # convex combination: every output coordinate inside the hull of the selected V rows
        assert np.all(got[h] <= Vs.max(axis=0) + 1e-12) and np.all(got[h] >= Vs.min(axis=0) - 1e-12)


def test_gather_attend_k1_returns_the_single_value_row():
    c = small_case(7)
    idx = np.array([[5], [9]], np.int32)
    got = oracle.gather_attend(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], idx)
    Vhat = c["A_v"] @ c["B_v"]
    n_rep, d_h = c["H_q"] // c["H_kv"], c["d_h"]
    for h in range(c["H_q"]):
        g = h // n_rep
        np.testing.assert_allclose(got[h], Vhat[idx[g, 0], g * d_h:(g + 1) * d_h], rtol=1e-12, atol=1e-13)


def test_gather_attend_invariant_to_order_of_indices():
    c = small_case(8)
    rng = np.random.default_rng(8)
    idx = np.stack([rng.choice(c["L"], 20, replace=False) for _ in range(c["H_kv"])]).astype(np.int32)
    a = oracle.gather_attend(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], idx)
    b = oracle.gather_attend(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], np.sort(idx, axis=1))
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------- dense and the k = L identity
def test_dense_matches_library_attention():
    import torch
    c = small_case(9, L=200)
    rng = np.random.default_rng(9)
    d = c["H_kv"] * c["d_h"]
    K, V = rng.standard_normal((c["L"], d)), rng.standard_normal((c["L"], d))
    scale = 1.0 / np.sqrt(c["d_h"])
    got = oracle.dense(K, V, c["q"], c["H_kv"])                   # default scale = 1/sqrt(d_h)
    np.testing.assert_allclose(got, np_softmax_attention(K, V, c["q"], c["H_kv"], scale), rtol=1e-11, atol=1e-13)
    # second opinion: torch SDPA in fp64 with enable_gqa-style head repetition done by hand
    n_rep = c["H_q"] // c["H_kv"]
    Kt = torch.from_numpy(K).view(c["L"], c["H_kv"], c["d_h"]).permute(1, 0, 2).repeat_interleave(n_rep, 0)
    Vt = torch.from_numpy(V).view(c["L"], c["H_kv"], c["d_h"]).permute(1, 0, 2).repeat_interleave(n_rep, 0)
    qt = torch.from_numpy(c["q"]).unsqueeze(1)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt).squeeze(1).numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_dense_invariant_to_logit_shift_and_peaked_limit():
    c = small_case(10)
    rng = np.random.default_rng(10)
    d = c["H_kv"] * c["d_h"]
    K, V = rng.standard_normal((c["L"], d)), rng.standard_normal((c["L"], d))
    # a huge scale makes softmax an argmax: output = the V row of the best-matching key
    got = oracle.dense(K, V, c["q"], c["H_kv"], scale=1e4)
    n_rep, d_h = c["H_q"] // c["H_kv"], c["d_h"]
    for h in range(c["H_q"]):
        g = h // n_rep
        t = np.argmax(K[:, g * d_h:(g + 1) * d_h] @ c["q"][h])
        np.testing.assert_allclose(got[h], V[t, g * d_h:(g + 1) * d_h], rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("H_kv,H_q", [(2, 6), (3, 3), (1, 4)])
def test_sr_with_k_equal_L_is_dense_attention_on_reconstruction(H_kv, H_q):
    """Dense reconstruction recovers the low-rank approximation exactly (Sec. 3.2), so selecting
    every token must give textbook attention on K = A^K B^K_l, V = A^V B^V_l."""
    c = small_case(11, H_kv=H_kv, H_q=H_q, L=80)
    out, idx, S32 = oracle.sr_decode(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], H_kv, k=c["L"])
    K, V = c["A_k"] @ c["B_k"], c["A_v"] @ c["B_v"]
    ref = np_softmax_attention(K, V, c["q"], H_kv, 1.0 / np.sqrt(c["d_h"]))
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(out, oracle.dense(K, V, c["q"], H_kv), rtol=1e-11, atol=1e-13)
    np.testing.assert_array_equal(idx, np.tile(np.arange(c["L"], dtype=np.int32), (H_kv, 1)))


def test_sr_decode_chain_matches_numpy_brute_force():
    """Whole step on a tiny input against an independent numpy pipeline."""
    c = small_case(12, L=120, H_kv=2, H_q=4)
    k = 9
    scale = 1.0 / np.sqrt(c["d_h"])
    out, idx, S32 = oracle.sr_decode(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], c["H_kv"], k)
    Khat, Vhat = c["A_k"] @ c["B_k"], c["A_v"] @ c["B_v"]
    d_h, n_rep = c["d_h"], 2
    for g in range(c["H_kv"]):
        per_head = np.stack([scale * Khat[:, g * d_h:(g + 1) * d_h] @ c["q"][h] for h in (2 * g, 2 * g + 1)])
        S = per_head.max(axis=0).astype(np.float32)
        np.testing.assert_allclose(S32[g], S, rtol=1e-6)
        sel = brute_topk(S32[g], k)
        np.testing.assert_array_equal(idx[g], sel)
        for h in (2 * g, 2 * g + 1):
            w = scipy.special.softmax(scale * Khat[sel, g * d_h:(g + 1) * d_h] @ c["q"][h])
            np.testing.assert_allclose(out[h], w @ Vhat[sel, g * d_h:(g + 1) * d_h], rtol=1e-10, atol=1e-12)


def _tail(c, T, seed):
    rng = np.random.default_rng(seed)
    shape = (c["H_kv"], T, c["d_h"])
    return rng.standard_normal(shape) * 0.5, rng.standard_normal(shape)


def test_sr_tail_with_empty_tail_is_plain_sr():
    """No uncompressed tokens: the tail variant must reduce to the SR step itself."""
    c = small_case(14, L=150, H_kv=2, H_q=6)
    K_t, V_t = _tail(c, 0, 1)
    out_t, idx_t = oracle.sr_decode_tail(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], c["H_kv"], 13, K_t, V_t)
    out, idx, _ = oracle.sr_decode(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], c["H_kv"], 13)
    np.testing.assert_array_equal(idx_t, idx)
    np.testing.assert_allclose(out_t, out, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("H_kv,H_q,T", [(2, 6, 7), (3, 3, 1), (1, 4, 40)])
def test_sr_tail_with_k_equal_L_is_dense_attention_on_the_whole_context(H_kv, H_q, T):
    """Selecting every compressed token and keeping T recent tokens uncompressed (Sec. 4, implementation details)
    is textbook attention over the L reconstructed rows followed by the T exact rows."""
    c = small_case(15, H_kv=H_kv, H_q=H_q, L=70)
    K_t, V_t = _tail(c, T, 2)
    out, idx = oracle.sr_decode_tail(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], H_kv, c["L"], K_t, V_t)
    as_rows = lambda X: X.transpose(1, 0, 2).reshape(T, H_kv * c["d_h"])       # [H_kv][T][d_h] -> [T][d]
    K = np.concatenate([c["A_k"] @ c["B_k"], as_rows(K_t)], axis=0)
    V = np.concatenate([c["A_v"] @ c["B_v"], as_rows(V_t)], axis=0)
    ref = np_softmax_attention(K, V, c["q"], H_kv, 1.0 / np.sqrt(c["d_h"]))
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(out, oracle.dense(K, V, c["q"], H_kv), rtol=1e-11, atol=1e-13)


def test_sr_tail_selection_ignores_the_tail_and_a_dominant_tail_token_wins():
    """The tail takes no part in the selection; a tail key aligned with the query at a huge scale takes all the
    weight, so the output is that token's value row."""
    c = small_case(16, L=90, H_kv=1, H_q=2)
    K_t, V_t = _tail(c, 5, 3)
    K_t[0, 3] = 50.0 * (c["q"][0] + c["q"][1])
    out, idx = oracle.sr_decode_tail(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], 1, 11, K_t, V_t, scale=10.0)
    _, idx_plain, _ = oracle.sr_decode(c["A_k"], c["A_v"], c["B_k"], c["B_v"], c["q"], 1, 11, 10.0)
    np.testing.assert_array_equal(idx, idx_plain)
    for h in range(2):
        np.testing.assert_allclose(out[h], V_t[0, 3], rtol=1e-9, atol=1e-12)


def test_sr_tiny_config_properties():
    """The benchmark's tiny configuration: selected tokens dominate, k distinct indices per head."""
    w = synth.TINY
    case = synth.make_case(w, seed=0)
    out, idx, S32 = oracle.sr_decode(case["A_k"][0], case["A_v"][0], case["B_k"][0, 0], case["B_v"][0, 0],
                                     case["q"][0, 0], w.H_kv, w.k)
    assert out.shape == (w.H_q, w.d_h) and idx.shape == (w.H_kv, w.k)
    for g in range(w.H_kv):
        assert len(set(idx[g].tolist())) == w.k
        mask = np.zeros(w.L, bool)
        mask[idx[g]] = True
        assert S32[g][mask].min() >= S32[g][~mask].max()


# ----------------------------------------------------------------- reconstruction / factorization
def test_reconstruct_matches_matmul():
    rng = np.random.default_rng(13)
    A, B = rng.standard_normal((40, 6)), rng.standard_normal((6, 10))
    np.testing.assert_allclose(oracle.reconstruct(A, B), A @ B, rtol=1e-13, atol=1e-13)


def test_factorize_reproduces_exactly_rank_r_input():
    rng = np.random.default_rng(14)
    L, G, d, r = 150, 3, 8, 6
    X = rng.standard_normal((L, r)) @ rng.standard_normal((r, G * d))
    A, B, sigma = oracle.factorize(X, r)
    assert np.abs(X - A @ B).max() <= 1e-11 * np.abs(X).max()
    np.testing.assert_allclose(B @ B.T, np.eye(r), atol=1e-12)          # B = V_r^T has orthonormal rows
    gram = A.T @ A                                                        # A = U Sigma: A^T A = Sigma^2, descending
    np.testing.assert_allclose(gram, np.diag(np.diag(gram)), atol=1e-9 * gram.max())
    assert np.all(np.diff(np.diag(gram)) <= 1e-9 * gram.max())
    # per-layer blocks reconstruct each layer's cache (Eq. 1)
    for l in range(G):
        np.testing.assert_allclose(A @ B[:, l * d:(l + 1) * d], X[:, l * d:(l + 1) * d], atol=1e-10)


def test_factorize_is_the_optimal_truncation():
    """Eckart-Young: squared Frobenius residual = sum of discarded sigma^2; sigma matches LAPACK."""
    rng = np.random.default_rng(15)
    L, n, r = 90, 20, 7
    X = rng.standard_normal((L, n)) * (np.arange(1, n + 1) ** -0.7)[None, :]
    A, B, sigma = oracle.factorize(X, r)
    sv = np.linalg.svd(X, compute_uv=False)
    np.testing.assert_allclose(sigma, sv, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(np.sum((X - A @ B) ** 2), np.sum(sv[r:] ** 2), rtol=1e-9)


# ----------------------------------------------------------------- printed numbers
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "compression_ratios.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append(line.split("|")[0].split())
    return rows


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: f"{r[0]}-W{r[2]}-r{r[5]}")
def test_compression_ratios_match_the_papers_tables(row):
    which, N, W, d, L, r_k, r_v, c, printed, tol = row
    got = oracle.compression_ratio(which, int(N), int(W), int(d), float(L), int(r_k), int(r_v), int(c))
    assert abs(got - float(printed)) <= float(tol), (got, printed)


def test_compression_ratio_special_forms():
    """With C_K = C_V = C and c = 8 the ratios reduce to 2/(1/C + 1/8) and 2/(2/C + 1/8) (App. C.6)."""
    C = oracle.compression_ratio("C_K", 32, 4, 1024, 65536, 512)
    assert abs(oracle.compression_ratio("C_V", 32, 4, 1024, 65536, 512, 512) - C) < 1e-12
    assert abs(oracle.compression_ratio("xK-SR-gpu", 32, 4, 1024, 65536, 512, 0, 8) - 2 / (1 / C + 1 / 8)) < 1e-12
    assert abs(oracle.compression_ratio("xKV-SR", 32, 4, 1024, 65536, 512, 512, 8) - 2 / (2 / C + 1 / 8)) < 1e-12
    # memory model: factors hold n_win*L*r + N*r*d scalars against N*L*d
    assert abs(C - (32 * 65536 * 1024) / (8 * 65536 * 512 + 32 * 512 * 1024)) < 1e-12


# ----------------------------------------------------------------- generator sanity (not the method)
def test_generator_recipe():
    w = synth.TINY
    case = synth.make_case(w, seed=3)
    B = case["B_k"][0, 1].astype(np.float64)
    sigma = np.arange(1, w.r_k + 1) ** -1.0
    np.testing.assert_allclose(B @ B.T, np.diag(sigma ** 2), atol=1e-6)
    again = synth.make_case(w, seed=3)
    for name in case:
        np.testing.assert_array_equal(case[name], again[name])
    bits = synth.f32_to_bf16_bits(np.array([1.0, 1.00390625, 1.01171875, -2.5], np.float32))
    np.testing.assert_array_equal(bits, [0x3F80, 0x3F80, 0x3F82, 0xC020])   # ties to even


# ----------------------------------------------------------------- landmark selector (App. B.1, Alg. 1-2)
def _rand_keys(rng, H_kv, L, d_h):
    return rng.standard_normal((H_kv, L, d_h))


def test_landmarks_are_chunk_means_with_a_short_last_chunk():
    rng = np.random.default_rng(41)
    K = _rand_keys(rng, 2, 22, 6)
    Lm, m, out = oracle.landmarks(K, 4)
    assert Lm.shape == (2, 6, 6) and m.shape == (2, 6) and out.shape == (2, 0)
    np.testing.assert_allclose(Lm[:, :5], K[:, :20].reshape(2, 5, 4, 6).mean(axis=2), rtol=1e-14)
    np.testing.assert_allclose(Lm[:, 5], K[:, 20:].mean(axis=1), rtol=1e-14)      # two tokens, divided by two


def test_chunks_of_one_token_are_their_own_landmarks():
    rng = np.random.default_rng(42)
    K = _rand_keys(rng, 3, 9, 5)
    Lm, m, _ = oracle.landmarks(K, 1)
    np.testing.assert_array_equal(Lm, K)
    np.testing.assert_allclose(m, 1.0, rtol=1e-14)


def test_minimum_cosine_has_its_closed_form_and_finds_the_planted_chunks():
    """A chunk of c - 1 copies of e1 and one copy of e2: landmark ((c-1) e1 + e2) / c, cosines (c-1)/s and 1/s with
    s = sqrt((c-1)^2 + 1); homogeneous chunks have cosine 1.  The outliers are exactly the planted chunks."""
    c, n_c, d = 4, 10, 8
    K = np.zeros((1, n_c * c, d))
    K[0, :, 0] = 1.0
    planted = [2, 7]
    for j in planted:
        K[0, j * c + 1] = 0.0
        K[0, j * c + 1, 1] = 1.0
    Lm, m, out = oracle.landmarks(K, c, o=2)
    s = np.sqrt((c - 1) ** 2 + 1.0)
    for j in range(n_c):
        assert abs(m[0, j] - ((1.0 / s) if j in planted else 1.0)) < 1e-14
    assert out[0].tolist() == planted
    np.testing.assert_allclose(Lm[0, 2, :2], [(c - 1) / c, 1 / c], rtol=1e-14)


def test_outlier_ties_go_to_the_smaller_chunk_and_zero_vectors_count_as_cosine_zero():
    K = np.ones((1, 12, 3))
    K[0, 4:8] = 0.0                      # an all-zero chunk: landmark 0, cosine defined as 0
    Lm, m, out = oracle.landmarks(K, 4, o=2)
    np.testing.assert_allclose(m[0], [1.0, 0.0, 1.0], atol=1e-15)
    assert out[0].tolist() == [0, 1]     # chunk 1 (smallest m), then the tie between 0 and 2 goes to 0


def test_landmark_scores_with_unit_chunks_are_the_pooled_scores_of_the_factors():
    """c = 1: scoring chunks against landmarks = scoring tokens against K = A B, which by associativity is what the
    factor path computes (steps 1-3)."""
    rng = np.random.default_rng(43)
    L, r, H_kv, H_q, d_h = 50, 7, 2, 6, 8
    A = rng.standard_normal((L, r))
    B = rng.standard_normal((r, H_kv * d_h))
    q = rng.standard_normal((H_q, d_h))
    K = oracle.reconstruct(A, B).reshape(L, H_kv, d_h).transpose(1, 0, 2)
    S_lm = oracle.chunk_scores(K, q)
    np.testing.assert_allclose(S_lm, oracle.pooled_scores(A, B, q, H_kv), rtol=1e-12, atol=1e-12)
    # and against the definition written out
    n_rep = H_q // H_kv
    for g in range(H_kv):
        ref = np.max(np.stack([K[g] @ q[h] for h in range(g * n_rep, (g + 1) * n_rep)]), axis=0) / np.sqrt(d_h)
        np.testing.assert_allclose(S_lm[g], ref, rtol=1e-13)


def test_chunk_budget_and_expansion():
    assert oracle.chunk_budget(2048, 8, 8192) == 256 and oracle.chunk_budget(10, 4, 100) == 3
    assert oracle.chunk_budget(1000, 8, 20) == 20
    rows = oracle.expand_chunks([5, 1], [1, 3], 4, 22)            # union {1, 3, 5}; chunk 5 has two tokens
    assert rows.tolist() == [4, 5, 6, 7, 12, 13, 14, 15, 20, 21]
    assert oracle.expand_chunks([0], [], 3, 10).tolist() == [0, 1, 2]


def test_selection_by_landmarks_brute_force():
    rng = np.random.default_rng(44)
    H_kv, H_q, L, d_h, c, k, o = 2, 4, 37, 6, 5, 11, 2
    K = _rand_keys(rng, H_kv, L, d_h)
    q = rng.standard_normal((H_q, d_h))
    Lm, m, out = oracle.landmarks(K, c, o)
    rows, S32 = oracle.select_rows_by_landmarks(Lm, out, q, k, c, L)
    n_c, k_ch = 8, 3
    for g in range(H_kv):
        sc = [max(float(Lm[g, j] @ q[h]) for h in (2 * g, 2 * g + 1)) / np.sqrt(d_h) for j in range(n_c)]
        top = sorted(range(n_c), key=lambda j: (-np.float32(sc[j]), j))[:k_ch]
        worst = sorted(range(n_c), key=lambda j: (np.float32(m[g, j]), j))[:o]
        want = sorted(t for j in set(top) | set(worst) for t in range(j * c, min(j * c + c, L)))
        assert rows[g].tolist() == want


def test_landmark_step_with_unit_chunks_equals_the_factor_step():
    """c = 1, no outliers, landmarks = rows of K^ = A^K B^K_l: the paper's selector and the factor-scoring selector
    pick the same tokens, and the outputs agree."""
    rng = np.random.default_rng(45)
    L, r, H_kv, H_q, d_h, k = 60, 6, 2, 4, 8, 9
    A_k, A_v = rng.standard_normal((L, r)), rng.standard_normal((L, r))
    B_k, B_v = rng.standard_normal((r, H_kv * d_h)), rng.standard_normal((r, H_kv * d_h))
    q = rng.standard_normal((H_q, d_h))
    out_f, idx_f, _ = oracle.sr_decode(A_k, A_v, B_k, B_v, q, H_kv, k)
    Lm = oracle.reconstruct(A_k, B_k).reshape(L, H_kv, d_h).transpose(1, 0, 2)
    out_l, rows, _ = oracle.sr_decode_landmark(A_k, A_v, B_k, B_v, q, Lm, np.zeros((H_kv, 0), np.int32), k, 1)
    for g in range(H_kv):
        assert rows[g].tolist() == idx_f[g].tolist()
    np.testing.assert_allclose(out_l, out_f, rtol=1e-11, atol=1e-13)
    # equal-length row lists: the numpy attention equals the C implementation
    np.testing.assert_allclose(oracle.gather_attend_rows(A_k, A_v, B_k, B_v, q, [idx_f[0], idx_f[1]]),
                               oracle.gather_attend(A_k, A_v, B_k, B_v, q, idx_f), rtol=1e-12, atol=1e-14)


def test_landmark_step_with_every_chunk_selected_is_dense_attention():
    rng = np.random.default_rng(46)
    L, r, H_kv, H_q, d_h, c = 45, 5, 1, 3, 4, 8
    A_k, A_v = rng.standard_normal((L, r)), rng.standard_normal((L, r))
    B_k, B_v = rng.standard_normal((r, d_h)), rng.standard_normal((r, d_h))
    q = rng.standard_normal((H_q, d_h))
    K = oracle.reconstruct(A_k, B_k)
    Lm, m, out = oracle.landmarks(K.reshape(L, 1, d_h).transpose(1, 0, 2), c, o=1)
    got, rows, _ = oracle.sr_decode_landmark(A_k, A_v, B_k, B_v, q, Lm, out, L, c)
    assert rows[0].tolist() == list(range(L))
    np.testing.assert_allclose(got, oracle.dense(K, oracle.reconstruct(A_v, B_v), q, H_kv), rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------- rotary embedding of reconstructed rows
def test_rope_is_a_rotation_of_each_channel_pair_by_position_times_frequency():
    """Independent form: the pair (x[j], x[j + d/2]) as a complex number times exp(i p theta^(-2j/d))."""
    rng = np.random.default_rng(51)
    n, d, theta = 7, 8, 10000.0
    X = rng.standard_normal((n, d))
    pos = np.array([0, 1, 2, 5, 100, 4097, 65535])
    got = oracle.rope(X, pos, theta)
    z = (X[:, :d // 2] + 1j * X[:, d // 2:]) * np.exp(1j * pos[:, None] * theta ** (-np.arange(d // 2) / (d // 2)))
    np.testing.assert_allclose(got[:, :d // 2], z.real, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(got[:, d // 2:], z.imag, rtol=1e-11, atol=1e-12)
    np.testing.assert_array_equal(got[0], X[0])                                  # position 0 is the identity
    np.testing.assert_allclose((got ** 2).sum(axis=1), (X ** 2).sum(axis=1), rtol=1e-12)
    # two channels, frequency 1: the textbook 2-D rotation by `position` radians
    np.testing.assert_allclose(oracle.rope(np.array([[1.0, 0.0]]), [3], 10000.0), [[np.cos(3.0), np.sin(3.0)]], rtol=1e-13)


def test_rope_scores_depend_on_the_distance_only():
    rng = np.random.default_rng(52)
    d, theta = 16, 500000.0
    q, k = rng.standard_normal((1, d)), rng.standard_normal((1, d))
    a = float((oracle.rope(q, [40], theta) @ oracle.rope(k, [33], theta).T)[0, 0])
    b = float((oracle.rope(q, [1007], theta) @ oracle.rope(k, [1000], theta).T)[0, 0])
    assert abs(a - b) <= 1e-10 * (np.abs(q).sum() * np.abs(k).sum())


def test_landmark_step_with_rope_and_every_chunk_selected_is_dense_attention_on_rotated_keys():
    rng = np.random.default_rng(53)
    L, r, H_kv, H_q, d_h, c, theta = 40, 5, 2, 4, 8, 4, 10000.0
    A_k, A_v = rng.standard_normal((L, r)), rng.standard_normal((L, r))
    B_k, B_v = rng.standard_normal((r, H_kv * d_h)), rng.standard_normal((r, H_kv * d_h))
    q = rng.standard_normal((H_q, d_h))
    K_pre = oracle.reconstruct(A_k, B_k).reshape(L, H_kv, d_h).transpose(1, 0, 2)
    K_rope = np.stack([oracle.rope(K_pre[g], np.arange(L), theta) for g in range(H_kv)])
    Lm, _, outl = oracle.landmarks(K_rope, c, o=1)
    got, rows, _ = oracle.sr_decode_landmark(A_k, A_v, B_k, B_v, q, Lm, outl, L, c, rope_theta=theta)
    assert all(rw.tolist() == list(range(L)) for rw in rows)
    K_flat = K_rope.transpose(1, 0, 2).reshape(L, H_kv * d_h)
    np.testing.assert_allclose(got, oracle.dense(K_flat, oracle.reconstruct(A_v, B_v), q, H_kv), rtol=1e-11, atol=1e-13)
    # without the rotation the result differs: the rotation is not a no-op in this check
    plain, _, _ = oracle.sr_decode_landmark(A_k, A_v, B_k, B_v, q, Lm, outl, L, c)
    assert np.abs(plain - got).max() > 1e-3


def test_landmark_step_with_an_uncompressed_tail():
    """Empty tail = no tail; every chunk selected + tail = dense attention over [rotated compressed keys ; tail]; and
    the same rows with the tail equals gather_attend_tail (written independently for equal-length row lists)."""
    rng = np.random.default_rng(54)
    L, T, r, H_kv, H_q, d_h, c, theta = 32, 5, 4, 2, 4, 8, 4, 10000.0
    A_k, A_v = rng.standard_normal((L, r)), rng.standard_normal((L, r))
    B_k, B_v = rng.standard_normal((r, H_kv * d_h)), rng.standard_normal((r, H_kv * d_h))
    q = rng.standard_normal((H_q, d_h))
    K_tail, V_tail = rng.standard_normal((H_kv, T, d_h)), rng.standard_normal((H_kv, T, d_h))
    K_pre = oracle.reconstruct(A_k, B_k).reshape(L, H_kv, d_h).transpose(1, 0, 2)
    K_rope = np.stack([oracle.rope(K_pre[g], np.arange(L), theta) for g in range(H_kv)])
    Lm, _, outl = oracle.landmarks(K_rope, c, o=0)
    none, rows0, _ = oracle.sr_decode_landmark(A_k, A_v, B_k, B_v, q, Lm, outl, 8, c, rope_theta=theta)
    empty, _, _ = oracle.sr_decode_landmark(A_k, A_v, B_k, B_v, q, Lm, outl, 8, c, rope_theta=theta,
                                            K_tail=K_tail[:, :0], V_tail=V_tail[:, :0])
    np.testing.assert_array_equal(none, empty)
    full, rows, _ = oracle.sr_decode_landmark(A_k, A_v, B_k, B_v, q, Lm, outl, L, c, rope_theta=theta, K_tail=K_tail,
                                              V_tail=V_tail)
    K_all = np.concatenate([K_rope, K_tail], axis=1).transpose(1, 0, 2).reshape(L + T, H_kv * d_h)
    V_cmp = oracle.reconstruct(A_v, B_v).reshape(L, H_kv, d_h).transpose(1, 0, 2)
    V_all = np.concatenate([V_cmp, V_tail], axis=1).transpose(1, 0, 2).reshape(L + T, H_kv * d_h)
    np.testing.assert_allclose(full, oracle.dense(K_all, V_all, q, H_kv), rtol=1e-11, atol=1e-13)
    same_len = np.stack(rows0)                                     # no outliers, full chunks: equal lengths
    np.testing.assert_allclose(
        oracle.gather_attend_rows(A_k, A_v, B_k, B_v, q, rows0, K_tail=K_tail, V_tail=V_tail),
        oracle.gather_attend_tail(A_k, A_v, B_k, B_v, q, same_len, K_tail, V_tail), rtol=1e-12, atol=1e-14)


def test_absorbed_form_equals_reconstruct_then_attend():
    """o_h = ((w^T A^V[I]) B^V) with logits taken from the head scores is the same number as attention over the
    reconstructed rows (associativity); the head scores pool to the scores the selection sees."""
    rng = np.random.default_rng(61)
    L, r_k, r_v, H_kv, H_q, d_h, k = 70, 6, 9, 2, 6, 8, 11
    A_k, A_v = rng.standard_normal((L, r_k)), rng.standard_normal((L, r_v))
    B_k, B_v = rng.standard_normal((r_k, H_kv * d_h)), rng.standard_normal((r_v, H_kv * d_h))
    q = rng.standard_normal((H_q, d_h))
    idx = np.stack([np.sort(rng.choice(L, size=k, replace=False)) for _ in range(H_kv)]).astype(np.int32)
    np.testing.assert_allclose(oracle.gather_attend_absorbed(A_k, A_v, B_k, B_v, q, idx),
                               oracle.gather_attend(A_k, A_v, B_k, B_v, q, idx), rtol=1e-11, atol=1e-13)
    s = oracle.head_scores(A_k, B_k, q, H_kv)
    np.testing.assert_allclose(oracle.pool(s, H_kv), oracle.pooled_scores(A_k, B_k, q, H_kv), rtol=1e-15)
    K = oracle.reconstruct(A_k, B_k)
    for h in range(H_q):
        g = h // (H_q // H_kv)
        np.testing.assert_allclose(s[h], K[:, g * d_h:(g + 1) * d_h] @ q[h] / np.sqrt(d_h), rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------------------ RTN quantisation of the token basis
def test_quantiser_reproduces_the_papers_two_compression_ratios():
    """App. 'Integrate with Quantization': 8x becomes 25.6x with 4 bits and 32x with 3 bits.  With one extra bit per
    element of side information (two 16-bit numbers per group of 32) 16-bit storage shrinks by 16/5 and 16/4."""
    assert oracle.quantized_bits_per_element(4) == 5.0 and oracle.quantized_bits_per_element(3) == 4.0
    assert abs(8.0 * 16 / oracle.quantized_bits_per_element(4) - 25.6) < 1e-12
    assert abs(8.0 * 16 / oracle.quantized_bits_per_element(3) - 32.0) < 1e-12
    # the packed 4-bit row really has that size: 5r/8 bytes against 2r
    codes, step, lo = oracle.quantize_rows(np.zeros((3, 128), np.float32))
    assert oracle.pack_q4(codes, step, lo).shape == (3, 80)
    # ranks that are not multiples of 128 are padded to whole 16-byte units: 5 * 96 / 8 = 60 -> 64, 576 -> 360 -> 368
    c96 = oracle.pack_q4(*oracle.quantize_rows(np.ones((2, 96), np.float32)))
    assert c96.shape == (2, 64) and not c96[:, 60:].any()
    assert oracle.pack_q4(*oracle.quantize_rows(np.zeros((1, 576), np.float32))).shape == (1, 368)


def test_quantiser_on_a_group_worked_by_hand():
    # 32 values 0, 0.5, ..., 15.5: lo = 0, step = 15.5/15 -> bf16(1.0333..) = 1.03125, inv = fp32(1/1.03125)
    x = (np.arange(32, dtype=np.float32) * 0.5)[None, :]
    codes, step, lo = oracle.quantize_rows(x)
    assert lo[0, 0] == 0.0 and step[0, 0] == np.float32(1.03125)
    want = np.clip(np.rint(x[0] / 1.03125), 0, 15)
    np.testing.assert_array_equal(codes[0], want)
    assert codes[0, 0] == 0 and codes[0, -1] == 15 and codes[0, 1] == 0 and codes[0, 2] == 1
    # a constant group: step falls back to 1, all codes 0, the value comes back exactly
    c2, s2, l2 = oracle.quantize_rows(np.full((1, 32), -0.75, np.float32))
    assert s2[0, 0] == 1.0 and not c2.any()
    np.testing.assert_array_equal(oracle.dequantize_rows(c2, s2, l2), np.full((1, 32), -0.75))


def test_quantiser_error_bound_and_extremes():
    rng = np.random.default_rng(4)
    x = synth.to_storage(rng.standard_normal((50, 256)) * np.exp(rng.standard_normal((50, 1))), "bf16")
    xf = oracle.widen(x)
    for bits in (3, 4, 8):
        codes, step, lo = oracle.quantize_rows(x, bits)
        assert codes.max() <= (1 << bits) - 1
        xh = oracle.dequantize_rows(codes, step, lo)
        g = xf.reshape(50, 8, 32)
        # the minimum of a group is reproduced exactly (lo is a bf16 element of the group, code 0)
        np.testing.assert_array_equal(xh.reshape(50, 8, 32).min(axis=2), g.min(axis=2))
        # half a step, plus what rounding the step to bf16 can clip at the top of the range
        span = g.max(axis=2) - g.min(axis=2)
        bound = 0.5 * step.astype(np.float64) + span * 2.0 ** -8
        assert (np.abs(xh - xf).reshape(50, 8, 32).max(axis=2) <= bound + 1e-12).all()
        # the maximum of a group gets the top code (the bf16 rounding of the step moves it by at most
        # (2^bits - 1) 2^-9 codes: nothing up to 4 bits, one code at 8 bits)
        top = codes.reshape(50, 8, 32)[np.arange(50)[:, None], np.arange(8)[None, :], g.argmax(axis=2)]
        assert (top >= (1 << bits) - (2 if bits == 8 else 1)).all()


def test_q4_pack_layout_and_round_trip():
    codes = (np.arange(64, dtype=np.uint8) % 16)[None, :].repeat(2, axis=0)
    codes[1] = codes[1, ::-1]
    step = np.array([[0.5, 2.0], [1.0, 0.25]], np.float32)
    lo = np.array([[-1.0, 3.0], [0.0, -8.0]], np.float32)
    p = oracle.pack_q4(codes, step, lo)
    assert p.shape == (2, 48) and p.dtype == np.uint8 and not p[:, 40:].any()   # 40 bytes, padded to 16-byte units
    # word 0 = ranks 0..7 = codes 0..7: even ranks 0,2,4,6 in bits 0..15, odd ranks 1,3,5,7 in bits 16..31
    assert p[0, 0:4].tolist() == [0x20, 0x64, 0x31, 0x75] and p[0, 4:8].tolist() == [0xA8, 0xEC, 0xB9, 0xFD]
    assert p[0, 32:36].tolist() == [0x00, 0x3F, 0x80, 0xBF]                 # bf16(0.5) = 0x3F00, bf16(-1) = 0xBF80
    c2, s2, l2 = oracle.unpack_q4(p, 64)
    np.testing.assert_array_equal(c2, codes)
    np.testing.assert_array_equal(s2, step)
    np.testing.assert_array_equal(l2, lo)


def test_q3_pack_layout_and_round_trip():
    """3-bit rows: one 16-byte piece per group of 32 ranks, 12 bytes of codes + (step, lo); r/2 bytes per row, which is
    the 4 bits per element behind the paper's 32x (App. 'Integrate with Quantization')."""
    codes = (np.arange(64, dtype=np.uint8) % 8)[None, :].repeat(2, axis=0)
    codes[1] = codes[1, ::-1]
    step = np.array([[0.5, 2.0], [1.0, 0.25]], np.float32)
    lo = np.array([[-1.0, 3.0], [0.0, -8.0]], np.float32)
    p = oracle.pack_q3(codes, step, lo)
    assert p.shape == (2, 32) and p.dtype == np.uint8                       # 64 ranks -> 32 bytes = 4 bits per element
    # unit 0 = ranks 0..7 = codes 0..7: even ranks 0,2,4,6 -> 0 | 2<<3 | 4<<6 | 6<<9 = 0xD10 in bits 0..11,
    # odd ranks 1,3,5,7 -> 1 | 3<<3 | 5<<6 | 7<<9 = 0xF59 in bits 12..23: the 24-bit unit is 0xF59D10
    assert p[0, 0:3].tolist() == [0x10, 0x9D, 0xF5]
    assert p[0, 3:6].tolist() == [0x10, 0x9D, 0xF5]                          # unit 1 holds the same codes (8..15 mod 8)
    assert p[0, 12:16].tolist() == [0x00, 0x3F, 0x80, 0xBF]                 # bf16(0.5) = 0x3F00, bf16(-1) = 0xBF80
    assert p[0, 28:32].tolist() == [0x00, 0x40, 0x40, 0x40]                 # bf16(2) = 0x4000, bf16(3) = 0x4040
    c2, s2, l2 = oracle.unpack_q3(p, 64)
    np.testing.assert_array_equal(c2, codes)
    np.testing.assert_array_equal(s2, step)
    np.testing.assert_array_equal(l2, lo)
    rng = np.random.default_rng(8)
    x = synth.to_storage(rng.standard_normal((9, 160)), "bf16")
    c, s, l = oracle.quantize_rows(x, 3)
    for a, b in zip(oracle.unpack_q3(oracle.pack_q3(c, s, l), 160), (c, s, l)):
        np.testing.assert_array_equal(a, b)


def test_three_bit_quantiser_on_a_group_worked_by_hand():
    # 32 values 0, 0.25, ..., 7.75: lo = 0, step = 7.75/7 = 1.10714.. -> bf16 = 1.109375 (0x3F8E), inv = fp32(1/step)
    x = (np.arange(32, dtype=np.float32) * 0.25)[None, :]
    codes, step, lo = oracle.quantize_rows(x, 3)
    assert lo[0, 0] == 0.0 and step[0, 0] == np.float32(1.109375)
    np.testing.assert_array_equal(codes[0], np.clip(np.rint(x[0] / 1.109375), 0, 7))
    assert codes[0, 0] == 0 and codes[0, -1] == 7 and codes[0, 2] == 0 and codes[0, 3] == 1


@pytest.mark.parametrize("bits", [4, 3])
def test_quantiser_codes_against_the_plain_definition_in_double_precision(bits):
    """The codes come from fp32 operations ((x - lo) times the rounded reciprocal of the step).  Against the plain
    definition rint((x - lo) / step) evaluated in float64 they may differ only where the exact quotient is a tie
    (fractional part exactly one half): there both neighbours are nearest, everywhere else the code is the same."""
    rng = np.random.default_rng(5)
    X = oracle._bf16_rne((rng.standard_normal((4000, 256)) / 16.0).astype(np.float32))
    codes, step, lo = oracle.quantize_rows(X, bits)
    g = X.reshape(4000, 8, 32).astype(np.float64)
    t = ((g - lo.astype(np.float64)[:, :, None]) / step.astype(np.float64)[:, :, None]).reshape(4000, 256)
    plain = np.clip(np.rint(t), 0, (1 << bits) - 1).astype(np.uint8)
    differ = plain != codes
    assert differ.mean() < 1e-3
    assert differ.any()          # the sample is large enough to contain ties, or the check below is empty
    frac = t[differ] - np.floor(t[differ])
    np.testing.assert_array_equal(frac, 0.5)
    assert np.abs(codes[differ].astype(np.int64) - plain[differ].astype(np.int64)).max() == 1
