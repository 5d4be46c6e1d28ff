"""GPU parity of xkv_factorize (Cross-Layer Factorization, Sec. 3.1, Eq. 1) against the CPU oracle.

The GPU path finds the rank-r subspace iteratively (App. B.3) and then rotates its basis to the singular vectors,
which are unique up to sign where the singular values are distinct; the comparison is on what is unique:
  * A^T A is diagonal and descending, its diagonal the squared singular values (also returned by
    xkv_factorize_svd), against the oracle's / LAPACK's where the iteration has converged (Eq. 1: A = U Sigma);
  * a leading block of r_out < r directions is the best rank-r_out approximation the subspace offers;
  * the approximation error ||X_cat - A B||_F^2 against the optimum sum_{i>r} sigma_i^2 of the oracle's exact
    truncated SVD (Eckart-Young), within 2 % of the optimum plus the rounding of A and B to the storage type;
  * the well-separated leading right singular vectors of the oracle lie in the row space of B;
  * B has orthonormal rows and A = X_cat B^T for the B that was stored (element by element);
  * an X_cat of rank r is reproduced, and decode attention computed from the GPU factors equals dense
    attention on the uncompressed cache.
Rounding terms: bf16 storage rounds A and B to 2^-9 relative each, i.e. about 2 * 2^-18 = 8e-6 of
||X_cat||_F^2 in the squared error (bound used: 3e-5); fp32 storage 1e-12.
"""
import numpy as np
import pytest

import oracle
from paper_2503_18893_amd import synth
from paper_2503_18893_amd import binding as xb

pytestmark = pytest.mark.gpu

ROUND_SQ = {"bf16": 3e-5, "f32": 1e-12}
ORTH = {"bf16": 4e-3, "f32": 1e-5}
ELEM = {"bf16": 2.0 ** -7, "f32": 1e-5}
ITERS = 8


def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def gpu_factorize(caches, G, H_kv, d_h, L, r, dtype, iters=ITERS, seed=7):
    """caches: list (one per sequence) of X [G][H_kv][L][d_h] storage arrays.  Returns float64 A [b][L][r],
    B_cat [b][r][n]."""
    torch = torch_mod()
    batch = len(caches)
    shape = xb.Shape(G=G, H_kv=H_kv, H_q=H_kv, d_h=d_h, r_k=r, r_v=r, L=L, k=1, batch=batch, dtype=dtype)
    X = synth.to_device({"X": np.stack(caches)}, dtype)["X"]
    dt = synth.torch_dtype(dtype)
    A = torch.zeros((batch, L, r), dtype=dt, device="cuda")
    B = torch.zeros((batch, G, r, H_kv * d_h), dtype=dt, device="cuda")
    ws = torch.empty(xb.xkv_factorize_workspace_bytes(shape, r), dtype=torch.uint8, device="cuda")
    xb.xkv_factorize(shape, X, r, iters, seed, A, B, ws)
    torch.cuda.synchronize()
    A64 = synth.storage_to_f64(synth.to_host(A))
    B64 = synth.storage_to_f64(synth.to_host(B)).transpose(0, 2, 1, 3).reshape(batch, r, G * H_kv * d_h)
    return A64, B64, (A, B)


CASES = {
    # name: G, H_kv, d_h, L, r, batch, dtype, decay
    "two_layers_bf16": (2, 2, 64, 1000, 48, 2, "bf16", 0.7),
    "ragged_tiles_bf16": (5, 1, 64, 2500, 100, 1, "bf16", 0.7),   # n = 320: a 256 tile and a 64 tail; r % 8 != 0
    "two_layers_f32": (2, 2, 64, 1000, 48, 1, "f32", 0.7),
    "steep_spectrum_bf16": (1, 2, 128, 700, 30, 1, "bf16", 1.2),
}


@pytest.mark.parametrize("name", list(CASES))
def test_factorize_against_exact_truncated_svd(name):
    G, H_kv, d_h, L, r, batch, dtype, decay = CASES[name]
    rng = np.random.default_rng(np.random.SeedSequence([31, len(name)]))
    caches = [synth.make_cache(rng, G, H_kv, d_h, L, decay, dtype=dtype) for _ in range(batch)]
    A, B, _ = gpu_factorize(caches, G, H_kv, d_h, L, r, dtype)
    for b in range(batch):
        X = synth.cache_as_matrix(caches[b])
        A_o, B_o, sigma = oracle.factorize(X, r)
        opt, tot = float(np.sum(sigma[r:] ** 2)), float(np.sum(sigma ** 2))
        res = float(np.sum((X - A[b] @ B[b]) ** 2))
        assert res >= opt * (1.0 - 1e-9)                        # nothing beats the truncated SVD
        assert res <= 1.02 * opt + ROUND_SQ[dtype] * tot, (name, b, res / opt)
        # orthonormal rows, and A is the projection coefficient of every token for the stored B
        assert np.abs(B[b] @ B[b].T - np.eye(r)).max() <= ORTH[dtype]
        ref_A = X @ B[b].T
        assert np.abs(A[b] - ref_A).max() <= ELEM[dtype] * np.abs(ref_A).max()
        # leading directions of the exact factorization (sigma_i >= 2.5 sigma_r) are inside the row space of B
        lead = int(np.sum(sigma[:r] >= 2.5 * sigma[r - 1]))
        assert lead >= 1
        inside = np.sum((B_o[:lead] @ B[b].T) ** 2, axis=1)
        assert inside.min() >= 1.0 - 1e-2, (name, b, inside.min())


@pytest.mark.parametrize("rank", [40, 24])
def test_factorize_reproduces_low_rank_cache(rank):
    """rank == r: A B = X_cat up to storage rounding (the first pin of the oracle's factorize, on the GPU);
    rank < r: the surplus directions must come out harmless (finite, nothing added to A B)."""
    G, H_kv, d_h, L, r, dtype = 2, 2, 64, 900, 40, "bf16"
    rng = np.random.default_rng(5 + rank)
    cache = synth.make_cache(rng, G, H_kv, d_h, L, 0.5, rank=rank, dtype=dtype)
    A, B, _ = gpu_factorize([cache], G, H_kv, d_h, L, r, dtype)
    X = synth.cache_as_matrix(cache)
    assert np.isfinite(A).all() and np.isfinite(B).all()
    # X itself was rounded to bf16, which adds rank-n noise of relative size 2^-9 that no rank-r product can follow
    assert np.sum((X - A[0] @ B[0]) ** 2) <= 4e-5 * np.sum(X ** 2)
    A_o, B_o, _ = oracle.factorize(X, r)
    assert np.abs(A[0] @ B[0] - A_o @ B_o).max() <= 2e-2 * np.abs(X).max()


def test_factorize_larger_matrix_several_tiles():
    """n = 1024 (a 4 x 4 grid of Gram tiles, 10 of them computed, token range split), L over several tiles of the
    A product.  The optimum comes from LAPACK's singular values, against which the oracle's are pinned."""
    G, H_kv, d_h, L, r, dtype = 2, 4, 128, 3000, 128, "bf16"
    rng = np.random.default_rng(77)
    cache = synth.make_cache(rng, G, H_kv, d_h, L, 1.0, dtype=dtype)
    A, B, _ = gpu_factorize([cache], G, H_kv, d_h, L, r, dtype)
    X = synth.cache_as_matrix(cache)
    sv = np.linalg.svd(X, compute_uv=False)
    opt, tot = float(np.sum(sv[r:] ** 2)), float(np.sum(sv ** 2))
    res = float(np.sum((X - A[0] @ B[0]) ** 2))
    assert opt * (1 - 1e-9) <= res <= 1.02 * opt + ROUND_SQ[dtype] * tot, res / opt
    assert np.abs(B[0] @ B[0].T - np.eye(r)).max() <= ORTH[dtype]
    ref_A = X @ B[0].T
    assert np.abs(A[0] - ref_A).max() <= ELEM[dtype] * np.abs(ref_A).max()


def test_more_iterations_do_not_hurt_and_one_is_worse():
    G, H_kv, d_h, L, r, dtype = 2, 2, 64, 1200, 32, "f32"
    rng = np.random.default_rng(3)
    cache = synth.make_cache(rng, G, H_kv, d_h, L, 0.6, dtype=dtype)
    X = synth.cache_as_matrix(cache)
    res = []
    for iters in (1, 4, 16):
        A, B, _ = gpu_factorize([cache], G, H_kv, d_h, L, r, dtype, iters=iters)
        res.append(float(np.sum((X - A[0] @ B[0]) ** 2)))
    sv = np.linalg.svd(X, compute_uv=False)
    opt = float(np.sum(sv[r:] ** 2))
    assert res[0] > res[1] > res[2] >= opt * (1 - 1e-9)
    assert res[2] <= 1.005 * opt


def test_decode_from_gpu_factors_matches_dense_attention_on_the_cache():
    """Caches of rank r, factorized on the GPU (keys and values separately), then one SR decode step with k = L:
    equals dense attention over the uncompressed cache (oracle), layer by layer."""
    torch = torch_mod()
    G, H_kv, H_q, d_h, L, r, dtype = 2, 2, 8, 64, 640, 32, "bf16"
    rng = np.random.default_rng(11)
    Kc = synth.make_cache(rng, G, H_kv, d_h, L, 0.3, rank=r, dtype=dtype)
    Vc = synth.make_cache(rng, G, H_kv, d_h, L, 0.3, rank=r, dtype=dtype)
    _, _, (A_k, B_k) = gpu_factorize([Kc], G, H_kv, d_h, L, r, dtype)
    _, _, (A_v, B_v) = gpu_factorize([Vc], G, H_kv, d_h, L, r, dtype, seed=8)
    shape = xb.Shape(G=G, H_kv=H_kv, H_q=H_q, d_h=d_h, r_k=r, r_v=r, L=L, k=L, batch=1, dtype=dtype)
    ws = xb.alloc_workspace(shape)
    q_host = synth.to_storage(rng.standard_normal((G, 1, H_q, d_h)) * 0.5, dtype)
    q_dev = synth.to_device({"q": q_host}, dtype)["q"]
    for layer in range(G):
        out = torch.empty((1, H_q, d_h), dtype=synth.torch_dtype(dtype), device="cuda")
        xb.xkv_sr_decode(shape, layer, A_k, A_v, B_k, B_v, q_dev[layer].contiguous(), out, None, None, ws)
        torch.cuda.synchronize()
        K = synth.storage_to_f64(Kc[layer]).transpose(1, 0, 2).reshape(L, H_kv * d_h)
        V = synth.storage_to_f64(Vc[layer]).transpose(1, 0, 2).reshape(L, H_kv * d_h)
        ref = oracle.dense(K, V, synth.storage_to_f64(q_host[layer, 0]), H_kv)
        got = synth.storage_to_f64(synth.to_host(out))[0]
        assert np.abs(got - ref).max() <= 2e-2 * np.abs(ref).max(), layer


def test_full_size_group_known_spectrum():
    """Llama-3.1-8B group at the bench's size (n = 4096, L = 65536, r = 512) on a cache whose singular values and
    right singular vectors are known by construction: X_cat = U diag(s) Q with U made of 16 signed, scaled
    permutation blocks (orthonormal columns).  Checked: energy captured by A against sum_{i<=r} s_i^2, the known
    leading directions inside the row space of B, orthonormal rows, sampled rows of A."""
    torch = torch_mod()
    G, H_kv, d_h, L, r, dtype = 4, 8, 128, 65536, 512, "bf16"
    n = G * H_kv * d_h
    rng = np.random.default_rng(2024)
    s = np.arange(1, n + 1, dtype=np.float64) ** -0.7
    Q = np.linalg.qr(rng.standard_normal((n, n)))[0].T
    SQ = torch.from_numpy((s[:, None] * Q * 0.25 * 64.0).astype(np.float32)).cuda()      # rows s_j Q_j / 4, scaled up
    blocks = []
    for b in range(L // n):
        perm = torch.from_numpy(rng.permutation(n)).cuda()
        sign = torch.from_numpy(rng.choice([-1.0, 1.0], size=n).astype(np.float32)).cuda()
        blocks.append(SQ[perm] * sign[:, None])
    Xcat = torch.cat(blocks).to(torch.bfloat16)                                           # [L][n]
    X = Xcat.view(L, G, H_kv, d_h).permute(1, 2, 0, 3).contiguous().unsqueeze(0)
    shape = xb.Shape(G=G, H_kv=H_kv, H_q=H_kv, d_h=d_h, r_k=r, r_v=r, L=L, k=1, batch=1, dtype=dtype)
    A = torch.zeros((1, L, r), dtype=torch.bfloat16, device="cuda")
    B = torch.zeros((1, G, r, H_kv * d_h), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(xb.xkv_factorize_workspace_bytes(shape, r), dtype=torch.uint8, device="cuda")
    xb.xkv_factorize(shape, X, r, ITERS, 99, A, B, ws)
    torch.cuda.synchronize()
    Bc = synth.storage_to_f64(synth.to_host(B))[0].transpose(1, 0, 2).reshape(r, n)
    assert np.abs(Bc @ Bc.T - np.eye(r)).max() <= ORTH[dtype]
    s_eff = s * 64.0                                     # singular values of X_cat (16 blocks x (1/4)^2 = 1)
    captured = float((A.double() ** 2).sum().item())
    total, best = float(np.sum(s_eff ** 2)), float(np.sum(s_eff[:r] ** 2))
    opt = total - best
    assert (total - captured) <= 1.02 * opt + ROUND_SQ[dtype] * total
    assert captured <= best * (1 + 1e-3)
    lead = int(np.sum(s[:r] >= 2.5 * s[r - 1]))
    inside = np.sum((Q[:lead] @ Bc.T) ** 2, axis=1)
    assert inside.min() >= 1.0 - 1e-2, inside.min()
    rows = rng.choice(L, size=64, replace=False)
    Xs = Xcat[torch.from_numpy(rows).cuda()].double().cpu().numpy()
    ref_A = Xs @ Bc.T
    got_A = synth.storage_to_f64(synth.to_host(A[0, torch.from_numpy(rows).cuda()]))
    assert np.abs(got_A - ref_A).max() <= ELEM[dtype] * np.abs(ref_A).max()


@pytest.mark.parametrize("G,H_kv,d_h,L,r,batch,dtype", [
    (1, 1, 64, 40, 1, 1, "f32"),        # one direction, a context shorter than one token tile
    (1, 1, 64, 500, 64, 1, "f32"),      # r = n: nothing is discarded
    (1, 2, 64, 300, 20, 18, "bf16"),    # more sequences than one pass takes (16 + 2)
    (3, 1, 64, 257, 33, 2, "bf16"),     # n = 192 (no full 256-row tile), odd sizes everywhere
])
def test_factorize_edge_shapes(G, H_kv, d_h, L, r, batch, dtype):
    rng = np.random.default_rng(G * 1000 + L)
    caches = [synth.make_cache(rng, G, H_kv, d_h, L, 0.8, dtype=dtype) for _ in range(batch)]
    A, B, _ = gpu_factorize(caches, G, H_kv, d_h, L, r, dtype, iters=12)
    n = G * H_kv * d_h
    for b in (0, batch - 1):
        X = synth.cache_as_matrix(caches[b])
        sv = np.linalg.svd(X, compute_uv=False)
        opt, tot = float(np.sum(sv[r:] ** 2)), float(np.sum(sv ** 2))
        res = float(np.sum((X - A[b] @ B[b]) ** 2))
        assert res <= 1.02 * opt + max(ROUND_SQ[dtype], 1e-9) * tot, (b, res, opt)
        assert np.abs(B[b] @ B[b].T - np.eye(r)).max() <= ORTH[dtype]
    if r == n:
        assert np.sum((synth.cache_as_matrix(caches[0]) - A[0] @ B[0]) ** 2) <= 1e-9 * tot


# what the rotation to singular vectors leaves of A^T A beside its diagonal, relative to the largest eigenvalue: the
# Rayleigh-Ritz matrix is formed from fp32 products (f32: 1e-6 sigma_1^2), and B is rounded to the storage type before A
# is formed from it (bf16: 2^-9 per element)
OFFDIAG = {"bf16": 1e-2, "f32": 1e-4}


def gpu_factorize_svd(caches, G, H_kv, d_h, L, r, r_out, dtype, iters=ITERS, seed=7):
    torch = torch_mod()
    batch = len(caches)
    shape = xb.Shape(G=G, H_kv=H_kv, H_q=H_kv, d_h=d_h, r_k=r, r_v=r, L=L, k=1, batch=batch, dtype=dtype)
    X = synth.to_device({"X": np.stack(caches)}, dtype)["X"]
    dt = synth.torch_dtype(dtype)
    A = torch.zeros((batch, L, r_out), dtype=dt, device="cuda")
    B = torch.zeros((batch, G, r_out, H_kv * d_h), dtype=dt, device="cuda")
    sig = torch.zeros((batch, r_out), dtype=torch.float32, device="cuda")
    ws = torch.empty(xb.xkv_factorize_workspace_bytes(shape, r), dtype=torch.uint8, device="cuda")
    xb.xkv_factorize_svd(shape, X, r, r_out, iters, seed, A, B, sig, ws)
    torch.cuda.synchronize()
    A64 = synth.storage_to_f64(synth.to_host(A))
    B64 = synth.storage_to_f64(synth.to_host(B)).transpose(0, 2, 1, 3).reshape(batch, r_out, G * H_kv * d_h)
    return A64, B64, sig.cpu().numpy().astype(np.float64)


SVD_CASES = {
    # name: G, H_kv, d_h, L, r, batch, dtype, decay, iters
    "f32_r48": (2, 2, 64, 1000, 48, 2, "f32", 0.7, 12),
    "bf16_r100": (5, 1, 64, 2500, 100, 1, "bf16", 0.7, 8),
    "bf16_steep_r30": (1, 2, 128, 700, 30, 1, "bf16", 1.2, 8),
    "bf16_r512_n1024": (2, 4, 128, 3000, 512, 1, "bf16", 0.8, 8),      # 32 column blocks of the eigen-solver
    "f32_r640_n1024": (2, 4, 128, 2000, 640, 1, "f32", 0.8, 8),        # the 16-column form of the eigen-solver
}


@pytest.mark.parametrize("name", list(SVD_CASES))
def test_factors_are_u_sigma_and_v_transposed(name):
    """Sec. 3.1, Eq. 1: A = U Sigma, B = V^T.  A^T A diagonal and descending, equal to the returned sigma^2; B B^T = I;
    singular values against the exact ones where the subspace iteration has separated them."""
    G, H_kv, d_h, L, r, batch, dtype, decay, iters = SVD_CASES[name]
    rng = np.random.default_rng(np.random.SeedSequence([41, len(name)]))
    caches = [synth.make_cache(rng, G, H_kv, d_h, L, decay, dtype=dtype) for _ in range(batch)]
    A, B, sig = gpu_factorize_svd(caches, G, H_kv, d_h, L, r, r, dtype, iters=iters)
    for b in range(batch):
        X = synth.cache_as_matrix(caches[b])
        sv = np.linalg.svd(X, compute_uv=False)
        AtA = A[b].T @ A[b]
        lam = np.diag(AtA)
        off = AtA - np.diag(lam)
        assert np.abs(off).max() <= OFFDIAG[dtype] * lam.max(), (name, b, np.abs(off).max() / lam.max())
        # descending (neighbours may swap inside the rounding of the storage type)
        assert (lam[1:] <= lam[:-1] * (1 + 4 * OFFDIAG[dtype])).all()
        np.testing.assert_allclose(sig[b] ** 2, lam, rtol=4 * OFFDIAG[dtype], atol=OFFDIAG[dtype] * lam.max())
        assert np.abs(B[b] @ B[b].T - np.eye(r)).max() <= ORTH[dtype]
        # converged part of the spectrum: singular values well above the last one kept
        lead = int(np.sum(sv[:r] >= 2.5 * sv[r - 1]))
        np.testing.assert_allclose(sig[b][:lead], sv[:lead], rtol=1e-2)
        # and the rotation has not changed the subspace: error against the optimum as before
        opt, tot = float(np.sum(sv[r:] ** 2)), float(np.sum(sv ** 2))
        res = float(np.sum((X - A[b] @ B[b]) ** 2))
        assert opt * (1 - 1e-9) <= res <= 1.02 * opt + ROUND_SQ[dtype] * tot, (name, b, res / opt)


def test_leading_block_of_a_larger_run_is_a_good_smaller_factorization():
    """r_out < r: the leading r_out directions of a run with r vectors.  They are the first rows of the full result
    (same run), their error is within 2 % of the rank-r_out optimum (the surplus vectors act as oversampling), and
    one run serves two ranks (keys at r_out, values at r: Sec. 4, r_K : r_V = 1 : 1.5)."""
    G, H_kv, d_h, L, r, r_out, dtype = 2, 2, 64, 1500, 96, 64, "bf16"
    rng = np.random.default_rng(17)
    cache = synth.make_cache(rng, G, H_kv, d_h, L, 0.7, dtype=dtype)
    X = synth.cache_as_matrix(cache)
    A_full, B_full, sig_full = gpu_factorize_svd([cache], G, H_kv, d_h, L, r, r, dtype)
    A_lead, B_lead, sig_lead = gpu_factorize_svd([cache], G, H_kv, d_h, L, r, r_out, dtype)
    np.testing.assert_array_equal(B_lead[0], B_full[0][:r_out])
    np.testing.assert_array_equal(sig_lead[0], sig_full[0][:r_out])
    np.testing.assert_allclose(A_lead[0], A_full[0][:, :r_out], rtol=0, atol=2.0 ** -7 * np.abs(A_full[0]).max())
    sv = np.linalg.svd(X, compute_uv=False)
    opt, tot = float(np.sum(sv[r_out:] ** 2)), float(np.sum(sv ** 2))
    res = float(np.sum((X - A_lead[0] @ B_lead[0]) ** 2))
    assert opt * (1 - 1e-9) <= res <= 1.02 * opt + ROUND_SQ[dtype] * tot, res / opt
    # a run with only r_out vectors and the same number of iterations is no better than the truncated larger run
    A_small, B_small, _ = gpu_factorize_svd([cache], G, H_kv, d_h, L, r_out, r_out, dtype)
    assert res <= float(np.sum((X - A_small[0] @ B_small[0]) ** 2)) * (1 + 1e-3)


def test_factorize_of_an_empty_batch_is_a_no_op():
    torch = torch_mod()
    shape = xb.Shape(G=1, H_kv=1, H_q=1, d_h=64, r_k=8, r_v=8, L=100, k=1, batch=0, dtype="bf16")
    ws = torch.empty(max(256, xb.xkv_factorize_workspace_bytes(shape, 8)), dtype=torch.uint8, device="cuda")
    dummy = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    xb.xkv_factorize(shape, dummy, 8, 4, 0, dummy, dummy, ws)
    torch.cuda.synchronize()
