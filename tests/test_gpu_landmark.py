"""GPU parity of the paper's landmark-guided selector (App. B.1, Alg. 1-2) and of SR decode driven by it.

Chain of strict links, as for the factor-scoring step (each stage is fed what the GPU fed the next one):
  (i)   xkv_landmarks: chunk means and minimum cosines vs oracle.landmarks                   within tolerance
        outliers                  vs oracle.select(-min cosine as the GPU computed it, o)    identical
  (ii)  xkv_sr_decode_landmark: pooled chunk scores vs oracle.chunk_scores(stored landmarks) within tolerance
        rows[:count]              vs oracle: top chunks of the GPU's scores, union, expansion identical
        out                       vs oracle.gather_attend_rows on the GPU's rows              within tolerance
  (iii) xkv_gather_attend_ex: row counts and the rotary embedding of the reconstructed key rows (Sec. 4) vs
        oracle.gather_attend_rows(rope_theta) on random rows over contexts up to 131072 tokens    within tolerance
  (iv)  factors of pre-RoPE keys + landmarks of post-RoPE keys + rotation of the reconstructed rows: the paper's
        arrangement, checked against dense attention over the rotated keys when every chunk is selected
In (i)-(ii) the post-RoPE keys are stood in for by K = A^K B^K_l and no rotation is applied.
Tolerance: max|gpu - ref| / max|ref|, 1e-5 for fp32 and 2e-2 for bf16 storage; cosines absolute 1e-4.
"""
import numpy as np
import pytest

import oracle
from paper_2503_18893_amd import synth
from paper_2503_18893_amd import binding as xb

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def max_rel(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


def keys_of(case, w, layer):
    """K = A^K B^K_l of every sequence, [batch][H_kv][L][d_h] in storage form (rounded once, like a real cache)."""
    K = np.empty((w.batch, w.H_kv, w.L, w.d_h))
    for b in range(w.batch):
        X = oracle.reconstruct(case["A_k"][b], case["B_k"][b, layer])
        K[b] = X.reshape(w.L, w.H_kv, w.d_h).transpose(1, 0, 2)
    return synth.to_storage(K, w.dtype)


CASES = {
    # name: workload fields, c, o
    "tiny_f32": (dict(G=2, H_kv=2, H_q=4, d_h=32, r_k=8, r_v=12, L=150, k=20, batch=2, dtype="f32"), 4, 2),
    "llama_heads_bf16": (dict(G=2, H_kv=2, H_q=8, d_h=128, r_k=64, r_v=96, L=3000, k=256, batch=2, dtype="bf16"), 8, 3),
    "ragged_context_bf16": (dict(G=1, H_kv=2, H_q=8, d_h=128, r_k=32, r_v=32, L=1001, k=100, batch=1, dtype="bf16"), 8, 0),
    "outliers_overlap_bf16": (dict(G=1, H_kv=2, H_q=4, d_h=128, r_k=32, r_v=32, L=160, k=80, batch=3, dtype="bf16"), 8, 6),
    "every_chunk_bf16": (dict(G=1, H_kv=1, H_q=4, d_h=128, r_k=16, r_v=16, L=333, k=333, batch=1, dtype="bf16"), 16, 1),
}


def workload(fields):
    return synth.Workload(name="landmark_case", a_scale=1.0, sigma_decay=0.5, q_scale=0.3, **fields)


@pytest.mark.parametrize("name", list(CASES))
def test_landmark_selector_chain(name):
    torch = torch_mod()
    fields, c, o = CASES[name]
    w = workload(fields)
    case = synth.make_case(w, seed=90 + len(name))
    layer = w.G - 1
    K_host = keys_of(case, w, layer)
    shape = xb.Shape.of(w)
    dev = synth.to_device(case, w.dtype)
    K_dev = synth.to_device({"K": K_host}, w.dtype)["K"]
    dt = synth.torch_dtype(w.dtype)
    n_c = -(-w.L // c)
    k_ch = oracle.chunk_budget(w.k, c, n_c)
    cap = (k_ch + o) * c
    ws = torch.empty(xb.xkv_landmark_workspace_bytes(shape, c, o), dtype=torch.uint8, device="cuda")
    Lm = torch.zeros((w.batch, w.H_kv, n_c, w.d_h), dtype=dt, device="cuda")
    negm = torch.zeros((w.batch, w.H_kv, n_c), dtype=torch.float32, device="cuda")
    outl = torch.zeros((w.batch, w.H_kv, max(o, 1)), dtype=torch.int32, device="cuda")
    xb.xkv_landmarks(shape, K_dev, c, o, Lm, negm, outl if o else None, ws)
    q = dev["q"][layer].contiguous()
    out = torch.zeros((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda")
    rows = torch.full((w.batch, w.H_kv, cap), -7, dtype=torch.int32, device="cuda")
    cnt = torch.zeros((w.batch, w.H_kv), dtype=torch.int32, device="cuda")
    S = torch.zeros((w.batch, w.H_kv, n_c), dtype=torch.float32, device="cuda")
    xb.xkv_sr_decode_landmark(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, Lm, outl if o else None,
                              c, o, out, rows, cnt, S, ws)
    out2 = torch.zeros_like(out)     # the same call without the optional outputs
    xb.xkv_sr_decode_landmark(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, Lm, outl if o else None,
                              c, o, out2, None, None, None, ws)
    torch.cuda.synchronize()
    Lm_h, negm_h, outl_h = synth.to_host(Lm), negm.cpu().numpy(), outl.cpu().numpy()
    rows_h, cnt_h, S_h = rows.cpu().numpy(), cnt.cpu().numpy(), S.cpu().numpy()
    out_h, out2_h = synth.storage_to_f64(synth.to_host(out)), synth.storage_to_f64(synth.to_host(out2))
    assert np.array_equal(out_h, out2_h)
    qh = synth.to_host(q)
    for b in range(w.batch):
        # (i) Alg. 1
        Lm_ref, m_ref, _ = oracle.landmarks(K_host[b], c, o)
        assert max_rel(synth.storage_to_f64(Lm_h[b]), Lm_ref) <= (2.0 ** -8 if w.dtype == "bf16" else 1e-6)
        assert np.abs(-negm_h[b].astype(np.float64) - m_ref).max() <= 1e-4
        if o:
            for g in range(w.H_kv):
                assert outl_h[b, g].tolist() == oracle.select(negm_h[b, g], o).tolist()
        # (ii) Alg. 2 on the stored landmarks
        S_ref = oracle.chunk_scores(Lm_h[b], qh[b])
        assert max_rel(S_h[b], S_ref) <= TOL[w.dtype]
        rows_b = []
        for g in range(w.H_kv):
            want = oracle.expand_chunks(oracle.select(S_h[b, g], k_ch), outl_h[b, g][:o], c, w.L)
            assert cnt_h[b, g] == len(want)
            assert rows_h[b, g, :cnt_h[b, g]].tolist() == want.tolist()
            assert not rows_h[b, g, cnt_h[b, g]:].any()          # padding
            rows_b.append(want)
        ref = oracle.gather_attend_rows(case["A_k"][b], case["A_v"][b], case["B_k"][b, layer], case["B_v"][b, layer],
                                        qh[b], rows_b)
        assert max_rel(out_h[b], ref) <= TOL[w.dtype], (name, b)
    if name == "every_chunk_bf16":      # every chunk selected: dense attention over the compressed cache
        Kd = oracle.reconstruct(case["A_k"][0], case["B_k"][0, layer])
        Vd = oracle.reconstruct(case["A_v"][0], case["B_v"][0, layer])
        assert max_rel(out_h[0], oracle.dense(Kd, Vd, qh[0], w.H_kv)) <= TOL[w.dtype]
        assert cnt_h[0, 0] == w.L
    if name == "outliers_overlap_bf16":  # the union is smaller than its capacity somewhere
        assert (cnt_h < cap).any()


def test_landmark_step_at_full_size_sampled():
    """The bench's Llama shape (batch 16, L = 65536, k = 4096) with c = 8 and 4 outlier chunks per head, in the
    launch configuration the library picks for it; checked on sampled (sequence, head) pairs."""
    torch = torch_mod()
    w = synth.LLAMA_FULL
    c, o, layer = 8, 4, 1
    g = synth.make_group_device(w, seed=5)
    shape = xb.Shape.of(w)
    dt = synth.torch_dtype(w.dtype)
    n_c = w.L // c
    k_ch = w.k // c
    cap = (k_ch + o) * c
    K = torch.empty((w.batch, w.H_kv, w.L, w.d_h), dtype=dt, device="cuda")
    xb.xkv_reconstruct(shape, layer, g["A_k"], g["B_k"], w.r_k, K)
    ws = torch.empty(xb.xkv_landmark_workspace_bytes(shape, c, o), dtype=torch.uint8, device="cuda")
    Lm = torch.zeros((w.batch, w.H_kv, n_c, w.d_h), dtype=dt, device="cuda")
    negm = torch.zeros((w.batch, w.H_kv, n_c), dtype=torch.float32, device="cuda")
    outl = torch.zeros((w.batch, w.H_kv, o), dtype=torch.int32, device="cuda")
    xb.xkv_landmarks(shape, K, c, o, Lm, negm, outl, ws)
    q = g["q"][layer].contiguous()
    out = torch.zeros((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda")
    rows = torch.zeros((w.batch, w.H_kv, cap), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((w.batch, w.H_kv), dtype=torch.int32, device="cuda")
    S = torch.zeros((w.batch, w.H_kv, n_c), dtype=torch.float32, device="cuda")
    xb.xkv_sr_decode_landmark(shape, layer, g["A_k"], g["A_v"], g["B_k"], g["B_v"], q, Lm, outl, c, o, out, rows, cnt, S, ws)
    torch.cuda.synchronize()
    n_rep = w.H_q // w.H_kv
    for b, h in ((0, 0), (7, 3), (15, 7)):
        Kh = synth.storage_to_f64(synth.to_host(K[b, h]))
        Lm_ref, m_ref, _ = oracle.landmarks(Kh[None, :4096], c)            # first 512 chunks of this head
        assert max_rel(synth.storage_to_f64(synth.to_host(Lm[b, h, :512])), Lm_ref[0]) <= 2.0 ** -8
        assert np.abs(-negm[b, h, :512].cpu().numpy() - m_ref[0]).max() <= 1e-4
        negm_h, S_h = negm[b, h].cpu().numpy(), S[b, h].cpu().numpy()
        outl_h = outl[b, h].cpu().numpy()
        assert outl_h.tolist() == oracle.select(negm_h, o).tolist()
        qh = synth.to_host(q[b, h * n_rep:(h + 1) * n_rep])
        S_ref = oracle.chunk_scores(synth.to_host(Lm[b, h])[None], qh)
        assert max_rel(S_h, S_ref[0]) <= TOL["bf16"]
        want = oracle.expand_chunks(oracle.select(S_h, k_ch), outl_h, c, w.L)
        n = int(cnt[b, h])
        assert n == len(want) and rows[b, h, :n].cpu().numpy().tolist() == want.tolist()
        cols = slice(h * w.d_h, (h + 1) * w.d_h)
        ref = oracle.gather_attend_rows(synth.to_host(g["A_k"][b]), synth.to_host(g["A_v"][b]),
                                        synth.to_host(g["B_k"][b, layer][:, cols]), synth.to_host(g["B_v"][b, layer][:, cols]),
                                        qh, [want])
        got = synth.storage_to_f64(synth.to_host(out[b, h * n_rep:(h + 1) * n_rep]))
        assert max_rel(got, ref) <= TOL["bf16"], (b, h)


# ----------------------------------------------------------------- rotary embedding of the reconstructed rows
ROPE_CASES = {
    # name: workload fields, theta   (k ids per head are drawn at random over the whole context)
    "generic_f32_dh32": (dict(G=1, H_kv=2, H_q=4, d_h=32, r_k=8, r_v=8, L=5000, k=40, batch=2, dtype="f32"), 10000.0),
    "generic_bf16_dh64": (dict(G=1, H_kv=2, H_q=4, d_h=64, r_k=16, r_v=16, L=3000, k=70, batch=1, dtype="bf16"), 10000.0),
    "mfma_bf16_dh128": (dict(G=2, H_kv=2, H_q=8, d_h=128, r_k=64, r_v=32, L=70000, k=300, batch=2, dtype="bf16"), 500000.0),
    "mfma_bf16_long_rows": (dict(G=1, H_kv=1, H_q=4, d_h=128, r_k=32, r_v=32, L=131072, k=1100, batch=1, dtype="bf16"), 1000000.0),
}


@pytest.mark.parametrize("name", list(ROPE_CASES))
def test_gather_attend_with_counts_and_rope(name):
    torch = torch_mod()
    fields, theta = ROPE_CASES[name]
    w = workload(fields)
    case = synth.make_case(w, seed=70 + len(name))
    layer = w.G - 1
    rng = np.random.default_rng(len(name))
    idx = np.stack([np.stack([np.sort(rng.choice(w.L, size=w.k, replace=False)) for _ in range(w.H_kv)])
                    for _ in range(w.batch)]).astype(np.int32)
    idx[:, :, -1] = w.L - 1                                   # the largest position is always there
    counts = rng.integers(1, w.k + 1, size=(w.batch, w.H_kv)).astype(np.int32)
    counts[0, 0] = w.k
    shape = xb.Shape.of(w)
    dev = synth.to_device(case, w.dtype)
    ws = xb.alloc_workspace(shape)
    q = dev["q"][layer].contiguous()
    qh = synth.to_host(q)
    idx_d, cnt_d = torch.from_numpy(idx).cuda(), torch.from_numpy(counts).cuda()
    out = torch.zeros((w.batch, w.H_q, w.d_h), dtype=synth.torch_dtype(w.dtype), device="cuda")
    for use_counts, th in ((True, theta), (False, theta), (True, 0.0)):
        xb.xkv_gather_attend_ex(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, idx_d,
                                cnt_d if use_counts else None, th, out, ws)
        torch.cuda.synchronize()
        got = synth.storage_to_f64(synth.to_host(out))
        for b in range(w.batch):
            rows = [idx[b, g, :(counts[b, g] if use_counts else w.k)] for g in range(w.H_kv)]
            ref = oracle.gather_attend_rows(case["A_k"][b], case["A_v"][b], case["B_k"][b, layer], case["B_v"][b, layer],
                                            qh[b], rows, rope_theta=(th if th > 0 else None))
            assert max_rel(got[b], ref) <= TOL[w.dtype], (name, use_counts, th, b)


def test_landmark_step_with_rope_is_the_papers_arrangement():
    """Factors of pre-RoPE keys, landmarks of post-RoPE keys, rotation re-applied to the reconstructed rows: with every
    chunk selected the step equals dense attention over the rotated keys; with a budget it equals the oracle on the
    GPU's rows."""
    torch = torch_mod()
    theta, c, o = 500000.0, 8, 2
    w = workload(dict(G=1, H_kv=2, H_q=8, d_h=128, r_k=32, r_v=32, L=1200, k=1200, batch=1, dtype="bf16"))
    case = synth.make_case(w, seed=123)
    K_pre = keys_of(case, w, 0)                                               # [1][H_kv][L][d_h], storage form
    K_rope = np.stack([oracle.rope(synth.storage_to_f64(K_pre[0, g]), np.arange(w.L), theta) for g in range(w.H_kv)])
    K_rope_s = synth.to_storage(K_rope[None], w.dtype)
    dev = synth.to_device(case, w.dtype)
    K_dev = synth.to_device({"K": K_rope_s}, w.dtype)["K"]
    dt = synth.torch_dtype(w.dtype)
    q = dev["q"][0].contiguous()
    qh = synth.to_host(q)
    for k in (w.L, 160):
        shape = xb.Shape.of(w, k=k)
        n_c = w.L // c
        k_ch = oracle.chunk_budget(k, c, n_c)
        cap = (k_ch + o) * c
        ws = torch.empty(xb.xkv_landmark_workspace_bytes(shape, c, o), dtype=torch.uint8, device="cuda")
        Lm = torch.zeros((1, w.H_kv, n_c, w.d_h), dtype=dt, device="cuda")
        outl = torch.zeros((1, w.H_kv, o), dtype=torch.int32, device="cuda")
        xb.xkv_landmarks(shape, K_dev, c, o, Lm, None, outl, ws)
        out = torch.zeros((1, w.H_q, w.d_h), dtype=dt, device="cuda")
        rows = torch.zeros((1, w.H_kv, cap), dtype=torch.int32, device="cuda")
        cnt = torch.zeros((1, w.H_kv), dtype=torch.int32, device="cuda")
        xb.xkv_sr_decode_landmark(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, Lm, outl, c, o, out, rows,
                                  cnt, None, ws, rope_theta=theta)
        torch.cuda.synchronize()
        got = synth.storage_to_f64(synth.to_host(out))[0]
        rows_h, cnt_h = rows.cpu().numpy()[0], cnt.cpu().numpy()[0]
        row_lists = [rows_h[g, :cnt_h[g]] for g in range(w.H_kv)]
        ref = oracle.gather_attend_rows(case["A_k"][0], case["A_v"][0], case["B_k"][0, 0], case["B_v"][0, 0], qh[0],
                                        row_lists, rope_theta=theta)
        assert max_rel(got, ref) <= TOL["bf16"], k
        if k == w.L:
            assert all(rl.tolist() == list(range(w.L)) for rl in row_lists)
            K_flat = synth.storage_to_f64(K_rope_s[0]).transpose(1, 0, 2).reshape(w.L, w.H_kv * w.d_h)
            V_flat = oracle.reconstruct(case["A_v"][0], case["B_v"][0, 0])
            assert max_rel(got, oracle.dense(K_flat, V_flat, qh[0], w.H_kv)) <= TOL["bf16"]


@pytest.mark.parametrize("L,c,o,k", [(5, 8, 1, 3), (64, 8, 8, 64), (100, 1, 0, 7), (1000, 16, 0, 1)])
def test_landmark_selector_edge_shapes(L, c, o, k):
    """A context shorter than one chunk; every chunk an outlier; chunks of one token; a budget of one token."""
    torch = torch_mod()
    w = workload(dict(G=1, H_kv=2, H_q=4, d_h=128, r_k=16, r_v=16, L=L, k=k, batch=2, dtype="bf16"))
    case = synth.make_case(w, seed=L + c)
    K_host = keys_of(case, w, 0)
    shape = xb.Shape.of(w)
    dev = synth.to_device(case, w.dtype)
    K_dev = synth.to_device({"K": K_host}, w.dtype)["K"]
    dt = synth.torch_dtype(w.dtype)
    n_c = -(-L // c)
    k_ch = oracle.chunk_budget(k, c, n_c)
    cap = (k_ch + o) * c
    ws = torch.empty(xb.xkv_landmark_workspace_bytes(shape, c, o), dtype=torch.uint8, device="cuda")
    Lm = torch.zeros((w.batch, w.H_kv, n_c, w.d_h), dtype=dt, device="cuda")
    outl = torch.zeros((w.batch, w.H_kv, max(o, 1)), dtype=torch.int32, device="cuda")
    negm = torch.zeros((w.batch, w.H_kv, n_c), dtype=torch.float32, device="cuda")
    xb.xkv_landmarks(shape, K_dev, c, o, Lm, negm, outl if o else None, ws)
    q = dev["q"][0].contiguous()
    out = torch.zeros((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda")
    rows = torch.zeros((w.batch, w.H_kv, cap), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((w.batch, w.H_kv), dtype=torch.int32, device="cuda")
    S = torch.zeros((w.batch, w.H_kv, n_c), dtype=torch.float32, device="cuda")
    xb.xkv_sr_decode_landmark(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, Lm, outl if o else None, c, o,
                              out, rows, cnt, S, ws)
    torch.cuda.synchronize()
    qh, S_h, rows_h, cnt_h = synth.to_host(q), S.cpu().numpy(), rows.cpu().numpy(), cnt.cpu().numpy()
    outl_h, negm_h = outl.cpu().numpy(), negm.cpu().numpy()
    got = synth.storage_to_f64(synth.to_host(out))
    for b in range(w.batch):
        row_lists = []
        for g in range(w.H_kv):
            if o:
                assert outl_h[b, g].tolist() == oracle.select(negm_h[b, g], o).tolist()
            want = oracle.expand_chunks(oracle.select(S_h[b, g], k_ch), outl_h[b, g][:o], c, L)
            assert cnt_h[b, g] == len(want) and rows_h[b, g, :len(want)].tolist() == want.tolist()
            row_lists.append(want)
        ref = oracle.gather_attend_rows(case["A_k"][b], case["A_v"][b], case["B_k"][b, 0], case["B_v"][b, 0], qh[b],
                                        row_lists)
        assert max_rel(got[b], ref) <= TOL["bf16"]


@pytest.mark.parametrize("T", [1, 77, 700])
def test_landmark_step_with_rope_and_uncompressed_tail(T):
    """The paper's complete decode arrangement: landmark selection, rotation of the reconstructed rows, and the T most
    recent tokens kept uncompressed in the same softmax."""
    torch = torch_mod()
    theta, c, o = 500000.0, 8, 2
    w = workload(dict(G=1, H_kv=2, H_q=8, d_h=128, r_k=32, r_v=48, L=2000, k=200, batch=2, dtype="bf16"))
    case = synth.make_case(w, seed=300 + T)
    rng = np.random.default_rng(T)
    K_pre = keys_of(case, w, 0)
    K_rope = np.stack([[oracle.rope(synth.storage_to_f64(K_pre[b, g]), np.arange(w.L), theta) for g in range(w.H_kv)]
                       for b in range(w.batch)])
    K_tail_h = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)) * 0.5, w.dtype)
    V_tail_h = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)), w.dtype)
    dev = synth.to_device(case, w.dtype)
    extra = synth.to_device({"K": synth.to_storage(K_rope, w.dtype), "Kt": K_tail_h, "Vt": V_tail_h}, w.dtype)
    shape = xb.Shape.of(w)
    dt = synth.torch_dtype(w.dtype)
    n_c = w.L // c
    cap = (oracle.chunk_budget(w.k, c, n_c) + o) * c
    ws = torch.empty(xb.xkv_landmark_workspace_bytes(shape, c, o), dtype=torch.uint8, device="cuda")
    Lm = torch.zeros((w.batch, w.H_kv, n_c, w.d_h), dtype=dt, device="cuda")
    outl = torch.zeros((w.batch, w.H_kv, o), dtype=torch.int32, device="cuda")
    xb.xkv_landmarks(shape, extra["K"], c, o, Lm, None, outl, ws)
    q = dev["q"][0].contiguous()
    out = torch.zeros((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda")
    rows = torch.zeros((w.batch, w.H_kv, cap), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((w.batch, w.H_kv), dtype=torch.int32, device="cuda")
    xb.xkv_sr_decode_landmark(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, Lm, outl, c, o, out, rows, cnt,
                              None, ws, rope_theta=theta, K_tail=extra["Kt"], V_tail=extra["Vt"], T=T)
    torch.cuda.synchronize()
    got = synth.storage_to_f64(synth.to_host(out))
    rows_h, cnt_h, qh = rows.cpu().numpy(), cnt.cpu().numpy(), synth.to_host(q)
    for b in range(w.batch):
        row_lists = [rows_h[b, g, :cnt_h[b, g]] for g in range(w.H_kv)]
        ref = oracle.gather_attend_rows(case["A_k"][b], case["A_v"][b], case["B_k"][b, 0], case["B_v"][b, 0], qh[b],
                                        row_lists, rope_theta=theta, K_tail=K_tail_h[b], V_tail=V_tail_h[b])
        assert max_rel(got[b], ref) <= TOL["bf16"], (T, b)
        no_tail = oracle.gather_attend_rows(case["A_k"][b], case["A_v"][b], case["B_k"][b, 0], case["B_v"][b, 0], qh[b],
                                            row_lists, rope_theta=theta)
        assert np.abs(no_tail - ref).max() > 1e-3 * np.abs(ref).max()      # the tail does matter in this case
