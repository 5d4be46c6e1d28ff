"""GPU parity: libxkv (through its C ABI) against the CPU oracle on the same seeded inputs.

Selection is discontinuous, so parity is a chain of strict links (each stage is fed exactly
what the GPU fed the next one):
  (i)   xkv_score                      vs oracle steps 1-3            within tolerance
  (ii)  xkv_topk(S_gpu)                vs oracle.select(S_gpu)        identical sets
  (iii) xkv_gather_attend(idx_gpu)     vs oracle steps 5-6 on idx_gpu within tolerance
  (iv)  xkv_sr_decode end to end       vs the whole oracle            within tolerance where the
        score gap at the k-th place exceeds rounding (fp32 tiny case), else reported
Tolerance: max|gpu - ref| / max|ref| per tensor, 1e-5 for fp32 and 2e-2 for bf16 storage with
fp32 accumulation.
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


def run_stages(w, case, layer, scale=0.0):
    """Run every stage entry point plus the fused call on the device; return host copies."""
    torch = torch_mod()
    shape = xb.Shape.of(w, scale=scale)
    dev = synth.to_device(case, w.dtype)
    ws = xb.alloc_workspace(shape)
    dt = synth.torch_dtype(w.dtype)
    q = dev["q"][layer].contiguous()
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    out_stage = torch.empty((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda")
    xb.xkv_score(shape, layer, dev["A_k"], dev["B_k"], q, S, ws)
    xb.xkv_topk(shape, S, idx, ws)
    xb.xkv_gather_attend(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, idx, out_stage, ws)
    S2 = torch.empty_like(S)
    idx2 = torch.empty_like(idx)
    out_fused = torch.empty_like(out_stage)
    xb.xkv_sr_decode(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out_fused, idx2, S2, ws)
    out_noaux = torch.empty_like(out_stage)
    xb.xkv_sr_decode(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out_noaux, None, None, ws)
    torch.cuda.synchronize()
    return dict(S=S.cpu().numpy(), idx=idx.cpu().numpy(), out_stage=synth.storage_to_f64(synth.to_host(out_stage)),
                S_fused=S2.cpu().numpy(), idx_fused=idx2.cpu().numpy(),
                out_fused=synth.storage_to_f64(synth.to_host(out_fused)),
                out_noaux=synth.storage_to_f64(synth.to_host(out_noaux)))


def check_chain(w, case, layer, scale=None, e2e_strict=False):
    tol = TOL[w.dtype]
    sc = oracle.default_scale(w.d_h) if scale is None else scale
    got = run_stages(w, case, layer, 0.0 if scale is None else scale)
    report = {}
    for b in range(w.batch):
        A_k, A_v = case["A_k"][b], case["A_v"][b]
        B_k, B_v = case["B_k"][b, layer], case["B_v"][b, layer]
        q = case["q"][layer, b]
        # (i) scores
        S_ref = oracle.pooled_scores(A_k, B_k, q, w.H_kv, sc)
        err_s = max_rel(got["S"][b], S_ref)
        assert err_s <= tol, f"score seq {b}: {err_s}"
        # (ii) selection on the GPU's own scores: identical sets, k distinct ids, ascending order
        for g in range(w.H_kv):
            ref_idx = oracle.select(got["S"][b, g], w.k)
            np.testing.assert_array_equal(np.sort(got["idx"][b, g]), ref_idx)
            np.testing.assert_array_equal(got["idx"][b, g], ref_idx)  # library writes ascending ids
        # (iii) reconstruct + attend on the GPU's index sets
        out_ref = oracle.gather_attend(A_k, A_v, B_k, B_v, q, got["idx"][b], sc)
        err_o = max_rel(got["out_stage"][b], out_ref)
        assert err_o <= tol, f"gather_attend seq {b}: {err_o}"
        # (iv) end to end
        out_e2e, idx_e2e, _ = oracle.sr_decode(A_k, A_v, B_k, B_v, q, w.H_kv, w.k, sc)
        jac = np.mean([len(set(got["idx_fused"][b, g]) & set(idx_e2e[g])) /
                       len(set(got["idx_fused"][b, g]) | set(idx_e2e[g])) for g in range(w.H_kv)])
        err_e = max_rel(got["out_fused"][b], out_e2e)
        report[b] = dict(score=err_s, attend=err_o, e2e=err_e, jaccard=jac)
        if e2e_strict:
            assert jac == 1.0 and err_e <= tol, report[b]
    # the fused call must reproduce the staged calls bit for bit (same kernels, same inputs)
    np.testing.assert_array_equal(got["S_fused"], got["S"])
    np.testing.assert_array_equal(got["idx_fused"], got["idx"])
    np.testing.assert_array_equal(got["out_fused"], got["out_stage"])
    np.testing.assert_array_equal(got["out_noaux"], got["out_stage"])
    return report


# ------------------------------------------------------------------------------ SR chain
def test_tiny_fp32_config_end_to_end():
    """Benchmark configuration 1 (fp32): every link strict, end to end included.

    The seed is one where the gap between the k-th and (k+1)-th pooled score is far above fp32
    rounding, so the GPU and the oracle must pick the same tokens."""
    w = synth.TINY
    case = synth.make_case(w, seed=0)
    for layer in range(w.G):
        _, _, S32 = oracle.sr_decode(case["A_k"][0], case["A_v"][0], case["B_k"][0, layer], case["B_v"][0, layer],
                                     case["q"][layer, 0], w.H_kv, w.k)
        srt = np.sort(S32[0])[::-1]
        assert (srt[w.k - 1] - srt[w.k]) > 1e-4 * np.abs(srt).max(), "pick a seed with a clear gap"
        rep = check_chain(w, case, layer, e2e_strict=True)
        print("tiny", layer, rep)


SMALL = [
    # name, workload: sizes span several tiles with ragged tails
    ("llama_small_bf16", synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=128, r_v=192, batch=2, G=2)),
    ("qwen_small_bf16", synth.QWEN.with_(L=5001, k=257, r_k=128, r_v=64, batch=1, G=1)),
    ("odd_f32", synth.Workload("odd_f32", G=3, H_kv=3, H_q=6, d_h=64, r_k=40, r_v=24, L=777, k=33, batch=2,
                               dtype="f32", a_scale=1.0, sigma_decay=0.5, q_scale=1.0)),
    ("odd_bf16_dh96", synth.Workload("odd_bf16", G=1, H_kv=2, H_q=10, d_h=96, r_k=72, r_v=56, L=1300, k=64, batch=1,
                                     dtype="bf16", a_scale=0.2, sigma_decay=0.8, q_scale=0.3)),
    ("mha_f32", synth.Workload("mha_f32", G=1, H_kv=4, H_q=4, d_h=32, r_k=16, r_v=16, L=300, k=7, batch=3,
                               dtype="f32", a_scale=1.0, sigma_decay=1.0, q_scale=1.0)),
    # bf16 shapes that exercise the matrix-core paths: several head blocks, padded head slots, ragged rank tails
    ("gqa8_bf16", synth.Workload("gqa8_bf16", G=1, H_kv=8, H_q=64, d_h=128, r_k=80, r_v=48, L=2100, k=96, batch=2,
                                 dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    ("gqa16_bf16", synth.Workload("gqa16_bf16", G=1, H_kv=3, H_q=48, d_h=64, r_k=48, r_v=32, L=1111, k=40, batch=1,
                                  dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    ("mha_bf16", synth.Workload("mha_bf16", G=2, H_kv=20, H_q=20, d_h=64, r_k=32, r_v=64, L=900, k=50, batch=1,
                                dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    ("gqa2_bf16", synth.Workload("gqa2_bf16", G=1, H_kv=5, H_q=10, d_h=128, r_k=256, r_v=128, L=4097, k=300, batch=1,
                                 dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    # enough selected tokens (4 x 8 x 2100) for the eight-wavefront form of the gather-attend kernel (the smaller
    # cases above run its four-wavefront form), ragged last tile
    ("llama_k2100_bf16", synth.LLAMA_GROUP.with_(L=6000, k=2100, r_k=64, r_v=96, batch=4, G=1)),
]


@pytest.mark.parametrize("name,w", SMALL, ids=[n for n, _ in SMALL])
def test_small_shapes_chain(name, w):
    case = synth.make_case(w, seed=11)
    rep = check_chain(w, case, layer=w.G - 1)
    print(name, rep)


def test_peaked_softmax_case():
    """Same data with the logit scale raised so that softmax is dominated by a few tokens and
    selection matters for the output."""
    w = synth.LLAMA_GROUP.with_(L=2048, k=128, r_k=64, r_v=64, batch=1, G=1, q_scale=1.0, a_scale=1.0)
    case = synth.make_case(w, seed=5)
    rep = check_chain(w, case, layer=0, scale=4.0)
    print("peaked", rep)


@pytest.mark.parametrize("k_kind", ["k1", "kL"])
def test_degenerate_k(k_kind):
    w = synth.TINY.with_(L=200, k=1 if k_kind == "k1" else 200, G=1)
    case = synth.make_case(w, seed=2)
    rep = check_chain(w, case, layer=0)
    if k_kind == "kL":  # selecting everything: SR equals dense attention on the reconstruction
        got = run_stages(w, case, 0)
        K = oracle.reconstruct(case["A_k"][0], case["B_k"][0, 0])
        V = oracle.reconstruct(case["A_v"][0], case["B_v"][0, 0])
        ref = oracle.dense(K, V, case["q"][0, 0], w.H_kv)
        assert max_rel(got["out_fused"][0], ref) <= TOL["f32"]
    print(k_kind, rep)


# ------------------------------------------------------------------------------ top-k on arbitrary arrays
def topk_gpu(rows_np, k):
    torch = torch_mod()
    n_rows, L = rows_np.shape
    shape = xb.Shape(G=1, H_kv=n_rows, H_q=n_rows, d_h=64, r_k=8, r_v=8, L=L, k=k, batch=1, dtype="f32")
    ws = xb.alloc_workspace(shape)
    S = torch.from_numpy(np.ascontiguousarray(rows_np, np.float32)).cuda().view(1, n_rows, L)
    idx = torch.full((1, n_rows, k), -1, dtype=torch.int32, device="cuda")
    xb.xkv_topk(shape, S, idx, ws)
    first = idx.cpu().numpy()[0]
    idx.fill_(-1)
    xb.xkv_topk(shape, S, idx, ws)   # determinism run to run
    np.testing.assert_array_equal(idx.cpu().numpy()[0], first)
    return first


@pytest.mark.parametrize("L", [1, 63, 64, 255, 256, 257, 1000, 4096, 10007, 32769, 65536, 65537, 70001])
def test_topk_adversarial_arrays(L):
    rng = np.random.default_rng(L)
    rows = [
        rng.standard_normal(L),                                   # generic
        np.full(L, 0.75),                                         # all equal: smallest ids win
        rng.integers(0, 4, L).astype(np.float64),                 # many duplicates
        np.where(rng.random(L) < 0.5, 0.0, -0.0),                 # signed zeros
        rng.standard_normal(L) * 1e-42,                           # denormals
        np.arange(L, dtype=np.float64),                           # sorted
        -np.arange(L, dtype=np.float64),                          # reverse sorted
        np.abs(rng.standard_normal(L)) * 1e-3 + 1.0,              # values sharing the high key bytes
        -np.abs(rng.standard_normal(L)) - 5.0,                    # all negative
    ]
    rows = np.stack(rows).astype(np.float32)
    for k in sorted({1, min(2, L), max(1, L // 16), max(1, L // 2), max(1, L - 1), L}):
        got = topk_gpu(rows, k)
        for r in range(rows.shape[0]):
            np.testing.assert_array_equal(got[r], oracle.select(rows[r], k), err_msg=f"L={L} k={k} row={r}")


# ------------------------------------------------------------------------------ dense baseline and reconstruction
DENSE = [
    ("tiny_f32", synth.TINY.with_(L=700)),
    ("llama_bf16", synth.LLAMA_GROUP.with_(L=4100, batch=2, r_k=64, r_v=64, G=1)),
    ("qwen_bf16", synth.QWEN.with_(L=2500, k=100, batch=1, r_k=64, r_v=64, G=1)),
    # ranks that span several 128-rank groups (odd and even counts, ragged last group), several workgroup tiles
    ("llama_r304_r512_bf16", synth.LLAMA_GROUP.with_(L=1801, k=100, batch=2, r_k=304, r_v=512, G=2)),
]


@pytest.mark.parametrize("name,w", DENSE, ids=[n for n, _ in DENSE])
def test_reconstruct_and_dense_decode(name, w):
    torch = torch_mod()
    case = synth.make_case(w, seed=21)
    dev = synth.to_device(case, w.dtype)
    shape = xb.Shape.of(w)
    ws = xb.alloc_workspace(shape)
    dt = synth.torch_dtype(w.dtype)
    K = torch.empty((w.batch, w.H_kv, w.L, w.d_h), dtype=dt, device="cuda")
    V = torch.empty_like(K)
    xb.xkv_reconstruct(shape, 0, dev["A_k"], dev["B_k"], w.r_k, K)
    xb.xkv_reconstruct(shape, 0, dev["A_v"], dev["B_v"], w.r_v, V)
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda")
    xb.xkv_dense_decode(shape, K, V, dev["q"][0].contiguous(), out, ws)
    torch.cuda.synchronize()
    Kh, Vh = synth.storage_to_f64(synth.to_host(K)), synth.storage_to_f64(synth.to_host(V))
    outh = synth.storage_to_f64(synth.to_host(out))
    for b in range(w.batch):
        K_ref = oracle.reconstruct(case["A_k"][b], case["B_k"][b, 0])      # [L][d]
        V_ref = oracle.reconstruct(case["A_v"][b], case["B_v"][b, 0])
        K_lm = Kh[b].transpose(1, 0, 2).reshape(w.L, w.d)                   # head-major -> [L][d]
        V_lm = Vh[b].transpose(1, 0, 2).reshape(w.L, w.d)
        assert max_rel(K_lm, K_ref) <= (2.0 ** -8 if w.dtype == "bf16" else 1e-5)
        assert max_rel(V_lm, V_ref) <= (2.0 ** -8 if w.dtype == "bf16" else 1e-5)
        # the dense kernel is checked on exactly the cache it read
        ref = oracle.dense(K_lm, V_lm, case["q"][0, b], w.H_kv)
        assert max_rel(outh[b], ref) <= TOL[w.dtype], name


# ------------------------------------------------------------------------------ full benchmark shapes
def test_llama_group_full_size():
    """Benchmark configuration 2 at full size (L=32768, r=512, k=2048, bf16), whole oracle."""
    w = synth.LLAMA_GROUP.with_(G=1)
    case = synth.make_case(w, seed=7)
    rep = check_chain(w, case, layer=0)
    print("llama_group_full", rep)


def _full_size_sampled(w, seqs, seed, scale=None, whole_rows=True):
    """One layer of a benchmark configuration at full size, in the launch configuration bench.py times (fused
    xkv_sr_decode_packed on device-generated factors, and xkv_sr_decode beside it), checked on the sampled sequences: every pooled score of the sequence
    (whole_rows; else token ranges at the start, in the middle and at the end), the complete selection (against the
    oracle's selection on the GPU's own scores), and the attention outputs."""
    torch = torch_mod()
    dev = synth.make_group_device(w, seed=seed)
    shape = xb.Shape.of(w, scale=0.0 if scale is None else scale)
    ws = xb.alloc_workspace(shape)
    layer = w.G - 1
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=synth.torch_dtype(w.dtype), device="cuda")
    # the call the benchmark times: B_l re-ordered once for the group, then the packed step (where the shape has one)
    if w.dtype == "bf16" and w.d_h == 128 and w.r_k % 16 == 0 and w.r_v % 16 == 0:
        packed = torch.empty(xb.xkv_packed_b_bytes(shape), dtype=torch.uint8, device="cuda")
        xb.xkv_pack_b(shape, dev["B_k"], dev["B_v"], packed)
        xb.xkv_sr_decode_packed(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], packed, dev["q"][layer].contiguous(),
                                out, idx, S, ws)
        torch.cuda.synchronize()
        packed_result = (out.clone(), idx.clone(), S.clone())
        del packed
        out.zero_(), idx.zero_(), S.zero_()
    else:
        packed_result = None
    xb.xkv_sr_decode(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], dev["q"][layer].contiguous(), out,
                     idx, S, ws)
    torch.cuda.synchronize()
    if packed_result is not None:    # same kernels on the same operands: the two calls agree bit for bit
        for a, b_ in zip(packed_result, (out, idx, S)):
            assert torch.equal(a, b_)
        del packed_result
    scale = oracle.default_scale(w.d_h) if scale is None else scale
    mid = w.L // 2
    ranges = [(0, w.L)] if whole_rows else [(0, 256), (mid - 128, mid + 128), (w.L - 256, w.L)]
    report = {}
    for b in seqs:
        B_k = synth.to_host(dev["B_k"][b, layer])
        B_v = synth.to_host(dev["B_v"][b, layer])
        q = synth.to_host(dev["q"][layer, b])
        err_s = 0.0
        for lo, hi in ranges:
            ref = oracle.pooled_scores(synth.to_host(dev["A_k"][b, lo:hi]), B_k, q, w.H_kv, scale)
            err_s = max(err_s, max_rel(S[b, :, lo:hi].cpu().numpy(), ref))
            assert err_s <= TOL[w.dtype], (b, lo, err_s)
        S_b, idx_b = S[b].cpu().numpy(), idx[b].cpu().numpy()
        for g in range(w.H_kv):
            np.testing.assert_array_equal(idx_b[g], oracle.select(S_b[g], w.k), err_msg=f"seq {b} head {g}")
        ref_out = oracle.gather_attend(synth.to_host(dev["A_k"][b]), synth.to_host(dev["A_v"][b]), B_k, B_v, q, idx_b,
                                       scale)
        err = max_rel(synth.storage_to_f64(synth.to_host(out[b])), ref_out)
        assert err <= TOL[w.dtype], (b, err)
        report[b] = dict(score=err_s, attend=err)
    return report


def test_llama_full_size_sampled():
    """Benchmark configuration 3 (batch 16, L = 65536, r = 512, k = 4096): first and last sequence, every token's
    pooled score (the four-rank-group instantiation of the streaming score kernel that the benchmark times)."""
    print(_full_size_sampled(synth.LLAMA_FULL, seqs=(0, synth.LLAMA_FULL.batch - 1), seed=31))


def test_qwen_full_size_sampled():
    """Benchmark configuration 4 (batch 4, L = 131072, r = 384, k = 4096, 7 query heads per KV head): two of the
    four sequences, every token's pooled score."""
    print(_full_size_sampled(synth.QWEN, seqs=(0, synth.QWEN.batch - 1), seed=32))


def test_llama_full_size_peaked_softmax():
    """Configuration 3's size and launch configuration with the logit scale raised 20000-fold: the workload's own
    logits have a spread of 2e-4 (softmax nearly uniform), here it is about 4, so that a few dozen of the 4096
    selected tokens carry the output and a mis-selected or mis-weighted token would show."""
    w = synth.LLAMA_FULL
    rep = _full_size_sampled(w, seqs=(w.batch - 1,), seed=33, scale=20000.0 / np.sqrt(w.d_h), whole_rows=False)
    print("peaked full size", rep)


# The sweep (benchmark configuration 5) publishes points at ranks 256, 512, 768, budgets from 1.5 % to 12.5 %, batches
# up to 32 and contexts up to 131072; the corners that no other test reaches, each in the sweep's own launch
# configuration (device-generated factors, fused call), on a sampled sequence.
SWEEP_CORNERS = [
    # rank 768: six rank groups per product in the gather-reconstruct kernel, the four-wavefront score stream
    ("r768_L64k_b16_k6pct", synth.llama_sweep_point(65536, 16, 768, 0.0625), (15,)),
    # the paper's own ranks at window 4, r_K : r_V = 1 : 1.5 (Sec. 4), on the bf16 gather-reconstruct path
    ("r384_576_L64k_b16", synth.LLAMA_FULL.with_(r_k=384, r_v=576, a_scale=384 ** -0.5), (7,)),
    # batch 32 x L = 131072: A holds more than 2^31 elements; the last sequence lies beyond that offset
    ("r512_L128k_b32_k3pct", synth.llama_sweep_point(131072, 32, 512, 0.03), (31,)),
    # smallest rank and budget, short context, single sequence (the four-wavefront gather kernel, short score kernel)
    ("r256_L16k_b1_k1.5pct", synth.llama_sweep_point(16384, 1, 256, 0.015), (0,)),
    # largest budget at rank 768 (the point where SR moves more bytes than dense attention)
    ("r768_L32k_b4_k12pct", synth.llama_sweep_point(32768, 4, 768, 0.125), (3,)),
]


@pytest.mark.parametrize("name,w,seqs", SWEEP_CORNERS, ids=[c[0] for c in SWEEP_CORNERS])
def test_sweep_corner_full_size_sampled(name, w, seqs):
    rep = _full_size_sampled(w.with_(n_groups=1), seqs=seqs, seed=41, whole_rows=w.L <= 65536)
    print(name, rep)


GA_RANKS = [
    ("r768_bf16", synth.LLAMA_GROUP.with_(L=9000, k=2100, r_k=768, r_v=768, batch=4, G=1, a_scale=768 ** -0.5)),
    ("r384_576_bf16", synth.LLAMA_GROUP.with_(L=9000, k=2100, r_k=384, r_v=576, batch=4, G=1, a_scale=384 ** -0.5)),
    ("r448_288_qwen_bf16", synth.QWEN.with_(L=7001, k=1111, r_k=448, r_v=288, batch=2, G=1, a_scale=448 ** -0.5)),
    # group counts (K, V) of the gather-reconstruct kernel: (1, 1) and (3, 3), where the softmax falls between the two
    # groups of one step; (2, 1) and (1, 2), where V is padded by a zero group; (3, 2), odd K with an even rest
    ("r128_128_bf16", synth.LLAMA_GROUP.with_(L=5000, k=700, r_k=128, r_v=128, batch=3, G=2, a_scale=128 ** -0.5)),
    ("r384_384_bf16", synth.LLAMA_GROUP.with_(L=5000, k=700, r_k=384, r_v=384, batch=3, G=2, a_scale=384 ** -0.5)),
    ("r256_128_bf16", synth.LLAMA_GROUP.with_(L=5000, k=700, r_k=256, r_v=128, batch=3, G=2, a_scale=256 ** -0.5)),
    ("r112_240_bf16", synth.LLAMA_GROUP.with_(L=5000, k=700, r_k=112, r_v=240, batch=3, G=2, a_scale=112 ** -0.5)),
    ("r368_256_bf16", synth.LLAMA_GROUP.with_(L=5000, k=700, r_k=368, r_v=256, batch=3, G=2, a_scale=368 ** -0.5)),
]


@pytest.mark.parametrize("name,w", GA_RANKS, ids=[n for n, _ in GA_RANKS])
def test_large_and_unequal_ranks_chain(name, w):
    """Every link of the chain, every sequence, on host-generated inputs at rank 768, at r_K : r_V = 1 : 1.5 and at
    ranks that are not whole 128-rank groups (bf16 gather-reconstruct kernel with six rank groups, with different group
    counts for K and V, with ragged last groups)."""
    case = synth.make_case(w, seed=13)
    rep = check_chain(w, case, layer=w.G - 1)
    print(name, rep)


# ------------------------------------------------------------------------------ B_l packed once per prompt
PACKED = [
    ("llama_small", synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=128, r_v=192, batch=2, G=3)),
    ("qwen_ragged_ranks", synth.QWEN.with_(L=5001, k=257, r_k=448, r_v=288, batch=2, G=2, a_scale=448 ** -0.5)),
    ("llama_k2100", synth.LLAMA_GROUP.with_(L=6000, k=2100, r_k=64, r_v=96, batch=4, G=2)),
]


@pytest.mark.parametrize("name,w", PACKED, ids=[n for n, _ in PACKED])
def test_packed_b_step_matches_plain_step(name, w):
    """xkv_pack_b once, then xkv_sr_decode_packed for every layer of the group: outputs, selections and scores
    bit for bit those of xkv_sr_decode (same kernels, same operands), and the outputs against the oracle on the
    step's own selection."""
    torch = torch_mod()
    case = synth.make_case(w, seed=19)
    dev = synth.to_device(case, w.dtype)
    shape = xb.Shape.of(w)
    ws = xb.alloc_workspace(shape)
    packed = torch.full((xb.xkv_packed_b_bytes(shape),), 0xAB, dtype=torch.uint8, device="cuda")
    xb.xkv_pack_b(shape, dev["B_k"], dev["B_v"], packed)
    dt = synth.torch_dtype(w.dtype)
    for layer in range(w.G):
        q = dev["q"][layer].contiguous()
        res = []
        for which in ("plain", "packed"):
            out = torch.full((w.batch, w.H_q, w.d_h), float("nan"), dtype=dt, device="cuda")
            idx = torch.full((w.batch, w.H_kv, w.k), -1, dtype=torch.int32, device="cuda")
            S = torch.full((w.batch, w.H_kv, w.L), float("nan"), dtype=torch.float32, device="cuda")
            if which == "plain":
                xb.xkv_sr_decode(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out, idx, S, ws)
            else:
                xb.xkv_sr_decode_packed(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], packed, q, out, idx, S, ws)
            torch.cuda.synchronize()
            res.append((synth.to_host(out), idx.cpu().numpy(), S.cpu().numpy()))
        for a, b_ in zip(res[0], res[1]):
            np.testing.assert_array_equal(a, b_)
        out_h, idx_h, _ = res[1]
        for b in range(w.batch):
            ref = oracle.gather_attend(case["A_k"][b], case["A_v"][b], case["B_k"][b, layer], case["B_v"][b, layer],
                                       case["q"][layer, b], idx_h[b])
            assert max_rel(synth.storage_to_f64(out_h[b]), ref) <= TOL[w.dtype], (name, layer, b)


def test_packed_b_rejects_shapes_of_the_general_kernels():
    torch_mod()
    with pytest.raises(xb.XkvError) as e:
        xb.xkv_packed_b_bytes(xb.Shape.of(synth.TINY))
    assert e.value.status == xb.XKV_ERR_UNSUPPORTED


# ------------------------------------------------------------------------------ uncompressed tail of recent tokens
TAIL = [
    ("tiny_f32", synth.TINY.with_(L=700, k=40), 37),
    ("llama_bf16", synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=128, r_v=192, batch=2, G=1), 1),
    ("llama_bf16_long_tail", synth.LLAMA_GROUP.with_(L=2000, k=300, r_k=64, r_v=64, batch=1, G=1), 1700),
    ("qwen_bf16", synth.QWEN.with_(L=2500, k=100, batch=2, r_k=64, r_v=64, G=1), 129),
]


@pytest.mark.parametrize("name,w,T", TAIL, ids=[n for n, _, _ in TAIL])
def test_sr_decode_with_uncompressed_tail(name, w, T):
    """xkv_sr_decode_tail: same scores and selection as the plain step, output against the oracle's attention over
    the selected rows plus the tail (fed the GPU's own index sets); T = 0 reproduces xkv_sr_decode bit for bit."""
    torch = torch_mod()
    case = synth.make_case(w, seed=23)
    dev = synth.to_device(case, w.dtype)
    rng = np.random.default_rng(5)
    K_t = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)) * 0.3, w.dtype)
    V_t = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)), w.dtype)
    tail = synth.to_device({"K": K_t, "V": V_t}, w.dtype)
    shape = xb.Shape.of(w)
    ws = xb.alloc_workspace(shape)
    dt = synth.torch_dtype(w.dtype)
    q = dev["q"][0].contiguous()
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda")
    out0, out_plain = torch.empty_like(out), torch.empty_like(out)
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    idx_plain = torch.empty_like(idx)
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    xb.xkv_sr_decode_tail(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, tail["K"], tail["V"], T, out, idx,
                          S, ws)
    xb.xkv_sr_decode_tail(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, None, None, 0, out0, None, None,
                          ws)
    xb.xkv_sr_decode(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out_plain, idx_plain, None, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(synth.to_host(out0), synth.to_host(out_plain))
    np.testing.assert_array_equal(idx.cpu().numpy(), idx_plain.cpu().numpy())
    if w.dtype == "bf16" and w.d_h == 128 and w.r_k % 16 == 0 and w.r_v % 16 == 0:
        # the same step on B_l re-ordered once for the group: bit for bit the same
        packed = torch.full((xb.xkv_packed_b_bytes(shape),), 0xAB, dtype=torch.uint8, device="cuda")
        xb.xkv_pack_b(shape, dev["B_k"], dev["B_v"], packed)
        out_p, idx_p, S_p = torch.empty_like(out), torch.empty_like(idx), torch.empty_like(S)
        xb.xkv_sr_decode_tail_packed(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], packed, q, tail["K"], tail["V"], T,
                                     out_p, idx_p, S_p, ws)
        torch.cuda.synchronize()
        assert torch.equal(out_p, out) and torch.equal(idx_p, idx) and torch.equal(S_p, S)
    outh, idxh, Sh = synth.storage_to_f64(synth.to_host(out)), idx.cpu().numpy(), S.cpu().numpy()
    for b in range(w.batch):
        for g in range(w.H_kv):
            np.testing.assert_array_equal(idxh[b, g], oracle.select(Sh[b, g], w.k))
        ref = oracle.gather_attend_tail(case["A_k"][b], case["A_v"][b], case["B_k"][b, 0], case["B_v"][b, 0],
                                        case["q"][0, b], idxh[b], K_t[b], V_t[b])
        assert max_rel(outh[b], ref) <= TOL[w.dtype], (name, b)


# ------------------------------------------------------------------------------ error paths (host side, no launch)
def test_error_codes():
    torch = torch_mod()
    w = synth.TINY
    shape = xb.Shape.of(w)
    ws = xb.alloc_workspace(shape)
    t = torch.zeros(16, device="cuda")
    with pytest.raises(xb.XkvError) as e:
        xb.xkv_topk(xb.Shape.of(w, k=w.L + 1), t, t, ws)
    assert e.value.status == xb.XKV_ERR_INVALID_ARG
    with pytest.raises(xb.XkvError) as e:
        xb.xkv_topk(shape, t, t, torch.empty(256, dtype=torch.uint8, device="cuda")[:16])
    assert e.value.status == xb.XKV_ERR_WORKSPACE
    with pytest.raises(xb.XkvError) as e:
        xb.xkv_topk(shape, None, t, ws)
    assert e.value.status == xb.XKV_ERR_INVALID_ARG
    with pytest.raises(xb.XkvError) as e:
        xb.xkv_sr_decode(shape, w.G, t, t, t, t, t, t, None, None, ws)   # layer out of range
    assert e.value.status == xb.XKV_ERR_INVALID_ARG
    xb.xkv_topk(xb.Shape.of(w, batch=0), t, t, ws)                         # empty batch: no-op
    torch.cuda.synchronize()


@pytest.mark.gpu
@pytest.mark.parametrize("r_k,H_kv,H_q", [(48, 2, 8), (256, 4, 8), (320, 5, 10)])
def test_score_long_stream(r_k, H_kv, H_q):
    """Score stage on a shape long enough for the streaming score kernel (one, two or three 128-rank groups per tile,
    ragged last tile), every pooled score against the oracle."""
    w = synth.Workload("long_stream", G=2, H_kv=H_kv, H_q=H_q, d_h=64, r_k=r_k, r_v=32, L=131072 + 5, k=64, batch=4,
                       dtype="bf16", a_scale=r_k ** -0.5, sigma_decay=0.8, q_scale=0.125)
    case = synth.make_case(w, seed=11)
    dev = synth.to_device(case, w.dtype)
    shape = xb.Shape.of(w)
    ws = xb.alloc_workspace(shape)
    torch = torch_mod()
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    layer = 1
    xb.xkv_score(shape, layer, dev["A_k"], dev["B_k"], dev["q"][layer].contiguous(), S, ws)
    torch.cuda.synchronize()
    got = S.cpu().numpy()
    scale = 1.0 / np.sqrt(w.d_h)
    for b in range(w.batch):
        ref = oracle.pooled_scores(synth.storage_to_f64(case["A_k"][b]), synth.storage_to_f64(case["B_k"][b, layer]),
                                   synth.storage_to_f64(case["q"][layer, b]), w.H_kv, scale)
        err = max_rel(got[b], ref)
        assert err <= TOL[w.dtype], (b, err)


@pytest.mark.gpu
@pytest.mark.parametrize("r_k,H_kv,H_q", [(48, 2, 8), (320, 5, 10)])
def test_long_stream_chain(r_k, H_kv, H_q):
    """Whole chain on a long-stream shape: here the score kernel also produces the first radix pass of the
    selection, so the fused call must still give exactly the ids the oracle selects from the same scores."""
    w = synth.Workload("long_stream_chain", G=2, H_kv=H_kv, H_q=H_q, d_h=64, r_k=r_k, r_v=64, L=131072 + 5, k=1000,
                       batch=4, dtype="bf16", a_scale=r_k ** -0.5, sigma_decay=0.8, q_scale=0.125)
    case = synth.make_case(w, seed=12)
    check_chain(w, case, layer=0)


@pytest.mark.gpu
def test_score_long_stream_large_rank():
    """Rank 768 leaves LDS room for only four wavefront tiles in the streaming score kernel: that variant, on
    device-generated inputs, checked on token ranges at the start, in the middle and at the ragged end."""
    torch = torch_mod()
    w = synth.Workload("long_stream_r768", G=1, H_kv=6, H_q=12, d_h=128, r_k=768, r_v=32, L=131072 + 9, k=64, batch=4,
                       dtype="bf16", a_scale=768 ** -0.5, sigma_decay=0.8, q_scale=128 ** -0.5)
    dev = synth.make_group_device(w, seed=21)
    shape = xb.Shape.of(w)
    ws = xb.alloc_workspace(shape)
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    xb.xkv_score(shape, 0, dev["A_k"], dev["B_k"], dev["q"][0].contiguous(), S, ws)
    torch.cuda.synchronize()
    scale = 1.0 / np.sqrt(w.d_h)
    ranges = [(0, 300), (65536 - 150, 65536 + 150), (w.L - 300, w.L)]
    for b in (0, w.batch - 1):
        B_k = synth.storage_to_f64(synth.to_host(dev["B_k"][b, 0]))
        q = synth.storage_to_f64(synth.to_host(dev["q"][0, b]))
        for lo, hi in ranges:
            A_rows = synth.storage_to_f64(synth.to_host(dev["A_k"][b, lo:hi]))
            ref = oracle.pooled_scores(A_rows, B_k, q, w.H_kv, scale)
            got = S[b, :, lo:hi].cpu().numpy()
            err = max_rel(got, ref)
            assert err <= TOL[w.dtype], (b, lo, err)


def test_step_can_be_recorded_into_a_graph_and_replayed():
    """The calls allocate nothing and synchronise nothing: a whole step can be recorded once and replayed.  Every replay
    is compared with the eager result, with the program's own eager work and synchronisations in between."""
    torch = torch_mod()
    w = synth.LLAMA_GROUP.with_(L=4096, k=512, batch=2)
    case = synth.make_case(w, seed=17)
    shape = xb.Shape.of(w)
    dev = synth.to_device(case, w.dtype)
    ws = xb.alloc_workspace(shape)
    dt = synth.torch_dtype(w.dtype)
    qs = [dev["q"][l].contiguous() for l in range(w.G)]
    outs = [torch.zeros((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda") for _ in range(w.G)]
    idxs = [torch.zeros((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda") for _ in range(w.G)]

    def step():
        for l in range(w.G):
            xb.xkv_sr_decode(shape, l, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], qs[l], outs[l], idxs[l], None, ws)

    step()
    torch.cuda.synchronize()
    want_out = [o.clone() for o in outs]
    want_idx = [i.clone() for i in idxs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        for o, i in zip(outs, idxs):
            o.zero_()
            i.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(w.G):
            assert torch.equal(outs[l], want_out[l]) and torch.equal(idxs[l], want_idx[l]), (rep, l)
        step()                       # eager work between the replays
        torch.cuda.synchronize()
