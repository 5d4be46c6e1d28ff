"""GPU parity of the absorbed form of the SR step (xkv_head_scores, xkv_attend_absorbed, xkv_sr_decode_absorbed)
against the CPU oracle, through the C ABI.

Links, each fed exactly what the GPU fed the next stage:
  (i)   xkv_head_scores                 vs oracle.head_scores               within tolerance; padding zero; the pooled
                                                                            score is bit for bit the max of the heads
  (ii)  xkv_topk(S_gpu)                 vs oracle.select(S_gpu)             identical sets
  (iii) xkv_attend_absorbed(idx_gpu)    vs oracle.gather_attend on idx_gpu  within tolerance (the reference is the
        reconstruct-then-attend definition, not the absorbed algebra, so the identity itself is under test too)
  (iv)  xkv_sr_decode_absorbed          reproduces the staged calls bit for bit
Tolerance as for the gather-reconstruct path: 1e-5 (fp32), 2e-2 (bf16 storage, fp32 accumulation).
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


def alloc_ws(shape):
    import torch
    return torch.empty(max(xb.xkv_absorbed_workspace_bytes(shape), 256), dtype=torch.uint8, device="cuda")


def run_absorbed(w, dev, layer, scale=0.0):
    torch = torch_mod()
    shape = xb.Shape.of(w, scale=scale)
    ws = alloc_ws(shape)
    dt = synth.torch_dtype(w.dtype)
    nrp = xb.head_pitch(shape)
    q = dev["q"][layer].contiguous()
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    heads = torch.full((w.batch, w.H_kv, w.L, nrp), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    out_stage = torch.empty((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda")
    xb.xkv_head_scores(shape, layer, dev["A_k"], dev["B_k"], q, S, heads, ws)
    xb.xkv_topk(shape, S, idx, ws)
    xb.xkv_attend_absorbed(shape, layer, dev["A_v"], dev["B_v"], heads, idx, out_stage, ws)
    S2, idx2, out_fused = torch.empty_like(S), torch.empty_like(idx), torch.empty_like(out_stage)
    xb.xkv_sr_decode_absorbed(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out_fused, idx2, S2, ws)
    out_noaux = torch.empty_like(out_stage)
    xb.xkv_sr_decode_absorbed(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out_noaux, None, None, ws)
    torch.cuda.synchronize()
    return dict(S=S, heads=heads, idx=idx, out_stage=out_stage, S_fused=S2, idx_fused=idx2, out_fused=out_fused,
                out_noaux=out_noaux, nrp=nrp, shape=shape)


def check_chain(w, case, layer, scale=None):
    tol = TOL[w.dtype]
    sc = oracle.default_scale(w.d_h) if scale is None else scale
    dev = synth.to_device(case, w.dtype)
    got = run_absorbed(w, dev, layer, 0.0 if scale is None else scale)
    n_rep = w.H_q // w.H_kv
    heads = got["heads"].cpu().numpy()
    S = got["S"].cpu().numpy()
    idx = got["idx"].cpu().numpy()
    out = synth.storage_to_f64(synth.to_host(got["out_stage"]))
    # the pooled score is the maximum of exactly the stored head scores; the padding is zero
    np.testing.assert_array_equal(S, heads[..., :n_rep].max(axis=-1))
    assert not np.isnan(heads).any()
    np.testing.assert_array_equal(heads[..., n_rep:], 0.0)
    report = {}
    for b in range(w.batch):
        A_k, A_v = case["A_k"][b], case["A_v"][b]
        B_k, B_v = case["B_k"][b, layer], case["B_v"][b, layer]
        q = case["q"][layer, b]
        s_ref = oracle.head_scores(A_k, B_k, q, w.H_kv, sc)                      # [H_q][L]
        s_gpu = heads[b, :, :, :n_rep].transpose(0, 2, 1).reshape(w.H_q, w.L)    # head h = g * n_rep + hh
        err_s = max_rel(s_gpu, s_ref)
        assert err_s <= tol, f"head scores seq {b}: {err_s}"
        for g in range(w.H_kv):
            np.testing.assert_array_equal(idx[b, g], oracle.select(S[b, g], w.k))
        ref = oracle.gather_attend(A_k, A_v, B_k, B_v, q, idx[b], sc)
        err_o = max_rel(out[b], ref)
        assert err_o <= tol, f"absorbed attention seq {b}: {err_o}"
        report[b] = dict(heads=err_s, attend=err_o)
    for a, b_ in (("S_fused", "S"), ("idx_fused", "idx")):
        np.testing.assert_array_equal(got[a].cpu().numpy(), got[b_].cpu().numpy())
    np.testing.assert_array_equal(synth.to_host(got["out_fused"]), synth.to_host(got["out_stage"]))
    np.testing.assert_array_equal(synth.to_host(got["out_noaux"]), synth.to_host(got["out_stage"]))
    return report


SMALL = [
    ("tiny_f32", synth.TINY),
    ("llama_small_bf16", synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=128, r_v=192, batch=2, G=2)),
    ("qwen_small_bf16", synth.QWEN.with_(L=5001, k=257, r_k=128, r_v=64, batch=1, G=1)),
    ("odd_f32", synth.Workload("odd_f32", G=3, H_kv=3, H_q=6, d_h=64, r_k=40, r_v=24, L=777, k=33, batch=2,
                               dtype="f32", a_scale=1.0, sigma_decay=0.5, q_scale=1.0)),
    ("odd_bf16_dh96", synth.Workload("odd_bf16", G=1, H_kv=2, H_q=10, d_h=96, r_k=72, r_v=56, L=1300, k=64, batch=1,
                                     dtype="bf16", a_scale=0.2, sigma_decay=0.8, q_scale=0.3)),
    ("mha_f32", synth.Workload("mha_f32", G=1, H_kv=4, H_q=4, d_h=32, r_k=16, r_v=16, L=300, k=7, batch=3,
                               dtype="f32", a_scale=1.0, sigma_decay=1.0, q_scale=1.0)),
    ("gqa16_bf16", synth.Workload("gqa16_bf16", G=1, H_kv=3, H_q=48, d_h=64, r_k=48, r_v=32, L=1111, k=40, batch=1,
                                  dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    ("gqa2_bf16", synth.Workload("gqa2_bf16", G=1, H_kv=5, H_q=10, d_h=128, r_k=256, r_v=128, L=4097, k=300, batch=1,
                                 dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    # several column blocks of A^V (r_v > 512 for bf16, > 256 for fp32) with a ragged last block, several splits
    ("wide_rv_bf16", synth.LLAMA_GROUP.with_(L=2500, k=700, r_k=64, r_v=776, batch=1, G=1)),
    ("wide_rv_f32", synth.Workload("wide_rv_f32", G=1, H_kv=6, H_q=12, d_h=64, r_k=32, r_v=300, L=900, k=130, batch=1,
                                   dtype="f32", a_scale=1.0, sigma_decay=0.5, q_scale=1.0)),
    # many selected tokens: splits of 512 with a ragged last one, d_h = 256
    ("k2100_dh256_bf16", synth.Workload("k2100", G=1, H_kv=2, H_q=8, d_h=256, r_k=64, r_v=96, L=6000, k=2100, batch=2,
                                        dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
]


@pytest.mark.parametrize("name,w", SMALL, ids=[n for n, _ in SMALL])
def test_absorbed_chain_small_shapes(name, w):
    case = synth.make_case(w, seed=13)
    print(name, check_chain(w, case, layer=w.G - 1), flush=True)


def test_absorbed_peaked_softmax():
    w = synth.LLAMA_GROUP.with_(L=2048, k=128, r_k=64, r_v=64, batch=1, G=1, q_scale=1.0, a_scale=1.0)
    case = synth.make_case(w, seed=5)
    print("peaked", check_chain(w, case, layer=0, scale=4.0), flush=True)


@pytest.mark.parametrize("k_kind", ["k1", "kL"])
def test_absorbed_degenerate_k(k_kind):
    w = synth.TINY.with_(L=200, k=1 if k_kind == "k1" else 200, G=1)
    case = synth.make_case(w, seed=2)
    print(k_kind, check_chain(w, case, layer=0), flush=True)


def test_absorbed_rejects_ragged_rows_and_small_workspace():
    torch = torch_mod()
    w = synth.TINY.with_(r_v=18, G=1)                       # fp32 rows that are not whole 16-byte pieces
    with pytest.raises(xb.XkvError) as ei:
        xb.xkv_absorbed_workspace_bytes(xb.Shape.of(w))
    assert ei.value.status == xb.XKV_ERR_UNSUPPORTED
    w = synth.TINY.with_(G=1)
    shape = xb.Shape.of(w)
    case = synth.make_case(w, seed=1)
    dev = synth.to_device(case, w.dtype)
    small = xb.alloc_workspace(shape)                       # the ordinary workspace is too small for the absorbed calls
    assert small.numel() < xb.xkv_absorbed_workspace_bytes(shape)
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=torch.float32, device="cuda")
    with pytest.raises(xb.XkvError) as ei:
        xb.xkv_sr_decode_absorbed(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], dev["q"][0].contiguous(), out,
                                  None, None, small)
    assert ei.value.status == xb.XKV_ERR_WORKSPACE


TAIL = [
    ("tiny_f32", synth.TINY.with_(L=700, k=40), 37),
    ("llama_bf16", synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=128, r_v=192, batch=2, G=1), 1),
    ("llama_bf16_long_tail", synth.LLAMA_GROUP.with_(L=2000, k=300, r_k=64, r_v=64, batch=1, G=1), 1700),
    ("qwen_bf16", synth.QWEN.with_(L=2500, k=100, batch=2, r_k=64, r_v=64, G=1), 129),
]


@pytest.mark.parametrize("name,w,T", TAIL, ids=[n for n, _, _ in TAIL])
def test_absorbed_with_uncompressed_tail(name, w, T):
    """Selected rows in the absorbed form plus T uncompressed recent tokens in one softmax, against the oracle's
    attention over reconstructed rows and tail (fed the GPU's own index sets); T = 0 is the plain absorbed step."""
    torch = torch_mod()
    case = synth.make_case(w, seed=23)
    dev = synth.to_device(case, w.dtype)
    rng = np.random.default_rng(5)
    K_t = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)) * 0.3, w.dtype)
    V_t = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)), w.dtype)
    tail = synth.to_device({"K": K_t, "V": V_t}, w.dtype)
    shape = xb.Shape.of(w)
    ws = alloc_ws(shape)
    q = dev["q"][0].contiguous()
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=synth.torch_dtype(w.dtype), device="cuda")
    out0, out_plain = torch.empty_like(out), torch.empty_like(out)
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    xb.xkv_sr_decode_absorbed(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out, idx, S, ws,
                              K_tail=tail["K"], V_tail=tail["V"], T=T)
    xb.xkv_sr_decode_absorbed(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out0, None, None, ws,
                              K_tail=None, V_tail=None, T=0)
    xb.xkv_sr_decode_absorbed(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out_plain, None, None, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(synth.to_host(out0), synth.to_host(out_plain))
    outh, idxh, Sh = synth.storage_to_f64(synth.to_host(out)), idx.cpu().numpy(), S.cpu().numpy()
    for b in range(w.batch):
        for g in range(w.H_kv):
            np.testing.assert_array_equal(idxh[b, g], oracle.select(Sh[b, g], w.k))
        ref = oracle.gather_attend_tail(case["A_k"][b], case["A_v"][b], case["B_k"][b, 0], case["B_v"][b, 0],
                                        case["q"][0, b], idxh[b], K_t[b], V_t[b])
        assert max_rel(outh[b], ref) <= TOL[w.dtype], (name, b)


def _full_size_sampled(w, seqs, seed):
    """One layer of a benchmark configuration at full size (device-generated factors, the launch configuration the
    benchmark times): the pooled scores and the selection are bit for bit those of xkv_sr_decode; head scores of
    token ranges at the start, middle and end of the sampled sequences and their attention outputs are checked
    against the oracle."""
    torch = torch_mod()
    dev = synth.make_group_device(w, seed=seed)
    shape = xb.Shape.of(w)
    ws = alloc_ws(shape)
    layer = w.G - 1
    n_rep = w.H_q // w.H_kv
    q_l = dev["q"][layer].contiguous()
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=synth.torch_dtype(w.dtype), device="cuda")
    xb.xkv_sr_decode_absorbed(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q_l, out, idx, S, ws)
    S0, idx0, out0 = torch.empty_like(S), torch.empty_like(idx), torch.empty_like(out)
    xb.xkv_sr_decode(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q_l, out0, idx0, S0, ws)
    heads = torch.empty((w.batch, w.H_kv, w.L, xb.head_pitch(shape)), dtype=torch.float32, device="cuda")
    S1 = torch.empty_like(S)
    xb.xkv_head_scores(shape, layer, dev["A_k"], dev["B_k"], q_l, S1, heads, ws)
    torch.cuda.synchronize()
    assert torch.equal(S, S0) and torch.equal(idx, idx0) and torch.equal(S1, S0)
    assert torch.equal(heads[..., :n_rep].max(dim=-1).values, S1)
    # the two forms of stages 3-4 agree with each other within twice the tolerance
    assert max_rel(synth.storage_to_f64(synth.to_host(out)), synth.storage_to_f64(synth.to_host(out0))) <= 2 * TOL[w.dtype]
    scale = oracle.default_scale(w.d_h)
    mid = w.L // 2
    for b in seqs:
        B_k = synth.to_host(dev["B_k"][b, layer])
        B_v = synth.to_host(dev["B_v"][b, layer])
        q = synth.to_host(dev["q"][layer, b])
        for lo, hi in [(0, 256), (mid - 128, mid + 128), (w.L - 256, w.L)]:
            ref = oracle.head_scores(synth.to_host(dev["A_k"][b, lo:hi]), B_k, q, w.H_kv, scale)
            got = heads[b, :, lo:hi, :n_rep].cpu().numpy().transpose(0, 2, 1).reshape(w.H_q, hi - lo)
            assert max_rel(got, ref) <= TOL[w.dtype], (b, lo)
        idx_b = idx[b].cpu().numpy()
        ref_out = oracle.gather_attend(synth.to_host(dev["A_k"][b]), synth.to_host(dev["A_v"][b]), B_k, B_v, q, idx_b,
                                       scale)
        err = max_rel(synth.storage_to_f64(synth.to_host(out[b])), ref_out)
        assert err <= TOL[w.dtype], (b, err)
        print("seq", b, "absorbed vs oracle", err, flush=True)


def test_absorbed_llama_full_size_sampled():
    _full_size_sampled(synth.LLAMA_FULL, seqs=(0, synth.LLAMA_FULL.batch - 1), seed=31)


def test_absorbed_qwen_full_size_sampled():
    _full_size_sampled(synth.QWEN, seqs=(synth.QWEN.batch - 1,), seed=32)
