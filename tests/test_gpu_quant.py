"""GPU parity of the 4-bit quantisation of the token basis and of the kernels that read quantised rows.

  xkv_quantize_rows      vs oracle.quantize_rows + pack_q4      bit for bit (codes, steps, offsets, byte layout)
  xkv_attend_absorbed_q4 vs oracle.gather_attend on the de-quantised A^V (x^ = step * code + lo, taken from the
                         GPU's own quantised rows, which equal the oracle's), within the bf16 tolerance
"""
import numpy as np
import pytest

import oracle
from paper_2503_18893_amd import synth
from paper_2503_18893_amd import binding as xb

pytestmark = pytest.mark.gpu

TOL = 2e-2


def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def max_rel(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


def quantize_gpu(x_bits):
    """x_bits: uint16 bf16 patterns [rows][r] -> packed uint8 [rows][5r/8] from the library."""
    torch = torch_mod()
    rows, r = x_bits.shape
    X = torch.from_numpy(x_bits.view(np.int16)).cuda()
    out = torch.full((rows, xb.xkv_quantized_row_bytes(r)), 0xAB, dtype=torch.uint8, device="cuda")
    xb.xkv_quantize_rows(X, rows, r, out)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("rows,r", [(1, 128), (7, 128), (333, 384), (1000, 512), (65, 2048), (0, 256), (50, 32),
                                    (77, 96), (500, 576)])
def test_quantiser_matches_the_oracle_bit_for_bit(rows, r):
    rng = np.random.default_rng(rows * 7 + r)
    x = rng.standard_normal((rows, r)) * np.exp(rng.standard_normal((rows, 1)))
    if rows > 2:
        x[1, :32] = 0.25                      # a constant group: step falls back to 1
        x[2, 32:64] = 0.0
        x[0, :32] = np.arange(32) * 0.5       # the group worked by hand in the CPU pins
    xbits = synth.to_storage(x, "bf16")
    got = quantize_gpu(xbits).cpu().numpy()
    codes, step, lo = oracle.quantize_rows(xbits)
    want = oracle.pack_q4(codes, step, lo) if rows else np.zeros((0, xb.xkv_quantized_row_bytes(r)), np.uint8)
    np.testing.assert_array_equal(got, want)


def test_quantiser_full_size_sampled():
    """A^V of one sequence group at benchmark size (16 x 65536 rows of 512): sampled rows against the oracle."""
    torch = torch_mod()
    w = synth.LLAMA_FULL
    dev = synth.make_group_device(w, seed=41)
    A = dev["A_v"]
    rows = w.batch * w.L
    out = torch.empty((rows, xb.xkv_quantized_row_bytes(w.r_v)), dtype=torch.uint8, device="cuda")
    xb.xkv_quantize_rows(A, rows, w.r_v, out)
    torch.cuda.synchronize()
    pick = np.unique(np.concatenate([np.arange(64), rows // 2 + np.arange(64), rows - 64 + np.arange(64),
                                     np.random.default_rng(1).integers(0, rows, 200)]))
    sel = torch.from_numpy(pick).cuda()
    a_host = synth.to_host(A.view(rows, w.r_v)[sel])
    codes, step, lo = oracle.quantize_rows(a_host)
    np.testing.assert_array_equal(out[sel].cpu().numpy(), oracle.pack_q4(codes, step, lo))


CASES = [
    ("llama_small", synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=128, r_v=256, batch=2, G=2)),
    ("qwen_small", synth.QWEN.with_(L=5001, k=257, r_k=128, r_v=128, batch=1, G=1)),
    ("wide_rv", synth.LLAMA_GROUP.with_(L=2500, k=700, r_k=64, r_v=640, batch=1, G=1)),
    ("paper_ranks_384_576", synth.LLAMA_GROUP.with_(L=2100, k=300, r_k=384, r_v=576, batch=1, G=1)),
    ("rv_96", synth.LLAMA_GROUP.with_(L=1500, k=100, r_k=64, r_v=96, batch=2, G=1)),
    ("gqa16_dh64", synth.Workload("gqa16", G=1, H_kv=3, H_q=48, d_h=64, r_k=48, r_v=128, L=1111, k=40, batch=1,
                                  dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    ("k2100_dh256", synth.Workload("k2100", G=1, H_kv=2, H_q=8, d_h=256, r_k=64, r_v=384, L=6000, k=2100, batch=2,
                                   dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
]


@pytest.mark.parametrize("name,w", CASES, ids=[n for n, _ in CASES])
def test_attend_absorbed_on_quantised_values(name, w):
    torch = torch_mod()
    case = synth.make_case(w, seed=17)
    dev = synth.to_device(case, w.dtype)
    shape = xb.Shape.of(w)
    layer = w.G - 1
    ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    q = dev["q"][layer].contiguous()
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    heads = torch.empty((w.batch, w.H_kv, w.L, xb.head_pitch(shape)), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=torch.bfloat16, device="cuda")
    Aq = torch.empty((w.batch, w.L, xb.xkv_quantized_row_bytes(w.r_v)), dtype=torch.uint8, device="cuda")
    xb.xkv_quantize_rows(dev["A_v"], w.batch * w.L, w.r_v, Aq)
    xb.xkv_head_scores(shape, layer, dev["A_k"], dev["B_k"], q, S, heads, ws)
    xb.xkv_topk(shape, S, idx, ws)
    xb.xkv_attend_absorbed_q4(shape, layer, Aq, dev["B_v"], heads, idx, out, ws)
    torch.cuda.synchronize()
    outh, idxh, Aqh = synth.storage_to_f64(synth.to_host(out)), idx.cpu().numpy(), Aq.cpu().numpy()
    sc = oracle.default_scale(w.d_h)
    for b in range(w.batch):
        codes, step, lo = oracle.quantize_rows(case["A_v"][b])
        np.testing.assert_array_equal(Aqh[b], oracle.pack_q4(codes, step, lo))
        A_v_hat = oracle.dequantize_rows(codes, step, lo)
        ref = oracle.gather_attend(case["A_k"][b], A_v_hat, case["B_k"][b, layer], case["B_v"][b, layer],
                                   case["q"][layer, b], idxh[b], sc)
        err = max_rel(outh[b], ref)
        assert err <= TOL, (name, b, err)
        # and the quantisation itself costs little at these spectra: against the unquantised values
        ref0 = oracle.gather_attend(case["A_k"][b], case["A_v"][b], case["B_k"][b, layer], case["B_v"][b, layer],
                                    case["q"][layer, b], idxh[b], sc)
        print(name, b, "vs quantised oracle", err, "quantisation effect", max_rel(ref, ref0), flush=True)


STEP_CASES = [
    ("llama_small", synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=128, r_v=256, batch=2, G=2)),
    ("qwen_small", synth.QWEN.with_(L=5001, k=257, r_k=384, r_v=128, batch=1, G=1)),
    ("gqa16_dh64", synth.Workload("gqa16", G=1, H_kv=3, H_q=48, d_h=64, r_k=128, r_v=128, L=1111, k=40, batch=1,
                                  dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    ("gqa2_many_heads", synth.Workload("gqa2", G=1, H_kv=20, H_q=40, d_h=128, r_k=256, r_v=128, L=4097, k=300, batch=1,
                                       dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    ("mha_r640", synth.Workload("mha", G=2, H_kv=20, H_q=20, d_h=64, r_k=640, r_v=256, L=900, k=50, batch=2,
                                dtype="bf16", a_scale=0.3, sigma_decay=0.8, q_scale=0.2)),
    # the paper's ranks at window 4 (r_K : r_V = 1 : 1.5); rows of A^V are padded from 360 to 368 bytes
    ("paper_ranks_384_576", synth.LLAMA_GROUP.with_(L=2100, k=300, r_k=384, r_v=576, batch=1, G=1)),
]


@pytest.mark.parametrize("name,w", STEP_CASES, ids=[n for n, _ in STEP_CASES])
def test_quantised_step_chain(name, w):
    """Head scores from quantised A^K, selection, absorbed attention over quantised A^V; then the fused call.
    References: the oracle on the de-quantised values (x^ = step * code + lo of the oracle's own quantiser, whose
    packed rows equal the GPU's bit for bit)."""
    torch = torch_mod()
    case = synth.make_case(w, seed=19)
    dev = synth.to_device(case, w.dtype)
    shape = xb.Shape.of(w)
    layer = w.G - 1
    n_rep = w.H_q // w.H_kv
    nrp = xb.head_pitch(shape)
    ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    q = dev["q"][layer].contiguous()
    Aqk = torch.empty((w.batch, w.L, xb.xkv_quantized_row_bytes(w.r_k)), dtype=torch.uint8, device="cuda")
    Aqv = torch.empty((w.batch, w.L, xb.xkv_quantized_row_bytes(w.r_v)), dtype=torch.uint8, device="cuda")
    xb.xkv_quantize_rows(dev["A_k"], w.batch * w.L, w.r_k, Aqk)
    xb.xkv_quantize_rows(dev["A_v"], w.batch * w.L, w.r_v, Aqv)
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    heads = torch.full((w.batch, w.H_kv, w.L, nrp), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=torch.bfloat16, device="cuda")
    xb.xkv_head_scores_q4(shape, layer, Aqk, dev["B_k"], q, S, heads, ws)
    xb.xkv_topk(shape, S, idx, ws)
    xb.xkv_attend_absorbed_q4(shape, layer, Aqv, dev["B_v"], heads, idx, out, ws)
    S2, idx2, out2 = torch.empty_like(S), torch.empty_like(idx), torch.empty_like(out)
    xb.xkv_sr_decode_absorbed_q4(shape, layer, Aqk, Aqv, dev["B_k"], dev["B_v"], q, out2, idx2, S2, ws)
    torch.cuda.synchronize()
    assert torch.equal(S2, S) and torch.equal(idx2, idx) and torch.equal(out2, out)
    Sh, hh, idxh = S.cpu().numpy(), heads.cpu().numpy(), idx.cpu().numpy()
    outh = synth.storage_to_f64(synth.to_host(out))
    np.testing.assert_array_equal(Sh, hh[..., :n_rep].max(axis=-1))
    np.testing.assert_array_equal(hh[..., n_rep:], 0.0)
    sc = oracle.default_scale(w.d_h)
    for b in range(w.batch):
        Ak_hat = oracle.dequantize_rows(*oracle.quantize_rows(case["A_k"][b]))
        Av_hat = oracle.dequantize_rows(*oracle.quantize_rows(case["A_v"][b]))
        s_ref = oracle.head_scores(Ak_hat, case["B_k"][b, layer], case["q"][layer, b], w.H_kv, sc)
        s_gpu = hh[b, :, :, :n_rep].transpose(0, 2, 1).reshape(w.H_q, w.L)
        err_s = max_rel(s_gpu, s_ref)
        assert err_s <= TOL, (name, b, err_s)
        for g in range(w.H_kv):
            np.testing.assert_array_equal(idxh[b, g], oracle.select(Sh[b, g], w.k))
        ref = oracle.gather_attend(Ak_hat, Av_hat, case["B_k"][b, layer], case["B_v"][b, layer], case["q"][layer, b],
                                   idxh[b], sc)
        err_o = max_rel(outh[b], ref)
        assert err_o <= TOL, (name, b, err_o)
        print(name, b, "head scores", err_s, "attention", err_o, flush=True)


@pytest.mark.parametrize("T", [1, 77, 700])
def test_quantised_step_with_uncompressed_tail(T):
    """The quantised step with T uncompressed recent tokens in the same softmax, against the oracle's attention over
    the de-quantised reconstructed rows plus the tail (fed the GPU's own index sets)."""
    torch = torch_mod()
    w = synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=128, r_v=256, batch=2, G=1)
    case = synth.make_case(w, seed=29)
    dev = synth.to_device(case, w.dtype)
    rng = np.random.default_rng(6)
    K_t = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)) * 0.3, w.dtype)
    V_t = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)), w.dtype)
    tail = synth.to_device({"K": K_t, "V": V_t}, w.dtype)
    shape = xb.Shape.of(w)
    ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    q = dev["q"][0].contiguous()
    Aqk = torch.empty((w.batch, w.L, xb.xkv_quantized_row_bytes(w.r_k)), dtype=torch.uint8, device="cuda")
    Aqv = torch.empty((w.batch, w.L, xb.xkv_quantized_row_bytes(w.r_v)), dtype=torch.uint8, device="cuda")
    xb.xkv_quantize_rows(dev["A_k"], w.batch * w.L, w.r_k, Aqk)
    xb.xkv_quantize_rows(dev["A_v"], w.batch * w.L, w.r_v, Aqv)
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=torch.bfloat16, device="cuda")
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    xb.xkv_sr_decode_absorbed_q4(shape, 0, Aqk, Aqv, dev["B_k"], dev["B_v"], q, out, idx, S, ws, K_tail=tail["K"],
                                 V_tail=tail["V"], T=T)
    torch.cuda.synchronize()
    outh, idxh, Sh = synth.storage_to_f64(synth.to_host(out)), idx.cpu().numpy(), S.cpu().numpy()
    for b in range(w.batch):
        for g in range(w.H_kv):
            np.testing.assert_array_equal(idxh[b, g], oracle.select(Sh[b, g], w.k))
        Ak_hat = oracle.dequantize_rows(*oracle.quantize_rows(case["A_k"][b]))
        Av_hat = oracle.dequantize_rows(*oracle.quantize_rows(case["A_v"][b]))
        ref = oracle.gather_attend_tail(Ak_hat, Av_hat, case["B_k"][b, 0], case["B_v"][b, 0], case["q"][0, b], idxh[b],
                                        K_t[b], V_t[b])
        assert max_rel(outh[b], ref) <= TOL, (T, b)


def test_quantised_step_full_size_sampled():
    """Benchmark configuration 3 with both token bases quantised, the launch configuration the benchmark times:
    sampled head scores, the complete selection of the sampled sequences, and their outputs."""
    torch = torch_mod()
    w = synth.LLAMA_FULL
    dev = synth.make_group_device(w, seed=43)
    shape = xb.Shape.of(w)
    layer = w.G - 1
    n_rep = w.H_q // w.H_kv
    ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    q_l = dev["q"][layer].contiguous()
    Aqk = torch.empty((w.batch, w.L, xb.xkv_quantized_row_bytes(w.r_k)), dtype=torch.uint8, device="cuda")
    Aqv = torch.empty((w.batch, w.L, xb.xkv_quantized_row_bytes(w.r_v)), dtype=torch.uint8, device="cuda")
    xb.xkv_quantize_rows(dev["A_k"], w.batch * w.L, w.r_k, Aqk)
    xb.xkv_quantize_rows(dev["A_v"], w.batch * w.L, w.r_v, Aqv)
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    heads = torch.empty((w.batch, w.H_kv, w.L, xb.head_pitch(shape)), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=torch.bfloat16, device="cuda")
    xb.xkv_sr_decode_absorbed_q4(shape, layer, Aqk, Aqv, dev["B_k"], dev["B_v"], q_l, out, idx, S, ws)
    S1 = torch.empty_like(S)
    xb.xkv_head_scores_q4(shape, layer, Aqk, dev["B_k"], q_l, S1, heads, ws)
    torch.cuda.synchronize()
    assert torch.equal(S1, S) and torch.equal(heads[..., :n_rep].max(dim=-1).values, S)
    sc = oracle.default_scale(w.d_h)
    mid = w.L // 2
    for b in (0, w.batch - 1):
        B_k, B_v = synth.to_host(dev["B_k"][b, layer]), synth.to_host(dev["B_v"][b, layer])
        q = synth.to_host(dev["q"][layer, b])
        Ak_hat = oracle.dequantize_rows(*oracle.quantize_rows(synth.to_host(dev["A_k"][b])))
        Av_hat = oracle.dequantize_rows(*oracle.quantize_rows(synth.to_host(dev["A_v"][b])))
        for lo_, hi_ in [(0, 256), (mid - 128, mid + 128), (w.L - 256, w.L)]:
            ref = oracle.head_scores(Ak_hat[lo_:hi_], B_k, q, w.H_kv, sc)
            got = heads[b, :, lo_:hi_, :n_rep].cpu().numpy().transpose(0, 2, 1).reshape(w.H_q, hi_ - lo_)
            assert max_rel(got, ref) <= TOL, (b, lo_)
        S_b, idx_b = S[b].cpu().numpy(), idx[b].cpu().numpy()
        for g in range(w.H_kv):
            np.testing.assert_array_equal(idx_b[g], oracle.select(S_b[g], w.k))
        ref_out = oracle.gather_attend(Ak_hat, Av_hat, B_k, B_v, q, idx_b, sc)
        err = max_rel(synth.storage_to_f64(synth.to_host(out[b])), ref_out)
        assert err <= TOL, (b, err)
        print("seq", b, "quantised step vs oracle", err, flush=True)


def test_prefill_to_decode_chain_factorize_quantise_decode():
    """The whole chain on the GPU: caches -> xkv_factorize (keys and values) -> xkv_quantize_rows ->
    xkv_sr_decode_absorbed_q4 with k = L.  Reference: the oracle's attention on the factors the GPU produced, with
    their token bases quantised by the oracle's quantiser (whose packed rows must equal the GPU's); and the
    bf16 absorbed and gather-reconstruct steps on the unquantised factors must agree with each other."""
    torch = torch_mod()
    G, H_kv, H_q, d_h, L, r, dtype = 2, 2, 8, 64, 640, 128, "bf16"
    rng = np.random.default_rng(12)
    caches = [synth.make_cache(rng, G, H_kv, d_h, L, 0.5, dtype=dtype) for _ in range(2)]   # keys, values (full rank)
    fshape = xb.Shape(G=G, H_kv=H_kv, H_q=H_kv, d_h=d_h, r_k=r, r_v=r, L=L, k=1, batch=1, dtype=dtype)
    fws = torch.empty(xb.xkv_factorize_workspace_bytes(fshape, r), dtype=torch.uint8, device="cuda")
    fac = []
    for i, X in enumerate(caches):
        Xd = synth.to_device({"X": X[None]}, dtype)["X"]
        A = torch.zeros((1, L, r), dtype=torch.bfloat16, device="cuda")
        B = torch.zeros((1, G, r, H_kv * d_h), dtype=torch.bfloat16, device="cuda")
        xb.xkv_factorize(fshape, Xd, r, 8, 7 + i, A, B, fws)
        fac.append((A, B))
    (A_k, B_k), (A_v, B_v) = fac
    shape = xb.Shape(G=G, H_kv=H_kv, H_q=H_q, d_h=d_h, r_k=r, r_v=r, L=L, k=L, batch=1, dtype=dtype)
    ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    Aqk = torch.empty((1, L, xb.xkv_quantized_row_bytes(r)), dtype=torch.uint8, device="cuda")
    Aqv = torch.empty_like(Aqk)
    xb.xkv_quantize_rows(A_k, L, r, Aqk)
    xb.xkv_quantize_rows(A_v, L, r, Aqv)
    q_host = synth.to_storage(rng.standard_normal((G, 1, H_q, d_h)) * 0.5, dtype)
    q_dev = synth.to_device({"q": q_host}, dtype)["q"]
    torch.cuda.synchronize()
    Ak_h, Av_h = synth.to_host(A_k[0]), synth.to_host(A_v[0])
    qk, qv = oracle.quantize_rows(Ak_h), oracle.quantize_rows(Av_h)
    np.testing.assert_array_equal(Aqk[0].cpu().numpy(), oracle.pack_q4(*qk))
    np.testing.assert_array_equal(Aqv[0].cpu().numpy(), oracle.pack_q4(*qv))
    Ak_hat, Av_hat = oracle.dequantize_rows(*qk), oracle.dequantize_rows(*qv)
    idx_all = np.tile(np.arange(L, dtype=np.int32), (H_kv, 1))
    for layer in range(G):
        outs = {}
        for kind in ("q4", "absorbed", "gather"):
            out = torch.empty((1, H_q, d_h), dtype=torch.bfloat16, device="cuda")
            ql = q_dev[layer].contiguous()
            if kind == "q4":
                xb.xkv_sr_decode_absorbed_q4(shape, layer, Aqk, Aqv, B_k, B_v, ql, out, None, None, ws)
            elif kind == "absorbed":
                xb.xkv_sr_decode_absorbed(shape, layer, A_k, A_v, B_k, B_v, ql, out, None, None, ws)
            else:
                xb.xkv_sr_decode(shape, layer, A_k, A_v, B_k, B_v, ql, out, None, None, ws)
            torch.cuda.synchronize()
            outs[kind] = synth.storage_to_f64(synth.to_host(out))[0]
        Bk_h, Bv_h = synth.to_host(B_k[0, layer]), synth.to_host(B_v[0, layer])
        ref_q = oracle.gather_attend(Ak_hat, Av_hat, Bk_h, Bv_h, q_host[layer, 0], idx_all)
        ref = oracle.gather_attend(Ak_h, Av_h, Bk_h, Bv_h, q_host[layer, 0], idx_all)
        assert max_rel(outs["q4"], ref_q) <= TOL, layer
        assert max_rel(outs["absorbed"], ref) <= TOL and max_rel(outs["gather"], ref) <= TOL, layer
        print("layer", layer, "q4 vs oracle on x^", max_rel(outs["q4"], ref_q), "4-bit vs bf16 factors",
              max_rel(ref_q, ref), flush=True)


def test_quantised_calls_reject_what_they_do_not_cover():
    torch = torch_mod()
    with pytest.raises(xb.XkvError) as ei:
        xb.xkv_quantized_row_bytes(100)
    assert ei.value.status == xb.XKV_ERR_UNSUPPORTED
    assert xb.xkv_quantized_row_bytes(128, bits=3) == 64           # 3-bit rows: r/2 bytes
    with pytest.raises(xb.XkvError) as ei:
        xb.xkv_quantized_row_bytes(128, bits=2)
    assert ei.value.status == xb.XKV_ERR_UNSUPPORTED
    w = synth.TINY.with_(r_v=128, G=1, H_kv=2, H_q=4)       # fp32 shape: quantised rows go with bf16 shapes only
    shape = xb.Shape.of(w)
    ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    t = torch.zeros(4096, device="cuda")
    with pytest.raises(xb.XkvError) as ei:
        xb.xkv_attend_absorbed_q4(shape, 0, t, t, t, t, t, ws)
    assert ei.value.status == xb.XKV_ERR_UNSUPPORTED
