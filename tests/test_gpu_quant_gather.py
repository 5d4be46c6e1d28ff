"""GPU parity of 3-bit rows and of the gather-reconstruct kernels reading quantised rows (4-bit and 3-bit).

  xkv_quantize_rows(bits=3)   vs oracle.quantize_rows(bits=3) + pack_q3      bit for bit
  xkv_gather_attend_q         vs oracle.gather_attend_rows on the de-quantised values x^ = step * code + lo (taken from
                              the oracle's codes, which equal the GPU's bytes), with row counts and the rotation
  xkv_sr_decode_landmark_q    the paper's arrangement (landmark selector, RoPE on reconstruction, uncompressed tail)
                              on a quantised cache: same rows as the unquantised call, output vs the oracle on x^
  xkv_sr_decode_q4            factor scoring from 4-bit rows, selection vs oracle.select on the GPU's scores, output vs
                              the oracle on x^
Tolerance 2e-2 (bf16 operands, fp32 accumulation), as for the unquantised path: the de-quantised value is rounded
once to bf16 on its way into the matrix cores.
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


def pack(codes, step, lo, bits):
    return oracle.pack_q4(codes, step, lo) if bits == 4 else oracle.pack_q3(codes, step, lo)


def quantise_on_gpu(torch, A_dev, rows, r, bits):
    out = torch.full((rows, xb.xkv_quantized_row_bytes(r, bits)), 0xAB, dtype=torch.uint8, device="cuda")
    xb.xkv_quantize_rows(A_dev, rows, r, out, bits=bits)
    torch.cuda.synchronize()
    return out


def quantised_case(torch, w, case, dev, bits):
    """Quantise A^K and A^V of every sequence on the GPU; check the bytes against the oracle's; return the device
    rows and the de-quantised values the oracle works on."""
    Aq_k = quantise_on_gpu(torch, dev["A_k"], w.batch * w.L, w.r_k, bits).view(w.batch, w.L, -1)
    Aq_v = quantise_on_gpu(torch, dev["A_v"], w.batch * w.L, w.r_v, bits).view(w.batch, w.L, -1)
    hat_k, hat_v = [], []
    for b in range(w.batch):
        for name, Aq, hats in (("A_k", Aq_k, hat_k), ("A_v", Aq_v, hat_v)):
            codes, step, lo = oracle.quantize_rows(case[name][b], bits)
            np.testing.assert_array_equal(Aq[b].cpu().numpy(), pack(codes, step, lo, bits))
            hats.append(oracle.dequantize_rows(codes, step, lo))
    return Aq_k, Aq_v, hat_k, hat_v


@pytest.mark.parametrize("rows,r", [(1, 128), (7, 32), (333, 384), (1000, 512), (65, 2048), (0, 256), (77, 96), (500, 576)])
def test_three_bit_quantiser_matches_the_oracle_bit_for_bit(rows, r):
    torch = torch_mod()
    rng = np.random.default_rng(rows * 5 + r)
    x = rng.standard_normal((rows, r)) * np.exp(rng.standard_normal((rows, 1)))
    if rows > 2:
        x[1, :32] = 0.25                      # a constant group: step falls back to 1
        x[0, :32] = np.arange(32) * 0.25      # the group worked by hand in the CPU pins
    xbits = synth.to_storage(x, "bf16")
    X = torch.from_numpy(xbits.view(np.int16)).cuda()
    got = quantise_on_gpu(torch, X, rows, r, 3).cpu().numpy()
    assert got.shape == (rows, r // 2)
    if rows:
        codes, step, lo = oracle.quantize_rows(xbits, 3)
        np.testing.assert_array_equal(got, oracle.pack_q3(codes, step, lo))


GA_CASES = [
    # name, workload, rope theta: four-wavefront kernel, ragged ranks (not whole 128- or 256-rank blocks)
    ("llama_small_r96_160", synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=96, r_v=160, batch=2, G=2, a_scale=0.1), 0.0),
    ("qwen_small_rope", synth.QWEN.with_(L=5001, k=257, r_k=128, r_v=64, batch=1, G=1), 1000000.0),
    # eight-wavefront kernel (4 x 8 x 2100 selected rows), the paper's ranks, several tiles with a ragged last one
    ("llama_384_576_rope", synth.LLAMA_GROUP.with_(L=9000, k=2100, r_k=384, r_v=576, batch=4, G=1, a_scale=384 ** -0.5),
     500000.0),
    ("llama_512", synth.LLAMA_GROUP.with_(L=6000, k=1100, r_k=512, r_v=512, batch=8, G=1), 0.0),
    ("llama_768_256", synth.LLAMA_GROUP.with_(L=4000, k=600, r_k=768, r_v=256, batch=1, G=1, a_scale=768 ** -0.5), 0.0),
]


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("name,w,theta", GA_CASES, ids=[c[0] for c in GA_CASES])
def test_gather_attend_from_quantised_rows(name, w, theta, bits):
    torch = torch_mod()
    case = synth.make_case(w, seed=23 + bits)
    dev = synth.to_device(case, w.dtype)
    layer = w.G - 1
    Aq_k, Aq_v, hat_k, hat_v = quantised_case(torch, w, case, dev, bits)
    rng = np.random.default_rng(len(name) + bits)
    idx = np.stack([np.stack([np.sort(rng.choice(w.L, size=w.k, replace=False)) for _ in range(w.H_kv)])
                    for _ in range(w.batch)]).astype(np.int32)
    idx[:, :, -1] = w.L - 1
    idx[:, :, 0] = 0
    counts = rng.integers(1, w.k + 1, size=(w.batch, w.H_kv)).astype(np.int32)
    counts[0, 0] = w.k
    shape = xb.Shape.of(w)
    ws = xb.alloc_workspace(shape)
    q = dev["q"][layer].contiguous()
    qh = synth.to_host(q)
    idx_d, cnt_d = torch.from_numpy(idx).cuda(), torch.from_numpy(counts).cuda()
    out = torch.zeros((w.batch, w.H_q, w.d_h), dtype=torch.bfloat16, device="cuda")
    for use_counts in (False, True):
        xb.xkv_gather_attend_q(shape, layer, Aq_k, Aq_v, bits, dev["B_k"], dev["B_v"], q, idx_d,
                               cnt_d if use_counts else None, theta, out, ws)
        torch.cuda.synchronize()
        got = synth.storage_to_f64(synth.to_host(out))
        for b in range(w.batch):
            rows = [idx[b, g, :(counts[b, g] if use_counts else w.k)] for g in range(w.H_kv)]
            ref = oracle.gather_attend_rows(hat_k[b], hat_v[b], case["B_k"][b, layer], case["B_v"][b, layer], qh[b], rows,
                                            rope_theta=(theta if theta > 0 else None))
            err = max_rel(got[b], ref)
            assert err <= TOL, (name, bits, use_counts, b, err)
    # what the quantisation itself does to this output (reported; white-noise bases are the worst case)
    ref0 = oracle.gather_attend_rows(case["A_k"][0], case["A_v"][0], case["B_k"][0, layer], case["B_v"][0, layer], qh[0],
                                     [idx[0, g, :counts[0, g]] for g in range(w.H_kv)],
                                     rope_theta=(theta if theta > 0 else None))
    print(name, bits, "last error vs oracle on x^", err, "| effect of quantisation on sequence 0", max_rel(got[0], ref0),
          flush=True)


@pytest.mark.parametrize("bits", [4, 3])
def test_landmark_step_on_a_quantised_cache(bits):
    """Factors of pre-RoPE keys quantised, landmarks of post-RoPE keys, rotation on the reconstructed rows, an
    uncompressed tail: the rows are those of the unquantised call (the selector never reads A), the output is the
    oracle's on the de-quantised values."""
    torch = torch_mod()
    theta, c, o, T = 500000.0, 8, 2, 77
    w = synth.LLAMA_GROUP.with_(L=4000, k=512, r_k=128, r_v=192, batch=2, G=1, a_scale=0.1)
    case = synth.make_case(w, seed=31)
    dev = synth.to_device(case, w.dtype)
    Aq_k, Aq_v, hat_k, hat_v = quantised_case(torch, w, case, dev, bits)
    rng = np.random.default_rng(3)
    # post-RoPE keys of the (unquantised) cache, as prefill would have seen them, for the landmarks
    K_rope = np.empty((w.batch, w.H_kv, w.L, w.d_h))
    for b in range(w.batch):
        K = oracle.reconstruct(case["A_k"][b], case["B_k"][b, 0])
        for g in range(w.H_kv):
            K_rope[b, g] = oracle.rope(K[:, g * w.d_h:(g + 1) * w.d_h], np.arange(w.L), theta)
    K_tail_h = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)) * 0.05, w.dtype)
    V_tail_h = synth.to_storage(rng.standard_normal((w.batch, w.H_kv, T, w.d_h)), w.dtype)
    extra = synth.to_device({"K": synth.to_storage(K_rope, w.dtype), "Kt": K_tail_h, "Vt": V_tail_h}, w.dtype)
    shape = xb.Shape.of(w)
    n_c = -(-w.L // c)
    cap = (oracle.chunk_budget(w.k, c, n_c) + o) * c
    ws = torch.empty(xb.xkv_landmark_workspace_bytes(shape, c, o), dtype=torch.uint8, device="cuda")
    Lm = torch.zeros((w.batch, w.H_kv, n_c, w.d_h), dtype=torch.bfloat16, device="cuda")
    outl = torch.zeros((w.batch, w.H_kv, o), dtype=torch.int32, device="cuda")
    xb.xkv_landmarks(shape, extra["K"], c, o, Lm, None, outl, ws)
    q = dev["q"][0].contiguous()
    qh = synth.to_host(q)
    res = {}
    for which in ("plain", "quantised"):
        out = torch.zeros((w.batch, w.H_q, w.d_h), dtype=torch.bfloat16, device="cuda")
        rows = torch.zeros((w.batch, w.H_kv, cap), dtype=torch.int32, device="cuda")
        cnt = torch.zeros((w.batch, w.H_kv), dtype=torch.int32, device="cuda")
        if which == "plain":
            xb.xkv_sr_decode_landmark(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, Lm, outl, c, o, out,
                                      rows, cnt, None, ws, rope_theta=theta, K_tail=extra["Kt"], V_tail=extra["Vt"], T=T)
        else:
            xb.xkv_sr_decode_landmark_q(shape, 0, Aq_k, Aq_v, bits, dev["B_k"], dev["B_v"], q, Lm, outl, c, o, out, rows,
                                        cnt, None, ws, rope_theta=theta, K_tail=extra["Kt"], V_tail=extra["Vt"], T=T)
        torch.cuda.synchronize()
        res[which] = (synth.storage_to_f64(synth.to_host(out)), rows.cpu().numpy(), cnt.cpu().numpy())
    np.testing.assert_array_equal(res["quantised"][1], res["plain"][1])
    np.testing.assert_array_equal(res["quantised"][2], res["plain"][2])
    # the same two calls on B_l re-ordered once for the group (xkv_pack_b): bit for bit the same results
    packed = torch.full((xb.xkv_packed_b_bytes(shape),), 0xAB, dtype=torch.uint8, device="cuda")
    xb.xkv_pack_b(shape, dev["B_k"], dev["B_v"], packed)
    for which, qb, Ak, Av in (("plain", 0, dev["A_k"], dev["A_v"]), ("quantised", bits, Aq_k, Aq_v)):
        out = torch.full((w.batch, w.H_q, w.d_h), float("nan"), dtype=torch.bfloat16, device="cuda")
        rows = torch.zeros((w.batch, w.H_kv, cap), dtype=torch.int32, device="cuda")
        cnt = torch.zeros((w.batch, w.H_kv), dtype=torch.int32, device="cuda")
        xb.xkv_sr_decode_landmark_packed(shape, 0, Ak, Av, qb, dev["B_k"], packed, q, Lm, outl, c, o, out, rows, cnt, None,
                                         ws, rope_theta=theta, K_tail=extra["Kt"], V_tail=extra["Vt"], T=T)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(synth.storage_to_f64(synth.to_host(out)), res[which][0])
        np.testing.assert_array_equal(rows.cpu().numpy(), res[which][1])
        np.testing.assert_array_equal(cnt.cpu().numpy(), res[which][2])
    got, rows_h, cnt_h = res["quantised"]
    for b in range(w.batch):
        row_lists = [rows_h[b, g, :cnt_h[b, g]] for g in range(w.H_kv)]
        ref = oracle.gather_attend_rows(hat_k[b], hat_v[b], case["B_k"][b, 0], case["B_v"][b, 0], qh[b], row_lists,
                                        rope_theta=theta, K_tail=K_tail_h[b], V_tail=V_tail_h[b])
        assert max_rel(got[b], ref) <= TOL, (bits, b)


Q4_STEP = [
    ("llama_small", synth.LLAMA_GROUP.with_(L=3000, k=200, r_k=128, r_v=256, batch=2, G=2)),
    ("qwen_384_128", synth.QWEN.with_(L=5001, k=257, r_k=384, r_v=128, batch=1, G=1)),
    ("llama_k2100_r256", synth.LLAMA_GROUP.with_(L=9000, k=2100, r_k=256, r_v=384, batch=4, G=1, a_scale=1 / 16.0)),
]


@pytest.mark.parametrize("name,w", Q4_STEP, ids=[n for n, _ in Q4_STEP])
def test_gather_reconstruct_step_on_four_bit_rows(name, w):
    torch = torch_mod()
    case = synth.make_case(w, seed=37)
    dev = synth.to_device(case, w.dtype)
    layer = w.G - 1
    Aq_k, Aq_v, hat_k, hat_v = quantised_case(torch, w, case, dev, 4)
    shape = xb.Shape.of(w)
    ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    q = dev["q"][layer].contiguous()
    out = torch.zeros((w.batch, w.H_q, w.d_h), dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    S = torch.zeros((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    xb.xkv_sr_decode_q4(shape, layer, Aq_k, Aq_v, dev["B_k"], dev["B_v"], q, out, idx, S, ws)
    S2 = torch.zeros_like(S)
    heads = torch.zeros((w.batch, w.H_kv, w.L, xb.head_pitch(shape)), dtype=torch.float32, device="cuda")
    xb.xkv_head_scores_q4(shape, layer, Aq_k, dev["B_k"], q, S2, heads, ws)
    out2 = torch.zeros_like(out)
    xb.xkv_sr_decode_q4(shape, layer, Aq_k, Aq_v, dev["B_k"], dev["B_v"], q, out2, None, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(S, S2) and torch.equal(out, out2)
    Sh, idxh, outh = S.cpu().numpy(), idx.cpu().numpy(), synth.storage_to_f64(synth.to_host(out))
    sc = oracle.default_scale(w.d_h)
    for b in range(w.batch):
        ref_S = oracle.pooled_scores(hat_k[b], case["B_k"][b, layer], case["q"][layer, b], w.H_kv, sc)
        assert max_rel(Sh[b], ref_S) <= TOL
        for g in range(w.H_kv):
            np.testing.assert_array_equal(idxh[b, g], oracle.select(Sh[b, g], w.k))
        ref = oracle.gather_attend(hat_k[b], hat_v[b], case["B_k"][b, layer], case["B_v"][b, layer], case["q"][layer, b],
                                   idxh[b], sc)
        assert max_rel(outh[b], ref) <= TOL, (name, b)


@pytest.mark.parametrize("bits", [4, 3])
def test_quantised_gather_reconstruct_full_size_sampled(bits):
    """Benchmark configuration 3's shape (batch 16, L = 65536, r = 512, k = 4096) with both bases quantised: the
    launch configuration the benchmark times, checked on one sequence against the oracle on its de-quantised rows."""
    torch = torch_mod()
    w = synth.LLAMA_FULL
    dev = synth.make_group_device(w, seed=43)
    shape = xb.Shape.of(w)
    layer = 1
    Aq_k = quantise_on_gpu(torch, dev["A_k"], w.batch * w.L, w.r_k, bits).view(w.batch, w.L, -1)
    Aq_v = quantise_on_gpu(torch, dev["A_v"], w.batch * w.L, w.r_v, bits).view(w.batch, w.L, -1)
    ws = xb.alloc_workspace(shape)
    q = dev["q"][layer].contiguous()
    gen = torch.Generator(device="cuda").manual_seed(9)
    idx = torch.stack([torch.stack([torch.randperm(w.L, generator=gen, device="cuda")[:w.k].sort().values
                                    for _ in range(w.H_kv)]) for _ in range(w.batch)]).to(torch.int32)
    out = torch.zeros((w.batch, w.H_q, w.d_h), dtype=torch.bfloat16, device="cuda")
    xb.xkv_gather_attend_q(shape, layer, Aq_k, Aq_v, bits, dev["B_k"], dev["B_v"], q, idx, None, 0.0, out, ws)
    torch.cuda.synchronize()
    b = w.batch - 1
    idx_b = idx[b].cpu().numpy()
    hats = []
    for name, Aq in (("A_k", Aq_k), ("A_v", Aq_v)):
        codes, step, lo = oracle.quantize_rows(synth.to_host(dev[name][b]), bits)
        touched = np.unique(idx_b)
        np.testing.assert_array_equal(Aq[b].cpu().numpy()[touched], pack(codes[touched], step[touched], lo[touched], bits))
        hats.append(oracle.dequantize_rows(codes, step, lo))
    ref = oracle.gather_attend(hats[0], hats[1], synth.to_host(dev["B_k"][b, layer]), synth.to_host(dev["B_v"][b, layer]),
                               synth.to_host(q[b]), idx_b)
    err = max_rel(synth.storage_to_f64(synth.to_host(out[b])), ref)
    print("full size", bits, err, flush=True)
    assert err <= TOL


def test_quantised_gather_calls_reject_what_they_do_not_cover():
    torch = torch_mod()
    t = torch.zeros(64, dtype=torch.uint8, device="cuda")
    ws = xb.alloc_workspace(xb.Shape.of(synth.TINY))
    with pytest.raises(xb.XkvError) as e:                       # fp32 shapes: the general kernel reads no quantised rows
        xb.xkv_gather_attend_q(xb.Shape.of(synth.TINY), 0, t, t, 4, t, t, t, t, None, 0.0, t, ws)
    assert e.value.status == xb.XKV_ERR_UNSUPPORTED
    w = synth.LLAMA_GROUP.with_(L=512, k=64, r_k=128, r_v=128, batch=1)
    ws = xb.alloc_workspace(xb.Shape.of(w))
    for bad_bits in (2, 5, 8):
        with pytest.raises(xb.XkvError) as e:
            xb.xkv_gather_attend_q(xb.Shape.of(w), 0, t, t, bad_bits, t, t, t, t, None, 0.0, t, ws)
        assert e.value.status == xb.XKV_ERR_UNSUPPORTED
    with pytest.raises(xb.XkvError) as e:                       # ranks must be whole quantisation groups
        xb.xkv_gather_attend_q(xb.Shape.of(w.with_(r_k=80)), 0, t, t, 4, t, t, t, t, None, 0.0, t, ws)
    assert e.value.status == xb.XKV_ERR_UNSUPPORTED
