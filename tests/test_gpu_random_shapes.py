"""Randomly drawn shapes within the documented limits, fixed seeds: what the hand-picked cases of the other files may
have missed.  Three sweeps, each against the oracle as in the files they are modelled on:

  the whole chain (stage calls and the fused call, bf16 and fp32, any head width)      as test_gpu_parity.check_chain
  the gather-reconstruct stage call on bf16, 4-bit and 3-bit rows (counts, rotation)   as test_gpu_quant_gather
  landmark construction and the landmark-guided step (plain and quantised rows, rotation, uncompressed tail)
                                                                                       as test_gpu_landmark
Shapes are printed before they run, so that a failure names its case.
"""
import numpy as np
import pytest

import oracle
from paper_2503_18893_amd import synth
from paper_2503_18893_amd import binding as xb
from test_gpu_parity import check_chain

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


def test_random_shapes_whole_chain():
    torch_mod()
    rng = np.random.default_rng(1)
    n_cases = 30
    for case_no in range(n_cases):
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        d_h = 128 if rng.random() < 0.7 else int(rng.choice([32, 64, 96, 128, 256]))
        H_kv = int(rng.choice([1, 2, 3, 4, 8]))
        n_rep = int(rng.choice([1, 2, 4, 5, 7, 8, 16]))
        d = H_kv * d_h
        rmax = min(640, d)
        step = 16 if rng.random() < 0.7 else 8
        r_k = int(rng.integers(1, rmax // step + 1)) * step
        r_v = int(rng.integers(1, rmax // step + 1)) * step
        L = int(rng.integers(1, 12000)) if rng.random() < 0.8 else int(rng.integers(60000, 72000))
        k = int(rng.integers(1, min(L, 1500) + 1))
        batch = int(rng.integers(1, 4)) if L < 20000 else 1
        G = int(rng.integers(1, 3))
        layer = int(rng.integers(0, G))
        w = synth.Workload(f"fuzz{case_no}", G=G, H_kv=H_kv, H_q=H_kv * n_rep, d_h=d_h, r_k=r_k, r_v=r_v, L=L, k=k, batch=batch,
                           dtype=dtype, a_scale=1.0 / np.sqrt(r_k), sigma_decay=0.8, q_scale=1.0 / np.sqrt(d_h))
        print(case_no, dict(dtype=dtype, d_h=d_h, H_kv=H_kv, n_rep=n_rep, r_k=r_k, r_v=r_v, L=L, k=k, batch=batch, G=G, layer=layer), flush=True)
        case = synth.make_case(w, seed=2000 + case_no)
        rep = check_chain(w, case, layer)
        print("   ", {b: {kk: round(vv, 6) for kk, vv in r.items()} for b, r in rep.items()}, flush=True)


def test_random_shapes_gather_reconstruct_on_plain_and_quantised_rows():
    torch = torch_mod()
    rng = np.random.default_rng(1)
    n_cases = 40
    worst = 0.0
    for case_no in range(n_cases):
        H_kv = int(rng.choice([1, 2, 4, 8]))
        n_rep = int(rng.choice([1, 2, 4, 5, 7, 8, 16]))
        d = H_kv * 128
        rmax = min(768, d)
        r_k = int(rng.integers(1, rmax // 32 + 1)) * 32
        r_v = int(rng.integers(1, rmax // 32 + 1)) * 32
        if rng.random() < 0.3:   # ranks that are multiples of 16 only: bf16 path alone
            r_k = min(rmax, r_k + 16) if r_k + 16 <= rmax else r_k
        L = int(rng.integers(1, 9000))
        k = int(rng.integers(1, min(L, 2500) + 1))
        batch = int(rng.integers(1, 4))
        G = int(rng.integers(1, 4))
        layer = int(rng.integers(0, G))
        theta = float(rng.choice([0.0, 10000.0, 500000.0]))
        w = synth.Workload(f"fuzz{case_no}", G=G, H_kv=H_kv, H_q=H_kv * n_rep, d_h=128, r_k=r_k, r_v=r_v, L=L, k=k, batch=batch,
                           dtype="bf16", a_scale=1.0 / np.sqrt(r_k), sigma_decay=0.8, q_scale=float(rng.choice([1 / np.sqrt(128.0), 1.0])))
        print(case_no, dict(H_kv=H_kv, n_rep=n_rep, r_k=r_k, r_v=r_v, L=L, k=k, batch=batch, G=G, layer=layer, theta=theta), flush=True)
        case = synth.make_case(w, seed=1000 + case_no)
        dev = synth.to_device(case, w.dtype)
        idx = np.stack([np.stack([np.sort(rng.choice(L, size=k, replace=False)) for _ in range(H_kv)]) for _ in range(batch)]).astype(np.int32)
        counts = rng.integers(0, k + 1, size=(batch, H_kv)).astype(np.int32)
        counts[0, 0] = k
        shape = xb.Shape.of(w)
        ws = xb.alloc_workspace(shape)
        q = dev["q"][layer].contiguous(); qh = synth.to_host(q)
        idx_d, cnt_d = torch.from_numpy(idx).cuda(), torch.from_numpy(counts).cuda()
        out = torch.zeros((batch, w.H_q, 128), dtype=torch.bfloat16, device="cuda")
        variants = [0] + ([4, 3] if r_k % 32 == 0 and r_v % 32 == 0 else [])
        for bits in variants:
            if bits:
                Aq, hats = {}, {}
                for nm, r in (("A_k", r_k), ("A_v", r_v)):
                    o = torch.full((batch * L, xb.xkv_quantized_row_bytes(r, bits)), 0xAB, dtype=torch.uint8, device="cuda")
                    xb.xkv_quantize_rows(dev[nm], batch * L, r, o, bits=bits)
                    Aq[nm] = o.view(batch, L, -1)
                    hats[nm] = []
                    for b in range(batch):
                        c, st, lo = oracle.quantize_rows(case[nm][b], bits)
                        hats[nm].append(oracle.dequantize_rows(c, st, lo))
            for use_counts in (False, True):
                out.fill_(float("nan"))
                if bits:
                    xb.xkv_gather_attend_q(shape, layer, Aq["A_k"], Aq["A_v"], bits, dev["B_k"], dev["B_v"], q, idx_d,
                                           cnt_d if use_counts else None, theta, out, ws)
                else:
                    xb.xkv_gather_attend_ex(shape, layer, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, idx_d,
                                            cnt_d if use_counts else None, theta, out, ws)
                torch.cuda.synchronize()
                got = synth.storage_to_f64(synth.to_host(out))
                for b in range(batch):
                    rows = [idx[b, g, :(counts[b, g] if use_counts else k)] for g in range(H_kv)]
                    Ak = hats["A_k"][b] if bits else case["A_k"][b]
                    Av = hats["A_v"][b] if bits else case["A_v"][b]
                    rows_eff = [rw if len(rw) else np.array([0]) for rw in rows]
                    ref = oracle.gather_attend_rows(Ak, Av, case["B_k"][b, layer], case["B_v"][b, layer], qh[b], rows_eff,
                                                    rope_theta=(theta if theta > 0 else None))
                    for g in range(H_kv):
                        if len(rows[g]) == 0:
                            ref[g * n_rep:(g + 1) * n_rep] = 0.0
                    # heads with no rows: the library writes zeros
                    for g in range(H_kv):
                        if len(rows[g]) == 0:
                            assert np.all(got[b, g * n_rep:(g + 1) * n_rep] == 0), ("empty head not zero", case_no, bits, b, g)
                    err = max_rel(got[b], ref)
                    worst = max(worst, err)
                    assert np.isfinite(got[b]).all() and err <= TOL, (case_no, bits, use_counts, b, err)
    print("worst error", worst)


def test_random_shapes_landmark_step():
    torch = torch_mod()
    rng = np.random.default_rng(1)
    n_cases = 20
    worst = 0.0
    for case_no in range(n_cases):
        H_kv = int(rng.choice([1, 2, 4]))
        n_rep = int(rng.choice([1, 2, 4, 7, 8]))
        d = H_kv * 128
        rmax = min(384, d)
        r_k = int(rng.integers(1, rmax // 32 + 1)) * 32
        r_v = int(rng.integers(1, rmax // 32 + 1)) * 32
        c = int(rng.choice([4, 8, 16, 32]))
        L = int(rng.integers(c, 6000))
        k = int(rng.integers(1, min(L, 1200) + 1))
        n_c = -(-L // c)
        o = int(rng.integers(0, min(6, n_c) + 1))
        batch = int(rng.integers(1, 3))
        T = int(rng.choice([0, 0, 1, 50, 300]))
        theta = float(rng.choice([0.0, 10000.0, 500000.0]))
        w = synth.Workload(f"fz{case_no}", G=1, H_kv=H_kv, H_q=H_kv * n_rep, d_h=128, r_k=r_k, r_v=r_v, L=L, k=k, batch=batch,
                           dtype="bf16", a_scale=1.0, sigma_decay=0.5, q_scale=0.3)
        print(case_no, dict(H_kv=H_kv, n_rep=n_rep, r_k=r_k, r_v=r_v, L=L, k=k, c=c, o=o, batch=batch, T=T, theta=theta), flush=True)
        case = synth.make_case(w, seed=3000 + case_no)
        dev = synth.to_device(case, w.dtype)
        K = np.empty((batch, H_kv, L, 128))
        for b in range(batch):
            X = oracle.reconstruct(case["A_k"][b], case["B_k"][b, 0])
            for g in range(H_kv):
                Kg = X[:, g * 128:(g + 1) * 128]
                K[b, g] = oracle.rope(Kg, np.arange(L), theta) if theta > 0 else Kg
        K_host = synth.to_storage(K, "bf16")
        extra = {"K": K_host}
        if T:
            Kt_h = synth.to_storage(rng.standard_normal((batch, H_kv, T, 128)) * 0.5, "bf16")
            Vt_h = synth.to_storage(rng.standard_normal((batch, H_kv, T, 128)), "bf16")
            extra.update(Kt=Kt_h, Vt=Vt_h)
        ex = synth.to_device(extra, "bf16")
        shape = xb.Shape.of(w)
        k_ch = oracle.chunk_budget(k, c, n_c)
        cap = (k_ch + o) * c
        ws = torch.empty(xb.xkv_landmark_workspace_bytes(shape, c, o), dtype=torch.uint8, device="cuda")
        Lm = torch.zeros((batch, H_kv, n_c, 128), dtype=torch.bfloat16, device="cuda")
        negm = torch.zeros((batch, H_kv, n_c), dtype=torch.float32, device="cuda")
        outl = torch.zeros((batch, H_kv, max(o, 1)), dtype=torch.int32, device="cuda")
        xb.xkv_landmarks(shape, ex["K"], c, o, Lm, negm, outl if o else None, ws)
        torch.cuda.synchronize()
        Lm_h, negm_h, outl_h = synth.to_host(Lm), negm.cpu().numpy(), outl.cpu().numpy()
        q = dev["q"][0].contiguous(); qh = synth.to_host(q)
        for b in range(batch):
            Lm_ref, m_ref, _ = oracle.landmarks(K_host[b], c, o)
            assert max_rel(synth.storage_to_f64(Lm_h[b]), Lm_ref) <= 2.0 ** -8, "landmarks"
            assert np.abs(-negm_h[b].astype(np.float64) - m_ref).max() <= 1e-4, "min cosine"
            for g in range(H_kv):
                if o:
                    assert outl_h[b, g].tolist() == oracle.select(negm_h[b, g], o).tolist(), "outliers"
        for bits in (0, 4, 3):
            if bits:
                Aq, hats = {}, {}
                for nm, r in (("A_k", r_k), ("A_v", r_v)):
                    oq = torch.full((batch * L, xb.xkv_quantized_row_bytes(r, bits)), 0xAB, dtype=torch.uint8, device="cuda")
                    xb.xkv_quantize_rows(dev[nm], batch * L, r, oq, bits=bits)
                    Aq[nm] = oq.view(batch, L, -1)
                    hats[nm] = []
                    for b in range(batch):
                        cd, st, lo = oracle.quantize_rows(case[nm][b], bits)
                        hats[nm].append(oracle.dequantize_rows(cd, st, lo))
            out = torch.full((batch, w.H_q, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
            rows = torch.full((batch, H_kv, cap), -7, dtype=torch.int32, device="cuda")
            cnt = torch.zeros((batch, H_kv), dtype=torch.int32, device="cuda")
            S = torch.zeros((batch, H_kv, n_c), dtype=torch.float32, device="cuda")
            kw = dict(rope_theta=theta)
            if T:
                kw.update(K_tail=ex["Kt"], V_tail=ex["Vt"], T=T)
            if bits:
                xb.xkv_sr_decode_landmark_q(shape, 0, Aq["A_k"], Aq["A_v"], bits, dev["B_k"], dev["B_v"], q, Lm, outl if o else None,
                                            c, o, out, rows, cnt, S, ws, **kw)
            else:
                xb.xkv_sr_decode_landmark(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, Lm, outl if o else None,
                                          c, o, out, rows, cnt, S, ws, **kw)
            torch.cuda.synchronize()
            got = synth.storage_to_f64(synth.to_host(out))
            rows_h, cnt_h, S_h = rows.cpu().numpy(), cnt.cpu().numpy(), S.cpu().numpy()
            for b in range(batch):
                S_ref = oracle.chunk_scores(Lm_h[b], qh[b])
                assert max_rel(S_h[b], S_ref) <= 2e-2, "chunk scores"
                rl = []
                for g in range(H_kv):
                    want = oracle.expand_chunks(oracle.select(S_h[b, g], k_ch), outl_h[b, g][:o], c, L)
                    assert cnt_h[b, g] == len(want), ("count", bits, b, g, cnt_h[b, g], len(want))
                    assert rows_h[b, g, :len(want)].tolist() == want.tolist(), "rows"
                    rl.append(want)
                Ak = hats["A_k"][b] if bits else case["A_k"][b]
                Av = hats["A_v"][b] if bits else case["A_v"][b]
                ref = oracle.gather_attend_rows(Ak, Av, case["B_k"][b, 0], case["B_v"][b, 0], qh[b], rl,
                                                rope_theta=(theta if theta > 0 else None),
                                                K_tail=(Kt_h[b] if T else None), V_tail=(Vt_h[b] if T else None))
                err = max_rel(got[b], ref)
                worst = max(worst, err)
                assert err <= TOL, (case_no, bits, b, err)
    print("worst error", worst)
