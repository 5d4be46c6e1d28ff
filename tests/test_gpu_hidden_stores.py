"""Regression test for the result stores that the streaming kernels issue from inline assembly.

The long-stream score kernel and the dense-reconstruction kernel write their results with hand-placed
global_store instructions (a store the compiler knows of inside their conditional code would make it drain the
prefetch queue every iteration).  A store of more than 64 bits reads its data registers shortly after issue, and
the kernels overwrite those registers with the next tile right away; the wait states that keep the two apart are
written by hand.  A missing wait state shows as a wrong value now and then, not on every call, so this test runs
the same call a few hundred times and compares every result bit for bit with the first, whose values are
themselves checked against the oracle (head scores) or against the staged product (reconstruction).  It stops at
the first mismatch.
"""
import numpy as np
import pytest

import oracle
from paper_2503_18893_amd import synth
from paper_2503_18893_amd import binding as xb

pytestmark = pytest.mark.gpu

REPEATS = 300


def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


# (query heads per KV head -> row length of the head-score array): 4 -> one 16-byte store per token,
# 7 -> two, 16 -> four; long enough (batch * L >= 512K tokens) for the long-stream kernel to be the one that runs
@pytest.mark.parametrize("H_kv,H_q,batch,L", [(8, 32, 16, 32768), (4, 28, 8, 65536), (2, 32, 16, 32768)])
def test_head_score_stores_are_stable_over_many_calls(H_kv, H_q, batch, L):
    torch = torch_mod()
    w = synth.Workload("hidden_stores", G=1, H_kv=H_kv, H_q=H_q, d_h=128, r_k=128, r_v=128, L=L, k=64, batch=batch,
                       dtype="bf16", a_scale=1.0 / np.sqrt(128.0), sigma_decay=0.8, q_scale=1.0 / np.sqrt(128.0))
    g = synth.make_group_device(w, seed=77)
    shape = xb.Shape.of(w)
    ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    q = g["q"][0].contiguous()
    nrp = xb.head_pitch(shape)
    n_rep = H_q // H_kv
    S0 = torch.empty((batch, H_kv, L), dtype=torch.float32, device="cuda")
    heads0 = torch.full((batch, H_kv, L, nrp), float("nan"), dtype=torch.float32, device="cuda")
    xb.xkv_head_scores(shape, 0, g["A_k"], g["B_k"], q, S0, heads0, ws)
    torch.cuda.synchronize()
    # the reference call itself: pooled = max of the stored heads, padding zero, a sampled range against the oracle
    assert torch.equal(S0, heads0[..., :n_rep].max(dim=-1).values)
    assert bool((heads0[..., n_rep:] == 0).all())
    b = batch - 1
    A_k = synth.to_host(g["A_k"][b, L - 4096:])
    ref = oracle.head_scores(A_k, synth.to_host(g["B_k"][b, 0]), synth.to_host(q[b]), H_kv, oracle.default_scale(w.d_h))
    got = heads0[b, :, L - 4096:, :n_rep].cpu().numpy().transpose(0, 2, 1).reshape(H_q, 4096)
    assert float(np.abs(got - ref).max() / np.abs(ref).max()) <= 2e-2
    # the pooled scores of the kernel variant without the head-score stores must be the same numbers
    S_plain = torch.empty_like(S0)
    xb.xkv_score(shape, 0, g["A_k"], g["B_k"], q, S_plain, ws)
    torch.cuda.synchronize()
    assert torch.equal(S_plain, S0)
    S = torch.empty_like(S0)
    heads = torch.empty_like(heads0)
    for it in range(REPEATS):
        heads.fill_(float("nan"))
        xb.xkv_head_scores(shape, 0, g["A_k"], g["B_k"], q, S, heads, ws)
        ok = bool(torch.equal(heads, heads0)) and bool(torch.equal(S, S0))
        if not ok:
            bad = int((heads != heads0).sum())
            pytest.fail(f"call {it}: {bad} head scores differ from the first call's")


def test_reconstruction_row_stores_are_stable_over_many_calls():
    torch = torch_mod()
    w = synth.LLAMA_GROUP.with_(L=40000, r_k=256, r_v=256, batch=2, G=1, a_scale=1.0 / 16.0)
    g = synth.make_group_device(w, seed=78)
    shape = xb.Shape.of(w)
    K0 = torch.empty((w.batch, w.H_kv, w.L, w.d_h), dtype=torch.bfloat16, device="cuda")
    xb.xkv_reconstruct(shape, 0, g["A_k"], g["B_k"], w.r_k, K0)
    torch.cuda.synchronize()
    # the reference call against the definition A B_l on a sampled token range
    t0 = w.L - 1000
    ref = oracle.reconstruct(synth.to_host(g["A_k"][1, t0:]), synth.to_host(g["B_k"][1, 0]))       # [1000][d]
    got = synth.storage_to_f64(synth.to_host(K0[1, :, t0:])).transpose(1, 0, 2).reshape(1000, w.d)
    assert float(np.abs(got - ref).max() / np.abs(ref).max()) <= 2e-2
    K = torch.empty_like(K0)
    for it in range(REPEATS // 3):
        K.zero_()
        xb.xkv_reconstruct(shape, 0, g["A_k"], g["B_k"], w.r_k, K)
        if not bool(torch.equal(K, K0)):
            pytest.fail(f"call {it}: {int((K != K0).sum())} reconstructed values differ from the first call's")
