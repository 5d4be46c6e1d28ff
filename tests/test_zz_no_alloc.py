"""xkv_sr_decode_static -- the SR step for callers that cannot allocate -- against xkv_sr_decode, through the C ABI.

Both run the same kernels, so outputs, index sets and pooled scores must agree bit for bit (which is inside the
tolerance of the parity tests: identical index sets, outputs within 2e-2 / 1e-5 of the oracle-checked call); the
output of the first call is also checked against the CPU oracle.  Two calls in a row share the library's built-in
scratch array, the second on a smaller input, so anything the first call left behind would show.  Shapes whose
workspace exceeds the built-in array are rejected on the host.
"""
import numpy as np
import pytest

import oracle
from paper_2503_18893_amd import synth
from paper_2503_18893_amd import binding as xb

pytestmark = pytest.mark.gpu


def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def run_both(torch, w, seed):
    case = synth.make_case(w, seed=seed)
    dev = synth.to_device(case, w.dtype)
    shape = xb.Shape.of(w)
    assert xb.xkv_workspace_bytes(shape) <= xb.STATIC_SCRATCH_BYTES
    dt = synth.torch_dtype(w.dtype)
    q = dev["q"][0].contiguous()
    res = {}
    for name in ("workspace", "static"):
        out = torch.full((w.batch, w.H_q, w.d_h), float("nan"), dtype=dt, device="cuda")
        idx = torch.full((w.batch, w.H_kv, w.k), -1, dtype=torch.int32, device="cuda")
        S = torch.full((w.batch, w.H_kv, w.L), float("nan"), dtype=torch.float32, device="cuda")
        if name == "workspace":
            ws = xb.alloc_workspace(shape)
            xb.xkv_sr_decode(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out, idx, S, ws)
        else:
            xb.xkv_sr_decode_static(shape, 0, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], q, out, idx, S)
        torch.cuda.synchronize()
        res[name] = (synth.to_host(out), idx.cpu().numpy(), S.cpu().numpy())
    return case, res


def check(w, case, res):
    out_w, idx_w, S_w = res["workspace"]
    out_s, idx_s, S_s = res["static"]
    np.testing.assert_array_equal(idx_s, idx_w)
    np.testing.assert_array_equal(S_s, S_w)
    np.testing.assert_array_equal(out_s, out_w)
    # and against the oracle, on the selection the call made (the selection itself against the oracle's on its scores)
    tol = 1e-5 if w.dtype == "f32" else 2e-2
    for b in range(w.batch):
        for g in range(w.H_kv):
            np.testing.assert_array_equal(idx_s[b, g], oracle.select(S_s[b, g], w.k))
        ref = oracle.gather_attend(case["A_k"][b], case["A_v"][b], case["B_k"][b, 0], case["B_v"][b, 0],
                                   case["q"][0, b], idx_s[b])
        got = synth.storage_to_f64(out_s[b])
        assert float(np.abs(got - ref).max() / np.abs(ref).max()) <= tol


def test_static_scratch_step_matches_workspace_step_on_two_calls_in_a_row():
    torch = torch_mod()
    # first a bf16 shape on the matrix-core kernels with rows above the one-launch selection's limit (so the
    # scratch holds histograms, packed B, partials), then a smaller one, then the tiny fp32 configuration
    big = synth.LLAMA_GROUP.with_(L=70001, k=1500, r_k=128, r_v=256, batch=2, G=1)
    small = synth.LLAMA_GROUP.with_(L=5000, k=300, r_k=128, r_v=128, batch=1, G=1)
    for w, seed in ((big, 5), (small, 6), (synth.TINY, 0)):
        case, res = run_both(torch, w, seed)
        check(w, case, res)


def test_static_scratch_rejects_shapes_beyond_its_size():
    torch = torch_mod()
    w = synth.LLAMA_FULL
    shape = xb.Shape.of(w)
    assert xb.xkv_workspace_bytes(shape) > xb.STATIC_SCRATCH_BYTES
    t = torch.zeros(16, dtype=torch.bfloat16, device="cuda")     # never read: the call must fail before any launch
    with pytest.raises(xb.XkvError) as err:
        xb.xkv_sr_decode_static(shape, 0, t, t, t, t, t, t, None, None)
    assert err.value.status == xb.XKV_ERR_WORKSPACE


def test_static_scratch_step_can_be_recorded_into_a_graph():
    """The callers the entry point is for: a step recorded once (after one eager call, which looks the scratch
    array's address up) and replayed, every replay compared with the eager result, eager calls in between."""
    torch = torch_mod()
    w = synth.LLAMA_GROUP.with_(L=4096, k=512, batch=2)
    case = synth.make_case(w, seed=17)
    shape = xb.Shape.of(w)
    dev = synth.to_device(case, w.dtype)
    qs = [dev["q"][l].contiguous() for l in range(w.G)]
    outs = [torch.zeros((w.batch, w.H_q, w.d_h), dtype=torch.bfloat16, device="cuda") for _ in range(w.G)]
    idxs = [torch.zeros((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda") for _ in range(w.G)]

    def step():
        for l in range(w.G):
            xb.xkv_sr_decode_static(shape, l, dev["A_k"], dev["A_v"], dev["B_k"], dev["B_v"], qs[l], outs[l], idxs[l], None)

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
    for rep in range(3):
        for o, i in zip(outs, idxs):
            o.zero_()
            i.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(w.G):
            assert torch.equal(outs[l], want_out[l]) and torch.equal(idxs[l], want_idx[l]), (rep, l)
        step()                       # eager work between the replays
        torch.cuda.synchronize()
