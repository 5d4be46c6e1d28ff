#!/usr/bin/env python3
"""Benchmark of xKV Selective-Reconstruction decode attention on one MI355X.

A "step" is one decode step of the attention path of the whole model shape: every layer of every
layer group calls xkv_sr_decode once for the whole batch (query projection, low-rank score
stream, GQA max-pool, per-head top-k, gather-reconstruct, sparse softmax.V).  Inputs are seeded
synthetic factors resident in HBM before the timed region.  The dense baseline (xkv_dense_decode
on the uncompressed bf16 cache K = A^K B^K_l, V = A^V B^V_l of the same shape) is timed next to it.

Prints ONE JSON line: whole-job SR tokens/s (= batch * steps/s), the roofline of the dominant
kernel, and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama_full", choices=["llama_group", "llama_full", "qwen"])
    ap.add_argument("--batch", type=int, default=None, help="override the workload's batch")
    ap.add_argument("--L", type=int, default=None)
    ap.add_argument("--r", type=int, default=None, help="rank of both token bases (r_k = r_v)")
    ap.add_argument("--r-v", type=int, default=None, help="rank of the value basis alone (e.g. 1.5 x r_k)")
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--groups", type=int, default=None, help="override the number of layer groups held in HBM")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense baseline")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-factorize", action="store_true", help="skip the timing of the prefill-side factorization")
    ap.add_argument("--no-landmark", action="store_true", help="skip the timing of the landmark-guided step")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--no-absorbed", action="store_true", help="skip the timing of the absorbed form of the step")
    ap.add_argument("--no-quantized", action="store_true", help="skip the timing of the step on 4-bit token bases")
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise 1 GiB copy kernel three times (reference point for hardware counters)")
    return ap.parse_args()


def time_loop(torch, fn, iters):
    """Average milliseconds per call of fn over iters calls, by HIP events on the current stream."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); the path shards by sequence "
              "with no communication (every sequence has its own factors and queries)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2503_18893_amd import binding as xb, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    xb.load()

    w = {"llama_group": synth.LLAMA_GROUP, "llama_full": synth.LLAMA_FULL, "qwen": synth.QWEN}[args.workload]
    over = {}
    if args.batch is not None:
        over["batch"] = args.batch
    if args.L is not None:
        over["L"] = args.L
    if args.r is not None:
        over.update(r_k=args.r, r_v=args.r, a_scale=1.0 / float(np.sqrt(args.r)))
    if args.r_v is not None:
        over["r_v"] = args.r_v
    if args.k is not None:
        over["k"] = args.k
    if args.groups is not None:
        over["n_groups"] = args.groups
    if over:
        w = w.with_(**over)
    # the single-group workload is timed over several independently seeded copies so that the timed
    # working set is far above the 256 MiB last-level cache
    copies = 1
    e = 2 if w.dtype == "bf16" else 4
    group_bytes = w.batch * w.L * (w.r_k + w.r_v) * e
    if w.n_groups * group_bytes < (2 << 30):
        copies = int(np.ceil((2 << 30) / (w.n_groups * group_bytes)))
    n_sets = w.n_groups * copies

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)   # an elementwise kernel that reads 1 GiB and writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    t0 = time.perf_counter()
    groups = [synth.make_group_device(w, args.seed + 1000 * s) for s in range(n_sets)]
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t0

    shape = xb.Shape.of(w)
    ws = xb.alloc_workspace(shape)
    dt = synth.torch_dtype(w.dtype)
    out = torch.empty((w.batch, w.H_q, w.d_h), dtype=dt, device="cuda")
    qs = [[g["q"][l].contiguous() for l in range(w.G)] for g in groups]

    state = {"set0": 0}

    # B_l of every factor set in the gather-reconstruct kernel's operand order, made once (as a serving stack would at
    # prefill: B_l does not change between decode steps).  Shapes the matrix-core kernel does not take keep the
    # plain-layout call.
    packs = None
    try:
        pack_bytes = xb.xkv_packed_b_bytes(shape)
        packs = [torch.empty(pack_bytes, dtype=torch.uint8, device="cuda") for _ in range(n_sets)]
        for s_i in range(n_sets):
            xb.xkv_pack_b(shape, groups[s_i]["B_k"], groups[s_i]["B_v"], packs[s_i])
        torch.cuda.synchronize()
    except xb.XkvError:
        packs = None

    def plain_step():
        base = state["set0"]
        for grp in range(w.n_groups):
            s = (base + grp) % n_sets
            g = groups[s]
            for l in range(w.G):
                xb.xkv_sr_decode(shape, l, g["A_k"], g["A_v"], g["B_k"], g["B_v"], qs[s][l], out, None, None, ws)
        state["set0"] = (base + w.n_groups) % n_sets

    def packed_step():
        base = state["set0"]
        for grp in range(w.n_groups):
            s = (base + grp) % n_sets
            g = groups[s]
            for l in range(w.G):
                xb.xkv_sr_decode_packed(shape, l, g["A_k"], g["A_v"], g["B_k"], packs[s], qs[s][l], out, None, None, ws)
        state["set0"] = (base + w.n_groups) % n_sets

    sr_step = packed_step if packs is not None else plain_step

    for _ in range(args.warmup):
        sr_step()
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    ms_sr = time_loop(torch, sr_step, args.steps)
    t_wall = time.perf_counter() - t_wall0
    tokens_per_s = w.batch / (ms_sr * 1e-3)
    plain_layout = None
    if packs is not None:          # the same step through the call that takes B_l in its plain layout
        plain_step()
        ms_plain = time_loop(torch, plain_step, max(2, min(args.steps, 5)))
        plain_layout = {"ms_per_step": round(ms_plain, 4), "tokens_per_s": round(w.batch / (ms_plain * 1e-3), 2),
                        "note": "xkv_sr_decode: B_l re-ordered for the matrix-core kernel on every call; `value` is "
                                "xkv_sr_decode_packed on B_l re-ordered once per prompt by xkv_pack_b"}
        state["set0"] = 0

    # The same step recorded once into a HIP graph and replayed: the calls allocate nothing and synchronise nothing, so
    # a serving loop can take the 5 launches per layer out of the host's hands.  Reported next to the eager figure.
    graph_replay = None
    if not args.no_graph:
        try:
            state["set0"] = 0
            sr_step()
            torch.cuda.synchronize()
            eager_out = out.clone()
            state["set0"] = 0
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    sr_step()
            torch.cuda.current_stream().wait_stream(side)
            same = True
            for _ in range(3):                      # replays interleaved with eager work, each checked
                out.zero_()
                graph.replay()
                torch.cuda.synchronize()
                same = same and bool(torch.equal(out, eager_out))
                S_scratch = torch.empty(1024, device="cuda").normal_()
                torch.cuda.synchronize()
            ms_graph = time_loop(torch, graph.replay, args.steps)
            graph_replay = {"ms_per_step": round(ms_graph, 4), "tokens_per_s": round(w.batch / (ms_graph * 1e-3), 2),
                            "identical_to_eager": same,
                            "note": "one recorded step (all layers) replayed as a HIP graph; `value` is the eager figure"}
            del graph
        except Exception as err:                    # graph capture is an extra; never fail the benchmark on it
            graph_replay = {"skipped": f"{type(err).__name__}: {err}"}
        state["set0"] = 0

    # ---------------------------------------------------------------- per-stage timing (same inputs)
    S = torch.empty((w.batch, w.H_kv, w.L), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
    n_launch = w.n_groups * w.G

    def stage_loop(kind):
        def fn():
            base = state["set0"]
            for grp in range(w.n_groups):
                s = (base + grp) % n_sets
                g = groups[s]
                for l in range(w.G):
                    if kind == "score":
                        xb.xkv_score(shape, l, g["A_k"], g["B_k"], qs[s][l], S, ws)
                    elif kind == "topk":
                        xb.xkv_topk(shape, S, idx, ws)
                    else:
                        xb.xkv_gather_attend(shape, l, g["A_k"], g["A_v"], g["B_k"], g["B_v"], qs[s][l], idx, out,
                                             ws)
            state["set0"] = (base + w.n_groups) % n_sets
        return fn

    stage_iters = max(2, min(args.steps, 5))
    stage_ms = {}
    for kind in ("score", "topk", "gather_attend"):
        fn = stage_loop(kind)
        fn()
        stage_ms[kind] = time_loop(torch, fn, stage_iters) / n_launch   # ms per layer call
    bytes_score = w.batch * (e * (w.L * w.r_k + w.r_k * w.d) + 4 * w.H_kv * w.L)
    bytes_gather = w.batch * (e * w.H_kv * w.k * (w.r_k + w.r_v) + e * (w.r_k + w.r_v) * w.d)
    bytes_topk = w.batch * (4 * w.H_kv * w.L + 4 * w.H_kv * w.k)
    stage_bytes = {"score": bytes_score, "topk": bytes_topk, "gather_attend": bytes_gather}
    stages = {kname: {"ms_per_layer": round(ms, 5), "alg_bytes": stage_bytes[kname],
                      "GBps": round(stage_bytes[kname] / (ms * 1e-3) / 1e9, 1)} for kname, ms in stage_ms.items()}
    # duration of the two big kernels alone: the library records an event pair around the kernel launch
    def kernel_ms(stage_id, call):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        ev1.record()                      # creates the HIP events; the library re-records them
        torch.cuda.synchronize()
        xb.xkv_profile_kernel(stage_id, ev0.cuda_event, ev1.cuda_event)
        total, count = 0.0, 0
        for s in range(min(n_sets, w.n_groups)):
            for l in range(w.G):
                call(s, l)
                torch.cuda.synchronize()
                total += ev0.elapsed_time(ev1)
                count += 1
        xb.xkv_profile_kernel(stage_id, None, None)
        return total / count

    kern_ms = {
        "score": kernel_ms(xb.STAGE_SCORE, lambda s, l: xb.xkv_score(shape, l, groups[s]["A_k"], groups[s]["B_k"],
                                                                     qs[s][l], S, ws)),
        "gather_attend": kernel_ms(xb.STAGE_GATHER_ATTEND,
                                   lambda s, l: xb.xkv_gather_attend(shape, l, groups[s]["A_k"], groups[s]["A_v"],
                                                                     groups[s]["B_k"], groups[s]["B_v"], qs[s][l],
                                                                     idx, out, ws)),
    }
    # algorithmic bytes of the kernels alone: the score kernel reads the projected queries, not B^K_l (the projection
    # pre-pass does), so the r_K d term of the score stage is left out; the gather-reconstruct kernel reads B^K_l and
    # B^V_l itself (in fragment order), so its figure is the stage's: selected rows plus B once
    kern_bytes = {"score": w.batch * (e * w.L * w.r_k + 4 * w.H_kv * w.L),
                  "gather_attend": bytes_gather}
    for kname in kern_ms:
        stages[kname]["kernel_ms"] = round(kern_ms[kname], 5)
        stages[kname]["kernel_GBps"] = round(kern_bytes[kname] / (kern_ms[kname] * 1e-3) / 1e9, 1)
    dom = max(("score", "gather_attend"), key=lambda kname: kern_ms[kname])
    achieved = kern_bytes[dom] / (kern_ms[dom] * 1e-3) / 1e9
    # HBM traffic per launch from the committed counter summary of this exact workload and kernel, if there is one
    # (a stored profile figure: counters are not collected inside this run); null otherwise
    traffic = None
    tfile = os.path.join(ROOT, "profiles", f"hbm_traffic_{dom}_{args.workload}.txt")
    if os.path.exists(tfile) and not over:
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(float(line.split(":")[1]))
    roofline = {"kernel": {"score": "score_stream_kernel / score_mfma_kernel (low-rank score stream + GQA max-pool)",
                           "gather_attend": "gather_attend_mfma_kernel (gather-reconstruct + sparse attention)"}[dom],
                "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "alg_bytes_per_launch": kern_bytes[dom], "ms_per_launch": round(kern_ms[dom], 5),
                # both big kernels, not only the longer one
                "kernels": {kname: {"achieved": round(kern_bytes[kname] / (kern_ms[kname] * 1e-3) / 1e9, 1),
                                    "frac": round(kern_bytes[kname] / (kern_ms[kname] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                    "alg_bytes_per_launch": kern_bytes[kname],
                                    "ms_per_launch": round(kern_ms[kname], 5)} for kname in kern_ms}}

    # ---------------------------------------------------------------- dense baseline on the uncompressed cache
    dense = None
    if not args.no_dense:
        layer_bytes = 2 * w.batch * w.L * w.d * e
        free_b, _ = torch.cuda.mem_get_info()
        n_dense_layers = int(min(n_sets * w.G, max(1, (free_b - (8 << 30)) // layer_bytes)))
        n_dense_layers = max(1, min(n_dense_layers, w.n_layers if copies == 1 else n_sets * w.G))
        Ks, Vs, dq = [], [], []
        for i in range(n_dense_layers):
            s, l = divmod(i, w.G)
            g = groups[s]
            K = torch.empty((w.batch, w.H_kv, w.L, w.d_h), dtype=dt, device="cuda")
            V = torch.empty_like(K)
            xb.xkv_reconstruct(shape, l, g["A_k"], g["B_k"], w.r_k, K)
            xb.xkv_reconstruct(shape, l, g["A_v"], g["B_v"], w.r_v, V)
            Ks.append(K)
            Vs.append(V)
            dq.append(qs[s][l])
        torch.cuda.synchronize()
        dstate = {"i": 0}

        def dense_step():
            for _ in range(w.n_layers):
                i = dstate["i"]
                xb.xkv_dense_decode(shape, Ks[i], Vs[i], dq[i], out, ws)
                dstate["i"] = (i + 1) % n_dense_layers

        dense_step()
        ms_dense = time_loop(torch, dense_step, max(2, min(args.steps, 5)))
        bytes_dense = w.batch * 2 * e * w.L * w.d
        dense = {"ms_per_step": round(ms_dense, 4), "tokens_per_s": round(w.batch / (ms_dense * 1e-3), 2),
                 "GBps": round(bytes_dense * w.n_layers / (ms_dense * 1e-3) / 1e9, 1),
                 "layers_resident": n_dense_layers,
                 "note": "all layers resident" if n_dense_layers >= w.n_layers else
                         f"timed over {n_dense_layers} resident layer caches visited round-robin"}
        # xKV decode without selection (Sec. 3.2): every layer reconstructs its whole K and V from the factors and
        # attends densely over them.  Two scratch caches, reused by every layer.
        if w.dtype == "bf16":
            Kr, Vr = Ks[0], Vs[0]

            def dense_reconstruct_step():
                for grp in range(w.n_groups):
                    g = groups[grp % n_sets]
                    for l in range(w.G):
                        xb.xkv_reconstruct(shape, l, g["A_k"], g["B_k"], w.r_k, Kr)
                        xb.xkv_reconstruct(shape, l, g["A_v"], g["B_v"], w.r_v, Vr)
                        xb.xkv_dense_decode(shape, Kr, Vr, qs[grp % n_sets][l], out, ws)

            dense_reconstruct_step()
            ms_dr = time_loop(torch, dense_reconstruct_step, 2)
            dense["reconstruct_then_dense"] = {"ms_per_step": round(ms_dr, 3),
                                               "tokens_per_s": round(w.batch / (ms_dr * 1e-3), 2),
                                               "note": "xKV without selection: K and V of every layer rebuilt from "
                                                       "the factors (A B_l), then dense attention"}
        del Ks, Vs

    # ---------------------------------------------------------------- the same step with the paper's own selector
    # Landmark-guided chunk selection (App. B.1): chunks of c = 8 tokens scored against their mean key, top
    # ceil(k / c) chunks plus 4 static outlier chunks per KV head, then the same reconstruction and attention.
    # Landmarks of every resident layer are built once from K = A^K B^K_l (stand-in for post-RoPE keys).
    landmark = None
    if not args.no_landmark and w.L >= 64:
        c_lm, o_lm = 8, 4
        n_c = -(-w.L // c_lm)
        lm_ws = torch.empty(xb.xkv_landmark_workspace_bytes(shape, c_lm, o_lm), dtype=torch.uint8, device="cuda")
        Kscr = torch.empty((w.batch, w.H_kv, w.L, w.d_h), dtype=dt, device="cuda")
        lms, outls = [], []
        n_lm_layers = min(n_sets, w.n_groups) * w.G
        ev_a, ev_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ms_build = 0.0
        for i in range(n_lm_layers):
            s_i, l_i = divmod(i, w.G)
            g = groups[s_i]
            xb.xkv_reconstruct(shape, l_i, g["A_k"], g["B_k"], w.r_k, Kscr)
            lm_t = torch.empty((w.batch, w.H_kv, n_c, w.d_h), dtype=dt, device="cuda")
            ol_t = torch.empty((w.batch, w.H_kv, o_lm), dtype=torch.int32, device="cuda")
            ev_a.record()
            xb.xkv_landmarks(shape, Kscr, c_lm, o_lm, lm_t, None, ol_t, lm_ws)
            ev_b.record()
            torch.cuda.synchronize()
            ms_build += ev_a.elapsed_time(ev_b)
            lms.append(lm_t)
            outls.append(ol_t)
        del Kscr
        lstate = {"i": 0}

        def landmark_call(i, s_i, l_i, theta):   # on B_l re-ordered once per prompt where the shape has that form
            g = groups[s_i]
            if packs is not None:
                xb.xkv_sr_decode_landmark_packed(shape, l_i, g["A_k"], g["A_v"], 0, g["B_k"], packs[s_i], qs[s_i][l_i],
                                                 lms[i], outls[i], c_lm, o_lm, out, None, None, None, lm_ws,
                                                 rope_theta=theta)
            else:
                xb.xkv_sr_decode_landmark(shape, l_i, g["A_k"], g["A_v"], g["B_k"], g["B_v"], qs[s_i][l_i], lms[i],
                                          outls[i], c_lm, o_lm, out, None, None, None, lm_ws, rope_theta=theta)

        def landmark_step():
            for _ in range(w.n_layers):
                i = lstate["i"]
                s_i, l_i = divmod(i, w.G)
                landmark_call(i, s_i, l_i, 0.0)
                lstate["i"] = (i + 1) % n_lm_layers

        landmark_step()
        ms_lm = time_loop(torch, landmark_step, max(2, min(args.steps, 5)))
        rope_theta = 500000.0     # Llama-3.1's rotary base; reconstructed key rows are rotated to their positions

        def landmark_rope_step():
            for _ in range(w.n_layers):
                i = lstate["i"]
                s_i, l_i = divmod(i, w.G)
                landmark_call(i, s_i, l_i, rope_theta)
                lstate["i"] = (i + 1) % n_lm_layers

        ms_lm_rope = None
        try:
            landmark_rope_step()
            ms_lm_rope = time_loop(torch, landmark_rope_step, max(2, min(args.steps, 5)))
        except xb.XkvError:
            pass                  # head widths the rotation does not cover
        landmark = {"ms_per_step": round(ms_lm, 4), "tokens_per_s": round(w.batch / (ms_lm * 1e-3), 2), "c": c_lm,
                    "outlier_chunks": o_lm, "rows_per_head_max": (min(-(-w.k // c_lm), n_c) + o_lm) * c_lm,
                    "landmark_build_ms_per_layer": round(ms_build / n_lm_layers, 4),
                    "with_rope": None if ms_lm_rope is None else {
                        "ms_per_step": round(ms_lm_rope, 4), "tokens_per_s": round(w.batch / (ms_lm_rope * 1e-3), 2),
                        "rope_theta": rope_theta},
                    "entry_point": "xkv_sr_decode_landmark_packed" if packs is not None else "xkv_sr_decode_landmark",
                    "note": "SR decode with landmark-guided chunk selection instead of scoring every token from the "
                            "factors; same reconstruction and attention kernels"}
        del lms, outls, lm_ws

    # ---------------------------------------------------------------- the absorbed form of the step (an extra)
    # Same scores and selection; stages 3-4 gather the selected tokens' head scores and sum rows of A^V instead of
    # rebuilding K^ and V^.  Valid where no rotation follows the reconstruction.  Not `value`.
    absorbed = None
    if not args.no_absorbed:
        try:
            ab_ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
            heads = torch.empty((w.batch, w.H_kv, w.L, xb.head_pitch(shape)), dtype=torch.float32, device="cuda")

            def absorbed_step():
                base = state["set0"]
                for grp in range(w.n_groups):
                    s = (base + grp) % n_sets
                    g = groups[s]
                    for l in range(w.G):
                        xb.xkv_sr_decode_absorbed(shape, l, g["A_k"], g["A_v"], g["B_k"], g["B_v"], qs[s][l], out, None,
                                                  None, ab_ws)
                state["set0"] = (base + w.n_groups) % n_sets

            absorbed_step()
            ms_ab = time_loop(torch, absorbed_step, max(2, min(args.steps, 5)))
            ab_kern = {
                "head_scores": kernel_ms(xb.STAGE_SCORE,
                                         lambda s, l: xb.xkv_head_scores(shape, l, groups[s]["A_k"], groups[s]["B_k"],
                                                                         qs[s][l], S, heads, ab_ws)),
                "absorb_rows": kernel_ms(xb.STAGE_ABSORB_ROWS,
                                         lambda s, l: xb.xkv_attend_absorbed(shape, l, groups[s]["A_v"], groups[s]["B_v"],
                                                                             heads, idx, out, ab_ws)),
            }
            ab_bytes = {"head_scores": w.batch * (e * w.L * w.r_k + 4 * w.H_kv * w.L * (1 + xb.head_pitch(shape))),
                        "absorb_rows": w.batch * w.H_kv * w.k * (e * w.r_v + 4 * xb.head_pitch(shape))}
            absorbed = {"ms_per_step": round(ms_ab, 4), "tokens_per_s": round(w.batch / (ms_ab * 1e-3), 2),
                        "speedup_vs_gather_reconstruct": round(ms_sr / ms_ab, 3),
                        "kernels": {kn: {"kernel_ms": round(ab_kern[kn], 5), "alg_bytes": ab_bytes[kn],
                                         "kernel_GBps": round(ab_bytes[kn] / (ab_kern[kn] * 1e-3) / 1e9, 1)}
                                    for kn in ab_kern},
                        "note": "xkv_sr_decode_absorbed: per-head scores kept by the score kernel, softmax over the "
                                "selected ones, weighted sum of rows of A^V, B^V applied once per head"}
            del ab_ws, heads
        except xb.XkvError as err:
            absorbed = {"skipped": str(err)}

    # ---------------------------------------------------------------- the absorbed step on 4-bit token bases (an extra)
    # A^K and A^V of every factor set quantised once (as prefill would), then the absorbed step straight from the
    # quantised rows.  What it computes is the step on the de-quantised values.  Not `value`.
    quantized = None
    if not args.no_quantized and w.dtype == "bf16":
        try:
            rb_k, rb_v = xb.xkv_quantized_row_bytes(w.r_k), xb.xkv_quantized_row_bytes(w.r_v)
            q_ws = torch.empty(xb.xkv_absorbed_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
            n_q = min(n_sets, w.n_groups)
            Aqk, Aqv = [], []
            ev_a, ev_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ms_quant = 0.0
            for s_i in range(n_q):
                ak = torch.empty((w.batch, w.L, rb_k), dtype=torch.uint8, device="cuda")
                av = torch.empty((w.batch, w.L, rb_v), dtype=torch.uint8, device="cuda")
                ev_a.record()
                xb.xkv_quantize_rows(groups[s_i]["A_k"], w.batch * w.L, w.r_k, ak)
                xb.xkv_quantize_rows(groups[s_i]["A_v"], w.batch * w.L, w.r_v, av)
                ev_b.record()
                torch.cuda.synchronize()
                ms_quant += ev_a.elapsed_time(ev_b)
                Aqk.append(ak)
                Aqv.append(av)
            qstate = {"set0": 0}

            def quantized_step():
                base = qstate["set0"]
                for grp in range(w.n_groups):
                    s_i = (base + grp) % n_q
                    g = groups[s_i]
                    for l in range(w.G):
                        xb.xkv_sr_decode_absorbed_q4(shape, l, Aqk[s_i], Aqv[s_i], g["B_k"], g["B_v"], qs[s_i][l], out,
                                                     None, None, q_ws)
                qstate["set0"] = (base + w.n_groups) % n_q

            quantized_step()
            ms_q = time_loop(torch, quantized_step, max(2, min(args.steps, 5)))
            heads_q = torch.empty((w.batch, w.H_kv, w.L, xb.head_pitch(shape)), dtype=torch.float32, device="cuda")

            qk = {
                "head_scores_q4": kernel_ms(xb.STAGE_SCORE,
                                              lambda s_i, l: xb.xkv_head_scores_q4(shape, l, Aqk[s_i], groups[s_i]["B_k"],
                                                                                   qs[s_i][l], S, heads_q, q_ws)),
                "absorb_rows_q4": kernel_ms(xb.STAGE_ABSORB_ROWS,
                                              lambda s_i, l: xb.xkv_attend_absorbed_q4(shape, l, Aqv[s_i],
                                                                                       groups[s_i]["B_v"], heads_q, idx,
                                                                                       out, q_ws)),
            }
            qb = {"head_scores_q4": w.batch * (w.L * rb_k + 4 * w.H_kv * w.L * (1 + xb.head_pitch(shape))),
                  "absorb_rows_q4": w.batch * w.H_kv * w.k * (rb_v + 4 * xb.head_pitch(shape))}
            quantized = {"ms_per_step": round(ms_q, 4), "tokens_per_s": round(w.batch / (ms_q * 1e-3), 2),
                         "speedup_vs_bf16_gather_reconstruct": round(ms_sr / ms_q, 3), "bits": 4,
                         "bytes_per_row": {"A_k": rb_k, "A_v": rb_v, "bf16": {"A_k": 2 * w.r_k, "A_v": 2 * w.r_v}},
                         "quantize_ms_per_group": round(ms_quant / n_q, 3),
                         "quantize_GBps": round(n_q * w.batch * w.L * (2 * (w.r_k + w.r_v) + rb_k + rb_v)
                                                / (ms_quant * 1e-3) / 1e9, 1),
                         "kernels": {kn: {"kernel_ms": round(qk[kn], 5), "alg_bytes": qb[kn],
                                          "kernel_GBps": round(qb[kn] / (qk[kn] * 1e-3) / 1e9, 1)} for kn in qk},
                         "note": "xkv_sr_decode_absorbed_q4: both token bases as 4-bit round-to-nearest rows (groups of "
                                 "32 ranks, bf16 step and offset), de-quantised inside the score and row-sum kernels"}
            # the gather-reconstruct form of the step on the same 4-bit rows (scores from the quantised A^K, Eq. 3 and
            # attention from quantised rows: the form that still allows a rotation of the reconstructed keys), and
            # its big kernel alone on 4-bit and on 3-bit rows
            try:
                def q4_gather_step():
                    base = qstate["set0"]
                    for grp in range(w.n_groups):
                        s_i = (base + grp) % n_q
                        g = groups[s_i]
                        for l in range(w.G):
                            xb.xkv_sr_decode_q4(shape, l, Aqk[s_i], Aqv[s_i], g["B_k"], g["B_v"], qs[s_i][l], out, None,
                                                None, q_ws)
                    qstate["set0"] = (base + w.n_groups) % n_q

                q4_gather_step()
                ms_qg = time_loop(torch, q4_gather_step, max(2, min(args.steps, 5)))
                gk = {}
                for bits in (4, 3):
                    rbk, rbv = xb.xkv_quantized_row_bytes(w.r_k, bits), xb.xkv_quantized_row_bytes(w.r_v, bits)
                    if bits == 4:
                        ak3, av3 = Aqk[0], Aqv[0]
                    else:
                        ak3 = torch.empty((w.batch, w.L, rbk), dtype=torch.uint8, device="cuda")
                        av3 = torch.empty((w.batch, w.L, rbv), dtype=torch.uint8, device="cuda")
                        xb.xkv_quantize_rows(groups[0]["A_k"], w.batch * w.L, w.r_k, ak3, bits=3)
                        xb.xkv_quantize_rows(groups[0]["A_v"], w.batch * w.L, w.r_v, av3, bits=3)
                    ms_k = kernel_ms(xb.STAGE_GATHER_ATTEND,
                                     lambda s_i, l: xb.xkv_gather_attend_q(shape, l, ak3, av3, bits, groups[0]["B_k"],
                                                                           groups[0]["B_v"], qs[0][l], idx, None, 0.0,
                                                                           out, ws))
                    gbytes = w.batch * w.H_kv * w.k * (rbk + rbv)
                    gk[f"gather_attend_q{bits}"] = {"kernel_ms": round(ms_k, 5), "alg_bytes": gbytes,
                                                    "kernel_GBps": round(gbytes / (ms_k * 1e-3) / 1e9, 1),
                                                    "bytes_per_row": {"A_k": rbk, "A_v": rbv}}
                quantized["gather_reconstruct"] = {
                    "ms_per_step": round(ms_qg, 4), "tokens_per_s": round(w.batch / (ms_qg * 1e-3), 2),
                    "speedup_vs_bf16_gather_reconstruct": round(ms_sr / ms_qg, 3), "kernels": gk,
                    "note": "xkv_sr_decode_q4: Eq. 3 and attention from 4-bit rows de-quantised in registers inside "
                            "the matrix-core kernel; 3-bit rows through xkv_gather_attend_q (kernel time only)"}
            except xb.XkvError as err:
                quantized["gather_reconstruct"] = {"skipped": str(err)}
            del Aqk, Aqv, q_ws, heads_q
        except xb.XkvError as err:
            quantized = {"skipped": str(err)}

    # ---------------------------------------------------------------- the step before the path: factorization
    # One layer group's key cache of every sequence (power-law spectrum, full rank) -> A^K, B^K (Eq. 1), as prefill
    # would do once per prompt and group, for keys and for values.  Not part of the decode step or of `value`.
    factorize = None
    n_cat = w.G * w.d
    if not args.no_factorize and w.dtype == "bf16" and w.d_h % 64 == 0 and w.r_k <= min(1024, n_cat):
        iters_f = 8
        try:
            fz_bytes = xb.xkv_factorize_workspace_bytes(shape, w.r_k)
            gen = torch.Generator(device="cuda").manual_seed(args.seed + 17)
            spec = torch.arange(1, n_cat + 1, device="cuda", dtype=torch.float32) ** -0.7
            mix = torch.linalg.qr(torch.randn((n_cat, n_cat), device="cuda", generator=gen))[0]
            Xc = torch.empty((w.batch, w.G, w.H_kv, w.L, w.d_h), dtype=dt, device="cuda")
            for b in range(w.batch):
                z = torch.randn((w.L, n_cat), device="cuda", generator=gen) * spec
                Xc[b] = (z @ mix.T).view(w.L, w.G, w.H_kv, w.d_h).permute(1, 2, 0, 3).to(dt)
                del z
            fz_ws = torch.empty(fz_bytes, dtype=torch.uint8, device="cuda")
            A_f = torch.empty((w.batch, w.L, w.r_k), dtype=dt, device="cuda")
            B_f = torch.empty((w.batch, w.G, w.r_k, w.d), dtype=dt, device="cuda")

            def fz_call():
                xb.xkv_factorize(shape, Xc, w.r_k, iters_f, args.seed, A_f, B_f, fz_ws)

            fz_call()
            ms_fz = time_loop(torch, fz_call, 2)
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            ev1.record()
            torch.cuda.synchronize()
            xb.xkv_profile_kernel(xb.STAGE_FACTORIZE_GRAM, ev0.cuda_event, ev1.cuda_event)
            fz_call()                    # with more than 16 sequences the events keep the last chunk's launch
            torch.cuda.synchronize()
            ms_gram = ev0.elapsed_time(ev1)
            xb.xkv_profile_kernel(xb.STAGE_FACTORIZE_GRAM, None, None)
            chunk = w.batch % 16 or min(w.batch, 16)     # sequences in the last launch (16 per launch)
            tiles = -(-n_cat // 256)
            gram_flops = chunk * (tiles * (tiles + 1) // 2) * 256 * 256 * 2 * w.L   # tiles on or below the diagonal
            captured = float((A_f[0].float() ** 2).sum() / (Xc[0].float() ** 2).sum())
            factorize = {"ms_per_call": round(ms_fz, 3), "sequences": w.batch, "iters": iters_f, "r": w.r_k, "n": n_cat,
                         "ms_per_sequence_and_group": round(ms_fz / w.batch, 3),
                         "gram_kernel": {"ms_per_launch": round(ms_gram, 4), "sequences_per_launch": chunk,
                                         "bound": "mfma", "achieved": round(gram_flops / (ms_gram * 1e-3) / 1e12, 1),
                                         "peak": 2500.0, "unit": "TFLOP/s",
                                         "frac": round(gram_flops / (ms_gram * 1e-3) / 2.5e15, 4)},
                         "energy_captured_seq0": round(captured, 5),
                         "note": "xkv_factorize on one group's key cache (synthetic, singular values ~ i^-0.7); "
                                 "prefill-side, outside the timed decode step"}
            del Xc, fz_ws, A_f, B_f
        except xb.XkvError as err:
            factorize = {"skipped": str(err)}

    # ---------------------------------------------------------------- CPU oracle on a bounded sample
    cpu = None
    parity = None
    if not args.no_cpu:
        import oracle
        g0 = groups[0]
        n_l = w.G if w.L * w.r_k <= 40e6 else 1
        host = {name: synth.to_host(g0[name][0]) for name in ("A_k", "A_v", "B_k", "B_v")}
        qh = synth.to_host(g0["q"][:, 0])
        out_s = torch.empty_like(out)
        idx_s = torch.empty((w.batch, w.H_kv, w.k), dtype=torch.int32, device="cuda")
        errs = []
        t_cpu = 0.0
        for l in range(n_l):
            if packs is not None:
                xb.xkv_sr_decode_packed(shape, l, g0["A_k"], g0["A_v"], g0["B_k"], packs[0], qs[0][l], out_s, idx_s, None,
                                        ws)
            else:
                xb.xkv_sr_decode(shape, l, g0["A_k"], g0["A_v"], g0["B_k"], g0["B_v"], qs[0][l], out_s, idx_s, None, ws)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            ref, ref_idx, _ = oracle.sr_decode(host["A_k"], host["A_v"], host["B_k"][l], host["B_v"][l], qh[l],
                                               w.H_kv, w.k)
            t_cpu += time.perf_counter() - t1
            # parity of the output given the GPU's own selection (selection near the k-th score may differ by rounding)
            ref_g = oracle.gather_attend(host["A_k"], host["A_v"], host["B_k"][l], host["B_v"][l], qh[l],
                                         idx_s[0].cpu().numpy())
            got = synth.storage_to_f64(synth.to_host(out_s[0]))
            errs.append(float(np.abs(got - ref_g).max() / np.abs(ref_g).max()))
        per_layer_seq = t_cpu / n_l
        cpu_tokens_per_s = 1.0 / (per_layer_seq * w.n_layers)     # one sequence through all layers
        cpu = {"value": round(cpu_tokens_per_s, 6), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"sequence 0, {n_l} layer(s) of group 0 ({per_layer_seq:.2f} s per layer-sequence), "
                         f"extrapolated linearly to {w.n_layers} layers; sequences are independent"}
        parity = {"max_rel_err_vs_oracle_on_sample": max(errs), "tolerance": 2e-2 if w.dtype == "bf16" else 1e-5}

    result = {
        "metric": "SR decode tokens/s (attention path, all layers; batch x decode steps/s)",
        "value": round(tokens_per_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_sr, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers": w.n_layers, "G": w.G, "batch": w.batch, "L": w.L, "r_k": w.r_k,
                   "r_v": w.r_v, "k": w.k, "H_kv": w.H_kv, "H_q": w.H_q, "d_h": w.d_h,
                   "factor_sets_in_hbm": n_sets, "copies_rotated": copies},
        "roofline": roofline, "cpu_baseline": cpu, "stages": stages, "dense_baseline": dense,
        "speedup_vs_dense": (round(dense["ms_per_step"] / ms_sr, 3) if dense else None),
        "entry_point": "xkv_sr_decode_packed" if packs is not None else "xkv_sr_decode", "plain_layout_step": plain_layout,
        "graph_replay": graph_replay, "landmark_selector": landmark, "absorbed": absorbed, "quantized": quantized, "factorize": factorize, "parity": parity, "setup_s": round(t_gen, 1), "timed_wall_s": round(t_wall, 2),
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
