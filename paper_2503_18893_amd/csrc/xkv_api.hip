// C ABI of libxkv: argument validation, workspace carving and launch sequencing.
// Every step of the path runs in the HIP kernels of this library; nothing here computes.
#include <cmath>
#include <cstring>

#include "xkv_common.h"

namespace xkv {

ProfileEvents g_profile[4] = {};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

static xkv_status validate(const xkv_shape *s)
{
    if (!s) return XKV_ERR_INVALID_ARG;
    if (s->G < 1 || s->H_kv < 1 || s->H_q < 1 || s->d_h < 1 || s->r_k < 1 || s->r_v < 1 || s->L < 1 || s->batch < 0)
        return XKV_ERR_INVALID_ARG;
    if (s->H_q % s->H_kv != 0) return XKV_ERR_INVALID_ARG;
    if (s->k < 1 || s->k > s->L) return XKV_ERR_INVALID_ARG;
    if (s->dtype != XKV_F32 && s->dtype != XKV_BF16) return XKV_ERR_INVALID_ARG;
    if (!(s->scale >= 0.0f) || !std::isfinite(s->scale)) return XKV_ERR_INVALID_ARG;
    if (s->d_h > 256) return XKV_ERR_UNSUPPORTED;
    if (s->H_q / s->H_kv > 16) return XKV_ERR_UNSUPPORTED;
    if ((long long)s->batch * s->H_kv > 65535LL) return XKV_ERR_UNSUPPORTED;  // grid.y limit
    return XKV_OK;
}

xkv_status make_plan(const xkv_shape &s, Plan &p)
{
    std::memset(&p, 0, sizeof p);
    p.n_rep = s.H_q / s.H_kv;
    p.rows = s.batch * s.H_kv;
    p.scale = s.scale > 0.0f ? s.scale : 1.0f / std::sqrt((float)s.d_h);
    const int rows = p.rows > 0 ? p.rows : 1;
    const int want = ceil_div(1024, rows);  // aim at ~4 workgroups per compute unit

    int chunks = clampi(want, 1, clampi(ceil_div(s.L, 1024), 1, 128));
    p.topk_chunk = ceil_div(ceil_div(s.L, chunks), 256) * 256;
    p.topk_chunks = ceil_div(s.L, p.topk_chunk);
    // When the long-stream score kernel can also histogram the top key digit, the top-k chunks are its
    // workgroups' token ranges.
    bool hist_fits = false;
    p.score_stream = score_stream_plan(s, &p.score_tpw, &hist_fits, &p.score_waves);
    p.topk_row = topk_row_shape_ok(s);  // then the selection needs no histogram from the score kernel
    p.score_hist = !p.topk_row && p.score_stream && hist_fits && ceil_div(s.L, 32 * p.score_tpw) <= 128;
    if (p.score_hist) {
        p.topk_chunk = 32 * p.score_tpw;
        p.topk_chunks = ceil_div(s.L, p.topk_chunk);
    }

    // the matrix-core kernel walks 32 selected tokens per wavefront and iteration, the general one 16 per workgroup
    p.ga_mfma = gather_attend_mfma_shape_ok(s);
    p.ga_waves = p.ga_mfma ? gather_attend_mfma_waves(s) : 0;
    const int gran = p.ga_mfma ? 32 * p.ga_waves : 64;
    // (its workgroups occupy a compute unit alone, so about one workgroup per compute unit; but at least four
    // splits per (sequence, KV head): the splits of a head share its packed B in their XCD's L2, and with fewer of
    // them more than 8 packs (2 MiB) are live per XCD and the re-streamed fragments start to miss)
    const int ga_splits = ceil_div(256, rows) < 4 ? 4 : ceil_div(256, rows);
    int splits = clampi(p.ga_mfma ? ga_splits : want, 1, clampi(ceil_div(s.k, gran), 1, 64));
    if (splits < ceil_div(s.k, 4096)) splits = ceil_div(s.k, 4096);  // a workgroup keeps at most 4096 token ids in LDS
    p.sr_chunk = ceil_div(ceil_div(s.k, splits), gran) * gran;
    p.sr_splits = ceil_div(s.k, p.sr_chunk);

    splits = clampi(want, 1, clampi(ceil_div(s.L, 256), 1, 128));
    p.dense_mfma = dense_mfma_shape_ok(s);
    p.dense_chunk = ceil_div(ceil_div(s.L, splits), 128) * 128;  // 4 wavefronts x 32-token blocks
    p.dense_splits = ceil_div(s.L, p.dense_chunk);

    p.max_splits = 4 * (p.sr_splits > p.dense_splits ? p.sr_splits : p.dense_splits);  // one partial per wavefront

    const size_t b = (size_t)(s.batch > 0 ? s.batch : 1);
    size_t off = 0;
    p.off_p = off;
    off = align_up(off + b * (size_t)(2 * s.H_q + 64) * (s.r_k + 128) * sizeof(float), 256);  // fp32 P or bf16 hi/lo fragments
    p.off_score = off;
    off = align_up(off + b * s.H_kv * (size_t)s.L * sizeof(float), 256);
    p.off_idx = off;
    off = align_up(off + b * s.H_kv * (size_t)s.k * sizeof(int32_t), 256);
    p.off_hist = off;
    off = align_up(off + (size_t)rows * p.topk_chunks * kTopkLevels * kTopkBins * sizeof(uint32_t), 256);
    p.off_state = off;
    // per row: state words, the row's digit histograms, per-chunk counts of keys above the threshold
    off = align_up(off + (size_t)rows * (kStateWords + kTopkLevels * kTopkBins + p.topk_chunks) * sizeof(uint32_t),
                   256);
    p.off_part_o = off;
    off = align_up(off + b * s.H_q * (size_t)p.max_splits * s.d_h * sizeof(float), 256);
    p.off_part_ml = off;
    off = align_up(off + b * s.H_q * (size_t)p.max_splits * 2 * sizeof(float), 256);
    p.off_bpack = off;
    if (p.ga_mfma) off = align_up(off + gather_attend_pack_bytes(s), 256);
    p.off_tail_o = off;
    off = align_up(off + b * s.H_q * (size_t)kTailParts * s.d_h * sizeof(float), 256);
    p.off_tail_ml = off;
    off = align_up(off + b * s.H_q * (size_t)kTailParts * 2 * sizeof(float), 256);
    p.total = off;
    return XKV_OK;
}

static inline xkv_status hip_status(hipError_t e) { return e == hipSuccess ? XKV_OK : XKV_ERR_HIP; }

static xkv_status prepare(const xkv_shape *s, void *ws, size_t ws_bytes, Plan &p)
{
    xkv_status st = validate(s);
    if (st != XKV_OK) return st;
    make_plan(*s, p);
    if (!ws) return XKV_ERR_INVALID_ARG;
    if (ws_bytes < p.total) return XKV_ERR_WORKSPACE;
    if (((uintptr_t)ws) & 255u) return XKV_ERR_INVALID_ARG;
    return XKV_OK;
}

template <typename T> static inline T *at(void *ws, size_t off) { return reinterpret_cast<T *>((char *)ws + off); }

}  // namespace xkv

using namespace xkv;

extern "C" {

xkv_status xkv_workspace_bytes(const xkv_shape *shape, size_t *bytes)
{
    if (!bytes) return XKV_ERR_INVALID_ARG;
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    Plan p;
    make_plan(*shape, p);
    *bytes = p.total;
    return XKV_OK;
}

xkv_status xkv_score(const xkv_shape *shape, int32_t layer, const void *A_k, const void *B_k, const void *q,
                     float *score_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Plan p;
    xkv_status st = prepare(shape, workspace, workspace_bytes, p);
    if (st != XKV_OK) return st;
    if (!A_k || !B_k || !q || !score_out || layer < 0 || layer >= shape->G) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    return hip_status(launch_score_stage(*shape, p, layer, A_k, B_k, q, at<void>(workspace, p.off_p), score_out,
                                         nullptr, nullptr, nullptr, nullptr, nullptr, stream));
}

xkv_status xkv_topk(const xkv_shape *shape, const float *score, int32_t *idx_out, void *workspace,
                    size_t workspace_bytes, void *hip_stream)
{
    Plan p;
    xkv_status st = prepare(shape, workspace, workspace_bytes, p);
    if (st != XKV_OK) return st;
    if (!score || !idx_out) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    return hip_status(launch_topk(*shape, p, score, idx_out, at<uint32_t>(workspace, p.off_hist),
                                  at<uint32_t>(workspace, p.off_state), false, (hipStream_t)hip_stream));
}

xkv_status xkv_gather_attend(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                             const void *B_k, const void *B_v, const void *q, const int32_t *idx, void *out,
                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Plan p;
    xkv_status st = prepare(shape, workspace, workspace_bytes, p);
    if (st != XKV_OK) return st;
    if (!A_k || !A_v || !B_k || !B_v || !q || !idx || !out || layer < 0 || layer >= shape->G)
        return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *part_o = at<float>(workspace, p.off_part_o);
    float *part_ml = at<float>(workspace, p.off_part_ml);
    void *pack_ws = at<void>(workspace, p.off_bpack);
    const bool mfma = gather_attend_uses_mfma(p, A_k, A_v, B_k, B_v, pack_ws);
    hipError_t e = launch_gather_attend(*shape, p, layer, A_k, A_v, B_k, B_v, q, idx, pack_ws, false, part_o, part_ml,
                                        stream);
    // the matrix-core kernel writes one partial per split, the general one one per wavefront
    if (e == hipSuccess) e = launch_combine(*shape, mfma ? p.sr_splits : p.sr_splits * 4, part_o, part_ml, out, stream);
    return hip_status(e);
}

// SR step; K_tail / V_tail (T > 0 tokens per KV head, uncompressed) are attended together with the selected rows.
static xkv_status sr_decode_impl(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                                 const void *B_k, const void *B_v, const void *q, const void *K_tail,
                                 const void *V_tail, int32_t T, void *out, int32_t *idx_out, float *score_out,
                                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Plan p;
    xkv_status st = prepare(shape, workspace, workspace_bytes, p);
    if (st != XKV_OK) return st;
    if (!A_k || !A_v || !B_k || !B_v || !q || !out || layer < 0 || layer >= shape->G) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *S = score_out ? score_out : at<float>(workspace, p.off_score);
    int32_t *idx = idx_out ? idx_out : at<int32_t>(workspace, p.off_idx);
    float *part_o = at<float>(workspace, p.off_part_o);
    float *part_ml = at<float>(workspace, p.off_part_ml);
    uint32_t *hist = at<uint32_t>(workspace, p.off_hist), *state = at<uint32_t>(workspace, p.off_state);
    bool level0_done = false;
    hipError_t e = hipSuccess;
    if (p.score_hist) e = launch_topk_init(p, state, stream);  // the score kernel adds to the zeroed row histograms
    // B is packed for the matrix-core gather-attend kernel in the same launch as the query projection
    void *pack_ws = at<void>(workspace, p.off_bpack);
    PackArgs pa{};
    const bool want_pack = gather_attend_uses_mfma(p, A_k, A_v, B_k, B_v, pack_ws);
    if (want_pack) pa = gather_attend_pack_args(*shape, layer, B_k, B_v, q, pack_ws);
    bool packed = false;
    if (e == hipSuccess)
        e = launch_score_stage(*shape, p, layer, A_k, B_k, q, at<void>(workspace, p.off_p), S,
                               p.score_hist ? topk_row_hist(p, state) : nullptr, p.score_hist ? hist : nullptr,
                               &level0_done, want_pack ? &pa : nullptr, &packed, stream);
    if (e == hipSuccess) e = launch_topk(*shape, p, S, idx, hist, state, level0_done, stream);
    if (e == hipSuccess)
        e = launch_gather_attend(*shape, p, layer, A_k, A_v, B_k, B_v, q, idx, pack_ws, packed, part_o, part_ml,
                                 stream);
    // The uncompressed tail goes through the dense kernel as a context of T tokens of its own (at most 8 splits),
    // into a second set of partials; the merge below is one softmax over selected rows and tail.
    int n_tail = 0;
    float *tail_o = at<float>(workspace, p.off_tail_o), *tail_ml = at<float>(workspace, p.off_tail_ml);
    if (T > 0 && e == hipSuccess) {
        xkv_shape ts = *shape;
        ts.L = T;
        Plan tp = p;
        const int splits = clampi(ceil_div(T, 512), 1, kTailParts / 4);
        tp.dense_chunk = ceil_div(ceil_div(T, splits), 128) * 128;
        tp.dense_splits = ceil_div(T, tp.dense_chunk);
        e = launch_dense(ts, tp, K_tail, V_tail, q, tail_o, tail_ml, stream);
        n_tail = dense_uses_mfma(tp, K_tail, V_tail, q) ? tp.dense_splits : tp.dense_splits * 4;
    }
    // the matrix-core kernel writes one partial per split, the general one one per wavefront
    if (e == hipSuccess)
        e = launch_combine(*shape, want_pack ? p.sr_splits : p.sr_splits * 4, part_o, part_ml, out, stream, n_tail,
                           tail_o, tail_ml);
    return hip_status(e);
}

xkv_status xkv_sr_decode(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v, const void *B_k,
                         const void *B_v, const void *q, void *out, int32_t *idx_out, float *score_out,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return sr_decode_impl(shape, layer, A_k, A_v, B_k, B_v, q, nullptr, nullptr, 0, out, idx_out, score_out, workspace,
                          workspace_bytes, hip_stream);
}

xkv_status xkv_sr_decode_tail(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                              const void *B_k, const void *B_v, const void *q, const void *K_tail,
                              const void *V_tail, int32_t T, void *out, int32_t *idx_out, float *score_out,
                              void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (T < 0 || (T > 0 && (!K_tail || !V_tail))) return XKV_ERR_INVALID_ARG;
    return sr_decode_impl(shape, layer, A_k, A_v, B_k, B_v, q, K_tail, V_tail, T, out, idx_out, score_out, workspace,
                          workspace_bytes, hip_stream);
}


xkv_status xkv_dense_decode(const xkv_shape *shape, const void *K, const void *V, const void *q, void *out,
                            void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Plan p;
    xkv_status st = prepare(shape, workspace, workspace_bytes, p);
    if (st != XKV_OK) return st;
    if (!K || !V || !q || !out) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *part_o = at<float>(workspace, p.off_part_o);
    float *part_ml = at<float>(workspace, p.off_part_ml);
    hipError_t e = launch_dense(*shape, p, K, V, q, part_o, part_ml, stream);
    // same test as launch_dense: the matrix-core kernel writes one partial per split, the general one one per wavefront
    const bool mfma = p.dense_mfma && ((((uintptr_t)K | (uintptr_t)V | (uintptr_t)q)) & 15u) == 0;
    if (e == hipSuccess) e = launch_combine(*shape, mfma ? p.dense_splits : p.dense_splits * 4, part_o, part_ml, out, stream);
    return hip_status(e);
}

xkv_status xkv_reconstruct(const xkv_shape *shape, int32_t layer, const void *A, const void *B, int32_t r,
                           void *X_out, void *hip_stream)
{
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    if (!A || !B || !X_out || r < 1 || layer < 0 || layer >= shape->G) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    return hip_status(launch_reconstruct(*shape, layer, A, B, r, X_out, (hipStream_t)hip_stream));
}

xkv_status xkv_factorize_workspace_bytes(const xkv_shape *shape, int32_t r, size_t *bytes)
{
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    if (!bytes || r < 1) return XKV_ERR_INVALID_ARG;
    if (!factorize_shape_ok(*shape, r)) return XKV_ERR_UNSUPPORTED;
    *bytes = factorize_workspace_bytes(*shape, r);
    return XKV_OK;
}

xkv_status xkv_factorize(const xkv_shape *shape, const void *X, int32_t r, int32_t iters, uint32_t seed, void *A_out,
                         void *B_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    if (!X || !A_out || !B_out || r < 1 || iters < 1) return XKV_ERR_INVALID_ARG;
    if (!factorize_shape_ok(*shape, r)) return XKV_ERR_UNSUPPORTED;
    if (shape->batch == 0) return XKV_OK;
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < factorize_workspace_bytes(*shape, r))
        return XKV_ERR_WORKSPACE;
    if ((((uintptr_t)X | (uintptr_t)A_out | (uintptr_t)B_out) & 15u) != 0) return XKV_ERR_INVALID_ARG;
    return hip_status(launch_factorize(*shape, X, r, iters, seed, A_out, B_out, workspace, (hipStream_t)hip_stream));
}

xkv_status xkv_profile_kernel(int32_t stage, void *start_event, void *stop_event)
{
    if (stage < 0 || stage > 3) return XKV_ERR_INVALID_ARG;
    g_profile[stage].start = (start_event && stop_event) ? (hipEvent_t)start_event : nullptr;
    g_profile[stage].stop = (start_event && stop_event) ? (hipEvent_t)stop_event : nullptr;
    return XKV_OK;
}

const char *xkv_status_string(xkv_status status)
{
    switch (status) {
    case XKV_OK: return "XKV_OK";
    case XKV_ERR_INVALID_ARG: return "XKV_ERR_INVALID_ARG";
    case XKV_ERR_UNSUPPORTED: return "XKV_ERR_UNSUPPORTED";
    case XKV_ERR_WORKSPACE: return "XKV_ERR_WORKSPACE";
    case XKV_ERR_HIP: return "XKV_ERR_HIP";
    default: return "XKV_ERR_UNKNOWN";
    }
}

int32_t xkv_version(void) { return 100; }

}  // extern "C"
