// C ABI of libxkv: argument validation, workspace carving and launch sequencing.
// Every step of the path runs in the HIP kernels of this library; nothing here computes.
#include <cmath>
#include <cstring>
#include <mutex>

#include "xkv_common.h"

namespace xkv {

thread_local ProfileEvents g_profile[5] = {};

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
    hipError_t e = launch_gather_attend(*shape, p, layer, A_k, A_v, B_k, B_v, q, idx, pack_ws, nullptr, false, part_o, part_ml,
                                        stream);
    // the matrix-core kernel writes one partial per split, the general one one per wavefront
    if (e == hipSuccess) e = launch_combine(*shape, mfma ? p.sr_splits : p.sr_splits * 4, part_o, part_ml, out, stream);
    return hip_status(e);
}

// SR step; K_tail / V_tail (T > 0 tokens per KV head, uncompressed) are attended together with the selected rows.
// Dense pass over the T uncompressed tail tokens (at most 8 splits) into their own set of partials; *n_part is how
// many partials per query head it wrote.
static hipError_t launch_tail(const xkv_shape &shape, const Plan &p, const void *K_tail, const void *V_tail, const void *q,
                              int T, float *tail_o, float *tail_ml, int *n_part, hipStream_t stream)
{
    xkv_shape ts = shape;
    ts.L = T;
    Plan tp = p;
    const int splits = clampi(ceil_div(T, 512), 1, kTailParts / 4);
    tp.dense_chunk = ceil_div(ceil_div(T, splits), 128) * 128;
    tp.dense_splits = ceil_div(T, tp.dense_chunk);
    const hipError_t e = launch_dense(ts, tp, K_tail, V_tail, q, tail_o, tail_ml, stream);
    *n_part = dense_uses_mfma(tp, K_tail, V_tail, q) ? tp.dense_splits : tp.dense_splits * 4;
    return e;
}

// B_packed (nullable): the group's B_l in fragment order from xkv_pack_b; B_v may then be NULL.
static xkv_status sr_decode_impl(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                                 const void *B_k, const void *B_v, const void *q, const void *K_tail,
                                 const void *V_tail, int32_t T, void *out, int32_t *idx_out, float *score_out,
                                 void *workspace, size_t workspace_bytes, void *hip_stream,
                                 const void *B_packed = nullptr)
{
    Plan p;
    xkv_status st = prepare(shape, workspace, workspace_bytes, p);
    if (st != XKV_OK) return st;
    if (!A_k || !A_v || !B_k || (!B_v && !B_packed) || !q || !out || layer < 0 || layer >= shape->G)
        return XKV_ERR_INVALID_ARG;
    if (B_packed && (!p.ga_mfma || ((((uintptr_t)A_k | (uintptr_t)A_v | (uintptr_t)B_k | (uintptr_t)B_packed)) & 15u)))
        return XKV_ERR_UNSUPPORTED;  // the packed form belongs to the matrix-core kernel
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *S = score_out ? score_out : at<float>(workspace, p.off_score);
    int32_t *idx = idx_out ? idx_out : at<int32_t>(workspace, p.off_idx);
    float *part_o = at<float>(workspace, p.off_part_o);
    float *part_ml = at<float>(workspace, p.off_part_ml);
    uint32_t *hist = at<uint32_t>(workspace, p.off_hist), *state = at<uint32_t>(workspace, p.off_state);
    bool level0_done = false;
    hipError_t e = hipSuccess;
    // B is packed for the matrix-core gather-attend kernel in the same launch as the query projection
    void *pack_ws = at<void>(workspace, p.off_bpack);
    PackArgs pa{};
    const bool want_pack = gather_attend_uses_mfma(p, A_k, A_v, B_k, B_packed ? B_k : B_v, pack_ws);
    if (want_pack) pa = gather_attend_pack_args(*shape, layer, B_k, B_v, q, pack_ws, B_packed == nullptr);
    bool packed = false;
    if (e == hipSuccess)
        e = launch_score_stage(*shape, p, layer, A_k, B_k, q, at<void>(workspace, p.off_p), S,
                               p.score_hist ? topk_row_hist(p, state) : nullptr,
                               p.score_hist ? hist : nullptr, &level0_done, want_pack ? &pa : nullptr, &packed, stream);
    if (e == hipSuccess) e = launch_topk(*shape, p, S, idx, hist, state, level0_done, stream);
    if (e == hipSuccess)
        e = launch_gather_attend(*shape, p, layer, A_k, A_v, B_k, B_packed ? B_k : B_v, q, idx, pack_ws, B_packed, packed,
                                 part_o, part_ml, stream);
    // The uncompressed tail goes through the dense kernel as a context of T tokens of its own (at most 8 splits),
    // into a second set of partials; the merge below is one softmax over selected rows and tail.
    int n_tail = 0;
    float *tail_o = at<float>(workspace, p.off_tail_o), *tail_ml = at<float>(workspace, p.off_tail_ml);
    if (T > 0 && e == hipSuccess) e = launch_tail(*shape, p, K_tail, V_tail, q, T, tail_o, tail_ml, &n_tail, stream);
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

xkv_status xkv_packed_b_bytes(const xkv_shape *shape, size_t *bytes)
{
    if (!bytes) return XKV_ERR_INVALID_ARG;
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    if (!gather_attend_mfma_shape_ok(*shape)) return XKV_ERR_UNSUPPORTED;
    *bytes = gather_attend_group_pack_bytes(*shape);
    return XKV_OK;
}

xkv_status xkv_pack_b(const xkv_shape *shape, const void *B_k, const void *B_v, void *packed_out, void *hip_stream)
{
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    if (!gather_attend_mfma_shape_ok(*shape)) return XKV_ERR_UNSUPPORTED;
    if (!B_k || !B_v || !packed_out) return XKV_ERR_INVALID_ARG;
    if ((((uintptr_t)B_k | (uintptr_t)B_v | (uintptr_t)packed_out)) & 15u) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    return hip_status(launch_pack_group(*shape, B_k, B_v, packed_out, (hipStream_t)hip_stream));
}

xkv_status xkv_sr_decode_packed(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v, const void *B_k,
                                const void *B_packed, const void *q, void *out, int32_t *idx_out, float *score_out,
                                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!B_packed) return XKV_ERR_INVALID_ARG;
    return sr_decode_impl(shape, layer, A_k, A_v, B_k, nullptr, q, nullptr, nullptr, 0, out, idx_out, score_out, workspace,
                          workspace_bytes, hip_stream, B_packed);
}

}  // extern "C"

// Scratch of xkv_sr_decode_static: one array per GPU, part of the loaded code object, never allocated or freed.
// Host code must not use the array's name as an address (on the host it is only a handle for the symbol lookup);
// static_scratch() resolves it once per device to that device's copy.
static __device__ __align__(256) unsigned char scratch[XKV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

xkv_status static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return XKV_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return XKV_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return XKV_OK;
}
}  // namespace

extern "C" {

xkv_status xkv_sr_decode_static(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v, const void *B_k,
                                const void *B_v, const void *q, void *out, int32_t *idx_out, float *score_out,
                                void *hip_stream)
{
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    Plan p;
    make_plan(*shape, p);
    if (p.total > (size_t)XKV_STATIC_SCRATCH_BYTES) return XKV_ERR_WORKSPACE;  // shape too large for the built-in scratch
    // (argument errors are reported before the device is touched, as in the other calls)
    if (!A_k || !A_v || !B_k || !B_v || !q || !out || layer < 0 || layer >= shape->G) return XKV_ERR_INVALID_ARG;
    void *ws = nullptr;
    if ((st = static_scratch(&ws)) != XKV_OK) return st;
    // Every array the step keeps in the scratch is written by the step's own kernels before it is read (the row
    // histograms of the long-row selection are cleared by the launch that precedes the score kernel), so the
    // contents a previous call left behind need no clearing here.
    return sr_decode_impl(shape, layer, A_k, A_v, B_k, B_v, q, nullptr, nullptr, 0, out, idx_out, score_out, ws,
                          XKV_STATIC_SCRATCH_BYTES, hip_stream);
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

// xkv_sr_decode_tail on B_l re-ordered once per prompt: what a serving loop calls once tokens have been generated.
xkv_status xkv_sr_decode_tail_packed(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                                     const void *B_k, const void *B_packed, const void *q, const void *K_tail,
                                     const void *V_tail, int32_t T, void *out, int32_t *idx_out, float *score_out,
                                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!B_packed) return XKV_ERR_INVALID_ARG;
    if (T < 0 || (T > 0 && (!K_tail || !V_tail))) return XKV_ERR_INVALID_ARG;
    return sr_decode_impl(shape, layer, A_k, A_v, B_k, nullptr, q, K_tail, V_tail, T, out, idx_out, score_out, workspace,
                          workspace_bytes, hip_stream, B_packed);
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

xkv_status xkv_factorize_svd(const xkv_shape *shape, const void *X, int32_t r, int32_t r_out, int32_t iters, uint32_t seed,
                             void *A_out, void *B_out, float *sigma_out, void *workspace, size_t workspace_bytes,
                             void *hip_stream)
{
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    if (!X || !A_out || !B_out || r < 1 || iters < 1 || r_out < 1 || r_out > r) return XKV_ERR_INVALID_ARG;
    if (!factorize_shape_ok(*shape, r)) return XKV_ERR_UNSUPPORTED;
    if (shape->batch == 0) return XKV_OK;
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < factorize_workspace_bytes(*shape, r))
        return XKV_ERR_WORKSPACE;
    if ((((uintptr_t)X | (uintptr_t)A_out | (uintptr_t)B_out) & 15u) != 0) return XKV_ERR_INVALID_ARG;
    return hip_status(launch_factorize(*shape, X, r, r_out, iters, seed, A_out, B_out, sigma_out, workspace,
                                       (hipStream_t)hip_stream));
}

xkv_status xkv_factorize(const xkv_shape *shape, const void *X, int32_t r, int32_t iters, uint32_t seed, void *A_out,
                         void *B_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return xkv_factorize_svd(shape, X, r, r, iters, seed, A_out, B_out, nullptr, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"

namespace {

// Shapes and workspace layout of the landmark-guided step: the reshaped scoring problem (one "sequence" per
// (sequence, KV head), landmarks in the place of A^K, identity in the place of B^K), the gather-attend problem with
// the row capacity as k, and where each lives in the workspace.
struct LandmarkPlan {
    int n_c, k_ch, k_cap;
    xkv_shape score_shape, attend_shape, outlier_shape;
    Plan score_plan, attend_plan, outlier_plan;
    size_t off_score_ws, off_identity, off_counts, total_decode, total_prefill;
};

xkv_status make_landmark_plan(const xkv_shape &s, int c, int o, LandmarkPlan &lp)
{
    if (c < 1 || o < 0) return XKV_ERR_INVALID_ARG;
    lp.n_c = ceil_div(s.L, c);
    if (o > lp.n_c) return XKV_ERR_INVALID_ARG;
    lp.k_ch = ceil_div(s.k, c) < lp.n_c ? ceil_div(s.k, c) : lp.n_c;
    if ((long long)(lp.k_ch + o) * c > (1LL << 30)) return XKV_ERR_UNSUPPORTED;
    lp.k_cap = (lp.k_ch + o) * c;
    lp.score_shape = s;
    lp.score_shape.G = 1;
    lp.score_shape.H_kv = 1;
    lp.score_shape.H_q = s.H_q / s.H_kv;
    lp.score_shape.r_k = lp.score_shape.r_v = s.d_h;
    lp.score_shape.L = lp.n_c;
    lp.score_shape.k = lp.k_ch;
    lp.score_shape.batch = s.batch * s.H_kv;
    if ((long long)lp.score_shape.batch > 65535LL) return XKV_ERR_UNSUPPORTED;
    make_plan(lp.score_shape, lp.score_plan);
    lp.attend_shape = s;
    lp.attend_shape.k = lp.k_cap;
    make_plan(lp.attend_shape, lp.attend_plan);
    lp.outlier_shape = s;
    lp.outlier_shape.L = lp.n_c;
    lp.outlier_shape.k = o > 0 ? o : 1;
    make_plan(lp.outlier_shape, lp.outlier_plan);
    const size_t esz = s.dtype == XKV_F32 ? 4 : 2, rows = (size_t)(s.batch > 0 ? s.batch : 1) * s.H_kv;
    lp.off_score_ws = align_up(lp.attend_plan.total, 256);
    lp.off_identity = align_up(lp.off_score_ws + lp.score_plan.total, 256);
    lp.off_counts = align_up(lp.off_identity + rows * s.d_h * s.d_h * esz, 256);
    lp.total_decode = align_up(lp.off_counts + rows * sizeof(int32_t), 256);
    lp.total_prefill = align_up(lp.outlier_plan.total + rows * (size_t)lp.n_c * sizeof(float), 256);
    return XKV_OK;
}

}  // namespace

extern "C" {

xkv_status xkv_landmark_workspace_bytes(const xkv_shape *shape, int32_t c, int32_t o, size_t *bytes)
{
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    if (!bytes) return XKV_ERR_INVALID_ARG;
    LandmarkPlan lp;
    if ((st = make_landmark_plan(*shape, c, o, lp)) != XKV_OK) return st;
    *bytes = lp.total_decode > lp.total_prefill ? lp.total_decode : lp.total_prefill;
    return XKV_OK;
}

xkv_status xkv_landmarks(const xkv_shape *shape, const void *K_rope, int32_t c, int32_t o, void *landmarks_out,
                         float *neg_min_cos_out, int32_t *outliers_out, void *workspace, size_t workspace_bytes,
                         void *hip_stream)
{
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    LandmarkPlan lp;
    if ((st = make_landmark_plan(*shape, c, o, lp)) != XKV_OK) return st;
    if (!K_rope || !landmarks_out || (o > 0 && !outliers_out)) return XKV_ERR_INVALID_ARG;
    if (o > 0 && (!workspace || ((uintptr_t)workspace & 255u))) return XKV_ERR_INVALID_ARG;
    if (o > 0 && workspace_bytes < lp.total_prefill) return XKV_ERR_WORKSPACE;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *neg_m = neg_min_cos_out;
    if (!neg_m && o > 0) neg_m = at<float>(workspace, align_up(lp.outlier_plan.total, 256));
    hipError_t e = launch_landmarks(*shape, K_rope, c, landmarks_out, neg_m, stream);
    if (e == hipSuccess && o > 0)
        e = launch_topk(lp.outlier_shape, lp.outlier_plan, neg_m, outliers_out, at<uint32_t>(workspace, lp.outlier_plan.off_hist),
                        at<uint32_t>(workspace, lp.outlier_plan.off_state), false, stream);
    return hip_status(e);
}

// qbits: 0 = A_k, A_v in shape->dtype; 4 or 3 = rows of 4-bit / 3-bit codes
// B_packed (nullable): the group's B_l in fragment order from xkv_pack_b; B_v may then be NULL.
static xkv_status sr_decode_landmark_impl(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                                          int qbits, const void *B_k, const void *B_v, const void *B_packed, const void *q,
                                          const void *landmarks, const int32_t *outliers, int32_t c, int32_t o,
                                          float rope_theta, const void *K_tail, const void *V_tail, int32_t T, void *out,
                                          int32_t *rows_out, int32_t *count_out, float *score_out, void *workspace,
                                          size_t workspace_bytes, void *hip_stream)
{
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    LandmarkPlan lp;
    if ((st = make_landmark_plan(*shape, c, o, lp)) != XKV_OK) return st;
    if (!A_k || !A_v || !B_k || (!B_v && !B_packed) || !q || !landmarks || !out || (o > 0 && !outliers) || layer < 0 ||
        layer >= shape->G)
        return XKV_ERR_INVALID_ARG;
    if (B_packed) B_v = B_k;  // never read: the gather-reconstruct kernel takes both products' B from the packed copy
    if (!(rope_theta >= 0.0f) || !std::isfinite(rope_theta)) return XKV_ERR_INVALID_ARG;
    if (T < 0 || (T > 0 && (!K_tail || !V_tail))) return XKV_ERR_INVALID_ARG;
    if (rope_theta > 0.0f && !rope_shape_ok(*shape)) return XKV_ERR_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255u)) return XKV_ERR_INVALID_ARG;
    if (workspace_bytes < lp.total_decode) return XKV_ERR_WORKSPACE;
    if (qbits != 0 && !gather_attend_quant_ok(lp.attend_shape, lp.attend_plan, A_k, A_v, B_k, B_v,
                                              at<void>(workspace, lp.attend_plan.off_bpack), qbits))
        return XKV_ERR_UNSUPPORTED;
    if (B_packed && (((uintptr_t)B_packed & 15u) ||
                     !gather_attend_uses_mfma(lp.attend_plan, A_k, A_v, B_k, B_v,
                                              at<void>(workspace, lp.attend_plan.off_bpack))))
        return XKV_ERR_UNSUPPORTED;  // only the matrix-core kernel reads the packed layout
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    const Plan &ps = lp.score_plan, &pa = lp.attend_plan;
    void *ws_s = at<void>(workspace, lp.off_score_ws);
    void *ident = at<void>(workspace, lp.off_identity);
    // Alg. 2, scores and pooling: the factor-scoring kernels on (landmarks, identity, queries of one KV head)
    float *S = score_out ? score_out : at<float>(ws_s, ps.off_score);
    int32_t *chunks = at<int32_t>(ws_s, ps.off_idx);
    uint32_t *hist = at<uint32_t>(ws_s, ps.off_hist), *state = at<uint32_t>(ws_s, ps.off_state);
    bool level0_done = false;
    // The identity in the place of B^K is written out only for the general score kernels; the matrix-core projection
    // generates it.  That launch also carries the operand packing of the gather-reconstruct kernel below (the Q
    // fragments, and B_l unless the caller brought the packed copy), as in xkv_sr_decode.
    void *pack_ws = at<void>(workspace, pa.off_bpack);
    const bool mfma = gather_attend_uses_mfma(pa, A_k, A_v, B_k, B_v, pack_ws);
    const bool gen_ident = score_stage_uses_mfma(lp.score_shape, landmarks, nullptr, q, at<void>(ws_s, ps.off_p), nullptr);
    PackArgs pk{};
    if (mfma) pk = gather_attend_pack_args(lp.attend_shape, layer, B_k, B_v, q, pack_ws, B_packed == nullptr);
    const bool fuse = gen_ident && mfma;
    bool packed = false;
    hipError_t e = gen_ident ? hipSuccess : launch_identity(*shape, ident, lp.score_shape.batch, stream);
    if (e == hipSuccess)
        e = launch_score_stage(lp.score_shape, ps, 0, landmarks, gen_ident ? nullptr : ident, q, at<void>(ws_s, ps.off_p), S,
                               ps.score_hist ? topk_row_hist(ps, state) : nullptr,
                               ps.score_hist ? hist : nullptr, &level0_done, fuse ? &pk : nullptr, &packed, stream);
    // top ceil(k / c) chunks per KV head, union with the outliers, expansion to rows
    if (e == hipSuccess) e = launch_topk(lp.score_shape, ps, S, chunks, hist, state, level0_done, stream);
    int32_t *rows = rows_out ? rows_out : at<int32_t>(workspace, pa.off_idx);
    int32_t *counts = count_out ? count_out : at<int32_t>(workspace, lp.off_counts);
    if (e == hipSuccess) e = launch_expand_chunks(*shape, chunks, lp.k_ch, outliers, o, c, rows, counts, stream);
    // Eq. 3 and attention over the rows that are real
    float *part_o = at<float>(workspace, pa.off_part_o), *part_ml = at<float>(workspace, pa.off_part_ml);
    if (e == hipSuccess)
        e = launch_gather_attend(lp.attend_shape, pa, layer, A_k, A_v, B_k, B_v, q, rows, pack_ws, B_packed, packed, part_o,
                                 part_ml, stream, counts, rope_theta, qbits);
    // the uncompressed tail, as in xkv_sr_decode_tail: a dense pass over its T tokens into a second set of partials
    int n_tail = 0;
    float *tail_o = at<float>(workspace, pa.off_tail_o), *tail_ml = at<float>(workspace, pa.off_tail_ml);
    if (T > 0 && e == hipSuccess) e = launch_tail(*shape, pa, K_tail, V_tail, q, T, tail_o, tail_ml, &n_tail, stream);
    if (e == hipSuccess)
        e = launch_combine(*shape, mfma ? pa.sr_splits : pa.sr_splits * 4, part_o, part_ml, out, stream, n_tail, tail_o,
                           tail_ml);
    return hip_status(e);
}

xkv_status xkv_sr_decode_landmark(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                                  const void *B_k, const void *B_v, const void *q, const void *landmarks,
                                  const int32_t *outliers, int32_t c, int32_t o, float rope_theta, const void *K_tail,
                                  const void *V_tail, int32_t T, void *out, int32_t *rows_out, int32_t *count_out,
                                  float *score_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return sr_decode_landmark_impl(shape, layer, A_k, A_v, 0, B_k, B_v, nullptr, q, landmarks, outliers, c, o, rope_theta,
                                   K_tail, V_tail, T, out, rows_out, count_out, score_out, workspace, workspace_bytes,
                                   hip_stream);
}

xkv_status xkv_sr_decode_landmark_q(const xkv_shape *shape, int32_t layer, const void *Aq_k, const void *Aq_v,
                                    int32_t bits, const void *B_k, const void *B_v, const void *q, const void *landmarks,
                                    const int32_t *outliers, int32_t c, int32_t o, float rope_theta, const void *K_tail,
                                    const void *V_tail, int32_t T, void *out, int32_t *rows_out, int32_t *count_out,
                                    float *score_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (bits != 4 && bits != 3) return XKV_ERR_UNSUPPORTED;
    return sr_decode_landmark_impl(shape, layer, Aq_k, Aq_v, bits, B_k, B_v, nullptr, q, landmarks, outliers, c, o,
                                   rope_theta, K_tail, V_tail, T, out, rows_out, count_out, score_out, workspace,
                                   workspace_bytes, hip_stream);
}

// The landmark-guided step on B_l re-ordered once per prompt (xkv_pack_b); bits 0 = rows of A in shape->dtype, 4 or 3 =
// quantised rows.
xkv_status xkv_sr_decode_landmark_packed(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                                         int32_t bits, const void *B_k, const void *B_packed, const void *q,
                                         const void *landmarks, const int32_t *outliers, int32_t c, int32_t o,
                                         float rope_theta, const void *K_tail, const void *V_tail, int32_t T, void *out,
                                         int32_t *rows_out, int32_t *count_out, float *score_out, void *workspace,
                                         size_t workspace_bytes, void *hip_stream)
{
    if (bits != 0 && bits != 4 && bits != 3) return XKV_ERR_UNSUPPORTED;
    if (!B_packed) return XKV_ERR_INVALID_ARG;
    return sr_decode_landmark_impl(shape, layer, A_k, A_v, bits, B_k, nullptr, B_packed, q, landmarks, outliers, c, o,
                                   rope_theta, K_tail, V_tail, T, out, rows_out, count_out, score_out, workspace,
                                   workspace_bytes, hip_stream);
}

}  // extern "C"

extern "C" {

// Stages 3-4 from rows of A^K, A^V given as 4-bit or 3-bit codes.
xkv_status xkv_gather_attend_q(const xkv_shape *shape, int32_t layer, const void *Aq_k, const void *Aq_v, int32_t bits,
                               const void *B_k, const void *B_v, const void *q, const int32_t *idx,
                               const int32_t *counts, float rope_theta, void *out, void *workspace,
                               size_t workspace_bytes, void *hip_stream)
{
    Plan p;
    xkv_status st = prepare(shape, workspace, workspace_bytes, p);
    if (st != XKV_OK) return st;
    if (!Aq_k || !Aq_v || !B_k || !B_v || !q || !idx || !out || layer < 0 || layer >= shape->G)
        return XKV_ERR_INVALID_ARG;
    if (!(rope_theta >= 0.0f) || !std::isfinite(rope_theta)) return XKV_ERR_INVALID_ARG;
    if (rope_theta > 0.0f && !rope_shape_ok(*shape)) return XKV_ERR_UNSUPPORTED;
    void *pack_ws = at<void>(workspace, p.off_bpack);
    if (!gather_attend_quant_ok(*shape, p, Aq_k, Aq_v, B_k, B_v, pack_ws, bits)) return XKV_ERR_UNSUPPORTED;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *part_o = at<float>(workspace, p.off_part_o), *part_ml = at<float>(workspace, p.off_part_ml);
    hipError_t e = launch_gather_attend(*shape, p, layer, Aq_k, Aq_v, B_k, B_v, q, idx, pack_ws, nullptr, false, part_o,
                                        part_ml, stream, counts, rope_theta, bits);
    if (e == hipSuccess) e = launch_combine(*shape, p.sr_splits, part_o, part_ml, out, stream);
    return hip_status(e);
}

xkv_status xkv_gather_attend_ex(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                                const void *B_k, const void *B_v, const void *q, const int32_t *idx,
                                const int32_t *counts, float rope_theta, void *out, void *workspace,
                                size_t workspace_bytes, void *hip_stream)
{
    Plan p;
    xkv_status st = prepare(shape, workspace, workspace_bytes, p);
    if (st != XKV_OK) return st;
    if (!A_k || !A_v || !B_k || !B_v || !q || !idx || !out || layer < 0 || layer >= shape->G)
        return XKV_ERR_INVALID_ARG;
    if (!(rope_theta >= 0.0f) || !std::isfinite(rope_theta)) return XKV_ERR_INVALID_ARG;
    if (rope_theta > 0.0f && !rope_shape_ok(*shape)) return XKV_ERR_UNSUPPORTED;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *part_o = at<float>(workspace, p.off_part_o);
    float *part_ml = at<float>(workspace, p.off_part_ml);
    void *pack_ws = at<void>(workspace, p.off_bpack);
    const bool mfma = gather_attend_uses_mfma(p, A_k, A_v, B_k, B_v, pack_ws);
    hipError_t e = launch_gather_attend(*shape, p, layer, A_k, A_v, B_k, B_v, q, idx, pack_ws, nullptr, false, part_o, part_ml,
                                        stream, counts, rope_theta);
    if (e == hipSuccess) e = launch_combine(*shape, mfma ? p.sr_splits : p.sr_splits * 4, part_o, part_ml, out, stream);
    return hip_status(e);
}

// Workspace of the absorbed calls: the ordinary plan's, then per-head scores and the partial row sums.
static xkv_status prepare_absorbed(const xkv_shape *s, void *ws, size_t ws_bytes, Plan &p, AbsorbPlan &a)
{
    xkv_status st = validate(s);
    if (st != XKV_OK) return st;
    if (!absorb_shape_ok(*s)) return XKV_ERR_UNSUPPORTED;
    make_plan(*s, p);
    a = make_absorb_plan(*s, p.total);
    if (!ws) return XKV_ERR_INVALID_ARG;
    if (ws_bytes < a.total) return XKV_ERR_WORKSPACE;
    if (((uintptr_t)ws) & 255u) return XKV_ERR_INVALID_ARG;
    return XKV_OK;
}

xkv_status xkv_absorbed_workspace_bytes(const xkv_shape *shape, size_t *bytes)
{
    if (!bytes) return XKV_ERR_INVALID_ARG;
    xkv_status st = validate(shape);
    if (st != XKV_OK) return st;
    if (!absorb_shape_ok(*shape)) return XKV_ERR_UNSUPPORTED;
    Plan p;
    make_plan(*shape, p);
    *bytes = make_absorb_plan(*shape, p.total).total;
    return XKV_OK;
}

xkv_status xkv_head_scores(const xkv_shape *shape, int32_t layer, const void *A_k, const void *B_k, const void *q,
                           float *score_out, float *heads_out, void *workspace, size_t workspace_bytes,
                           void *hip_stream)
{
    Plan p;
    AbsorbPlan a;
    xkv_status st = prepare_absorbed(shape, workspace, workspace_bytes, p, a);
    if (st != XKV_OK) return st;
    if (!A_k || !B_k || !q || !heads_out || layer < 0 || layer >= shape->G) return XKV_ERR_INVALID_ARG;
    if (((uintptr_t)heads_out) & 15u) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    float *S = score_out ? score_out : at<float>(workspace, p.off_score);
    return hip_status(launch_score_stage(*shape, p, layer, A_k, B_k, q, at<void>(workspace, p.off_p), S, nullptr, nullptr,
                                         nullptr, nullptr, nullptr, (hipStream_t)hip_stream, heads_out));
}

xkv_status xkv_attend_absorbed(const xkv_shape *shape, int32_t layer, const void *A_v, const void *B_v,
                               const float *head_scores, const int32_t *idx, void *out, void *workspace,
                               size_t workspace_bytes, void *hip_stream);

static xkv_status attend_absorbed_impl(const xkv_shape *shape, int32_t layer, const void *A_v, const void *B_v,
                                       const float *head_scores, const int32_t *idx, void *out, void *workspace,
                                       size_t workspace_bytes, void *hip_stream, bool q4)
{
    Plan p;
    AbsorbPlan a;
    xkv_status st = prepare_absorbed(shape, workspace, workspace_bytes, p, a);
    if (st != XKV_OK) return st;
    if (q4 && (shape->dtype != XKV_BF16 || !quant_rank_ok(shape->r_v))) return XKV_ERR_UNSUPPORTED;
    if (!A_v || !B_v || !head_scores || !idx || !out || layer < 0 || layer >= shape->G) return XKV_ERR_INVALID_ARG;
    if ((((uintptr_t)A_v) | ((uintptr_t)head_scores)) & 15u) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *po = at<float>(workspace, a.off_po), *pml = at<float>(workspace, a.off_pml);
    hipError_t e = launch_absorbed(*shape, a, layer, A_v, B_v, head_scores, idx, po, pml,
                                   at<float>(workspace, a.off_part_u), at<float>(workspace, a.off_part_ml), stream, q4);
    if (e == hipSuccess) e = launch_combine(*shape, a.slices, po, pml, out, stream);
    return hip_status(e);
}

xkv_status xkv_attend_absorbed(const xkv_shape *shape, int32_t layer, const void *A_v, const void *B_v,
                               const float *head_scores, const int32_t *idx, void *out, void *workspace,
                               size_t workspace_bytes, void *hip_stream)
{
    return attend_absorbed_impl(shape, layer, A_v, B_v, head_scores, idx, out, workspace, workspace_bytes, hip_stream,
                                false);
}

xkv_status xkv_quantized_row_bytes(int32_t r, int32_t bits, size_t *bytes)
{
    if (!bytes || r < 1) return XKV_ERR_INVALID_ARG;
    if ((bits != 4 && bits != 3) || !quant_rank_ok(r)) return XKV_ERR_UNSUPPORTED;
    *bytes = quant_row_bytes(r, bits);
    return XKV_OK;
}

xkv_status xkv_quantize_rows(const void *X, int64_t rows, int32_t r, int32_t bits, void *out, void *hip_stream)
{
    if (rows < 0 || r < 1) return XKV_ERR_INVALID_ARG;
    if ((bits != 4 && bits != 3) || !quant_rank_ok(r)) return XKV_ERR_UNSUPPORTED;
    if (rows == 0) return XKV_OK;
    if (!X || !out || ((((uintptr_t)X) | ((uintptr_t)out)) & 15u)) return XKV_ERR_INVALID_ARG;
    return hip_status(launch_quantize_rows(X, rows, r, bits, out, (hipStream_t)hip_stream));
}

xkv_status xkv_attend_absorbed_q4(const xkv_shape *shape, int32_t layer, const void *Aq_v, const void *B_v,
                                  const float *head_scores, const int32_t *idx, void *out, void *workspace,
                                  size_t workspace_bytes, void *hip_stream)
{
    return attend_absorbed_impl(shape, layer, Aq_v, B_v, head_scores, idx, out, workspace, workspace_bytes, hip_stream,
                                true);
}

static xkv_status sr_decode_absorbed_impl(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                                          const void *B_k, const void *B_v, const void *q, const void *K_tail,
                                          const void *V_tail, int32_t T, void *out, int32_t *idx_out, float *score_out,
                                          void *workspace, size_t workspace_bytes, void *hip_stream, bool q4)
{
    if (T < 0 || (T > 0 && (!K_tail || !V_tail))) return XKV_ERR_INVALID_ARG;
    Plan p;
    AbsorbPlan a;
    xkv_status st = prepare_absorbed(shape, workspace, workspace_bytes, p, a);
    if (st != XKV_OK) return st;
    if (q4 && (!score_q4_shape_ok(*shape) || !quant_rank_ok(shape->r_v))) return XKV_ERR_UNSUPPORTED;
    if (!A_k || !A_v || !B_k || !B_v || !q || !out || layer < 0 || layer >= shape->G) return XKV_ERR_INVALID_ARG;
    if (((uintptr_t)A_v) & 15u) return XKV_ERR_INVALID_ARG;
    if (q4 && ((((uintptr_t)A_k) | ((uintptr_t)B_k) | ((uintptr_t)q)) & 15u)) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *S = score_out ? score_out : at<float>(workspace, p.off_score);
    int32_t *idx = idx_out ? idx_out : at<int32_t>(workspace, p.off_idx);
    float *heads = at<float>(workspace, a.off_heads);
    uint32_t *hist = at<uint32_t>(workspace, p.off_hist), *state = at<uint32_t>(workspace, p.off_state);
    bool level0_done = false;
    hipError_t e =
        q4 ? launch_score_q4_stage(*shape, p, layer, A_k, B_k, q, at<void>(workspace, p.off_p), S, heads, stream)
           : launch_score_stage(*shape, p, layer, A_k, B_k, q, at<void>(workspace, p.off_p), S,
                                p.score_hist ? topk_row_hist(p, state) : nullptr,
                                p.score_hist ? hist : nullptr, &level0_done, nullptr, nullptr, stream, heads);
    if (e == hipSuccess) e = launch_topk(*shape, p, S, idx, hist, state, level0_done, stream);
    float *po = at<float>(workspace, a.off_po), *pml = at<float>(workspace, a.off_pml);
    if (e == hipSuccess)
        e = launch_absorbed(*shape, a, layer, A_v, B_v, heads, idx, po, pml, at<float>(workspace, a.off_part_u),
                            at<float>(workspace, a.off_part_ml), stream, q4);
    // the uncompressed tail, if any, joins the same softmax through its own set of partials (as in xkv_sr_decode_tail)
    int n_tail = 0;
    float *tail_o = at<float>(workspace, p.off_tail_o), *tail_ml = at<float>(workspace, p.off_tail_ml);
    if (T > 0 && e == hipSuccess) e = launch_tail(*shape, p, K_tail, V_tail, q, T, tail_o, tail_ml, &n_tail, stream);
    if (e == hipSuccess) e = launch_combine(*shape, a.slices, po, pml, out, stream, n_tail, tail_o, tail_ml);
    return hip_status(e);
}

xkv_status xkv_sr_decode_absorbed(const xkv_shape *shape, int32_t layer, const void *A_k, const void *A_v,
                                  const void *B_k, const void *B_v, const void *q, const void *K_tail,
                                  const void *V_tail, int32_t T, void *out, int32_t *idx_out, float *score_out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return sr_decode_absorbed_impl(shape, layer, A_k, A_v, B_k, B_v, q, K_tail, V_tail, T, out, idx_out, score_out,
                                   workspace, workspace_bytes, hip_stream, false);
}

xkv_status xkv_sr_decode_absorbed_q4(const xkv_shape *shape, int32_t layer, const void *Aq_k, const void *Aq_v,
                                     const void *B_k, const void *B_v, const void *q, const void *K_tail,
                                     const void *V_tail, int32_t T, void *out, int32_t *idx_out, float *score_out,
                                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return sr_decode_absorbed_impl(shape, layer, Aq_k, Aq_v, B_k, B_v, q, K_tail, V_tail, T, out, idx_out, score_out,
                                   workspace, workspace_bytes, hip_stream, true);
}

// The gather-reconstruct step on 4-bit rows: scores from the quantised A^K (which also leaves the per-head scores in
// the workspace, unused here), selection, then Eq. 3 and attention from the quantised rows.
xkv_status xkv_sr_decode_q4(const xkv_shape *shape, int32_t layer, const void *Aq_k, const void *Aq_v, const void *B_k,
                            const void *B_v, const void *q, float rope_theta, const void *K_tail, const void *V_tail,
                            int32_t T, void *out, int32_t *idx_out, float *score_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    if (T < 0 || (T > 0 && (!K_tail || !V_tail))) return XKV_ERR_INVALID_ARG;
    Plan p;
    AbsorbPlan a;
    xkv_status st = prepare_absorbed(shape, workspace, workspace_bytes, p, a);
    if (st != XKV_OK) return st;
    if (!Aq_k || !Aq_v || !B_k || !B_v || !q || !out || layer < 0 || layer >= shape->G) return XKV_ERR_INVALID_ARG;
    if (!(rope_theta >= 0.0f) || !std::isfinite(rope_theta)) return XKV_ERR_INVALID_ARG;
    if (rope_theta > 0.0f && !rope_shape_ok(*shape)) return XKV_ERR_UNSUPPORTED;
    void *pack_ws = at<void>(workspace, p.off_bpack);
    if (!score_q4_shape_ok(*shape) || !gather_attend_quant_ok(*shape, p, Aq_k, Aq_v, B_k, B_v, pack_ws, 4))
        return XKV_ERR_UNSUPPORTED;
    if (((uintptr_t)q) & 15u) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    float *S = score_out ? score_out : at<float>(workspace, p.off_score);
    int32_t *idx = idx_out ? idx_out : at<int32_t>(workspace, p.off_idx);
    uint32_t *hist = at<uint32_t>(workspace, p.off_hist), *state = at<uint32_t>(workspace, p.off_state);
    float *part_o = at<float>(workspace, p.off_part_o), *part_ml = at<float>(workspace, p.off_part_ml);
    hipError_t e = launch_score_q4_stage(*shape, p, layer, Aq_k, B_k, q, at<void>(workspace, p.off_p), S,
                                         at<float>(workspace, a.off_heads), stream);
    if (e == hipSuccess) e = launch_topk(*shape, p, S, idx, hist, state, false, stream);
    if (e == hipSuccess)
        e = launch_gather_attend(*shape, p, layer, Aq_k, Aq_v, B_k, B_v, q, idx, pack_ws, nullptr, false, part_o, part_ml,
                                 stream, nullptr, rope_theta, 4);
    int n_tail = 0;
    float *tail_o = at<float>(workspace, p.off_tail_o), *tail_ml = at<float>(workspace, p.off_tail_ml);
    if (T > 0 && e == hipSuccess) e = launch_tail(*shape, p, K_tail, V_tail, q, T, tail_o, tail_ml, &n_tail, stream);
    if (e == hipSuccess) e = launch_combine(*shape, p.sr_splits, part_o, part_ml, out, stream, n_tail, tail_o, tail_ml);
    return hip_status(e);
}

xkv_status xkv_head_scores_q4(const xkv_shape *shape, int32_t layer, const void *Aq_k, const void *B_k, const void *q,
                              float *score_out, float *heads_out, void *workspace, size_t workspace_bytes,
                              void *hip_stream)
{
    Plan p;
    AbsorbPlan a;
    xkv_status st = prepare_absorbed(shape, workspace, workspace_bytes, p, a);
    if (st != XKV_OK) return st;
    if (!score_q4_shape_ok(*shape)) return XKV_ERR_UNSUPPORTED;
    if (!Aq_k || !B_k || !q || !heads_out || layer < 0 || layer >= shape->G) return XKV_ERR_INVALID_ARG;
    if ((((uintptr_t)heads_out) | ((uintptr_t)Aq_k) | ((uintptr_t)B_k) | ((uintptr_t)q)) & 15u) return XKV_ERR_INVALID_ARG;
    if (shape->batch == 0) return XKV_OK;
    float *S = score_out ? score_out : at<float>(workspace, p.off_score);
    return hip_status(launch_score_q4_stage(*shape, p, layer, Aq_k, B_k, q, at<void>(workspace, p.off_p), S, heads_out,
                                            (hipStream_t)hip_stream));
}

xkv_status xkv_profile_kernel(int32_t stage, void *start_event, void *stop_event)
{
    if (stage < 0 || stage > 4) return XKV_ERR_INVALID_ARG;
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
