// Shared device helpers and the internal launch interface of libxkv (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "xkv.h"

namespace xkv {

constexpr int kWave = 64;  // CDNA wavefront width

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// round-to-nearest-even; inputs are finite by contract
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_to_f32(x); }

template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return f32_to_bf16(x); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

// monotone unsigned image of an fp32 bit pattern: a > b as floats (with -0 < +0) <=> key(a) > key(b)
__device__ __forceinline__ uint32_t order_key(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ---------------------------------------------------------------------------------------------
// Host-side plan: how a shape is split over workgroups and where each scratch array lives.
// ---------------------------------------------------------------------------------------------
struct Plan {
    int n_rep;         // query heads per KV head
    int rows;          // batch * H_kv independent top-k problems
    int topk_chunks;   // chunks each score row is split into
    int topk_chunk;    // elements per chunk (multiple of 256)
    int sr_splits;     // splits of the k selected tokens per (sequence, KV head)
    int sr_chunk;      // selected tokens per split
    int dense_splits;  // splits of the L tokens per (sequence, KV head)
    int dense_chunk;   // tokens per split
    int max_splits;
    float scale;
    // byte offsets into the workspace
    size_t off_p, off_score, off_idx, off_hist, off_state, off_part_o, off_part_ml, off_bpack, off_tail_o, off_tail_ml, total;
    bool dense_mfma;   // shape fits the matrix-core dense kernel
    bool ga_mfma;      // shape fits the matrix-core gather-attend kernel
    int ga_waves;      // ... with this many wavefronts (32 selected tokens each) per workgroup
    bool topk_row;     // rows short enough for the one-launch, register-resident selection
    bool score_stream; // shape fits the long-stream score kernel
    bool score_hist;   // ... and that kernel can also histogram the top digit of its scores for the top-k stage
    int score_tpw;     // 32-token tiles per workgroup of that kernel (topk_chunk = 32 * score_tpw when score_hist)
    int score_waves;   // wavefronts per workgroup of that kernel (8, or 4 at large ranks)
};

constexpr int kTailParts = 32;   // partials per query head for the uncompressed tail (8 splits x 4 wavefronts)
constexpr int kTopkLevels = 4;   // 8-bit digits of the 32-bit order key
constexpr int kTopkBins = 256;
constexpr int kStateWords = 8;   // per row: (prefix, k_rem) for each resolved level

xkv_status make_plan(const xkv_shape &s, Plan &p);

// Optional event pair recorded around the main kernel of a stage (0 score, 1 gather-attend, 2 dense,
// 3 Gram-matrix product of the factorization, 4 row sums of the absorbed attention).  Kept per host thread: the
// thread that asks for a measurement is the one whose calls are measured, and no other thread sees the pair.
struct ProfileEvents {
    hipEvent_t start, stop;
};
extern thread_local ProfileEvents g_profile[5];
inline void profile_begin(int stage, hipStream_t st)
{
    if (g_profile[stage].start && g_profile[stage].stop) (void)hipEventRecord(g_profile[stage].start, st);
}
inline void profile_end(int stage, hipStream_t st)
{
    if (g_profile[stage].start && g_profile[stage].stop) (void)hipEventRecord(g_profile[stage].stop, st);
}

// Arguments of the two small passes over B_l (see prepass.h): the query projection into hi/lo bf16 fragments
// and the packing of B_l and the query heads into matrix-core fragment order.
typedef __attribute__((ext_vector_type(4))) uint32_t pack_u32x4_t;
struct ProjArgs {
    const bf16_t *B_k, *q;
    bf16_t *Pfrag;
    int G, layer, r_k, H_kv, H_q, d_h, F8;
    int blocks_x;  // 256-thread blocks per sequence
};
struct PackArgs {
    const bf16_t *B_k, *B_v, *q;
    pack_u32x4_t *pack;    // packed B, [batch][dst_G][H_kv][(F8k + F8v) * 256] pieces of 16 B
    pack_u32x4_t *pack_q;  // Q^T fragments, [batch][H_kv][512] pieces
    int G, layer, r_k, r_v, H_kv, H_q, F8k, F8v, batch;
    int dst_G, dst_layer;  // the destination holds dst_G layers per sequence; this call fills dst_layer
    int blocks_per_head;   // 256-item blocks per (sequence, KV head) for the B items (0: B is already packed)
};
constexpr int kPackQBlocks = 2;  // 256-item blocks per (sequence, KV head) for the Q^T fragments

// Raises a kernel's dynamic-LDS limit the first time the kernel is launched on each device.  One static instance
// per kernel; safe for concurrent host threads (the attribute call is idempotent, the flag word is atomic).
struct DynamicLdsOnce {
    std::atomic<uint64_t> done{0};  // bit d: set on device d (devices 64 and up share bits: they repeat the call)
    hipError_t ensure(const void *kernel, size_t bytes)
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const uint64_t bit = 1ull << (dev & 63);
        if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
        return e;
    }
};

// Kernel launchers (each enqueues on `st`; shapes were validated by the caller).
// Top-k scratch (uint32 words).  `state` region: [rows][8] state words, then the row histograms
// [rows][4][256], then chunk_gt [rows][chunks]; `hist` region: [rows][chunks][4][256].
inline uint32_t *topk_row_hist(const Plan &p, uint32_t *state) { return state + (size_t)p.rows * kStateWords; }
bool score_stream_plan(const xkv_shape &s, int *tiles_per_wg, bool *hist_fits, int *waves);
// fuse_pack (nullable): also pack B for the gather-attend kernel in the projection launch (matrix-core path
// only; *packed_done tells whether it did).  If row_hist/chunk_hist are given and the long-stream kernel runs, the
// projection launch also clears the row histograms (all levels) and the score kernel adds the histogram of the top
// 8 key bits of every pooled score to them and stores the per-chunk histograms; *hist_done tells whether it did
// (if not, the row histograms were not touched).
hipError_t launch_score_stage(const xkv_shape &s, const Plan &p, int layer, const void *A_k, const void *B_k,
                              const void *q, void *P_ws, float *S, uint32_t *row_hist, uint32_t *chunk_hist,
                              bool *hist_done, const PackArgs *fuse_pack, bool *packed_done, hipStream_t st,
                              float *S_heads = nullptr);
// Whether that stage runs on the matrix-core kernels for these operands.  Only then may B_k be NULL, which stands for
// an identity B_l (landmark scoring): the projection generates its rows instead of reading them.
bool score_stage_uses_mfma(const xkv_shape &s, const void *A_k, const void *B_k, const void *q, const void *P_ws,
                           const float *S_heads);
// S_heads (nullable): also store every query head's score, [batch][H_kv][L][head_pitch(H_q / H_kv)] fp32 with the
// padding zero; S is then the maximum of exactly the stored values.
inline int head_pitch_of(int n_rep) { return n_rep <= 1 ? 1 : n_rep <= 2 ? 2 : n_rep <= 4 ? 4 : n_rep <= 8 ? 8 : 16; }
bool topk_row_shape_ok(const xkv_shape &s);
hipError_t launch_topk_init(const Plan &p, uint32_t *state, hipStream_t st);
// level0_done: launch_topk_init ran and the level-0 histograms were already accumulated by the score stage.
hipError_t launch_topk(const xkv_shape &s, const Plan &p, const float *S, int32_t *idx, uint32_t *hist,
                       uint32_t *state, bool level0_done, hipStream_t st);
// pack_ws: workspace for the operands in fragment order (Q^T fragments, then this layer's packed B).
// B_packed (nullable): the group's B already in fragment order (xkv_pack_b), then nothing of B is packed per call.
// packed: pack_ws already holds this call's fragments (written by the launch that projected the queries).
// counts (nullable): [batch][H_kv], how many of the s.k ids of each row are real; the rest is ignored.
hipError_t launch_gather_attend(const xkv_shape &s, const Plan &p, int layer, const void *A_k, const void *A_v,
                                const void *B_k, const void *B_v, const void *q, const int32_t *idx, void *pack_ws,
                                const void *B_packed, bool packed, float *part_o, float *part_ml, hipStream_t st,
                                const int32_t *counts = nullptr, float rope_theta = 0.0f, int qbits = 0);
// qbits 4 or 3: A_k and A_v are rows of 4-bit / 3-bit codes (quant.hip); matrix-core shapes with ranks that are
// multiples of 32 only (gather_attend_quant_ok).
bool gather_attend_quant_ok(const xkv_shape &s, const Plan &p, const void *Aq_k, const void *Aq_v, const void *B_k,
                            const void *B_v, const void *pack_ws, int qbits);
// rope_theta > 0: the reconstructed key rows are rotated to their positions (RoPE base theta) before the scores.
bool rope_shape_ok(const xkv_shape &s);
bool gather_attend_uses_mfma(const Plan &p, const void *A_k, const void *A_v, const void *B_k, const void *B_v,
                             const void *pack_ws);
// with_b: also pack B_l into the workspace (false when the caller supplies the group's packed B)
PackArgs gather_attend_pack_args(const xkv_shape &s, int layer, const void *B_k, const void *B_v, const void *q,
                                 void *pack_ws, bool with_b);
bool gather_attend_mfma_shape_ok(const xkv_shape &s);
int gather_attend_mfma_waves(const xkv_shape &s);
size_t gather_attend_pack_bytes(const xkv_shape &s);        // Q^T fragments + one layer's packed B (workspace)
size_t gather_attend_group_pack_bytes(const xkv_shape &s);  // packed B of all G layers of a group (xkv_pack_b)
hipError_t launch_pack_group(const xkv_shape &s, const void *B_k, const void *B_v, void *packed, hipStream_t st);
hipError_t launch_gather_attend_mfma(const xkv_shape &s, const Plan &p, int layer, const void *A_k, const void *A_v,
                                     const void *B_k, const void *B_v, const void *q, const int32_t *idx,
                                     void *pack_ws, const void *B_packed, bool packed, float *part_o, float *part_ml,
                                     hipStream_t st, const int32_t *counts = nullptr, float rope_theta = 0.0f,
                                     int qbits = 0);
hipError_t launch_dense(const xkv_shape &s, const Plan &p, const void *K, const void *V, const void *q, float *part_o,
                        float *part_ml, hipStream_t st);
bool dense_mfma_shape_ok(const xkv_shape &s);
hipError_t launch_combine(const xkv_shape &s, int n_part, const float *part_o, const float *part_ml, void *out,
                          hipStream_t st, int n_part2 = 0, const float *part_o2 = nullptr,
                          const float *part_ml2 = nullptr);
bool dense_uses_mfma(const Plan &p, const void *K, const void *V, const void *q);
hipError_t launch_reconstruct(const xkv_shape &s, int layer, const void *A, const void *B, int r, void *X,
                              hipStream_t st);
// Attention over selected tokens in the absorbed form (see absorbed.hip): extra workspace laid out behind the
// `base_bytes` of the ordinary plan.
struct AbsorbPlan {
    int nrp;         // row length of the per-head score array
    int chunk;       // selected tokens per split
    int splits;
    int col_blocks;  // blocks of 64 sixteen-byte pieces of a row of A^V
    int slices;      // attention partials per query head that the projection with B^V leaves
    size_t off_heads, off_part_u, off_part_ml, off_po, off_pml, total;
};
bool absorb_shape_ok(const xkv_shape &s);
AbsorbPlan make_absorb_plan(const xkv_shape &s, size_t base_bytes);
hipError_t launch_absorbed(const xkv_shape &s, const AbsorbPlan &a, int layer, const void *A_v, const void *B_v,
                           const float *S_heads, const int32_t *idx, float *po, float *pml, float *part_u,
                           float *part_ml, hipStream_t st, bool q4 = false);
// 4-bit round-to-nearest rows (see quant.hip): r a multiple of 32; 5 r / 8 bytes per row, padded with zero bytes to
// a multiple of 16 (no padding when r is a multiple of 128).  The score kernels take multiples of 128 only.
inline bool quant_rank_ok(int r) { return r > 0 && r % 32 == 0; }
__host__ __device__ inline size_t quant_row_bytes(int r) { return ((size_t)r * 5 / 8 + 15) / 16 * 16; }
// 3-bit rows: one 16-byte piece per group of 32 ranks (96 bits of codes, then step and offset), r / 2 bytes per row.
__host__ __device__ inline size_t quant_row_bytes(int r, int bits) { return bits == 3 ? (size_t)r / 2 : quant_row_bytes(r); }
bool score_q4_shape_ok(const xkv_shape &s);
hipError_t launch_score_q4_stage(const xkv_shape &s, const Plan &p, int layer, const void *Aq_k, const void *B_k,
                                 const void *q, void *P_ws, float *S, float *S_heads, hipStream_t st);
hipError_t launch_quantize_rows(const void *X, long long rows, int r, int bits, void *out, hipStream_t st);
// Cross-layer factorization of the caches of one group (see factorize.hip).
bool factorize_shape_ok(const xkv_shape &s, int r);
size_t factorize_workspace_bytes(const xkv_shape &s, int r);
// The paper's landmark-guided chunk selector (see landmark.hip).
hipError_t launch_landmarks(const xkv_shape &s, const void *K_rope, int c, void *landmarks, float *neg_min_cos,
                            hipStream_t st);
hipError_t launch_identity(const xkv_shape &s, void *B, int copies, hipStream_t st);
hipError_t launch_expand_chunks(const xkv_shape &s, const int32_t *chunks, int k_ch, const int32_t *outliers, int o, int c,
                                int32_t *rows, int32_t *counts, hipStream_t st);
// r_out <= r: how many of the leading singular directions are written; sigma_out (nullable) [batch][r_out].
hipError_t launch_factorize(const xkv_shape &s, const void *X, int r, int r_out, int iters, uint32_t seed, void *A_out,
                            void *B_out, float *sigma_out, void *ws, hipStream_t st);

}  // namespace xkv
