// Query projection into the rank space and the low-rank score stream with GQA max-pooling.
//   p_h = B^K_{l,rho(h)} q_h                      (Eq. 3 regrouped by associativity)
//   s[h,t] = scale * A^K[t,:] . p_h               (App. B.1 Alg. 2, scaled scores, per token)
//   S[g,t] = max_{h: rho(h)=g} s[h,t]             (App. B.1 Alg. 2, GQA pooling)
#include "xkv_common.h"
#include "prepass.h"

namespace xkv {

// ------------------------------------------------------------------------------------------
// project_q: one wavefront per (rank index i, KV head g); lanes run over the head dimension.
// P is written as fp32 [batch][H_q][r_k].
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void project_q_kernel(const T *__restrict__ B_k,  // [batch][G][r_k][d]
                                                        const T *__restrict__ q,    // [batch][H_q][d_h]
                                                        float *__restrict__ P,      // [batch][H_q][r_k]
                                                        int G, int layer, int r_k, int H_kv, int H_q, int d_h)
{
    const int b = blockIdx.y;
    const int item = blockIdx.x * 4 + wave_id();  // (i, g) pair
    if (item >= r_k * H_kv) return;
    const int i = item / H_kv, g = item % H_kv;
    const int n_rep = H_q / H_kv, d = H_kv * d_h;
    const int lane = lane_id();
    const T *Brow = B_k + (((size_t)b * G + layer) * r_k + i) * d + (size_t)g * d_h;
    const T *qg = q + ((size_t)b * H_q + (size_t)g * n_rep) * d_h;
    float acc[16];
#pragma unroll
    for (int hh = 0; hh < 16; ++hh) acc[hh] = 0.0f;
    for (int j = lane; j < d_h; j += kWave) {
        const float bv = to_f32(Brow[j]);
#pragma unroll
        for (int hh = 0; hh < 16; ++hh)
            if (hh < n_rep) acc[hh] = fmaf(bv, to_f32(qg[(size_t)hh * d_h + j]), acc[hh]);
    }
#pragma unroll
    for (int hh = 0; hh < 16; ++hh) {
        if (hh < n_rep) {
            const float v = wave_sum(acc[hh]);
            if (lane == 0) P[((size_t)b * H_q + g * n_rep + hh) * r_k + i] = v;
        }
    }
}

// ------------------------------------------------------------------------------------------
// score, general path: one thread per token, fp32 FMA.  Each thread walks its row of A^K once
// per block of up to 8 query heads; P is read through wave-uniform (scalar) loads.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void score_generic_kernel(const T *__restrict__ A_k,      // [batch][L][r_k]
                                                            const float *__restrict__ P,   // [batch][H_q][r_k]
                                                            float *__restrict__ S,         // [batch][H_kv][L]
                                                            int L, int r_k, int H_kv, int H_q, float scale)
{
    const int b = blockIdx.y;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= L) return;
    const int n_rep = H_q / H_kv;
    const T *Arow = A_k + ((size_t)b * L + t) * r_k;
    const float *Pb = P + (size_t)b * H_q * r_k;
    for (int g = 0; g < H_kv; ++g) {
        float best = -INFINITY;
        for (int h0 = 0; h0 < n_rep; h0 += 8) {
            float acc[8];
#pragma unroll
            for (int hh = 0; hh < 8; ++hh) acc[hh] = 0.0f;
            const float *Pg = Pb + (size_t)(g * n_rep + h0) * r_k;
            const int nh = n_rep - h0 < 8 ? n_rep - h0 : 8;
            for (int i = 0; i < r_k; ++i) {
                const float a = to_f32(Arow[i]);
#pragma unroll
                for (int hh = 0; hh < 8; ++hh)
                    if (hh < nh) acc[hh] = fmaf(a, Pg[(size_t)hh * r_k + i], acc[hh]);
            }
#pragma unroll
            for (int hh = 0; hh < 8; ++hh)
                if (hh < nh) best = fmaxf(best, scale * acc[hh]);
        }
        S[((size_t)b * H_kv + g) * L + t] = best;
    }
}

// Same walk, but every query head's score is kept as well: S_heads is [batch][H_kv][L][nrp] with nrp the
// number of query heads per KV head rounded up to a power of two (the padding is written as zero).  The pooled
// score is the maximum of exactly the values stored, so a softmax over stored head scores agrees with the
// selection made on S.
template <typename T>
__global__ __launch_bounds__(256) void score_heads_generic_kernel(const T *__restrict__ A_k,     // [batch][L][r_k]
                                                                  const float *__restrict__ P,  // [batch][H_q][r_k]
                                                                  float *__restrict__ S,        // [batch][H_kv][L]
                                                                  float *__restrict__ S_heads, int L, int r_k,
                                                                  int H_kv, int H_q, int nrp, float scale)
{
    const int b = blockIdx.y;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= L) return;
    const int n_rep = H_q / H_kv;
    const T *Arow = A_k + ((size_t)b * L + t) * r_k;
    const float *Pb = P + (size_t)b * H_q * r_k;
    for (int g = 0; g < H_kv; ++g) {
        float best = -INFINITY;
        float *dst = S_heads + (((size_t)b * H_kv + g) * L + t) * nrp;
        for (int h0 = 0; h0 < nrp; h0 += 8) {
            float acc[8];
#pragma unroll
            for (int hh = 0; hh < 8; ++hh) acc[hh] = 0.0f;
            const float *Pg = Pb + (size_t)(g * n_rep + h0) * r_k;
            const int nh = n_rep - h0 < 8 ? n_rep - h0 : 8;  // may be <= 0 inside the padding
            for (int i = 0; i < r_k && nh > 0; ++i) {
                const float a = to_f32(Arow[i]);
#pragma unroll
                for (int hh = 0; hh < 8; ++hh)
                    if (hh < nh) acc[hh] = fmaf(a, Pg[(size_t)hh * r_k + i], acc[hh]);
            }
#pragma unroll
            for (int hh = 0; hh < 8; ++hh) {
                if (hh < nh) best = fmaxf(best, scale * acc[hh]);
                if (h0 + hh < nrp) dst[h0 + hh] = hh < nh ? scale * acc[hh] : 0.0f;
            }
        }
        S[((size_t)b * H_kv + g) * L + t] = best;
    }
}

// ==========================================================================================
// bf16 MFMA path.  The contraction S^T = P_slots (32 x r) . A^T (r x tokens) runs on
// v_mfma_f32_32x32x16_bf16: the MFMA "A" operand is a fragment of P (32 head slots x 16 ranks)
// read from LDS, the "B" operand is 16 B of a token's row of A^K loaded straight from global
// memory (lane (n, hf) holds ranks 16f + 8hf .. +7 of token n for fragment f), so A^K is
// streamed exactly once and never staged.  In the 32x32 result lane (n, hf) holds, for token n,
// the 16 head slots 8(v/4) + 4hf + v%4, v = 0..15.  Query heads are placed in slots so that all
// heads of a KV head sit in one lane's registers: the GQA max-pool needs no cross-lane traffic.
//
// Slot map: half hf holds gph = 16 / n_rep KV heads; KV head g sits in block g / (2 gph), half
// (g % (2 gph)) / gph, position u = g % gph, and its query head hh in register v = u n_rep + hh.
// P is kept as a sum of two bf16 values (high part and remainder) so that the scores carry
// fp32-accumulation accuracy even though the MFMA operands are bf16.
// ==========================================================================================
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;


__global__ __launch_bounds__(256) void project_q_frag_kernel(ProjArgs a)
{
    project_q_frag_block(a, blockIdx.x, blockIdx.y);
}

// One launch for the small passes that precede the score kernel: blocks [0, n_proj) project the queries, the next
// n_pack put the Q^T fragments and (unless the caller brought a packed B) B_l into fragment order for the
// gather-attend kernel (see prepass.h), the rest clear the row histograms that the score kernel adds to (zero_words a
// multiple of 4).
__global__ __launch_bounds__(256) void prepass_kernel(ProjArgs pj, PackArgs pk, int n_proj, int n_pack,
                                                      uint32_t *__restrict__ zero, int zero_words)
{
    if ((int)blockIdx.x < n_proj) {
        project_q_frag_block(pj, (int)blockIdx.x % pj.blocks_x, (int)blockIdx.x / pj.blocks_x);
    } else if ((int)blockIdx.x < n_proj + n_pack) {
        const int per_head = pk.blocks_per_head + kPackQBlocks;
        const int pl = (int)blockIdx.x - n_proj, blk = pl % per_head;
        const int g = (pl / per_head) % pk.H_kv, b = pl / (per_head * pk.H_kv);
        if (blk < pk.blocks_per_head)
            pack_b_block(pk, blk, g, b);
        else
            pack_q_block(pk, blk - pk.blocks_per_head, g, b);
    } else {
        const int i = 4 * (((int)blockIdx.x - n_proj - n_pack) * 256 + (int)threadIdx.x);
        if (i < zero_words) *reinterpret_cast<u32x4_t *>(zero + i) = u32x4_t{0u, 0u, 0u, 0u};
    }
}

// Heads per KV head rounded up to a power of two: the row length of the per-head score array.
constexpr int head_pitch(int n_rep) { return n_rep <= 1 ? 1 : n_rep <= 2 ? 2 : n_rep <= 4 ? 4 : n_rep <= 8 ? 8 : 16; }

// HEADS: also write every query head's score, S_heads [batch][H_kv][L][head_pitch(N_REP)] (padding zero); the
// pooled score is the maximum of exactly those values.
template <int N_REP, bool HEADS>
__global__ __launch_bounds__(256) void score_mfma_kernel(const bf16_t *__restrict__ A_k,    // [batch][L][r_k]
                                                         const bf16_t *__restrict__ Pfrag,  // see above
                                                         float *__restrict__ S,             // [batch][H_kv][L]
                                                         int L, int r_k, int H_kv, int F8, int tiles_per_wg,
                                                         float scale, float *__restrict__ S_heads)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4_t *Pl = reinterpret_cast<u32x4_t *>(smem);  // [2][F8][64] fragments of 16 B per lane
    constexpr int GPH = 16 / N_REP;
    const int b = blockIdx.z, blk = blockIdx.y, nblk = gridDim.y;
    const int lane = lane_id(), w = wave_id();
    const int n = lane & 31, hf = lane >> 5;
    const int F = r_k / 16;

    // stage this block's P fragments (hi and lo parts) in LDS, eight 16 B loads in flight per thread
    {
        const u32x4_t *src = reinterpret_cast<const u32x4_t *>(Pfrag) + ((size_t)b * nblk + blk) * 2 * F8 * 64;
        const int total = 2 * F8 * 64;  // a multiple of 4 * 256
        for (int e0 = threadIdx.x; e0 < total; e0 += 4 * 256) {
            u32x4_t tmp[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) tmp[j] = src[e0 + j * 256];
#pragma unroll
            for (int j = 0; j < 4; ++j) Pl[e0 + j * 256] = tmp[j];
        }
    }
    __syncthreads();

    const bf16_t *Ab = A_k + (size_t)b * L * r_k;
    const int n_tiles = (L + 31) / 32;
    const int tile_begin = blockIdx.x * tiles_per_wg;
    const int tile_end = tile_begin + tiles_per_wg < n_tiles ? tile_begin + tiles_per_wg : n_tiles;
    const int n_steps = F8 / 8;  // steps of 8 fragments per tile
    // 16 B pieces of a token's row for one step; fragments beyond the rank meet zero P fragments, so the
    // address is only clamped, never skipped: the loop body is straight-line code
    auto load_step = [&](int tile, int step, u32x4_t (&a)[8]) __attribute__((always_inline)) {
        const int t = tile * 32 + n;
        const u32x4_t *row = reinterpret_cast<const u32x4_t *>(Ab + (size_t)(t < L ? t : L - 1) * r_k) + hf;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int f = step * 8 + j;
            a[j] = row[2 * (f < F ? f : F - 1)];
        }
    };
    int tile = tile_begin + w;
    if (tile >= tile_end) return;
    u32x4_t a_cur[8], a_nxt[8];
    load_step(tile, 0, a_cur);
    f32x16_t acc_h, acc_l;  // separate chains for the high parts and the remainders of P
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_h[v] = acc_l[v] = 0.0f;
    int step = 0;
    while (true) {
        // pieces of the next step (of this tile, or the first of the wavefront's next tile) before this step's MFMAs
        const bool last_step = step + 1 == n_steps;
        const int tile_n = last_step ? tile + 4 : tile, step_n = last_step ? 0 : step + 1;
        load_step(tile_n < tile_end ? tile_n : tile, step_n, a_nxt);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const u32x4_t ph = Pl[(step * 8 + j) * 64 + lane];
            const u32x4_t pl = Pl[(F8 + step * 8 + j) * 64 + lane];
            acc_h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ph),
                                                            __builtin_bit_cast(bf16x8_t, a_cur[j]), acc_h, 0, 0, 0);
            acc_l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, pl),
                                                            __builtin_bit_cast(bf16x8_t, a_cur[j]), acc_l, 0, 0, 0);
        }
        if (last_step) {
            const int t = tile * 32 + n;
            if (t < L) {
#pragma unroll
                for (int u = 0; u < GPH; ++u) {
                    const int g = blk * 2 * GPH + hf * GPH + u;
                    if constexpr (HEADS) {
                        constexpr int NRP = head_pitch(N_REP);
                        float hv[16];
#pragma unroll
                        for (int hh = 0; hh < 16; ++hh)
                            hv[hh] = hh < N_REP ? scale * (acc_h[(u * N_REP + hh) & 15] + acc_l[(u * N_REP + hh) & 15]) : 0.0f;
                        float best = hv[0];
#pragma unroll
                        for (int hh = 1; hh < N_REP; ++hh) best = fmaxf(best, hv[hh]);
                        if (g < H_kv) {
                            S[((size_t)b * H_kv + g) * L + t] = best;
                            float *dst = S_heads + (((size_t)b * H_kv + g) * L + t) * NRP;
                            if constexpr (NRP >= 4) {
#pragma unroll
                                for (int c = 0; c < NRP / 4; ++c)
                                    *reinterpret_cast<float4 *>(dst + 4 * c) =
                                        make_float4(hv[4 * c], hv[4 * c + 1], hv[4 * c + 2], hv[4 * c + 3]);
                            } else {
#pragma unroll
                                for (int hh = 0; hh < NRP; ++hh) dst[hh] = hv[hh];
                            }
                        }
                    } else {
                        float best = acc_h[u * N_REP] + acc_l[u * N_REP];
#pragma unroll
                        for (int hh = 1; hh < N_REP; ++hh)
                            best = fmaxf(best, acc_h[u * N_REP + hh] + acc_l[u * N_REP + hh]);
                        if (g < H_kv) __builtin_nontemporal_store(scale * best, &S[((size_t)b * H_kv + g) * L + t]);
                    }
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) acc_h[v] = acc_l[v] = 0.0f;
            if (tile_n >= tile_end) break;
        }
        tile = tile_n;
        step = step_n;
#pragma unroll
        for (int j = 0; j < 8; ++j) a_cur[j] = a_nxt[j];
    }
}

// Variant for long streams: the same contraction, but A^K is fetched line-wise and turned into operand
// fragments through a wavefront-private LDS tile.  A group is 128 ranks (256 B) of each of the wavefront's 32
// token rows; instruction j of a group covers rows 4j..4j+3, lane l loading the 16 B piece l%16 of row 4j + l/16,
// so every 128 B line is requested by exactly one instruction (with one lane per row, four instructions share
// each line and the stream runs well below the memory rate).  The tile is written row-wise, rotated by the row
// number so that neither side has bank conflicts (piece c of row t at 16 t + (c + t) % 16, in 16 B units), and
// read back as one fragment per step.  Two groups are in flight in registers per wavefront; nothing in the
// main loop needs a barrier (P is read-only in LDS, the tiles are private).
constexpr int kScoreWaves = 8;  // wavefronts per workgroup; 4 when the P fragments leave no room for 8 tiles

template <int SLOT0>
__device__ __forceinline__ void score_group(f32x16_t &acc_h, f32x16_t &acc_l, u32x4_t (&areg)[16], u32x4_t *At,
                                            const u32x4_t *Ph, const u32x4_t *Pl_, const u32x4_t *arow, int pieces,
                                            int t0, int row_step, int L, const int (&woff)[4], int rbase)
{
    // all but the 8 youngest loads (the other half of the ring) have landed: vmcnt(8), other counters untouched
    __builtin_amdgcn_s_waitcnt(8 | (7 << 4) | (0xF << 8));
#pragma unroll
    for (int j = 0; j < 8; ++j) At[64 * j + woff[j & 3]] = areg[SLOT0 + j];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int fl = 0; fl < 8; ++fl) {
        const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, At[(rbase & ~15) + ((rbase + 2 * fl) & 15)]);
        acc_h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, Ph[fl * 64]), a0, acc_h, 0, 0, 0);
        acc_l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, Pl_[fl * 64]), a0, acc_l, 0, 0, 0);
        // instruction fl of the group two groups on, into the ring entry written out above
        const int t = t0 + row_step * fl;
        areg[SLOT0 + fl] = __builtin_nontemporal_load(&arow[(size_t)(t < L ? t : L - 1) * pieces]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// One token's head scores (NRP consecutive floats, v[] already zero beyond the real heads), as hidden stores
// like the pooled ones below.
template <int NRP> __device__ __forceinline__ void store_head_row(float *dst, const float (&v)[16])
{
    if constexpr (NRP == 1) {
        asm volatile("global_store_dword %0, %1, off" : : "v"(dst), "v"(v[0]) : "memory");
    } else if constexpr (NRP == 2) {
        const f32x2_t x = {v[0], v[1]};
        asm volatile("global_store_dwordx2 %0, %1, off" : : "v"(dst), "v"(x) : "memory");
    } else {
#pragma unroll
        for (int c = 0; c < NRP / 4; ++c) {
            const f32x4_t x = {v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]};
            // (a store of more than 64 bits reads its data registers a cycle or two after issue; the compiler inserts
            // the wait states for stores it knows, not for these)
            asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 1" : : "v"(dst + 4 * c), "v"(x) : "memory");
        }
    }
}

// HEADS: also write every query head's score, S_heads [batch][H_kv][L][head_pitch(N_REP)] (padding zero); the
// pooled score is the maximum of exactly those values.
template <int N_REP, int WAVES, bool HEADS>
__global__ __launch_bounds__(WAVES * 64) void score_stream_kernel(const bf16_t *__restrict__ A_k,
                                                                        const bf16_t *__restrict__ Pfrag,
                                                                        float *__restrict__ S, int L, int r_k,
                                                                        int H_kv, int F8, int tiles_per_wg,
                                                                        float scale, uint32_t *__restrict__ row_hist,
                                                                        uint32_t *__restrict__ chunk_hist,
                                                                        float *__restrict__ S_heads)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4_t *Pl = reinterpret_cast<u32x4_t *>(smem);  // [2][F8][64] fragments of 16 B per lane
    constexpr int GPH = 16 / N_REP;
    // Pooled scores are kept in registers and written in bursts of RT tiles: 4 B per (KV head, token) are only 3 %
    // of the bytes, but dribbled out between the reads they cost the memory system as much as 15 % of the stream.
    // (with HEADS all 16 head slots of a tile are kept instead, and bursts are four tiles)
    constexpr int RT = HEADS ? 4 : 64 / GPH;
    constexpr int RW = HEADS ? 16 : GPH;
    constexpr int NRP = head_pitch(N_REP);
    const int b = blockIdx.z, blk = blockIdx.y, nblk = gridDim.y;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int n = lane & 31, hf = lane >> 5;
    u32x4_t *At = Pl + 2 * F8 * 64 + w * 512;
    // Optional first pass of the top-k stage: histogram of the top 8 bits of the order key of every pooled
    // score of this workgroup, one 256-bin histogram per KV head slot of the block.
    uint32_t *hist = reinterpret_cast<uint32_t *>(Pl + 2 * F8 * 64 + WAVES * 512);  // [2 GPH][256]
    const bool do_hist = row_hist != nullptr;
    if (do_hist)
        for (int i = tid; i < 2 * GPH * kTopkBins; i += WAVES * 64) hist[i] = 0;

    const int pieces = r_k >> 3;  // 16 B pieces per row
    const u32x4_t *Ab = reinterpret_cast<const u32x4_t *>(A_k + (size_t)b * L * r_k);
    const int n_tiles = (L + 31) / 32;
    const int n_groups = F8 / 8;  // groups per tile
    const int wg_end = (blockIdx.x + 1) * tiles_per_wg < n_tiles ? (blockIdx.x + 1) * tiles_per_wg : n_tiles;
    // The wavefronts of a workgroup interleave their tiles (stride TS), so that at any moment the workgroup reads
    // one compact window of the sequence: measurably faster than eight separate runs per workgroup.
    constexpr int TS = WAVES;
    int tile = blockIdx.x * tiles_per_wg + w;
    const int tile_end = wg_end;
    const bool has_work = tile < tile_end;  // wave-uniform

    int woff[4];
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) woff[qd] = 16 * (lane >> 4) + (((lane & 15) + (lane >> 4) + 4 * qd) & 15);
    const int rbase = 16 * n + ((hf + n) & 15);
    // this lane's piece of group S (beyond the row: piece 0, it meets zero P fragments) and first row of a tile
    auto piece_of = [&](int S_) __attribute__((always_inline)) {
        const int pc = 16 * S_ + (lane & 15);
        return pc < pieces ? pc : 0;
    };
    const int trow = lane >> 4;

    // first part of this block's P fragments (hi and lo parts), eight 16 B loads in flight per thread ...
    const u32x4_t *psrc = reinterpret_cast<const u32x4_t *>(Pfrag) + ((size_t)b * nblk + blk) * 2 * F8 * 64;
    const int total = 2 * F8 * 64;  // a multiple of 1024
    u32x4_t ptmp[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int e0 = tid + j * WAVES * 64;
        ptmp[j] = psrc[e0 < total ? e0 : tid];
    }
    // ... and behind them already the first two groups of A^K.  (tile, group) two groups ahead of the one being
    // multiplied; past the end it stays on the last tile.
    int tile_p = has_work ? tile : 0, S_p = 0;
    // (the prefetches keep being issued past the wavefront's last tile -- the waits count outstanding loads -- but
    // then every one of them goes to one row, a cache hit, instead of streaming the last tile from memory again)
    int row_step = 4, row_lane = 1;  // rows between the instructions of a group, and between a lane's row and lane/16
    auto advance_p = [&]() __attribute__((always_inline)) {
        if (++S_p == n_groups) {
            S_p = 0;
            if (tile_p + TS < tile_end) {
                tile_p += TS;
            } else {
                row_step = 0;
                row_lane = 0;
            }
        }
    };
    u32x4_t areg[16];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const u32x4_t *arow = Ab + piece_of(S_p);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int t = tile_p * 32 + trow + 4 * j;
            areg[half * 8 + j] = __builtin_nontemporal_load(&arow[(size_t)(t < L ? t : L - 1) * pieces]);
            __builtin_amdgcn_sched_barrier(0);
        }
        advance_p();
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int e0 = tid + j * WAVES * 64;
        if (e0 < total) Pl[e0] = ptmp[j];
    }
    for (int e0 = tid + 8 * WAVES * 64; e0 < total; e0 += 2 * WAVES * 64) {
        u32x4_t tmp[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) tmp[j] = psrc[e0 + j * WAVES * 64];
#pragma unroll
        for (int j = 0; j < 2; ++j) Pl[e0 + j * WAVES * 64] = tmp[j];
    }
    __syncthreads();
    if (has_work) {
    f32x16_t acc_h, acc_l;  // separate chains for the high parts and the remainders of P
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_h[v] = acc_l[v] = 0.0f;
    float res[RT][RW];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int u = 0; u < RW; ++u) res[i][u] = 0.0f;
    int S_c = 0, ti = 0, tile0 = tile;  // group within the tile, tiles held in res, first of them
    // Stores go through inline assembly: a store the compiler knows of inside conditional code makes its count of
    // outstanding memory operations uncertain, and it then waits for *all* prefetches at the top of the loop.
    // Unknown to it, the stores only make those waits stricter for a moment.
    auto flush = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            const int t = (tile0 + i * TS) * 32 + n;
            if (i < ti && t < L) {
#pragma unroll
                for (int u = 0; u < GPH; ++u) {
                    const int g = blk * 2 * GPH + hf * GPH + u;
                    if (g < H_kv) {
                        float *dst = S + ((size_t)b * H_kv + g) * L + t;
                        if constexpr (HEADS) {
                            float hv[16];
#pragma unroll
                            for (int hh = 0; hh < 16; ++hh) hv[hh] = hh < N_REP ? res[i][(u * N_REP + hh) & 15] : 0.0f;
                            float best = hv[0];
#pragma unroll
                            for (int hh = 1; hh < N_REP; ++hh) best = fmaxf(best, hv[hh]);
                            asm volatile("global_store_dword %0, %1, off" : : "v"(dst), "v"(best) : "memory");
                            store_head_row<NRP>(S_heads + (((size_t)b * H_kv + g) * L + t) * NRP, hv);
                        } else {
                            asm volatile("global_store_dword %0, %1, off" : : "v"(dst), "v"(res[i][u]) : "memory");
                        }
                    }
                }
            }
        }
        tile0 += ti * TS;
        ti = 0;
    };
    auto finish_group = [&]() __attribute__((always_inline)) {  // closes a tile after its last group
        if (++S_c < n_groups) return;
        S_c = 0;
#pragma unroll
        for (int u = 0; u < GPH; ++u) {
            float best = acc_h[u * N_REP] + acc_l[u * N_REP];
#pragma unroll
            for (int hh = 1; hh < N_REP; ++hh) best = fmaxf(best, acc_h[u * N_REP + hh] + acc_l[u * N_REP + hh]);
            best *= scale;
            if constexpr (HEADS) {
#pragma unroll
                for (int hh = 0; hh < N_REP; ++hh) {
                    const float hs = scale * (acc_h[u * N_REP + hh] + acc_l[u * N_REP + hh]);
#pragma unroll
                    for (int i = 0; i < RT; ++i) res[i][u * N_REP + hh] = (i == ti) ? hs : res[i][u * N_REP + hh];
                }
            } else {
#pragma unroll
                for (int i = 0; i < RT; ++i) res[i][u] = (i == ti) ? best : res[i][u];
            }
            if (do_hist) {
                // Done per tile, where it hides behind the other wavefronts' memory waits.  Scores cluster in few
                // bins: one LDS add per distinct (head slot, bin) of the wavefront.
                const int g = blk * 2 * GPH + hf * GPH + u;
                const uint32_t slot = (uint32_t)(hf * GPH + u) * kTopkBins + (order_key(best) >> 24);
                const bool active = tile * 32 + n < L && g < H_kv;
                uint64_t m = __ballot(active);
                while (m != 0) {
                    const int first = __ffsll((unsigned long long)m) - 1;
                    const uint32_t s0 = (uint32_t)__builtin_amdgcn_readlane((int)slot, first);
                    const uint64_t same = __ballot(active && slot == s0);
                    if (lane == first) atomicAdd(&hist[s0], (uint32_t)__popcll(same));
                    m &= ~same;
                }
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_h[v] = acc_l[v] = 0.0f;
        tile += TS;
        ++ti;
    };
    // groups of this wavefront, two per iteration (one per half of the ring); an odd total leaves one surplus
    // group at the end, which multiplies re-fetched rows of the last tile and is dropped
    const int my_groups = (tile_end - tile + TS - 1) / TS * n_groups;
    for (int gi = 0; gi < my_groups; gi += 2) {
        {
            const u32x4_t *arow = Ab + piece_of(S_p);
            const int t0 = tile_p * 32 + trow * row_lane, rs = row_step;
            advance_p();
            score_group<0>(acc_h, acc_l, areg, At, Pl + (S_c * 8) * 64 + lane, Pl + (F8 + S_c * 8) * 64 + lane, arow,
                           pieces, t0, rs, L, woff, rbase);
            finish_group();
        }
        {
            const u32x4_t *arow = Ab + piece_of(S_p);
            const int t0 = tile_p * 32 + trow * row_lane, rs = row_step;
            advance_p();
            score_group<8>(acc_h, acc_l, areg, At, Pl + (S_c * 8) * 64 + lane, Pl + (F8 + S_c * 8) * 64 + lane, arow,
                           pieces, t0, rs, L, woff, rbase);
            if (gi + 1 < my_groups) finish_group();
        }
        if (ti > RT - 2) flush();  // up to two tiles complete per iteration
    }
    flush();
    }
    if (do_hist) {
        // this workgroup is chunk blockIdx.x of its rows: keep the chunk histograms, add them to the rows'
        __syncthreads();
        const int chunks = gridDim.x;
        for (int i = tid; i < 2 * GPH * kTopkBins; i += WAVES * 64) {
            const int g = blk * 2 * GPH + i / kTopkBins, bin = i % kTopkBins;
            if (g < H_kv) {
                const size_t row = (size_t)b * H_kv + g;
                const uint32_t cnt = hist[i];
                chunk_hist[(row * chunks + blockIdx.x) * kTopkLevels * kTopkBins + bin] = cnt;
                if (cnt != 0) atomicAdd(&row_hist[row * kTopkLevels * kTopkBins + bin], cnt);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Scores from a 4-bit quantised token basis (quant.hip: per row r/8 words of codes, then (step, lo) per group of
// 32 ranks).  Same contraction and head-slot layout as above, with the codes themselves as the matrix-core
// operand: a code c in 0..15 is the bf16 number 128 + c when 0x4300 is or-ed on top of it, and a pair of adjacent
// ranks is one shift and one mask away from a packed bf16 pair.  Per group g and token t the matrix cores give
//   acc_g[slot] = sum_{i in g} (128 + c_ti) p[slot][i]      (exact products, fp32 sums, P as bf16 hi + lo)
// and the affine map of the group is applied to the sum, not to the elements:
//   s[slot] += step_tg (acc_g[slot] - 128 Ps_g[slot]) + lo_tg Ps_g[slot],   Ps_g[slot] = sum_{i in g} p[slot][i].
// (In this kernel the second part is kept in fp32 multiply-adds; the line-wise kernel below runs it on the matrix
// cores with exact three-way splits.)
// Lane (n, hf) loads the 16 bytes of each of token n's groups (both halves load the same pieces) and the parameter
// words.  Always writes the per-head scores as well as the pooled ones.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ bf16x8_t q4_fragment(uint32_t w)
{
    u32x4_t o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = ((w >> (4 * i)) & 0x000F000Fu) | 0x43004300u;
    return __builtin_bit_cast(bf16x8_t, o);
}

// One pass of a token's quantised row: GP groups of codes from group g0 on (clamped to the last real group) and
// their parameter words.  n_groups is a multiple of 4.
template <int GP>
__device__ __forceinline__ void q4_load_pass(u32x4_t (&cw)[GP], u32x4_t (&pw)[GP / 4], const unsigned char *Ab, size_t pitch,
                                             int r_k, int t, int L, int g0, int n_groups)
{
    const unsigned char *rowp = Ab + (size_t)(t < L ? t : L - 1) * pitch;
    const u32x4_t *codes = reinterpret_cast<const u32x4_t *>(rowp);
    const u32x4_t *params = reinterpret_cast<const u32x4_t *>(rowp + (r_k >> 1));
#pragma unroll
    for (int j = 0; j < GP; ++j) cw[j] = codes[g0 + j < n_groups ? g0 + j : n_groups - 1];
#pragma unroll
    for (int j = 0; j < GP / 4; ++j) pw[j] = params[g0 + 4 * j < n_groups ? (g0 >> 2) + j : (n_groups >> 2) - 1];
}

template <int N_REP, int WAVES, int GP>
__global__ __launch_bounds__(WAVES * 64) void score_q4_kernel(const unsigned char *__restrict__ Aq,  // [batch][L][5 r_k / 8]
                                                       const bf16_t *__restrict__ Pfrag, float *__restrict__ S,
                                                       float *__restrict__ S_heads, int L, int r_k, int H_kv, int F8,
                                                       int tiles_per_wg, float scale)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4_t *Pl = reinterpret_cast<u32x4_t *>(smem);                   // [2][F8][64] fragments of 16 B per lane
    float *Ps = reinterpret_cast<float *>(Pl + 2 * F8 * 64);            // [F8 / 2 groups][32 slots]
    constexpr int GPH = 16 / N_REP;
    constexpr int NRP = head_pitch(N_REP);
    const int b = blockIdx.z, blk = blockIdx.y, nblk = gridDim.y;
    const int lane = lane_id(), w = wave_id();
    const int n = lane & 31, hf = lane >> 5;
    const int n_groups = r_k >> 5;  // = F8 / 2 for the ranks this kernel takes (multiples of 128)
    {
        const u32x4_t *src = reinterpret_cast<const u32x4_t *>(Pfrag) + ((size_t)b * nblk + blk) * 2 * F8 * 64;
        const int total = 2 * F8 * 64;  // a multiple of 1024
        for (int e0 = threadIdx.x; e0 < total; e0 += 4 * WAVES * 64) {
            u32x4_t tmp[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) tmp[j] = src[e0 + j * WAVES * 64 < total ? e0 + j * WAVES * 64 : e0];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (e0 + j * WAVES * 64 < total) Pl[e0 + j * WAVES * 64] = tmp[j];
        }
    }
    __syncthreads();
    // Ps: lane (slot m, hf) sums its 8 ranks of both fragments and both parts of a group, the halves are added
    for (int g = w; g < F8 / 2; g += WAVES) {
        float sum = 0.0f;
#pragma unroll
        for (int part = 0; part < 2; ++part)
#pragma unroll
            for (int ff = 0; ff < 2; ++ff) {
                const u32x4_t v = Pl[(part * F8 + 2 * g + ff) * 64 + lane];
#pragma unroll
                for (int e = 0; e < 4; ++e) sum += __uint_as_float(v[e] << 16) + __uint_as_float(v[e] & 0xFFFF0000u);
            }
        sum += __shfl_xor(sum, 32, kWave);
        if (hf == 0) Ps[g * 32 + n] = sum;
    }
    __syncthreads();

    const size_t pitch = (size_t)r_k * 5 / 8;
    const unsigned char *Ab = Aq + (size_t)b * L * pitch;
    const int n_tiles = (L + 31) / 32;
    const int tile_begin = blockIdx.x * tiles_per_wg;
    const int tile_end = tile_begin + tiles_per_wg < n_tiles ? tile_begin + tiles_per_wg : n_tiles;
    // A token's row is requested a pass at a time (a pass = GP groups = 16 GP bytes of codes and 4 GP bytes of
    // parameters per lane), and the next pass -- of this tile or of the wavefront's next tile -- is requested
    // before the products of the current one: with one group in flight per lane the stream is bound by load
    // latency, not by bytes.
    const int n_pass = (n_groups + GP - 1) / GP;
    int tile = tile_begin + w;
    if (tile >= tile_end) return;
    u32x4_t cw[GP], pw[GP / 4];
    q4_load_pass<GP>(cw, pw, Ab, pitch, r_k, tile * 32 + n, L, 0, n_groups);
    f32x16_t tot;
#pragma unroll
    for (int v = 0; v < 16; ++v) tot[v] = 0.0f;
    const f32x16_t zero = tot;
    int pass = 0;
    while (true) {
        const bool last_pass = pass + 1 == n_pass;
        const int tile_n = last_pass ? tile + WAVES : tile, pass_n = last_pass ? 0 : pass + 1;
        u32x4_t cw_n[GP], pw_n[GP / 4];
        q4_load_pass<GP>(cw_n, pw_n, Ab, pitch, r_k, (tile_n < tile_end ? tile_n : tile) * 32 + n, L, pass_n * GP, n_groups);
        const int g0 = pass * GP;
#pragma unroll
        for (int j = 0; j < GP; ++j) {
            const int g = g0 + j;
            if (g < n_groups) {  // wave-uniform
                f32x16_t acc = zero;
#pragma unroll
                for (int ff = 0; ff < 2; ++ff) {
                    // fragment 2g + ff covers ranks 32g + 16ff ..; this half takes word 2ff + hf of the group
                    const uint32_t word = hf ? (ff ? cw[j][3] : cw[j][1]) : (ff ? cw[j][2] : cw[j][0]);
                    const bf16x8_t bop = q4_fragment(word);
                    const u32x4_t ph = Pl[(2 * g + ff) * 64 + lane];
                    const u32x4_t pl = Pl[(F8 + 2 * g + ff) * 64 + lane];
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ph), bop, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, pl), bop, acc, 0, 0, 0);
                }
                const uint32_t pword = pw[j >> 2][j & 3];
                const float step = __uint_as_float(pword << 16), lo = __uint_as_float(pword & 0xFFFF0000u);
                const float c2 = fmaf(-128.0f, step, lo);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float4 ps = *reinterpret_cast<const float4 *>(Ps + g * 32 + 8 * i + 4 * hf);
                    tot[4 * i + 0] = fmaf(step, acc[4 * i + 0], fmaf(c2, ps.x, tot[4 * i + 0]));
                    tot[4 * i + 1] = fmaf(step, acc[4 * i + 1], fmaf(c2, ps.y, tot[4 * i + 1]));
                    tot[4 * i + 2] = fmaf(step, acc[4 * i + 2], fmaf(c2, ps.z, tot[4 * i + 2]));
                    tot[4 * i + 3] = fmaf(step, acc[4 * i + 3], fmaf(c2, ps.w, tot[4 * i + 3]));
                }
            }
        }
#pragma unroll
        for (int j = 0; j < GP; ++j) cw[j] = cw_n[j];
#pragma unroll
        for (int j = 0; j < GP / 4; ++j) pw[j] = pw_n[j];
        if (!last_pass) {
            pass = pass_n;
            continue;
        }
        const int t = tile * 32 + n;
        if (t < L) {
#pragma unroll
            for (int u = 0; u < GPH; ++u) {
                const int g = blk * 2 * GPH + hf * GPH + u;
                if (g < H_kv) {
                    float hv[16];
#pragma unroll
                    for (int hh = 0; hh < 16; ++hh) hv[hh] = hh < N_REP ? scale * tot[(u * N_REP + hh) & 15] : 0.0f;
                    float best = hv[0];
#pragma unroll
                    for (int hh = 1; hh < N_REP; ++hh) best = fmaxf(best, hv[hh]);
                    S[((size_t)b * H_kv + g) * L + t] = best;
                    float *dst = S_heads + (((size_t)b * H_kv + g) * L + t) * NRP;
                    if constexpr (NRP >= 4) {
#pragma unroll
                        for (int c = 0; c < NRP / 4; ++c)
                            *reinterpret_cast<float4 *>(dst + 4 * c) =
                                make_float4(hv[4 * c], hv[4 * c + 1], hv[4 * c + 2], hv[4 * c + 3]);
                    } else {
#pragma unroll
                        for (int hh = 0; hh < NRP; ++hh) dst[hh] = hv[hh];
                    }
                }
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) tot[v] = 0.0f;
        if (tile_n >= tile_end) break;
        tile = tile_n;
        pass = 0;
    }
}

// The same kernel with the rows fetched line-wise: the 32 token rows of a tile are one contiguous block of
// 32 * 5r/8 bytes, which a wavefront requests as whole 1 KiB runs (lane l = 16-byte piece i * 64 + l, NL requests)
// and passes to the lanes that need them through a wavefront-private LDS tile.  With one lane per row (kernel
// above) every request touches 32 different lines and the load path, not the arithmetic, bounds the kernel (measured:
// 81 of 175 us).  Rows sit in the tile at a pitch of an odd number of 16-byte units, so the per-row reads are free
// of bank conflicts.  The next tile waits in registers while the current one is multiplied; nothing needs a
// barrier (P is read-only, the tiles are private).
constexpr int kQ4TileWaves = 8;
constexpr int kQ4MaxLoads = 10;  // 16-byte requests per lane and tile: 32 rows * 5r/8 bytes <= 10 KiB, r <= 512

__host__ __device__ inline int q4_tile_pitch(int r) { return r * 5 / 8 + ((r / 128) % 2 == 0 ? 16 : 0); }  // bytes
// (the offset term reads a row's parameters in runs of 64 bytes; the last run may reach up to 48 bytes past the
// row, into the next row of the tile or, for the last row, the 64 bytes of slack behind the wavefront's tile)
constexpr int kQ4TileSlack = 64;

template <int N_REP>
__global__ __launch_bounds__(kQ4TileWaves * 64) void score_q4_tile_kernel(const unsigned char *__restrict__ Aq,
                                                                          const bf16_t *__restrict__ Pfrag,
                                                                          float *__restrict__ S,
                                                                          float *__restrict__ S_heads, int L, int r_k,
                                                                          int H_kv, int F8, int tiles_per_wg, float scale)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int WAVES = kQ4TileWaves;
    u32x4_t *Pl = reinterpret_cast<u32x4_t *>(smem);         // [2][F8][64] fragments of 16 B per lane
    float *Ps = reinterpret_cast<float *>(Pl + 2 * F8 * 64);  // [F8 / 2 groups][32 slots]
    constexpr int GPH = 16 / N_REP;
    constexpr int NRP = head_pitch(N_REP);
    const int b = blockIdx.z, blk = blockIdx.y, nblk = gridDim.y;
    const int lane = lane_id(), w = wave_id();
    const int n = lane & 31, hf = lane >> 5;
    const int n_groups = r_k >> 5;
    const int tpitch = q4_tile_pitch(r_k);
    const int n_pass = (n_groups + 15) >> 4;  // passes of 16 groups of the offset term
    u32x4_t *PsF = reinterpret_cast<u32x4_t *>(Ps + (F8 / 2) * 32);  // [n_pass][3 parts][64]: Ps as operand fragments
    unsigned char *tile_lds = reinterpret_cast<unsigned char *>(PsF + n_pass * 3 * 64) + (size_t)w * (32 * tpitch + kQ4TileSlack);
    {
        const u32x4_t *src = reinterpret_cast<const u32x4_t *>(Pfrag) + ((size_t)b * nblk + blk) * 2 * F8 * 64;
        const int total = 2 * F8 * 64;  // a multiple of 1024
        for (int e0 = threadIdx.x; e0 < total; e0 += 4 * WAVES * 64) {
            u32x4_t tmp[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) tmp[j] = src[e0 + j * WAVES * 64 < total ? e0 + j * WAVES * 64 : e0];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (e0 + j * WAVES * 64 < total) Pl[e0 + j * WAVES * 64] = tmp[j];
        }
    }
    __syncthreads();
    for (int g = w; g < F8 / 2; g += WAVES) {
        float sum = 0.0f;
#pragma unroll
        for (int part = 0; part < 2; ++part)
#pragma unroll
            for (int ff = 0; ff < 2; ++ff) {
                const u32x4_t v = Pl[(part * F8 + 2 * g + ff) * 64 + lane];
#pragma unroll
                for (int e = 0; e < 4; ++e) sum += __uint_as_float(v[e] << 16) + __uint_as_float(v[e] & 0xFFFF0000u);
            }
        sum += __shfl_xor(sum, 32, kWave);
        if (hf == 0) Ps[g * 32 + n] = sum;
    }
    __syncthreads();
    // The offset term sum_g (lo_tg - 128 step_tg) Ps_g[slot] is a product [slots x groups] . [groups x tokens] and
    // runs on the matrix cores, 16 groups per instruction.  Because 128 step Ps cancels against the first term it
    // needs full fp32 accuracy: both factors are split *exactly* into three bf16 numbers (8 + 8 + 8 mantissa bits,
    // by truncation) and the six largest of the nine partial products are taken; the dropped ones are below 2^-24
    // of the term.  Here: Ps as operand fragments, lane (slot m, hf), position e = group 16 pass + 8 hf + e.
    for (int ps = w; ps < n_pass; ps += WAVES) {
        u32x4_t f3[3];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            uint32_t part[2][3];
#pragma unroll
            for (int o = 0; o < 2; ++o) {
                const int g = 16 * ps + 8 * hf + 2 * e2 + o;
                float v = g < n_groups ? Ps[g * 32 + n] : 0.0f;
#pragma unroll
                for (int q3 = 0; q3 < 3; ++q3) {
                    part[o][q3] = __float_as_uint(v) & 0xFFFF0000u;
                    v -= __uint_as_float(part[o][q3]);
                }
            }
#pragma unroll
            for (int q3 = 0; q3 < 3; ++q3) f3[q3][e2] = (part[0][q3] >> 16) | part[1][q3];
        }
#pragma unroll
        for (int q3 = 0; q3 < 3; ++q3) PsF[(ps * 3 + q3) * 64 + lane] = f3[q3];
    }
    __syncthreads();

    const int pitch = r_k * 5 / 8;
    const int ppr = pitch >> 4;            // 16-byte pieces per row
    const int pieces = 32 * ppr;           // per tile
    const unsigned char *Ab = Aq + (size_t)b * L * pitch;
    const size_t seq_last = (size_t)L * pitch - 16;  // last piece of the sequence: requests beyond it are redirected
    const int n_tiles = (L + 31) / 32;
    const int tile_begin = blockIdx.x * tiles_per_wg;
    const int tile_end = tile_begin + tiles_per_wg < n_tiles ? tile_begin + tiles_per_wg : n_tiles;
    int tile = tile_begin + w;
    if (tile >= tile_end) return;
    // where this lane's pieces go in the LDS tile (the same for every tile); -1: no such piece
    int dst_off[kQ4MaxLoads];
#pragma unroll
    for (int i = 0; i < kQ4MaxLoads; ++i) {
        const int pc = i * 64 + lane;
        dst_off[i] = pc < pieces ? (pc / ppr) * tpitch + (pc % ppr) * 16 : -1;
    }
    u32x4_t stage[kQ4MaxLoads];
#define XKV_Q4_REQUEST(TL)                                                                              \
    _Pragma("unroll") for (int i = 0; i < kQ4MaxLoads; ++i)                                             \
    {                                                                                                   \
        const size_t off = (size_t)(TL) * 32 * pitch + (size_t)(i * 64 + lane) * 16;                    \
        stage[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(Ab + (off < seq_last ? off : seq_last))); \
    }
    XKV_Q4_REQUEST(tile);
    f32x16_t tot;
#pragma unroll
    for (int v = 0; v < 16; ++v) tot[v] = 0.0f;
    const f32x16_t zero = tot;
    const unsigned char *my_row = tile_lds + n * tpitch;
    constexpr int kQ4Burst = 4;
    float res[kQ4Burst][16];
#pragma unroll
    for (int i = 0; i < kQ4Burst; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) res[i][v] = 0.0f;
    int ti = 0, tile0 = tile;  // tiles held in res, first of them
    while (true) {
#pragma unroll
        for (int i = 0; i < kQ4MaxLoads; ++i)
            if (dst_off[i] >= 0) *reinterpret_cast<u32x4_t *>(tile_lds + dst_off[i]) = stage[i];
        const int tile_n = tile + WAVES;
        XKV_Q4_REQUEST(tile_n < tile_end ? tile_n : tile);
        for (int ps = 0; ps < n_pass; ++ps) {
            // (lo - 128 step) of this half's eight groups of the pass, split like Ps
            const u32x4_t *par = reinterpret_cast<const u32x4_t *>(my_row + (r_k >> 1) + 64 * ps + 32 * hf);
            const u32x4_t pa = par[0], pb = par[1];
            u32x4_t c3[3];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                uint32_t part[2][3];
#pragma unroll
                for (int o = 0; o < 2; ++o) {
                    const int e = 2 * e2 + o;
                    const uint32_t pword = e < 4 ? pa[e & 3] : pb[e & 3];
                    float v = fmaf(-128.0f, __uint_as_float(pword << 16), __uint_as_float(pword & 0xFFFF0000u));
                    v = 16 * ps + 8 * hf + e < n_groups ? v : 0.0f;  // beyond the row: whatever the tile holds there
#pragma unroll
                    for (int q3 = 0; q3 < 3; ++q3) {
                        part[o][q3] = __float_as_uint(v) & 0xFFFF0000u;
                        v -= __uint_as_float(part[o][q3]);
                    }
                }
#pragma unroll
                for (int q3 = 0; q3 < 3; ++q3) c3[q3][e2] = (part[0][q3] >> 16) | part[1][q3];
            }
            const u32x4_t *pf = PsF + ps * 3 * 64 + lane;
            const bf16x8_t p0 = __builtin_bit_cast(bf16x8_t, pf[0]), p1 = __builtin_bit_cast(bf16x8_t, pf[64]);
            const bf16x8_t p2 = __builtin_bit_cast(bf16x8_t, pf[128]);
            const bf16x8_t c0 = __builtin_bit_cast(bf16x8_t, c3[0]), c1 = __builtin_bit_cast(bf16x8_t, c3[1]);
            const bf16x8_t c2v = __builtin_bit_cast(bf16x8_t, c3[2]);
            // smallest products first
            tot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p1, c1, tot, 0, 0, 0);
            tot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p2, c0, tot, 0, 0, 0);
            tot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p0, c2v, tot, 0, 0, 0);
            tot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p1, c0, tot, 0, 0, 0);
            tot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p0, c1, tot, 0, 0, 0);
            tot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p0, c0, tot, 0, 0, 0);
        }
        for (int g = 0; g < n_groups; ++g) {
            const u32x4_t cw = *reinterpret_cast<const u32x4_t *>(my_row + 16 * g);
            const uint32_t pword = *reinterpret_cast<const uint32_t *>(my_row + (r_k >> 1) + 4 * g);
            f32x16_t acc = zero;
#pragma unroll
            for (int ff = 0; ff < 2; ++ff) {
                const uint32_t word = hf ? (ff ? cw[3] : cw[1]) : (ff ? cw[2] : cw[0]);
                const bf16x8_t bop = q4_fragment(word);
                const u32x4_t ph = Pl[(2 * g + ff) * 64 + lane];
                const u32x4_t pl = Pl[(F8 + 2 * g + ff) * 64 + lane];
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ph), bop, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, pl), bop, acc, 0, 0, 0);
            }
            const float step = __uint_as_float(pword << 16);
#pragma unroll
            for (int v = 0; v < 16; ++v) tot[v] = fmaf(step, acc[v], tot[v]);
        }
        // results wait in registers and are written in bursts of kQ4Burst tiles (as in the bf16 stream kernel:
        // stores dribbled out between the reads cost the memory system more than their bytes)
#pragma unroll
        for (int i = 0; i < kQ4Burst; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) res[i][v] = (i == ti) ? scale * tot[v] : res[i][v];
        ++ti;
#pragma unroll
        for (int v = 0; v < 16; ++v) tot[v] = 0.0f;
        const bool done = tile_n >= tile_end;
        if (ti == kQ4Burst || done) {
#pragma unroll
            for (int i = 0; i < kQ4Burst; ++i) {
                const int t = (tile0 + i * WAVES) * 32 + n;
                if (i < ti && t < L) {
#pragma unroll
                    for (int u = 0; u < GPH; ++u) {
                        const int g = blk * 2 * GPH + hf * GPH + u;
                        if (g < H_kv) {
                            float hv[16];
#pragma unroll
                            for (int hh = 0; hh < 16; ++hh) hv[hh] = hh < N_REP ? res[i][(u * N_REP + hh) & 15] : 0.0f;
                            float best = hv[0];
#pragma unroll
                            for (int hh = 1; hh < N_REP; ++hh) best = fmaxf(best, hv[hh]);
                            S[((size_t)b * H_kv + g) * L + t] = best;
                            float *dst = S_heads + (((size_t)b * H_kv + g) * L + t) * NRP;
                            if constexpr (NRP >= 4) {
#pragma unroll
                                for (int c = 0; c < NRP / 4; ++c)
                                    *reinterpret_cast<float4 *>(dst + 4 * c) =
                                        make_float4(hv[4 * c], hv[4 * c + 1], hv[4 * c + 2], hv[4 * c + 3]);
                            } else {
#pragma unroll
                                for (int hh = 0; hh < NRP; ++hh) dst[hh] = hv[hh];
                            }
                        }
                    }
                }
            }
            tile0 += ti * WAVES;
            ti = 0;
        }
        if (done) break;
        tile = tile_n;
    }
#undef XKV_Q4_REQUEST
}

static bool score_mfma_ok(const xkv_shape &s, const void *A_k)
{
    const int n_rep = s.H_q / s.H_kv;
    const bool rep_ok = (n_rep >= 1 && n_rep <= 8) || n_rep == 16;
    return s.dtype == XKV_BF16 && rep_ok && s.r_k % 16 == 0 && s.d_h % 16 == 0 && (((uintptr_t)A_k) & 15u) == 0 &&
           s.r_k <= 2048;
}

static hipError_t launch_score_generic(const xkv_shape &s, const Plan &p, int layer, const void *A_k,
                                       const void *B_k, const void *q, float *P, float *S, float *S_heads,
                                       hipStream_t st)
{
    dim3 pgrid((s.r_k * s.H_kv + 3) / 4, s.batch), grid((s.L + 255) / 256, s.batch), block(256);
    if (S_heads) {
        const int nrp = head_pitch(s.H_q / s.H_kv);
        if (s.dtype == XKV_F32) {
            hipLaunchKernelGGL(project_q_kernel<float>, pgrid, block, 0, st, (const float *)B_k, (const float *)q, P,
                               s.G, layer, s.r_k, s.H_kv, s.H_q, s.d_h);
            profile_begin(0, st);
            hipLaunchKernelGGL(score_heads_generic_kernel<float>, grid, block, 0, st, (const float *)A_k, P, S, S_heads,
                               s.L, s.r_k, s.H_kv, s.H_q, nrp, p.scale);
            profile_end(0, st);
        } else {
            hipLaunchKernelGGL(project_q_kernel<bf16_t>, pgrid, block, 0, st, (const bf16_t *)B_k, (const bf16_t *)q,
                               P, s.G, layer, s.r_k, s.H_kv, s.H_q, s.d_h);
            profile_begin(0, st);
            hipLaunchKernelGGL(score_heads_generic_kernel<bf16_t>, grid, block, 0, st, (const bf16_t *)A_k, P, S,
                               S_heads, s.L, s.r_k, s.H_kv, s.H_q, nrp, p.scale);
            profile_end(0, st);
        }
        return hipGetLastError();
    }
    if (s.dtype == XKV_F32) {
        hipLaunchKernelGGL(project_q_kernel<float>, pgrid, block, 0, st, (const float *)B_k, (const float *)q, P, s.G,
                           layer, s.r_k, s.H_kv, s.H_q, s.d_h);
        profile_begin(0, st);
        hipLaunchKernelGGL(score_generic_kernel<float>, grid, block, 0, st, (const float *)A_k, P, S, s.L, s.r_k,
                           s.H_kv, s.H_q, p.scale);
        profile_end(0, st);
    } else {
        hipLaunchKernelGGL(project_q_kernel<bf16_t>, pgrid, block, 0, st, (const bf16_t *)B_k, (const bf16_t *)q, P,
                           s.G, layer, s.r_k, s.H_kv, s.H_q, s.d_h);
        profile_begin(0, st);
        hipLaunchKernelGGL(score_generic_kernel<bf16_t>, grid, block, 0, st, (const bf16_t *)A_k, P, S, s.L, s.r_k,
                           s.H_kv, s.H_q, p.scale);
        profile_end(0, st);
    }
    return hipGetLastError();
}

// Whether a shape goes to the long-stream kernel, with how many 32-token tiles per workgroup, and whether its
// LDS also has room for the top-digit histograms.  One 8-wavefront workgroup per compute unit in a single
// round; every wavefront gets at least 8 tiles of its own.
bool score_stream_plan(const xkv_shape &s, int *tiles_per_wg, bool *hist_fits, int *waves)
{
    *tiles_per_wg = 0;
    *hist_fits = false;
    *waves = 0;
    if (s.H_kv <= 0 || s.H_q % s.H_kv != 0) return false;
    const int n_rep = s.H_q / s.H_kv;
    const bool rep_ok = (n_rep >= 1 && n_rep <= 8) || n_rep == 16;
    if (s.dtype != XKV_BF16 || !rep_ok || s.r_k % 16 != 0 || s.d_h % 16 != 0 || s.r_k > 2048) return false;
    const int F8 = (s.r_k / 16 + 7) / 8 * 8;
    const int n_tiles = (s.L + 31) / 32;
    const int pairs = s.batch * mfma_blocks(s.H_kv, n_rep);
    if ((long long)pairs * n_tiles < 256LL * kScoreWaves * 8) return false;
    const size_t lds_max = 160 * 1024 - 512, lds_p = (size_t)2 * F8 * 64 * 16;
    const size_t lds_hist = (size_t)2 * mfma_gph(n_rep) * kTopkBins * 4;
    int wv = kScoreWaves;
    if (lds_p + (size_t)wv * 512 * 16 > lds_max) wv = 4;
    if (lds_p + (size_t)wv * 512 * 16 > lds_max) return false;
    const int wgs = pairs >= 256 ? 1 : 256 / pairs;
    const int tpw = (n_tiles + wgs - 1) / wgs;
    *tiles_per_wg = (tpw + kScoreWaves - 1) / kScoreWaves * kScoreWaves;
    *hist_fits = lds_p + (size_t)wv * 512 * 16 + lds_hist <= lds_max;
    *waves = wv;
    return true;
}

// The long-stream kernel, with or without the per-head output (S_heads only read when HEADS).
template <int N_REP, int WAVES, bool HEADS>
static hipError_t launch_score_stream_t(const xkv_shape &s, const Plan &p, const bf16_t *A_k, const bf16_t *Pfrag,
                                        float *S, int F8, dim3 sgrid, size_t lds_stream, uint32_t *row_hist,
                                        uint32_t *chunk_hist, float *S_heads, hipStream_t st)
{
    static DynamicLdsOnce attr;
    if (hipError_t e0 = attr.ensure((const void *)score_stream_kernel<N_REP, WAVES, HEADS>, 160 * 1024 - 512); e0 != hipSuccess)
        return e0;
    profile_begin(0, st);
    hipLaunchKernelGGL((score_stream_kernel<N_REP, WAVES, HEADS>), sgrid, dim3(WAVES * 64), lds_stream, st, A_k, Pfrag, S,
                       s.L, s.r_k, s.H_kv, F8, p.score_tpw, p.scale, row_hist, chunk_hist, S_heads);
    profile_end(0, st);
    return hipGetLastError();
}

template <int N_REP>
static hipError_t launch_score_mfma_t(const xkv_shape &s, const Plan &p, const bf16_t *A_k, const bf16_t *Pfrag,
                                      float *S, int F8, uint32_t *row_hist, uint32_t *chunk_hist, bool *hist_done,
                                      float *S_heads, hipStream_t st)
{
    const int nblk = mfma_blocks(s.H_kv, N_REP);
    const int n_tiles = (s.L + 31) / 32;
    const size_t lds = (size_t)2 * F8 * 64 * 16;
    if (p.score_stream) {
        const bool with_hist = p.score_hist && row_hist && chunk_hist;
        const size_t lds_stream = lds + (size_t)p.score_waves * 512 * 16 +
                                  (with_hist ? (size_t)2 * mfma_gph(N_REP) * kTopkBins * 4 : 0);
        dim3 sgrid((n_tiles + p.score_tpw - 1) / p.score_tpw, nblk, s.batch);
        uint32_t *rh = with_hist ? row_hist : nullptr, *ch = with_hist ? chunk_hist : nullptr;
        hipError_t e;
        if (p.score_waves == kScoreWaves)
            e = S_heads ? launch_score_stream_t<N_REP, kScoreWaves, true>(s, p, A_k, Pfrag, S, F8, sgrid, lds_stream, rh,
                                                                          ch, S_heads, st)
                        : launch_score_stream_t<N_REP, kScoreWaves, false>(s, p, A_k, Pfrag, S, F8, sgrid, lds_stream,
                                                                           rh, ch, nullptr, st);
        else
            e = S_heads ? launch_score_stream_t<N_REP, 4, true>(s, p, A_k, Pfrag, S, F8, sgrid, lds_stream, rh, ch,
                                                                S_heads, st)
                        : launch_score_stream_t<N_REP, 4, false>(s, p, A_k, Pfrag, S, F8, sgrid, lds_stream, rh, ch,
                                                                 nullptr, st);
        if (e != hipSuccess) return e;
        if (hist_done) *hist_done = with_hist;
        return hipSuccess;
    }
    // about two workgroups per compute unit in a single round, each streaming one contiguous range of a
    // sequence (staging P costs a fixed 2 KiB per rank-16 fragment, so fewer, longer workgroups win)
    const int pairs = s.batch * nblk;
    const int wgs_per_pair = pairs >= 512 ? 1 : 512 / pairs;
    int tiles_per_wg = (n_tiles + wgs_per_pair - 1) / wgs_per_pair;
    tiles_per_wg = tiles_per_wg < 4 ? 4 : tiles_per_wg;
    tiles_per_wg = (tiles_per_wg + 3) / 4 * 4;
    static DynamicLdsOnce attr_pooled, attr_heads;
    if (hipError_t e0 = attr_pooled.ensure((const void *)score_mfma_kernel<N_REP, false>, 160 * 1024 - 512); e0 != hipSuccess)
        return e0;
    if (hipError_t e0 = attr_heads.ensure((const void *)score_mfma_kernel<N_REP, true>, 160 * 1024 - 512); e0 != hipSuccess)
        return e0;
    dim3 grid((n_tiles + tiles_per_wg - 1) / tiles_per_wg, nblk, s.batch), block(256);
    profile_begin(0, st);
    if (S_heads)
        hipLaunchKernelGGL((score_mfma_kernel<N_REP, true>), grid, block, lds, st, A_k, Pfrag, S, s.L, s.r_k, s.H_kv, F8,
                           tiles_per_wg, p.scale, S_heads);
    else
        hipLaunchKernelGGL((score_mfma_kernel<N_REP, false>), grid, block, lds, st, A_k, Pfrag, S, s.L, s.r_k, s.H_kv, F8,
                           tiles_per_wg, p.scale, (float *)nullptr);
    profile_end(0, st);
    return hipGetLastError();
}

bool score_stage_uses_mfma(const xkv_shape &s, const void *A_k, const void *B_k, const void *q, const void *P_ws,
                           const float *S_heads)
{
    return score_mfma_ok(s, A_k) && ((((uintptr_t)B_k | (uintptr_t)q | (uintptr_t)P_ws)) & 15u) == 0 &&
           (!S_heads || (((uintptr_t)S_heads) & 15u) == 0);
}

hipError_t launch_score_stage(const xkv_shape &s, const Plan &p, int layer, const void *A_k, const void *B_k,
                              const void *q, void *P_ws, float *S, uint32_t *row_hist, uint32_t *chunk_hist,
                              bool *hist_done, const PackArgs *fuse_pack, bool *packed_done, hipStream_t st,
                              float *S_heads)
{
    if (hist_done) *hist_done = false;
    if (packed_done) *packed_done = false;
    // per-head scores come from either matrix-core kernel, or from the general one
    const bool mfma = score_stage_uses_mfma(s, A_k, B_k, q, P_ws, S_heads);
    if (!mfma && !B_k) return hipErrorInvalidValue;  // only the matrix-core projection generates an identity B_l
    if (!mfma) return launch_score_generic(s, p, layer, A_k, B_k, q, (float *)P_ws, S, S_heads, st);
    const int n_rep = s.H_q / s.H_kv;
    const int F8 = (s.r_k / 16 + 7) / 8 * 8;
    const int gph = mfma_gph(n_rep), nblk = mfma_blocks(s.H_kv, n_rep);
    bf16_t *Pfrag = (bf16_t *)P_ws;
    ProjArgs pj;
    pj.B_k = (const bf16_t *)B_k;
    pj.q = (const bf16_t *)q;
    pj.Pfrag = Pfrag;
    pj.G = s.G;
    pj.layer = layer;
    pj.r_k = s.r_k;
    pj.H_kv = s.H_kv;
    pj.H_q = s.H_q;
    pj.d_h = s.d_h;
    pj.F8 = F8;
    pj.blocks_x = ((F8 / 2) * 2 * gph * nblk + 3) / 4;
    // the row histograms of the top-k stage are cleared in the same launch when the score kernel will add to them
    const bool zero_hist = p.score_stream && p.score_hist && row_hist && chunk_hist;
    const int zero_words = zero_hist ? p.rows * kTopkLevels * kTopkBins : 0;  // a multiple of 1024
    if (fuse_pack || zero_hist) {
        const int n_proj = pj.blocks_x * s.batch;
        const int n_pack = fuse_pack ? (fuse_pack->blocks_per_head + kPackQBlocks) * fuse_pack->H_kv * fuse_pack->batch : 0;
        hipLaunchKernelGGL(prepass_kernel, dim3(n_proj + n_pack + zero_words / 1024), dim3(256), 0, st, pj,
                           fuse_pack ? *fuse_pack : PackArgs{}, n_proj, n_pack, row_hist, zero_words);
        if (packed_done) *packed_done = fuse_pack != nullptr;
    } else {
        hipLaunchKernelGGL(project_q_frag_kernel, dim3(pj.blocks_x, s.batch), dim3(256), 0, st, pj);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const bf16_t *A = (const bf16_t *)A_k;
    switch (n_rep) {
    case 1: return launch_score_mfma_t<1>(s, p, A, Pfrag, S, F8, row_hist, chunk_hist, hist_done, S_heads, st);
    case 2: return launch_score_mfma_t<2>(s, p, A, Pfrag, S, F8, row_hist, chunk_hist, hist_done, S_heads, st);
    case 3: return launch_score_mfma_t<3>(s, p, A, Pfrag, S, F8, row_hist, chunk_hist, hist_done, S_heads, st);
    case 4: return launch_score_mfma_t<4>(s, p, A, Pfrag, S, F8, row_hist, chunk_hist, hist_done, S_heads, st);
    case 5: return launch_score_mfma_t<5>(s, p, A, Pfrag, S, F8, row_hist, chunk_hist, hist_done, S_heads, st);
    case 6: return launch_score_mfma_t<6>(s, p, A, Pfrag, S, F8, row_hist, chunk_hist, hist_done, S_heads, st);
    case 7: return launch_score_mfma_t<7>(s, p, A, Pfrag, S, F8, row_hist, chunk_hist, hist_done, S_heads, st);
    case 8: return launch_score_mfma_t<8>(s, p, A, Pfrag, S, F8, row_hist, chunk_hist, hist_done, S_heads, st);
    default: return launch_score_mfma_t<16>(s, p, A, Pfrag, S, F8, row_hist, chunk_hist, hist_done, S_heads, st);
    }
}

// The line-wise kernel (eight wavefronts, one workgroup per compute unit) whenever its LDS fits -- ranks up to 512 --
// else the kernel with one lane per row (four wavefronts, long passes).
template <int N_REP>
static hipError_t launch_score_q4_t(const xkv_shape &s, const Plan &p, const unsigned char *Aq, const bf16_t *Pfrag, float *S,
                                    float *S_heads, int F8, hipStream_t st)
{
    const int nblk = mfma_blocks(s.H_kv, N_REP);
    const int n_tiles = (s.L + 31) / 32;
    const size_t lds = (size_t)2 * F8 * 64 * 16 + (size_t)(F8 / 2) * 32 * 4;
    const size_t lds_tile = lds + (size_t)((F8 / 2 + 15) / 16) * 3 * 64 * 16 +
                            (size_t)kQ4TileWaves * (32 * q4_tile_pitch(s.r_k) + kQ4TileSlack);
    const bool tiled = lds_tile <= 160 * 1024 - 512 && 32 * (s.r_k * 5 / 8) <= kQ4MaxLoads * 1024;
    const int waves = tiled ? kQ4TileWaves : 4;
    // one (line-wise) or two workgroups per compute unit, each over one contiguous range of a sequence
    const int pairs = s.batch * nblk;
    const int want = tiled ? 256 : 512;
    const int wgs_per_pair = pairs >= want ? 1 : want / pairs;
    int tiles_per_wg = (n_tiles + wgs_per_pair - 1) / wgs_per_pair;
    tiles_per_wg = tiles_per_wg < waves ? waves : (tiles_per_wg + waves - 1) / waves * waves;
    dim3 grid((n_tiles + tiles_per_wg - 1) / tiles_per_wg, nblk, s.batch);
    hipError_t e = hipSuccess;
    if (tiled) {
        static DynamicLdsOnce attr8;
        e = attr8.ensure((const void *)score_q4_tile_kernel<N_REP>, 160 * 1024 - 512);
        if (e != hipSuccess) return e;
        profile_begin(0, st);
        hipLaunchKernelGGL((score_q4_tile_kernel<N_REP>), grid, dim3(kQ4TileWaves * 64), lds_tile, st, Aq, Pfrag, S, S_heads,
                           s.L, s.r_k, s.H_kv, F8, tiles_per_wg, p.scale);
        profile_end(0, st);
    } else {
        static DynamicLdsOnce attr4;
        e = attr4.ensure((const void *)score_q4_kernel<N_REP, 4, 16>, 160 * 1024 - 512);
        if (e != hipSuccess) return e;
        profile_begin(0, st);
        hipLaunchKernelGGL((score_q4_kernel<N_REP, 4, 16>), grid, dim3(256), lds, st, Aq, Pfrag, S, S_heads, s.L, s.r_k,
                           s.H_kv, F8, tiles_per_wg, p.scale);
        profile_end(0, st);
    }
    return hipGetLastError();
}

bool score_q4_shape_ok(const xkv_shape &s)
{
    if (s.H_kv <= 0 || s.H_q % s.H_kv != 0) return false;
    const int n_rep = s.H_q / s.H_kv;
    const bool rep_ok = (n_rep >= 1 && n_rep <= 8) || n_rep == 16;
    return s.dtype == XKV_BF16 && rep_ok && s.r_k > 0 && s.r_k % 128 == 0 && s.r_k <= 2048 && s.d_h % 16 == 0;
}

// Projection (as for the bf16 stream) and the score kernel over quantised rows; S and S_heads are both written.
hipError_t launch_score_q4_stage(const xkv_shape &s, const Plan &p, int layer, const void *Aq_k, const void *B_k,
                                 const void *q, void *P_ws, float *S, float *S_heads, hipStream_t st)
{
    const int n_rep = s.H_q / s.H_kv;
    const int F8 = (s.r_k / 16 + 7) / 8 * 8;
    const int gph = mfma_gph(n_rep), nblk = mfma_blocks(s.H_kv, n_rep);
    bf16_t *Pfrag = (bf16_t *)P_ws;
    ProjArgs pj;
    pj.B_k = (const bf16_t *)B_k;
    pj.q = (const bf16_t *)q;
    pj.Pfrag = Pfrag;
    pj.G = s.G;
    pj.layer = layer;
    pj.r_k = s.r_k;
    pj.H_kv = s.H_kv;
    pj.H_q = s.H_q;
    pj.d_h = s.d_h;
    pj.F8 = F8;
    pj.blocks_x = ((F8 / 2) * 2 * gph * nblk + 3) / 4;
    hipLaunchKernelGGL(project_q_frag_kernel, dim3(pj.blocks_x, s.batch), dim3(256), 0, st, pj);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const unsigned char *A = (const unsigned char *)Aq_k;
    switch (n_rep) {
    case 1: return launch_score_q4_t<1>(s, p, A, Pfrag, S, S_heads, F8, st);
    case 2: return launch_score_q4_t<2>(s, p, A, Pfrag, S, S_heads, F8, st);
    case 3: return launch_score_q4_t<3>(s, p, A, Pfrag, S, S_heads, F8, st);
    case 4: return launch_score_q4_t<4>(s, p, A, Pfrag, S, S_heads, F8, st);
    case 5: return launch_score_q4_t<5>(s, p, A, Pfrag, S, S_heads, F8, st);
    case 6: return launch_score_q4_t<6>(s, p, A, Pfrag, S, S_heads, F8, st);
    case 7: return launch_score_q4_t<7>(s, p, A, Pfrag, S, S_heads, F8, st);
    case 8: return launch_score_q4_t<8>(s, p, A, Pfrag, S, S_heads, F8, st);
    default: return launch_score_q4_t<16>(s, p, A, Pfrag, S, S_heads, F8, st);
    }
}

}  // namespace xkv
