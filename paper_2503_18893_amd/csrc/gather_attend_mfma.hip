// bf16 matrix-core path of selective reconstruction + sparse attention (Sec. 3.2, Eq. 3):
//   K^_g = A^K[I_g,:] B^K_{l,g},  V^_g = A^V[I_g,:] B^V_{l,g},  out_h = softmax(scale K^_g q_h)^T V^_g.
//
// Everything is one chain of v_mfma_f32_32x32x16_bf16 whose operand layouts are chosen so that the
// result registers of one product are, after a bf16 pack, directly the operand of the next:
//   (1) K^T tile [dims x tokens]  = B^K_g^T (LDS fragment)  x  gathered rows of A^K (global, 16 B/lane)
//   (2) Z^T [tokens x head slots] = K^ (registers of (1))   x  Q^T fragments (registers)
//   (3) V^ tile [tokens x dims]   = gathered rows of A^V    x  B^V_g (LDS fragment)
//   (4) O [head slots x dims]    += W = exp(Z^T - max) (registers of (2))  x  V^ (registers of (3))
// In a 32x32 result lane (n, hf) holds column n and rows 8(v/4) + 4hf + v%4, v = 0..15; eight
// consecutive registers are a valid 16-deep operand fragment for the next product because both of
// its operands then agree on which row sits at which position.  Nothing is staged for a transpose.
//
// A wavefront owns 64 selected tokens per iteration (two 32-token blocks), a workgroup 256; the
// reconstruction matrices are pre-packed into fragment order (pack_b_kernel) and streamed through
// LDS 64 ranks at a time, shared by the four wavefronts.  Each wavefront keeps its own online
// softmax state and writes one partial per query head; combine_kernel merges them.
#include <type_traits>

#include "xkv_common.h"

namespace xkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) float f32x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

constexpr int kMaxChunkTokens = 8192;  // selected tokens per workgroup (their ids sit in LDS)
constexpr int kGroup = 8;  // fragments (of 16 ranks) per LDS stage: 8 x 4 KiB = 32 KiB, double-buffered

// Pack B_{l,g} (r x 128 slice of B_l) into MFMA fragment order:
//   pack[f][db][hf*32 + c][e] = B[16f + 8hf + e][g*128 + db*32 + c],  zero beyond r.
// Output per (sequence, KV head): F8k fragment rows for K then F8v for V, 4 KiB each, F8 = roundup(r/16, 8).
__global__ __launch_bounds__(256) void pack_b_kernel(const bf16_t *__restrict__ B_k, const bf16_t *__restrict__ B_v,
                                                     u32x4_t *__restrict__ pack, int G, int layer, int r_k, int r_v,
                                                     int H_kv, int F8k, int F8v)
{
    // one thread per (fragment f, half hf, dim block db, 4 columns): 8 rows x 8 B in, 4 lanes' 16 B pieces out
    const int g = blockIdx.y, b = blockIdx.z;
    const int d = H_kv * 128;
    const int item = blockIdx.x * 256 + threadIdx.x;
    if (item >= (F8k + F8v) * 64) return;
    const int c4 = item & 7, db = (item >> 3) & 3, hf = (item >> 5) & 1, fa = item >> 6;
    const bool is_v = fa >= F8k;
    const int f = is_v ? fa - F8k : fa;
    const int r = is_v ? r_v : r_k;
    const bf16_t *src = (is_v ? B_v : B_k) + ((size_t)b * G + layer) * r * d + (size_t)g * 128 + db * 32 + c4 * 4;
    uint64_t wd[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int i = 16 * f + 8 * hf + e;
        wd[e] = i < r ? *reinterpret_cast<const uint64_t *>(src + (size_t)i * d) : 0ull;
    }
    u32x4_t *dst = pack + ((size_t)b * H_kv + g) * (size_t)(F8k + F8v) * 256 + (size_t)(fa * 4 + db) * 64 + hf * 32 +
                   c4 * 4;
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
        u32x4_t o;
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const uint32_t lo = (uint32_t)(wd[2 * e2] >> (16 * cc)) & 0xFFFFu;
            const uint32_t hi = (uint32_t)(wd[2 * e2 + 1] >> (16 * cc)) & 0xFFFFu;
            o[e2] = lo | (hi << 16);
        }
        dst[cc] = o;
    }
}

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t &c, int j)
{
    f32x8_t x;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = c[8 * j + e];
    return __builtin_convertvector(x, bf16x8_t);
}

// One group of 8 fragment steps.  IS_K selects which product the fragments feed.
// While the group is multiplied out of LDS buffer gg%2, the thread writes its slice of group gg+1's B
// fragments (loaded one group earlier) into the other buffer, loads its slice of group gg+2 (bsrc2),
// and loads the A pieces its lane needs in group gg+1 (rows an0/an1, fragments fn0.. of Fn).
template <bool IS_K>
__device__ __forceinline__ void run_group(f32x16_t (&acc)[2][4], u32x4_t (&areg)[kGroup][2], u32x4_t (&breg)[kGroup],
                                          u32x4_t *Bl, const u32x4_t *bsrc2, int gg, int NG, const u32x4_t *an0,
                                          const u32x4_t *an1, int fn0, int Fn, int tid, int lane)
{
    // Buffer gg%2 is complete and nobody still reads buffer (gg+1)%2.  The barrier orders LDS traffic only:
    // the global loads in flight are this thread's own prefetch and must stay in flight across it.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    // Past the last group the "next" sources wrap around to valid memory (the packed B of the first groups,
    // clamped token rows), so every load and LDS write below is unconditional: the group is one straight
    // line of code and the wait counters stay exact.
    (void)NG;
    u32x4_t *bdst = Bl + ((gg + 1) & 1) * (kGroup * 256) + tid;
    const u32x4_t *bcur = Bl + (gg & 1) * (kGroup * 256) + lane;
    u32x4_t bf_cur[4], bf_nxt[4];
#pragma unroll
    for (int db = 0; db < 4; ++db) bf_cur[db] = bcur[db * 64];
#pragma unroll
    for (int fl = 0; fl < kGroup; ++fl) {
        bdst[fl * 256] = breg[fl];
        breg[fl] = bsrc2[fl * 256];
        const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, areg[fl][0]);
        const bf16x8_t a1 = __builtin_bit_cast(bf16x8_t, areg[fl][1]);
        if (fl + 1 < kGroup) {
#pragma unroll
            for (int db = 0; db < 4; ++db) bf_nxt[db] = bcur[((fl + 1) * 4 + db) * 64];  // LDS reads one step ahead
        }
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const bf16x8_t bf = __builtin_bit_cast(bf16x8_t, bf_cur[db]);
            if constexpr (IS_K) {  // (1) K^T tile: rows = head dims, columns = tokens
                acc[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, a0, acc[0][db], 0, 0, 0);
                acc[1][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, a1, acc[1][db], 0, 0, 0);
            } else {  // (3) V^ tile: rows = tokens, columns = head dims
                acc[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bf, acc[0][db], 0, 0, 0);
                acc[1][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bf, acc[1][db], 0, 0, 0);
            }
        }
#pragma unroll
        for (int db = 0; db < 4; ++db) bf_cur[db] = bf_nxt[db];
        // the lane's A pieces for the same step of the next group, loaded into the registers just consumed
        const int f = fn0 + fl < Fn ? fn0 + fl : 0;
        areg[fl][0] = an0[2 * f];
        areg[fl][1] = an1[2 * f];
        __builtin_amdgcn_sched_barrier(0);  // keep each step's loads where they are written: they are the prefetch
    }
}

// Software pipeline.  The work of a workgroup is a linear sequence of groups of 8 fragment steps:
// per 256-token tile first the K groups, then the V groups.  While group gg is multiplied out of LDS
// buffer gg%2, every thread (a) writes into the other buffer the slice of group gg+1's B fragments it
// loaded one group earlier and loads its slice of group gg+2, and (b) loads, one group ahead, the 16 B
// pieces of the gathered A rows its own lane will need.  One barrier per group.
__global__ __launch_bounds__(256, 1) void gather_attend_mfma_kernel(
    const bf16_t *__restrict__ A_k, const bf16_t *__restrict__ A_v, const u32x4_t *__restrict__ pack,
    const bf16_t *__restrict__ q, const int32_t *__restrict__ idx, float *__restrict__ part_o,
    float *__restrict__ part_ml, int L, int r_k, int r_v, int H_kv, int H_q, int k, int splits, int chunk, int F8k,
    int F8v, float scale)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    u32x4_t *Bl = reinterpret_cast<u32x4_t *>(smem_raw);  // [2][kGroup][4][64] 16-byte fragments = 64 KiB
    // workgroup id -> (KV head fastest, so that a head's packed B stays in one XCD's L2), split, sequence
    const int g = blockIdx.x % H_kv;
    const int split = (blockIdx.x / H_kv) % splits;
    const int b = blockIdx.x / (H_kv * splits);
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int n = lane & 31, hf = lane >> 5;
    const int n_rep = H_q / H_kv;
    const int Fk = r_k / 16, Fv = r_v / 16;
    const int GK = F8k / kGroup, GT = (F8k + F8v) / kGroup;

    // Q^T fragments, kept in LDS (shared by the four wavefronts): lane (head slot n, hf), position e of
    // fragment (db, j) holds q[n][db*32 + 8(2j + e/4) + 4hf + e%4]
    u32x4_t *Ql = Bl + 2 * kGroup * 256;  // [8][64]
    if (w == 0) {
        const bf16_t *qh = q + ((size_t)b * H_q + (size_t)g * n_rep + (n < n_rep ? n : 0)) * 128;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                u32x4_t raw;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int e = 2 * e2;
                    const int dim = db * 32 + 8 * (2 * j + e / 4) + 4 * hf + e % 4;  // e and e+1 are adjacent dims
                    const uint32_t lo = n < n_rep ? qh[dim] : 0u, hi = n < n_rep ? qh[dim + 1] : 0u;
                    raw[e2] = lo | (hi << 16);
                }
                Ql[(db * 2 + j) * 64 + lane] = raw;
            }
    }

    const u32x4_t *packg = pack + ((size_t)b * H_kv + g) * (size_t)(F8k + F8v) * 256;
    const bf16_t *Ak = A_k + (size_t)b * L * r_k;
    const bf16_t *Av = A_v + (size_t)b * L * r_v;
    const int32_t *ids = idx + ((size_t)b * H_kv + g) * k;
    const int m_begin = split * chunk;
    const int m_end = m_begin + chunk < k ? m_begin + chunk : k;
    const int n_tiles = (m_end - m_begin + 255) / 256;
    const int NG = n_tiles * GT;

    // The split's token ids are staged in LDS once (clamped into [0, L)), so that the main loop issues no
    // global load other than its prefetches: a wait on an id would otherwise drain the whole prefetch queue.
    int *tok_lds = reinterpret_cast<int *>(Ql + 8 * 64);  // [chunk]
    for (int m = tid; m < m_end - m_begin; m += 256) {
        const int t = ids[m_begin + m];
        tok_lds[m] = t < 0 ? 0 : (t >= L ? L - 1 : t);
    }
    __syncthreads();
    // token ids gathered by this lane (both 32-token blocks) of a tile
    auto tile_tokens = [&](int tile, int (&tk)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            int m = tile * 256 + w * 64 + tb * 32 + n;
            m = m < m_end - m_begin ? m : m_end - m_begin - 1;
            tk[tb] = tok_lds[m];
        }
    };
    // 16-byte pieces of a gathered row, already offset by the lane's half
    auto krow = [&](int t) __attribute__((always_inline)) {
        return reinterpret_cast<const u32x4_t *>(Ak + (size_t)t * r_k) + hf;
    };
    auto vrow = [&](int t) __attribute__((always_inline)) {
        return reinterpret_cast<const u32x4_t *>(Av + (size_t)t * r_v) + hf;
    };
    int tok[2], tok_n[2];
    tile_tokens(0, tok);
    tile_tokens(n_tiles > 1 ? 1 : 0, tok_n);

    float m_run = -INFINITY, l_run = 0.0f;
    f32x16_t O[4], acc[2][4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) O[db][v] = acc[0][db][v] = acc[1][db][v] = 0.0f;
    bf16x8_t Wf[2][2];

    // ---- prologue: B group 0 straight into buffer 0, B group 1 into registers, A pieces of group 0
    u32x4_t breg[kGroup], areg[kGroup][2];
#pragma unroll
    for (int fl = 0; fl < kGroup; ++fl) Bl[fl * 256 + tid] = packg[fl * 256 + tid];
#pragma unroll
    for (int fl = 0; fl < kGroup; ++fl) {
        breg[fl] = packg[(size_t)((1 % GT) * kGroup + fl) * 256 + tid];
        const int f = fl < Fk ? fl : 0;  // beyond the rank the B fragment is zero: any finite A piece will do
        areg[fl][0] = krow(tok[0])[2 * f];
        areg[fl][1] = krow(tok[1])[2 * f];
        __builtin_amdgcn_sched_barrier(0);  // same issue order as in the steady state (keeps the wait counts exact)
    }

    int gg = 0;
    for (int tile = 0; tile < n_tiles; ++tile) {
        const int base = m_begin + tile * 256 + w * 64;
        for (int wi = 0; wi < GK; ++wi, ++gg) {
            const bool next_k = wi + 1 < GK;  // the group after this one: K or the first V group of this tile
            run_group<true>(acc, areg, breg, Bl, packg + (size_t)(((wi + 2) % GT) * kGroup) * 256 + tid, gg, NG,
                            next_k ? krow(tok[0]) : vrow(tok[0]), next_k ? krow(tok[1]) : vrow(tok[1]),
                            next_k ? (wi + 1) * kGroup : 0, next_k ? Fk : Fv, tid, lane);
        }
        {
            // (2) Z^T = K^ Q^T: lane (head slot n, hf), register v <-> token 8(v/4) + 4hf + v%4 of block tb
            f32x16_t Z[2];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) Z[tb][v] = 0.0f;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const bf16x8_t qf = __builtin_bit_cast(bf16x8_t, Ql[(db * 2 + j) * 64 + lane]);
                        Z[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pack8(acc[tb][db], j), qf, Z[tb], 0, 0, 0);
                    }
            }
            // online softmax; selected tokens beyond the end of this split get weight 0
            float m_loc = -INFINITY;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int tt = base + tb * 32 + 8 * (v / 4) + 4 * hf + (v % 4);
                    Z[tb][v] = tt < m_end ? scale * Z[tb][v] : -INFINITY;
                    m_loc = fmaxf(m_loc, Z[tb][v]);
                }
            m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32, kWave));
            const float m_new = fmaxf(m_run, m_loc);
            const float alpha = (m_new == -INFINITY) ? 1.0f : __expf(m_run - m_new);
            float l_add = 0.0f;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float wv = (Z[tb][v] == -INFINITY) ? 0.0f : __expf(Z[tb][v] - m_new);
                    Z[tb][v] = wv;
                    l_add += wv;
                }
                Wf[tb][0] = pack8(Z[tb], 0);
                Wf[tb][1] = pack8(Z[tb], 1);
            }
            l_run = l_run * alpha + l_add;
            m_run = m_new;
            // rescale O now: rows are head slots, register v of half hf is slot 8(v/4) + 4hf + v%4
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                const float a = __shfl(alpha, 8 * (v / 4) + 4 * hf + (v % 4), kWave);
#pragma unroll
                for (int db = 0; db < 4; ++db) O[db][v] *= a;
            }
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[tb][db][v] = 0.0f;
        }
        for (int wi = GK; wi < GT; ++wi, ++gg) {
            const bool wrap = wi + 1 == GT;  // the next group is the first K group of the next tile
            run_group<false>(acc, areg, breg, Bl, packg + (size_t)(((wi + 2) % GT) * kGroup) * 256 + tid, gg, NG,
                             wrap ? krow(tok_n[0]) : vrow(tok[0]), wrap ? krow(tok_n[1]) : vrow(tok[1]),
                             wrap ? 0 : (wi + 1 - GK) * kGroup, wrap ? Fk : Fv, tid, lane);
        }
        {
            // (4) O += W V^
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int db = 0; db < 4; ++db)
                        O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Wf[tb][j], pack8(acc[tb][db], j), O[db], 0, 0,
                                                                        0);
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[tb][db][v] = 0.0f;
            // rotate the token ids and fetch those of the tile after next
            tok[0] = tok_n[0];
            tok[1] = tok_n[1];
            tile_tokens(tile + 2 < n_tiles ? tile + 2 : n_tiles - 1, tok_n);
        }
    }

    // merge the four wavefronts in LDS, then write one partial per (split, query head)
    __syncthreads();
    float *mg = reinterpret_cast<float *>(smem_raw);  // [4][16][132]
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    if (lane < n_rep) {
        mg[(w * 16 + lane) * 132 + 128] = m_run;
        mg[(w * 16 + lane) * 132 + 129] = l_tot;
    }
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const int hh = 8 * (v / 4) + 4 * hf + (v % 4);
        if (hh < n_rep) {
#pragma unroll
            for (int db = 0; db < 4; ++db) mg[(w * 16 + hh) * 132 + db * 32 + n] = O[db][v];
        }
    }
    __syncthreads();
    for (int item = tid; item < n_rep * 128; item += 256) {
        const int hh = item >> 7, dim = item & 127;
        float M = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) M = fmaxf(M, mg[(ww * 16 + hh) * 132 + 128]);
        float num = 0.0f, den = 0.0f;
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) {
            const float mw = mg[(ww * 16 + hh) * 132 + 128];
            const float wgt = (mw == -INFINITY) ? 0.0f : __expf(mw - M);
            num = fmaf(wgt, mg[(ww * 16 + hh) * 132 + dim], num);
            den = fmaf(wgt, mg[(ww * 16 + hh) * 132 + 129], den);
        }
        const size_t slot = ((size_t)b * H_q + g * n_rep + hh) * splits + split;
        part_o[slot * 128 + dim] = num;
        if (dim == 0) {
            part_ml[slot * 2 + 0] = M;
            part_ml[slot * 2 + 1] = den;
        }
    }
}

bool gather_attend_mfma_shape_ok(const xkv_shape &s)
{
    return s.dtype == XKV_BF16 && s.d_h == 128 && s.r_k % 16 == 0 && s.r_v % 16 == 0;
}

size_t gather_attend_pack_bytes(const xkv_shape &s)
{
    const int F8k = (s.r_k / 16 + 7) / 8 * 8, F8v = (s.r_v / 16 + 7) / 8 * 8;
    return (size_t)(s.batch > 0 ? s.batch : 1) * s.H_kv * (size_t)(F8k + F8v) * 4 * 1024;
}

hipError_t launch_gather_attend_mfma(const xkv_shape &s, const Plan &p, int layer, const void *A_k, const void *A_v,
                                     const void *B_k, const void *B_v, const void *q, const int32_t *idx,
                                     void *pack_ws, float *part_o, float *part_ml, hipStream_t st)
{
    const int F8k = (s.r_k / 16 + 7) / 8 * 8, F8v = (s.r_v / 16 + 7) / 8 * 8;
    dim3 pgrid(((F8k + F8v) * 64 + 255) / 256, s.H_kv, s.batch), block(256);
    hipLaunchKernelGGL(pack_b_kernel, pgrid, block, 0, st, (const bf16_t *)B_k, (const bf16_t *)B_v,
                       (u32x4_t *)pack_ws, s.G, layer, s.r_k, s.r_v, s.H_kv, F8k, F8v);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t lds = 2 * kGroup * 256 * 16 + 8 * 64 * 16 + (size_t)p.sr_chunk * 4;  // B fragments, Q fragments, token ids
    static bool attr_set = false;
    if (!attr_set) {
        e = hipFuncSetAttribute((const void *)gather_attend_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                2 * kGroup * 256 * 16 + 8 * 64 * 16 + kMaxChunkTokens * 4);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)((long long)p.sr_splits * s.H_kv * s.batch));
    profile_begin(1, st);
    hipLaunchKernelGGL(gather_attend_mfma_kernel, grid, block, lds, st, (const bf16_t *)A_k, (const bf16_t *)A_v,
                       (const u32x4_t *)pack_ws, (const bf16_t *)q, idx, part_o, part_ml, s.L, s.r_k, s.r_v, s.H_kv,
                       s.H_q, s.k, p.sr_splits, p.sr_chunk, F8k, F8v, p.scale);
    profile_end(1, st);
    return hipGetLastError();
}

}  // namespace xkv
