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
#include "xkv_common.h"

namespace xkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) float f32x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

constexpr int kFragsPerChunk = 4;  // 64 ranks of B per LDS stage

// Pack B_{l,g} (r x 128 slice of B_l) into MFMA fragment order:
//   pack[f][db][hf*32 + c][e] = B[16f + 8hf + e][g*128 + db*32 + c],  zero beyond r.
// Output per (sequence, KV head, K|V): F4 * 4 fragments of 1 KiB, F4 = roundup(r/16, 4).
__global__ __launch_bounds__(256) void pack_b_kernel(const bf16_t *__restrict__ B_k, const bf16_t *__restrict__ B_v,
                                                     u32x4_t *__restrict__ pack, int G, int layer, int r_k, int r_v,
                                                     int H_kv, int F4k, int F4v)
{
    const int g = blockIdx.y, b = blockIdx.z;
    const int d = H_kv * 128;
    const int total = (F4k + F4v) * 4 * 64;
    u32x4_t *dst = pack + ((size_t)b * H_kv + g) * total;
    for (int e16 = blockIdx.x * 256 + threadIdx.x; e16 < total; e16 += gridDim.x * 256) {
        const bool is_v = e16 >= F4k * 4 * 64;
        const int loc = is_v ? e16 - F4k * 4 * 64 : e16;
        const int lane = loc % 64, db = (loc / 64) % 4, f = loc / 256;
        const int c = lane & 31, hf = lane >> 5;
        const int r = is_v ? r_v : r_k;
        const bf16_t *src = (is_v ? B_v : B_k) + ((size_t)b * G + layer) * r * d + (size_t)g * 128 + db * 32 + c;
        uint32_t wds[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const int i0 = 16 * f + 8 * hf + 2 * e2;
            const uint32_t lo = i0 < r ? src[(size_t)i0 * d] : 0u;
            const uint32_t hi = i0 + 1 < r ? src[(size_t)(i0 + 1) * d] : 0u;
            wds[e2] = lo | (hi << 16);
        }
        dst[e16] = u32x4_t{wds[0], wds[1], wds[2], wds[3]};
    }
}

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t &c, int j)
{
    f32x8_t x;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = c[8 * j + e];
    return __builtin_convertvector(x, bf16x8_t);
}

__global__ __launch_bounds__(256, 1) void gather_attend_mfma_kernel(
    const bf16_t *__restrict__ A_k, const bf16_t *__restrict__ A_v, const u32x4_t *__restrict__ pack,
    const bf16_t *__restrict__ q, const int32_t *__restrict__ idx, float *__restrict__ part_o,
    float *__restrict__ part_ml, int L, int r_k, int r_v, int H_kv, int H_q, int k, int splits, int chunk, int F4k,
    int F4v, float scale)
{
    __shared__ u32x4_t Bl[kFragsPerChunk * 4 * 64];  // 16 KiB
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = lane_id(), w = wave_id();
    const int n = lane & 31, hf = lane >> 5;
    const int n_rep = H_q / H_kv;
    const int Fk = r_k / 16, Fv = r_v / 16;

    // Q^T fragments: lane (head slot n, hf), position e of fragment (db, j) holds q[n][db*32 + 8(2j + e/4) + 4hf + e%4]
    bf16x8_t Qf[4][2];
    {
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
                Qf[db][j] = __builtin_bit_cast(bf16x8_t, raw);
            }
    }

    const u32x4_t *packK = pack + ((size_t)b * H_kv + g) * (size_t)(F4k + F4v) * 256;
    const u32x4_t *packV = packK + (size_t)F4k * 256;
    const bf16_t *Ak = A_k + (size_t)b * L * r_k;
    const bf16_t *Av = A_v + (size_t)b * L * r_v;
    const int32_t *ids = idx + ((size_t)b * H_kv + g) * k;
    const int m_begin = split * chunk;
    const int m_end = m_begin + chunk < k ? m_begin + chunk : k;

    float m_run = -INFINITY, l_run = 0.0f;
    f32x16_t O[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) O[db][v] = 0.0f;

    for (int tile0 = m_begin; tile0 < m_end; tile0 += 256) {  // uniform over the workgroup
        const int base = tile0 + w * 64;
        const u32x4_t *rowK[2], *rowV[2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            int m = base + tb * 32 + n;
            m = m < m_end ? m : m_end - 1;
            int t = ids[m];
            t = t < 0 ? 0 : (t >= L ? L - 1 : t);
            rowK[tb] = reinterpret_cast<const u32x4_t *>(Ak + (size_t)t * r_k) + hf;
            rowV[tb] = reinterpret_cast<const u32x4_t *>(Av + (size_t)t * r_v) + hf;
        }
        f32x16_t acc[2][4];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tb][db][v] = 0.0f;

        // (1) K^T tile: rows = head dims, columns = tokens
        for (int c0 = 0; c0 < F4k; c0 += kFragsPerChunk) {
            __syncthreads();
            for (int e = threadIdx.x; e < kFragsPerChunk * 256; e += 256) Bl[e] = packK[(size_t)c0 * 256 + e];
            __syncthreads();
#pragma unroll
            for (int fl = 0; fl < kFragsPerChunk; ++fl) {
                const int f = c0 + fl;
                if (f < Fk) {
                    const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, rowK[0][2 * f]);
                    const bf16x8_t a1 = __builtin_bit_cast(bf16x8_t, rowK[1][2 * f]);
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        const bf16x8_t bf = __builtin_bit_cast(bf16x8_t, Bl[(fl * 4 + db) * 64 + lane]);
                        acc[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, a0, acc[0][db], 0, 0, 0);
                        acc[1][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, a1, acc[1][db], 0, 0, 0);
                    }
                }
            }
        }

        // (2) Z^T = K^ Q^T: lane (head slot n, hf), register v <-> token 8(v/4) + 4hf + v%4 of block tb
        f32x16_t Z[2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) Z[tb][v] = 0.0f;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    Z[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pack8(acc[tb][db], j), Qf[db][j], Z[tb], 0, 0, 0);
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
        bf16x8_t Wf[2][2];
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

        // (3) V^ tile: rows = tokens, columns = head dims
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tb][db][v] = 0.0f;
        for (int c0 = 0; c0 < F4v; c0 += kFragsPerChunk) {
            __syncthreads();
            for (int e = threadIdx.x; e < kFragsPerChunk * 256; e += 256) Bl[e] = packV[(size_t)c0 * 256 + e];
            __syncthreads();
#pragma unroll
            for (int fl = 0; fl < kFragsPerChunk; ++fl) {
                const int f = c0 + fl;
                if (f < Fv) {
                    const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, rowV[0][2 * f]);
                    const bf16x8_t a1 = __builtin_bit_cast(bf16x8_t, rowV[1][2 * f]);
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        const bf16x8_t bf = __builtin_bit_cast(bf16x8_t, Bl[(fl * 4 + db) * 64 + lane]);
                        acc[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bf, acc[0][db], 0, 0, 0);
                        acc[1][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bf, acc[1][db], 0, 0, 0);
                    }
                }
            }
        }

        // (4) O = alpha O + W V^ ; O rows are head slots: register v of half hf is slot 8(v/4) + 4hf + v%4
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const float a = __shfl(alpha, 8 * (v / 4) + 4 * hf + (v % 4), kWave);
#pragma unroll
            for (int db = 0; db < 4; ++db) O[db][v] *= a;
        }
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int db = 0; db < 4; ++db)
                    O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Wf[tb][j], pack8(acc[tb][db], j), O[db], 0, 0, 0);
    }

    // one partial per wavefront and query head
    const int n_part = splits * 4, part = split * 4 + w;
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    if (lane < n_rep) {
        const size_t slot = ((size_t)b * H_q + g * n_rep + lane) * n_part + part;
        part_ml[slot * 2 + 0] = m_run;
        part_ml[slot * 2 + 1] = l_tot;
    }
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const int hh = 8 * (v / 4) + 4 * hf + (v % 4);
        if (hh < n_rep) {
            const size_t slot = ((size_t)b * H_q + g * n_rep + hh) * n_part + part;
#pragma unroll
            for (int db = 0; db < 4; ++db) part_o[slot * 128 + db * 32 + n] = O[db][v];
        }
    }
}

bool gather_attend_mfma_shape_ok(const xkv_shape &s)
{
    return s.dtype == XKV_BF16 && s.d_h == 128 && s.r_k % 16 == 0 && s.r_v % 16 == 0;
}

size_t gather_attend_pack_bytes(const xkv_shape &s)
{
    const int F4k = (s.r_k / 16 + 3) / 4 * 4 + 4, F4v = (s.r_v / 16 + 3) / 4 * 4 + 4;
    return (size_t)(s.batch > 0 ? s.batch : 1) * s.H_kv * (size_t)(F4k + F4v) * 4 * 1024;
}

hipError_t launch_gather_attend_mfma(const xkv_shape &s, const Plan &p, int layer, const void *A_k, const void *A_v,
                                     const void *B_k, const void *B_v, const void *q, const int32_t *idx,
                                     void *pack_ws, float *part_o, float *part_ml, hipStream_t st)
{
    const int F4k = (s.r_k / 16 + 3) / 4 * 4, F4v = (s.r_v / 16 + 3) / 4 * 4;
    const int total = (F4k + F4v) * 256;
    dim3 pgrid((total + 255) / 256 < 8 ? (total + 255) / 256 : 8, s.H_kv, s.batch), block(256);
    hipLaunchKernelGGL(pack_b_kernel, pgrid, block, 0, st, (const bf16_t *)B_k, (const bf16_t *)B_v,
                       (u32x4_t *)pack_ws, s.G, layer, s.r_k, s.r_v, s.H_kv, F4k, F4v);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid(p.sr_splits, s.H_kv, s.batch);
    hipLaunchKernelGGL(gather_attend_mfma_kernel, grid, block, 0, st, (const bf16_t *)A_k, (const bf16_t *)A_v,
                       (const u32x4_t *)pack_ws, (const bf16_t *)q, idx, part_o, part_ml, s.L, s.r_k, s.r_v, s.H_kv,
                       s.H_q, s.k, p.sr_splits, p.sr_chunk, F4k, F4v, p.scale);
    return hipGetLastError();
}

}  // namespace xkv
