// Query projection into the rank space and the low-rank score stream with GQA max-pooling.
//   p_h = B^K_{l,rho(h)} q_h                      (Eq. 3 regrouped by associativity)
//   s[h,t] = scale * A^K[t,:] . p_h               (App. B.1 Alg. 2, scaled scores, per token)
//   S[g,t] = max_{h: rho(h)=g} s[h,t]             (App. B.1 Alg. 2, GQA pooling)
#include "xkv_common.h"

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

hipError_t launch_project_q(const xkv_shape &s, const Plan &p, int layer, const void *B_k, const void *q, float *P,
                            hipStream_t st)
{
    (void)p;
    dim3 grid((s.r_k * s.H_kv + 3) / 4, s.batch), block(256);
    if (s.dtype == XKV_F32)
        hipLaunchKernelGGL(project_q_kernel<float>, grid, block, 0, st, (const float *)B_k, (const float *)q, P, s.G,
                           layer, s.r_k, s.H_kv, s.H_q, s.d_h);
    else
        hipLaunchKernelGGL(project_q_kernel<bf16_t>, grid, block, 0, st, (const bf16_t *)B_k, (const bf16_t *)q, P,
                           s.G, layer, s.r_k, s.H_kv, s.H_q, s.d_h);
    return hipGetLastError();
}

hipError_t launch_score(const xkv_shape &s, const Plan &p, const void *A_k, const float *P, float *S, hipStream_t st)
{
    dim3 grid((s.L + 255) / 256, s.batch), block(256);
    if (s.dtype == XKV_F32)
        hipLaunchKernelGGL(score_generic_kernel<float>, grid, block, 0, st, (const float *)A_k, P, S, s.L, s.r_k,
                           s.H_kv, s.H_q, p.scale);
    else
        hipLaunchKernelGGL(score_generic_kernel<bf16_t>, grid, block, 0, st, (const bf16_t *)A_k, P, S, s.L, s.r_k,
                           s.H_kv, s.H_q, p.scale);
    return hipGetLastError();
}

}  // namespace xkv
