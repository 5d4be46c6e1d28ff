// Selective reconstruction of the chosen rows (Sec. 3.2, Eq. 3) fused with softmax attention
// over them for the query heads of each KV head:
//   K^_g[m,:] = A^K[I_g[m],:] B^K_{l,g},  V^_g[m,:] = A^V[I_g[m],:] B^V_{l,g},
//   out_h = softmax(scale * K^_g q_h)^T V^_g   for every h with rho(h) = g.
// The selected tokens of a (sequence, KV head) are split over workgroups and wavefronts; each
// wavefront keeps an online-softmax partial (max, sum, unnormalised output) per query head and
// writes it out; combine_kernel (dense.hip) merges the partials.
#include "xkv_common.h"

namespace xkv {

// ------------------------------------------------------------------------------------------
// General path (any dtype, any rank): fp32 FMA.  Lanes run over the head dimension (JP values
// per lane), a wavefront reconstructs TM selected rows at a time so every element of B is
// loaded once per TM rows; the A values of a row are wave-uniform.
// ------------------------------------------------------------------------------------------
template <typename T, int JP>
__global__ __launch_bounds__(256) void gather_attend_generic_kernel(
    const T *__restrict__ A_k, const T *__restrict__ A_v, const T *__restrict__ B_k, const T *__restrict__ B_v,
    const T *__restrict__ q, const int32_t *__restrict__ idx, const int32_t *__restrict__ counts,
    float *__restrict__ part_o, float *__restrict__ part_ml, int G, int layer, int L, int r_k, int r_v, int H_kv,
    int H_q, int d_h, int k, int splits, int chunk, float scale, float rope_theta)
{
    constexpr int TM = 4;
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int n_rep = H_q / H_kv, d = H_kv * d_h;
    const int lane = lane_id(), w = wave_id();

    float qreg[16][JP], o[16][JP], mx[16], den[16];
#pragma unroll
    for (int hh = 0; hh < 16; ++hh) {
        mx[hh] = -INFINITY;
        den[hh] = 0.0f;
#pragma unroll
        for (int jj = 0; jj < JP; ++jj) {
            const int j = lane + jj * kWave;
            o[hh][jj] = 0.0f;
            qreg[hh][jj] = (hh < n_rep && j < d_h) ? to_f32(q[((size_t)b * H_q + g * n_rep + hh) * d_h + j]) : 0.0f;
        }
    }

    const T *Bk = B_k + ((size_t)b * G + layer) * r_k * d + (size_t)g * d_h;
    const T *Bv = B_v + ((size_t)b * G + layer) * r_v * d + (size_t)g * d_h;
    const T *Ak = A_k + (size_t)b * L * r_k;
    const T *Av = A_v + (size_t)b * L * r_v;
    const int32_t *ids = idx + ((size_t)b * H_kv + g) * k;
    int k_eff = k;  // with `counts`, only the first counts[sequence][head] ids of a row are attended over
    if (counts) {
        const int cn = counts[b * H_kv + g];
        k_eff = cn < k ? (cn > 0 ? cn : 0) : k;
    }
    const int m_begin = split * chunk;
    const int m_end = (m_begin + chunk < k_eff) ? m_begin + chunk : k_eff;

    for (int m0 = m_begin + w * TM; m0 < m_end; m0 += 4 * TM) {
        int tok[TM];
#pragma unroll
        for (int mm = 0; mm < TM; ++mm) {
            const int m = (m0 + mm < m_end) ? m0 + mm : m_end - 1;
            int t = __builtin_amdgcn_readfirstlane(ids[m]);
            t = t < 0 ? 0 : (t >= L ? L - 1 : t);  // ids are validated by contract; never read out of bounds
            tok[mm] = t;
        }
        float kh[TM][JP], vh[TM][JP], vrot[TM][JP];
#pragma unroll
        for (int mm = 0; mm < TM; ++mm)
#pragma unroll
            for (int jj = 0; jj < JP; ++jj) kh[mm][jj] = vh[mm][jj] = 0.0f;

        for (int i = 0; i < r_k; ++i) {
            float bv[JP];
#pragma unroll
            for (int jj = 0; jj < JP; ++jj) {
                const int j = lane + jj * kWave;
                bv[jj] = j < d_h ? to_f32(Bk[(size_t)i * d + j]) : 0.0f;
            }
#pragma unroll
            for (int mm = 0; mm < TM; ++mm) {
                const float a = to_f32(Ak[(size_t)tok[mm] * r_k + i]);
#pragma unroll
                for (int jj = 0; jj < JP; ++jj) kh[mm][jj] = fmaf(a, bv[jj], kh[mm][jj]);
            }
        }
        for (int i = 0; i < r_v; ++i) {
            float bv[JP];
#pragma unroll
            for (int jj = 0; jj < JP; ++jj) {
                const int j = lane + jj * kWave;
                bv[jj] = j < d_h ? to_f32(Bv[(size_t)i * d + j]) : 0.0f;
            }
#pragma unroll
            for (int mm = 0; mm < TM; ++mm) {
                const float a = to_f32(Av[(size_t)tok[mm] * r_v + i]);
#pragma unroll
                for (int jj = 0; jj < JP; ++jj) vh[mm][jj] = fmaf(a, bv[jj], vh[mm][jj]);
            }
        }
        if (rope_theta > 0.0f) {
            // The reconstructed key rows are pre-RoPE: rotate each to its position (its row number).  Channel
            // j < d_h/2 is paired with j + d_h/2; the partner sits in this lane's other register when d_h/2 is a
            // multiple of 64, else (d_h <= 64) in lane j +- d_h/2 of the same register.  Angles in double.
            const int half = d_h / 2;
#pragma unroll
            for (int mm = 0; mm < TM; ++mm)
#pragma unroll
                for (int jj = 0; jj < JP; ++jj) {
                    const int j = lane + jj * kWave;
                    const bool low = j < half;
                    float partner;
                    if constexpr (JP >= 2)
                        partner = kh[mm][(jj + JP / 2) % JP];  // d_h = 64 JP: the partner is JP / 2 registers away
                    else
                        partner = __shfl(kh[mm][jj], low ? lane + half : lane - half, kWave);
                    const int jf = low ? j : j - half;
                    float cs = 1.0f, sn = 0.0f;
                    if (j < d_h) {
                        const double ang = (double)tok[mm] * pow((double)rope_theta, -2.0 * (double)jf / (double)d_h);
                        cs = (float)cos(ang);
                        sn = (float)sin(ang);
                    }
                    vrot[mm][jj] = low ? kh[mm][jj] * cs - partner * sn : kh[mm][jj] * cs + partner * sn;
                }
#pragma unroll
            for (int mm = 0; mm < TM; ++mm)
#pragma unroll
                for (int jj = 0; jj < JP; ++jj) kh[mm][jj] = vrot[mm][jj];
        }
#pragma unroll
        for (int mm = 0; mm < TM; ++mm) {
            if (m0 + mm < m_end) {  // wave-uniform
#pragma unroll
                for (int hh = 0; hh < 16; ++hh) {
                    if (hh < n_rep) {
                        float part = 0.0f;
#pragma unroll
                        for (int jj = 0; jj < JP; ++jj) part = fmaf(kh[mm][jj], qreg[hh][jj], part);
                        const float z = scale * wave_sum(part);
                        const float m_new = fmaxf(mx[hh], z);
                        const float alpha = expf(mx[hh] - m_new);  // exp(-inf) = 0 on the first row
                        const float pw = expf(z - m_new);
                        den[hh] = den[hh] * alpha + pw;
#pragma unroll
                        for (int jj = 0; jj < JP; ++jj) o[hh][jj] = fmaf(pw, vh[mm][jj], o[hh][jj] * alpha);
                        mx[hh] = m_new;
                    }
                }
            }
        }
    }

    const int n_part = splits * 4, part = split * 4 + w;
#pragma unroll
    for (int hh = 0; hh < 16; ++hh) {
        if (hh < n_rep) {
            const size_t slot = ((size_t)b * H_q + g * n_rep + hh) * n_part + part;
#pragma unroll
            for (int jj = 0; jj < JP; ++jj) {
                const int j = lane + jj * kWave;
                if (j < d_h) part_o[slot * d_h + j] = o[hh][jj];
            }
            if (lane == 0) {
                part_ml[slot * 2 + 0] = mx[hh];
                part_ml[slot * 2 + 1] = den[hh];
            }
        }
    }
}

template <typename T>
static hipError_t launch_generic(const xkv_shape &s, const Plan &p, int layer, const void *A_k, const void *A_v,
                                 const void *B_k, const void *B_v, const void *q, const int32_t *idx, float *part_o,
                                 float *part_ml, hipStream_t st, const int32_t *counts, float rope_theta)
{
    dim3 grid(p.sr_splits, s.H_kv, s.batch), block(256);
#define XKV_GA_LAUNCH(JP)                                                                                          \
    hipLaunchKernelGGL((gather_attend_generic_kernel<T, JP>), grid, block, 0, st, (const T *)A_k, (const T *)A_v,  \
                       (const T *)B_k, (const T *)B_v, (const T *)q, idx, counts, part_o, part_ml, s.G, layer,     \
                       s.L, s.r_k, s.r_v, s.H_kv, s.H_q, s.d_h, s.k, p.sr_splits, p.sr_chunk, p.scale, rope_theta)
    profile_begin(1, st);
    if (s.d_h <= 64)
        XKV_GA_LAUNCH(1);
    else if (s.d_h <= 128)
        XKV_GA_LAUNCH(2);
    else
        XKV_GA_LAUNCH(4);
    profile_end(1, st);
#undef XKV_GA_LAUNCH
    return hipGetLastError();
}

// Channel pairs (j, j + d_h/2) must sit in one lane or in one register of the general kernel.
bool rope_shape_ok(const xkv_shape &s) { return s.d_h % 2 == 0 && (s.d_h <= 64 || (s.d_h / 2) % 64 == 0); }

bool gather_attend_uses_mfma(const Plan &p, const void *A_k, const void *A_v, const void *B_k, const void *B_v,
                             const void *pack_ws)
{
    return p.ga_mfma &&
           ((((uintptr_t)A_k | (uintptr_t)A_v | (uintptr_t)B_k | (uintptr_t)B_v | (uintptr_t)pack_ws)) & 15u) == 0;
}

bool gather_attend_quant_ok(const xkv_shape &s, const Plan &p, const void *Aq_k, const void *Aq_v, const void *B_k,
                            const void *B_v, const void *pack_ws, int qbits)
{
    return (qbits == 4 || qbits == 3) && quant_rank_ok(s.r_k) && quant_rank_ok(s.r_v) &&
           gather_attend_uses_mfma(p, Aq_k, Aq_v, B_k, B_v, pack_ws);
}

hipError_t launch_gather_attend(const xkv_shape &s, const Plan &p, int layer, const void *A_k, const void *A_v,
                                const void *B_k, const void *B_v, const void *q, const int32_t *idx, void *pack_ws,
                                const void *B_packed, bool packed, float *part_o, float *part_ml, hipStream_t st,
                                const int32_t *counts, float rope_theta, int qbits)
{
    if (gather_attend_uses_mfma(p, A_k, A_v, B_k, B_v, pack_ws))
        return launch_gather_attend_mfma(s, p, layer, A_k, A_v, B_k, B_v, q, idx, pack_ws, B_packed, packed, part_o,
                                         part_ml, st, counts, rope_theta, qbits);
    if (qbits != 0) return hipErrorInvalidValue;  // quantised rows are read by the matrix-core kernel only
    if (s.dtype == XKV_F32)
        return launch_generic<float>(s, p, layer, A_k, A_v, B_k, B_v, q, idx, part_o, part_ml, st, counts, rope_theta);
    return launch_generic<bf16_t>(s, p, layer, A_k, A_v, B_k, B_v, q, idx, part_o, part_ml, st, counts, rope_theta);
}

}  // namespace xkv
