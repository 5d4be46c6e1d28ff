// Dense decode attention on an uncompressed cache (the "Full Attention" baseline of Sec. 5):
//   out_h = softmax(scale * K_{rho(h)} q_h)^T V_{rho(h)}  over all L tokens,
// split over the tokens flash-decoding style, plus the kernel that merges split partials
// (shared with the SR path).
#include "xkv_common.h"

namespace xkv {

// ------------------------------------------------------------------------------------------
// General path: lanes run over the head dimension, a wavefront walks TM tokens at a time.
// K, V: [batch][H_kv][L][d_h].
// ------------------------------------------------------------------------------------------
template <typename T, int JP>
__global__ __launch_bounds__(256) void dense_generic_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                            const T *__restrict__ q, float *__restrict__ part_o,
                                                            float *__restrict__ part_ml, int L, int H_kv, int H_q,
                                                            int d_h, int splits, int chunk, float scale)
{
    constexpr int TM = 4;
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int n_rep = H_q / H_kv;
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
    const T *Kg = K + ((size_t)b * H_kv + g) * L * d_h;
    const T *Vg = V + ((size_t)b * H_kv + g) * L * d_h;
    const int t_begin = split * chunk;
    const int t_end = (t_begin + chunk < L) ? t_begin + chunk : L;

    for (int t0 = t_begin + w * TM; t0 < t_end; t0 += 4 * TM) {
        float kr[TM][JP], vr[TM][JP];
#pragma unroll
        for (int mm = 0; mm < TM; ++mm) {
            const int t = (t0 + mm < t_end) ? t0 + mm : t_end - 1;
#pragma unroll
            for (int jj = 0; jj < JP; ++jj) {
                const int j = lane + jj * kWave;
                kr[mm][jj] = j < d_h ? to_f32(Kg[(size_t)t * d_h + j]) : 0.0f;
                vr[mm][jj] = j < d_h ? to_f32(Vg[(size_t)t * d_h + j]) : 0.0f;
            }
        }
#pragma unroll
        for (int mm = 0; mm < TM; ++mm) {
            if (t0 + mm < t_end) {  // wave-uniform
#pragma unroll
                for (int hh = 0; hh < 16; ++hh) {
                    if (hh < n_rep) {
                        float part = 0.0f;
#pragma unroll
                        for (int jj = 0; jj < JP; ++jj) part = fmaf(kr[mm][jj], qreg[hh][jj], part);
                        const float z = scale * wave_sum(part);
                        const float m_new = fmaxf(mx[hh], z);
                        const float alpha = expf(mx[hh] - m_new);
                        const float pw = expf(z - m_new);
                        den[hh] = den[hh] * alpha + pw;
#pragma unroll
                        for (int jj = 0; jj < JP; ++jj) o[hh][jj] = fmaf(pw, vr[mm][jj], o[hh][jj] * alpha);
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

// ------------------------------------------------------------------------------------------
// Merge the split partials of one (sequence, query head) with the log-sum-exp rule and write
// the normalised output in the storage dtype.  A partial that saw no token has max = -inf.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ part_o,
                                                      const float *__restrict__ part_ml, T *__restrict__ out,
                                                      int H_q, int d_h, int n_part)
{
    const int h = blockIdx.x, b = blockIdx.y;
    const size_t base = ((size_t)b * H_q + h) * n_part;
    float M = -INFINITY;
    for (int s = 0; s < n_part; ++s) M = fmaxf(M, part_ml[(base + s) * 2]);
    for (int j = threadIdx.x; j < d_h; j += blockDim.x) {
        float num = 0.0f, den = 0.0f;
        for (int s = 0; s < n_part; ++s) {
            const float m = part_ml[(base + s) * 2];
            const float wgt = (m == -INFINITY) ? 0.0f : expf(m - M);
            num = fmaf(wgt, part_o[(base + s) * d_h + j], num);
            den = fmaf(wgt, part_ml[(base + s) * 2 + 1], den);
        }
        out[((size_t)b * H_q + h) * d_h + j] = from_f32<T>(num / den);
    }
}

template <typename T>
static hipError_t launch_dense_generic(const xkv_shape &s, const Plan &p, const void *K, const void *V, const void *q,
                                       float *part_o, float *part_ml, hipStream_t st)
{
    dim3 grid(p.dense_splits, s.H_kv, s.batch), block(256);
#define XKV_DENSE_LAUNCH(JP)                                                                                    \
    hipLaunchKernelGGL((dense_generic_kernel<T, JP>), grid, block, 0, st, (const T *)K, (const T *)V,           \
                       (const T *)q, part_o, part_ml, s.L, s.H_kv, s.H_q, s.d_h, p.dense_splits, p.dense_chunk, \
                       p.scale)
    if (s.d_h <= 64)
        XKV_DENSE_LAUNCH(1);
    else if (s.d_h <= 128)
        XKV_DENSE_LAUNCH(2);
    else
        XKV_DENSE_LAUNCH(4);
#undef XKV_DENSE_LAUNCH
    return hipGetLastError();
}

hipError_t launch_dense(const xkv_shape &s, const Plan &p, const void *K, const void *V, const void *q, float *part_o,
                        float *part_ml, hipStream_t st)
{
    if (s.dtype == XKV_F32) return launch_dense_generic<float>(s, p, K, V, q, part_o, part_ml, st);
    return launch_dense_generic<bf16_t>(s, p, K, V, q, part_o, part_ml, st);
}

hipError_t launch_combine(const xkv_shape &s, int n_splits, const float *part_o, const float *part_ml, void *out,
                          hipStream_t st)
{
    dim3 grid(s.H_q, s.batch), block(s.d_h <= 64 ? 64 : (s.d_h <= 128 ? 128 : 256));
    const int n_part = n_splits * 4;
    if (s.dtype == XKV_F32)
        hipLaunchKernelGGL(combine_kernel<float>, grid, block, 0, st, part_o, part_ml, (float *)out, s.H_q, s.d_h,
                           n_part);
    else
        hipLaunchKernelGGL(combine_kernel<bf16_t>, grid, block, 0, st, part_o, part_ml, (bf16_t *)out, s.H_q, s.d_h,
                           n_part);
    return hipGetLastError();
}

}  // namespace xkv
