// landmark.hip -- the paper's own token selector for Selective Reconstruction (App. B.1): landmark construction
// at prefill (Alg. 1) and the pieces of the landmark-guided chunk selection at decode (Alg. 2) that are not
// already kernels of the factor-scoring path.
//
// At decode, scoring chunks against landmarks is the same computation as scoring tokens against the key factors
// with the landmarks of one KV head in the place of A^K (n_c rows of d_h values), the head's queries in the place
// of the projected queries, and an identity matrix in the place of B^K: the score kernels, the GQA max-pool and
// the radix top-k are used unchanged on that reshaped problem.  What is new here: the chunk means and the
// within-chunk minimum cosine (Alg. 1), the union of the top chunks with the static outliers and its expansion
// to token rows (Alg. 2, last two steps).
#include "xkv_common.h"

namespace xkv {
namespace {

// One wavefront per chunk: lane l holds channels l, l + 64, ... of the d_h <= 256 channels.  Landmark = mean of the
// chunk's keys (a shorter last chunk: mean over the tokens it has), rounded once to the storage type; the cosine
// of every key with the fp32 mean, its minimum over the chunk negated into neg_min_cos (so that the chunks with
// the smallest minimum are the top of ArgTopK(-m, o), Alg. 1).  A zero key or a zero mean counts as cosine 0.
template <typename T>
__global__ __launch_bounds__(256) void landmark_kernel(const T *__restrict__ K, T *__restrict__ Lm, float *__restrict__ neg_m,
                                                       int L, int d_h, int c, int n_c)
{
    const int j = blockIdx.x * 4 + wave_id(), row = blockIdx.y;  // chunk, (sequence, KV head)
    if (j >= n_c) return;
    const int lane = lane_id();
    const int t0 = j * c, t1 = (t0 + c < L) ? t0 + c : L;
    const T *Kr = K + (size_t)row * L * d_h;
    float mean[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int t = t0; t < t1; ++t)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ch = lane + 64 * u;
            if (ch < d_h) mean[u] += to_f32(Kr[(size_t)t * d_h + ch]);
        }
    const float inv = 1.0f / (float)(t1 - t0);
    float mm = 0.0f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        mean[u] *= inv;
        mm += mean[u] * mean[u];
        const int ch = lane + 64 * u;
        if (ch < d_h) Lm[((size_t)row * n_c + j) * d_h + ch] = from_f32<T>(mean[u]);
    }
    mm = wave_sum(mm);
    float worst = INFINITY;
    for (int t = t0; t < t1; ++t) {
        float xm = 0.0f, xx = 0.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ch = lane + 64 * u;
            const float x = ch < d_h ? to_f32(Kr[(size_t)t * d_h + ch]) : 0.0f;
            xm += x * mean[u];
            xx += x * x;
        }
        xm = wave_sum(xm);
        xx = wave_sum(xx);
        const float den = sqrtf(xx) * sqrtf(mm);
        worst = fminf(worst, den > 0.0f ? xm / den : 0.0f);
    }
    if (lane == 0 && neg_m) neg_m[(size_t)row * n_c + j] = -worst;
}

// The same for bf16 keys of 128 channels and chunks of 4, 8, 12 or 16 tokens, read once and line-wise: an
// instruction covers 4 rows (lane l: row l / 16, the 16 B piece l % 16), the rows of a chunk stay in registers for
// the cosine pass, sums over channels run across the 16 lanes of a row, sums over rows across the 4 lane groups.
typedef __attribute__((ext_vector_type(4))) uint32_t lm_u32x4_t;
__global__ __launch_bounds__(256) void landmark_bf16_128_kernel(const bf16_t *__restrict__ K, bf16_t *__restrict__ Lm,
                                                                float *__restrict__ neg_m, int L, int c, int n_c)
{
    const int j = blockIdx.x * 4 + wave_id(), row = blockIdx.y;
    if (j >= n_c) return;
    const int lane = lane_id(), rg = lane >> 4, pc = lane & 15;
    const int t0 = j * c, t1 = (t0 + c < L) ? t0 + c : L;
    const lm_u32x4_t *Kr = reinterpret_cast<const lm_u32x4_t *>(K + (size_t)row * L * 128);
    lm_u32x4_t xs[4];
    float sum[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) sum[e] = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = t0 + 4 * i + rg;
        xs[i] = lm_u32x4_t{0u, 0u, 0u, 0u};
        if (4 * i < c && t < t1) xs[i] = Kr[(size_t)t * 16 + pc];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sum[2 * e] += __uint_as_float(xs[i][e] << 16);
            sum[2 * e + 1] += __uint_as_float(xs[i][e] & 0xFFFF0000u);
        }
    }
    const float inv = 1.0f / (float)(t1 - t0);
    float mean[8], mm = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float v = sum[e];
        v += __shfl_xor(v, 16, kWave);
        v += __shfl_xor(v, 32, kWave);
        mean[e] = v * inv;
        mm += mean[e] * mean[e];
    }
#pragma unroll
    for (int o2 = 1; o2 < 16; o2 <<= 1) mm += __shfl_xor(mm, o2, kWave);
    if (rg == 0) {
        lm_u32x4_t pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (uint32_t)f32_to_bf16(mean[2 * e]) | ((uint32_t)f32_to_bf16(mean[2 * e + 1]) << 16);
        reinterpret_cast<lm_u32x4_t *>(Lm + ((size_t)row * n_c + j) * 128)[pc] = pk;
    }
    float worst = INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float xm = 0.0f, xx = 0.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x0 = __uint_as_float(xs[i][e] << 16), x1 = __uint_as_float(xs[i][e] & 0xFFFF0000u);
            xm += x0 * mean[2 * e] + x1 * mean[2 * e + 1];
            xx += x0 * x0 + x1 * x1;
        }
#pragma unroll
        for (int o2 = 1; o2 < 16; o2 <<= 1) {
            xm += __shfl_xor(xm, o2, kWave);
            xx += __shfl_xor(xx, o2, kWave);
        }
        const float den = sqrtf(xx) * sqrtf(mm);
        const float cs = den > 0.0f ? xm / den : 0.0f;
        if (4 * i < c && t0 + 4 * i + rg < t1) worst = fminf(worst, cs);
    }
    worst = fminf(worst, __shfl_xor(worst, 16, kWave));
    worst = fminf(worst, __shfl_xor(worst, 32, kWave));
    if (lane == 0 && neg_m) neg_m[(size_t)row * n_c + j] = -worst;
}

// `copies` identity matrices [d_h][d_h] in the storage type.
template <typename T> __global__ __launch_bounds__(256) void identity_kernel(T *__restrict__ B, int d_h, long long count)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const int col = (int)(i % d_h), rw = (int)((i / d_h) % d_h);
    B[i] = from_f32<T>(rw == col ? 1.0f : 0.0f);
}

// Alg. 2, last steps, one workgroup per (sequence, KV head): union of the k_ch selected chunks (ascending, no
// repeats) with the o static outliers (ascending, no repeats), expanded to token rows in ascending order.  rows gets
// (k_ch + o) * c entries, of which the first counts[row] are real (only the context's last chunk can be short, and
// it can only be the last of the union); the rest is filled with row 0 and ignored by the attention kernel.
__global__ __launch_bounds__(256) void expand_chunks_kernel(const int32_t *__restrict__ chunks, int k_ch,
                                                            const int32_t *__restrict__ outliers, int o, int c, int L, int n_c,
                                                            int32_t *__restrict__ rows, int32_t *__restrict__ counts)
{
    extern __shared__ int32_t lds_i[];
    int32_t *ch_s = lds_i, *ou_s = ch_s + k_ch, *lb_s = ou_s + o, *dup_s = lb_s + o, *merged = dup_s + o;  // [k_ch + o]
    __shared__ int n_merged;
    const int row = blockIdx.x, cap = (k_ch + o) * c, tid = threadIdx.x;
    auto clampc = [&](int v) { return v < 0 ? 0 : (v >= n_c ? n_c - 1 : v); };
    for (int a = tid; a < k_ch; a += 256) ch_s[a] = clampc(chunks[(size_t)row * k_ch + a]);
    for (int b = tid; b < o; b += 256) ou_s[b] = clampc(outliers[(size_t)row * o + b]);
    __syncthreads();
    // both lists are ascending without repeats: an element's place in the union is its own index plus the number of
    // elements of the other list in front of it (outliers that are also selected chunks are dropped)
    for (int b = tid; b < o; b += 256) {
        int lo = 0, hi = k_ch;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (ch_s[mid] < ou_s[b]) lo = mid + 1; else hi = mid;
        }
        lb_s[b] = lo;
        dup_s[b] = (lo < k_ch && ch_s[lo] == ou_s[b]) ? 1 : 0;
    }
    __syncthreads();
    for (int a = tid; a < k_ch; a += 256) {
        int before = 0;
        for (int b = 0; b < o; ++b) before += (!dup_s[b] && ou_s[b] < ch_s[a]) ? 1 : 0;
        merged[a + before] = ch_s[a];
    }
    for (int b = tid; b < o; b += 256) {
        if (!dup_s[b]) {
            int before = 0;
            for (int b2 = 0; b2 < b; ++b2) before += dup_s[b2] ? 0 : 1;
            merged[lb_s[b] + before] = ou_s[b];
        }
    }
    if (tid == 0) {
        int n = k_ch;
        for (int b = 0; b < o; ++b) n += dup_s[b] ? 0 : 1;
        n_merged = n;
    }
    __syncthreads();
    const int n = n_merged;
    int total = n * c;
    if (n > 0 && merged[n - 1] == n_c - 1) total -= n_c * c - L;  // the short last chunk
    int32_t *out = rows + (size_t)row * cap;
    for (int i = tid; i < cap; i += 256) out[i] = i < total ? merged[i / c] * c + i % c : 0;
    if (tid == 0) counts[row] = total;
}

}  // namespace

hipError_t launch_landmarks(const xkv_shape &s, const void *K_rope, int c, void *landmarks, float *neg_min_cos,
                            hipStream_t st)
{
    const int n_c = (s.L + c - 1) / c;
    dim3 grid((n_c + 3) / 4, s.batch * s.H_kv);
    if (s.dtype == XKV_BF16 && s.d_h == 128 && c % 4 == 0 && c <= 16 && (((uintptr_t)K_rope | (uintptr_t)landmarks) & 15u) == 0) {
        hipLaunchKernelGGL(landmark_bf16_128_kernel, grid, dim3(256), 0, st, (const bf16_t *)K_rope, (bf16_t *)landmarks,
                           neg_min_cos, s.L, c, n_c);
        return hipGetLastError();
    }
    if (s.dtype == XKV_F32)
        hipLaunchKernelGGL(landmark_kernel<float>, grid, dim3(256), 0, st, (const float *)K_rope, (float *)landmarks,
                           neg_min_cos, s.L, s.d_h, c, n_c);
    else
        hipLaunchKernelGGL(landmark_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t *)K_rope, (bf16_t *)landmarks,
                           neg_min_cos, s.L, s.d_h, c, n_c);
    return hipGetLastError();
}

hipError_t launch_identity(const xkv_shape &s, void *B, int copies, hipStream_t st)
{
    const long long count = (long long)copies * s.d_h * s.d_h;
    const unsigned blocks = (unsigned)((count + 255) / 256);
    if (s.dtype == XKV_F32)
        hipLaunchKernelGGL(identity_kernel<float>, dim3(blocks), dim3(256), 0, st, (float *)B, s.d_h, count);
    else
        hipLaunchKernelGGL(identity_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, (bf16_t *)B, s.d_h, count);
    return hipGetLastError();
}

hipError_t launch_expand_chunks(const xkv_shape &s, const int32_t *chunks, int k_ch, const int32_t *outliers, int o, int c,
                                int32_t *rows, int32_t *counts, hipStream_t st)
{
    const int n_c = (s.L + c - 1) / c;
    hipLaunchKernelGGL(expand_chunks_kernel, dim3(s.batch * s.H_kv), dim3(256), (size_t)(2 * k_ch + 4 * o) * sizeof(int32_t), st,
                       chunks, k_ch, outliers, o, c, s.L, n_c, rows, counts);
    return hipGetLastError();
}

}  // namespace xkv
