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
constexpr int kMaxCombineParts = 1024;  // partials per query head that one merge takes (splits and tail together)

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ part_o,
                                                      const float *__restrict__ part_ml, T *__restrict__ out,
                                                      int H_q, int d_h, int n_part,
                                                      const float *__restrict__ part_o2,
                                                      const float *__restrict__ part_ml2, int n_part2)
{
    // the second set of partials (n_part2 may be 0) has the same layout; it holds the uncompressed tail tokens
    const int h = blockIdx.x, b = blockIdx.y;
    const size_t base = ((size_t)b * H_q + h) * n_part, base2 = ((size_t)b * H_q + h) * n_part2;
    // (maximum, sum) of every partial into LDS with all loads in flight at once, then one weight per partial; the
    // accumulation below runs four partials at a time for the same reason (the kernel is a chain of small dependent
    // loads otherwise: its time is their latency)
    __shared__ float sm_m[kMaxCombineParts], sm_w[kMaxCombineParts];
    __shared__ float sm_den;
    const int n_all = n_part + n_part2;
    for (int s = threadIdx.x; s < n_all; s += blockDim.x)
        sm_m[s] = s < n_part ? part_ml[(base + s) * 2] : part_ml2[(base2 + (s - n_part)) * 2];
    __syncthreads();
    float M = -INFINITY;
    for (int s = 0; s < n_all; ++s) M = fmaxf(M, sm_m[s]);
    __syncthreads();
    for (int s = threadIdx.x; s < n_all; s += blockDim.x) {
        const float m = sm_m[s];
        sm_w[s] = (m == -INFINITY) ? 0.0f : expf(m - M);
        sm_m[s] = s < n_part ? part_ml[(base + s) * 2 + 1] : part_ml2[(base2 + (s - n_part)) * 2 + 1];  // now the sums
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float den = 0.0f;
        for (int s = 0; s < n_all; ++s) den = fmaf(sm_w[s], sm_m[s], den);
        sm_den = den;
    }
    __syncthreads();
    const float den = sm_den;
    for (int j = threadIdx.x; j < d_h; j += blockDim.x) {
        float num = 0.0f;
        int s = 0;
        for (; s + 4 <= n_part; s += 4) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = part_o[(base + s + u) * d_h + j];
#pragma unroll
            for (int u = 0; u < 4; ++u) num = fmaf(sm_w[s + u], v[u], num);
        }
        for (; s < n_part; ++s) num = fmaf(sm_w[s], part_o[(base + s) * d_h + j], num);
        for (int s2 = 0; s2 < n_part2; ++s2) num = fmaf(sm_w[n_part + s2], part_o2[(base2 + s2) * d_h + j], num);
        // a head with no token at all (every list empty, no tail) has den == 0: its output is defined as zero
        out[((size_t)b * H_q + h) * d_h + j] = from_f32<T>(den > 0.0f ? num / den : 0.0f);
    }
}

// ==========================================================================================
// bf16 matrix-core path (d_h = 128).  A wavefront walks 32-token blocks of its workgroup's range:
//   Z^T [tokens x head slots] = K block (loaded line-wise, operand fragments through an LDS tile)  x  Q^T (registers)
//   O [head slots x dims]    += W = exp(Z^T - max) (the result registers of Z^T, packed)   x  V block
// The contraction of the second product runs over tokens, so each lane needs eight token rows of one
// column of V: the V block goes through a wavefront-private LDS tile (row pitch 272 B, conflict-free)
// and is read back transposed.  The four wavefronts merge their partials in LDS before writing.
// ==========================================================================================
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) float f32x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

constexpr int kVPitch = 272;  // bytes per token row of the LDS tile of V (256 + 16: rows 4 apart land 64 B apart)

__device__ __forceinline__ bf16x8_t pack8_bf16(const f32x16_t &c, int j)
{
    f32x8_t x;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = c[8 * j + e];
    return __builtin_convertvector(x, bf16x8_t);
}

__global__ __launch_bounds__(256, 2) void dense_mfma_kernel(const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
                                                            const bf16_t *__restrict__ q, float *__restrict__ part_o,
                                                            float *__restrict__ part_ml, int L, int H_kv, int H_q,
                                                            int splits, int chunk, float scale)
{
    // per wavefront a V tile (32 x 272 B) and a K tile (32 x 256 B); 66 KiB; the V part is reused for the merge
    __shared__ __attribute__((aligned(16))) unsigned char smem[4 * 32 * kVPitch + 4 * 32 * 256];
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = lane_id(), w = wave_id();
    const int n = lane & 31, hf = lane >> 5;
    const int n_rep = H_q / H_kv;

    // Q^T fragments: lane (head slot n, hf), fragment f, position e: q[n][16 f + 8 hf + e]
    bf16x8_t Qf[8];
    {
        const u32x4_t *qh = reinterpret_cast<const u32x4_t *>(q + ((size_t)b * H_q + (size_t)g * n_rep +
                                                                    (n < n_rep ? n : 0)) * 128);
#pragma unroll
        for (int f = 0; f < 8; ++f) {
            u32x4_t raw = qh[2 * f + hf];
            if (n >= n_rep) raw = u32x4_t{0u, 0u, 0u, 0u};
            Qf[f] = __builtin_bit_cast(bf16x8_t, raw);
        }
    }
    const bf16_t *Kg = K + ((size_t)b * H_kv + g) * (size_t)L * 128;
    const bf16_t *Vg = V + ((size_t)b * H_kv + g) * (size_t)L * 128;
    const int t_begin = split * chunk;
    const int t_end = t_begin + chunk < L ? t_begin + chunk : L;
    unsigned char *vt = smem + w * 32 * kVPitch;  // this wavefront's V tile
    // ... and its K tile, in 16 B units: piece c of token row t sits at 16 t + (c + t) % 16 (conflict-free for the
    // row-wise writes and for the fragment reads: lane (n, hf) reads piece 2 f + hf of row n)
    u32x4_t *kt = reinterpret_cast<u32x4_t *>(smem + 4 * 32 * kVPitch) + w * 512;
    const int kw_row = lane >> 4, kw_piece = lane & 15;
    const int kr_base = 16 * n, kr_rot = hf + n;

    float m_run = -INFINITY, l_run = 0.0f;
    // Only head slots 0..15 can hold a query head (n_rep <= 16): of the 16 result registers of an O tile the
    // first 8 (slots 8(v/4) + 4hf + v%4, v < 8) are kept between blocks, the rest is dropped.
    float O[4][8];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 8; ++v) O[db][v] = 0.0f;

    for (int t0 = t_begin + w * 32; t0 < t_end; t0 += 128) {
        // K and V rows, whole lines per instruction: 16 lanes cover one 256 B row, the wavefront 4 rows per load
        // (with one lane per row four instructions would share every 128 B line, which streams measurably slower)
        u32x4_t kr[8], vr[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = i * 4 + (lane >> 4);
            const int tv = t0 + row < t_end ? t0 + row : t_end - 1;
            kr[i] = __builtin_nontemporal_load(&reinterpret_cast<const u32x4_t *>(Kg + (size_t)tv * 128)[lane & 15]);
            vr[i] = __builtin_nontemporal_load(&reinterpret_cast<const u32x4_t *>(Vg + (size_t)tv * 128)[lane & 15]);
        }
        // K through its LDS tile: written row-wise, read back as the operand fragment of each 16 head dims
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = i * 4 + kw_row;
            kt[16 * row + ((kw_piece + row) & 15)] = kr[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        f32x16_t Z;
#pragma unroll
        for (int v = 0; v < 16; ++v) Z[v] = 0.0f;
#pragma unroll
        for (int f = 0; f < 8; ++f) {
            const u32x4_t kf = kt[kr_base + ((kr_rot + 2 * f) & 15)];
            Z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf), Qf[f], Z, 0, 0, 0);
        }
        // lane (head slot n, hf): register v is token 8(v/4) + 4hf + v%4 of the block
        float m_loc = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int tt = t0 + 8 * (v / 4) + 4 * hf + (v % 4);
            Z[v] = tt < t_end ? scale * Z[v] : -INFINITY;
            m_loc = fmaxf(m_loc, Z[v]);
        }
        m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32, kWave));
        const float m_new = fmaxf(m_run, m_loc);
        const float alpha = (m_new == -INFINITY) ? 1.0f : __expf(m_run - m_new);
        float l_add = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float wv = (Z[v] == -INFINITY) ? 0.0f : __expf(Z[v] - m_new);
            Z[v] = wv;
            l_add += wv;
        }
        l_run = l_run * alpha + l_add;
        m_run = m_new;
        const bf16x8_t W0 = pack8_bf16(Z, 0), W1 = pack8_bf16(Z, 1);

        // stage V in LDS and read it back as [8 tokens of one column] fragments
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = i * 4 + (lane >> 4);
            *reinterpret_cast<u32x4_t *>(vt + row * kVPitch + (lane & 15) * 16) = vr[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const float a = __shfl(alpha, 8 * (v / 4) + 4 * hf + (v % 4), kWave);
#pragma unroll
            for (int db = 0; db < 4; ++db) O[db][v] *= a;
        }
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            f32x16_t ot;
#pragma unroll
            for (int v = 0; v < 16; ++v) ot[v] = 0.0f;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                u32x4_t raw;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int e = 2 * e2;
                    const int tok = 8 * (2 * j + e / 4) + 4 * hf + (e % 4);  // e, e+1 are adjacent tokens
                    const uint32_t lo = *reinterpret_cast<const uint16_t *>(vt + tok * kVPitch + (db * 32 + n) * 2);
                    const uint32_t hi =
                        *reinterpret_cast<const uint16_t *>(vt + (tok + 1) * kVPitch + (db * 32 + n) * 2);
                    raw[e2] = lo | (hi << 16);
                }
                ot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(j == 0 ? W0 : W1, __builtin_bit_cast(bf16x8_t, raw), ot, 0,
                                                             0, 0);
            }
#pragma unroll
            for (int v = 0; v < 8; ++v) O[db][v] += ot[v];
        }
        __builtin_amdgcn_wave_barrier();
    }

    // merge the four wavefronts: LDS holds per (wavefront, head) the max, the sum and 128 outputs
    __syncthreads();
    float *mg = reinterpret_cast<float *>(smem);  // [4][16][132]
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
    for (int item = threadIdx.x; item < n_rep * 128; item += 256) {
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

template <typename T>
static hipError_t launch_dense_generic(const xkv_shape &s, const Plan &p, const void *K, const void *V, const void *q,
                                       float *part_o, float *part_ml, hipStream_t st)
{
    dim3 grid(p.dense_splits, s.H_kv, s.batch), block(256);
#define XKV_DENSE_LAUNCH(JP)                                                                                    \
    hipLaunchKernelGGL((dense_generic_kernel<T, JP>), grid, block, 0, st, (const T *)K, (const T *)V,           \
                       (const T *)q, part_o, part_ml, s.L, s.H_kv, s.H_q, s.d_h, p.dense_splits, p.dense_chunk, \
                       p.scale)
    profile_begin(2, st);
    if (s.d_h <= 64)
        XKV_DENSE_LAUNCH(1);
    else if (s.d_h <= 128)
        XKV_DENSE_LAUNCH(2);
    else
        XKV_DENSE_LAUNCH(4);
    profile_end(2, st);
#undef XKV_DENSE_LAUNCH
    return hipGetLastError();
}

bool dense_mfma_shape_ok(const xkv_shape &s) { return s.dtype == XKV_BF16 && s.d_h == 128; }

bool dense_uses_mfma(const Plan &p, const void *K, const void *V, const void *q);

hipError_t launch_dense(const xkv_shape &s, const Plan &p, const void *K, const void *V, const void *q, float *part_o,
                        float *part_ml, hipStream_t st)
{
    if (dense_uses_mfma(p, K, V, q)) {
        dim3 grid(p.dense_splits, s.H_kv, s.batch), block(256);
        profile_begin(2, st);
        hipLaunchKernelGGL(dense_mfma_kernel, grid, block, 0, st, (const bf16_t *)K, (const bf16_t *)V,
                           (const bf16_t *)q, part_o, part_ml, s.L, s.H_kv, s.H_q, p.dense_splits, p.dense_chunk,
                           p.scale);
        profile_end(2, st);
        return hipGetLastError();
    }
    if (s.dtype == XKV_F32) return launch_dense_generic<float>(s, p, K, V, q, part_o, part_ml, st);
    return launch_dense_generic<bf16_t>(s, p, K, V, q, part_o, part_ml, st);
}

hipError_t launch_combine(const xkv_shape &s, int n_part, const float *part_o, const float *part_ml, void *out,
                          hipStream_t st, int n_part2, const float *part_o2, const float *part_ml2)
{
    if (n_part + n_part2 > kMaxCombineParts) return hipErrorInvalidValue;
    dim3 grid(s.H_q, s.batch), block(s.d_h <= 64 ? 64 : (s.d_h <= 128 ? 128 : 256));
    if (s.dtype == XKV_F32)
        hipLaunchKernelGGL(combine_kernel<float>, grid, block, 0, st, part_o, part_ml, (float *)out, s.H_q, s.d_h,
                           n_part, part_o2, part_ml2, n_part2);
    else
        hipLaunchKernelGGL(combine_kernel<bf16_t>, grid, block, 0, st, part_o, part_ml, (bf16_t *)out, s.H_q, s.d_h,
                           n_part, part_o2, part_ml2, n_part2);
    return hipGetLastError();
}

// Whether launch_dense takes the matrix-core kernel (one partial per split) or the general one (one per wavefront).
bool dense_uses_mfma(const Plan &p, const void *K, const void *V, const void *q)
{
    return p.dense_mfma && ((((uintptr_t)K | (uintptr_t)V | (uintptr_t)q)) & 15u) == 0;
}

}  // namespace xkv
