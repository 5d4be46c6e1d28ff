// Dense reconstruction X^_l = A B_l for all L tokens (Sec. 3.2), written head-major
// [batch][H_kv][L][d_h].  Builds the uncompressed cache the dense baseline reads.
#include "xkv_common.h"

namespace xkv {

// 64 x 64 output tile per workgroup, 4 x 4 outputs per thread, rank walked 16 at a time via LDS.
template <typename T>
__global__ __launch_bounds__(256) void reconstruct_kernel(const T *__restrict__ A,  // [batch][L][r]
                                                          const T *__restrict__ B,  // [batch][G][r][d]
                                                          T *__restrict__ X,        // [batch][H_kv][L][d_h]
                                                          int G, int layer, int L, int r, int H_kv, int d_h)
{
    __shared__ float sA[16][64 + 1];
    __shared__ float sB[16][64 + 1];
    const int b = blockIdx.z, d = H_kv * d_h;
    const int t0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const T *Ab = A + (size_t)b * L * r;
    const T *Bb = B + ((size_t)b * G + layer) * r * d;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] = 0.0f;

    for (int i0 = 0; i0 < r; i0 += 16) {
        for (int e = threadIdx.x; e < 64 * 16; e += 256) {
            const int tt = e / 16, ii = e % 16;  // A tile: consecutive threads read along the rank
            const int t = t0 + tt, i = i0 + ii;
            sA[ii][tt] = (t < L && i < r) ? to_f32(Ab[(size_t)t * r + i]) : 0.0f;
            const int i2 = e / 64, cc = e % 64;  // B tile: consecutive threads read along the columns
            const int ib = i0 + i2, c = c0 + cc;
            sB[i2][cc] = (ib < r && c < d) ? to_f32(Bb[(size_t)ib * d + c]) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int ii = 0; ii < 16; ++ii) {
            float av[4], bv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) av[a] = sA[ii][ty * 4 + a];
#pragma unroll
            for (int c = 0; c < 4; ++c) bv[c] = sB[ii][tx * 4 + c];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[a][c] = fmaf(av[a], bv[c], acc[a][c]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int t = t0 + ty * 4 + a;
        if (t >= L) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int col = c0 + tx * 4 + c;
            if (col >= d) continue;
            const int g = col / d_h, j = col % d_h;
            X[(((size_t)b * H_kv + g) * L + t) * d_h + j] = from_f32<T>(acc[a][c]);
        }
    }
}

hipError_t launch_reconstruct(const xkv_shape &s, int layer, const void *A, const void *B, int r, void *X,
                              hipStream_t st)
{
    const int d = s.H_kv * s.d_h;
    dim3 grid((d + 63) / 64, (s.L + 63) / 64, s.batch), block(256);
    if (s.dtype == XKV_F32)
        hipLaunchKernelGGL(reconstruct_kernel<float>, grid, block, 0, st, (const float *)A, (const float *)B,
                           (float *)X, s.G, layer, s.L, r, s.H_kv, s.d_h);
    else
        hipLaunchKernelGGL(reconstruct_kernel<bf16_t>, grid, block, 0, st, (const bf16_t *)A, (const bf16_t *)B,
                           (bf16_t *)X, s.G, layer, s.L, r, s.H_kv, s.d_h);
    return hipGetLastError();
}

}  // namespace xkv
