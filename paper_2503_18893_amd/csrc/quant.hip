// 4-bit round-to-nearest quantisation of rows of the token basis A (App. "Integrate with Quantization": a plain
// RTN quantiser on the compressed cache; the format below is the one the two published ratios imply -- one extra
// bit per element of side information = two 16-bit numbers per group of 32 elements).
//
// Row layout, r a multiple of 32:  r/8 32-bit words of codes (word j holds ranks 8j..8j+7: rank 8j+2i in bits
// [4i, 4i+4), rank 8j+2i+1 in bits [16+4i, 16+4i+4), so two adjacent ranks are one shift and one mask away from a
// packed pair of 16-bit numbers), then r/32 pairs (step, lo) of bf16: 5r/8 bytes, then zero bytes up to the next
// multiple of 16 (none when r is a multiple of 128), so that every row and every group is 16-byte aligned.
//   lo = min of the group, step = bf16((max - lo) / 15) (1 if that is 0), code = clip(rint((x - lo) * (1 / step)), 0, 15),
// each a single fp32 operation (the same sequence as the CPU oracle: the codes agree bit for bit);  x^ = step * code + lo.
#include "xkv_common.h"

namespace xkv {

typedef __attribute__((ext_vector_type(4))) uint32_t q_u32x4_t;

// One lane per 16-byte piece (8 ranks); the four lanes of a group share min and max through two exchanges.  A
// wavefront reads 1 KiB of contiguous input and writes 256 B of codes and 64 B of parameters, both contiguous.
__global__ __launch_bounds__(256) void quantize_rows_q4_kernel(const bf16_t *__restrict__ X, unsigned char *__restrict__ out,
                                                               long long pieces, int r)
{
    const long long p = (long long)blockIdx.x * 256 + threadIdx.x;
    // pieces is a multiple of 4 (r % 32 == 0), so a group's four lanes are all inside or all outside
    const bool in = p < pieces;
    const int ppr = r >> 3;  // pieces per row
    const long long row = (in ? p : 0) / ppr;
    const int pc = (int)((in ? p : 0) % ppr);
    const q_u32x4_t raw = in ? *reinterpret_cast<const q_u32x4_t *>(X + row * r + (long long)pc * 8) : q_u32x4_t{0u, 0u, 0u, 0u};
    float x[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = __uint_as_float(raw[e] << 16);
        x[2 * e + 1] = __uint_as_float(raw[e] & 0xFFFF0000u);
    }
    float mn = x[0], mx = x[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) {
        mn = fminf(mn, x[e]);
        mx = fmaxf(mx, x[e]);
    }
#pragma unroll
    for (int off = 1; off <= 2; off <<= 1) {
        mn = fminf(mn, __shfl_xor(mn, off, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    }
    const float lo = mn;  // a bf16 value
    float step = bf16_to_f32(f32_to_bf16((mx - lo) / 15.0f));
    step = step > 0.0f ? step : 1.0f;
    const float inv = 1.0f / step;
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float t = (x[e] - lo) * inv;
        const float c = fminf(fmaxf(rintf(t), 0.0f), 15.0f);
        word |= (uint32_t)c << (4 * (e >> 1) + 16 * (e & 1));
    }
    if (!in) return;
    unsigned char *orow = out + row * (long long)quant_row_bytes(r);
    reinterpret_cast<uint32_t *>(orow)[pc] = word;
    if ((pc & 3) == 0)
        reinterpret_cast<uint32_t *>(orow + (r >> 1))[pc >> 2] = (uint32_t)f32_to_bf16(step) | ((uint32_t)f32_to_bf16(lo) << 16);
    if (pc == 0)  // the row's padding
        for (int i = (r >> 3) + (r >> 5); i < (int)(quant_row_bytes(r) >> 2); ++i) reinterpret_cast<uint32_t *>(orow)[i] = 0u;
}

hipError_t launch_quantize_rows(const void *X, long long rows, int r, void *out, hipStream_t st)
{
    const long long pieces = rows * (long long)(r >> 3);
    if (pieces == 0) return hipSuccess;
    const long long blocks = (pieces + 255) / 256;
    if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(quantize_rows_q4_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t *)X,
                       (unsigned char *)out, pieces, r);
    return hipGetLastError();
}

}  // namespace xkv
