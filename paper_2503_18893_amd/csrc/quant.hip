// 4-bit and 3-bit round-to-nearest quantisation of rows of the token basis A (App. "Integrate with Quantization": a
// plain RTN quantiser on the compressed cache, 25.6x at 4 bits and 32x at 3 bits; the formats below are what the two
// published ratios imply -- one extra bit per element of side information = two 16-bit numbers per group of 32).
//
// 3-bit row layout: one 16-byte piece per group of 32 ranks -- 96 bits of codes (little-endian over three words),
// then the word (step, lo) of two bf16 -- so r/2 bytes per row.  The 96 bits are four units of 24 bits, unit u for
// ranks 8u..8u+7 of the group; inside a unit the even ranks sit in the low 12 bits (rank 8u+2i at bits [3i, 3i+3))
// and the odd ranks in the high 12 (rank 8u+2i+1 at bits [12+3i, 12+3i+3)), so that moving the high half up to bit
// 16 gives the same "two adjacent ranks 16 bits apart" word as the 4-bit format.  step = bf16((max - lo) / 7).
//
// 4-bit row layout, r a multiple of 32:  r/8 32-bit words of codes (word j holds ranks 8j..8j+7: rank 8j+2i in bits
// [4i, 4i+4), rank 8j+2i+1 in bits [16+4i, 16+4i+4), so two adjacent ranks are one shift and one mask away from a
// packed pair of 16-bit numbers), then r/32 pairs (step, lo) of bf16: 5r/8 bytes, then zero bytes up to the next
// multiple of 16 (none when r is a multiple of 128), so that every row and every group is 16-byte aligned.
//   lo = min of the group, step = bf16((max - lo) / 15) (1 if that is 0), code = clip(rint((x - lo) * (1 / step)), 0, 15),
// each a single fp32 operation (the same sequence as the CPU oracle: the codes agree bit for bit);  x^ = step * code + lo.
#include "xkv_common.h"

namespace xkv {

typedef __attribute__((ext_vector_type(4))) uint32_t q_u32x4_t;

// One lane per 16-byte piece (8 ranks); the four lanes of a group share min and max through two exchanges.  A
// wavefront reads 1 KiB of contiguous input and writes 256 B of codes and 64 B of parameters, both contiguous (4-bit
// rows), or 256 B of whole group pieces (3-bit rows).
template <int BITS>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const bf16_t *__restrict__ X, unsigned char *__restrict__ out,
                                                            long long pieces, int r)
{
    constexpr float kQmax = (float)((1 << BITS) - 1);
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
    float step = bf16_to_f32(f32_to_bf16((mx - lo) / kQmax));
    step = step > 0.0f ? step : 1.0f;
    const float inv = 1.0f / step;
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float t = (x[e] - lo) * inv;
        const float c = fminf(fmaxf(rintf(t), 0.0f), kQmax);
        // even ranks in the low half, odd ranks in the high half (16 bits up for 4-bit codes, 12 for 3-bit codes)
        word |= (uint32_t)c << (BITS * (e >> 1) + (BITS == 4 ? 16 : 12) * (e & 1));
    }
    if constexpr (BITS == 3) {
        // the group's four 24-bit units into three words; the group's first lane writes the 16-byte piece
        const uint32_t u1 = __shfl_down(word, 1, kWave), u2 = __shfl_down(word, 2, kWave), u3 = __shfl_down(word, 3, kWave);
        if (!in || (pc & 3) != 0) return;
        q_u32x4_t piece;
        piece[0] = word | (u1 << 24);
        piece[1] = (u1 >> 8) | (u2 << 16);
        piece[2] = (u2 >> 16) | (u3 << 8);
        piece[3] = (uint32_t)f32_to_bf16(step) | ((uint32_t)f32_to_bf16(lo) << 16);
        *reinterpret_cast<q_u32x4_t *>(out + row * (long long)(r >> 1) + (long long)(pc >> 2) * 16) = piece;
        return;
    }
    if (!in) return;
    unsigned char *orow = out + row * (long long)quant_row_bytes(r);
    reinterpret_cast<uint32_t *>(orow)[pc] = word;
    if ((pc & 3) == 0)
        reinterpret_cast<uint32_t *>(orow + (r >> 1))[pc >> 2] = (uint32_t)f32_to_bf16(step) | ((uint32_t)f32_to_bf16(lo) << 16);
    if (pc == 0)  // the row's padding
        for (int i = (r >> 3) + (r >> 5); i < (int)(quant_row_bytes(r) >> 2); ++i) reinterpret_cast<uint32_t *>(orow)[i] = 0u;
}

hipError_t launch_quantize_rows(const void *X, long long rows, int r, int bits, void *out, hipStream_t st)
{
    const long long pieces = rows * (long long)(r >> 3);
    if (pieces == 0) return hipSuccess;
    const long long blocks = (pieces + 255) / 256;
    if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    if (bits == 3)
        hipLaunchKernelGGL(quantize_rows_kernel<3>, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t *)X,
                           (unsigned char *)out, pieces, r);
    else
        hipLaunchKernelGGL(quantize_rows_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t *)X,
                           (unsigned char *)out, pieces, r);
    return hipGetLastError();
}

}  // namespace xkv
