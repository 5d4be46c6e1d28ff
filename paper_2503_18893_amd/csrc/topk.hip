// Per-row ArgTopK by radix select on the monotone 32-bit image of the fp32 scores
// (App. B.1 Alg. 2, top-k step, applied per token).  Bit-exact, deterministic, no global atomics.
//
// A row of L scores is split into chunks; one workgroup owns one (row, chunk).  Four passes
// resolve the 32-bit key of the k-th largest element 8 bits at a time: each pass histograms,
// per chunk, the current digit of the keys that still match the resolved prefix.  The next
// launch sums the per-chunk histograms of its row (every workgroup redundantly, so that no
// cross-workgroup wait exists), finds the bin holding the k-th element and refines the prefix.
// The last launch knows the threshold key T and how many keys equal to T are still needed
// (ties go to the smaller token id), derives each chunk's output offset from the stored
// histograms and writes the selected ids in ascending order using wavefront ballots.
#include "xkv_common.h"

namespace xkv {

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Sum the per-chunk histograms of `level` for this row and find the bin b with
// (#keys in bins above b) < k_rem <= (#keys in bins >= b).  All 256 threads take part.
__device__ __forceinline__ void resolve_level(const uint32_t *__restrict__ hist_row, int chunks, int level,
                                              uint32_t k_rem, uint32_t *sh /* >= 8 words */, uint32_t &digit,
                                              uint32_t &k_rem_out)
{
    const int b = threadIdx.x, lane = lane_id(), w = wave_id();
    uint32_t c = 0;
    for (int ch = 0; ch < chunks; ++ch) c += hist_row[((size_t)ch * kTopkLevels + level) * kTopkBins + b];
    uint32_t s = c;  // inclusive suffix sum inside the wavefront
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t n = __shfl_down(s, off, kWave);
        if (lane + off < kWave) s += n;
    }
    __syncthreads();  // sh may still be read by a previous use
    if (lane == 0) sh[w] = s;
    __syncthreads();
    uint32_t higher = 0;
    for (int ww = w + 1; ww < 4; ++ww) higher += sh[ww];
    const uint32_t incl = s + higher, above = incl - c;
    if (above < k_rem && k_rem <= incl) {
        sh[4] = (uint32_t)b;
        sh[5] = k_rem - above;
    }
    __syncthreads();
    digit = sh[4];
    k_rem_out = sh[5];
}

template <int LEVEL>
__global__ __launch_bounds__(256) void topk_hist_kernel(const float *__restrict__ S, uint32_t *__restrict__ hist,
                                                        uint32_t *__restrict__ state, int L, int k, int chunks,
                                                        int chunk)
{
    __shared__ uint32_t sh_hist[kTopkBins];
    __shared__ uint32_t sh_misc[8];
    const int row = blockIdx.y, c = blockIdx.x;
    uint32_t *hist_row = hist + (size_t)row * chunks * kTopkLevels * kTopkBins;
    uint32_t prefix = 0, k_rem = (uint32_t)k;
    if constexpr (LEVEL > 0) {
        if constexpr (LEVEL > 1) {
            prefix = state[(size_t)row * kStateWords + 2 * (LEVEL - 2)];
            k_rem = state[(size_t)row * kStateWords + 2 * (LEVEL - 2) + 1];
        }
        uint32_t digit, k_new;
        resolve_level(hist_row, chunks, LEVEL - 1, k_rem, sh_misc, digit, k_new);
        prefix = (prefix << 8) | digit;
        k_rem = k_new;
        if (c == 0 && threadIdx.x == 0) {
            state[(size_t)row * kStateWords + 2 * (LEVEL - 1)] = prefix;
            state[(size_t)row * kStateWords + 2 * (LEVEL - 1) + 1] = k_rem;
        }
    }
    sh_hist[threadIdx.x] = 0;
    __syncthreads();
    const float *Srow = S + (size_t)row * L;
    const int lane = lane_id();
    const int base = c * chunk;
    for (int i0 = 0; i0 < chunk; i0 += 1024) {  // chunk is a multiple of 256: every trip count is uniform
        float val[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {  // four independent coalesced loads in flight
            const int t = base + i0 + u * 256 + (int)threadIdx.x;
            val[u] = (i0 + u * 256 < chunk && t < L) ? Srow[t] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (i0 + u * 256 >= chunk) break;
            const int t = base + i0 + u * 256 + (int)threadIdx.x;
            const uint32_t key = order_key(val[u]);
            bool active = t < L;
            if constexpr (LEVEL > 0) active = active && ((key >> (32 - 8 * LEVEL)) == prefix);
            const uint32_t digit = (key >> (24 - 8 * LEVEL)) & 0xFFu;
            // scores cluster in few bins at the top levels: add the leader's bin once per wavefront
            const uint64_t m = __ballot(active);
            if (m != 0) {
                const int first = __ffsll((unsigned long long)m) - 1;
                const uint32_t d0 = __shfl(digit, first, kWave);
                const uint64_t same = __ballot(active && digit == d0);
                if (lane == first) atomicAdd(&sh_hist[d0], (uint32_t)__popcll(same));
                if (active && digit != d0) atomicAdd(&sh_hist[digit], 1u);
            }
        }
    }
    __syncthreads();
    hist_row[((size_t)c * kTopkLevels + LEVEL) * kTopkBins + threadIdx.x] = sh_hist[threadIdx.x];
}

__global__ __launch_bounds__(256) void topk_write_kernel(const float *__restrict__ S,
                                                         const uint32_t *__restrict__ hist,
                                                         const uint32_t *__restrict__ state,
                                                         int32_t *__restrict__ idx_out, int L, int k, int chunks,
                                                         int chunk)
{
    __shared__ uint32_t sh_misc[8];
    __shared__ uint32_t sh_red[2][4];
    __shared__ uint32_t sh_cnt[2][4];
    const int row = blockIdx.y, c = blockIdx.x;
    const uint32_t *hist_row = hist + (size_t)row * chunks * kTopkLevels * kTopkBins;
    uint32_t prefix = state[(size_t)row * kStateWords + 4];
    uint32_t k_rem = state[(size_t)row * kStateWords + 5];
    uint32_t digit, need_eq;
    resolve_level(hist_row, chunks, 3, k_rem, sh_misc, digit, need_eq);
    const uint32_t T = (prefix << 8) | digit;  // key of the k-th largest element

    // selected elements that precede this chunk: keys above T (found level by level) and keys equal to T
    const int lane = lane_id(), w = wave_id();
    const uint32_t b = threadIdx.x;
    uint32_t gt = 0, eq = 0;
    for (int ch = 0; ch < c; ++ch) {
        const uint32_t *h = hist_row + (size_t)ch * kTopkLevels * kTopkBins;
#pragma unroll
        for (int lv = 0; lv < kTopkLevels; ++lv) {
            const uint32_t dl = (T >> (24 - 8 * lv)) & 0xFFu;
            if (b > dl) gt += h[lv * kTopkBins + b];
            if (lv == 3 && b == dl) eq += h[lv * kTopkBins + b];
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        gt += __shfl_xor(gt, off, kWave);
        eq += __shfl_xor(eq, off, kWave);
    }
    if (lane == 0) {
        sh_red[0][w] = gt;
        sh_red[1][w] = eq;
    }
    __syncthreads();
    const uint32_t gt_before = sh_red[0][0] + sh_red[0][1] + sh_red[0][2] + sh_red[0][3];
    const uint32_t eq_before = sh_red[1][0] + sh_red[1][1] + sh_red[1][2] + sh_red[1][3];

    // each wavefront owns a contiguous quarter of the chunk; first count, then write in order
    const float *Srow = S + (size_t)row * L;
    const int sub = chunk / 4;
    const int begin = c * chunk + w * sub;
    uint32_t my_gt = 0, my_eq = 0;
    for (int i0 = 0; i0 < sub; i0 += 4 * kWave) {  // sub is a multiple of 64
        float val[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = begin + i0 + u * kWave + lane;
            val[u] = (i0 + u * kWave < sub && t < L) ? Srow[t] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = begin + i0 + u * kWave + lane;
            const bool in = i0 + u * kWave < sub && t < L;
            const uint32_t key = order_key(val[u]);
            my_gt += (uint32_t)__popcll(__ballot(in && key > T));
            my_eq += (uint32_t)__popcll(__ballot(in && key == T));
        }
    }
    if (lane == 0) {
        sh_cnt[0][w] = my_gt;
        sh_cnt[1][w] = my_eq;
    }
    __syncthreads();
    uint32_t gt_run = gt_before, eq_run = eq_before;
    for (int ww = 0; ww < w; ++ww) {
        gt_run += sh_cnt[0][ww];
        eq_run += sh_cnt[1][ww];
    }
    int32_t *out = idx_out + (size_t)row * k;
    for (int i0 = 0; i0 < sub; i0 += 4 * kWave) {
        float val[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = begin + i0 + u * kWave + lane;
            val[u] = (i0 + u * kWave < sub && t < L) ? Srow[t] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = begin + i0 + u * kWave + lane;
            const bool in = i0 + u * kWave < sub && t < L;
            const uint32_t key = order_key(val[u]);
            const bool is_gt = in && key > T, is_eq = in && key == T;
            const uint64_t mg = __ballot(is_gt), me = __ballot(is_eq);
            const uint32_t gt_me = gt_run + lanes_below(mg), eq_me = eq_run + lanes_below(me);
            if (is_gt || (is_eq && eq_me < need_eq)) {
                const uint32_t pos = gt_me + (eq_me < need_eq ? eq_me : need_eq);
                if (pos < (uint32_t)k) out[pos] = t;
            }
            gt_run += (uint32_t)__popcll(mg);
            eq_run += (uint32_t)__popcll(me);
        }
    }
}

hipError_t launch_topk(const xkv_shape &s, const Plan &p, const float *S, int32_t *idx, uint32_t *hist,
                       uint32_t *state, hipStream_t st)
{
    dim3 grid(p.topk_chunks, p.rows), block(256);
    hipLaunchKernelGGL(topk_hist_kernel<0>, grid, block, 0, st, S, hist, state, s.L, s.k, p.topk_chunks, p.topk_chunk);
    hipLaunchKernelGGL(topk_hist_kernel<1>, grid, block, 0, st, S, hist, state, s.L, s.k, p.topk_chunks, p.topk_chunk);
    hipLaunchKernelGGL(topk_hist_kernel<2>, grid, block, 0, st, S, hist, state, s.L, s.k, p.topk_chunks, p.topk_chunk);
    hipLaunchKernelGGL(topk_hist_kernel<3>, grid, block, 0, st, S, hist, state, s.L, s.k, p.topk_chunks, p.topk_chunk);
    hipLaunchKernelGGL(topk_write_kernel, grid, block, 0, st, S, hist, state, idx, s.L, s.k, p.topk_chunks,
                       p.topk_chunk);
    return hipGetLastError();
}

}  // namespace xkv
