// Per-row ArgTopK by radix select on the monotone 32-bit image of the fp32 scores
// (App. B.1 Alg. 2, top-k step, applied per token).  Bit-exact and deterministic.
//
// A row of L scores is split into chunks; one workgroup owns one (row, chunk).  Four passes resolve the
// 32-bit key of the k-th largest element 8 bits at a time.  A pass histograms, per chunk, the current
// digit of the keys that still match the resolved prefix, keeps the chunk's histogram and adds it to the
// row's histogram with integer atomics (order-independent, so the result is deterministic).  Launch
// boundaries are the only synchronisation: every workgroup of the next launch reads the row histogram
// (1 KiB), finds the bin holding the k-th element, refines the prefix, and counts from its own chunk's
// stored histogram how many of its keys are thereby known to lie above the threshold.  The last launch
// knows the threshold key T and how many keys equal to T are still needed (ties go to the smaller token
// id), sums the counts of the chunks before its own and writes the selected ids in ascending order with
// wavefront ballots.
#include "xkv_common.h"

namespace xkv {

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// scratch arrays (uint32 words), carved by launch_topk
struct TopkScratch {
    uint32_t *hist;      // [rows][chunks][4][256] per-chunk digit histograms (level 3: suffix sums)
    uint32_t *state;     // [rows][8]  (prefix, k_rem) after each level
    uint32_t *row_hist;  // [rows][4][256] per-row digit histograms (zeroed by topk_init_kernel)
    uint32_t *chunk_gt;  // [rows][chunks] keys of the chunk above the threshold by levels 0..2
};

__global__ void topk_init_kernel(uint32_t *row_hist, int words)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;  // every level of every row
    if (i < words) row_hist[i] = 0;
}

// Inclusive suffix sum over the 256 bins held one per thread.  All 256 threads take part.
__device__ __forceinline__ uint32_t suffix_sum_256(uint32_t c, uint32_t *sh /* >= 4 words */)
{
    const int lane = lane_id(), w = wave_id();
    uint32_t s = c;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t nb = __shfl_down(s, off, kWave);
        if (lane + off < kWave) s += nb;
    }
    __syncthreads();  // sh may still be read by a previous use
    if (lane == 0) sh[w] = s;
    __syncthreads();
    for (int ww = w + 1; ww < 4; ++ww) s += sh[ww];
    return s;
}

// From the row histogram of `level`: the bin b with (#keys in bins above b) < k_rem <= (#keys in bins >= b).
__device__ __forceinline__ void resolve_level(const uint32_t *__restrict__ row_hist_level, uint32_t k_rem,
                                              uint32_t *sh /* >= 8 words */, uint32_t &digit, uint32_t &k_rem_out)
{
    const uint32_t c = row_hist_level[threadIdx.x];
    const uint32_t incl = suffix_sum_256(c, sh), above = incl - c;
    if (above < k_rem && k_rem <= incl) {
        sh[4] = threadIdx.x;
        sh[5] = k_rem - above;
    }
    __syncthreads();
    digit = sh[4];
    k_rem_out = sh[5];
}

template <int LEVEL>
__global__ __launch_bounds__(256) void topk_hist_kernel(const float *__restrict__ S, TopkScratch ws, int L, int k,
                                                        int chunks, int chunk)
{
    __shared__ uint32_t sh_hist[kTopkBins];
    __shared__ uint32_t sh_misc[8];
    const int row = blockIdx.y, c = blockIdx.x;
    uint32_t *row_hist = ws.row_hist + (size_t)row * kTopkLevels * kTopkBins;
    uint32_t *my_hist = ws.hist + ((size_t)row * chunks + c) * kTopkLevels * kTopkBins;
    uint32_t prefix = 0, k_rem = (uint32_t)k;
    if constexpr (LEVEL > 0) {
        if constexpr (LEVEL > 1) {
            prefix = ws.state[(size_t)row * kStateWords + 2 * (LEVEL - 2)];
            k_rem = ws.state[(size_t)row * kStateWords + 2 * (LEVEL - 2) + 1];
        }
        uint32_t digit, k_new;
        resolve_level(row_hist + (LEVEL - 1) * kTopkBins, k_rem, sh_misc, digit, k_new);
        prefix = (prefix << 8) | digit;
        k_rem = k_new;
        if (c == 0 && threadIdx.x == 0) {
            ws.state[(size_t)row * kStateWords + 2 * (LEVEL - 1)] = prefix;
            ws.state[(size_t)row * kStateWords + 2 * (LEVEL - 1) + 1] = k_rem;
        }
        // keys of this chunk that matched the old prefix and have a larger digit lie above the threshold
        const uint32_t mine = my_hist[(LEVEL - 1) * kTopkBins + threadIdx.x];
        const uint32_t incl = suffix_sum_256(threadIdx.x > digit ? mine : 0u, sh_misc);
        if (threadIdx.x == 0) {
            uint32_t *cg = ws.chunk_gt + (size_t)row * chunks + c;
            *cg = (LEVEL == 1 ? 0u : *cg) + incl;
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
    const uint32_t cnt = sh_hist[threadIdx.x];
    if (cnt != 0) atomicAdd(&row_hist[LEVEL * kTopkBins + threadIdx.x], cnt);
    if constexpr (LEVEL < 3) {
        my_hist[LEVEL * kTopkBins + threadIdx.x] = cnt;
    } else {
        // last level: keep the suffix sums, so that "keys above digit d" is one load for the writer
        my_hist[LEVEL * kTopkBins + threadIdx.x] = suffix_sum_256(cnt, sh_misc);
    }
}

__global__ __launch_bounds__(256) void topk_write_kernel(const float *__restrict__ S, TopkScratch ws,
                                                         int32_t *__restrict__ idx_out, int L, int k, int chunks,
                                                         int chunk)
{
    __shared__ uint32_t sh_misc[8];
    __shared__ uint32_t sh_red[2][4];
    __shared__ uint32_t sh_cnt[2][4];
    const int row = blockIdx.y, c = blockIdx.x;
    const uint32_t *row_hist = ws.row_hist + (size_t)row * kTopkLevels * kTopkBins;
    const uint32_t *hist_row = ws.hist + (size_t)row * chunks * kTopkLevels * kTopkBins;
    const uint32_t prefix = ws.state[(size_t)row * kStateWords + 4];
    const uint32_t k_rem = ws.state[(size_t)row * kStateWords + 5];
    uint32_t digit, need_eq;
    resolve_level(row_hist + 3 * kTopkBins, k_rem, sh_misc, digit, need_eq);
    const uint32_t T = (prefix << 8) | digit;  // key of the k-th largest element

    // selected keys of the chunks before this one: above T (levels 0..2 counted earlier, level 3 from the
    // stored suffix sums) and equal to T
    const int lane = lane_id(), w = wave_id();
    uint32_t gt = 0, eq = 0;
    for (int ch = threadIdx.x; ch < c; ch += 256) {
        const uint32_t *h3 = hist_row + ((size_t)ch * kTopkLevels + 3) * kTopkBins;
        const uint32_t ge = h3[digit], above = digit < 255u ? h3[digit + 1] : 0u;
        gt += ws.chunk_gt[(size_t)row * chunks + ch] + above;
        eq += ge - above;
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

// ------------------------------------------------------------------------------------------
// Rows of up to 65536 scores: the whole selection in one launch.  One workgroup of 16 wavefronts owns a row
// and keeps its keys in registers (NV per thread; wavefront w holds the contiguous segment
// [w 64 NV, (w+1) 64 NV), element j of a lane is w 64 NV + 64 j + lane), so the row is read from memory once
// and nothing but the ids is written.  The four 8-bit radix passes histogram into LDS counters that are
// replicated per lane pair ([bin][lane/2], two 16-bit halves per word: a lane position sees at most
// 16 NV <= 1024 keys), so the clustered top digits cost no serialised atomics; the replicas are summed, the
// first wavefront finds the bin of the k-th key, and the pass repeats on the next digit.  The ordered write
// is the same ballot scheme as topk_write_kernel, fed from the registers.
// ------------------------------------------------------------------------------------------
constexpr int kRowWaves = 16;

template <int NV>
__global__ __launch_bounds__(kRowWaves * 64) void topk_row_kernel(const float *__restrict__ S,
                                                                 int32_t *__restrict__ idx_out, int L, int k)
{
    __shared__ uint32_t hist[kTopkBins * 32];
    __shared__ uint32_t bins[kTopkBins];
    __shared__ uint32_t sh[3 + 2 * kRowWaves];
    const int row = blockIdx.x, tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const float *Srow = S + (size_t)row * L;
    const int base = w * 64 * NV + lane;

    uint32_t key[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int t = base + 64 * j;
        key[j] = __float_as_uint(Srow[t < L ? t : L - 1]);
        if (j % 8 == 7) __builtin_amdgcn_sched_barrier(0);  // bounds the address registers alive at once
    }
    // Positions beyond the row get key 0, below every real key (those are clamped to >= 1; only one NaN pattern
    // maps to 0): they can then be histogrammed and compared like the rest and are never selected, k <= L.
    // (Each phase recomputes its positions from an opaque copy of `base`; otherwise the compiler keeps all NV of
    // them in registers from the loads to the final write.)
    int base_v = base;
    asm volatile("" : "+v"(base_v));
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const uint32_t kk = order_key(__uint_as_float(key[j]));
        key[j] = base_v + 64 * j < L ? (kk > 1u ? kk : 1u) : 0u;
    }

    // Levels 0..2 histogram into `hist`.  While many keys still match the prefix the counters are replicated per
    // lane pair ([bin][lane/2], two 16-bit halves per word); once at most 4096 match (known exactly from the
    // previous level's bin count) a plain 256-word histogram is cheaper to clear and to sum.  Level 3 histograms
    // per wavefront ([wavefront][bin]), so that each wavefront can read off afterwards how many of its own keys
    // lie above / at the threshold without another pass over its registers.
    uint32_t prefix = 0, k_rem = (uint32_t)k, n_match = (uint32_t)L;
    uint32_t above24 = 0;  // level 3: keys of this wavefront whose upper 24 bits are already above the prefix
#pragma unroll
    for (int level = 0; level < kTopkLevels; ++level) {
        const bool per_wave = level == 3;
        const bool direct = !per_wave && level > 0 && n_match <= 4096u;  // uniform over the workgroup
        if (per_wave) {
            for (int i = tid; i < kRowWaves * kTopkBins; i += kRowWaves * 64) hist[i] = 0;
        } else if (direct) {
            if (tid < kTopkBins) hist[tid] = 0;
        } else {
            for (int i = tid; i < kTopkBins * 32; i += kRowWaves * 64) hist[i] = 0;
        }
        __syncthreads();
        const uint32_t inc = (per_wave || direct) ? 1u : 1u << (16 * (lane & 1));
        const uint32_t slot0 = per_wave ? (uint32_t)w * kTopkBins : direct ? 0u : (uint32_t)(lane >> 1);
        const uint32_t dmul = (per_wave || direct) ? 1u : 32u;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const uint32_t upper = level == 0 ? 0u : key[j] >> (32 - 8 * level);
            const bool match = level == 0 || upper == prefix;
            const uint32_t digit = (key[j] >> (24 - 8 * level)) & 0xFFu;
            if (match) atomicAdd(&hist[digit * dmul + slot0], inc);
            if (level == 3) {
                above24 += (uint32_t)__popcll(__ballot(upper > prefix));
                asm volatile("" : "+s"(above24));
            }
            if (j % 4 == 3) __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        if (per_wave) {
            if (tid < kTopkBins) {
                uint32_t sum = 0;
#pragma unroll
                for (int ww = 0; ww < kRowWaves; ++ww) sum += hist[ww * kTopkBins + tid];
                bins[tid] = sum;
            }
        } else if (direct) {
            if (tid < kTopkBins) bins[tid] = hist[tid];
        } else {  // sum the replicas: four threads per bin, eight words each
            const int bin = tid >> 2, part = tid & 3;
            uint32_t sum = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t v = hist[bin * 32 + part * 8 + i];
                sum += (v & 0xFFFFu) + (v >> 16);
            }
            sum += __shfl_xor(sum, 1, kWave);
            sum += __shfl_xor(sum, 2, kWave);
            if (part == 0) bins[bin] = sum;
        }
        __syncthreads();
        if (w == 0) {  // the bin b with (#keys in bins above b) < k_rem <= (#keys in bins >= b)
            uint32_t c[4], tot = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                c[i] = bins[4 * lane + i];
                tot += c[i];
            }
            uint32_t sfx = tot;  // keys in the bins of this lane and of all higher lanes
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t nb = __shfl_down(sfx, off, kWave);
                if (lane + off < kWave) sfx += nb;
            }
            uint32_t above = sfx - tot;
#pragma unroll
            for (int i = 3; i >= 0; --i) {
                const uint32_t incl = above + c[i];
                if (above < k_rem && k_rem <= incl) {
                    sh[0] = (uint32_t)(4 * lane + i);
                    sh[1] = k_rem - above;
                    sh[2] = c[i];
                }
                above = incl;
            }
        }
        __syncthreads();
        prefix = (prefix << 8) | sh[0];
        k_rem = sh[1];
        n_match = sh[2];
    }
    const uint32_t T = prefix, need_eq = k_rem;  // key of the k-th largest; how many keys equal to it are taken

    // keys above / equal to T in this wavefront's segment: those above in the upper 24 bits were counted during
    // the last pass, the rest sit in the wavefront's own level-3 histogram (lane l sums bins 4l .. 4l+3)
    uint32_t my_gt, my_eq;
    {
        const uint32_t d3 = T & 0xFFu;
        uint32_t g = 0, e = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t bin = 4 * lane + i, c = hist[w * kTopkBins + bin];
            g += bin > d3 ? c : 0u;
            e += bin == d3 ? c : 0u;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            g += __shfl_xor(g, off, kWave);
            e += __shfl_xor(e, off, kWave);
        }
        my_gt = above24 + g;
        my_eq = e;
    }
    if (lane == 0) {
        sh[3 + w] = my_gt;
        sh[3 + kRowWaves + w] = my_eq;
    }
    __syncthreads();
    uint32_t gt_run = 0, eq_run = 0;
    for (int ww = 0; ww < w; ++ww) {
        gt_run += sh[3 + ww];
        eq_run += sh[3 + kRowWaves + ww];
    }
    int32_t *out = idx_out + (size_t)row * k;
    // The comparisons are redone rather than kept: 2 NV lane masks would not fit the scalar registers.  The empty
    // statement hides from the compiler that Tw is T.
    uint32_t Tw = T;
    int base_w = base;
    asm volatile("" : "+v"(Tw), "+v"(base_w));
    if (my_eq == 0) {
        // no key of this segment equals the threshold (the usual case): only the keys above it matter
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const bool is_gt = key[j] > Tw;
            const uint64_t mg = __ballot(is_gt);
            if (is_gt) {
                const uint32_t pos = gt_run + lanes_below(mg) + (eq_run < need_eq ? eq_run : need_eq);
                if (pos < (uint32_t)k) out[pos] = base_w + 64 * j;
            }
            gt_run += (uint32_t)__popcll(mg);
            if (j % 4 == 3) __builtin_amdgcn_sched_barrier(0);
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int t = base_w + 64 * j;
        const bool is_gt = key[j] > Tw, is_eq = key[j] == Tw;
        const uint64_t mg = __ballot(is_gt), me = __ballot(is_eq);
        const uint32_t gt_me = gt_run + lanes_below(mg), eq_me = eq_run + lanes_below(me);
        if (is_gt || (is_eq && eq_me < need_eq)) {
            const uint32_t pos = gt_me + (eq_me < need_eq ? eq_me : need_eq);
            if (pos < (uint32_t)k) out[pos] = t;
        }
        gt_run += (uint32_t)__popcll(mg);
        eq_run += (uint32_t)__popcll(me);
        if (j % 4 == 3) __builtin_amdgcn_sched_barrier(0);
    }
}

bool topk_row_shape_ok(const xkv_shape &s) { return s.L <= kRowWaves * 64 * 64; }

template <int NV>
static void launch_topk_row_t(const xkv_shape &s, const Plan &p, const float *S, int32_t *idx, hipStream_t st)
{
    hipLaunchKernelGGL(topk_row_kernel<NV>, dim3(p.rows), dim3(kRowWaves * 64), 0, st, S, idx, s.L, s.k);
}

hipError_t launch_topk_init(const Plan &p, uint32_t *state, hipStream_t st)
{
    const int words = p.rows * kTopkLevels * kTopkBins;
    hipLaunchKernelGGL(topk_init_kernel, dim3((words + 255) / 256), dim3(256), 0, st, topk_row_hist(p, state), words);
    return hipGetLastError();
}

hipError_t launch_topk(const xkv_shape &s, const Plan &p, const float *S, int32_t *idx, uint32_t *hist,
                       uint32_t *state, bool level0_done, hipStream_t st)
{
    if (p.topk_row) {
        const int per_thread = (s.L + kRowWaves * 64 - 1) / (kRowWaves * 64);
        if (per_thread <= 8)
            launch_topk_row_t<8>(s, p, S, idx, st);
        else if (per_thread <= 16)
            launch_topk_row_t<16>(s, p, S, idx, st);
        else if (per_thread <= 32)
            launch_topk_row_t<32>(s, p, S, idx, st);
        else
            launch_topk_row_t<64>(s, p, S, idx, st);
        return hipGetLastError();
    }
    TopkScratch ws;
    ws.hist = hist;
    ws.state = state;
    ws.row_hist = topk_row_hist(p, state);
    ws.chunk_gt = ws.row_hist + (size_t)p.rows * kTopkLevels * kTopkBins;
    dim3 grid(p.topk_chunks, p.rows), block(256);
    if (!level0_done) {
        hipError_t e = launch_topk_init(p, state, st);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(topk_hist_kernel<0>, grid, block, 0, st, S, ws, s.L, s.k, p.topk_chunks, p.topk_chunk);
    }
    hipLaunchKernelGGL(topk_hist_kernel<1>, grid, block, 0, st, S, ws, s.L, s.k, p.topk_chunks, p.topk_chunk);
    hipLaunchKernelGGL(topk_hist_kernel<2>, grid, block, 0, st, S, ws, s.L, s.k, p.topk_chunks, p.topk_chunk);
    hipLaunchKernelGGL(topk_hist_kernel<3>, grid, block, 0, st, S, ws, s.L, s.k, p.topk_chunks, p.topk_chunk);
    hipLaunchKernelGGL(topk_write_kernel, grid, block, 0, st, S, ws, idx, s.L, s.k, p.topk_chunks, p.topk_chunk);
    return hipGetLastError();
}

}  // namespace xkv
