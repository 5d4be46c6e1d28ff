// factorize.hip -- Cross-Layer Factorization (Sec. 3.1, Eq. 1) on the GPU: the caches of the G layers of a
// group, concatenated along the feature axis into X_cat [L][n] (n = G * H_kv * d_h), are replaced by a shared
// token basis A [L][r] and per-layer reconstruction matrices B_l [r][d] with A [B_1 .. B_G] the best rank-r
// approximation of X_cat.
//
// How it is computed here.  n is a few thousand while L is tens of thousands, so the right singular subspace
// is taken from the n x n Gram matrix C = X_cat^T X_cat, which is built once on the matrix cores and then
// stays in cache:
//   1. X_cat is rewritten channel-major (Xt [n][Lp], tokens contiguous, zero-padded to a multiple of 64) so
//      that both operands of the Gram product are contiguous along the summation index;
//   2. C = Xt Xt^T (lower tiles, split over the tokens, fp32 accumulation), mirrored to the full matrix;
//   3. block power iteration on C: V <- orth(C V) for a random start V [r][n], `iters` times.  The product
//      runs on the fp32 matrix cores; orth() is a Cholesky-QR in fp64 (Gram matrix of the r vectors,
//      Cholesky factor, forward substitution), which keeps r directions apart whose lengths differ by many
//      orders of magnitude after the multiplication by C;
//   4. B = V rounded to the storage type (rows of B are an orthonormal basis of the dominant right singular
//      subspace), A = X_cat B^T (matrix cores again).
// A B is then X_cat projected onto the span of B's rows.  The factors differ from (U Sigma, V^T) of Eq. 1 by an
// r x r rotation inside that span, which leaves every product A B_l, and with it every quantity the decode path
// computes, unchanged.  (Randomised subspace iteration with Cholesky-QR is also what App. B.3 describes for
// the paper's own implementation; working on the Gram matrix instead of X_cat is this implementation's choice.)
#include "xkv_common.h"

#include <algorithm>

namespace xkv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 fz_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float fz_f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t fz_u32x4_t;
typedef __attribute__((ext_vector_type(4))) float fz_f32x4_t;
typedef __attribute__((address_space(3))) void fz_lds_void_t;

__device__ __forceinline__ void fz_copy16_global_to_lds(const void *gptr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(gptr) : "memory", "m0");
}
// s_waitcnt bounding only the number of outstanding vector-memory operations (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
#define FZ_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (7 << 4) | (0xF << 8) | (((n) >> 4) << 14))

__device__ __forceinline__ void fz_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ------------------------------------------------------------------------------------------------
// (1) X [G*H_kv][L][d_h] (one sequence, every layer and head of the group) -> Xt [n][Lp], row
//     cb * d_h + j = channel j of column block cb, zero beyond token L.  64 x 64 tiles through LDS.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void xt_pack_kernel(const T *__restrict__ X, T *__restrict__ Xt, int L, int Lp, int d_h,
                                                      long long x_seq, long long xt_seq)
{
    X += (size_t)blockIdx.z * x_seq;
    Xt += (size_t)blockIdx.z * xt_seq;
    constexpr int V = 16 / sizeof(T);  // elements per 16 B
    constexpr int PPR = 64 / V;        // 16 B pieces per tile row
    __shared__ __attribute__((aligned(16))) T tile[64][64 + V];
    const int t0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    const int cb = n0 / d_h, c0 = n0 % d_h;
    const T *src = X + (size_t)cb * L * d_h + c0;
    for (int i = threadIdx.x; i < 64 * PPR; i += 256) {
        const int tt = i / PPR, p = i % PPR;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (t0 + tt < L) v = *reinterpret_cast<const uint4 *>(src + (size_t)(t0 + tt) * d_h + p * V);
        *reinterpret_cast<uint4 *>(&tile[tt][p * V]) = v;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * PPR; i += 256) {
        const int c = i / PPR, p = i % PPR;
        __attribute__((aligned(16))) T vals[V];
#pragma unroll
        for (int e = 0; e < V; ++e) vals[e] = tile[p * V + e][c];
        *reinterpret_cast<uint4 *>(Xt + (size_t)(n0 + c) * Lp + t0 + p * V) = *reinterpret_cast<const uint4 *>(vals);
    }
}

// ------------------------------------------------------------------------------------------------
// (2) out[m][n] = sum_k P[m][k] Q[n][k] on the matrix cores, both operands contiguous along k.
//
// Element (row, k) of an operand lives at base + (k / kbw) * kblk + row * pitch + k % kbw: a plain row-major
// matrix has kbw = K, and a cache stored as [column block][token][d_h] is read as X_cat [token][n] with
// kbw = d_h, kblk = L * d_h, pitch = d_h.  K is consumed in slabs of 128 B per row (64 bf16 or 32 fp32
// values); kbw is a multiple of the slab.
//
// Workgroup: 8 wavefronts, a 256 x 256 output tile, wavefront (wm, wn) owns rows 64 wm .. +63 and columns
// 128 wn .. +127 as 2 x 4 accumulator tiles of 32 x 32.  A slab of the 256 + 256 operand rows (64 KiB) is
// copied global -> LDS directly, two stages: one copy instruction moves 8 rows x 128 B, lane l fetching the 16 B
// piece (l % 8) ^ (row / 2) % 8 of row l / 8, so that a row's pieces sit in LDS xor-swizzled by (row / 2) % 8 and
// the fragment reads (consecutive rows, same piece) spread over all 64 banks.  Rows beyond the operand's end are
// clamped to its last row; what they produce is never stored.
// Output: fp32 partial planes out_f32[split][m][n] (summed by a second kernel), or, with one split, the
// final matrix in fp32 or bf16.  With lower_only (P == Q) only tiles on or below the diagonal are computed.
// ------------------------------------------------------------------------------------------------
struct GemmOperand {
    const void *base;
    long long pitch, kblk;  // elements
    int kbw, rows;
    long long seq;  // elements between the matrices of consecutive sequences (blockIdx.z)
};
struct GemmArgs {
    GemmOperand P, Q;
    int n_slabs, splits, lower_only, tiles_n, tiles;  // tiles: output tiles per split (lower_only: on or below the diagonal)
    float *out_f32;
    bf16_t *out_bf16;
    long long ldo, plane, out_seq;
};

constexpr int kGemmThreads = 512, kGemmTile = 256, kGemmStages = 2, kGemmStage = 512 * 128, kGemmLds = kGemmStages * kGemmStage;

// Decoding of a linear index into a pair (bi, bj), bj <= bi, enumerated row by row.
__device__ __forceinline__ void fz_lower_pair(int t, int &bi, int &bj)
{
    int m = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
    while ((m + 1) * (m + 2) / 2 <= t) ++m;
    while (m * (m + 1) / 2 > t) --m;
    bi = m;
    bj = t - m * (m + 1) / 2;
}

// The t-th tile on or below the diagonal of a T x T tile grid, counted patch by patch (patches of 4 x 4 tiles,
// row by row; inside a patch row by row).
__device__ __forceinline__ void fz_lower_patch_tile(int t, int T, int &tm, int &tn)
{
    const int PT = (T + 3) / 4;
    for (int pr = 0; pr < PT; ++pr)
        for (int pc = 0; pc <= pr; ++pc) {
            const int m0 = 4 * pr, n0 = 4 * pc, m1 = (m0 + 4 < T) ? m0 + 4 : T, n1 = (n0 + 4 < T) ? n0 + 4 : T;
            for (int m = m0; m < m1; ++m) {
                const int hi = (n1 - 1 < m) ? n1 - 1 : m, cnt = hi - n0 + 1;  // tiles (m, n0 .. hi)
                if (cnt <= 0) continue;
                if (t < cnt) {
                    tm = m;
                    tn = n0 + t;
                    return;
                }
                t -= cnt;
            }
        }
    tm = tn = 0;  // not reached for t < T (T + 1) / 2
}

// The eight copy instructions of a wavefront for one slab: its 64 operand rows, 8 rows x 128 B each.
__device__ __forceinline__ void fz_issue_slab(const unsigned char *const (&rowp)[8], size_t off, uint32_t dst)
{
#pragma unroll
    for (int j = 0; j < 8; ++j) fz_copy16_global_to_lds(rowp[j] + off, dst + j * 1024);
}

// One k-step of a wavefront: its 2 + 4 operand fragments (32 rows each, the lane's 16 B piece), and the 8 products.
__device__ __forceinline__ void fz_read_frags(fz_u32x4_t (&af)[2], fz_u32x4_t (&qf)[4], const fz_u32x4_t *st, int arow, int qrow,
                                              int slot)
{
#pragma unroll
    for (int i = 0; i < 2; ++i) af[i] = st[arow + i * 256 + slot];
#pragma unroll
    for (int j = 0; j < 4; ++j) qf[j] = st[qrow + j * 256 + slot];
}

template <typename T>
__device__ __forceinline__ void fz_multiply(fz_f32x16_t (&acc)[2][4], const fz_u32x4_t (&af)[2], const fz_u32x4_t (&qf)[4])
{
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(fz_bf16x8_t, af[i]),
                                                                    __builtin_bit_cast(fz_bf16x8_t, qf[j]), acc[i][j], 0, 0, 0);
    } else {
        // a 16 B piece holds 4 consecutive k of the lane's row; step e pairs k = 8 s + e (lanes 0-31) with
        // k = 8 s + 4 + e (lanes 32-63) on both operands
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(fz_f32x4_t, af[i])[e],
                                                                     __builtin_bit_cast(fz_f32x4_t, qf[j])[e], acc[i][j], 0, 0, 0);
    }
}

template <typename T>
__global__ __launch_bounds__(kGemmThreads) void gemm_nt_kernel(const GemmArgs a)
{
    constexpr int E = 128 / (int)sizeof(T);  // elements per slab row
    extern __shared__ __attribute__((aligned(16))) unsigned char fz_smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = wave_id();
    const int m32 = lane & 31, h = lane >> 5;

    // Work item -> compute-unit die.  Workgroups go to the 8 dies (each with its own L2) round-robin by their
    // linear id, so die x = blockIdx.x % 8 takes the x-th eighth of the item list, in order: the items a die
    // works on at the same time are neighbours in the list, and the list is ordered so that neighbours share
    // operand rows (same range of k; tiles in 4 x 4 patches, or side by side along n).
    const int items = a.tiles * a.splits, per_die = (items + 7) / 8;
    const int q = (int)(blockIdx.x & 7) * per_die + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_die || q >= items) return;
    const int split = q / a.tiles, t = q % a.tiles;
    int tm, tn;
    if (a.lower_only) {
        fz_lower_patch_tile(t, a.tiles_n, tm, tn);
    } else {
        tm = t / a.tiles_n;
        tn = t % a.tiles_n;
    }
    const int sb_begin = (int)((long long)a.n_slabs * split / a.splits);
    const int sb_end = (int)((long long)a.n_slabs * (split + 1) / a.splits);

    // ---- copy side: wavefronts 0-3 bring in P rows 64 w .. +63 of the tile, wavefronts 4-7 the Q rows
    const bool is_p = w < 4;
    const unsigned char *op_base = reinterpret_cast<const unsigned char *>(is_p ? a.P.base : a.Q.base) +
                                   (size_t)blockIdx.z * (size_t)(is_p ? a.P.seq : a.Q.seq) * sizeof(T);
    const long long op_pitch = is_p ? a.P.pitch : a.Q.pitch, op_kblk = is_p ? a.P.kblk : a.Q.kblk;
    const int op_kbw = is_p ? a.P.kbw : a.Q.kbw, op_rows = is_p ? a.P.rows : a.Q.rows;
    const int origin = (is_p ? tm : tn) * kGemmTile + (w & 3) * 64;
    const unsigned char *rowp[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int R = origin + 8 * j + (lane >> 3);
        R = R < op_rows ? R : op_rows - 1;
        const int piece = (lane & 7) ^ ((4 * j + (lane >> 4)) & 7);  // slot ^ (stage row / 2) % 8
        rowp[j] = op_base + (size_t)((long long)R * op_pitch) * sizeof(T) + piece * 16;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(fz_lds_void_t *)fz_smem + (uint32_t)(w * 8 * 1024);
    // Byte offset of the next slab to request within an operand row, advanced without divisions: slabs are
    // requested in order, and past the last one the last one again.
    const long long kk0 = (long long)sb_begin * E;
    int kin = (int)(kk0 % op_kbw);
    size_t slab_off = (size_t)((kk0 / op_kbw) * op_kblk + kin) * sizeof(T);
    const size_t blk_jump = (size_t)(op_kblk - op_kbw) * sizeof(T);
    int to_advance = sb_end - sb_begin - 1;  // how many more times the offset moves on
    auto next_slab = [&]() __attribute__((always_inline)) {
        const size_t cur = slab_off;
        if (to_advance > 0) {
            --to_advance;
            kin += E;
            slab_off += E * sizeof(T);
            if (kin >= op_kbw) {
                kin = 0;
                slab_off += blk_jump;
            }
        }
        return cur;
    };

    // ---- compute side
    const int wm = w & 3, wn = w >> 2;
    fz_f32x16_t acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    // 16 B index of (row, piece c) in a stage: row * 8 + (c ^ (row / 2) % 8); (row / 2) % 8 == (m32 / 2) % 8 for every row
    // read here.  With 64 banks of 4 B, 16 consecutive rows x one piece then cover every bank exactly once.
    const int arow = (64 * wm + m32) * 8, qrow = (256 + 128 * wn + m32) * 8, sw = (m32 >> 1) & 7;

    // Two stages of 128 B per row (a whole cache line per row and request: row-scattered 64 B pieces reach only about
    // 60 % of the L2 -> LDS rate of whole lines): the next slab is requested right after the barrier that retires
    // the previous one, while the current one is multiplied.  Within a slab the fragments of a step are read during
    // the products of the step before (the scheduling fences keep that order).
    const int n_sb = sb_end - sb_begin;
    fz_issue_slab(rowp, next_slab(), lds0);
    fz_u32x4_t a0[2], q0[4], a1[2], q1[4];
    for (int i = 0; i < n_sb; ++i) {
        FZ_WAIT_VMCNT(0);   // slab i is in LDS
        fz_lds_barrier();   // ... for every wavefront; and nobody reads the other stage any more
        if (i + 1 < n_sb) fz_issue_slab(rowp, next_slab(), lds0 + (uint32_t)(((i + 1) & 1) * kGemmStage));
        const fz_u32x4_t *st = reinterpret_cast<const fz_u32x4_t *>(fz_smem + (i & 1) * kGemmStage);
        fz_read_frags(a0, q0, st, arow, qrow, h ^ sw);
        __builtin_amdgcn_sched_barrier(0);
        fz_read_frags(a1, q1, st, arow, qrow, (2 + h) ^ sw);
        __builtin_amdgcn_sched_barrier(0);
        fz_multiply<T>(acc, a0, q0);
        __builtin_amdgcn_sched_barrier(0);
        fz_read_frags(a0, q0, st, arow, qrow, (4 + h) ^ sw);
        __builtin_amdgcn_sched_barrier(0);
        fz_multiply<T>(acc, a1, q1);
        __builtin_amdgcn_sched_barrier(0);
        fz_read_frags(a1, q1, st, arow, qrow, (6 + h) ^ sw);
        __builtin_amdgcn_sched_barrier(0);
        fz_multiply<T>(acc, a0, q0);
        __builtin_amdgcn_sched_barrier(0);
        fz_multiply<T>(acc, a1, q1);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- store: accumulator register v of a 32 x 32 tile is row 8 (v / 4) + 4 h + v % 4, column m32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = tn * kGemmTile + 128 * wn + 32 * j + m32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = tm * kGemmTile + 64 * wm + 32 * i + 8 * (v / 4) + 4 * h + (v % 4);
                if (row < a.P.rows && col < a.Q.rows) {
                    const size_t o = (size_t)blockIdx.z * a.out_seq + (size_t)row * a.ldo + col;
                    if (a.out_bf16)
                        a.out_bf16[o] = f32_to_bf16(acc[i][j][v]);
                    else
                        a.out_f32[(size_t)split * a.plane + o] = acc[i][j][v];
                }
            }
        }
}

// (2b) C = sum of the split planes of the lower 64 x 64 blocks, mirrored into the upper triangle.
__global__ __launch_bounds__(256) void gram_finish_kernel(const float *__restrict__ part, float *__restrict__ C, int n,
                                                          int splits, long long plane, long long part_seq)
{
    part += (size_t)blockIdx.z * part_seq;
    C += (size_t)blockIdx.z * n * n;
    const int bm = blockIdx.y, bn = blockIdx.x;
    if (bn > bm) return;
    __shared__ float tile[64][65];
    for (int i = threadIdx.x; i < 4096; i += 256) {
        const int rr = i >> 6, cc = i & 63, m = bm * 64 + rr, c = bn * 64 + cc;
        float v = 0.0f;
        if (m < n && c < n) {
            for (int s = 0; s < splits; ++s) v += part[(size_t)s * plane + (size_t)m * n + c];
            C[(size_t)m * n + c] = v;
        }
        tile[rr][cc] = v;
    }
    __syncthreads();
    if (bn == bm) return;
    for (int i = threadIdx.x; i < 4096; i += 256) {
        const int rr = i >> 6, cc = i & 63, m = bn * 64 + rr, c = bm * 64 + cc;  // element (m, c) of the upper block
        if (m < n && c < n) C[(size_t)m * n + c] = tile[cc][rr];
    }
}

// (2c) out = sum of `splits` planes of `count` floats.
__global__ __launch_bounds__(256) void sum_planes_kernel(const float *__restrict__ part, float *__restrict__ out,
                                                         long long count, int splits, long long plane, long long part_seq)
{
    part += (size_t)blockIdx.z * part_seq;
    out += (size_t)blockIdx.z * count;
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float v = 0.0f;
    for (int s = 0; s < splits; ++s) v += part[(size_t)s * plane + i];
    out[i] = v;
}

// (3a) Start block of the iteration: r x n values in (-1, 1) from a counter hash of (seed, index).
__global__ __launch_bounds__(256) void init_v_kernel(float *__restrict__ Vt, long long count, uint32_t seed)
{
    Vt += (size_t)blockIdx.z * count;
    seed += 0x9E37u * blockIdx.z;
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    uint32_t x = (uint32_t)i * 0x9E3779B9u + seed * 0x85EBCA6Bu + (uint32_t)(i >> 32) * 0xC2B2AE35u + 0x27D4EB2Fu;
    x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
    Vt[i] = ((float)(x >> 8) + 0.5f) * (2.0f / 16777216.0f) - 1.0f;
}

// fp64 matrix-core instruction v_mfma_f64_16x16x4_f64: D[16][16] += A[16][4] B[4][16], one double per lane for A
// (row lane % 16, k = lane / 16) and for B (column lane % 16, k = lane / 16); lane l holds D[l / 16 + 4 v][l % 16]
// in element v of its four results.
typedef __attribute__((ext_vector_type(4))) double fz_f64x4_t;

__device__ __forceinline__ void fz_gram_fetch(float (&fa)[8][2], float (&fb)[8][2], const float *__restrict__ Wn, int n0,
                                              int n_begin, int n_end, int r, const int (&ci)[2], const int (&cj)[2], int kk)
{
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int row = n0 + 4 * q + kk;
        const bool ok = row < n_end;
        const float *wr = Wn + (size_t)(ok ? row : n_begin) * r;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            fa[q][u] = (ok && ci[u] < r) ? wr[ci[u]] : 0.0f;
            fb[q][u] = (ok && cj[u] < r) ? wr[cj[u]] : 0.0f;
        }
    }
}

// (3b) Gram matrix of the r vectors, products and sums in fp64: G[i][j] = sum_n W[n][i] W[n][j].  One wavefront
// per 32 x 32 block on or below the diagonal and per range of n (one partial plane per range, added up in a
// fixed order by gram_sum_kernel); a step multiplies 4 rows of W, widened to fp64 as they are loaded.
__global__ __launch_bounds__(256) void gram_f64_kernel(const float *__restrict__ Wn, double *__restrict__ planes, int n,
                                                       int r, int splits, int n_pairs)
{
    Wn += (size_t)blockIdx.z * n * r;
    planes += (size_t)blockIdx.z * splits * r * r;
    const int pair = blockIdx.x * 4 + wave_id();
    if (pair >= n_pairs) return;
    int bi, bj;
    fz_lower_pair(pair, bi, bj);
    const int split = blockIdx.y, lane = lane_id(), col = lane & 15, kk = lane >> 4;
    const int n_begin = (int)((long long)n * split / splits), n_end = (int)((long long)n * (split + 1) / splits);
    fz_f64x4_t acc[2][2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 2; ++v) acc[u][v] = fz_f64x4_t{0.0, 0.0, 0.0, 0.0};
    int ci[2], cj[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        ci[u] = bi * 32 + 16 * u + col;
        cj[u] = bj * 32 + 16 * u + col;
    }
    // eight steps (32 rows of W) at a time; the loads of the next eight are requested before the 32 products of
    // the current ones
    float fa[8][2], fb[8][2];
    fz_gram_fetch(fa, fb, Wn, n_begin, n_begin, n_end, r, ci, cj, kk);
    for (int n0 = n_begin; n0 < n_end; n0 += 32) {
        double da[8][2], db[8][2];
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                da[q][u] = (double)fa[q][u];
                db[q][u] = (double)fb[q][u];
            }
        if (n0 + 32 < n_end) fz_gram_fetch(fa, fb, Wn, n0 + 32, n_begin, n_end, r, ci, cj, kk);
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int v = 0; v < 2; ++v)
                    acc[u][v] = __builtin_amdgcn_mfma_f64_16x16x4f64(da[q][u], db[q][v], acc[u][v], 0, 0, 0);
    }
    double *out = planes + (size_t)split * r * r;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 2; ++v)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = bi * 32 + 16 * u + kk + 4 * e, j = bj * 32 + 16 * v + col;
                if (i < r && j < r) out[(size_t)i * r + j] = acc[u][v][e];
            }
}

__global__ __launch_bounds__(256) void gram_sum_kernel(const double *__restrict__ planes, double *__restrict__ G,
                                                       double *__restrict__ diag0, int r, int splits)
{
    planes += (size_t)blockIdx.z * splits * r * r;
    G += (size_t)blockIdx.z * r * r;
    diag0 += (size_t)blockIdx.z * r;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)r * r) return;
    const int i = (int)(idx / r), j = (int)(idx % r);
    if ((j >> 5) > (i >> 5)) return;
    double v = 0.0;
    for (int s = 0; s < splits; ++s) v += planes[(size_t)s * r * r + idx];
    G[idx] = v;
    if (i == j) diag0[i] = v;
}

__device__ __forceinline__ double fz_readlane(double v, int l)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), l), hi = __builtin_amdgcn_readlane(__double2hiint(v), l);
    return __hiloint2double(hi, lo);
}

// (3c) Cholesky factor Lc of G + shift I, right-looking, one launch per panel of pb columns [c0, c0 + pb).
// Workgroup j owns rows i0 = c0 + 32 j .. i0 + 31 of G and touches nothing else, so the workgroups of a launch do
// not depend on each other; what they need of the panel beyond their own rows they recompute:
//   1. every workgroup factors the pb x pb diagonal block (current values of G, shift added) in LDS;
//   2. it solves for the panel entries Lc[j'][c0 .. c0 + pb) of all rows j' from the diagonal block down to
//      its own last row (one thread per row, substitution in registers) and keeps them in LDS;
//   3. it subtracts the panel's outer product from its own rows of the trailing matrix, G[i][j'] -= Lc[i] . Lc[j'].
// Own rows of the panel are written to Lt transposed (Lt[k][i] = Lc[i][k], i >= k), so that the column of Lc a
// later substitution needs is a contiguous row.
// shift = 1e-13 * max diagonal of the original G (diag0) keeps the factor defined when the r vectors are
// numerically dependent (an X_cat of rank below r): such directions come out short instead of normalised and
// contribute nothing to A B.
constexpr int kCholRB = 32;
__global__ __launch_bounds__(256) void chol_panel_kernel(double *__restrict__ G, double *__restrict__ Lt,
                                                         const double *__restrict__ diag0, int r, int c0, int pb)
{
    G += (size_t)blockIdx.z * r * r;
    Lt += (size_t)blockIdx.z * r * r;
    diag0 += (size_t)blockIdx.z * r;
    extern __shared__ __attribute__((aligned(16))) unsigned char fz_smem[];
    const int RP = r - c0, P1 = pb + 1;
    double *LS = reinterpret_cast<double *>(fz_smem);  // [pb][pb + 1] factor of the diagonal block
    double *dinvs = LS + pb * P1;                       // [pb] reciprocals of its diagonal
    double *Lp = dinvs + pb;                            // [pb][RP]: Lc[c0 + rr][c0 + c] at c * RP + rr
    __shared__ double red[4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int pwc = (r - c0) < pb ? (r - c0) : pb;
    const int i0 = c0 + blockIdx.x * kCholRB;
    const int own_end = (i0 + kCholRB) < r ? (i0 + kCholRB) : r;
    const int nrows = own_end - c0;

    // panel entries of G for this thread's first row below the diagonal block: requested now, used in step 2
    double g0[32];
    {
        const bool pre = tid >= pwc && tid < nrows;
#pragma unroll
        for (int c = 0; c < 32; ++c) g0[c] = (pre && c < pwc) ? G[(size_t)(c0 + tid) * r + c0 + c] : 0.0;
    }
    double mx = 0.0;
    for (int i = tid; i < r; i += 256) mx = fmax(mx, diag0[i]);
    for (int o = 32; o > 0; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o));
    if (lane == 0) red[tid >> 6] = mx;
    __syncthreads();
    const double shift = fmax(1e-13 * fmax(fmax(red[0], red[1]), fmax(red[2], red[3])), 1e-300);

    // ---- 1. diagonal block, by wavefront 0 alone and without LDS traffic: lane a keeps row a in registers, the
    // entries of the pivot column are passed around with readlane.  Rows beyond the panel are identity rows.
    if (wave_id() == 0) {
        const int a = lane & 31;
        double x[32];
#pragma unroll
        for (int b2 = 0; b2 < 32; ++b2) {
            double v = a == b2 ? 1.0 : 0.0;
            if (a < pwc && b2 <= a) v = G[(size_t)(c0 + a) * r + c0 + b2] + (a == b2 ? shift : 0.0);
            x[b2] = v;
        }
#pragma unroll
        for (int c = 0; c < 32; ++c) {
            const double piv = fz_readlane(x[c], c);
            const double dinv = rsqrt(piv > shift * 1e-3 ? piv : shift * 1e-3);
            const double l = x[c] * dinv;  // lane a > c: Lc[a][c]; lane c: the square root of the pivot
            x[c] = l;
            if (lane == 0 && c < pb) dinvs[c] = dinv;
#pragma unroll
            for (int b2 = c + 1; b2 < 32; ++b2) x[b2] -= l * fz_readlane(l, b2);
        }
        if (lane < pb) {
#pragma unroll
            for (int c = 0; c < 32; ++c)
                if (c < pb) LS[lane * P1 + c] = c <= lane ? x[c] : 0.0;
        }
    }
    __syncthreads();

    // ---- 2. panel entries of the rows c0 .. own_end - 1
    for (int rr = tid; rr < nrows; rr += 256) {
        const int row = c0 + rr;
        double x[32];
        if (rr < pwc) {
#pragma unroll
            for (int c = 0; c < 32; ++c) x[c] = (c < pb && c <= rr) ? LS[rr * P1 + c] : 0.0;
        } else {
#pragma unroll
            for (int c = 0; c < 32; ++c) {
                double v = 0.0;
                if (c < pwc) {
                    v = rr == tid ? g0[c] : G[(size_t)row * r + c0 + c];
#pragma unroll
                    for (int c2 = 0; c2 < c; ++c2) v -= x[c2] * LS[c * P1 + c2];
                    v *= dinvs[c];
                }
                x[c] = v;
            }
        }
#pragma unroll
        for (int c = 0; c < 32; ++c)
            if (c < pb) {
                Lp[(size_t)c * RP + rr] = x[c];
                if (row >= i0 && c < pwc && row >= c0 + c) Lt[(size_t)(c0 + c) * r + row] = x[c];
            }
    }
    __syncthreads();

    // ---- 3. own rows of the trailing matrix: thread = (column lane, group of 8 rows)
    const int cl = tid & 63, rg = tid >> 6;
    for (int jc = c0 + pwc + cl; jc < own_end; jc += 64) {
        double acc[8];
#pragma unroll
        for (int v = 0; v < 8; ++v) acc[v] = 0.0;
        for (int c = 0; c < pwc; ++c) {
            const double lj = Lp[(size_t)c * RP + (jc - c0)];
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                const int irow = i0 + rg * 8 + v;  // rows beyond own_end read zeros or stale LDS, and are not stored
                acc[v] += (irow < own_end ? Lp[(size_t)c * RP + (irow - c0)] : 0.0) * lj;
            }
        }
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const int irow = i0 + rg * 8 + v;
            if (irow < own_end && jc <= irow) G[(size_t)irow * r + jc] -= acc[v];
        }
    }
}

// (3c') Inverses of the 16 x 16 diagonal blocks of Lc: Minv[b][ii][jj] = (Lc_bb^-1)[ii][jj] (rows beyond r: identity).
constexpr int kSolveIB = 16;
__global__ __launch_bounds__(256) void diag_inverse_kernel(const double *__restrict__ Lt, double *__restrict__ Minv, int r)
{
    Lt += (size_t)blockIdx.z * r * r;
    Minv += (size_t)blockIdx.z * ((r + kSolveIB - 1) / kSolveIB) * (kSolveIB * kSolveIB);
    const int t = blockIdx.x * 256 + threadIdx.x, b = t / kSolveIB, jj = t % kSolveIB;
    if (b * kSolveIB >= r) return;
    double x[kSolveIB];
#pragma unroll
    for (int ii = 0; ii < kSolveIB; ++ii) {
        double v = ii == jj ? 1.0 : 0.0;
        const int row = b * kSolveIB + ii;
        if (ii > jj && row < r) {
#pragma unroll
            for (int k = 0; k < ii; ++k)
                if (k >= jj) v -= Lt[(size_t)(b * kSolveIB + k) * r + row] * x[k];
        }
        if (ii >= jj && row < r) v /= Lt[(size_t)row * r + row];
        x[ii] = ii >= jj ? v : 0.0;
    }
#pragma unroll
    for (int ii = 0; ii < kSolveIB; ++ii) Minv[(size_t)b * (kSolveIB * kSolveIB) + ii * kSolveIB + jj] = x[ii];
}

// (3d) V = Lc^-1 W by blocked forward substitution on the fp64 matrix cores.  Rows of W^T (Wn [n][r]) are
// independent; a workgroup of 4 wavefronts takes 16 RT of them and keeps them in registers as 16 x 16 accumulator
// tiles (tile t = columns 16 t .. 16 t + 15, owned by wavefront t % 4).  For tile I in turn: its owner hands the
// values to LDS, the threads multiply them by the inverse of the diagonal block (the final rows 16 I .. 16 I + 15
// of V for these n, written out as fp32), and every wavefront subtracts V_I Lc[16 t .., 16 I ..]^T from its tiles
// t > I (four matrix-core steps per tile and row group; the Lc operands come straight from global memory and are
// requested before the block inverse is applied, the block inverse itself one block ahead).
template <int MAXT, int RT>  // tiles per wavefront (r <= 64 MAXT), groups of 16 rows per workgroup
__global__ __launch_bounds__(256) void orth_solve_kernel(const float *__restrict__ Wn, const double *__restrict__ Lt,
                                                         const double *__restrict__ Minv, float *__restrict__ Vt, int n, int r)
{
    Wn += (size_t)blockIdx.z * n * r;
    Lt += (size_t)blockIdx.z * r * r;
    Minv += (size_t)blockIdx.z * ((r + 15) / 16) * 256;
    Vt += (size_t)blockIdx.z * n * r;
    __shared__ double wt[16 * RT][17], vblk[16 * RT][17], minv_s[16][17];
    const int tid = threadIdx.x, lane = tid & 63, w = wave_id(), col = lane & 15, kk = lane >> 4;
    const int n0 = blockIdx.x * (16 * RT), n_tiles = (r + 15) / 16;
    fz_f64x4_t acc[RT][MAXT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int u = 0; u < MAXT; ++u) {
            const int c = 16 * (w + 4 * u) + col;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = n0 + 16 * rt + kk + 4 * e;
                acc[rt][u][e] = (c < r && row < n) ? (double)Wn[(size_t)row * r + c] : 0.0;
            }
        }
    const int s_row = tid >> 4, s_ii = tid & 15;  // role when the block inverse is applied: outputs (s_row + 16 rt, ii)
    double mi = Minv[tid];
    for (int I = 0; I < n_tiles; ++I) {
        // operands of the update for this wavefront's tiles behind I: Lc[16 t + col][16 I + 4 g + kk]
        double bop[MAXT][4];
#pragma unroll
        for (int u = 0; u < MAXT; ++u) {
            const int t = w + 4 * u, c = 16 * t + col;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int lrow = 16 * I + 4 * g + kk;
                bop[u][g] = (t > I && c < r && lrow < r) ? Lt[(size_t)lrow * r + c] : 0.0;
            }
        }
        if ((I & 3) == w) {
#pragma unroll
            for (int u = 0; u < MAXT; ++u)
                if (u == (I >> 2)) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                        for (int e = 0; e < 4; ++e) wt[16 * rt + kk + 4 * e][col] = acc[rt][u][e];
                }
        }
        minv_s[tid >> 4][tid & 15] = mi;
        if (I + 1 < n_tiles) mi = Minv[(size_t)(I + 1) * 256 + tid];
        __syncthreads();
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            double v = 0.0;
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) v += minv_s[s_ii][jj] * wt[16 * rt + s_row][jj];  // entries jj > ii of the inverse are zero
            vblk[16 * rt + s_row][s_ii] = v;
            const int row = n0 + 16 * rt + s_row;
            if (16 * I + s_ii < r && row < n) Vt[(size_t)(16 * I + s_ii) * n + row] = (float)v;
        }
        __syncthreads();
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            double aop[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) aop[g] = -vblk[16 * rt + col][4 * g + kk];
#pragma unroll
            for (int u = 0; u < MAXT; ++u) {
                if (w + 4 * u > I && w + 4 * u < n_tiles) {
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        acc[rt][u] = __builtin_amdgcn_mfma_f64_16x16x4f64(aop[g], bop[u][g], acc[rt][u], 0, 0, 0);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// (5) Rotation to singular vectors (Sec. 3.1 Eq. 1: A = U Sigma, B = V^T).  The iteration leaves an orthonormal basis
// V of the dominant subspace; within it the Rayleigh-Ritz matrix M = V C V^T (= A^T A for A = X_cat V^T) is
// diagonalised, M = R Lambda R^T, and V is replaced by R^T V with the eigenvalues in descending order, after which
// A^T A = Lambda is diagonal and descending and any leading block of rows of B spans the best subspace of that size
// that the basis contains.  M is r x r, symmetric positive semi-definite, fp64.
//
// Eigen-solver: one-sided (Hestenes) Jacobi on the columns of M itself, in blocks.  Plane rotations J are applied from
// the right until the columns of M J are mutually orthogonal; then J^T M^2 J is diagonal, so J holds the eigenvectors
// of M^2, which are those of M, and the column norms are the eigenvalues.  Both M J and J are stored transposed (row c
// = column vector c), so a rotation touches two contiguous rows.  The r columns are cut into blocks of NC / 2; a launch
// is one round of a round-robin tournament between blocks, workgroup = one pair of blocks: it loads its NC column
// vectors into LDS, runs an inner tournament over them (wavefront = one column pair per inner round: three dot
// products, one rotation; all pairs in a sweep's first round, only the pairs between the two blocks afterwards, so that
// every pair of columns meets exactly once per sweep), writes them back, and applies the accumulated NC x NC transform
// to its NC rows of J^T (a 32 x 32 by 32 x r product on the fp64 matrix cores).
// Workgroups of a launch touch disjoint rows; launch boundaries are the only synchronisation between rounds.
// The launches of kJacobiSweeps sweeps are all enqueued up front (no value is read back by the host); a sequence is
// finished early on the device: every sweep counts, per sequence, the rotations whose two columns had a cosine above
// kJacobiSettled, and the workgroups of the sweeps after one with a count of zero return at once.  Convergence is
// quadratic by then: what a sweep without such a rotation leaves behind is of the order of the square of that bound.
// ------------------------------------------------------------------------------------------------

// (4z) Wn[c][i] = Vt[i][c]: the basis in the layout the orthonormalisation reads, for its second pass.
__global__ __launch_bounds__(256) void transpose_v_kernel(const float *__restrict__ Vt, float *__restrict__ Wn, int n, int r)
{
    __shared__ float tile[32][33];
    Vt += (size_t)blockIdx.z * r * n;
    Wn += (size_t)blockIdx.z * n * r;
    const int c0 = blockIdx.x * 32, i0 = blockIdx.y * 32, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = i0 + ty + 8 * u, c = c0 + tx;
        tile[ty + 8 * u][tx] = (i < r && c < n) ? Vt[(size_t)i * n + c] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int c = c0 + ty + 8 * u, i = i0 + tx;
        if (c < n && i < r) Wn[(size_t)c * r + i] = tile[tx][ty + 8 * u];
    }
}

// (5a) M = V W with W = C V^T, fp64 accumulation: 32 x 32 tile per workgroup.
__global__ __launch_bounds__(256) void ritz_matrix_kernel(const float *__restrict__ Vt, const float *__restrict__ Wn,
                                                          double *__restrict__ M, int n, int r)
{
    __shared__ double sv[32][33], sw[32][33];
    Vt += (size_t)blockIdx.z * r * n;
    Wn += (size_t)blockIdx.z * n * r;
    M += (size_t)blockIdx.z * r * r;
    const int i0 = blockIdx.y * 32, j0 = blockIdx.x * 32, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // ty 0..7
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int c0 = 0; c0 < n; c0 += 32) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = ty + 8 * u;
            sv[row][tx] = (i0 + row < r && c0 + tx < n) ? (double)Vt[(size_t)(i0 + row) * n + c0 + tx] : 0.0;
            sw[row][tx] = (c0 + row < n && j0 + tx < r) ? (double)Wn[(size_t)(c0 + row) * r + j0 + tx] : 0.0;
        }
        __syncthreads();
#pragma unroll 8
        for (int c = 0; c < 32; ++c) {
            const double wv = sw[c][tx];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = fma(sv[ty + 8 * u][c], wv, acc[u]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (i0 + ty + 8 * u < r && j0 + tx < r) M[(size_t)(i0 + ty + 8 * u) * r + j0 + tx] = acc[u];
}

constexpr int kJacobiSweeps = 10;        // most sweeps of the block Jacobi eigen-solver (each: every pair of column blocks once)
constexpr double kJacobiSettled = 1e-7;  // a sweep whose rotations all stayed below this cosine was the last one needed

// (5b) Gt = (M + M^T) / 2 (row c = column c of the symmetric matrix), Jt = identity, rotation counts zero.
__global__ __launch_bounds__(256) void jacobi_init_kernel(const double *__restrict__ M, double *__restrict__ Gt,
                                                          double *__restrict__ Jt, int *__restrict__ rotations, int r)
{
    if (blockIdx.x == 0 && threadIdx.x < kJacobiSweeps) rotations[blockIdx.z * kJacobiSweeps + threadIdx.x] = 0;
    M += (size_t)blockIdx.z * r * r;
    Gt += (size_t)blockIdx.z * r * r;
    Jt += (size_t)blockIdx.z * r * r;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)r * r) return;
    const int i = (int)(idx / r), j = (int)(idx % r);
    Gt[idx] = 0.5 * (M[idx] + M[(size_t)j * r + i]);
    Jt[idx] = i == j ? 1.0 : 0.0;
}

// Opponent of player `who` in round `round` of a round-robin tournament of m players (m even): player m - 1 stays,
// the others rotate.  Every pair meets exactly once in m - 1 rounds.
__device__ __forceinline__ int fz_opponent(int who, int round, int m)
{
    const int q = m - 1;
    if (who == q) return round % q;
    if (who == round % q) return q;
    return ((2 * round - who) % q + q) % q;
}

__device__ __forceinline__ double fz_wave_sum_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// The same sum for code where every lane of the wavefront is active, through the data-parallel lane permutations of
// the vector ALU instead of LDS round trips: four steps leave the sum of each row of 16 lanes in all of its lanes
// (neighbour, other pair of the quad, other quad of the half row, other half row), the four row sums are then read
// out as scalars.  CTRL: quad_perm(1,0,3,2) = 0xB1, quad_perm(2,3,0,1) = 0x4E, row_half_mirror = 0x141, row_mirror =
// 0x140.
template <int CTRL> __device__ __forceinline__ double fz_dpp_f64(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double fz_wave_sum_all_lanes_f64(double v)
{
    v += fz_dpp_f64<0xB1>(v);
    v += fz_dpp_f64<0x4E>(v);
    v += fz_dpp_f64<0x141>(v);
    v += fz_dpp_f64<0x140>(v);
    double sum = 0.0;
#pragma unroll
    for (int row = 0; row < kWave; row += 16)
        sum += __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), row),
                                __builtin_amdgcn_readlane(__double2loint(v), row));
    return sum;
}

// (5c) one tournament round between column blocks.  NC local columns (two blocks of NC / 2), NC / 2 wavefronts.
template <int NC>
__global__ __launch_bounds__(NC / 2 * 64) void jacobi_round_kernel(double *__restrict__ Gt, double *__restrict__ Jt,
                                                                  int *rotations, int r, int n_blocks,
                                                                  int sweep, int round)
{
    // rotations[sequence][sweep]: written by the launches of that sweep only, read by those of the next
    rotations += blockIdx.z * kJacobiSweeps;
    if (sweep > 0 && rotations[sweep - 1] == 0) return;  // same value for the whole workgroup
    __shared__ int big_rotations;
    if (threadIdx.x == 0) big_rotations = 0;
    extern __shared__ double fz_sm[];
    // r <= 64 kMaxIt (512 for NC = 32, 1024 for NC = 16); the local columns are kept at that pitch and zero beyond r,
    // so that the loops over a column need no per-element bounds (zeros rotate into zeros)
    constexpr int kMaxIt = NC == 32 ? 8 : 16, RP = kMaxIt * kWave;
    double *cols = fz_sm;                 // [NC][RP]
    double *T = fz_sm + (size_t)NC * RP;  // [NC][NC]: row c = coefficients of local column c in terms of the old ones
    Gt += (size_t)blockIdx.z * r * r;
    Jt += (size_t)blockIdx.z * r * r;
    constexpr int BS = NC / 2, THREADS = NC / 2 * 64;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    // this workgroup's pair of blocks: the blockIdx.x-th pair of the round
    int P = -1, Q = -1;
    {
        int seen = 0;
        for (int a = 0; a < n_blocks && P < 0; ++a) {
            const int bq = fz_opponent(a, round, n_blocks);
            if (a < bq) {
                if (seen == (int)blockIdx.x) {
                    P = a;
                    Q = bq;
                }
                ++seen;
            }
        }
    }
    auto gcol = [&](int c) { return c < BS ? P * BS + c : Q * BS + (c - BS); };  // columns >= r do not exist
    // Rows move between memory and LDS a wavefront at a time: local column w and w + NC / 2, 64 consecutive elements
    // per request, all requests of a wavefront issued before the first is awaited.
    auto rows_to_lds = [&](const double *__restrict__ src) __attribute__((always_inline)) {
        double v[2][kMaxIt];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int gc = gcol(w + BS * u);
#pragma unroll
            for (int it = 0; it < kMaxIt; ++it) {
                const int i = lane + kWave * it;
                v[u][it] = (gc < r && i < r) ? src[(size_t)gc * r + i] : 0.0;
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int it = 0; it < kMaxIt; ++it) cols[(w + BS * u) * RP + lane + kWave * it] = v[u][it];
    };
    rows_to_lds(Gt);
    for (int idx = tid; idx < NC * NC; idx += THREADS) T[idx] = (idx / NC == idx % NC) ? 1.0 : 0.0;
    __syncthreads();
    // In the sweep's first round the inner tournament is complete (every pair of the NC columns: that is where the
    // pairs inside a block meet, once per sweep, every block being in exactly one workgroup of the round); in the
    // other rounds only the BS x BS pairs between the two blocks are left to visit.
    const bool complete = round == 0;
    const int inner_rounds = complete ? NC - 1 : BS;
    for (int t = 0; t < inner_rounds; ++t) {
        // wavefront w plays the w-th pair of the inner round
        int a, b;
        if (complete) {
            // the pairs of round t of the tournament (fz_opponent): the last player meets t, and player t + j meets
            // player t - j (modulo NC - 1) for j = 1 .. NC / 2 - 1; wavefront w takes pair number w of that list
            constexpr int q = NC - 1;
            const int x = w == 0 ? t % q : (t + w) % q, y = w == 0 ? q : (t - w + q) % q;
            a = x < y ? x : y;
            b = x < y ? y : x;
        } else {
            a = w;
            b = BS + (w + t) % BS;
        }
        if (gcol(a) < r && gcol(b) < r) {
            double *ga = cols + a * RP + lane, *gb = cols + b * RP + lane;
            // the lane's elements of both columns stay in registers from the dot products to the rotation
            // (all LDS reads are requested before the first wait)
            double x[kMaxIt], y[kMaxIt];
#pragma unroll
            for (int it = 0; it < kMaxIt; ++it) {
                x[it] = ga[kWave * it];
                y[it] = gb[kWave * it];
            }
            double alpha = 0.0, beta = 0.0, gamma = 0.0;
#pragma unroll
            for (int it = 0; it < kMaxIt; ++it) {
                alpha = fma(x[it], y[it], alpha);
                beta = fma(x[it], x[it], beta);
                gamma = fma(y[it], y[it], gamma);
            }
            alpha = fz_wave_sum_all_lanes_f64(alpha);
            beta = fz_wave_sum_all_lanes_f64(beta);
            gamma = fz_wave_sum_all_lanes_f64(gamma);
            // rotate unless the two columns are already orthogonal to working accuracy (or one of them is zero)
            // (cosine of the two columns)^2 = alpha^2 / (beta gamma).  The rotation angle: tan(2 theta) = 2 alpha /
            // (gamma - beta), the smaller root of the tangent written with one square root and one division.
            const double a_sq = alpha * alpha, bg = beta * gamma;
            if (a_sq > 1e-30 * bg && beta > 0.0 && gamma > 0.0) {
                if (lane == 0 && a_sq > kJacobiSettled * kJacobiSettled * bg) atomicAdd(&big_rotations, 1);
                const double dif = gamma - beta, a2 = 2.0 * alpha;
                const double hyp = sqrt(dif * dif + a2 * a2);
                const double tn = (dif >= 0.0 ? a2 : -a2) / (fabs(dif) + hyp);
                const double cs = rsqrt(1.0 + tn * tn), sn = cs * tn;
#pragma unroll
                for (int it = 0; it < kMaxIt; ++it) {
                    ga[kWave * it] = cs * x[it] - sn * y[it];
                    gb[kWave * it] = sn * x[it] + cs * y[it];
                }
                if (lane < NC) {
                    const double x = T[a * NC + lane], y = T[b * NC + lane];
                    T[a * NC + lane] = cs * x - sn * y;
                    T[b * NC + lane] = sn * x + cs * y;
                }
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int gc = gcol(w + BS * u);
#pragma unroll
        for (int it = 0; it < kMaxIt; ++it) {
            const int i = lane + kWave * it;
            if (gc < r && i < r) Gt[(size_t)gc * r + i] = cols[(w + BS * u) * RP + i];
        }
    }
    if (tid == 0 && big_rotations > 0) atomicAdd(&rotations[sweep], big_rotations);
    __syncthreads();
    // the same transform on this workgroup's rows of J^T: load them where the columns were, combine, store
    rows_to_lds(Jt);
    __syncthreads();
    // J^T_new = T J^T_old on the fp64 matrix cores: result tiles of 16 local rows x 16 positions, NC / 4 steps each.
    // A wavefront keeps its A operands (the NC x NC transform) in registers and walks the position tiles; its B
    // operands are the old rows in LDS, so writing the new rows to memory in place disturbs nothing.
    {
        constexpr int MT = NC / 16, KS = NC / 4;
        const int lr = lane & 15, lk = lane >> 4;
        double ta[MT][KS];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) ta[mt][ks] = T[(16 * mt + lr) * NC + 4 * ks + lk];
        const int n_tiles = (r + 15) / 16;
        for (int nt = w; nt < n_tiles; nt += NC / 2) {
            const int i = 16 * nt + lr;
            double tb[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) tb[ks] = cols[(4 * ks + lk) * RP + i];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                fz_f64x4_t acc = fz_f64x4_t{0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(ta[mt][ks], tb[ks], acc, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int gc = gcol(16 * mt + lk + 4 * v);
                    if (gc < r && i < r) Jt[(size_t)gc * r + i] = acc[v];
                }
            }
        }
    }
}

// (5d) eigenvalues = norms of the rows of Gt; order[k] = the column with the k-th largest one (ties: smaller index);
// sigma (nullable) receives the singular values sqrt(lambda) of the leading r_out, in that order.
__global__ __launch_bounds__(1024) void ritz_order_kernel(const double *__restrict__ Gt, int *__restrict__ order,
                                                          float *__restrict__ sigma, int r, int r_out)
{
    __shared__ double lam[1024];
    Gt += (size_t)blockIdx.x * r * r;
    order += (size_t)blockIdx.x * r;
    const int lane = lane_id(), w = wave_id();
    for (int c = w; c < r; c += 16) {
        double sum = 0.0;
        for (int i = lane; i < r; i += kWave) sum = fma(Gt[(size_t)c * r + i], Gt[(size_t)c * r + i], sum);
        sum = fz_wave_sum_f64(sum);
        if (lane == 0) lam[c] = sqrt(sum);
    }
    __syncthreads();
    const int c = threadIdx.x;
    if (c < r) {
        int rank = 0;
        const double mine = lam[c];
        for (int j = 0; j < r; ++j) rank += (lam[j] > mine || (lam[j] == mine && j < c)) ? 1 : 0;
        order[rank] = c;
        if (sigma && rank < r_out) sigma[(size_t)blockIdx.x * r_out + rank] = (float)sqrt(mine);
    }
}

// (5e) the leading r_out rotated basis vectors: Vr[k][c] = sum_j Jt[order[k]][j] Vt[j][c], thread = column c, eight k.
__global__ __launch_bounds__(256) void rotate_basis_kernel(const double *__restrict__ Jt, const int *__restrict__ order,
                                                           const float *__restrict__ Vt, float *__restrict__ Vr, int n,
                                                           int r, int r_out, long long vr_seq)
{
    Jt += (size_t)blockIdx.z * r * r;
    order += (size_t)blockIdx.z * r;
    Vt += (size_t)blockIdx.z * r * n;
    Vr += (size_t)blockIdx.z * vr_seq;
    const int c = blockIdx.x * 256 + threadIdx.x, k0 = blockIdx.y * 8;
    const double *jrow[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) jrow[u] = Jt + (size_t)order[k0 + u < r_out ? k0 + u : r_out - 1] * r;
    double acc[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    const int cc = c < n ? c : n - 1;
    for (int j = 0; j < r; ++j) {
        const double v = (double)Vt[(size_t)j * n + cc];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[u] = fma(jrow[u][j], v, acc[u]);
    }
    if (c < n)
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u < r_out) Vr[(size_t)(k0 + u) * n + c] = (float)acc[u];
}

// (4a) B_out[l][i][c] = Vt[i][l * d + c] in the storage type.
template <typename T>
__global__ __launch_bounds__(256) void write_b_kernel(const float *__restrict__ Vt, long long vt_seq, T *__restrict__ B,
                                                      int G, int r, int d)
{
    Vt += (size_t)blockIdx.z * vt_seq;
    B += (size_t)blockIdx.z * G * r * d;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)G * r * d) return;
    const int c = (int)(idx % d), i = (int)((idx / d) % r), l = (int)(idx / ((long long)d * r));
    B[idx] = from_f32<T>(Vt[(size_t)i * ((size_t)G * d) + (size_t)l * d + c]);
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Sequences are processed `bc` at a time (grid dimension z of every kernel), which is what keeps the many small
// launches of the orthonormalisation busy; the workspace holds the intermediates of one such chunk.
constexpr int kFzChunk = 16;

struct FzLayout {
    int n, Lp, bc, gram_tiles, gram_splits, w_splits, g_splits, chol_pb;
    size_t esz, xt_seq, part_seq, off_xt, off_part, off_c, off_vt, off_wn, off_g, off_lt, off_planes, off_diag, off_minv,
        off_rot, total;
};

FzLayout fz_layout(const xkv_shape &s, int r)
{
    FzLayout f{};
    f.esz = s.dtype == XKV_F32 ? 4 : 2;
    f.n = s.G * s.H_kv * s.d_h;
    f.Lp = (s.L + 63) / 64 * 64;
    // a row pitch that is a multiple of 4 KiB would put the same piece of every row of a tile on the same cache
    // channel; 64 more (zero) tokens move consecutive rows one 128 B line apart
    if (((size_t)f.Lp * f.esz) % 4096 == 0) f.Lp += 64;
    f.bc = std::max(1, std::min(s.batch, kFzChunk));
    const int t = (f.n + kGemmTile - 1) / kGemmTile;
    f.gram_tiles = t * (t + 1) / 2;
    const int slab = 128 / (int)f.esz, gram_slabs = f.Lp / slab;
    auto splits_for = [&](int wgs_per_seq, int target, int most) {  // enough workgroups to fill the chip twice over
        const int wgs = wgs_per_seq * f.bc;
        return std::max(1, std::min(std::min(16, most), (target + wgs - 1) / wgs));
    };
    f.gram_splits = splits_for(f.gram_tiles, 512, gram_slabs);
    f.w_splits = splits_for(t * ((r + kGemmTile - 1) / kGemmTile), 256, f.n / 32);
    const int gb = (r + 31) / 32;
    f.g_splits = splits_for((gb * (gb + 1) / 2 + 3) / 4, 1024, f.n / 64);
    f.chol_pb = r <= 512 ? 32 : 16;
    f.xt_seq = (size_t)f.n * f.Lp;
    f.part_seq = std::max((size_t)f.gram_splits * f.n * f.n, (size_t)f.w_splits * f.n * r);
    const size_t bc = (size_t)f.bc;
    size_t o = 0;
    f.off_xt = o;     o += align256(bc * f.xt_seq * f.esz);
    f.off_part = o;   o += align256(bc * f.part_seq * 4);
    f.off_c = o;      o += align256(bc * f.n * f.n * 4);
    f.off_vt = o;     o += align256(bc * r * f.n * 4);
    f.off_wn = o;     o += align256(bc * f.n * r * 4);
    f.off_g = o;      o += align256(bc * r * r * 8);
    f.off_lt = o;     o += align256(bc * r * r * 8);
    f.off_planes = o; o += align256(bc * f.g_splits * r * r * 8);
    f.off_diag = o;   o += align256(bc * r * 8);
    f.off_minv = o;   o += align256(bc * ((r + 15) / 16) * 256 * 8);
    f.off_rot = o;    o += align256(bc * 16 * 4);
    f.total = o;
    return f;
}

template <typename T> hipError_t launch_gemm(const GemmArgs &a, int tiles, int nseq, hipStream_t st)
{
    static DynamicLdsOnce attr;
    if (hipError_t e0 = attr.ensure((const void *)gemm_nt_kernel<T>, kGemmLds); e0 != hipSuccess) return e0;
    GemmArgs b = a;
    b.tiles = tiles;
    const int per_die = (tiles * a.splits + 7) / 8;
    hipLaunchKernelGGL(gemm_nt_kernel<T>, dim3(8 * per_die, 1, nseq), dim3(kGemmThreads), kGemmLds, st, b);
    return hipGetLastError();
}

inline unsigned blocks256(long long count) { return (unsigned)((count + 255) / 256); }

template <typename T>
hipError_t factorize_typed(const xkv_shape &s, const FzLayout &f, const void *X, int r, int r_out, int iters, uint32_t seed,
                           void *A_out, void *B_out, float *sigma_out, unsigned char *ws, hipStream_t st)
{
    const int n = f.n, d = s.H_kv * s.d_h, tn = (n + kGemmTile - 1) / kGemmTile, tr = (r + kGemmTile - 1) / kGemmTile;
    constexpr int E = 128 / (int)sizeof(T);
    T *Xt = reinterpret_cast<T *>(ws + f.off_xt);
    float *part = reinterpret_cast<float *>(ws + f.off_part), *C = reinterpret_cast<float *>(ws + f.off_c);
    float *Vt = reinterpret_cast<float *>(ws + f.off_vt), *Wn = reinterpret_cast<float *>(ws + f.off_wn);
    double *Gm = reinterpret_cast<double *>(ws + f.off_g), *Lt = reinterpret_cast<double *>(ws + f.off_lt);
    double *planes = reinterpret_cast<double *>(ws + f.off_planes), *diag0 = reinterpret_cast<double *>(ws + f.off_diag);
    double *Minv = reinterpret_cast<double *>(ws + f.off_minv);
    int *rotations = reinterpret_cast<int *>(ws + f.off_rot);
    static_assert(kJacobiSweeps <= 16, "the rotation counters have 16 slots per sequence");
    static DynamicLdsOnce attr;
    if (hipError_t e0 = attr.ensure((const void *)chol_panel_kernel, 160 * 1024 - 256); e0 != hipSuccess) return e0;
    hipError_t e = hipSuccess;
    const long long vcount = (long long)r * n, x_seq = (long long)n * s.L;
    for (int b0 = 0; b0 < s.batch && e == hipSuccess; b0 += f.bc) {
        const int nb = std::min(f.bc, s.batch - b0);  // sequences of this chunk
        const T *Xb = reinterpret_cast<const T *>(X) + (size_t)b0 * x_seq;
        hipLaunchKernelGGL(xt_pack_kernel<T>, dim3(f.Lp / 64, n / 64, nb), dim3(256), 0, st, Xb, Xt, s.L, f.Lp, s.d_h, x_seq,
                           (long long)f.xt_seq);
        {  // C = Xt Xt^T
            GemmArgs a{};
            a.P = GemmOperand{Xt, f.Lp, 0, f.Lp, n, (long long)f.xt_seq};
            a.Q = a.P;
            a.n_slabs = f.Lp / E; a.splits = f.gram_splits; a.lower_only = 1; a.tiles_n = tn;
            a.out_f32 = part; a.out_bf16 = nullptr; a.ldo = n; a.plane = (long long)n * n; a.out_seq = (long long)f.part_seq;
            profile_begin(3, st);
            e = launch_gemm<T>(a, f.gram_tiles, nb, st);
            profile_end(3, st);
            if (e != hipSuccess) break;
            const int n64 = (n + 63) / 64;
            hipLaunchKernelGGL(gram_finish_kernel, dim3(n64, n64, nb), dim3(256), 0, st, part, C, n, f.gram_splits, a.plane,
                               (long long)f.part_seq);
        }
        hipLaunchKernelGGL(init_v_kernel, dim3(blocks256(vcount), 1, nb), dim3(256), 0, st, Vt, vcount,
                           seed + 0x9E37u * (uint32_t)b0);
        // Vt <- orthonormal basis of the columns of Wn (Cholesky-QR: r x r Gram matrix, Cholesky factor, solve; fp64)
        auto orthonormalise = [&]() {
            const int gb = (r + 31) / 32, pairs = gb * (gb + 1) / 2;
            hipLaunchKernelGGL(gram_f64_kernel, dim3((pairs + 3) / 4, f.g_splits, nb), dim3(256), 0, st, Wn, planes, n, r,
                               f.g_splits, pairs);
            hipLaunchKernelGGL(gram_sum_kernel, dim3(blocks256((long long)r * r), 1, nb), dim3(256), 0, st, planes, Gm, diag0, r,
                               f.g_splits);
            for (int c0 = 0; c0 < r; c0 += f.chol_pb) {
                const int pb = f.chol_pb;
                const size_t lds = ((size_t)pb * (pb + 1) + pb + (size_t)pb * (r - c0)) * 8;
                hipLaunchKernelGGL(chol_panel_kernel, dim3((r - c0 + kCholRB - 1) / kCholRB, 1, nb), dim3(256), lds, st, Gm, Lt,
                                   diag0, r, c0, pb);
            }
            hipLaunchKernelGGL(diag_inverse_kernel, dim3(blocks256((r + 15) / 16 * 16), 1, nb), dim3(256), 0, st, Lt, Minv, r);
            if (r <= 512)
                hipLaunchKernelGGL((orth_solve_kernel<8, 2>), dim3((n + 31) / 32, 1, nb), dim3(256), 0, st, Wn, Lt, Minv, Vt, n, r);
            else
                hipLaunchKernelGGL((orth_solve_kernel<16, 1>), dim3((n + 15) / 16, 1, nb), dim3(256), 0, st, Wn, Lt, Minv, Vt, n, r);
        };
        for (int it = 0; it < iters; ++it) {
            GemmArgs a{};  // Wn [n][r] = C Vt^T
            a.P = GemmOperand{C, n, 0, n, n, (long long)n * n};
            a.Q = GemmOperand{Vt, n, 0, n, r, vcount};
            a.n_slabs = n / 32; a.splits = f.w_splits; a.lower_only = 0; a.tiles_n = tr;
            a.out_f32 = f.w_splits > 1 ? part : Wn; a.out_bf16 = nullptr; a.ldo = r; a.plane = vcount;
            a.out_seq = f.w_splits > 1 ? (long long)f.part_seq : vcount;
            if ((e = launch_gemm<float>(a, tn * tr, nb, st)) != hipSuccess) break;
            if (f.w_splits > 1)
                hipLaunchKernelGGL(sum_planes_kernel, dim3(blocks256(vcount), 1, nb), dim3(256), 0, st, part, Wn, vcount,
                                   f.w_splits, vcount, (long long)f.part_seq);
            orthonormalise();
        }
        if (e != hipSuccess) break;
        // Cholesky-QR once more on the basis itself: after the last multiplication by C the weakest directions are
        // orthonormal only to fp32 rounding times the spread of the spectrum; a second pass on a matrix that is already
        // nearly orthonormal brings them to fp32 rounding
        hipLaunchKernelGGL(transpose_v_kernel, dim3((n + 31) / 32, (r + 31) / 32, nb), dim3(256), 0, st, Vt, Wn, n, r);
        orthonormalise();
        if (e != hipSuccess) break;
        // ---- rotation to singular vectors (5): Wn = C Vt^T once more, M = Vt Wn, eigenvectors of M by block Jacobi
        {
            GemmArgs a{};
            a.P = GemmOperand{C, n, 0, n, n, (long long)n * n};
            a.Q = GemmOperand{Vt, n, 0, n, r, vcount};
            a.n_slabs = n / 32; a.splits = f.w_splits; a.lower_only = 0; a.tiles_n = tr;
            a.out_f32 = f.w_splits > 1 ? part : Wn; a.out_bf16 = nullptr; a.ldo = r; a.plane = vcount;
            a.out_seq = f.w_splits > 1 ? (long long)f.part_seq : vcount;
            if ((e = launch_gemm<float>(a, tn * tr, nb, st)) != hipSuccess) break;
            if (f.w_splits > 1)
                hipLaunchKernelGGL(sum_planes_kernel, dim3(blocks256(vcount), 1, nb), dim3(256), 0, st, part, Wn, vcount,
                                   f.w_splits, vcount, (long long)f.part_seq);
        }
        double *Mr = planes, *Gt = Gm, *Jt = Lt;  // r x r each per sequence
        int *order = reinterpret_cast<int *>(Minv);
        const int rb = (r + 31) / 32;
        hipLaunchKernelGGL(ritz_matrix_kernel, dim3(rb, rb, nb), dim3(256), 0, st, Vt, Wn, Mr, n, r);
        hipLaunchKernelGGL(jacobi_init_kernel, dim3(blocks256((long long)r * r), 1, nb), dim3(256), 0, st, Mr, Gt, Jt, rotations, r);
        {
            const int nc = r <= 512 ? 32 : 16, bs = nc / 2;
            const int n_blocks = std::max(2, ((r + bs - 1) / bs + 1) / 2 * 2);  // an even number of column blocks
            const size_t lds = ((size_t)nc * (nc == 32 ? 512 : 1024) + (size_t)nc * nc) * 8;  // columns at their full pitch
            static DynamicLdsOnce attr32, attr16;
            e = nc == 32 ? attr32.ensure((const void *)jacobi_round_kernel<32>, 160 * 1024 - 256)
                         : attr16.ensure((const void *)jacobi_round_kernel<16>, 160 * 1024 - 256);
            if (e != hipSuccess) break;
            for (int sweep = 0; sweep < kJacobiSweeps; ++sweep)
                for (int round = 0; round < n_blocks - 1; ++round) {
                    if (nc == 32)
                        hipLaunchKernelGGL(jacobi_round_kernel<32>, dim3(n_blocks / 2, 1, nb), dim3(16 * 64), lds, st, Gt, Jt,
                                           rotations, r, n_blocks, sweep, round);
                    else
                        hipLaunchKernelGGL(jacobi_round_kernel<16>, dim3(n_blocks / 2, 1, nb), dim3(8 * 64), lds, st, Gt, Jt,
                                           rotations, r, n_blocks, sweep, round);
                }
        }
        hipLaunchKernelGGL(ritz_order_kernel, dim3(nb), dim3(1024), 0, st, Gt, order,
                           sigma_out ? sigma_out + (size_t)b0 * r_out : nullptr, r, r_out);
        float *Vr = Wn;  // [r_out][n] per sequence, in the place of W
        hipLaunchKernelGGL(rotate_basis_kernel, dim3((n + 255) / 256, (r_out + 7) / 8, nb), dim3(256), 0, st, Jt, order, Vt,
                           Vr, n, r, r_out, vcount);
        if ((e = hipGetLastError()) != hipSuccess) break;
        T *Bb = reinterpret_cast<T *>(B_out) + (size_t)b0 * s.G * r_out * d;
        T *Ab = reinterpret_cast<T *>(A_out) + (size_t)b0 * s.L * r_out;
        const long long bcount = (long long)s.G * r_out * d;
        const int tro = (r_out + kGemmTile - 1) / kGemmTile;
        hipLaunchKernelGGL(write_b_kernel<T>, dim3(blocks256(bcount), 1, nb), dim3(256), 0, st, Vr, vcount, Bb, s.G, r_out, d);
        {  // A = X_cat B^T
            GemmArgs a{};
            a.P = GemmOperand{Xb, s.d_h, (long long)s.L * s.d_h, s.d_h, s.L, x_seq};
            a.Q = GemmOperand{Bb, d, (long long)r_out * d, d, r_out, bcount};
            a.n_slabs = n / E; a.splits = 1; a.lower_only = 0; a.tiles_n = tro;
            a.out_f32 = sizeof(T) == 4 ? reinterpret_cast<float *>(Ab) : nullptr;
            a.out_bf16 = sizeof(T) == 2 ? reinterpret_cast<bf16_t *>(Ab) : nullptr;
            a.ldo = r_out; a.plane = 0; a.out_seq = (long long)s.L * r_out;
            e = launch_gemm<T>(a, ((s.L + kGemmTile - 1) / kGemmTile) * tro, nb, st);
        }
        if (e == hipSuccess) e = hipGetLastError();
    }
    return e;
}

}  // namespace

bool factorize_shape_ok(const xkv_shape &s, int r)
{
    const long long n = (long long)s.G * s.H_kv * s.d_h;
    return s.d_h % 64 == 0 && r >= 1 && r <= 1024 && r <= n && n <= 16384;
}

size_t factorize_workspace_bytes(const xkv_shape &s, int r) { return fz_layout(s, r).total; }

hipError_t launch_factorize(const xkv_shape &s, const void *X, int r, int r_out, int iters, uint32_t seed, void *A_out,
                            void *B_out, float *sigma_out, void *ws, hipStream_t st)
{
    const FzLayout f = fz_layout(s, r);
    if (s.dtype == XKV_F32)
        return factorize_typed<float>(s, f, X, r, r_out, iters, seed, A_out, B_out, sigma_out,
                                      reinterpret_cast<unsigned char *>(ws), st);
    return factorize_typed<bf16_t>(s, f, X, r, r_out, iters, seed, A_out, B_out, sigma_out,
                                   reinterpret_cast<unsigned char *>(ws), st);
}

}  // namespace xkv
