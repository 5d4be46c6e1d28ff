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

// ==========================================================================================
// bf16 matrix-core path (d_h = 128, rank a multiple of 16): X^[tokens x 128 dims of one KV head] on
// v_mfma_f32_32x32x16_bf16, the same building blocks as the gather-attend kernel's V^ product.
// A workgroup of 8 wavefronts owns one (sequence, KV head) and a range of tokens; per iteration every wavefront
// takes 32 tokens (256 per workgroup).  The rank is walked in groups of 128:
//  - A arrives line-wise (256 B pieces of 4 rows per instruction, non-temporal), two groups in flight per
//    wavefront in registers, and becomes operand fragments in a wavefront-private LDS tile (rotated layout,
//    conflict-free on both sides);
//  - the 128 x 128 block of B_l of the group is loaded row-wise by the whole workgroup one group ahead and
//    scattered into MFMA fragment order in one of two LDS buffers (the contraction index must be the per-lane
//    contiguous one, B is stored with the head dims contiguous: a transpose is unavoidable);
//  - the result tile [tokens x dims] is rounded to bf16 once, staged through the wavefront's LDS tile and stored
//    as whole 256 B rows.
// Barriers order LDS only, so the prefetches of A stay in flight across them.
// ==========================================================================================
typedef __attribute__((ext_vector_type(8))) __bf16 rc_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float rc_f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t rc_u32x4_t;

constexpr int kRcWaves = 8;
constexpr int kRcLdsB = 2 * 8 * 256 * 16;         // two buffers of 8 fragment rows x 4 dim blocks x 64 lanes x 16 B
constexpr int kRcLdsA = kRcWaves * 512 * 16;      // one 32 x 256 B tile per wavefront

__device__ __forceinline__ void rc_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// One group of 8 fragment steps for one wavefront; SLOT0 selects the half of the ring of A pieces it consumes.
template <int SLOT0>
__device__ __forceinline__ void rc_group(rc_f32x16_t (&acc)[4], rc_u32x4_t (&areg)[16], rc_u32x4_t *At,
                                         const rc_u32x4_t *Bcur, const rc_u32x4_t *arow, int pieces, int t0, int L,
                                         const int (&woff)[4], int rbase, int lane)
{
#pragma unroll
    for (int j = 0; j < 8; ++j) At[64 * j + woff[j & 3]] = areg[SLOT0 + j];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int fl = 0; fl < 8; ++fl) {
        const rc_bf16x8_t a0 = __builtin_bit_cast(rc_bf16x8_t, At[(rbase & ~15) + ((rbase + 2 * fl) & 15)]);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const rc_bf16x8_t bf = __builtin_bit_cast(rc_bf16x8_t, Bcur[(fl * 4 + db) * 64 + lane]);
            acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, a0, acc[db], 0, 0, 0);  // rows dims, columns tokens
        }
        // instruction fl of the gather two groups on, into the ring entry written out above
        const int t = t0 + 4 * fl;
        areg[SLOT0 + fl] = __builtin_nontemporal_load(&arow[(size_t)(t < L ? t : L - 1) * pieces]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

__global__ __launch_bounds__(kRcWaves * 64) void reconstruct_mfma_kernel(const bf16_t *__restrict__ A,
                                                                        const bf16_t *__restrict__ B,
                                                                        bf16_t *__restrict__ X, int G, int layer,
                                                                        int L, int r, int H_kv, int tiles_per_wg)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char rc_smem[];
    rc_u32x4_t *Bl = reinterpret_cast<rc_u32x4_t *>(rc_smem);
    const int g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int n = lane & 31, hf = lane >> 5;
    rc_u32x4_t *At = reinterpret_cast<rc_u32x4_t *>(rc_smem + kRcLdsB) + w * 512;
    const int d = H_kv * 128;
    const int pieces = r >> 3;            // 16 B pieces per row of A
    const int NG = (r + 127) / 128;       // groups of 128 ranks
    const rc_u32x4_t *Ab = reinterpret_cast<const rc_u32x4_t *>(A + (size_t)b * L * r);
    const bf16_t *Bg = B + ((size_t)b * G + layer) * (size_t)r * d + (size_t)g * 128;
    bf16_t *Xg = X + ((size_t)b * H_kv + g) * (size_t)L * 128;
    const int n_tiles = (L + 255) / 256;  // 256-token workgroup tiles
    const int tile_begin = blockIdx.x * tiles_per_wg;
    const int tile_end = tile_begin + tiles_per_wg < n_tiles ? tile_begin + tiles_per_wg : n_tiles;
    if (tile_begin >= tile_end) return;   // whole workgroup

    int woff[4];
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) woff[qd] = 16 * (lane >> 4) + (((lane & 15) + (lane >> 4) + 4 * qd) & 15);
    const int rbase = 16 * n + ((hf + n) & 15);
    const int trow = lane >> 4;
    auto piece_of = [&](int S) __attribute__((always_inline)) {
        const int pc = 16 * S + (lane & 15);
        return pc < pieces ? pc : 0;  // beyond the row: any finite piece, it meets zero rows of B
    };
    // This thread's four 16 B pieces of a 128 x 128 block of B.  Piece i is row ri(i), dims 8 cp(i) .. +7 with
    //   cp = lane % 8 + 8 (hi % 2),  ri = (lane / 8) % 8 + 8 (hi / 2),  hi = 4 w + i:
    // eight lanes read one 128 B line, and (see scatter_b) one store instruction of the wavefront hits all 32 banks.
    const int sc_k = lane & 7, sc_e = (lane >> 3) & 7;
    auto load_b = [&](int S, rc_u32x4_t (&breg)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int hi = 4 * w + i, cp = sc_k + 8 * (hi & 1), ri = S * 128 + sc_e + 8 * (hi >> 1);
            const rc_u32x4_t v = *reinterpret_cast<const rc_u32x4_t *>(Bg + (size_t)(ri < r ? ri : 0) * d + cp * 8);
            breg[i] = ri < r ? v : rc_u32x4_t{0u, 0u, 0u, 0u};
        }
    };
    // ... scattered into fragment order: element B[16 f + 8 hf' + e][32 db + c] is element e of lane (c, hf') of
    // fragment (f, db), i.e. the eight dims of a piece go to eight lanes, 2 B each.  The bank of such a store is
    // 4 (c % 8) + e / 2, so a thread writes its dims in the rotated order (j + lane % 8) % 8: then the 64 lanes of
    // one instruction cover 8 values of c % 8 and 8 of e.  The piece is rotated once in registers for that.
    auto scatter_b = [&](int buf, const rc_u32x4_t (&breg)[4]) __attribute__((always_inline)) {
        unsigned char *base = reinterpret_cast<unsigned char *>(Bl + buf * (8 * 256));
        const int kw = sc_k >> 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int hi = 4 * w + i, cp = sc_k + 8 * (hi & 1), ri = sc_e + 8 * (hi >> 1);
            const int f = ri >> 4, hfb = (ri >> 3) & 1, db = cp >> 2, c0 = (cp & 3) * 8;
            uint32_t t[4], rot[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) {  // words rotated by kw
                const uint32_t a0 = breg[i][m], a1 = breg[i][(m + 1) & 3], a2 = breg[i][(m + 2) & 3], a3 = breg[i][(m + 3) & 3];
                t[m] = kw == 0 ? a0 : kw == 1 ? a1 : kw == 2 ? a2 : a3;
            }
#pragma unroll
            for (int m = 0; m < 4; ++m)  // ... and by one more element when lane % 8 is odd
                rot[m] = (sc_k & 1) ? __builtin_amdgcn_alignbit(t[(m + 1) & 3], t[m], 16) : t[m];
            unsigned char *dst = base + (((f * 4 + db) * 64 + hfb * 32 + c0) * 16) + 2 * sc_e;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t word = rot[j >> 1];
                *reinterpret_cast<uint16_t *>(dst + 16 * ((j + sc_k) & 7)) =
                    (uint16_t)((j & 1) ? (word >> 16) : (word & 0xFFFFu));
            }
        }
    };

    // linear sequence of groups: group gi is rank group gi % NG of workgroup tile tile_begin + gi / NG
    const int total = (tile_end - tile_begin) * NG;
    auto tok0 = [&](int gi) __attribute__((always_inline)) {
        const int tl = tile_begin + (gi < total ? gi : total - 1) / NG;
        return tl * 256 + w * 32 + trow;
    };
    rc_u32x4_t areg[16], breg[4];
    load_b(0, breg);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int gi = half < total ? half : total - 1;
        const rc_u32x4_t *arow = Ab + piece_of(gi % NG);
        const int t0 = tok0(gi);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int t = t0 + 4 * j;
            areg[half * 8 + j] = __builtin_nontemporal_load(&arow[(size_t)(t < L ? t : L - 1) * pieces]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    scatter_b(0, breg);

    rc_f32x16_t acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[db][v] = 0.0f;

    // After the last rank group of a tile: lane (token n, hf) holds dims 32 db + 8 (v/4) + 4 hf + v%4.  Round once,
    // stage [32 tokens][16 pieces of 8 dims] in the wavefront's tile (same rotation as for A), store whole rows.
    // The stores go through inline assembly so that the compiler's count of outstanding loads stays exact around
    // this conditional code.
    auto finish_tile = [&](int gi) __attribute__((always_inline)) {
        const int tl = tile_begin + gi / NG;
        int nn = n;  // opaque copy: keeps the 16 tile addresses from being computed once and held in registers
        asm volatile("" : "+v"(nn));
        unsigned char *ot = reinterpret_cast<unsigned char *>(At) + hf * 8;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int c = db * 4 + q4;  // 16 B piece of the output row
                uint2 pk;
                pk.x = (uint32_t)f32_to_bf16(acc[db][4 * q4 + 0]) | ((uint32_t)f32_to_bf16(acc[db][4 * q4 + 1]) << 16);
                pk.y = (uint32_t)f32_to_bf16(acc[db][4 * q4 + 2]) | ((uint32_t)f32_to_bf16(acc[db][4 * q4 + 3]) << 16);
                *reinterpret_cast<uint2 *>(ot + (16 * nn + ((c + nn) & 15)) * 16) = pk;
            }
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[db][v] = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int tt = 4 * j + (lane >> 4), t = tl * 256 + w * 32 + tt;
            const rc_u32x4_t val = At[16 * tt + (((lane & 15) + tt) & 15)];
            if (t < L) {
                rc_u32x4_t *dst = reinterpret_cast<rc_u32x4_t *>(Xg + (size_t)t * 128) + (lane & 15);
                // (wait states: a store of more than 64 bits reads its data registers after issue, and the compiler
                // does not cover stores it cannot see)
                asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 1" : : "v"(dst), "v"(val) : "memory");
            }
        }
    };

    for (int gi = 0; gi < total; gi += 2) {
        {
            rc_lds_barrier();  // B of group gi is in buffer 0; nobody reads buffer 1 any more
            load_b((gi + 1) % NG, breg);
            const int g2 = gi + 2;
            const rc_u32x4_t *arow = Ab + piece_of((g2 < total ? g2 : total - 1) % NG);
            rc_group<0>(acc, areg, At, Bl, arow, pieces, tok0(g2), L, woff, rbase, lane);
            if (gi % NG == NG - 1) finish_tile(gi);
            scatter_b(1, breg);
        }
        {
            rc_lds_barrier();
            load_b((gi + 2) % NG, breg);
            const int g3 = gi + 3;
            const rc_u32x4_t *arow = Ab + piece_of((g3 < total ? g3 : total - 1) % NG);
            rc_group<8>(acc, areg, At, Bl + 8 * 256, arow, pieces, tok0(g3), L, woff, rbase, lane);
            if (gi + 1 < total && (gi + 1) % NG == NG - 1) finish_tile(gi + 1);
            scatter_b(0, breg);
        }
    }
}

static bool reconstruct_mfma_ok(const xkv_shape &s, int r, const void *A, const void *B, const void *X)
{
    return s.dtype == XKV_BF16 && s.d_h == 128 && r % 16 == 0 && r >= 16 &&
           ((((uintptr_t)A | (uintptr_t)B | (uintptr_t)X)) & 15u) == 0;
}

hipError_t launch_reconstruct(const xkv_shape &s, int layer, const void *A, const void *B, int r, void *X,
                              hipStream_t st)
{
    if (reconstruct_mfma_ok(s, r, A, B, X)) {
        static DynamicLdsOnce attr;
        if (hipError_t e0 = attr.ensure((const void *)reconstruct_mfma_kernel, kRcLdsB + kRcLdsA); e0 != hipSuccess) return e0;
        // about two workgroups per compute unit over the launch (one resident at a time)
        const int n_tiles = (s.L + 255) / 256, rows = s.batch * s.H_kv;
        int chunks = rows >= 512 ? 1 : (512 + rows - 1) / rows;
        chunks = chunks > n_tiles ? n_tiles : chunks;
        const int tiles_per_wg = (n_tiles + chunks - 1) / chunks;
        dim3 mgrid((n_tiles + tiles_per_wg - 1) / tiles_per_wg, s.H_kv, s.batch);
        hipLaunchKernelGGL(reconstruct_mfma_kernel, mgrid, dim3(kRcWaves * 64), kRcLdsB + kRcLdsA, st,
                           (const bf16_t *)A, (const bf16_t *)B, (bf16_t *)X, s.G, layer, s.L, r, s.H_kv, tiles_per_wg);
        return hipGetLastError();
    }
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
