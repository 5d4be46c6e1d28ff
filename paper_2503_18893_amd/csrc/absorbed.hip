// Attention over the selected tokens without rebuilding their key and value rows: the absorbed form of the
// paper's selective reconstruction.  The paper does not describe it; it is a re-association of Eq. 3,
// (A[S] B_l) q = A[S] (B_l q) and w^T (A^V[S] B^V_l) = (w^T A^V[S]) B^V_l: the per-layer factor B is folded into the
// query and into the output instead of into every token.
//
//   logits  : the selected tokens' per-head scores  scale * (A^K[t] . B^K_g q_h)  were already computed by the
//             score stage for every token, so they are gathered, not recomputed;
//   values  : o_h = ( sum_j w_hj A^V[I_j] ) B^V_g  -- the softmax-weighted sum runs over rows of A^V (r_v numbers
//             per token, read once, whole cache lines per request), and B^V is applied once per head at the end.
//
// Compared with gather-reconstruct-attend this reads half the bytes per selected token (no A^K rows) and does
// n_rep * r_v instead of (r_k + r_v) * d_h multiply-adds per token, so it is bound by the row gather alone.
// It is only valid where the keys need no per-token treatment after reconstruction (no rotary embedding).
#include "xkv_common.h"

namespace xkv {

typedef __attribute__((ext_vector_type(4))) uint32_t ab_u32x4_t;

constexpr int kAbsorbWaves = 4;   // wavefronts per workgroup of the row-sum kernel
constexpr int kAbsorbUnroll = 8;  // rows in flight per wavefront
constexpr int kProjRows = 64;     // ranks per workgroup of the projection kernel

template <typename T> struct Piece;  // the E elements of a 16 B piece as fp32
template <> struct Piece<float> {
    static constexpr int E = 4;
    static __device__ __forceinline__ void unpack(const ab_u32x4_t &r, float (&x)[4])
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = __uint_as_float(r[e]);
    }
};
template <> struct Piece<bf16_t> {
    static constexpr int E = 8;
    static __device__ __forceinline__ void unpack(const ab_u32x4_t &r, float (&x)[8])
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[2 * e] = __uint_as_float(r[e] << 16);
            x[2 * e + 1] = __uint_as_float(r[e] & 0xFFFF0000u);
        }
    }
};

// ------------------------------------------------------------------------------------------
// Row sums.  Workgroup (split, column block, row = sequence * H_kv + KV head): `chunk` of the row's k selected
// tokens, 64 * E columns of A^V.  Lane l owns the 16 B piece l of the column block, so one load instruction of a
// wavefront is one token's contiguous run of 1 KiB.  Output per workgroup: the un-normalised sums
// U[hh][col] = sum_j exp(logit_hj - m_h) A^V[I_j][col] and, from column block 0, (m_h, l_h).
// ------------------------------------------------------------------------------------------
//
// Q4: the rows of A^V are 4-bit quantised (quant.hip: r_v/2 bytes of codes, then (step, offset) as two bf16 per
// group of 32 ranks; 5 r_v / 8 bytes per row).  Lane l owns one dword of codes = 8 ranks, so a wavefront load is a
// token's contiguous 256 B, and the dword with its group's parameters.  The affine map is taken out of the inner
// loop: sum_j w_j (step_j c_je + lo_j) = sum_j (w_j step_j) c_je + sum_j w_j lo_j, the second sum once per lane.
template <typename T, int NRP, bool Q4>
__global__ __launch_bounds__(kAbsorbWaves * 64) void absorb_rows_kernel(const T *__restrict__ A_v,          // [batch][L][r_v]
                                                                        const float *__restrict__ S_heads,  // [batch][H_kv][L][NRP]
                                                                        const int32_t *__restrict__ idx,    // [batch][H_kv][k]
                                                                        float *__restrict__ part_u,   // [rows][splits][NRP][r_v]
                                                                        float *__restrict__ part_ml,  // [rows][splits][2][NRP]
                                                                        int L, int r_v, int H_kv, int k, int chunk)
{
    constexpr int E = Q4 ? 8 : Piece<T>::E;
    constexpr int CW = 64 * E;  // columns per block
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int32_t *tok = reinterpret_cast<int32_t *>(smem);                // [chunk]
    float *wl = reinterpret_cast<float *>(smem + (size_t)chunk * 4);  // [chunk][NRP] logits, then weights
    float *red = wl + (size_t)chunk * NRP;                            // [NRP][CW]
    float *stat = red + NRP * CW;                                     // [kAbsorbWaves][NRP]
    const int row = blockIdx.z, split = blockIdx.x, splits = gridDim.x;
    const int b = row / H_kv;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int j0 = split * chunk;
    const int n = k - j0 < chunk ? k - j0 : chunk;  // >= 1 by construction of the grid

    // logits of this split's tokens and their maxima
    float mx[NRP];
#pragma unroll
    for (int hh = 0; hh < NRP; ++hh) mx[hh] = -INFINITY;
    for (int j = tid; j < n; j += kAbsorbWaves * 64) {
        int t = idx[(size_t)row * k + j0 + j];
        t = t < 0 ? 0 : (t >= L ? L - 1 : t);
        tok[j] = t;
        const float *src = S_heads + ((size_t)row * L + t) * NRP;
        float v[NRP];
        if constexpr (NRP >= 4) {
#pragma unroll
            for (int c = 0; c < NRP / 4; ++c) {
                const float4 x = *reinterpret_cast<const float4 *>(src + 4 * c);
                v[4 * c] = x.x, v[4 * c + 1] = x.y, v[4 * c + 2] = x.z, v[4 * c + 3] = x.w;
            }
        } else {
#pragma unroll
            for (int hh = 0; hh < NRP; ++hh) v[hh] = src[hh];
        }
#pragma unroll
        for (int hh = 0; hh < NRP; ++hh) {
            wl[j * NRP + hh] = v[hh];
            mx[hh] = fmaxf(mx[hh], v[hh]);
        }
    }
#pragma unroll
    for (int hh = 0; hh < NRP; ++hh) {
        const float m = wave_max(mx[hh]);
        if (lane == 0) stat[w * NRP + hh] = m;
    }
    __syncthreads();
    float sum[NRP];
#pragma unroll
    for (int hh = 0; hh < NRP; ++hh) {
        float m = stat[hh];
#pragma unroll
        for (int ww = 1; ww < kAbsorbWaves; ++ww) m = fmaxf(m, stat[ww * NRP + hh]);
        mx[hh] = m;
        sum[hh] = 0.0f;
    }
    __syncthreads();  // everyone has read the maxima before stat is reused for the sums
    for (int j = tid; j < n; j += kAbsorbWaves * 64) {
#pragma unroll
        for (int hh = 0; hh < NRP; ++hh) {
            const float e = expf(wl[j * NRP + hh] - mx[hh]);
            wl[j * NRP + hh] = e;
            sum[hh] += e;
        }
    }
#pragma unroll
    for (int hh = 0; hh < NRP; ++hh) {
        const float s = wave_sum(sum[hh]);
        if (lane == 0) stat[w * NRP + hh] = s;
    }
    __syncthreads();
    if (blockIdx.y == 0 && tid < NRP) {
        float s = 0.0f;
#pragma unroll
        for (int ww = 0; ww < kAbsorbWaves; ++ww) s += stat[ww * NRP + tid];
        float *ml = part_ml + ((size_t)row * splits + split) * 2 * NRP;
        // mx[] is indexed at compile time only; pick this thread's head through a select chain
        float m = mx[0];
#pragma unroll
        for (int hh = 1; hh < NRP; ++hh) m = tid == hh ? mx[hh] : m;
        ml[tid] = m;
        ml[NRP + tid] = s;
    }

    // weighted sum of the rows
    const int pieces = r_v / E;
    const int pc = blockIdx.y * 64 + lane;
    const bool active = pc < pieces;
    float acc[NRP][E];
#pragma unroll
    for (int hh = 0; hh < NRP; ++hh)
#pragma unroll
        for (int e = 0; e < E; ++e) acc[hh][e] = 0.0f;
    if constexpr (Q4) {
        if (active) {
            const size_t pitch = quant_row_bytes(r_v);
            const unsigned char *Ab = reinterpret_cast<const unsigned char *>(A_v) + (size_t)b * L * pitch;
            const size_t par_off = (size_t)(r_v >> 1) + 4 * (size_t)(pc >> 2);
            float accl[NRP];
#pragma unroll
            for (int hh = 0; hh < NRP; ++hh) accl[hh] = 0.0f;
            for (int jb = w * kAbsorbUnroll; jb < n; jb += kAbsorbWaves * kAbsorbUnroll) {
                uint32_t cw[kAbsorbUnroll], pw[kAbsorbUnroll];
#pragma unroll
                for (int u = 0; u < kAbsorbUnroll; ++u) {
                    const int j = jb + u < n ? jb + u : n - 1;
                    const int t = __builtin_amdgcn_readfirstlane(tok[j]);
                    const unsigned char *rowp = Ab + (size_t)t * pitch;
                    cw[u] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(rowp) + pc);
                    pw[u] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(rowp + par_off));
                }
#pragma unroll
                for (int u = 0; u < kAbsorbUnroll; ++u) {
                    if (jb + u < n) {  // wave-uniform
                        const float step = __uint_as_float(pw[u] << 16), lo = __uint_as_float(pw[u] & 0xFFFF0000u);
                        const uint32_t t0 = cw[u] & 0x0F0F0F0Fu, t1 = (cw[u] >> 4) & 0x0F0F0F0Fu;
                        // rank 2i sits in bits [4i, 4i+4), rank 2i+1 in bits [16+4i, 16+4i+4): after the two masks
                        // every code is a byte of t0 (i even) or t1 (i odd)
                        float c[8];
                        c[0] = (float)(t0 & 0xFFu), c[4] = (float)((t0 >> 8) & 0xFFu);
                        c[1] = (float)((t0 >> 16) & 0xFFu), c[5] = (float)(t0 >> 24);
                        c[2] = (float)(t1 & 0xFFu), c[6] = (float)((t1 >> 8) & 0xFFu);
                        c[3] = (float)((t1 >> 16) & 0xFFu), c[7] = (float)(t1 >> 24);
#pragma unroll
                        for (int hh = 0; hh < NRP; ++hh) {
                            const float wv = wl[(jb + u) * NRP + hh];
                            const float ws = wv * step;
                            accl[hh] = fmaf(wv, lo, accl[hh]);
#pragma unroll
                            for (int e = 0; e < E; ++e) acc[hh][e] = fmaf(ws, c[e], acc[hh][e]);
                        }
                    }
                }
            }
#pragma unroll
            for (int hh = 0; hh < NRP; ++hh)
#pragma unroll
                for (int e = 0; e < E; ++e) acc[hh][e] += accl[hh];
        }
    } else if (active) {
        const ab_u32x4_t *Ab = reinterpret_cast<const ab_u32x4_t *>(A_v + (size_t)b * L * r_v) + pc;
        for (int jb = w * kAbsorbUnroll; jb < n; jb += kAbsorbWaves * kAbsorbUnroll) {
            ab_u32x4_t r[kAbsorbUnroll];
#pragma unroll
            for (int u = 0; u < kAbsorbUnroll; ++u) {
                const int j = jb + u < n ? jb + u : n - 1;
                const int t = __builtin_amdgcn_readfirstlane(tok[j]);
                r[u] = __builtin_nontemporal_load(&Ab[(size_t)t * pieces]);
            }
#pragma unroll
            for (int u = 0; u < kAbsorbUnroll; ++u) {
                if (jb + u < n) {  // wave-uniform
                    float x[E];
                    Piece<T>::unpack(r[u], x);
#pragma unroll
                    for (int hh = 0; hh < NRP; ++hh) {
                        const float wv = wl[(jb + u) * NRP + hh];
#pragma unroll
                        for (int e = 0; e < E; ++e) acc[hh][e] = fmaf(wv, x[e], acc[hh][e]);
                    }
                }
            }
        }
    }
    // the wavefronts' sums are added in a fixed order, so the result does not depend on timing
    for (int ww = 0; ww < kAbsorbWaves; ++ww) {
        if (w == ww && active) {
#pragma unroll
            for (int hh = 0; hh < NRP; ++hh)
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    float *dst = &red[hh * CW + lane * E + e];
                    *dst = (ww == 0 ? 0.0f : *dst) + acc[hh][e];
                }
        }
        __syncthreads();
    }
    float *dst = part_u + ((size_t)row * splits + split) * NRP * r_v;
    const int c0 = blockIdx.y * CW;
    for (int i = tid; i < NRP * CW; i += kAbsorbWaves * 64) {
        const int hh = i / CW, c = i % CW;
        if (c0 + c < r_v) dst[(size_t)hh * r_v + c0 + c] = red[i];
    }
}

// ------------------------------------------------------------------------------------------
// Merge of the splits and product with B^V_g.  Workgroup (slice, KV head, sequence): kProjRows ranks.
//   f_s = exp(m_s - m),  m = max_s m_s,  l = sum_s f_s l_s,  U = sum_s f_s U_s   (its kProjRows columns),
//   partial o[hh][:] = U[hh][slice] . B^V_g[slice][:]
// written in the layout of the attention partials (one per slice, all with maximum m; slice 0 carries l, the
// others 0), so that the ordinary merge kernel sums the slices and divides -- and can take the partials of an
// uncompressed tail into the same softmax.
// ------------------------------------------------------------------------------------------
//
// WIDE: rows of B^V_g are fetched 16 bytes per lane, 64 / lpr rows per request (lpr = lanes per row, a power of
// two), instead of one element per lane.  With one element per lane a request is 128 bytes and the number of
// requests a compute unit can have in flight caps the whole chip at about 1.5 TB/s: phase timestamps showed 11 of
// the kernel's 15 us waiting for these 16 MB.
template <typename T, int NRP, bool WIDE>
__global__ __launch_bounds__(256) void absorb_project_kernel(const float *__restrict__ part_u,
                                                             const float *__restrict__ part_ml,
                                                             const T *__restrict__ B_v,   // [batch][G][r_v][d]
                                                             float *__restrict__ po,      // [batch][H_q][slices][d_h]
                                                             float *__restrict__ pml,     // [batch][H_q][slices][2]
                                                             int G, int layer, int r_v, int H_kv, int H_q, int d_h,
                                                             int splits)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *ml = reinterpret_cast<float *>(smem);  // [splits][2][NRP]
    float *fs = ml + (size_t)splits * 2 * NRP;     // [splits][NRP]
    float *tot = fs + (size_t)splits * NRP;        // [2][NRP]: m, l
    float *U = tot + 2 * NRP;                      // [NRP][kProjRows]
    float *red = U + NRP * kProjRows;              // [4][NRP][d_h]
    const int slice = blockIdx.x, n_slices = gridDim.x, g = blockIdx.y, b = blockIdx.z;
    const int row = b * H_kv + g;
    const int n_rep = H_q / H_kv, d = H_kv * d_h;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int c0 = slice * kProjRows;
    const int cn = r_v - c0 < kProjRows ? r_v - c0 : kProjRows;
    // This kernel is a chain of short dependent steps, so it is bound by load latency: the rows of B^V, which
    // depend on nothing, are requested first and wait in registers (rows w, w + 4, ... of the slice per wavefront).
    constexpr int DI = 4;               // d_h <= 256
    constexpr int RPW = kProjRows / 4;  // rows per wavefront
    constexpr int E = Piece<T>::E;
    const T *Bg = B_v + (((size_t)b * G + layer) * r_v + c0) * d + (size_t)g * d_h;
    T xraw[WIDE ? 1 : RPW][DI];
    ab_u32x4_t xwide[WIDE ? RPW : 1];
    // WIDE: wavefront w takes rows 16 w .. 16 w + 15, request u covers rows 16 w + u rpl + sub
    const int lpr = d_h / E, rpl = 64 / lpr;
    const int sub = lane / lpr, pc = lane - sub * lpr;
    const int n_req = RPW / rpl > 0 ? RPW / rpl : 1;
    if constexpr (WIDE) {
#pragma unroll
        for (int u = 0; u < RPW; ++u) {
            const int c = RPW * w + u * rpl + sub;
            if (u < n_req)
                xwide[u] = *reinterpret_cast<const ab_u32x4_t *>(Bg + (size_t)(c < cn ? c : 0) * d + pc * E);
        }
    } else {
#pragma unroll
        for (int u = 0; u < RPW; ++u) {
            const int c = w + 4 * u;
            const T *brow = Bg + (size_t)(c < cn ? c : 0) * d;
#pragma unroll
            for (int i = 0; i < DI; ++i) {
                const int col = lane + 64 * i;
                xraw[u][i] = col < d_h ? brow[col] : T(0);
            }
        }
    }
    for (int i = tid; i < splits * 2 * NRP; i += 256) ml[i] = part_ml[(size_t)row * splits * 2 * NRP + i];
    __syncthreads();
    if (tid < NRP) {
        float m = -INFINITY;
        for (int s = 0; s < splits; ++s) m = fmaxf(m, ml[s * 2 * NRP + tid]);
        float l = 0.0f;
        for (int s = 0; s < splits; ++s) {
            const float f = expf(ml[s * 2 * NRP + tid] - m);
            fs[s * NRP + tid] = f;
            l = fmaf(f, ml[s * 2 * NRP + NRP + tid], l);
        }
        tot[tid] = m;
        tot[NRP + tid] = l;
    }
    __syncthreads();
    const float *pu = part_u + (size_t)row * splits * NRP * r_v;
    for (int i = tid; i < NRP * kProjRows; i += 256) {
        const int hh = i / kProjRows, c = i % kProjRows;
        float u = 0.0f;
        if (c < cn) {
            for (int s0 = 0; s0 < splits; s0 += 8) {  // eight splits' values in flight
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    v[j] = s0 + j < splits ? pu[((size_t)(s0 + j) * NRP + hh) * r_v + c0 + c] : 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (s0 + j < splits) u = fmaf(fs[(s0 + j) * NRP + hh], v[j], u);
            }
        }
        U[i] = u;
    }
    __syncthreads();
    if constexpr (WIDE) {
        float accw[NRP][E];
#pragma unroll
        for (int hh = 0; hh < NRP; ++hh)
#pragma unroll
            for (int e = 0; e < E; ++e) accw[hh][e] = 0.0f;
#pragma unroll
        for (int u = 0; u < RPW; ++u) {
            const int c = RPW * w + u * rpl + sub;
            if (u < n_req && c < cn) {
                float x[E];
                Piece<T>::unpack(xwide[u], x);
#pragma unroll
                for (int hh = 0; hh < NRP; ++hh) {
                    const float uv = U[hh * kProjRows + c];
#pragma unroll
                    for (int e = 0; e < E; ++e) accw[hh][e] = fmaf(uv, x[e], accw[hh][e]);
                }
            }
        }
        // the rows of a request sit lpr lanes apart: fold them onto the first lpr lanes, always in the same order
        for (int off = lpr; off < 64; off <<= 1) {
#pragma unroll
            for (int hh = 0; hh < NRP; ++hh)
#pragma unroll
                for (int e = 0; e < E; ++e) accw[hh][e] += __shfl_xor(accw[hh][e], off, kWave);
        }
        if (sub == 0) {
#pragma unroll
            for (int hh = 0; hh < NRP; ++hh)
#pragma unroll
                for (int e = 0; e < E; ++e) red[((size_t)w * NRP + hh) * d_h + pc * E + e] = accw[hh][e];
        }
    } else {
    float acc[NRP][DI];
#pragma unroll
    for (int hh = 0; hh < NRP; ++hh)
#pragma unroll
        for (int i = 0; i < DI; ++i) acc[hh][i] = 0.0f;
#pragma unroll
    for (int u = 0; u < RPW; ++u) {
        const int c = w + 4 * u;
        if (c < cn) {  // wave-uniform
#pragma unroll
            for (int hh = 0; hh < NRP; ++hh) {
                const float uv = U[hh * kProjRows + c];
#pragma unroll
                for (int i = 0; i < DI; ++i) acc[hh][i] = fmaf(uv, to_f32(xraw[u][i]), acc[hh][i]);
            }
        }
    }
#pragma unroll
    for (int hh = 0; hh < NRP; ++hh)
#pragma unroll
        for (int i = 0; i < DI; ++i) {
            const int col = lane + 64 * i;
            if (col < d_h) red[((size_t)w * NRP + hh) * d_h + col] = acc[hh][i];
        }
    }
    __syncthreads();
    for (int i = tid; i < n_rep * d_h; i += 256) {
        const int hh = i / d_h, col = i % d_h;
        float v = red[(size_t)hh * d_h + col];
#pragma unroll
        for (int ww = 1; ww < 4; ++ww) v += red[((size_t)ww * NRP + hh) * d_h + col];
        const size_t slot = ((size_t)b * H_q + (size_t)g * n_rep + hh) * n_slices + slice;
        po[slot * d_h + col] = v;
        if (col == 0) {
            pml[slot * 2] = tot[hh];
            pml[slot * 2 + 1] = slice == 0 ? tot[NRP + hh] : 0.0f;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
static inline int ab_ceil_div(int a, int b) { return (a + b - 1) / b; }

bool absorb_shape_ok(const xkv_shape &s)
{
    const int E = s.dtype == XKV_F32 ? 4 : 8;
    return s.r_v % E == 0 && s.d_h <= 256 && s.H_q / s.H_kv <= 16;
}

AbsorbPlan make_absorb_plan(const xkv_shape &s, size_t base_bytes)
{
    AbsorbPlan a{};
    const int E = s.dtype == XKV_F32 ? 4 : 8;
    a.nrp = head_pitch_of(s.H_q / s.H_kv);
    a.col_blocks = ab_ceil_div(s.r_v, 64 * E);
    const int rows = s.batch * s.H_kv > 0 ? s.batch * s.H_kv : 1;
    // about four workgroups per compute unit (more, shorter splits only add partial sums to write and to merge);
    // a split holds 64..512 tokens (ids and weights live in LDS)
    const int want = ab_ceil_div(1024, rows * a.col_blocks);
    int chunk = ab_ceil_div(ab_ceil_div(s.k, want), 32) * 32;
    chunk = chunk < 64 ? 64 : (chunk > 512 ? 512 : chunk);
    a.chunk = chunk;
    a.splits = ab_ceil_div(s.k, chunk);
    const size_t b = (size_t)(s.batch > 0 ? s.batch : 1);
    size_t off = (base_bytes + 255) / 256 * 256;
    a.off_heads = off;
    off += (b * s.H_kv * (size_t)s.L * a.nrp * sizeof(float) + 255) / 256 * 256;
    a.off_part_u = off;
    off += (b * s.H_kv * (size_t)a.splits * a.nrp * s.r_v * sizeof(float) + 255) / 256 * 256;
    a.off_part_ml = off;
    off += (b * s.H_kv * (size_t)a.splits * 2 * a.nrp * sizeof(float) + 255) / 256 * 256;
    a.slices = ab_ceil_div(s.r_v, kProjRows);
    a.off_po = off;
    off += (b * s.H_q * (size_t)a.slices * s.d_h * sizeof(float) + 255) / 256 * 256;
    a.off_pml = off;
    off += (b * s.H_q * (size_t)a.slices * 2 * sizeof(float) + 255) / 256 * 256;
    a.total = off;
    return a;
}

template <typename T, int NRP, bool Q4>
static hipError_t launch_absorbed_t(const xkv_shape &s, const AbsorbPlan &a, int layer, const T *A_v, const T *B_v,
                                    const float *S_heads, const int32_t *idx, float *po, float *pml, float *part_u, float *part_ml,
                                    hipStream_t st)
{
    constexpr int E = Q4 ? 8 : Piece<T>::E;
    const size_t lds_rows = (size_t)a.chunk * 4 + ((size_t)a.chunk * NRP + NRP * 64 * E + kAbsorbWaves * NRP) * 4;
    const size_t lds_comb = ((size_t)a.splits * 3 * NRP + 2 * NRP + NRP * kProjRows + (size_t)4 * NRP * s.d_h) * 4;
    const size_t lds_max = 160 * 1024 - 512;
    if (lds_rows > lds_max || lds_comb > lds_max) return hipErrorInvalidValue;
    static DynamicLdsOnce attr_rows, attr_proj, attr_proj_wide;
    if (hipError_t e0 = attr_rows.ensure((const void *)absorb_rows_kernel<T, NRP, Q4>, lds_max); e0 != hipSuccess) return e0;
    if (hipError_t e0 = attr_proj.ensure((const void *)absorb_project_kernel<T, NRP, false>, lds_max); e0 != hipSuccess)
        return e0;
    if (hipError_t e0 = attr_proj_wide.ensure((const void *)absorb_project_kernel<T, NRP, true>, lds_max); e0 != hipSuccess)
        return e0;
    profile_begin(4, st);
    hipLaunchKernelGGL((absorb_rows_kernel<T, NRP, Q4>), dim3(a.splits, a.col_blocks, s.batch * s.H_kv),
                       dim3(kAbsorbWaves * 64), lds_rows, st, A_v, S_heads, idx, part_u, part_ml, s.L, s.r_v, s.H_kv,
                       s.k, a.chunk);
    profile_end(4, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // rows of B^V 16 bytes per lane when a row of the head is a power-of-two number (4..64) of aligned pieces
    const int lpr = s.d_h % E == 0 ? s.d_h / E : 0;
    const bool wide = lpr >= 4 && lpr <= 64 && (lpr & (lpr - 1)) == 0 && (((uintptr_t)B_v) & 15u) == 0;
    if (wide)
        hipLaunchKernelGGL((absorb_project_kernel<T, NRP, true>), dim3(a.slices, s.H_kv, s.batch), dim3(256), lds_comb, st,
                           part_u, part_ml, B_v, po, pml, s.G, layer, s.r_v, s.H_kv, s.H_q, s.d_h, a.splits);
    else
        hipLaunchKernelGGL((absorb_project_kernel<T, NRP, false>), dim3(a.slices, s.H_kv, s.batch), dim3(256), lds_comb, st,
                           part_u, part_ml, B_v, po, pml, s.G, layer, s.r_v, s.H_kv, s.H_q, s.d_h, a.splits);
    return hipGetLastError();
}

template <typename T, bool Q4>
static hipError_t launch_absorbed_n(const xkv_shape &s, const AbsorbPlan &a, int layer, const T *A_v, const T *B_v,
                                    const float *S_heads, const int32_t *idx, float *po, float *pml, float *part_u,
                                    float *part_ml, hipStream_t st)
{
    switch (a.nrp) {
    case 1: return launch_absorbed_t<T, 1, Q4>(s, a, layer, A_v, B_v, S_heads, idx, po, pml, part_u, part_ml, st);
    case 2: return launch_absorbed_t<T, 2, Q4>(s, a, layer, A_v, B_v, S_heads, idx, po, pml, part_u, part_ml, st);
    case 4: return launch_absorbed_t<T, 4, Q4>(s, a, layer, A_v, B_v, S_heads, idx, po, pml, part_u, part_ml, st);
    case 8: return launch_absorbed_t<T, 8, Q4>(s, a, layer, A_v, B_v, S_heads, idx, po, pml, part_u, part_ml, st);
    default: return launch_absorbed_t<T, 16, Q4>(s, a, layer, A_v, B_v, S_heads, idx, po, pml, part_u, part_ml, st);
    }
}

// Leaves a.slices attention partials per query head in po / pml; the caller merges them with launch_combine.
// q4: A_v holds 4-bit rows (bf16 shapes only; B_v and the output stay bf16).
hipError_t launch_absorbed(const xkv_shape &s, const AbsorbPlan &a, int layer, const void *A_v, const void *B_v,
                           const float *S_heads, const int32_t *idx, float *po, float *pml, float *part_u,
                           float *part_ml, hipStream_t st, bool q4)
{
    if (q4) {
        if (s.dtype != XKV_BF16) return hipErrorInvalidValue;
        return launch_absorbed_n<bf16_t, true>(s, a, layer, (const bf16_t *)A_v, (const bf16_t *)B_v, S_heads, idx, po, pml,
                                               part_u, part_ml, st);
    }
    if (s.dtype == XKV_F32)
        return launch_absorbed_n<float, false>(s, a, layer, (const float *)A_v, (const float *)B_v, S_heads, idx, po, pml,
                                               part_u, part_ml, st);
    return launch_absorbed_n<bf16_t, false>(s, a, layer, (const bf16_t *)A_v, (const bf16_t *)B_v, S_heads, idx, po, pml,
                                            part_u, part_ml, st);
}

}  // namespace xkv
