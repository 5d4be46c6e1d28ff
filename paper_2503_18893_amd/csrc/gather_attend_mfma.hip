// bf16 matrix-core path of selective reconstruction + sparse attention (Sec. 3.2, Eq. 3):
//   K^_g = A^K[I_g,:] B^K_{l,g},  V^_g = A^V[I_g,:] B^V_{l,g},  out_h = softmax(scale K^_g q_h)^T V^_g.
//
// Everything is one chain of v_mfma_f32_32x32x16_bf16 whose operand layouts are chosen so that the
// result registers of one product are, after a bf16 pack, directly the operand of the next:
//   (1) K^T tile [dims x tokens]  = B^K_g^T (LDS fragment)  x  gathered rows of A^K (fragment from the LDS tile)
//   (2) Z^T [tokens x head slots] = K^ (registers of (1))   x  Q^T fragments (LDS)
//   (3) V^ tile [tokens x dims]   = gathered rows of A^V    x  B^V_g (LDS fragment)
//   (4) O [head slots x dims]    += W = exp(Z^T - max) (registers of (2))  x  V^ (registers of (3))
// In a 32x32 result lane (n, hf) holds column n and rows 8(v/4) + 4hf + v%4, v = 0..15; eight
// consecutive registers are a valid 16-deep operand fragment for the next product because both of
// its operands then agree on which row sits at which position: K^ and V^ never leave the registers.
//
// A workgroup is eight wavefronts (four for small problems) of 32 selected tokens each (256 per tile).  The reconstruction matrices
// are pre-packed into fragment order (pack_b_block) and streamed through two LDS buffers 128 ranks at a
// time, shared by the wavefronts; the gathered rows arrive line-wise and are turned into operand fragments
// in a wavefront-private LDS tile.  Each wavefront keeps its own online softmax state; the workgroup
// merges them and writes one partial per query head and split; combine_kernel merges the splits.
#include <type_traits>

#include "xkv_common.h"

#include <cmath>
#include "prepass.h"

namespace xkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) float f32x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

constexpr int kMaxChunkTokens = 4096;  // selected tokens per workgroup (their ids sit in LDS)
constexpr int kGroup = 8;  // fragments (of 16 ranks) per LDS stage: 8 x 4 KiB = 32 KiB, two stages

// blocks [0, blocks_per_head) of a (sequence, KV head) pack B, the next kPackQBlocks the Q^T fragments
__global__ __launch_bounds__(256) void pack_b_kernel(PackArgs a)
{
    if ((int)blockIdx.x < a.blocks_per_head)
        pack_b_block(a, blockIdx.x, blockIdx.y, blockIdx.z);
    else if (a.pack_q)
        pack_q_block(a, (int)blockIdx.x - a.blocks_per_head, blockIdx.y, blockIdx.z);
}

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t &c, int j)
{
    f32x8_t x;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = c[8 * j + e];
    return __builtin_convertvector(x, bf16x8_t);
}

typedef __attribute__((address_space(3))) void lds_void_t;

// 16 B per lane straight from global memory into LDS at lds_base + lane * 16 (lds_base is wave-uniform).
// Issued as inline assembly on purpose: the compiler then does not tie later LDS reads of the *other*
// buffer to this copy (it cannot tell the buffers apart and would drain the whole vector-memory queue before
// every group); completion is awaited explicitly with XKV_WAIT_VMCNT before the barrier that publishes
// the buffer.  The copy still counts as one outstanding vector-memory operation, which only makes the
// compiler's own waits for register loads more conservative, never less.
__device__ __forceinline__ void copy16_global_to_lds(const void *gptr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(gptr) : "memory", "m0");
}

// s_waitcnt that only bounds the number of outstanding vector-memory operations (gfx9 encoding: vmcnt is
// split over bits 3:0 and 15:14; expcnt and lgkmcnt are left at "no wait").
#define XKV_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (7 << 4) | (0xF << 8) | (((n) >> 4) << 14))

// Wavefronts per workgroup (WAVES, template parameter): 8 with 32 selected tokens each per tile (256 tokens);
// 4 when there are too few selected tokens to give every compute unit a 256-token tile.
// LDS map (bytes): B fragments [2][kGroup][4][64][16] | A tiles [WAVES][512][16] | Q fragments [8][64][16] | ids
constexpr int kLdsB = 2 * kGroup * 256 * 16, kLdsQ = 8 * 64 * 16;
constexpr int lds_a_bytes(int waves) { return waves * 512 * 16; }

// What a wavefront gathers for one group of 8 fragment steps: 128 ranks = 256 B of each of its 32 rows.
// Instruction j (0..7) covers rows 4j..4j+3 whole-line-wise: lane l loads the 16 B piece l%16 of row 4j + l/16,
// so every 128 B line is touched by exactly one instruction (this is what keeps random-row gathers near the
// streaming rate; one lane per row with 32 B runs does not).  `piece` is the lane's 16 B piece within the row,
// already clamped into the row; `pieces` is the row length in 16 B units.
struct AStage {
    const u32x4_t *base;  // A^K or A^V of this sequence
    int pieces;
    int piece;
};

// One group of 8 fragment steps.  IS_K selects which product the fragments feed, SLOT0 (0 or 8) which half of
// the two-group-deep ring of gathered pieces the group consumes.  The wavefront
//  - waits until its copies of this group's B fragments (issued one group ago) have landed, and publishes them,
//  - starts the global -> LDS copies of the next group's B fragments into the other buffer,
//  - transposes its gathered pieces through its private LDS tile: written row-wise (rotated by the row number,
//    so that neither side has bank conflicts), read back as one 16-rank operand fragment per step,
//  - refills the ring, one instruction per step, with the pieces of the group two groups on,
//  - per step multiplies the step's four B fragments with the A fragment.
template <bool IS_K, int SLOT0, int WAVES>
__device__ __forceinline__ void run_group(f32x16_t (&acc)[4], u32x4_t (&areg)[2 * kGroup], const u32x4_t *Bl,
                                          u32x4_t *At, int buf, uint32_t dma_dst, const u32x4_t *bsrc_next,
                                          const AStage &an, const int (&tk)[kGroup], const int (&woff)[4], int rbase,
                                          int lane)
{
    // Outstanding at this point, youngest first: the 8 gathers issued during the previous group, then the B copies
    // for this group, then older gathers.  The barrier orders LDS only: the gathers stay in flight across it.
    XKV_WAIT_VMCNT(kGroup);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
#pragma unroll
    for (int i = 0; i < 32 / WAVES; ++i) copy16_global_to_lds(bsrc_next + i * (WAVES * 64), dma_dst + i * (WAVES * 1024));
#pragma unroll
    for (int j = 0; j < kGroup; ++j) At[64 * j + woff[j & 3]] = areg[SLOT0 + j];
    __builtin_amdgcn_sched_barrier(0);
    const u32x4_t *bcur = Bl + buf * (kGroup * 256) + lane;
#pragma unroll
    for (int fl = 0; fl < kGroup; ++fl) {
        const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, At[(rbase & ~15) + ((rbase + 2 * fl) & 15)]);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const bf16x8_t bf = __builtin_bit_cast(bf16x8_t, bcur[(fl * 4 + db) * 64]);
            if constexpr (IS_K)  // (1) K^T tile: rows = head dims, columns = tokens
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, a0, acc[db], 0, 0, 0);
            else  // (3) V^ tile: rows = tokens, columns = head dims
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bf, acc[db], 0, 0, 0);
        }
        // instruction fl of the gather two groups on, into the ring entry written out above
        areg[SLOT0 + fl] = an.base[(size_t)tk[fl] * an.pieces + an.piece];
        __builtin_amdgcn_sched_barrier(0);  // keep each step's memory operations where they are written
    }
}

// ---- rows of A given as 4-bit or 3-bit round-to-nearest codes (quant.hip) --------------------------------------
// The gathers then move the codes and parameters of a pair of groups (256 ranks) of the wavefront's 32 rows at a
// time -- 4 instructions of 8 rows x 128 B of codes, and for 4-bit rows one more for the 32 B of parameters of
// each row (3-bit rows carry them inside the 16-byte group pieces) -- into a wavefront-private LDS tile that keeps
// them as they are; a fragment step reads one word of codes (8 ranks) and the group's (step, lo) back and
// de-quantises in registers, x^ = step * code + lo rounded once to bf16, which is the matrix-core operand.
template <int QB> struct QuantTile {
    static constexpr int NG = QB == 4 ? 5 : 4;          // gather instructions per pair of groups and wavefront
    static constexpr int PITCH = QB == 4 ? 176 : 144;   // bytes per row of the code tile (pieces stay 16-byte aligned)
};

// A word with eight codes, even ranks in the low half and odd ranks in the high half, QB bits apart (two adjacent
// ranks are 16 bits apart), and the group's (step, lo) word -> eight bf16 operands.  A code c or-ed onto 0x4300 is
// the bf16 number 128 + c, so x^ = step (128 + c) + (lo - 128 step) is one fused multiply-add per element.
template <int QB> __device__ __forceinline__ bf16x8_t dequant8(uint32_t codes, uint32_t param)
{
    constexpr uint32_t kMask = QB == 4 ? 0x000F000Fu : 0x00070007u;
    const float step = __uint_as_float(param << 16), lo = __uint_as_float(param & 0xFFFF0000u);
    const float lo2 = fmaf(-128.0f, step, lo);
    f32x8_t x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t pr = ((codes >> (QB * i)) & kMask) | 0x43004300u;
        x[2 * i] = fmaf(step, __uint_as_float(pr << 16), lo2);
        x[2 * i + 1] = fmaf(step, __uint_as_float(pr & 0xFFFF0000u), lo2);
    }
    return __builtin_convertvector(x, bf16x8_t);
}

// Gather descriptor of one pair of groups of quantised rows.
struct QStage {
    const unsigned char *base;  // quantised A^K or A^V of this sequence
    size_t pitch;               // bytes per row
    int code_off;               // byte offset of this lane's 16-byte piece of codes within a row
    int par_off;                // byte offset of this lane's 16 bytes of parameters (4-bit rows)
};

// The eight fragment steps of one group (gsel: first or second group of the pair held in the code tile).
template <bool IS_K, int QB>
__device__ __forceinline__ void q_steps(f32x16_t (&acc)[4], const u32x4_t *bcur, const unsigned char *crow, int gsel, int hf)
{
    u32x4_t piece = u32x4_t{0u, 0u, 0u, 0u};
    // 4-bit rows: the group's four (step, lo) words are one 16-byte piece; the codes are read a piece (two steps of
    // both half-wavefronts) at a time as well -- one-word reads of rows 176 bytes apart would collide pairwise
    u32x4_t pars = u32x4_t{0u, 0u, 0u, 0u};
    if constexpr (QB == 4) pars = *reinterpret_cast<const u32x4_t *>(crow + 128 + 16 * gsel);
#pragma unroll
    for (int fl = 0; fl < kGroup; ++fl) {
        uint32_t codes, param;
        if constexpr (QB == 4) {
            // word 16 gsel + 2 fl + hf of the row = word 2 (fl % 2) + hf of piece 4 gsel + fl / 2
            if (fl % 2 == 0) piece = *reinterpret_cast<const u32x4_t *>(crow + 16 * (4 * gsel + fl / 2));
            codes = fl % 2 == 0 ? (hf ? piece[1] : piece[0]) : (hf ? piece[3] : piece[2]);
            param = pars[fl / 2];
        } else {
            // the group's 16-byte piece: 96 bits of codes (four units of 24, unit 2 (fl % 2) + hf is this lane's), then (step, lo)
            if (fl % 2 == 0) piece = *reinterpret_cast<const u32x4_t *>(crow + 16 * (4 * gsel + fl / 2));
            uint32_t u;
            if (fl % 2 == 0)
                u = hf ? ((piece[0] >> 24) | (piece[1] << 8)) : piece[0];
            else
                u = hf ? (piece[2] >> 8) : ((piece[1] >> 16) | (piece[2] << 16));
            codes = (u & 0xFFFu) | ((u << 4) & 0x0FFF0000u);  // odd ranks (bits 12..23) up to bit 16
            param = piece[3];
        }
        const bf16x8_t a0 = dequant8<QB>(codes, param);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const bf16x8_t bf = __builtin_bit_cast(bf16x8_t, bcur[(fl * 4 + db) * 64]);
            if constexpr (IS_K)
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, a0, acc[db], 0, 0, 0);
            else
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bf, acc[db], 0, 0, 0);
        }
    }
}

// One pair of groups from quantised rows.  Vector-memory operations complete in order, so the copies of the B
// fragments must never be the youngest ones when they are awaited: the pair's first group waits for everything (its B
// fragments and this pair's rows, both issued a whole group or more ago), then starts the copy of the second group's B
// fragments and, behind it, the gathers of the next pair; the second group waits until only those gathers are left.
template <bool IS_K, int WAVES, int QB>
__device__ __forceinline__ void run_pair_q(f32x16_t (&acc)[4], u32x4_t (&creg)[QuantTile<QB>::NG], const u32x4_t *Bl,
                                           unsigned char *Ct, uint32_t dma_buf0, uint32_t dma_buf1, const u32x4_t *bsrc1,
                                           const u32x4_t *bsrc2, const QStage &qn, const int (&tkc)[4], int tkp, int lane)
{
    constexpr int NG = QuantTile<QB>::NG, PITCH = QuantTile<QB>::PITCH;
    const int n = lane & 31, hf = lane >> 5;
    XKV_WAIT_VMCNT(0);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
#pragma unroll
    for (int i = 0; i < 32 / WAVES; ++i) copy16_global_to_lds(bsrc1 + i * (WAVES * 64), dma_buf1 + i * (WAVES * 1024));
    // this pair's codes (and parameters) into the code tile, then the registers take the next pair's
#pragma unroll
    for (int i = 0; i < 4; ++i)
        *reinterpret_cast<u32x4_t *>(Ct + (8 * i + (lane >> 3)) * PITCH + 16 * (lane & 7)) = creg[i];
    if constexpr (QB == 4) *reinterpret_cast<u32x4_t *>(Ct + (lane >> 1) * PITCH + 128 + 16 * (lane & 1)) = creg[4];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        creg[i] = *reinterpret_cast<const u32x4_t *>(qn.base + (size_t)tkc[i] * qn.pitch + qn.code_off);
        __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (QB == 4) {
        creg[4] = *reinterpret_cast<const u32x4_t *>(qn.base + (size_t)tkp * qn.pitch + qn.par_off);
        __builtin_amdgcn_sched_barrier(0);
    }
    q_steps<IS_K, QB>(acc, Bl + lane, Ct + n * PITCH, 0, hf);
    __builtin_amdgcn_sched_barrier(0);
    XKV_WAIT_VMCNT(NG);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
#pragma unroll
    for (int i = 0; i < 32 / WAVES; ++i) copy16_global_to_lds(bsrc2 + i * (WAVES * 64), dma_buf0 + i * (WAVES * 1024));
    __builtin_amdgcn_sched_barrier(0);
    q_steps<IS_K, QB>(acc, Bl + kGroup * 256 + lane, Ct + n * PITCH, 1, hf);
    __builtin_amdgcn_sched_barrier(0);
}

// Software pipeline.  The work of a workgroup is a linear sequence of groups of 8 fragment steps, taken in
// pairs: per 256-token tile first the K pairs, then the V pairs (ranks are padded to a multiple of 256 with
// zero fragments).  While a group is multiplied out of one of two LDS buffers, the B fragments of the next
// group are copied straight from global memory into the other, and every wavefront has the gathered pieces of
// the next two groups in flight in registers.
// Eight wavefronts of 32 tokens each: two share a SIMD, so one multiplies while the other waits for memory.
// ROPE: the reconstructed key rows are pre-RoPE (Sec. 4, App. C.6 "Setup") and are rotated to their position (the
// row number) before they meet the query: channel j < 64 is paired with channel j + 64 (Llama / Qwen2 convention) and
// the pair is turned by position * theta^(-j/64).  In the K^T tile both channels of a pair sit in the same lane (blocks
// db and db + 2, same register), so the rotation is register-local.  The angle in revolutions is formed from the
// position split into position / 256 and position % 256 against two per-channel constants (the fraction of 256
// revolutions and of one), which keeps it accurate to 2^-16 of a turn over the whole context, and goes through the
// hardware sine and cosine; the kernel is bound by its gathers, so the extra arithmetic is hidden.
struct RopeTable {
    float f0[64], f1[64];  // theta^(-j/64) / 2 pi, and frac(256 * that)
};

// QB: 0 = rows of A in bf16; 4 or 3 = rows given as 4-bit / 3-bit codes (A_k, A_v then point to quantised rows).
template <int WAVES, bool ROPE, int QB>
__global__ __launch_bounds__(WAVES * 64, 2) void gather_attend_mfma_kernel(
    const bf16_t *__restrict__ A_k, const bf16_t *__restrict__ A_v, const u32x4_t *__restrict__ pack,
    size_t pack_seq_stride, const u32x4_t *__restrict__ pack_q, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ counts,
    float *__restrict__ part_o, float *__restrict__ part_ml, int L, int r_k, int r_v, int H_kv, int H_q, int k,
    int splits, int chunk, int F16k, int F16v, float scale, const RopeTable rope)
{
    constexpr int kLdsA = lds_a_bytes(WAVES), TILE = WAVES * 32;  // selected tokens per workgroup iteration
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    u32x4_t *Bl = reinterpret_cast<u32x4_t *>(smem_raw);
    // workgroup id -> (KV head fastest, so that a head's packed B stays in one XCD's L2), split, sequence
    const int g = blockIdx.x % H_kv;
    const int split = (blockIdx.x / H_kv) % splits;
    const int b = blockIdx.x / (H_kv * splits);
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int n = lane & 31, hf = lane >> 5;
    const int n_rep = H_q / H_kv;
    const int PK = F16k / (2 * kGroup), PT = (F16k + F16v) / (2 * kGroup);  // pairs of groups per tile: K, total

    // this head's B fragments (pack_seq_stride pieces from one sequence to the next: a per-call pack holds one layer,
    // a group's pack all of its layers) and its Q^T fragments, the latter kept in LDS for all wavefronts
    const u32x4_t *packg = pack + (size_t)b * pack_seq_stride + (size_t)g * ((size_t)(F16k + F16v) * 256);
    u32x4_t *At = reinterpret_cast<u32x4_t *>(smem_raw + kLdsB) + w * 512;
    u32x4_t *Ql = reinterpret_cast<u32x4_t *>(smem_raw + kLdsB + kLdsA);  // [8][64]
    for (int i = tid; i < 8 * 64; i += WAVES * 64) Ql[i] = pack_q[((size_t)b * H_kv + g) * 512 + i];

    const u32x4_t *Ak = reinterpret_cast<const u32x4_t *>(A_k + (size_t)b * L * r_k);
    const u32x4_t *Av = reinterpret_cast<const u32x4_t *>(A_v + (size_t)b * L * r_v);
    const int32_t *ids = idx + ((size_t)b * H_kv + g) * k;
    // with `counts`, only the first counts[sequence][head] of the k ids of a row are attended over; a split that
    // lies behind them contributes an empty partial (weight 0 in the merge)
    int k_eff = k;
    if (counts) {
        const int cn = counts[b * H_kv + g];
        k_eff = cn < k ? (cn > 0 ? cn : 0) : k;
    }
    const int m_begin = split * chunk;
    const int m_end_raw = m_begin + chunk < k_eff ? m_begin + chunk : k_eff;
    const int m_end = m_end_raw > m_begin ? m_end_raw : m_begin;
    const int n_tiles = (m_end - m_begin + TILE - 1) / TILE;

    // The split's token ids are staged in LDS once (clamped into [0, L)), so that the main loop issues no
    // global load other than its prefetches: a wait on an id would otherwise drain the whole prefetch queue.
    float *rope_lds = reinterpret_cast<float *>(smem_raw + kLdsB + kLdsA + kLdsQ);  // [128] (ROPE only)
    if constexpr (ROPE) {
        if (tid < 64) rope_lds[tid] = rope.f0[tid];
        else if (tid < 128) rope_lds[tid] = rope.f1[tid - 64];
    }
    int *tok_lds = reinterpret_cast<int *>(smem_raw + kLdsB + kLdsA + kLdsQ + (ROPE ? 512 : 0));  // [chunk]
    for (int m = tid; m < m_end - m_begin; m += WAVES * 64) {
        const int t = ids[m_begin + m];
        tok_lds[m] = t < 0 ? 0 : (t >= L ? L - 1 : t);
    }
    if (m_end == m_begin && tid == 0) tok_lds[0] = 0;  // the prologue below still gathers one (unused) tile
    __syncthreads();
    // the eight rows this lane gathers from in a tile: row 4j + lane/16 of the wavefront's 32-token block.  Past the
    // last tile the pipeline still issues its prefetches (the count of outstanding loads is what its waits rely
    // on); they then all go to the split's first row, which costs a cache hit instead of a tile's worth of memory
    // traffic.
    auto tile_tokens = [&](int tile, int (&tk)[kGroup]) __attribute__((always_inline)) {
        const bool past = tile >= n_tiles;
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            int m = tile * TILE + w * 32 + 4 * j + (lane >> 4);
            m = m < m_end - m_begin ? m : (m_end > m_begin ? m_end - m_begin - 1 : 0);
            tk[j] = tok_lds[past ? 0 : m];
        }
    };
    // gather descriptor of group S (128 ranks each) of the K or V rows; pieces beyond the row are replaced by
    // piece 0 (they meet zero B fragments: any finite value will do)
    auto stage_of = [&](bool is_k, int S) __attribute__((always_inline)) {
        AStage st;
        st.base = is_k ? Ak : Av;
        st.pieces = (is_k ? r_k : r_v) >> 3;
        const int pc = 16 * S + (lane & 15);
        st.piece = pc < st.pieces ? pc : 0;
        return st;
    };
    // LDS tile addressing in 16 B units: piece c of row t sits at 16 t + (c + t) % 16
    int woff[4];
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) woff[qd] = 16 * (lane >> 4) + (((lane & 15) + (lane >> 4) + 4 * qd) & 15);
    const int rbase = 16 * n + ((hf + n) & 15);  // step fl reads (rbase & ~15) + (rbase + 2 fl) % 16

    float m_run = -INFINITY, l_run = 0.0f;
    // Only head slots 0..15 can hold a query head (n_rep <= 16): of the 16 result registers of an O tile the
    // first 8 (slots 8(v/4) + 4hf + v%4, v < 8) are kept between tiles, the rest is dropped.
    float O[4][8];
    f32x16_t acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db) {
#pragma unroll
        for (int v = 0; v < 8; ++v) O[db][v] = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[db][v] = 0.0f;
    }
    bf16x8_t Wf[2];

    // this wavefront's slice of a B buffer as the target of the global -> LDS copies (the hardware adds
    // lane * 16 B): one copy instruction of the workgroup covers two fragment rows (8 KiB)
    const uint32_t lds_b0 = (uint32_t)(uintptr_t)(lds_void_t *)Bl;
    auto dma_base = [&](int bufi) __attribute__((always_inline)) {
        return lds_b0 + (uint32_t)((bufi * (kGroup * 256) + w * 64) * 16);
    };

    // quantised rows: descriptors of a pair of groups, and the rows each lane gathers from (instruction i covers rows
    // 8i .. 8i+7 with 8 pieces of codes each, the parameter instruction rows lane/2)
    constexpr int NGq = QuantTile<QB>::NG;
    const size_t qpitch_k = quant_row_bytes(r_k, QB), qpitch_v = quant_row_bytes(r_v, QB);
    const unsigned char *Qk = reinterpret_cast<const unsigned char *>(A_k) + (size_t)b * L * qpitch_k;
    const unsigned char *Qv = reinterpret_cast<const unsigned char *>(A_v) + (size_t)b * L * qpitch_v;
    unsigned char *Ct = reinterpret_cast<unsigned char *>(At);
    auto qstage_of = [&](bool is_k, int pidx) __attribute__((always_inline)) {
        QStage st;
        const int r = is_k ? r_k : r_v, ng = r >> 5;  // quantisation groups of 32 ranks in a row
        st.base = is_k ? Qk : Qv;
        st.pitch = is_k ? qpitch_k : qpitch_v;
        // groups beyond the row are replaced by group 0 (finite values that meet zero B fragments)
        const int grp = 8 * pidx + (lane & 7), pg = 8 * pidx + 4 * (lane & 1);
        st.code_off = 16 * (grp < ng ? grp : 0);
        st.par_off = (r >> 1) + 4 * (pg < ng ? pg : 0);
        return st;
    };
    auto q_tokens = [&](int tile, int (&tkc)[4], int &tkp) __attribute__((always_inline)) {
        const int last = m_end > m_begin ? m_end - m_begin - 1 : 0;
        const bool past = tile >= n_tiles;  // prefetches past the last tile: all to the split's first row
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = tile * TILE + w * 32 + 8 * i + (lane >> 3);
            tkc[i] = tok_lds[past ? 0 : (m < m_end - m_begin ? m : last)];
        }
        const int mp = tile * TILE + w * 32 + (lane >> 1);
        tkp = tok_lds[past ? 0 : (mp < m_end - m_begin ? mp : last)];
    };

    // ---- prologue, in the order the steady state expects: B fragments of group 0, gathers of groups 0 and 1
#pragma unroll
    for (int i = 0; i < 32 / WAVES; ++i)
        copy16_global_to_lds(packg + i * (WAVES * 64) + tid, dma_base(0) + i * (WAVES * 1024));
    u32x4_t areg[QB == 0 ? 2 * kGroup : 1];
    u32x4_t creg[NGq];
    if constexpr (QB == 0) {
        const AStage s0 = stage_of(true, 0), s1 = stage_of(true, 1);
        int tk0[kGroup];
        tile_tokens(0, tk0);
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            areg[j] = s0.base[(size_t)tk0[j] * s0.pieces + s0.piece];
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            areg[kGroup + j] = s1.base[(size_t)tk0[j] * s1.pieces + s1.piece];
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        const QStage q0 = qstage_of(true, 0);
        int tkc[4], tkp;
        q_tokens(0, tkc, tkp);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            creg[i] = *reinterpret_cast<const u32x4_t *>(q0.base + (size_t)tkc[i] * q0.pitch + q0.code_off);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (QB == 4) creg[4] = *reinterpret_cast<const u32x4_t *>(q0.base + (size_t)tkp * q0.pitch + q0.par_off);
    }

    int gg = 0;  // group counter: group gg is read from buffer gg % 2
    for (int tile = 0; tile < n_tiles; ++tile) {
        const int base = m_begin + tile * TILE + w * 32;
        // descriptors of the pair after pair `pi`: K or V of this tile, or the first K pair of the next tile
#define XKV_NEXT_PAIR(pi)                                                                                     \
    const bool wrap = (pi) + 1 == PT;                                                                         \
    const int pn = wrap ? 0 : (pi) + 1;                                                                       \
    const bool next_k = pn < PK;                                                                              \
    const int S0 = (next_k ? pn : pn - PK) * 2;                                                               \
    const AStage an0 = stage_of(next_k, S0), an1 = stage_of(next_k, S0 + 1);                                  \
    int tkn[kGroup]; /* rows of the tile that pair belongs to */                                              \
    tile_tokens(wrap ? tile + 1 : tile, tkn);                                                                 \
    const u32x4_t *bs1 = packg + (size_t)((pi) * 2 + 1) * (kGroup * 256) + tid; /* second group of this pair */ \
    const u32x4_t *bs2 = packg + (size_t)(pn * 2) * (kGroup * 256) + tid;       /* first group of next pair */  \
    const int buf0 = gg & 1, buf1 = buf0 ^ 1
        // the same for quantised rows: the pair after pair `pi`, its rows, and where the B fragments come from
#define XKV_NEXT_PAIR_Q(pi)                                                                                   \
    const bool wrap = (pi) + 1 == PT;                                                                         \
    const int pn = wrap ? 0 : (pi) + 1;                                                                       \
    const bool next_k = pn < PK;                                                                              \
    const QStage qn = qstage_of(next_k, next_k ? pn : pn - PK);                                               \
    int tkc[4], tkp;                                                                                          \
    q_tokens(wrap ? tile + 1 : tile, tkc, tkp);                                                               \
    const u32x4_t *bs1 = packg + (size_t)((pi) * 2 + 1) * (kGroup * 256) + tid;                               \
    const u32x4_t *bs2 = packg + (size_t)(pn * 2) * (kGroup * 256) + tid
        for (int pi = 0; pi < PK; ++pi, gg += 2) {
            if constexpr (QB == 0) {
                XKV_NEXT_PAIR(pi);
                run_group<true, 0, WAVES>(acc, areg, Bl, At, buf0, dma_base(buf1), bs1, an0, tkn, woff, rbase, lane);
                run_group<true, kGroup, WAVES>(acc, areg, Bl, At, buf1, dma_base(buf0), bs2, an1, tkn, woff, rbase, lane);
            } else {
                XKV_NEXT_PAIR_Q(pi);
                run_pair_q<true, WAVES, QB>(acc, creg, Bl, Ct, dma_base(0), dma_base(1), bs1, bs2, qn, tkc, tkp, lane);
            }
        }
        {
                if constexpr (ROPE) {
                    // K^T tile: lane (token n, hf), register v of block db <-> channel 32 db + 8(v/4) + 4hf + v%4
                    int ml = tile * TILE + w * 32 + n;
                    ml = ml < m_end - m_begin ? ml : (m_end > m_begin ? m_end - m_begin - 1 : 0);
                    const int tpos = tok_lds[ml];
                    const float t_hi = (float)(tpos >> 8), t_lo = (float)(tpos & 255);
#pragma unroll
                    for (int db = 0; db < 2; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int j = 32 * db + 8 * (v / 4) + 4 * hf + (v % 4);
                            const float rev = __builtin_amdgcn_fractf(t_hi * rope_lds[64 + j] + t_lo * rope_lds[j]);
                            const float sn = __builtin_amdgcn_sinf(rev), cs = __builtin_amdgcn_cosf(rev);
                            const float x = acc[db][v], y = acc[db + 2][v];
                            acc[db][v] = x * cs - y * sn;
                            acc[db + 2][v] = y * cs + x * sn;
                        }
                }
                // (2) Z^T = K^ Q^T: lane (head slot n, hf), register v <-> token 8(v/4) + 4hf + v%4 of the block
                f32x16_t Z;
#pragma unroll
                for (int v = 0; v < 16; ++v) Z[v] = 0.0f;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const bf16x8_t qf = __builtin_bit_cast(bf16x8_t, Ql[(db * 2 + j) * 64 + lane]);
                        Z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pack8(acc[db], j), qf, Z, 0, 0, 0);
                    }
                // online softmax; selected tokens beyond the end of this split get weight 0
                float m_loc = -INFINITY;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int tt = base + 8 * (v / 4) + 4 * hf + (v % 4);
                    Z[v] = tt < m_end ? scale * Z[v] : -INFINITY;
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
                Wf[0] = pack8(Z, 0);
                Wf[1] = pack8(Z, 1);
                l_run = l_run * alpha + l_add;
                m_run = m_new;
                // rescale O now: rows are head slots, register v of half hf is slot 8(v/4) + 4hf + v%4
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const float a = __shfl(alpha, 8 * (v / 4) + 4 * hf + (v % 4), kWave);
#pragma unroll
                    for (int db = 0; db < 4; ++db) O[db][v] *= a;
                }
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[db][v] = 0.0f;
        }
        for (int pi = PK; pi < PT; ++pi, gg += 2) {
            if constexpr (QB == 0) {
                XKV_NEXT_PAIR(pi);
                run_group<false, 0, WAVES>(acc, areg, Bl, At, buf0, dma_base(buf1), bs1, an0, tkn, woff, rbase, lane);
                run_group<false, kGroup, WAVES>(acc, areg, Bl, At, buf1, dma_base(buf0), bs2, an1, tkn, woff, rbase, lane);
            } else {
                XKV_NEXT_PAIR_Q(pi);
                run_pair_q<false, WAVES, QB>(acc, creg, Bl, Ct, dma_base(0), dma_base(1), bs1, bs2, qn, tkc, tkp, lane);
            }
        }
#undef XKV_NEXT_PAIR
#undef XKV_NEXT_PAIR_Q
        {
                // (4) O += W V^, one dim block at a time through a scratch result tile
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    f32x16_t ot;
#pragma unroll
                    for (int v = 0; v < 16; ++v) ot[v] = 0.0f;
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        ot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Wf[j], pack8(acc[db], j), ot, 0, 0, 0);
#pragma unroll
                    for (int v = 0; v < 8; ++v) O[db][v] += ot[v];
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[db][v] = 0.0f;
                }
        }
    }

    // all global -> LDS copies must have landed before the buffers are reused for the merge
    XKV_WAIT_VMCNT(0);
    __syncthreads();
    // merge the eight wavefronts in LDS, then write one partial per (split, query head)
    float *mg = reinterpret_cast<float *>(smem_raw);  // [WAVES][16][132]
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
    for (int item = tid; item < n_rep * 128; item += WAVES * 64) {
        const int hh = item >> 7, dim = item & 127;
        float M = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < WAVES; ++ww) M = fmaxf(M, mg[(ww * 16 + hh) * 132 + 128]);
        float num = 0.0f, den = 0.0f;
#pragma unroll
        for (int ww = 0; ww < WAVES; ++ww) {
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

bool gather_attend_mfma_shape_ok(const xkv_shape &s)
{
    return s.dtype == XKV_BF16 && s.d_h == 128 && s.r_k % 16 == 0 && s.r_v % 16 == 0;
}

static inline int frag_rows(int r) { return (r / 16 + 15) / 16 * 16; }  // fragments of 16 ranks, padded to whole pairs of groups

// one layer's packed B, all sequences
static size_t layer_pack_bytes(const xkv_shape &s)
{
    return (size_t)(s.batch > 0 ? s.batch : 1) * s.H_kv * (size_t)(frag_rows(s.r_k) + frag_rows(s.r_v)) * 4 * 1024;
}
static size_t q_pack_bytes(const xkv_shape &s) { return (size_t)(s.batch > 0 ? s.batch : 1) * s.H_kv * 8 * 1024; }

size_t gather_attend_pack_bytes(const xkv_shape &s) { return q_pack_bytes(s) + layer_pack_bytes(s); }
size_t gather_attend_group_pack_bytes(const xkv_shape &s) { return layer_pack_bytes(s) * (size_t)s.G; }

PackArgs gather_attend_pack_args(const xkv_shape &s, int layer, const void *B_k, const void *B_v, const void *q,
                                  void *pack_ws, bool with_b)
{
    PackArgs a;
    a.B_k = (const bf16_t *)B_k;
    a.B_v = (const bf16_t *)B_v;
    a.q = (const bf16_t *)q;
    a.pack_q = (pack_u32x4_t *)pack_ws;
    a.pack = (pack_u32x4_t *)((char *)pack_ws + q_pack_bytes(s));
    a.G = s.G;
    a.layer = layer;
    a.r_k = s.r_k;
    a.r_v = s.r_v;
    a.H_kv = s.H_kv;
    a.H_q = s.H_q;
    a.F8k = frag_rows(s.r_k);
    a.F8v = frag_rows(s.r_v);
    a.batch = s.batch;
    a.dst_G = 1;
    a.dst_layer = 0;
    a.blocks_per_head = with_b ? ((a.F8k + a.F8v) * 64 + 255) / 256 : 0;
    return a;
}

// B of every layer of a group into fragment order, [batch][G][H_kv][...]: what xkv_sr_decode_packed reads.
hipError_t launch_pack_group(const xkv_shape &s, const void *B_k, const void *B_v, void *packed, hipStream_t st)
{
    for (int layer = 0; layer < s.G; ++layer) {
        PackArgs a = gather_attend_pack_args(s, layer, B_k, B_v, nullptr, nullptr, true);
        a.pack = (pack_u32x4_t *)packed;
        a.pack_q = nullptr;
        a.dst_G = s.G;
        a.dst_layer = layer;
        hipLaunchKernelGGL(pack_b_kernel, dim3(a.blocks_per_head, s.H_kv, s.batch), dim3(256), 0, st, a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_gather_attend_mfma(const xkv_shape &s, const Plan &p, int layer, const void *A_k, const void *A_v,
                                     const void *B_k, const void *B_v, const void *q, const int32_t *idx,
                                     void *pack_ws, const void *B_packed, bool packed, float *part_o, float *part_ml,
                                     hipStream_t st, const int32_t *counts, float rope_theta, int qbits)
{
    RopeTable rope{};
    const bool use_rope = rope_theta > 0.0f;
    if (use_rope)
        for (int j = 0; j < 64; ++j) {
            const double f = std::pow((double)rope_theta, -(double)j / 64.0) / 6.283185307179586476925286766559;
            const double f256 = 256.0 * f;
            rope.f0[j] = (float)f;
            rope.f1[j] = (float)(f256 - std::floor(f256));
        }
    const PackArgs pa = gather_attend_pack_args(s, layer, B_k, B_v, q, pack_ws, B_packed == nullptr);
    const int F8k = pa.F8k, F8v = pa.F8v;
    hipError_t e = hipSuccess;
    if (!packed) {
        hipLaunchKernelGGL(pack_b_kernel, dim3(pa.blocks_per_head + kPackQBlocks, s.H_kv, s.batch), dim3(256), 0, st, pa);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (p.sr_chunk > kMaxChunkTokens) return hipErrorInvalidValue;
    // where the kernel finds B: this layer of the group's pack, or the one layer packed into the workspace
    const size_t per_head = (size_t)(F8k + F8v) * 256;  // pieces of 16 B
    const u32x4_t *bsrc = B_packed ? (const u32x4_t *)B_packed + (size_t)layer * s.H_kv * per_head : (const u32x4_t *)pa.pack;
    const size_t seq_stride = (B_packed ? (size_t)s.G : 1) * s.H_kv * per_head;
    dim3 grid((unsigned)((long long)p.sr_splits * s.H_kv * s.batch));
#define XKV_GA_LAUNCH(WV, RP, QB)                                                                                  \
    do {                                                                                                           \
        /* B, A tiles, Q, (rotation constants,) token ids */                                                      \
        const size_t lds = kLdsB + lds_a_bytes(WV) + kLdsQ + (RP ? 512 : 0) + (size_t)p.sr_chunk * 4;              \
        static DynamicLdsOnce attr;                                                                                \
        e = attr.ensure((const void *)gather_attend_mfma_kernel<WV, RP, QB>,                                       \
                        kLdsB + lds_a_bytes(WV) + kLdsQ + 512 + kMaxChunkTokens * 4);                              \
        if (e != hipSuccess) return e;                                                                             \
        profile_begin(1, st);                                                                                      \
        hipLaunchKernelGGL((gather_attend_mfma_kernel<WV, RP, QB>), grid, dim3(WV * 64), lds, st,                  \
                           (const bf16_t *)A_k, (const bf16_t *)A_v, bsrc, seq_stride, (const u32x4_t *)pa.pack_q, \
                           idx, counts, part_o, part_ml, s.L, s.r_k, s.r_v, s.H_kv, s.H_q, s.k, p.sr_splits,       \
                           p.sr_chunk, F8k, F8v, p.scale, rope);                                                   \
        profile_end(1, st);                                                                                        \
    } while (0)
#define XKV_GA_LAUNCH_Q(WV, RP)                                                                                    \
    do {                                                                                                           \
        if (qbits == 4)                                                                                            \
            XKV_GA_LAUNCH(WV, RP, 4);                                                                              \
        else if (qbits == 3)                                                                                       \
            XKV_GA_LAUNCH(WV, RP, 3);                                                                              \
        else                                                                                                       \
            XKV_GA_LAUNCH(WV, RP, 0);                                                                              \
    } while (0)
    if (p.ga_waves == 8) {
        if (use_rope)
            XKV_GA_LAUNCH_Q(8, true);
        else
            XKV_GA_LAUNCH_Q(8, false);
    } else {
        if (use_rope)
            XKV_GA_LAUNCH_Q(4, true);
        else
            XKV_GA_LAUNCH_Q(4, false);
    }
#undef XKV_GA_LAUNCH_Q
#undef XKV_GA_LAUNCH
    return hipGetLastError();
}

// Wavefronts per workgroup for a shape: full 256-token tiles when there are enough selected tokens to give every
// compute unit one, else 128-token tiles so that more compute units take part (64-token tiles lose again: every
// workgroup streams the whole packed B, and two wavefronts do not hide each other's latencies).
int gather_attend_mfma_waves(const xkv_shape &s)
{
    const long long tokens = (long long)s.batch * s.H_kv * s.k;
    return tokens >= 256LL * 256 ? 8 : 4;
}

}  // namespace xkv
