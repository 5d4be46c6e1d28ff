/*
 * xkv.h -- C ABI of libxkv: xKV Selective-Reconstruction (SR) decode attention over a
 * cross-layer factorized KV cache, hand-written for AMD MI355X (gfx950), one GPU.
 *
 * Method (arXiv 2503.18893): a group of G adjacent layers stores its key cache as
 * K_l ~= A^K B^K_l and its value cache as V_l ~= A^V B^V_l, with the token bases
 * A^K [L][r_k], A^V [L][r_v] shared by the group and one small reconstruction matrix
 * B_l [r][d] per layer, d = H_kv * d_h (Sec. 3.1, Eq. 1-2; App. C.6 "Setup").  A decode
 * step of layer l scores every token from the factors, pools the scores of the query
 * heads of each KV head, picks the k best tokens per KV head, reconstructs only those
 * rows (Sec. 3.2, Eq. 3) and runs softmax attention over them.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller (row-major, contiguous,
 *     16-byte aligned).  `shape` and `bytes` are HOST pointers.  `hip_stream` is a
 *     hipStream_t passed as void* (NULL = the default stream).
 *   - Calls validate on the host, enqueue kernels on the stream and return; they do not
 *     allocate, free or synchronise.  Inputs are read-only.  `workspace` is scratch of
 *     at least xkv_workspace_bytes() bytes (256-byte aligned); no state is carried
 *     between calls; two calls in flight at once need two workspaces.
 *   - Errors are returned, never thrown: XKV_ERR_INVALID_ARG for a bad shape or a null
 *     required pointer (nothing is launched), XKV_ERR_WORKSPACE for a workspace that is
 *     too small, XKV_ERR_UNSUPPORTED for a shape no kernel handles, XKV_ERR_HIP when a
 *     launch fails.
 *   - GQA map: rho(h) = h / (H_q / H_kv) (contiguous groups of query heads).
 *   - dtype is the element type of A, B, q, K, V and out; all accumulation is fp32;
 *     scores are fp32 and indices int32.  Inputs must be finite.
 *   - Layouts: A_k [batch][L][r_k], A_v [batch][L][r_v], B_k [batch][G][r_k][H_kv*d_h],
 *     B_v [batch][G][r_v][H_kv*d_h] (KV head g = columns g*d_h .. g*d_h+d_h-1),
 *     q/out [batch][H_q][d_h], pooled scores [batch][H_kv][L], idx [batch][H_kv][k],
 *     dense K/V [batch][H_kv][L][d_h].
 */
#ifndef XKV_H
#define XKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define XKV_API __attribute__((visibility("default")))

typedef enum {
    XKV_OK = 0,
    XKV_ERR_INVALID_ARG = -1,
    XKV_ERR_UNSUPPORTED = -2,
    XKV_ERR_WORKSPACE = -3,
    XKV_ERR_HIP = -4
} xkv_status;

typedef enum { XKV_F32 = 0, XKV_BF16 = 1 } xkv_dtype;

typedef struct xkv_shape {
    int32_t G;     /* layers per group (the paper's window size W, Sec. 3.1)          */
    int32_t H_kv;  /* KV heads                                                        */
    int32_t H_q;   /* query heads, a multiple of H_kv                                 */
    int32_t d_h;   /* per-head width (<= 256)                                         */
    int32_t r_k;   /* rank of the key token basis A^K                                 */
    int32_t r_v;   /* rank of the value token basis A^V (App. C.6 allows r_k != r_v)  */
    int32_t L;     /* tokens in the compressed context                                */
    int32_t k;     /* tokens selected per KV head, 1 <= k <= L                        */
    int32_t batch; /* independent sequences                                           */
    int32_t dtype; /* xkv_dtype                                                       */
    float scale;   /* logit scale, > 0; 0 means 1/sqrt(d_h) (App. B.1, Alg. 2)        */
} xkv_shape;

/* Bytes of scratch any entry point below needs for this shape (host call, no GPU work). */
XKV_API xkv_status xkv_workspace_bytes(const xkv_shape *shape, size_t *bytes);

/*
 * One SR decode step of one layer for every sequence of the batch (Sec. 3.2, Eq. 3, with
 * the scoring, GQA max-pooling and per-KV-head ArgTopK of App. B.1 Alg. 2 applied per
 * token to scores computed from the factors):
 *   p_h = B^K_{l,rho(h)} q_h;  s[h,t] = scale * A^K[t,:] . p_h;  S[g,t] = max_{rho(h)=g} s[h,t];
 *   I_g = the k tokens with the largest S[g,.] (ties: smaller index first);
 *   K^_g = A^K[I_g,:] B^K_{l,g},  V^_g = A^V[I_g,:] B^V_{l,g};
 *   out_h = softmax(scale * K^_{rho(h)} q_h)^T V^_{rho(h)}.
 * layer_in_group in [0, G) picks B_k[:, layer_in_group], B_v[:, layer_in_group].
 * idx_out (nullable) receives the selected token ids, ascending per KV head;
 * score_out (nullable) receives the pooled fp32 scores S.
 */
XKV_API xkv_status xkv_sr_decode(const xkv_shape *shape, int32_t layer_in_group,
                                 const void *A_k, const void *A_v, const void *B_k, const void *B_v,
                                 const void *q, void *out, int32_t *idx_out, float *score_out,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The same step for a context whose T most recent tokens are still uncompressed (Sec. 4, "Implementation
 * details": newly generated tokens are kept uncompressed; Sec. 7, long-generation scenario).  Scoring, pooling
 * and selection run over the L compressed tokens exactly as in xkv_sr_decode; attention then runs over the k
 * reconstructed rows of each KV head together with all T tail rows, one softmax over the union:
 *   out_h = softmax(scale * [K^_{rho(h)} ; K_tail_{rho(h)}] q_h)^T [V^_{rho(h)} ; V_tail_{rho(h)}].
 * K_tail, V_tail: [batch][H_kv][T][d_h] in shape->dtype, T >= 0 (T = 0: identical to xkv_sr_decode, the tail
 * pointers may then be NULL).  XKV_ERR_INVALID_ARG for T < 0 or a missing tail pointer.
 */
XKV_API xkv_status xkv_sr_decode_tail(const xkv_shape *shape, int32_t layer_in_group, const void *A_k,
                                      const void *A_v, const void *B_k, const void *B_v, const void *q,
                                      const void *K_tail, const void *V_tail, int32_t T, void *out,
                                      int32_t *idx_out, float *score_out, void *workspace,
                                      size_t workspace_bytes, void *hip_stream);

/*
 * The same step with the reconstruction matrices prepared once per prompt.  B_l does not change between decode steps
 * (Sec. 3.2: the factors are computed at prefill and kept), but the matrix-core gather-reconstruct kernel reads
 * B^K_{l,g} and B^V_{l,g} in its operand-fragment order, and xkv_sr_decode re-orders them on every call so that it can
 * take the plain layout.  A serving loop re-orders once:
 *   xkv_packed_b_bytes: size of the re-ordered copy of one group's B_k and B_v (all G layers, all sequences); about
 *     the size of B_k and B_v themselves, ranks padded to multiples of 256.
 *   xkv_pack_b: B_k [batch][G][r_k][d], B_v [batch][G][r_v][d] -> packed_out (device, 16-byte aligned, opaque:
 *     [batch][G][H_kv] blocks of 16-rank operand fragments, keys then values, zero beyond the rank).
 *   xkv_sr_decode_packed: xkv_sr_decode with B_v replaced by the packed copy; B_k is still read in its plain layout
 *     by the query projection.  Same kernels otherwise, bit for bit the same results as xkv_sr_decode.
 *   xkv_sr_decode_tail_packed: xkv_sr_decode_tail (K_tail, V_tail, T as there) with B_v replaced by the packed copy.
 *   xkv_sr_decode_landmark_packed: the landmark-guided step (xkv_sr_decode_landmark below, all its arguments) with B_v
 *     replaced by the packed copy; bits = 0 for rows of A in shape->dtype, 4 or 3 for quantised rows
 *     (xkv_sr_decode_landmark_q).  Same results as those calls, bit for bit.
 * XKV_ERR_UNSUPPORTED for shapes the matrix-core kernel does not take (dtype bf16, d_h = 128, ranks multiples of 16,
 * all pointers 16-byte aligned): those callers use xkv_sr_decode.
 */
XKV_API xkv_status xkv_packed_b_bytes(const xkv_shape *shape, size_t *bytes);
XKV_API xkv_status xkv_pack_b(const xkv_shape *shape, const void *B_k, const void *B_v, void *packed_out,
                              void *hip_stream);
XKV_API xkv_status xkv_sr_decode_packed(const xkv_shape *shape, int32_t layer_in_group, const void *A_k,
                                        const void *A_v, const void *B_k, const void *B_packed, const void *q,
                                        void *out, int32_t *idx_out, float *score_out, void *workspace,
                                        size_t workspace_bytes, void *hip_stream);
XKV_API xkv_status xkv_sr_decode_tail_packed(const xkv_shape *shape, int32_t layer_in_group, const void *A_k,
                                             const void *A_v, const void *B_k, const void *B_packed, const void *q,
                                             const void *K_tail, const void *V_tail, int32_t T, void *out,
                                             int32_t *idx_out, float *score_out, void *workspace,
                                             size_t workspace_bytes, void *hip_stream);
XKV_API xkv_status xkv_sr_decode_landmark_packed(const xkv_shape *shape, int32_t layer_in_group, const void *A_k,
                                                 const void *A_v, int32_t bits, const void *B_k, const void *B_packed,
                                                 const void *q, const void *landmarks, const int32_t *outliers,
                                                 int32_t c, int32_t o, float rope_theta, const void *K_tail,
                                                 const void *V_tail, int32_t T, void *out, int32_t *rows_out,
                                                 int32_t *count_out, float *score_out, void *workspace,
                                                 size_t workspace_bytes, void *hip_stream);

/*
 * xkv_sr_decode for callers that cannot allocate device memory or keep a workspace of their own: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit for bit the same
 * results as xkv_sr_decode, but the scratch is an array of XKV_STATIC_SCRATCH_BYTES bytes that is part of the library's
 * code object (each GPU the library runs on holds its own copy until the process ends); the call allocates and frees
 * nothing.  The first call on a device looks the array's address up once (hipGetSymbolAddress).
 * XKV_ERR_WORKSPACE when xkv_workspace_bytes(shape) exceeds XKV_STATIC_SCRATCH_BYTES (nothing is launched): use
 * xkv_sr_decode with a workspace of the caller's then.  All calls on one GPU share the array: calls that may overlap
 * on one GPU (different streams, or different host threads) race and must be serialised by the caller; consecutive
 * calls on one stream are fine.  Nothing in the array is carried from one call to the next.
 */
#define XKV_STATIC_SCRATCH_BYTES (40u << 20)
XKV_API xkv_status xkv_sr_decode_static(const xkv_shape *shape, int32_t layer_in_group, const void *A_k,
                                        const void *A_v, const void *B_k, const void *B_v, const void *q, void *out,
                                        int32_t *idx_out, float *score_out, void *hip_stream);

/*
 * Dense decode attention on an uncompressed cache, the speedup baseline (Sec. 5, "Full
 * Attention"): out_h = softmax(scale * K_{rho(h)} q_h)^T V_{rho(h)} over all L tokens.
 * K, V: [batch][H_kv][L][d_h].  shape->r_k, r_v, k, G are ignored.
 */
XKV_API xkv_status xkv_dense_decode(const xkv_shape *shape, const void *K, const void *V, const void *q,
                                    void *out, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Stage 1 of xkv_sr_decode on its own: pooled scores S [batch][H_kv][L] (fp32) from the
 * key factors and the queries (query projection, low-rank score stream, GQA max-pool). */
XKV_API xkv_status xkv_score(const xkv_shape *shape, int32_t layer_in_group, const void *A_k, const void *B_k,
                             const void *q, float *score_out, void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/* Stage 2 on its own: per-row ArgTopK (App. B.1 Alg. 2, top-k step) of ANY finite fp32 array
 * score [batch][H_kv][L] -> idx_out [batch][H_kv][k].  Order: value descending under the
 * IEEE bit-pattern order (-0.0 < +0.0), ties broken towards the smaller index; exactly k
 * distinct ids per row, written in ascending id order; bit-exact and deterministic. */
XKV_API xkv_status xkv_topk(const xkv_shape *shape, const float *score, int32_t *idx_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/* Stages 3-4 on their own: reconstruct the rows idx [batch][H_kv][k] of K and V (Eq. 3)
 * and attend over them.  Ids must lie in [0, L); they need not be sorted or distinct. */
XKV_API xkv_status xkv_gather_attend(const xkv_shape *shape, int32_t layer_in_group, const void *A_k,
                                     const void *A_v, const void *B_k, const void *B_v, const void *q,
                                     const int32_t *idx, void *out, void *workspace, size_t workspace_bytes,
                                     void *hip_stream);

/* Dense reconstruction X^_l = A B_l for all L tokens (Sec. 3.2), written head-major as
 * X_out [batch][H_kv][L][d_h] in shape->dtype (accumulated in fp32, rounded once).  A is
 * [batch][L][r], B is [batch][G][r][H_kv*d_h]; r is given explicitly so the same call serves
 * keys and values.  Used to build the dense baseline's cache from the factors. */
XKV_API xkv_status xkv_reconstruct(const xkv_shape *shape, int32_t layer_in_group, const void *A, const void *B,
                                   int32_t r, void *X_out, void *hip_stream);

/*
 * Cross-Layer Factorization of one layer group (Sec. 3.1, Eq. 1; run once per prompt at prefill, separately for
 * keys and for values, App. C.6): the caches of the G layers, X [batch][G][H_kv][L][d_h] in shape->dtype (layer l's
 * cache in the dense K/V layout above), are read as X_cat [L][n], n = G * H_kv * d_h, column l*d + g*d_h + j =
 * channel j of KV head g of layer l, and replaced by
 *   B_out [batch][G][r][H_kv*d_h]  B = V^T: the r leading right singular vectors of X_cat as orthonormal rows (before
 *                                  rounding to shape->dtype), in descending order of their singular values, cut into
 *                                  the per-layer blocks B_l,
 *   A_out [batch][L][r]            A = U Sigma = X_cat B^T, so that A^T A = Sigma^2 is diagonal and descending and
 *                                  A [B_1 .. B_G] is the rank-r approximation of Eq. 1.
 * The dominant subspace is found by `iters` rounds of block power iteration on X_cat^T X_cat from a pseudo-random start
 * chosen by `seed` (randomised subspace iteration with Cholesky-QR as in App. B.3); inside it the r x r Rayleigh-Ritz
 * matrix is diagonalised in fp64 (block Jacobi) and the basis rotated to the singular vectors.  The approximation
 * error ||X_cat - A B||_F approaches the optimum of Eq. 1 (the truncated SVD) as iters grows, 8 is a good default;
 * singular vectors are unique up to sign (and up to rotations among equal singular values).
 * xkv_factorize_svd is the same with two options: r_out <= r writes only the leading r_out directions (A_out
 * [batch][L][r_out], B_out [batch][G][r_out][H_kv*d_h]) of a subspace iteration run with r vectors -- the surplus
 * r - r_out act as oversampling, and one run can serve ranks r_K != r_V (Sec. 4: r_K : r_V = 1 : 1.5) by truncation
 * after the fact -- and sigma_out (nullable, device, fp32 [batch][r_out]) receives the singular values.
 * The layouts of A_out and B_out are those xkv_sr_decode takes.  shape->r_k, r_v, k, H_q, scale are ignored.
 * XKV_ERR_UNSUPPORTED unless d_h % 64 == 0, r <= min(1024, n) and n <= 16384; XKV_ERR_INVALID_ARG for iters < 1 or
 * r_out outside [1, r].  workspace: at least xkv_factorize_workspace_bytes() bytes (for r), 256-byte aligned.
 */
XKV_API xkv_status xkv_factorize_workspace_bytes(const xkv_shape *shape, int32_t r, size_t *bytes);
XKV_API xkv_status xkv_factorize(const xkv_shape *shape, const void *X, int32_t r, int32_t iters, uint32_t seed,
                                 void *A_out, void *B_out, void *workspace, size_t workspace_bytes, void *hip_stream);
XKV_API xkv_status xkv_factorize_svd(const xkv_shape *shape, const void *X, int32_t r, int32_t r_out, int32_t iters,
                                     uint32_t seed, void *A_out, void *B_out, float *sigma_out, void *workspace,
                                     size_t workspace_bytes, void *hip_stream);

/*
 * The paper's own selector for Selective Reconstruction (App. B.1 "Landmark-guided Chunk Selector", after ShadowKV),
 * next to the factor-scoring selector of xkv_sr_decode.  The context is cut into n_c = ceil(L / c) chunks of c
 * tokens (the last one may be shorter).
 *
 * xkv_landmarks (Alg. 1, prefill): K_rope [batch][H_kv][L][d_h] post-RoPE keys in shape->dtype ->
 *   landmarks_out   [batch][H_kv][n_c][d_h]  chunk means (fp32 sums, rounded once to shape->dtype),
 *   neg_min_cos_out [batch][H_kv][n_c] fp32 (nullable)  minus the smallest cosine between a key of the chunk and
 *                   its (unrounded) landmark; a zero vector counts as cosine 0,
 *   outliers_out    [batch][H_kv][o] int32 (required when o > 0)  ArgTopK(neg_min_cos, o): the o chunks whose
 *                   minimum cosine is smallest, in the order of xkv_topk (ties: smaller chunk first), ascending.
 * xkv_sr_decode_landmark (Alg. 2 + Eq. 3, decode): P[h][j] = scale <q_h, landmark[rho(h)][j]>, pooled with the
 *   maximum over the query heads of a KV head, top k_ch = min(ceil(k / c), n_c) chunks per KV head (k = shape->k is
 *   the token budget), union with the head's outliers, expansion to token rows; those rows of K and V are
 *   reconstructed and attended over exactly as in xkv_sr_decode.  The union has between k_ch and k_ch + o chunks:
 *   rows_out (nullable) [batch][H_kv][(k_ch + o) * c] receives the rows in ascending order, of which the first
 *   count_out[batch][H_kv] (nullable) are real, the rest 0; score_out (nullable) [batch][H_kv][n_c] the pooled
 *   chunk scores.  landmarks / outliers are xkv_landmarks' outputs (outliers may be NULL when o == 0).  rope_theta
 *   as in xkv_gather_attend_ex below: with landmarks of post-RoPE keys and factors of pre-RoPE keys this is the
 *   paper's arrangement; 0 leaves the reconstructed rows as they are.  K_tail, V_tail, T as in xkv_sr_decode_tail:
 *   the T most recent, uncompressed tokens (keys as the model stored them, i.e. already rotated) join the softmax;
 *   T = 0 and NULL for none.
 * workspace for both: xkv_landmark_workspace_bytes() bytes, 256-byte aligned (xkv_landmarks needs none for o == 0).
 * XKV_ERR_INVALID_ARG for c < 1, o < 0 or o > n_c.
 */
XKV_API xkv_status xkv_landmark_workspace_bytes(const xkv_shape *shape, int32_t c, int32_t o, size_t *bytes);
XKV_API xkv_status xkv_landmarks(const xkv_shape *shape, const void *K_rope, int32_t c, int32_t o, void *landmarks_out,
                                 float *neg_min_cos_out, int32_t *outliers_out, void *workspace, size_t workspace_bytes,
                                 void *hip_stream);
XKV_API xkv_status xkv_sr_decode_landmark(const xkv_shape *shape, int32_t layer_in_group, const void *A_k,
                                          const void *A_v, const void *B_k, const void *B_v, const void *q,
                                          const void *landmarks, const int32_t *outliers, int32_t c, int32_t o,
                                          float rope_theta, const void *K_tail, const void *V_tail, int32_t T,
                                          void *out, int32_t *rows_out, int32_t *count_out, float *score_out,
                                          void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * xkv_gather_attend with two options (stages 3-4 of the step on their own):
 *   counts (nullable) [batch][H_kv]: only the first counts[..] of the k ids of a row are attended over (row lists of
 *     different lengths, as the landmark selector produces them; the other ids must still lie in [0, L)); a KV head
 *     whose count is 0 attends over nothing and its query heads' outputs are written as zeros;
 *   rope_theta > 0: the cache was factorized before the rotary position embedding (Sec. 4 "Implementation details",
 *     App. C.6 "Setup"), so every reconstructed key row is rotated to its position, which is its row number t, before
 *     it meets the (already rotated) query: channel j < d_h/2 is paired with channel j + d_h/2 (Llama / Qwen2
 *     convention) and the pair is turned by t * rope_theta^(-2j/d_h).  Values are not rotated.  0 = no rotation.
 *     XKV_ERR_UNSUPPORTED unless d_h is even and (d_h <= 64 or d_h/2 is a multiple of 64).
 */
XKV_API xkv_status xkv_gather_attend_ex(const xkv_shape *shape, int32_t layer_in_group, const void *A_k,
                                        const void *A_v, const void *B_k, const void *B_v, const void *q,
                                        const int32_t *idx, const int32_t *counts, float rope_theta, void *out,
                                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The SR step in the absorbed form.  Not in the paper: it is this library's re-association of Eq. 3,
 * (A[S] B_l) q = A[S] (B_l q) for the logits and w^T (A^V[S] B^V_l) = (w^T A^V[S]) B^V_l for the output, so that B_l is
 * multiplied into the query and into the output once instead of into every selected token.  Stages 1-2 are unchanged -- same scores, same index sets as
 * xkv_sr_decode -- but the score kernel also keeps every query head's score; stages 3-4 then become
 *     w_h = softmax_j( s_h[I_j] ),      o_h = ( sum_j w_hj A^V[I_j, :] ) B^V_g,
 * which equals softmax(q_h K^_g^T / sqrt(d_h)) V^_g with K^ = A^K[I] B^K, V^ = A^V[I] B^V up to rounding order
 * (K^ and V^ are never rounded to the storage type here).  Only valid where nothing is applied to the reconstructed
 * rows -- not with the rotary embedding of Sec. 4 "Implementation details" applied after reconstruction.  xkv_sr_decode remains the named
 * gather-reconstruct path; this is an additional one.
 *   xkv_head_scores: stage 1 + 2a; heads_out [batch][H_kv][L][nrp] fp32 (device, 16-byte aligned), nrp = H_q/H_kv
 *     rounded up to a power of two, padding written as 0; score_out (nullable) [batch][H_kv][L] is the pooled
 *     score and is the maximum of exactly the values in heads_out.
 *   xkv_attend_absorbed: stages 3-4 from given head scores and ids idx [batch][H_kv][k] (each in [0, L); ids
 *     outside are clamped); out [batch][H_q][d_h] in the shape's dtype.
 *   xkv_sr_decode_absorbed: the whole step; idx_out / score_out nullable as in xkv_sr_decode; K_tail, V_tail, T as
 *     in xkv_sr_decode_tail (the T most recent tokens, uncompressed, join the softmax; T = 0 and NULL for none).
 * workspace for all three: xkv_absorbed_workspace_bytes() bytes, 256-byte aligned (it contains the head scores of
 * one layer, batch * H_kv * L * nrp * 4 bytes).  XKV_ERR_UNSUPPORTED unless rows of A^V are whole 16-byte pieces
 * (r_v a multiple of 8 for bf16, of 4 for fp32); A_v must be 16-byte aligned.
 */
XKV_API xkv_status xkv_absorbed_workspace_bytes(const xkv_shape *shape, size_t *bytes);
XKV_API xkv_status xkv_head_scores(const xkv_shape *shape, int32_t layer_in_group, const void *A_k, const void *B_k,
                                   const void *q, float *score_out, float *heads_out, void *workspace,
                                   size_t workspace_bytes, void *hip_stream);
XKV_API xkv_status xkv_attend_absorbed(const xkv_shape *shape, int32_t layer_in_group, const void *A_v,
                                       const void *B_v, const float *head_scores, const int32_t *idx, void *out,
                                       void *workspace, size_t workspace_bytes, void *hip_stream);
XKV_API xkv_status xkv_sr_decode_absorbed(const xkv_shape *shape, int32_t layer_in_group, const void *A_k,
                                          const void *A_v, const void *B_k, const void *B_v, const void *q,
                                          const void *K_tail, const void *V_tail, int32_t T, void *out,
                                          int32_t *idx_out, float *score_out, void *workspace, size_t workspace_bytes,
                                          void *hip_stream);

/*
 * 4-bit round-to-nearest quantisation of the token basis (App. "Integrate with Quantization": a plain RTN quantiser
 * applied to the compressed cache, 25.6x total at 4 bits).  The paper gives no format; this one is what its ratios
 * imply (one extra bit per element: two 16-bit numbers per group of 32).  A row of r bf16 numbers (r a multiple of
 * 32) becomes 5r/8 bytes, padded with zero bytes to a multiple of 16 (no padding when r is a multiple of 128): r/8 little-endian 32-bit words of codes (word j holds ranks 8j..8j+7: rank 8j+2i in bits
 * [4i, 4i+4), rank 8j+2i+1 in bits [16+4i, 16+4i+4), i = 0..3), then r/32 pairs (step, lo) of bf16.  Per group of 32 consecutive ranks: lo = min, step = bf16((max - lo) / 15)
 * (1 if that is 0), code = clip(rint((x - lo) * (1 / step)), 0, 15) in fp32; the value every later stage sees is
 * x^ = step * code + lo.
 *   xkv_quantized_row_bytes: the row size, or XKV_ERR_UNSUPPORTED (bits not 4 or 3, r not a multiple of 32).
 *   xkv_quantize_rows: X [rows][r] bf16 -> out [rows][row size] bytes (both device, 16-byte aligned).
 *   xkv_attend_absorbed_q4: xkv_attend_absorbed with A^V given as quantised rows Aq_v [batch][L][row size]; the
 *     rows are de-quantised in registers inside the row-sum kernel, so the gather moves 5/16 of the bytes.  bf16
 *     shapes only; B_v, head_scores, idx, out and the workspace as in xkv_attend_absorbed.
 *   xkv_head_scores_q4: xkv_head_scores with A^K given as quantised rows Aq_k [batch][L][5 r_k / 8]: the codes are
 *     the matrix-core operand and a group's (step, lo) is applied to the group's partial sum, so the score stream
 *     is 5/16 of the bytes.  bf16 shapes with at most 8, or 16, query heads per KV head, r_k a multiple of 128.
 *   xkv_sr_decode_absorbed_q4: xkv_sr_decode_absorbed on quantised A^K and A^V (B_k, B_v, q, the tail and the
 *     output stay bf16).  What it computes is the absorbed step on the de-quantised values x^.
 */
/*
 * 3-bit rows (App. "Integrate with Quantization": 32x total at 3 bits = 4 bits per element with the same side
 * information) and the quantised cache in the gather-reconstruct kernels.  bits = 3 in xkv_quantized_row_bytes /
 * xkv_quantize_rows gives r/2 bytes per row: one 16-byte piece per group of 32 ranks, 96 bits of codes read as one
 * little-endian number -- unit u (ranks 8u..8u+7 of the group) in bits [24u, 24u+24), inside a unit rank 8u+2i at bits
 * [3i, 3i+3) and rank 8u+2i+1 at bits [12+3i, 12+3i+3) -- then (step, lo) as two bf16; step = bf16((max - lo) / 7).
 * The calls below run stages 3-4 (Eq. 3 and attention) straight from quantised rows of A^K and A^V: codes and
 * parameters are gathered as they are, de-quantised in registers (x^ = step * code + lo, rounded once to bf16 as the
 * matrix-core operand) and multiplied with B_l, so a rotation can still be applied to the reconstructed key rows -- the
 * paper's own arrangement (factors of pre-RoPE keys, landmark selector, RoPE on reconstruction; Sec. 4 "Implementation
 * details", App. B.1) on a quantised cache.  What they compute is the named step on the de-quantised values x^.
 * bf16 shapes with d_h = 128 and ranks that are multiples of 32 (XKV_ERR_UNSUPPORTED otherwise); bits 4 or 3.
 *   xkv_gather_attend_q: xkv_gather_attend_ex with Aq_k [batch][L][row bytes of r_k], Aq_v likewise.
 *   xkv_sr_decode_landmark_q: xkv_sr_decode_landmark on quantised rows (landmarks stay in shape->dtype).
 *   xkv_sr_decode_q4: the factor-scoring step of xkv_sr_decode on 4-bit rows -- scores from the quantised A^K
 *     (xkv_head_scores_q4's kernel), selection, gather-reconstruct and attention from the quantised rows; rope_theta
 *     and the tail as above; workspace of xkv_absorbed_workspace_bytes() bytes.  (No score kernel reads 3-bit rows:
 *     a 3-bit cache goes with the landmark selector.)
 */
XKV_API xkv_status xkv_gather_attend_q(const xkv_shape *shape, int32_t layer_in_group, const void *Aq_k,
                                       const void *Aq_v, int32_t bits, const void *B_k, const void *B_v, const void *q,
                                       const int32_t *idx, const int32_t *counts, float rope_theta, void *out,
                                       void *workspace, size_t workspace_bytes, void *hip_stream);
XKV_API xkv_status xkv_sr_decode_landmark_q(const xkv_shape *shape, int32_t layer_in_group, const void *Aq_k,
                                            const void *Aq_v, int32_t bits, const void *B_k, const void *B_v,
                                            const void *q, const void *landmarks, const int32_t *outliers, int32_t c,
                                            int32_t o, float rope_theta, const void *K_tail, const void *V_tail,
                                            int32_t T, void *out, int32_t *rows_out, int32_t *count_out,
                                            float *score_out, void *workspace, size_t workspace_bytes, void *hip_stream);
XKV_API xkv_status xkv_sr_decode_q4(const xkv_shape *shape, int32_t layer_in_group, const void *Aq_k, const void *Aq_v,
                                    const void *B_k, const void *B_v, const void *q, float rope_theta,
                                    const void *K_tail, const void *V_tail, int32_t T, void *out, int32_t *idx_out,
                                    float *score_out, void *workspace, size_t workspace_bytes, void *hip_stream);

XKV_API xkv_status xkv_quantized_row_bytes(int32_t r, int32_t bits, size_t *bytes);
XKV_API xkv_status xkv_quantize_rows(const void *X, int64_t rows, int32_t r, int32_t bits, void *out, void *hip_stream);
XKV_API xkv_status xkv_attend_absorbed_q4(const xkv_shape *shape, int32_t layer_in_group, const void *Aq_v,
                                          const void *B_v, const float *head_scores, const int32_t *idx, void *out,
                                          void *workspace, size_t workspace_bytes, void *hip_stream);
XKV_API xkv_status xkv_head_scores_q4(const xkv_shape *shape, int32_t layer_in_group, const void *Aq_k, const void *B_k,
                                      const void *q, float *score_out, float *heads_out, void *workspace,
                                      size_t workspace_bytes, void *hip_stream);
XKV_API xkv_status xkv_sr_decode_absorbed_q4(const xkv_shape *shape, int32_t layer_in_group, const void *Aq_k,
                                             const void *Aq_v, const void *B_k, const void *B_v, const void *q,
                                             const void *K_tail, const void *V_tail, int32_t T, void *out,
                                             int32_t *idx_out, float *score_out, void *workspace,
                                             size_t workspace_bytes, void *hip_stream);

/* Measurement aid for callers that want the duration of one kernel rather than of a whole call.
 * Not part of the method.  For stage = 0 (low-rank score kernel), 1 (gather-reconstruct + sparse
 * attention kernel), 2 (dense decode kernel), 3 (the Gram-matrix product X_cat^T X_cat of xkv_factorize, all
 * sequences of a chunk in one launch) or 4 (the row-sum kernel of xkv_attend_absorbed), every later call that launches that kernel records
 * start_event on the call's stream right before the launch and stop_event right after it.  Both are
 * hipEvent_t created by the caller with timing enabled (HOST handles, passed as void*); NULL for
 * either switches the recording off.  The setting belongs to the calling host thread: only that thread's later calls
 * record, other threads are not affected. */
XKV_API xkv_status xkv_profile_kernel(int32_t stage, void *start_event, void *stop_event);

/* Human-readable name of a status code (static storage). */
XKV_API const char *xkv_status_string(xkv_status status);

/* Library version, major*10000 + minor*100 + patch. */
XKV_API int32_t xkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* XKV_H */
