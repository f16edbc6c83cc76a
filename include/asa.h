/*
 * libasa -- Adaptive Block-Sparse Attention (ASA) for AMD MI355X (gfx950).
 *
 * C ABI.  Plain pointers and sizes only.  Every tensor pointer is a DEVICE pointer
 * unless it says HOST.  The caller owns every buffer; the library allocates no device
 * memory, keeps no state between calls and only borrows pointers until the work it
 * enqueued on `hip_stream` has completed.  All calls are asynchronous on that stream
 * (0 / NULL = the default stream); the caller synchronises.
 *
 * Method: "BLADE: Block-Sparse Attention Meets Step Distillation for Efficient Video
 * Generation", Sec. 3.3 (Adaptive Block-Sparse Attention) and appendix "Pseudocode"
 * (Alg. 1 GetMaxPooledAttnMap, Alg. 2 Compute Block Importance Score, Alg. 3 ASA Mask
 * Generation).
 *
 * Layout.  Q, K, V, O, dO, dQ, dK, dV are bf16 tensors [B, H, L, d] with d contiguous.
 * Sequence positions are split into Nb = ceil(L / block) blocks of `block` tokens; the
 * last block may be partial.  A "slab" is one (batch, head) pair, slab index = b*H + h.
 *
 * Errors.  Every entry point returns ASA_OK (0) or a negative asa_status.  Arguments are
 * checked before anything is enqueued, so a failed call writes nothing.  No C++ exception
 * crosses this boundary.
 */
#ifndef ASA_H_
#define ASA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ASA_VERSION 100

typedef enum asa_status {
  ASA_OK = 0,
  ASA_ERR_INVALID_ARG = -1, /* null pointer, bad size, bad parameter, misaligned pointer */
  ASA_ERR_UNSUPPORTED = -2, /* (block, d) pair or size the kernels were not built for     */
  ASA_ERR_WORKSPACE = -3,   /* workspace missing or smaller than the *_workspace_bytes     */
  ASA_ERR_HIP = -4,         /* a HIP call failed; see asa_last_hip_error()                 */
  ASA_ERR_TOO_LARGE = -5    /* asa_attn_bwd_noalloc: the problem needs more scratch memory than
                               ASA_NOALLOC_SCRATCH_BYTES                                      */
} asa_status;

/*
 * Problem description shared by all entry points.
 *
 * Supported: d in {64, 128}; block in {64, 128}; 1 <= L; Nb = ceil(L/block) <= 1024;
 * 1 <= k_samples <= 16, or k_samples == block: every token sampled, the exact importance map
 * that Sec. 3.3 Step 1 defines and the sampling approximates (mask generation then costs as
 * much as dense attention scores and takes L <= 16 384).
 */
typedef struct asa_params {
  int32_t B, H, L, d;
  int32_t block;                 /* b of Sec. 3.3: query-block size == key-block size        */
  int32_t k_samples;             /* k of Alg. 2/3: sampled tokens per block (paper: 16)       */
  const int32_t *sample_offsets; /* HOST pointer to k strictly ascending offsets in [0, b),
                                    the same for every block, head, Q and K (the sampling of
                                    Alg. 3 step 3 is drawn by the caller); NULL selects the
                                    strided default u * (b / k).  Read during the call.      */
  float tau;                     /* cumulative-score threshold of Alg. 3 step 9              */
  float r_min, r_max;            /* minimum / maximum retention ratios of Alg. 3 step 9:
                                    m is clamped to [max(1, ceil(r_min*Nb)),
                                    max(that, floor(r_max*Nb))]; 0 <= r_min <= r_max <= 1     */
  int32_t n_prefix_dense;        /* tokens [0, n): every block holding one is always kept as
                                    a row and as a column (CogVideoX text tokens); 0 = none  */
  float scale;                   /* soft-max scale; 0 selects 1/sqrt(d)                      */
  /* Element strides of the B, H and L axes; d has stride 1.  All zero selects the packed
     layout {H*L*d, L*d, d}.  q_stride also applies to dQ, k_stride to dK, v_stride to dV,
     o_stride to dO.  Strides must be multiples of 8 elements (16-byte rows); the L stride
     must be below 2^24 elements (the kernels address the 64 rows of a tile with 32-bit
     byte offsets).  Anything else: ASA_ERR_INVALID_ARG.                                     */
  int64_t q_stride[3], k_stride[3], v_stride[3], o_stride[3];
} asa_params;

int asa_version(void);
const char *asa_error_string(int status); /* static string, never freed                     */
const char *asa_last_hip_error(void);     /* text of the last HIP failure on this thread    */

/* Workspace sizes in bytes for the calls below (256-byte aligned device memory).           */
size_t asa_mask_workspace_bytes(const asa_params *p);
size_t asa_fwd_workspace_bytes(const asa_params *p);
size_t asa_bwd_workspace_bytes(const asa_params *p);

/*
 * Mask generation (Sec. 3.3 Steps 1 and 2.1; Alg. 2 -> Alg. 1 -> Alg. 3 steps 6-11).
 *
 * From every block of Q and K the k sampled tokens are read; for each sampled query the
 * soft-max over ALL sampled keys of its slab is formed (online, Alg. 1) and max-pooled to
 * the block importance map P_imp [Nb, Nb] (fp32).  Each row of P_imp is then ranked by
 * (score descending, block index ascending); with c_r the fp64 running sum of the r best
 * scores and T the row total, m* = #{r : c_r < tau*T}; m = clamp(m*, m_min, m_max); the m
 * best blocks are kept.  Tokens past L take no part.  A NaN score counts as 0.  The
 * always-kept prefix rows/columns are OR-ed in afterwards.  Every row keeps >= 1 block.
 *
 * Outputs (all device):
 *   mask    [B*H, Nb, Nb] uint8, 1 = keep
 *   row_ptr [B*H, Nb+1]   int32, offsets into this slab's part of col_idx
 *   col_idx [B*H, Nb*Nb]  int32, kept key blocks of each row, ascending; entries past
 *                          row_ptr[Nb] of a slab are left untouched
 *   col_ptr, row_idx      the same mask by columns (for the backward pass); both NULL to skip
 *   p_imp   [B*H, Nb, Nb] fp32 importance map, or NULL
 * The workspace (asa_mask_workspace_bytes) is always needed: it holds the probe's per-row
 * block maxima and, when p_imp is NULL, the importance map.
 */
int asa_build_mask(const asa_params *p, const void *q, const void *k, uint8_t *mask,
                   int32_t *row_ptr, int32_t *col_idx, int32_t *col_ptr, int32_t *row_idx,
                   float *p_imp, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * asa_build_mask with seeded random sampling (Alg. 3 step 2, "randomly sample k tokens from
 * each block", made reproducible): the sample_offsets of `p` are ignored; instead every block
 * of every (batch, head) slab draws its own k_samples positions with a counter-based generator.
 * Position j of block blk of slab s = batch * H + head gets the first word of Philox-4x32-10
 * (Salmon et al., SC'11) with counter (j, blk, s, 0) and key (seed low word, seed high word);
 * the k_samples positions with the smallest (word, j) are the sample, used in ascending order
 * for both Q and K.  asa_sample_offsets writes that table alone:
 *   table [B*H, Nb, k_samples] uint8 (DEVICE).
 * Workspace of the seeded build: asa_mask_seeded_workspace_bytes.
 */
size_t asa_mask_seeded_workspace_bytes(const asa_params *p);
int asa_build_mask_seeded(const asa_params *p, uint64_t seed, const void *q, const void *k,
                          uint8_t *mask, int32_t *row_ptr, int32_t *col_idx, int32_t *col_ptr,
                          int32_t *row_idx, float *p_imp, void *workspace, size_t workspace_bytes,
                          void *hip_stream);
int asa_sample_offsets(const asa_params *p, uint64_t seed, uint8_t *table, void *hip_stream);

/*
 * The selection rule alone (Alg. 3 steps 6-11) on caller-supplied scores
 * [B*H, Nb, Nb] fp32 -> mask [B*H, Nb, Nb] uint8 (prefix rows/columns included).
 */
int asa_mask_from_scores(const asa_params *p, const float *scores, uint8_t *mask,
                         void *hip_stream);

/* Index lists of a caller-supplied mask; same layouts as asa_build_mask.                   */
int asa_csr_from_mask(const asa_params *p, const uint8_t *mask, int32_t *row_ptr,
                      int32_t *col_idx, int32_t *col_ptr, int32_t *row_idx, void *hip_stream);

/*
 * Block-sparse attention forward (Sec. 3.3 Step 2.2, standard ASA).  Query block i attends
 * to the key blocks col_idx[row_ptr[i] .. row_ptr[i+1]) of its slab and to nothing else:
 *   S = scale * Q_i K_j^T (keys >= L excluded),  LSE = log sum exp S,  O = exp(S - LSE) V.
 * o    [B, H, L, d] bf16 (o_stride); rows >= L do not exist and nothing is written there
 * o_lo [B, H, L, d] bf16 (o_stride), optional (NULL to skip): the part of the fp32 result
 *      that rounding to bf16 dropped, o_lo = bf16(O_fp32 - o).  Saved for the backward pass,
 *      whose Delta = rowsum(dO * O) cancels against dO V^T in sharply peaked rows and needs
 *      more than the 8 significant bits of o there.
 * lse  [B*H, L] fp32, natural logarithm; a row with an empty list gets O = 0, LSE = -inf
 * bf16 products accumulate in fp32; probabilities are rounded to bf16 before P V.
 * row_ptr = col_idx = NULL selects the dense specialisation (every key block, no index
 * lists read): the dense attention of the first two sampling steps (Sec. 4.3) and the
 * in-house dense baseline of the kernel-speedup ratio (Table 2); exactly one of them NULL is
 * ASA_ERR_INVALID_ARG.
 */
int asa_attn_fwd(const asa_params *p, const void *q, const void *k, const void *v,
                 const int32_t *row_ptr, const int32_t *col_idx, void *o, void *o_lo, float *lse,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Block-sparse attention backward with the mask held constant (the mask restricts
 * attention "during both training and inference", Sec. 3.3 Step 2.1).  With
 * P = exp(S - LSE), Delta = rowsum(dO * O), dS = P * (dO V^T - Delta):
 *   dV = P^T dO,  dK = scale * dS^T Q,  dQ = scale * dS K     over the kept tiles only.
 * o, o_lo, lse are the forward's outputs; col_ptr/row_idx is the mask by columns.
 * o_lo may be NULL (the plain call): Delta is then not taken from o at all but formed as
 * sum_c P_c (dO V_c^T) over the kept tiles in fp32, by one more walk over the row lists before
 * the gradient kernels (two tile products; about a quarter more time at the Wan2.1 shape).
 * With o_lo, Delta = rowsum(dO * (o + o_lo)) costs one pass over three tensors.  Both meet the
 * same tolerance; Delta from the bf16 o alone would not where keys and queries are large.
 * dq, dk, dv [B, H, L, d] bf16 (q/k/v strides); every row < L is written.
 * All four index-list pointers NULL selects the dense specialisation (see asa_attn_fwd);
 * some but not all NULL is ASA_ERR_INVALID_ARG.
 */
int asa_attn_bwd(const asa_params *p, const void *q, const void *k, const void *v, const void *o,
                 const void *o_lo, const void *d_o, const float *lse, const int32_t *row_ptr,
                 const int32_t *col_idx, const int32_t *col_ptr, const int32_t *row_idx, void *dq,
                 void *dk, void *dv, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * asa_attn_bwd for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving / training loops, harnesses that forbid hipMalloc.
 * Same arguments, results and kernels as asa_attn_bwd, minus the workspace: the scratch memory
 * of the call (the backward's row statistics and the order of its dK / dV workgroups) lives in
 * a device array of ASA_NOALLOC_SCRATCH_BYTES that is part of the library (every GPU the library
 * is used on holds one copy until the process ends).  The call allocates and frees nothing.
 *   - The device that is current at the call must be the device of `hip_stream` and of the
 *     tensors; its array's address is looked up once per device, at the first call there.
 *   - asa_bwd_workspace_bytes(p) > ASA_NOALLOC_SCRATCH_BYTES: ASA_ERR_TOO_LARGE, nothing is
 *     enqueued (the need is 12 bytes per padded token row of all slabs plus 4 bytes per block
 *     row: 8 MiB cover B * H * L up to about 690 000 tokens; the Wan2.1 layer needs 4.7 MiB).
 *   - All calls on one GPU share that GPU's array: two calls whose work overlaps in time on
 *     one GPU (different streams, or several host threads) race; calls on one stream do not.
 *     The array keeps the previous call's contents; no call depends on them.
 */
#define ASA_NOALLOC_SCRATCH_BYTES (8u << 20)
int asa_attn_bwd_noalloc(const asa_params *p, const void *q, const void *k, const void *v,
                         const void *o, const void *o_lo, const void *d_o, const float *lse,
                         const int32_t *row_ptr, const int32_t *col_idx, const int32_t *col_ptr,
                         const int32_t *row_idx, void *dq, void *dk, void *dv, void *hip_stream);

/*
 * ASA with global tokens, ASA_G (Sec. 3.3, "ASA with Global Tokens"): K and V are extended by
 * mean-pooled copies of themselves, K_aug = Concat(K, MeanPool_n(K)) and likewise V.  A query
 * sees the original keys through the block mask exactly as in asa_attn_fwd and, in addition,
 * EVERY pooled key, with ln(n) added to its pre-soft-max score.
 *
 * The pooled part is kept in tensors of its own:
 *   kg, vg [B, H, G, d] bf16, contiguous, G = asa_global_token_count(p, n) = ceil(L/n) rounded
 *   up to a multiple of `block`.  Row w < ceil(L/n) is the mean of tokens [w n, min(L, (w+1) n))
 *   formed in fp32 and rounded to bf16 (the tensor type); rows past ceil(L/n) are zero and are
 *   never attended.  The bias is ln(n) for every window, the short last one included.
 * asa_global_tokens writes kg and vg from k and v.  n: 1 <= n <= L; ceil(L/block) +
 * G/block may not exceed 1024 (ASA_ERR_UNSUPPORTED).
 */
size_t asa_global_token_count(const asa_params *p, int n);   /* 0 on invalid arguments */
int asa_global_tokens(const asa_params *p, int n, const void *k, const void *v, void *kg,
                      void *vg, void *hip_stream);

/*
 * Forward of ASA_G: as asa_attn_fwd with the pooled keys / values kg, vg of window n appended
 * (NULL index lists: dense over the original keys, plus the pooled ones).  LSE covers both
 * parts.  Workspace: asa_fwd_g_workspace_bytes.  ASA_ERR_UNSUPPORTED here: a (batch, head) slab
 * of K spanning 4 GiB or more, and K rows that are not contiguous (k_stride[2] != d).
 */
size_t asa_fwd_g_workspace_bytes(const asa_params *p, int n);
int asa_attn_fwd_g(const asa_params *p, int n, const void *q, const void *k, const void *v,
                   const void *kg, const void *vg, const int32_t *row_ptr, const int32_t *col_idx,
                   void *o, void *o_lo, float *lse, void *workspace, size_t workspace_bytes,
                   void *hip_stream);

/*
 * Backward of ASA_G with the mask held constant.  o, o_lo, lse are asa_attn_fwd_g's outputs.
 * dq, dk, dv [B, H, L, d] bf16 hold the complete gradients: dk and dv include what flows back
 * through the pooling, the gradient of pooled token w divided by the number of tokens of its
 * window, added in fp32 before the one rounding to bf16.  Workspace: asa_bwd_g_workspace_bytes.
 */
size_t asa_bwd_g_workspace_bytes(const asa_params *p, int n);
int asa_attn_bwd_g(const asa_params *p, int n, const void *q, const void *k, const void *v,
                   const void *kg, const void *vg, const void *o, const void *o_lo, const void *d_o,
                   const float *lse, const int32_t *row_ptr, const int32_t *col_idx,
                   const int32_t *col_ptr, const int32_t *row_idx, void *dq, void *dk, void *dv,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Token rearrangement along a Gilbert (generalised Hilbert) curve (Sec. 3.3 "Preprocessing and
 * Importance Estimation"; Alg. 3 step 1): before the sequence is cut into blocks, the tokens of
 * the T x Y x X video grid are put into the order in which a space-filling curve visits them, so
 * that a block holds tokens that are neighbours in the video.  The paper names the curve and does
 * not define it; this library's curve visits every cell once, moves one cell along one axis per
 * step for every grid (its major axis is the longest axis of even length, the longest axis if
 * all are odd), and is the classical Hilbert curve on a 2^k square.
 *
 * asa_gilbert_order -- HOST function, no GPU work.  order, inverse: HOST arrays of
 * n_prefix + T*Y*X int32 (inverse may be NULL).  Position i of the rearranged sequence holds the
 * token that raster order (t major, then y, then x; after n_prefix leading tokens, which keep
 * their places) holds at order[i]; inverse[order[i]] = i.  At most 2^30 tokens.
 *
 * asa_reorder_tokens -- dst[t][b, h, i, :] = src[t][b, h, index[i], :] for t < n_tensors <= 3
 * tensors [B, H, L, d] bf16 in one launch (Q, K, V with index = order before the attention
 * calls; O, dQ, dK, dV with index = inverse after them).  index: DEVICE [L] int32; an entry
 * outside [0, L) gives a zero row.  src, dst: HOST arrays of n_tensors device pointers, read
 * during the call; a tensor cannot be its own destination.  src_stride / dst_stride: element
 * strides {B, H, L} of all sources / all destinations, NULL = packed (the strides in `p` are not
 * used).  Of `p` only B, H, L, d have a meaning here.
 */
int asa_gilbert_order(int32_t T, int32_t Y, int32_t X, int32_t n_prefix, int32_t *order,
                      int32_t *inverse);
int asa_reorder_tokens(const asa_params *p, int32_t n_tensors, const void *const *src,
                       void *const *dst, const int64_t *src_stride, const int64_t *dst_stride,
                       const int32_t *index, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ASA_H_ */
