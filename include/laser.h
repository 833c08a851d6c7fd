/*
 * laser.h - C ABI of the MI355X (gfx950) implementation of LASER's hot path
 * (arxiv 2602.11562): Segmented Target Attention (STA) over a long per-user
 * behaviour history, then Global Stacked Target Attention (GSTA) over the
 * compressed segments.
 *
 * Problem statement (paper Sec. 3.1, generalised from one target item to the C
 * candidates a ranking request scores for one user): a user u has a history of
 * up to L items; item j carries a key K[u,j,:] in R^{d_q} and a value V[u,j,:]
 * in R^{d} (K = H W_k, V = H W_v, already projected); candidate c carries a
 * query Q[u,c,:] in R^{d_q} (Q = t W_q) and a target vector t[u,c,:] in R^{d}.
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer (HBM), caller-owned, row-major,
 *     contiguous, 16-byte aligned. Nothing is copied to or from the host.
 *   - The library allocates nothing, keeps no state and never synchronises: work
 *     is enqueued on `stream` (a hipStream_t; NULL = the default stream). (One exception
 *     to "no state": laser_sta_backward_static owns a fixed scratch array per GPU.)
 *   - Outputs are overwritten in full, including exact zeros for empty segments.
 *   - Return value only; no exception or abort crosses the ABI. Arguments are
 *     validated on the host before anything is launched, so an error return means
 *     no kernel ran. `lens` is device data and cannot be checked on the host: each
 *     value is clamped to [0, L] on the device.
 *   - dtype `dt` is the storage type of q, k, v, t0, the GSTA weights and H'
 *     (LASER_F32 or LASER_BF16). Arithmetic accumulates in fp32. z is always fp32.
 *   - Segment i covers items [i*w, min((i+1)*w, L)); S = ceil(L / w).
 *     Item j of user u is valid iff j < lens[u]. Padded rows are never multiplied
 *     in, so they may hold anything, including NaN or Inf.
 */
#ifndef LASER_H_
#define LASER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LASER_OK = 0,
  LASER_ERR_NULL = 1,        /* a required pointer is NULL                       */
  LASER_ERR_SHAPE = 2,       /* a size is <= 0, too large, or inconsistent       */
  LASER_ERR_DTYPE = 3,       /* dt is not a laser_dtype                          */
  LASER_ERR_UNSUPPORTED = 4, /* valid request that no kernel here implements     */
  LASER_ERR_LAUNCH = 5,      /* the HIP runtime refused a launch                 */
  LASER_ERR_ALIGN = 6,       /* a pointer is not 16-byte aligned                 */
  LASER_STATUS_ANY_INT = 0x7fffffff
} laser_status;

/* (The *_ANY_INT members below name no value of their own: they make every non-negative int a representable value of
 * the enumeration, so that a caller's out-of-range number reaches the library's own check, which answers with
 * LASER_ERR_DTYPE or LASER_ERR_UNSUPPORTED, instead of being undefined behaviour at the call.) */
typedef enum { LASER_F32 = 0, LASER_BF16 = 1, LASER_DTYPE_ANY_INT = 0x7fffffff } laser_dtype;

/* Which STA kernel runs. AUTO picks by (dt, C, d_q, d, w); the others force one
 * and return LASER_ERR_UNSUPPORTED when the shape is outside that kernel's range. */
typedef enum {
  LASER_STA_AUTO = 0,
  LASER_STA_GENERIC = 1, /* fp32 FMA, any shape, either dtype                        */
  LASER_STA_MFMA = 2,    /* bf16 MFMA, many candidates per user                      */
  LASER_STA_STREAM = 3,  /* bf16, few candidates per user, HBM streaming             */
  LASER_STA_MFMA_CACHED = 4, /* LASER_STA_MFMA with H' stored cacheable instead of with the non-temporal hint: for a
                              * caller whose next launch reads H' back (this is the form laser_forward launches) */
  LASER_STA_VARIANT_ANY_INT = 0x7fffffff
} laser_sta_variant;

/* Which GSTA kernel runs. */
typedef enum {
  LASER_GSTA_AUTO = 0,
  LASER_GSTA_GENERIC = 1, /* fp32 FMA, one workgroup per pair, any shape              */
  LASER_GSTA_TILED = 2,   /* bf16 storage, a tile of pairs per workgroup, MFMA, any M */
  LASER_GSTA_SPLIT = 3,   /* bf16 storage, M = 1: projection / streaming / output kernels; z_out is the scratch */
  LASER_GSTA_ONE = 4,     /* bf16 storage, M = 1: the same three steps in one launch, 32 pairs per workgroup */
  LASER_GSTA_VARIANT_ANY_INT = 0x7fffffff
} laser_gsta_variant;

/*
 * Segmented Target Attention, forward (paper Sec. 3.4.2, the STA equation
 *   s_i = Sigmoid(Q K_i^T / gamma) V_i,
 * in the "global scores, then per-segment aggregation" form of Sec. 3.5.1):
 *   seg_out[u,c,i,:] = sum over valid j in segment i of
 *                      sigmoid(dot(q[u,c,:], k[u,j,:]) / gamma) * v[u,j,:]
 *   seg_cnt[u,i]     = number of valid items in segment i
 *
 *   q       [U,C,d_q]  candidate queries
 *   k       [U,L,d_q]  history keys
 *   v       [U,L,d]    history values
 *   lens    [U] int32  valid lengths; NULL means every user has L valid items
 *   gamma   score scale (> 0); the paper leaves its value open
 *   seg_out [U,C,S,d]  H', dtype dt (fp32 sums rounded once to dt)
 *   seg_cnt [U,S] int32, may be NULL
 * Limits: U,C,L,d_q,d,w >= 1; d_q, d <= 1024 and multiples of 8; every tensor < 2^31 elements.
 */
laser_status laser_sta_forward(const void* q, const void* k, const void* v, const int32_t* lens,
                               int U, int C, int L, int d_q, int d, int w, float gamma, laser_dtype dt,
                               void* seg_out, int32_t* seg_cnt, void* stream);

/* Same operation with the kernel chosen by the caller (tests and benchmarks). */
laser_status laser_sta_forward_variant(const void* q, const void* k, const void* v, const int32_t* lens,
                                       int U, int C, int L, int d_q, int d, int w, float gamma, laser_dtype dt,
                                       void* seg_out, int32_t* seg_cnt, void* stream, laser_sta_variant variant);

/*
 * STA with several attention heads (paper Sec. 4.1.2 runs the compression module with 2 heads, d_q = 16 per head, and
 * a value width equal to the embedding width). The paper gives the head count and the widths only; here, as in
 * multi-head attention, head h owns columns [h d_q/heads, (h+1) d_q/heads) of q and k and columns
 * [h d/heads, (h+1) d/heads) of v and seg_out: every head is the STA above on its own columns, with the same gamma,
 * and the heads' outputs lie side by side, so all shapes and layouts are those of laser_sta_forward. heads = 1 is
 * laser_sta_forward_variant. heads must divide d_q and d (1 <= heads <= 64), else LASER_ERR_SHAPE. The streaming
 * kernel takes 1 or 2 heads (d_q/heads and d/heads multiples of 8); the matrix-core kernel takes 1, 2 or 4 heads (d_q / heads a multiple of 16, d / heads of 32); other
 * cases run on the generic kernel (AUTO picks; a forced variant that does not take the case returns
 * LASER_ERR_UNSUPPORTED). Everything else as for laser_sta_forward.
 */
laser_status laser_sta_forward_heads(const void* q, const void* k, const void* v, const int32_t* lens,
                                     int U, int C, int L, int d_q, int d, int w, float gamma, int heads,
                                     laser_dtype dt, void* seg_out, int32_t* seg_cnt, void* stream,
                                     laser_sta_variant variant);

/*
 * The ablation variant of paper Sec. 4.4.1 / Table 4, STA with a softmax over the items in the place of its sigmoid
 * gates:  seg_out[u,c,i,:] = sum_j softmax_j(dot(q[u,c,:], k[u,j,:]) / gamma) * v[u,j,:], the softmax taken over the
 * valid items j of segment i (per head on the head's own columns, as in laser_sta_forward_heads); segments without a
 * valid item give zeros. Arguments, layouts, limits and errors as for laser_sta_forward_heads. Kernels: the streaming
 * kernel for short segments (C <= 8, bf16, w below one step of its long form), the matrix-core kernel (C >= 9, bf16,
 * 1, 2 or 4 heads, its usual widths) and the generic kernel; the long-segment streaming kernel carries sigmoid gates only
 * (a forced variant that does not take the case returns LASER_ERR_UNSUPPORTED).
 */
laser_status laser_sta_forward_softmax(const void* q, const void* k, const void* v, const int32_t* lens,
                                       int U, int C, int L, int d_q, int d, int w, float gamma, int heads,
                                       laser_dtype dt, void* seg_out, int32_t* seg_cnt, void* stream,
                                       laser_sta_variant variant);

/*
 * Global Stacked Target Attention, forward (paper Sec. 3.4.3): for l = 1..M
 *   a_l = softmax((t_{l-1} W_q^l)(H' W_k^l)^T / sqrt(d)),  o_l = a_l (H' W_v^l),  t_l = t_{l-1} + o_l
 * with t_0 = t0 and z = t_M. The softmax runs over the segments of user u that hold at
 * least one valid item (the first ceil(lens[u] / w)); with none, z = t0.
 *
 *   seg   [U,C,S,d]  H' (dtype dt), S = ceil(L / w)
 *   t0    [U,C,d]    target vectors (dtype dt)
 *   wq, wk, wv [M,d,d] each (dtype dt), applied as y = x W (row vector times matrix)
 *   lens  [U] int32 or NULL (all L)
 *   z_out [U,C,d] fp32
 * Limits: d <= 1024 and a multiple of 8; S <= 4096; M >= 1.
 */
laser_status laser_gsta_forward(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                const int32_t* lens, int U, int C, int L, int d, int w, int M, laser_dtype dt,
                                float* z_out, void* stream);

laser_status laser_gsta_forward_variant(const void* seg, const void* t0, const void* wq, const void* wk,
                                        const void* wv, const int32_t* lens, int U, int C, int L, int d, int w,
                                        int M, laser_dtype dt, float* z_out, void* stream,
                                        laser_gsta_variant variant);

/*
 * The whole path: STA, then GSTA on the segment vectors it produced (paper Sec. 3.2,
 * "compress-then-refine"; the per-segment FFN + LayerNorm of Sec. 3.4.2 is not applied,
 * which is the paper's "-FFN+LayerNorm" ablation variant). Arguments as above; seg_cnt may be NULL.
 * seg_out [U,C,S,d] is the buffer GSTA reads: GSTA consumes H' as stored there, i.e. after rounding to dt.
 * seg_out may be NULL when H' is not wanted (M = 1 only; M > 1 returns LASER_ERR_UNSUPPORTED, because every further
 * layer reads every segment vector again): the call is then laser_forward_fused below without a work buffer, i.e.
 * one launch in which every workgroup walks a whole history and nothing but z_out (and seg_cnt) is written.
 */
laser_status laser_forward(const void* q, const void* k, const void* v, const void* t0,
                           const void* wq, const void* wk, const void* wv, const int32_t* lens,
                           int U, int C, int L, int d_q, int d, int w, float gamma, int M, laser_dtype dt,
                           void* seg_out, int32_t* seg_cnt, float* z_out, void* stream);

/*
 * The whole path with one GSTA layer and H' never stored (paper Sec. 3.4.2 and 3.4.3): the attention of Sec. 3.4.3,
 *   a = softmax((t0 W_q)(H' W_k)^T / sqrt(d)),  z = t0 + a (H' W_v),
 * is applied to each segment vector while it is still in registers, as an online softmax over the segments (running
 * maximum, denominator and weighted sum per pair), with the products re-associated (H' (W_k (t0 W_q)^T) and (a H') W_v:
 * exact). Same arguments, layouts, masks and limits as laser_forward with M = 1 (wq, wk, wv [d,d]); the segment vectors
 * enter the layer as fp32 sums, not rounded to dt, so z_out agrees with laser_forward's within the tolerance, not bit
 * for bit. seg_cnt [U,S] may be NULL.
 * work: with few users a history must be cut into runs of segments that different workgroups walk, and each run
 * leaves a partial result (maximum, denominator, weighted sum) per pair that a second, small launch merges in run
 * order (fixed order: results are reproducible). work is caller-owned device scratch for those partial results, 16-byte
 * aligned, at least laser_forward_fused_work_bytes(...) bytes (contents unspecified on return; 0 bytes are needed when
 * there are enough users to fill the machine, or when no kernel here cuts histories for the shape). work may be NULL:
 * every workgroup then walks a whole history, which is always correct and needs no scratch, but leaves compute units
 * idle when U * ceil(C / 128) is small. Kernels: bf16 with d_q in {32, 64, 128} and d in {64, 128} on the matrix cores;
 * everything else (fp32 storage, other widths) on a generic fp32 kernel, one run per user.
 * Errors: as laser_forward, and LASER_ERR_ALIGN (work), LASER_ERR_SHAPE (work_bytes too small). Nothing is launched
 * on an error.
 */
size_t laser_forward_fused_work_bytes(int U, int C, int L, int d_q, int d, int w, laser_dtype dt);   /* host only */
laser_status laser_forward_fused(const void* q, const void* k, const void* v, const void* t0,
                                 const void* wq, const void* wk, const void* wv, const int32_t* lens,
                                 int U, int C, int L, int d_q, int d, int w, float gamma, laser_dtype dt,
                                 int32_t* seg_cnt, float* z_out, void* work, size_t work_bytes, void* stream);

/*
 * Ragged candidate counts per user (serving batches: every request brings its own number of candidates). The pair
 * tensors are packed: q [P,d_q], t0 [P,d], seg_out [P,S,d], z_out [P,d] hold the P pairs of the batch one after the
 * other, user by user, and cand_off [U+1] int32 (device) gives each user's rows, cand_off[u] .. cand_off[u+1]-1, with
 * cand_off[0] = 0, non-decreasing, cand_off[U] = P, and at most C_max rows per user (C_max sizes the launch; users
 * without candidates are allowed). Everything else (k, v, lens, seg_cnt [U,S], weights, arithmetic, kernels, limits
 * with C_max in the place of C) is as in laser_sta_forward / laser_gsta_forward / laser_forward, and with equal
 * counts the results are those of the dense entry points bit for bit. The host cannot see the offsets: on the device
 * they are clamped so that no access leaves the P rows (a user's first row into [0, P], its count into
 * [0, min(C_max, P - first)]); offsets that break the rules above give unspecified values in the rows concerned,
 * never a fault. Rows that belong to no user are not written.
 * Errors: as for the dense entry points, and LASER_ERR_NULL (cand_off), LASER_ERR_ALIGN (cand_off not 4-byte aligned),
 * LASER_ERR_SHAPE (P < 1, P > U * C_max, P * S * d >= 2^31). Nothing is launched on an error.
 */
laser_status laser_sta_forward_ragged(const void* q, const void* k, const void* v, const int32_t* lens,
                                      const int32_t* cand_off, int U, int C_max, int P, int L, int d_q, int d, int w,
                                      float gamma, laser_dtype dt, void* seg_out, int32_t* seg_cnt, void* stream);
laser_status laser_gsta_forward_ragged(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                       const int32_t* lens, const int32_t* cand_off, int U, int C_max, int P, int L,
                                       int d, int w, int M, laser_dtype dt, float* z_out, void* stream);
laser_status laser_forward_ragged(const void* q, const void* k, const void* v, const void* t0, const void* wq,
                                  const void* wk, const void* wv, const int32_t* lens, const int32_t* cand_off, int U,
                                  int C_max, int P, int L, int d_q, int d, int w, float gamma, int M, laser_dtype dt,
                                  void* seg_out, int32_t* seg_cnt, float* z_out, void* stream);

/* The views of Sec. 3.4.4 and the segment FFN + LayerNorm step of Sec. 3.4.2 on packed pairs: seg [P,S,d], pool_out
 * [P,d], recent_out [P,r,d], seg_out [P,S,d]; cand_off, C_max and P as above, everything else as for
 * laser_multires_forward and laser_segment_ffn_forward (kernel chosen as by LASER_FFN_AUTO). */
laser_status laser_multires_forward_ragged(const void* seg, const int32_t* lens, const int32_t* cand_off, int U,
                                           int C_max, int P, int L, int d, int w, int r, laser_dtype dt, void* pool_out,
                                           void* recent_out, void* stream);
laser_status laser_segment_ffn_forward_ragged(const void* seg, const int32_t* lens, const int32_t* cand_off,
                                              const void* w1, const float* b1, const void* w2, const float* b2,
                                              const float* ln_g, const float* ln_b, int U, int C_max, int P, int L,
                                              int d, int d_ff, int w, float eps, laser_dtype dt, void* seg_out,
                                              void* stream);

/*
 * Segment feed-forward step (paper Sec. 3.4.2, the equation after the STA paragraph): every segment vector of H'
 * becomes s <- LN(FFN(s) + s). The paper names neither the network's shape nor the normalisation's constants; here
 *   FFN(s) = relu(s W1 + b1) W2 + b2,  W1 [d, d_ff], W2 [d_ff, d]  (row vector times matrix, as everywhere),
 *   LN(x)  = (x - mean(x)) / sqrt(var(x) + eps) * ln_g + ln_b       over the d components, biased variance.
 * seg [U,C,S,d] dt (H' as stored), lens [U] or NULL as for laser_gsta_forward; w1, w2 in dt; b1 [d_ff], b2 [d],
 * ln_g [d], ln_b [d] in fp32; d_ff a multiple of 8, at most 4096; eps >= 0. seg_out [U,C,S,d] dt is fully
 * overwritten and may be seg itself (in place). Vectors of segments without a valid item (i*w >= lens[u]) are
 * written as zeros. Arithmetic in fp32 (bf16 products on the matrix cores for bf16 storage, the hidden layer
 * rounded to bf16 between the two products); the result is rounded to dt once.
 * All pointers are device pointers, caller-owned; 16-byte alignment for seg, w1, w2, seg_out, 4-byte for the rest.
 * Errors: LASER_ERR_NULL, LASER_ERR_SHAPE, LASER_ERR_DTYPE, LASER_ERR_ALIGN, LASER_ERR_UNSUPPORTED (a forced variant
 * that does not take the shape), LASER_ERR_LAUNCH. Nothing is launched on an error.
 */
typedef enum {
  LASER_FFN_AUTO = 0,
  LASER_FFN_GENERIC = 1, /* fp32 FMA, any d and d_ff, either dtype                                   */
  LASER_FFN_MFMA = 2,    /* bf16 MFMA, d = 128, d_ff in {64, 128}, both weight matrices in LDS     */
  LASER_FFN_VARIANT_ANY_INT = 0x7fffffff
} laser_ffn_variant;

laser_status laser_segment_ffn_forward(const void* seg, const int32_t* lens, const void* w1, const float* b1,
                                       const void* w2, const float* b2, const float* ln_g, const float* ln_b,
                                       int U, int C, int L, int d, int d_ff, int w, float eps, laser_dtype dt,
                                       void* seg_out, void* stream);
laser_status laser_segment_ffn_forward_variant(const void* seg, const int32_t* lens, const void* w1, const float* b1,
                                               const void* w2, const float* b2, const float* ln_g, const float* ln_b,
                                               int U, int C, int L, int d, int d_ff, int w, float eps, laser_dtype dt,
                                               void* seg_out, void* stream, laser_ffn_variant variant);

/*
 * The segment feed-forward step followed by GSTA (paper Sec. 3.4.2, the FFN + LayerNorm equation, then Sec. 3.4.3):
 * z = GSTA(t0; s) with s = LN(FFN(H') + H') as laser_segment_ffn_forward defines it, rounded to dt once as if it
 * were stored. Arguments as for laser_segment_ffn_forward (seg, lens, w1 .. ln_b, d_ff, eps) and laser_gsta_forward
 * (t0, wq, wk, wv, M, z_out); all pointers are device pointers, caller-owned, aligned as there.
 * seg_out [U,C,S,d] dt receives s (fully overwritten, zeros for segments without a valid item); it may be seg itself,
 * and it may be NULL when s is not wanted. bf16, d = 128, d_ff in {64, 128}, M = 1: one pass over H', s is scored
 * and pooled while it is on chip, z_out holds intermediate values until the last of three launches has run. Any
 * other shape: laser_segment_ffn_forward into seg_out, then laser_gsta_forward on it, and LASER_ERR_UNSUPPORTED if
 * seg_out is NULL. Results agree with those two calls in a row up to the order of fp32 sums.
 * Errors: those of the two entry points (seg_out may be NULL), everything validated before the first launch.
 */
laser_status laser_ffn_gsta_forward(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                    const int32_t* lens, const void* w1, const float* b1, const void* w2,
                                    const float* b2, const float* ln_g, const float* ln_b, int U, int C, int L, int d,
                                    int d_ff, int w, int M, float eps, laser_dtype dt, void* seg_out, float* z_out,
                                    void* stream);

/*
 * laser_ffn_gsta_forward with the two other views of Sec. 3.4.4 taken from the transformed rows s (the complete head
 * on a stored H'): pool_out [U,C,d] dt, recent_out [U,C,r,d] dt and r as for laser_multires_forward, everything else
 * as for laser_ffn_gsta_forward, everything validated before the first launch. Where that entry point makes one pass
 * over H' the views come from the same pass; otherwise laser_segment_ffn_forward into seg_out (required then), then
 * laser_gsta_forward_multires on it. z_out, pool_out and recent_out agree with those two calls in a row: the views
 * bit for bit, z_out up to the order of fp32 sums.
 */
laser_status laser_ffn_gsta_forward_multires(const void* seg, const void* t0, const void* wq, const void* wk,
                                             const void* wv, const int32_t* lens, const void* w1, const float* b1,
                                             const void* w2, const float* b2, const float* ln_g, const float* ln_b,
                                             int U, int C, int L, int d, int d_ff, int w, int M, float eps,
                                             laser_dtype dt, void* seg_out, float* z_out, int r, void* pool_out,
                                             void* recent_out, void* stream);

/*
 * Multi-resolution feature fusion (paper Sec. 3.4.4): besides the global context z, the representation holds
 * max_pool(H') and the r most recent segments s_1 .. s_r. Both are taken from a stored H':
 *   pool_out   [U,C,d]   dt   component-wise maximum over the segment vectors of the pair that hold at least one
 *                             valid item (segment i of user u is valid iff i*w < lens[u], as in GSTA); zeros when
 *                             there is none. Exact: a maximum of stored values. May be NULL (not wanted).
 *   recent_out [U,C,r,d] dt   rows 0 .. r-1 of H' (the paper counts the history from its most recent item, so
 *                             s_1 is row 0), copied as stored (zeros for segments without a valid item).
 *                             0 <= r <= S; NULL exactly when r == 0.
 * seg [U,C,S,d] dt and lens [U] (NULL = all L) as for laser_gsta_forward; all pointers are device pointers,
 * caller-owned, 16-byte aligned (lens 4-byte); outputs are fully overwritten; work is enqueued on `stream`.
 * Errors: LASER_ERR_NULL (seg NULL, or both outputs NULL), LASER_ERR_SHAPE (sizes, r out of range, r and
 * recent_out disagree), LASER_ERR_DTYPE, LASER_ERR_ALIGN, LASER_ERR_LAUNCH. Nothing is launched on an error.
 */
laser_status laser_multires_forward(const void* seg, const int32_t* lens, int U, int C, int L, int d, int w, int r,
                                    laser_dtype dt, void* pool_out, void* recent_out, void* stream);

/*
 * The whole path with all three views of Sec. 3.4.4: laser_forward followed by laser_multires_forward on the
 * stored H', same arguments, same results, same errors; everything is validated before the first launch. Where
 * the GSTA kernel holds a pair's H' block in registers (bf16, M = 1, d in {64, 128}, S up to 32 * 64 / (d / 8)) the
 * views are written by that kernel from the same pass over H'; otherwise a third launch reads H' again.
 */
laser_status laser_forward_multires(const void* q, const void* k, const void* v, const void* t0,
                                    const void* wq, const void* wk, const void* wv, const int32_t* lens,
                                    int U, int C, int L, int d_q, int d, int w, float gamma, int M, laser_dtype dt,
                                    void* seg_out, int32_t* seg_cnt, float* z_out,
                                    int r, void* pool_out, void* recent_out, void* stream);

/*
 * GSTA and the two other views of Sec. 3.4.4 from a stored H' (for callers that put a step of their own between STA
 * and GSTA, such as laser_segment_ffn_forward): laser_gsta_forward followed by laser_multires_forward on the same seg,
 * same arguments, same results (z_out, pool_out and recent_out bit for bit), same errors, everything validated before
 * the first launch; H' is read once where the GSTA kernel holds a pair's block in registers (see above), twice
 * otherwise.
 */
laser_status laser_gsta_forward_multires(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                         const int32_t* lens, int U, int C, int L, int d, int w, int M, laser_dtype dt,
                                         float* z_out, int r, void* pool_out, void* recent_out, void* stream);

/*
 * The linear maps ahead of STA (paper Sec. 3.5.1, first two equations): Q = t W_q for the targets, and K = H W_k,
 * V = H W_v for every item of the raw history, both from one pass over H. Row vector times matrix, no bias.
 *   t   [U,C,d_in] dt   target embeddings          w_q [d_in,d_q] dt     q_out [U,C,d_q] dt
 *   h   [U,L,d_in] dt   raw history embeddings     w_k [d_in,d_q] dt     k_out [U,L,d_q] dt
 *                                                  w_v [d_in,d]   dt     v_out [U,L,d]   dt
 * The outputs are the q, k, v arguments of laser_sta_forward / laser_forward (items past a user's valid length are
 * projected like any other; STA never reads them). Products in fp32 (bf16 operands on the matrix cores for bf16
 * storage), accumulated over d_in in fp32, rounded to dt once. 1 <= d_in, d_q, d <= 4096.
 * All pointers are device pointers, caller-owned, 16-byte aligned; outputs are fully overwritten and must not
 * overlap the inputs; work is enqueued on `stream`.
 * Errors: LASER_ERR_NULL, LASER_ERR_SHAPE, LASER_ERR_DTYPE, LASER_ERR_ALIGN, LASER_ERR_UNSUPPORTED (a forced variant
 * that does not take the shape), LASER_ERR_LAUNCH. Nothing is launched on an error.
 */
typedef enum {
  LASER_PROJECT_AUTO = 0,
  LASER_PROJECT_GENERIC = 1, /* fp32 FMA, any sizes, either dtype                                               */
  LASER_PROJECT_MFMA = 2,    /* bf16 MFMA, d_in = 128, output widths multiples of 32, each <= 128, weights in LDS */
  LASER_PROJECT_VARIANT_ANY_INT = 0x7fffffff
} laser_project_variant;

laser_status laser_project_q_forward(const void* t, const void* w_q, int U, int C, int d_in, int d_q, laser_dtype dt,
                                     void* q_out, void* stream);
laser_status laser_project_q_forward_variant(const void* t, const void* w_q, int U, int C, int d_in, int d_q,
                                             laser_dtype dt, void* q_out, void* stream,
                                             laser_project_variant variant);
laser_status laser_project_kv_forward(const void* h, const void* w_k, const void* w_v, int U, int L, int d_in, int d_q,
                                      int d, laser_dtype dt, void* k_out, void* v_out, void* stream);
laser_status laser_project_kv_forward_variant(const void* h, const void* w_k, const void* w_v, int U, int L, int d_in,
                                              int d_q, int d, laser_dtype dt, void* k_out, void* v_out, void* stream,
                                              laser_project_variant variant);

/*
 * Folded form of projections + STA for few candidates per user (paper Sec. 3.5.1: the matrices do not depend on the
 * position, so the products can be re-associated; here that is taken one step further than the paper does). K and V
 * are never formed and the raw history is read once:
 *   score of head h for item j   (t W_q)_h . (h_j W_k)_h  =  (t A_h) . h_j,     A_h = W_q,h W_k,h^T  [d_in, d_in]
 *   segment vector of head h     sum_j g_j (h_j W_v,h)    =  (sum_j g_j h_j) W_v,h
 * with W_x,h head h's run of columns (d_q / heads of W_q and W_k, d / heads of W_v), as in laser_sta_forward_heads.
 *
 * laser_fold_query_weights: a_out [d_in, heads * d_in] dt, A = [A_1 | ... | A_heads], from w_q, w_k [d_in, d_q] dt
 *   (fp32 sums rounded once to dt). Done once per model.
 * laser_project_heads_forward: y[p, i, h b + e] = sum_k x[p, h, i, k] w_v[k, h b + e], b = d / heads;
 *   x [P, heads, S, d_in] dt, w_v [d_in, d] dt, y [P, S, d] dt. d_in, d multiples of 8, heads divides d.
 * laser_sta_folded_forward: the whole chain from raw embeddings to H':
 *   qf_work [U, C * heads, d_in] dt   <- t A                      (laser_project_q_forward with A)
 *   g_work  [U, C * heads, S, d_in] dt <- STA(qf_work, h, h)      (laser_sta_forward: keys = values = raw items)
 *   seg_out [U, C, S, d] dt           <- laser_project_heads_forward(g_work, w_v)
 *   t [U,C,d_in], h [U,L,d_in], a_fold from laser_fold_query_weights, lens / seg_cnt / gamma as for
 *   laser_sta_forward. The two work buffers are caller-owned scratch (contents on return: the intermediates above,
 *   each rounded to dt); the library allocates nothing. Equal to projections followed by STA in exact arithmetic;
 *   in bf16 the intermediates are rounded at other places, so the two forms differ within the tolerance.
 * All pointers are device pointers, caller-owned, 16-byte aligned (lens, seg_cnt 4-byte); work is enqueued on
 * `stream`. Errors as for laser_sta_forward and laser_project_kv_forward; nothing is launched on an error.
 */
laser_status laser_fold_query_weights(const void* w_q, const void* w_k, int d_in, int d_q, int heads, laser_dtype dt,
                                      void* a_out, void* stream);
laser_status laser_project_heads_forward(const void* x, const void* w_v, int P, int S, int d_in, int d, int heads,
                                         laser_dtype dt, void* y, void* stream, laser_project_variant variant);
laser_status laser_sta_folded_forward(const void* t, const void* h, const void* a_fold, const void* w_v,
                                      const int32_t* lens, int U, int C, int L, int d_in, int d, int w, float gamma,
                                      int heads, laser_dtype dt, void* qf_work, void* g_work, void* seg_out,
                                      int32_t* seg_cnt, void* stream);

/*
 * Backward pass of STA (the derivatives of the forward equations of paper Sec. 3.4.2; the paper trains the module,
 * Sec. 4.1.2, and prints no backward formulas). Given dseg = d loss / d H' [U,C,S,d] (dt), with
 *   g_cj = sigmoid(q_c . k_j / gamma)   and   ds_cj = (dseg[c, i(j), :] . v_j) g_cj (1 - g_cj),   i(j) = j / w:
 *   dv_out[u,j,:] = sum_c g_cj dseg[u,c,i(j),:]           [U,L,d]   fp32
 *   dk_out[u,j,:] = sum_c ds_cj q[u,c,:] / gamma          [U,L,d_q] fp32
 *   dq_out[u,c,:] = sum_j ds_cj k[u,j,:] / gamma          [U,C,d_q] fp32
 * over the valid items j < lens[u]; items at or past the valid length get zeros (all outputs are fully overwritten).
 * q, k, v, lens, sizes and gamma as for laser_sta_forward (one head, sigmoid gates). Arithmetic in fp32 from the stored
 * inputs; sums in a fixed order (results are reproducible run to run).
 * Built for training batches, which hold one or a few targets per sample: d_q, d <= 256 (wider rows return
 * LASER_ERR_UNSUPPORTED), and up to eight candidates per user in one pass over k and v; more are taken eight at a
 * time, one pass each, the later passes adding to dk_out and dv_out (correct for any C, fast for few). work is caller-owned scratch of at least laser_sta_backward_work_bytes(U, C, L, d_q, w)
 * bytes (partial dq sums; contents unspecified on return); the library allocates nothing.
 * All pointers are device pointers, 16-byte aligned (lens 4-byte); work is enqueued on `stream`.
 * Errors: LASER_ERR_NULL, LASER_ERR_SHAPE (sizes, gamma, work_bytes too small), LASER_ERR_DTYPE, LASER_ERR_ALIGN,
 * LASER_ERR_UNSUPPORTED, LASER_ERR_LAUNCH. Nothing is launched on an error.
 */
size_t laser_sta_backward_work_bytes(int U, int C, int L, int d_q, int w);   /* host only; 0 for invalid sizes */
laser_status laser_sta_backward(const void* q, const void* k, const void* v, const int32_t* lens, const void* dseg,
                                int U, int C, int L, int d_q, int d, int w, float gamma, laser_dtype dt,
                                float* dq_out, float* dk_out, float* dv_out, void* work, size_t work_bytes,
                                void* stream);

/*
 * The same with bf16 inputs and the two large gradients in bf16 as well: dk_out [U,L,d_q] and dv_out [U,L,d] in the
 * storage type of k and v (fp32 sums rounded once), dq_out [U,C,d_q] fp32. Half the bytes of the pass's largest
 * outputs. C <= 4, d_q in {32, 64, 128}, d in {64, 128}; otherwise LASER_ERR_UNSUPPORTED. Everything else as above.
 */
laser_status laser_sta_backward_bf16(const void* q, const void* k, const void* v, const int32_t* lens, const void* dseg,
                                     int U, int C, int L, int d_q, int d, int w, float gamma, float* dq_out,
                                     void* dk_out, void* dv_out, void* work, size_t work_bytes, void* stream);

/*
 * laser_sta_backward for callers that cannot allocate device memory at all (code under HIP graph capture, tight
 * serving or training loops, harnesses that forbid hipMalloc): the same operation, kernels, results (bit for bit) and
 * errors, with the scratch of partial dq sums taken from a fixed array inside the library instead of a caller's
 * buffer. The array is device memory of the library's own code object, LASER_STATIC_SCRATCH_BYTES per GPU, held by
 * every GPU the library runs on until the process ends; its address is looked up once per device, on the first call
 * with that device current (a symbol lookup, no allocation). The call allocates and frees nothing.
 * Limit: laser_sta_backward_work_bytes(U, C, L, d_q, w) <= LASER_STATIC_SCRATCH_BYTES, else LASER_ERR_SHAPE and
 * nothing is launched (the paper's training batch of 2048 x 1 targets, L = 1000, w = 10, d_q = 32 needs 2.4 MB).
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on the same GPU (two streams, two
 * threads) race on it and must be serialised by the caller; calls in order on one stream are safe. Nothing in the
 * array has to start at zero (every partial sum that is read is written first by the same call).
 */
#define LASER_STATIC_SCRATCH_BYTES (8u << 20)
laser_status laser_sta_backward_static(const void* q, const void* k, const void* v, const int32_t* lens,
                                       const void* dseg, int U, int C, int L, int d_q, int d, int w, float gamma,
                                       laser_dtype dt, float* dq_out, float* dk_out, float* dv_out, void* stream);

/*
 * Backward pass of GSTA (the derivatives of the forward equations of paper Sec. 3.4.3: per layer q' = t W_q,
 * e = (H' W_k) q' / sqrt(d), a = softmax over the valid segments, t <- t + a (H' W_v); the paper prints no backward
 * formulas). Given dz = d loss / d z [U,C,d] (fp32):
 *   dseg_out [U,C,S,d] dt    d loss / d H' through GSTA (rows of segments without a valid item are zeros); this is the
 *                            dseg argument of laser_sta_backward (add the other consumers of H' first, if any)
 *   dt0_out  [U,C,d]   fp32  d loss / d t0
 *   dwq_out, dwk_out, dwv_out [M,d,d] fp32, summed over all pairs in a fixed order
 * seg, t0, wq, wk, wv, lens and the sizes as for laser_gsta_forward. Arithmetic in fp32 from the stored inputs; dseg_out
 * is rounded once to dt. Generic kernels (one workgroup per pair, H' and, with several layers, its gradient in LDS): d <= 256,
 * M <= 8 and S d sizeof(dt) + ((M > 1 ? S d : 0) + (M + 7) d + 2 S + 4) * 4 bytes <= 150 KB; other shapes return LASER_ERR_UNSUPPORTED. work is caller-owned scratch
 * of at least laser_gsta_backward_work_bytes(U, C, d, M) bytes (six d-vectors per pair and layer, whose outer products
 * are the weight gradients, and partial sums of those); the library allocates nothing.
 * All pointers are device pointers, 16-byte aligned (lens 4-byte); outputs are fully overwritten; work is enqueued on
 * `stream`. Errors: LASER_ERR_NULL, LASER_ERR_SHAPE (sizes, work_bytes too small), LASER_ERR_DTYPE, LASER_ERR_ALIGN,
 * LASER_ERR_UNSUPPORTED, LASER_ERR_LAUNCH. Nothing is launched on an error.
 */
size_t laser_gsta_backward_work_bytes(int U, int C, int d, int M);   /* host only; 0 for invalid sizes */
laser_status laser_gsta_backward(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                 const int32_t* lens, const float* dz, int U, int C, int L, int d, int w, int M,
                                 laser_dtype dt, void* dseg_out, float* dt0_out, float* dwq_out, float* dwk_out,
                                 float* dwv_out, void* work, size_t work_bytes, void* stream);

/* Name of the STA / GSTA kernel AUTO would pick for a shape (static strings; host only, no GPU needed). */
const char* laser_sta_kernel_name(int C, int d_q, int d, int w, laser_dtype dt);
const char* laser_gsta_kernel_name(int C, int S, int d, laser_dtype dt);               /* one layer (M = 1) */
const char* laser_gsta_kernel_name_layers(int C, int S, int d, int M, laser_dtype dt);

/* Static, human-readable name of a status code. Never NULL. */
const char* laser_status_string(laser_status s);

/* Library version as major * 10000 + minor * 100 + patch. */
int laser_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LASER_H_ */
