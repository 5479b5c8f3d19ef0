/*
 * kvzap.h -- C ABI of the KVzap prune step for AMD MI355X (gfx950).
 *
 * KVzap (arXiv 2601.07891) prunes a transformer layer's KV cache in three
 * steps (Sec. 3.3, Algorithm 1): a small per-layer surrogate maps every
 * token's hidden state to one importance score per KV head; scores are compared
 * with one global threshold tau, the most recent `window` positions being kept
 * unconditionally; the surviving K/V rows of every head are gathered, in
 * position order, into a cache whose length differs from head to head (Sec. 5).
 * While decoding, the same rule is applied one token at a time, with a buffer
 * of the scores of the tokens still inside the window (caption of Algorithm 1).
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer into memory owned by the caller, unless
 *     a parameter says "host".  The library allocates no device memory, keeps no
 *     pointer after a call returns, and never synchronises: every call only
 *     enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  The caller keeps all buffers alive until the stream has
 *     drained.
 *   - bf16 tensors are raw 16-bit patterns (upper half of an IEEE fp32).
 *   - All tensors are dense, row-major, in the index order written beside them.
 *     Base pointers must be 16-byte aligned (KVZAP_ERR_ALIGN otherwise).
 *   - Scratch memory comes from a caller-provided workspace whose minimum size
 *     is given by kvzap_workspace_bytes(); it must be 256-byte aligned and is
 *     free for reuse once the call's kernels have run.
 *   - Return value: KVZAP_OK (0) or a negative kvzap_status.  Arguments are
 *     validated on the host before anything is enqueued; on error nothing is
 *     launched and no output is written.  No call throws or aborts.
 *   - Supported shapes: H (KV heads) in [1, 16]; D (head dim) a multiple of 8
 *     with D <= 512 (rows are moved in 16-byte pieces); D_h a multiple of 64;
 *     the MLP width M a multiple of 128 with M <= 640; at most 65535 (sequence, head)
 *     rows per call (B*H) and T <= 2^31 - 2^20 - 1 positions in the calls that index
 *     positions (mask, top-k, compaction).  Anything else returns KVZAP_ERR_UNSUPPORTED;
 *     there is no fallback path.
 *   - Weight storage is output-major, the way a PyTorch linear module stores
 *     it: the paper's W1 in R^{D_h x M} (App. B) is passed as its transpose
 *     [M, D_h], W2 in R^{M x H} as [H, M], the linear surrogate's D_h x H matrix
 *     as [H, D_h].  Every output unit's D_h inputs are therefore contiguous.
 */
#ifndef KVZAP_H_
#define KVZAP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum kvzap_status {
  KVZAP_OK = 0,
  KVZAP_ERR_NULL = -1,        /* a required pointer is NULL                    */
  KVZAP_ERR_SHAPE = -2,       /* a size is negative, zero where it may not be, or overflows */
  KVZAP_ERR_ALIGN = -3,       /* a base pointer is not 16-byte aligned         */
  KVZAP_ERR_UNSUPPORTED = -4, /* legal but outside the supported shapes        */
  KVZAP_ERR_CAPACITY = -5,    /* an output buffer is too small for the worst case */
  KVZAP_ERR_WORKSPACE = -6,   /* workspace missing, misaligned or too small    */
  KVZAP_ERR_RUNTIME = -7,     /* a HIP launch failed (see hipGetLastError)     */
  KVZAP_ERR_STATIC_LIMIT = -8 /* input larger than kvzap_mask_static's built-in scratch */
} kvzap_status;

/* Which call a workspace query is for. */
typedef enum kvzap_call {
  KVZAP_CALL_SCORE = 0,
  KVZAP_CALL_MASK = 1,
  KVZAP_CALL_COMPACT = 2,
  KVZAP_CALL_DECODE_EVICT = 3,
  KVZAP_CALL_ATTEND_DECODE = 4,  /* pass T = max_rows, Dh = HQ, M = window (also for the paged form) */
  KVZAP_CALL_ASSIGN_PAGES = 5,   /* only B and H matter (pass T = 1) */
  KVZAP_CALL_TOPK_THRESHOLD = 6, /* pass M = per_layer (0 or 1) */
  KVZAP_CALL_TEACHER_SCORES = 7, /* pass B = 1, T = prompt length, Dh = HQ, M = Tq */
  KVZAP_CALL_COMPRESS = 8,       /* as KVZAP_CALL_SCORE: the larger of the score and mask needs */
  KVZAP_CALL_MASK_COMPACT = 9    /* as KVZAP_CALL_MASK */
} kvzap_call;

/* Text for a status code (host pointer to a static string, never NULL). */
const char* kvzap_status_string(int status);

/* Library version, "major.minor.patch" (host pointer to a static string). */
const char* kvzap_version(void);

/*
 * Minimum workspace size in bytes for one call.  For KVZAP_CALL_DECODE_EVICT
 * pass T = 1 (one new token per sequence).  Returns 0 for calls that need no
 * workspace and for invalid arguments.  Pure host function.
 * KVZAP_CALL_SCORE with M > 0 needs M*Dh*2 bytes: every call copies W1 there in
 * the order the matrix-core loads want it (a few microseconds); for inputs too short
 * to fill the chip (B*T up to about 16k tokens) it needs more, for the fp32 partial sums
 * of a first projection that is split over K -- so query with the B and T of the call.
 */
size_t kvzap_workspace_bytes(int which_call, int B, int T, int Dh, int M, int H);

/*
 * kvzap_score -- the surrogate forward (Sec. 3.3; Sec. 4.1; App. B Eq. 5-6).
 *
 *   M == 0 : KVzap-Linear   scores[b,h,t] = sum_k hidden[b,t,k] * W1[h,k] + b1[h]
 *   M  > 0 : KVzap-MLP      z = hidden[b,t,:] . W1[m,:] + b1[m]        (m < M)
 *                           g = GELU(z) = z * Phi(z)  (erf form, not the tanh one; evaluated in
 *                               fp32 to 2.6e-5 absolute, see "Arithmetic")
 *                           scores[b,h,t] = sum_m g[m] * W2[h,m] + b2[h]
 *
 *   hidden  bf16 [B, T, Dh]
 *   W1      bf16 [M, Dh] (MLP) or [H, Dh] (linear)
 *   b1      bf16 [M] (MLP) or [H] (linear); NULL = zero
 *   W2      bf16 [H, M]; must be NULL iff M == 0
 *   b2      bf16 [H]; NULL = zero; must be NULL if M == 0
 *   scores  fp32 [B, H, T]  (positions on the last axis, as Algorithm 1 indexes
 *           them); fully overwritten.
 *
 * workspace: see kvzap_workspace_bytes(KVZAP_CALL_SCORE, ...); may be NULL when
 * that is 0 (linear surrogate).  KVZAP_ERR_WORKSPACE if missing, misaligned or small.
 *
 * Arithmetic: bf16 products accumulated in fp32 on the matrix cores (the accumulation starts
 * from b1).  In the single-kernel path GELU is z * sigmoid(z * p(z^2)) with a fitted cubic p,
 * within 2.6e-5 (absolute) of z * Phi(z) for every z, evaluated in fp32; its result is rounded
 * to fp16 (relative 2^-11; values beyond 65504 become infinite) and W2 is converted to fp16
 * (exact for bf16 magnitudes in [2^-14, 65504], subnormal or infinite beyond) for the second
 * projection on the matrix cores, accumulated in fp32.  Short inputs (see the workspace
 * query) take a split first projection whose GELU (erf to 1.5e-7) and second projection are
 * plain fp32.  Both are far inside the 1e-2 score tolerance.  The sum order is fixed for a
 * given shape, so results are run-to-run deterministic; the same token scored in calls of
 * different B*T may differ in the last bits.  B*T == 0 is a no-op.
 */
int kvzap_score(const void* hidden, const void* W1, const void* b1,
                const void* W2, const void* b2, float* scores,
                int B, int T, int Dh, int M, int H,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_prepare_scorer_rmsnorm / kvzap_score_rmsnorm -- the MLP surrogate fused into the
 * layer's input normalisation (Sec. 3: the surrogate is applied to the layer's input hidden
 * states; Sec. 5: what an inference engine has to fuse).  The caller holds the un-normalised
 * residual stream x; the layer's input RMSNorm
 *
 *     hidden[b,t,k] = x[b,t,k] * rstd[b,t] * gain[k],   rstd = 1 / sqrt(mean_k x[b,t,k]^2 + eps)
 *
 * and kvzap_score on `hidden` become one kernel that reads x once: the gain is folded into
 * the prepared copy of W1 (W1[m,k] * gain[k], rounded to bf16, in the matrix cores' operand
 * order), the sum of squares of every token is accumulated beside the first projection, and
 * rstd is applied to the accumulators before b1 and GELU:
 *
 *     z[m] = rstd * sum_k x[k] * (W1[m,k] * gain[k]) + b1[m]
 *
 *   x            bf16 [B, T, Dh]   the residual stream (layer input before its norm)
 *   gain         bf16 [Dh]
 *   eps          >= 0
 *   W1_prepared  from kvzap_prepare_scorer_rmsnorm(W1 bf16 [M, Dh], gain): device, 256-byte
 *                aligned, at least M*Dh*2 bytes rounded up to 256, not overlapping W1
 *   b1, W2, b2   as kvzap_score (MLP form)
 *   scores       fp32 [B, H, T], fully overwritten
 *   rstd         fp32 [B, T], fully overwritten: all that a consumer which folds the gain into
 *                its own weights (as done here) needs in order to apply the norm in its epilogue
 *   normed       bf16 [B, T, Dh] or NULL.  If given, it receives x * rstd * gain rounded to bf16
 *                -- the states the layer's projections read.  A token's rstd is known only when
 *                its whole row has passed, so each thread block then goes over its 128 (96) rows
 *                a second time: x is read twice and `normed` written once, which is the traffic
 *                of the separate norm and scorer, but inside one launch.  Must not overlap x.
 *
 * MLP surrogates only (M > 0; M == 0 returns KVZAP_ERR_UNSUPPORTED), Dh >= 256; always the
 * single-kernel path (no workspace).  Arithmetic as kvzap_score's single-kernel path; the sum
 * of squares is accumulated in fp32 from bf16 pairs.  Scores equal those of kvzap_score on a
 * separately normalised input up to the bf16 rounding that pipeline applies to `hidden` and
 * this one to W1 * gain: both are within the score tolerance of the un-rounded definition.
 */
int kvzap_prepare_scorer_rmsnorm(const void* W1, const void* gain, int Dh, int M,
                                 void* W1_prepared, size_t prepared_bytes, void* stream);
int kvzap_score_rmsnorm(const void* x, const void* W1_prepared, const void* gain, float eps,
                        const void* b1, const void* W2, const void* b2,
                        float* scores, float* rstd, void* normed,
                        int B, int T, int Dh, int M, int H, void* stream);

/*
 * kvzap_mask -- threshold plus sliding window (Sec. 3.3; Algorithm 1).
 *
 *   keep[b,h,t] = t < T_b  and  ( t >= T_b - window  or  scores[b,h,t] >= tau )
 *
 * with T_b = seq_lens[b] (or T when seq_lens is NULL).  Equality keeps; a NaN
 * score is dropped unless the window protects it; window = 0 protects nothing;
 * window >= T_b keeps everything; tau may be +-infinity.
 *
 *   scores    fp32 [B, H, T]
 *   seq_lens  int32 [B], 0 <= seq_lens[b] <= T, or NULL   (right-padded batch)
 *   keep_idx  int32, capacity B*H*T entries: kept positions t, ascending within
 *             a head, heads packed back to back in (b,h) row-major order; head
 *             (b,h) occupies keep_idx[offsets[b*H+h] .. +lengths[b,h])
 *   lengths   int32 [B, H]     number of kept positions
 *   offsets   int64 [B*H + 1]  exclusive prefix sum of lengths; the last entry
 *             is the total number of kept rows
 *
 * Exactly one result is correct and it is reproduced bit for bit.
 */
int kvzap_mask(const float* scores, float tau, int window,
               const int32_t* seq_lens, int B, int H, int T,
               int32_t* keep_idx, int32_t* lengths, int64_t* offsets,
               void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_mask_static -- kvzap_mask for callers that cannot allocate device memory or hand over
 * a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (minus the workspace), same kernels, same result bit for bit.
 * The scratch kvzap_mask keeps in its workspace lives in a buffer built into the library
 * instead (KVZAP_MASK_STATIC_MAX_CHUNKS * 12 bytes = 768 KiB per GPU, held until the process
 * ends), so the call allocates nothing and frees nothing.
 *
 * Limit: B * H * ceil(T / 1024) <= KVZAP_MASK_STATIC_MAX_CHUNKS (64 Mi score entries, e.g.
 * 8 heads of 8 Mi positions); beyond it KVZAP_ERR_STATIC_LIMIT, nothing launched.
 * All calls on one GPU share that GPU's buffer: calls whose kernels may overlap on one GPU
 * (different streams, no dependency between them) race; calls on one stream, or ordered by
 * events, are fine.  Nothing in the buffer needs clearing between calls.  The first call on a
 * device looks up the buffer's address on that device (hipGetSymbolAddress, with that device
 * current); make that call once outside any stream capture.  KVZAP_ERR_RUNTIME if the lookup
 * fails or the device ordinal is 64 or more.
 */
#define KVZAP_MASK_STATIC_MAX_CHUNKS 65536
int kvzap_mask_static(const float* scores, float tau, int window,
                      const int32_t* seq_lens, int B, int H, int T,
                      int32_t* keep_idx, int32_t* lengths, int64_t* offsets,
                      void* stream);

/*
 * kvzap_prepare_scorer / kvzap_score_prepared -- kvzap_score for MLP surrogates (Sec. 3.3,
 * App. B Eq. 5) whose weights do not change between calls: kvzap_score re-orders W1 into the
 * matrix cores' operand order in its workspace on every call; kvzap_prepare_scorer does that
 * once, into a buffer the caller keeps (W1_prepared: device, 256-byte aligned, at least
 * M * Dh * 2 bytes rounded up to 256, not overlapping W1), and
 * kvzap_score_prepared takes that buffer in place of W1 and needs no workspace.  Scores are
 * bit-identical to kvzap_score's when that runs the same single kernel (from about 16k
 * tokens); for shorter inputs kvzap_score splits the first projection over K (it has the
 * workspace for the partial sums) and the two agree within fp32 rounding.  M > 0 only (the linear surrogate has nothing to prepare);
 * other arguments, layouts and errors as kvzap_score.  The prepared layout is private to
 * the library version that wrote it.
 */
int kvzap_prepare_scorer(const void* W1, int Dh, int M, void* W1_prepared, size_t prepared_bytes,
                         void* stream);
int kvzap_score_prepared(const void* hidden, const void* W1_prepared, const void* b1,
                         const void* W2, const void* b2, float* scores, int B, int T, int Dh,
                         int M, int H, void* stream);

/*
 * kvzap_topk_threshold -- thresholds for the fixed-budget variants (Sec. 3.3: keeping a
 * fixed fraction; Sec. 4 ablation: fixed-ratio top-k per head, or per layer as in AdaKV).
 * The population of head (b,h) is its non-window positions t < T_b - window whose score is
 * not NaN.  per_layer == 0: tau_out[b,h] = the k-th largest score of that population.
 * per_layer != 0: the populations of the H heads of sequence b are pooled and
 * tau_out[b,:] = the k-th largest of the pool (one budget of k shared by the heads).
 * k <= 0 gives +inf, k >= the population size gives -inf.  Feeding tau_out to
 * kvzap_mask_per_head keeps {score >= tau} plus the window: exactly k non-window entries
 * per head (per sequence) when scores are distinct, all entries tied with the k-th largest
 * otherwise.  Exact (a radix select on the bits): no tolerance.
 *   scores fp32 [B,H,T]; seq_lens int32 [B] or NULL; tau_out fp32 [B,H] (device).
 *   workspace: kvzap_workspace_bytes(KVZAP_CALL_TOPK_THRESHOLD, B, T, 0, per_layer, H).
 */
int kvzap_topk_threshold(const float* scores, int window, const int32_t* seq_lens,
                         int64_t k, int per_layer, int B, int H, int T, float* tau_out,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_mask_per_head -- kvzap_mask with one threshold per (sequence, head), read from
 * device memory: tau fp32 [B,H] (NaN entries keep nothing but the window).  Everything else
 * as kvzap_mask, including the workspace.
 */
int kvzap_mask_per_head(const float* scores, const float* tau, int window,
                        const int32_t* seq_lens, int B, int H, int T,
                        int32_t* keep_idx, int32_t* lengths, int64_t* offsets,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_compact -- the ragged per-head gather (Algorithm 1, last line; Sec. 5).
 *
 *   K_out[offsets[b*H+h] + j, :] = K[b, h, keep_idx[offsets[b*H+h] + j], :]
 *   for j < lengths[b,h]; the same for V.  Rows are copied byte for byte.
 *
 *   K, V          bf16 [B, H, T, D]
 *   keep_idx, lengths, offsets   as written by kvzap_mask (device memory)
 *   K_out, V_out  bf16 [cap_rows, D]; must not overlap K or V
 *   cap_rows      rows available in K_out and V_out.  The kept total lives on
 *                 the device, so it cannot be checked on the host: rows at or
 *                 beyond cap_rows are not written (never out of bounds), and
 *                 cap_rows = B*H*T is always sufficient.
 */
int kvzap_compact(const void* K, const void* V, const int32_t* keep_idx,
                  const int32_t* lengths, const int64_t* offsets,
                  void* K_out, void* V_out, int64_t cap_rows,
                  int B, int H, int T, int D, void* stream);

/*
 * kvzap_mask_compact -- the last three lines of Algorithm 1 (window, threshold, gather) in one
 * call: kvzap_mask followed by kvzap_compact, with the arguments and the results of those two
 * calls, bit for bit (keep_idx, lengths and offsets are written as kvzap_mask writes them).
 * The kernels are those of the two calls (a gather fused into the ranking kernel measured
 * slower than the separate gather, whose one-row-per-thread grid keeps more of HBM busy); what
 * the single call adds is that all checks of both happen before the first launch.
 * workspace: kvzap_workspace_bytes(KVZAP_CALL_MASK_COMPACT, B, T, 0, 0, H), as for kvzap_mask.
 */
int kvzap_mask_compact(const float* scores, float tau, int window, const int32_t* seq_lens,
                       const void* K, const void* V, int32_t* keep_idx, int32_t* lengths,
                       int64_t* offsets, void* K_out, void* V_out, int64_t cap_rows,
                       int B, int H, int T, int D,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_compress -- the whole of Algorithm 1 for one layer in one call: kvzap_score, then
 * kvzap_mask_compact on the same stream, with the arguments of those calls (`scores`
 * receives the surrogate's scores and is part of the result).  Identical, bit for bit, to
 * making the three calls kvzap_score, kvzap_mask, kvzap_compact; validation of all three
 * happens before the first launch.  (Counting the kept scores inside the scorer, to save the
 * mask's first kernel, measured no faster end to end and is not done.)
 * workspace: kvzap_workspace_bytes(KVZAP_CALL_COMPRESS, B, T, Dh, M, H).
 */
int kvzap_compress(const void* hidden, const void* W1, const void* b1, const void* W2,
                   const void* b2, const void* K, const void* V, float tau, int window,
                   const int32_t* seq_lens, float* scores, int32_t* keep_idx,
                   int32_t* lengths, int64_t* offsets, void* K_out, void* V_out,
                   int64_t cap_rows, int B, int T, int Dh, int M, int H, int D,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_decode_evict -- one decoding step of one layer for B sequences
 * (caption of Algorithm 1; Sec. 2 "delayed eviction with a sliding window";
 * Sec. 3.3: the surrogate needs only the hidden state, so it runs at decode).
 *
 * For sequence b at position p = seq_pos[b], for every head h:
 *   1. s = surrogate(hidden_new[b])[h]                   (as kvzap_score)
 *   2. q = p - window is the position leaving the window.  If q >= 0, its
 *      score is score_ring[b,h,q mod window]; if that score >= tau the pair is
 *      appended to the head's kept prefix, otherwise it is dropped.
 *   3. the new pair and s are stored in ring slot p mod window.
 * Then seq_pos[b] = p + 1.  After the step, prefix + ring hold exactly the
 * positions Algorithm 1 keeps on the first p+1 tokens.
 *
 * Cache layout (device memory, caller-owned, updated in place):
 *   K_prefix, V_prefix  bf16 [total_rows, D]: head (b,h) owns the slab of rows
 *                 slab_offsets[b*H+h] .. + slab_capacity[b*H+h]; its first
 *                 lengths[b,h] rows are the kept pairs older than the window,
 *                 in ascending position order (append-only)
 *   prefix_pos    int32 [total_rows]: position of every prefix row
 *   K_ring, V_ring  bf16 [B, H, window, D]: the pairs inside the window, the
 *                 pair of position t in slot t mod window
 *   score_ring    fp32 [B, H, window]: their scores
 *   lengths       int32 [B, H], seq_pos int32 [B]
 * With window == 0 the ring pointers may be NULL: the new token itself is
 * tested and goes to the prefix or nowhere.
 *
 *   hidden_new    bf16 [B, Dh];  k_new, v_new  bf16 [B, H, D]
 *   W1, b1, W2, b2, Dh, M       as in kvzap_score
 *   error_flag    int32 [1], may be NULL: set to 1 on the device if a kept pair
 *                 found its slab full (the pair is then not appended and the
 *                 head's length stays at capacity); never cleared by the library
 *
 * Calls on the same state must be ordered on one stream.
 */
int kvzap_decode_evict(const void* hidden_new, const void* W1, const void* b1,
                       const void* W2, const void* b2, int Dh, int M,
                       const void* k_new, const void* v_new,
                       void* K_prefix, void* V_prefix, int32_t* prefix_pos,
                       const int64_t* slab_offsets, const int32_t* slab_capacity,
                       void* K_ring, void* V_ring, float* score_ring,
                       int32_t* lengths, int32_t* seq_pos,
                       float tau, int window, int B, int H, int D,
                       int32_t* error_flag,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_attend_decode -- one decoding step of attention over the ragged cache the
 * prune step produces (Sec. 5: the non-uniform per-head lengths need an attention
 * kernel that handles them; the weights are the a_ji of Sec. 3.2, Eq. 2).
 *
 * For sequence b and query head g (grouped-query attention, KV head h = g / (HQ/H)):
 *   out[b,g,:] = sum_i softmax_i( scale * q[b,g,:] . K_i ) * V_i
 * over the rows i of head (b,h): its lengths[b,h] packed rows followed, when
 * window > 0, by the min(seq_pos[b], window) pairs still inside the window ring.
 * The two parts are exactly the state kvzap_decode_evict maintains (call it first,
 * then attend: seq_pos counts the new token, which sits in the ring).  A prefill
 * result of kvzap_compact is attended to with window = 0, row_offsets = offsets,
 * lengths = lengths (its window tokens are among the packed rows).
 *
 *   q            bf16 [B, HQ, D]
 *   K_rows, V_rows  bf16 [total_rows, D]; head (b,h) owns rows
 *                row_offsets[b*H+h] .. + lengths[b,h].  The kernel never reads
 *                outside [0, total_rows): a head whose offset is out of range is
 *                treated as empty and a length is cut at total_rows.
 *   row_offsets  int64 [B*H];  lengths int32 [B, H]
 *   K_ring, V_ring  bf16 [B, H, window, D], seq_pos int32 [B]; all three NULL iff window == 0
 *   max_rows     host-side upper bound on lengths[b,h] (e.g. the slab capacity or the
 *                prompt length).  It only sizes the launch and the workspace; a head
 *                longer than the bound is still attended to in full, only slower.
 *   scale        usually 1/sqrt(D)
 *   out          bf16 [B, HQ, D], fully overwritten.  A head with no row yields zeros.
 *   workspace    kvzap_workspace_bytes(KVZAP_CALL_ATTEND_DECODE, B, T = max_rows,
 *                Dh = HQ, M = window, H)
 *
 * Supported: D = 128, HQ a multiple of H with HQ/H <= 16.  Arithmetic: bf16 products
 * accumulated in fp32 on the matrix cores; the softmax weights enter the second
 * product rounded to bf16 and the denominator sums those rounded weights, so the
 * output is a convex combination of the V rows up to fp32 rounding, then rounded to
 * bf16.  Fixed combination order (run-to-run deterministic); the result does not
 * depend on the order of the rows beyond rounding.
 */
int kvzap_attend_decode(const void* q, const void* K_rows, const void* V_rows,
                        int64_t total_rows, const int64_t* row_offsets,
                        const int32_t* lengths, const void* K_ring, const void* V_ring,
                        const int32_t* seq_pos, int window, int max_rows, float scale,
                        void* out, int B, int H, int HQ, int D,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Paged layout of the ragged cache (Sec. 1, third criterion: a pruning method has to work
 * with paged attention; Sec. 5: per-head lengths need pages per head).  The kept rows of
 * head (b,h) live in pages of page_rows rows taken from one pool:
 *
 *   K_pool, V_pool  bf16 [num_pages, page_rows, D]
 *   block_table     int32 [B*H, max_pages]: row j of head (b,h) is row j % page_rows of
 *                   page block_table[b*H+h][j / page_rows]; unused entries are -1
 *   page_rows       a power of two >= 16
 *
 * kvzap_assign_pages -- fills the block table from the lengths kvzap_mask produced: head
 * (b,h), in (b,h) order, takes the next ceil((lengths[b,h] + reserve_rows) / page_rows)
 * entries of free_pages (first fit in list order; reserve_rows leaves room for tokens
 * appended later).  result (device int32 [2]): [0] = entries of free_pages consumed,
 * [1] = 0 on success, 1 if the free list is too short, 2 if a head needs more than
 * max_pages; on failure every table entry is -1 and nothing is consumed.  The library
 * never reads the pool here and keeps no allocator state: the caller removes the first
 * result[0] entries from its free list.
 *   lengths int32 [B,H]; free_pages int32 [n_free] (4-byte alignment is enough, so the
 *   unconsumed tail of a list can be passed on); block_table fully overwritten.
 *   workspace: kvzap_workspace_bytes(KVZAP_CALL_ASSIGN_PAGES, B, 1, 0, 0, H).
 */
int kvzap_assign_pages(const int32_t* lengths, int B, int H, int page_rows, int reserve_rows,
                       const int32_t* free_pages, int n_free, int32_t* block_table,
                       int max_pages, int32_t* result,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_extend_pages -- the same assignment for a cache that grows (decoding): head (b,h)
 * already owns the first page_counts[b,h] entries of its table row and is brought up to
 * ceil((lengths[b,h] + reserve_rows) / page_rows) pages by appending the next entries of
 * free_pages behind them (heads in (b,h) order); page_counts (int32 [B,H], in/out) is
 * updated, every other table entry is left as it is.  result and failure as above (on
 * failure nothing changes).  With reserve_rows >= the number of tokens decoded until the
 * next call, kvzap_decode_evict_paged always finds room.  Same workspace as
 * kvzap_assign_pages.
 */
int kvzap_extend_pages(const int32_t* lengths, int32_t* page_counts, int B, int H,
                       int page_rows, int reserve_rows, const int32_t* free_pages, int n_free,
                       int32_t* block_table, int max_pages, int32_t* result,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_compact_paged -- the gather of kvzap_compact written through a block table
 * (Algorithm 1, last line, into the layout above).  keep_idx, lengths and offsets are
 * kvzap_mask's outputs (offsets only locates each head's slice of keep_idx).  A kept row
 * whose page slot is beyond max_pages or whose table entry is not in [0, num_pages) is
 * skipped; rows of a page beyond the head's length are left untouched.  K, V must not
 * overlap the pools.  D in {64, 128, 256}.
 */
int kvzap_compact_paged(const void* K, const void* V, const int32_t* keep_idx,
                        const int32_t* lengths, const int64_t* offsets,
                        const int32_t* block_table, int max_pages, int page_rows,
                        void* K_pool, void* V_pool, int num_pages,
                        int B, int H, int T, int D, void* stream);

/*
 * kvzap_attend_decode_paged -- kvzap_attend_decode over the paged layout: the packed rows
 * of head (b,h) are its first lengths[b,h] rows in block-table order, the window ring is
 * as before.  A table entry outside [0, num_pages) is clamped into the pool (the call never
 * reads outside it; the result for that head is then meaningless), lengths are cut at
 * max_pages * page_rows.  Same arithmetic, workspace and limits as kvzap_attend_decode.
 */
int kvzap_attend_decode_paged(const void* q, const void* K_pool, const void* V_pool,
                              int num_pages, const int32_t* block_table, int max_pages,
                              int page_rows, const int32_t* lengths, const void* K_ring,
                              const void* V_ring, const int32_t* seq_pos, int window,
                              int max_rows, float scale, void* out, int B, int H, int HQ,
                              int D, void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_decode_evict_paged -- kvzap_decode_evict with the kept prefix in pages (caption of
 * Algorithm 1; layout above).  Row j of head (b,h)'s prefix is row j % page_rows of page
 * block_table[b*H+h][j / page_rows] in K_pool / V_pool, its position in the same place of
 *   pos_pool  int32 [num_pages, page_rows].
 * A kept pair is appended at row lengths[b,h]; if that table slot is beyond max_pages or
 * does not hold a page of the pool, error_flag is set, the pair is not appended and the
 * length stays (as a full slab does in kvzap_decode_evict).  Ring, scores, lengths, seq_pos,
 * workspace and every other argument as in kvzap_decode_evict.
 */
int kvzap_decode_evict_paged(const void* hidden_new, const void* W1, const void* b1,
                             const void* W2, const void* b2, int Dh, int M,
                             const void* k_new, const void* v_new,
                             void* K_pool, void* V_pool, int32_t* pos_pool, int num_pages,
                             const int32_t* block_table, int max_pages, int page_rows,
                             void* K_ring, void* V_ring, float* score_ring,
                             int32_t* lengths, int32_t* seq_pos,
                             float tau, int window, int B, int H, int D,
                             int32_t* error_flag,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvzap_teacher_scores -- the scores the surrogate is trained on, for one layer of one
 * extended prompt "prompt, instruction, repeated prompt" (Sec. 3.1 Eq. 1: KVzip; Sec. 3.2
 * Eq. 3: KVzip+), in log space (Sec. 3.3: the surrogate regresses log s+).
 *
 *   q      bf16 [HQ, Tq, D]  queries of the Tq positions of the repeated prompt, which sit
 *                            at positions P0 .. P0+Tq-1 of the extended prompt, P0 = Tk - Tq
 *   k      bf16 [H, Tk, D]   keys of all Tk positions
 *   vnorm  fp32 [H, T] or NULL (= 1): ||W_O v_i|| for the T <= P0 prompt positions
 *   hnorm  fp32 [Tq]   or NULL (= 1): ||h_j||
 *   log_s  fp32 [H, T]: log max_{j, g in group(h)} a_ji * vnorm[h,i] / hnorm[j], where a is
 *          the causal softmax of scale * q_gj . k_i' over the keys i' <= P0 + j and the
 *          group of KV head h is its HQ/H query heads.  NULL norms give Eq. 1.
 * Supported: D = 128, HQ a multiple of H, scale > 0.  bf16 products accumulated in fp32 on the
 * matrix cores, softmax statistics in fp32; the maximum is taken on the logits, so no weight
 * underflows.  Deterministic.  workspace:
 * kvzap_workspace_bytes(KVZAP_CALL_TEACHER_SCORES, 1, T, Dh = HQ, M = Tq, H).
 */
int kvzap_teacher_scores(const void* q, const void* k, const float* vnorm, const float* hnorm,
                         float scale, float* log_s, int H, int HQ, int Tq, int Tk, int T,
                         int D, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVZAP_H_ */
