/*
 * dd.h -- C ABI of the DualDiffusion draft-then-verify hot path on MI355X (gfx950).
 *
 * One draft-then-verify cycle (Alg. 1) is K drafter unmasking steps followed by one
 * verifier pass and a verification rule.  This library provides the three operations
 * that dominate it:
 *
 *   dd_bidir_attention         the verifier's attention over ALL positions -- the
 *                              O(N^2)-per-step cost Sec. 1 and Sec. 2.2 name as the
 *                              bottleneck of masked diffusion models;
 *   dd_block_attention_cached  the drafter's attention: only the active block's
 *                              queries, keys/values of the other positions read from
 *                              a block-wise approximate KV cache (Sec. 2.3, Sec. 3.1);
 *   dd_verify_remask           the verification rule of Sec. 3.2 over the vocabulary:
 *                              verifier confidence (Eq. 7) and argmax, KL(drafter ||
 *                              verifier) (Eq. 5), and the Trust (Eq. 4) / KL-threshold /
 *                              KL-probabilistic (Eq. 6) / confidence-threshold /
 *                              confidence-probabilistic remask decision.
 *
 * Common rules
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates, frees or synchronises.  Work is enqueued on `stream` (a hipStream_t
 *     passed as void*; NULL = the default stream).  Inputs are never written; outputs
 *     are fully overwritten; identical inputs give bit-identical outputs.
 *   - `workspace` is device memory of at least dd_*_workspace_bytes(...) bytes (same
 *     shape arguments), 256-byte aligned, contents undefined on entry and exit.  It may
 *     be NULL when the query function returns 0.  Calls that share a workspace must be
 *     ordered on one stream.
 *   - All tensors are dense, row-major, contiguous, base pointers 16-byte aligned.
 *   - Return value: DD_OK, or a negative dd_status.  Arguments are validated on the
 *     host before any GPU call; on error nothing is launched and no output is touched.
 */
#ifndef DD_H
#define DD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DD_OK = 0,
    DD_ERR_NULL = -1,       /* a required pointer is NULL */
    DD_ERR_SHAPE = -2,      /* a size is out of range or inconsistent */
    DD_ERR_DTYPE = -3,      /* unsupported element type / combination */
    DD_ERR_MODE = -4,       /* unknown remask mode */
    DD_ERR_WORKSPACE = -5,  /* workspace NULL / too small / misaligned */
    DD_ERR_ALIGN = -6,      /* a pointer or row pitch is not 16-byte aligned */
    DD_ERR_LAUNCH = -7,     /* the HIP runtime refused a launch */
    DD_STATUS_INT_RANGE_LO = -0x7fffffff - 1, DD_STATUS_INT_RANGE_HI = 0x7fffffff
} dd_status;

/* (The *_INT_RANGE_* enumerators of the enumerations in this header only give them the value range of int, so that
 * an integer a C caller passes for them - valid or not - is a value the library may legally inspect and refuse.) */

typedef enum {
    DD_F32 = 0,        /* IEEE binary32 */
    DD_BF16 = 1,       /* upper 16 bits of binary32 */
    DD_FP8_E4M3 = 2,   /* OCP e4m3 (bias 7, max 448, no infinities); Q and K only */
    DD_DTYPE_INT_RANGE_LO = -0x7fffffff - 1, DD_DTYPE_INT_RANGE_HI = 0x7fffffff
} dd_dtype;

typedef enum {
    DD_TRUST = 0,        /* Eq. 4: keep the drafter's sequence, remask nothing */
    DD_KL_THRESH = 1,    /* remask i iff KL_i > threshold                      (Sec. 3.2.2) */
    DD_CONF_THRESH = 2,  /* remask i iff c_V,i < threshold                     (Sec. 3.2.3) */
    DD_KL_PROB = 3,      /* remask i with probability KL_i / sum_j KL_j (Eq. 6) */
    DD_CONF_PROB = 4,    /* remask i with probability 1 - c_V,i                (Sec. 3.2.3) */
    /* Budgeted forms of the two rules above (not rules of the paper, which only thresholds or draws):
     * per sequence, the k = floor(threshold) worst eligible positions are remasked. */
    DD_KL_TOPK = 5,      /* the k eligible positions with the largest KL_i   */
    DD_CONF_TOPK = 6,    /* the k eligible positions with the smallest c_V,i */
    DD_MODE_INT_RANGE_LO = -0x7fffffff - 1, DD_MODE_INT_RANGE_HI = 0x7fffffff
} dd_mode;

/* Human-readable text for a dd_status (static storage; never NULL). */
const char *dd_strerror(int status);

/* Library version as major * 10000 + minor * 100 + patch. */
int dd_version(void);

/*
 * Verifier attention (Sec. 2.2; Alg. 1, verification phase):
 *     O[b,h,i,:] = sum_j softmax_j( Q[b,h,i,:] . K[b,g,j,:] / sqrt(d) ) V[b,g,j,:],   j = 0..N-1
 * i.e. the softmax(Q K^T / sqrt(d_k)) V of Eq. 3 with the key range being every position
 * (bidirectional: no causal or padding mask).  Query head h reads kv head g = h*Hkv/H
 * (consecutive groups; Hkv == H is plain multi-head attention).
 *
 *   Q  [B,H,N,d]    qk_dtype          K [B,Hkv,N,d]  qk_dtype
 *   V  [B,Hkv,N,d]  v_dtype           O [B,H,N,d]    v_dtype   (written)
 *   q_scale [B*H], k_scale [B*Hkv]  fp32 per-(batch,head) multipliers of the decoded
 *       values (must be > 0); required for DD_FP8_E4M3, optional (NULL = 1) otherwise.
 * Supported: (qk_dtype, v_dtype) in {(F32,F32), (BF16,BF16), (FP8_E4M3,BF16)};
 *            d in {64, 128}; H % Hkv == 0; B, H, N >= 1; B*H*N*d < 2^40.
 * Arithmetic: F32 path in fp32 throughout; BF16/FP8 paths multiply on the matrix cores
 *            with fp32 accumulation, fp32 online softmax, probabilities rounded to bf16
 *            before the PV product.
 * Workspace: none needed (dd_bidir_attention_workspace_bytes returns 0).
 */
int dd_bidir_attention(const void *Q, const void *K, const void *V, void *O,
                       int B, int H, int Hkv, int N, int d,
                       dd_dtype qk_dtype, dd_dtype v_dtype,
                       const float *q_scale, const float *k_scale,
                       void *workspace, size_t workspace_bytes, void *stream);
size_t dd_bidir_attention_workspace_bytes(int B, int H, int Hkv, int N, int d,
                                          dd_dtype qk_dtype, dd_dtype v_dtype);

/*
 * Drafter attention over a block-wise approximate KV cache (Sec. 2.3: keys/values of the
 * other blocks are cached and reused across the denoising steps inside a block; prefix
 * and suffix are both cached).  Same formula as above, but only for the block_len queries
 * of the active block; key/value row j is
 *     Kblk/Vblk[b,g,j-block_start,:]  if Kblk != NULL and block_start <= j < block_start+block_len
 *     Kc/Vc[b,g,j,:]                  otherwise (whatever the cache holds, stale or not).
 * With Kblk == Vblk == NULL the caller has already refreshed the block's rows in the cache.
 *
 *   Qblk [B,H,block_len,d] qk_dtype     Kc [B,Hkv,N,d] qk_dtype    Vc [B,Hkv,N,d] v_dtype
 *   Kblk [B,Hkv,block_len,d] qk_dtype   Vblk [B,Hkv,block_len,d] v_dtype  (both or neither)
 *   O    [B,H,block_len,d] v_dtype  (written)
 *   k_scale applies to cache rows and block rows alike.
 * Requires 0 <= block_start, 1 <= block_len, block_start + block_len <= N;
 *          dtypes / d / heads as for dd_bidir_attention.
 * The key range is split over several workgroups whose partial (max, sum, unnormalised
 * output) states live in `workspace` and are merged by a second kernel.
 */
int dd_block_attention_cached(const void *Qblk, const void *Kc, const void *Vc, void *O,
                              int block_start, int block_len,
                              const void *Kblk, const void *Vblk,
                              int B, int H, int Hkv, int N, int d,
                              dd_dtype qk_dtype, dd_dtype v_dtype,
                              const float *q_scale, const float *k_scale,
                              void *workspace, size_t workspace_bytes, void *stream);
size_t dd_block_attention_cached_workspace_bytes(int block_len, int B, int H, int Hkv, int N, int d,
                                                 dd_dtype qk_dtype, dd_dtype v_dtype);

/*
 * Second precision workload: the two attention calls with V stored like K - OCP e4m3 codes with one fp32 scale per
 * (batch, kv head), real value = scale x decoded code - which halves the bytes of V in memory, the quantity the
 * drafter's call is bound by.  (The paper fixes no storage precision; Sec. 4.1 runs stock models.)  Same formulas
 * as dd_bidir_attention / dd_block_attention_cached:
 *   Q, K, V (and Qblk, Kc, Vc, Kblk, Vblk): DD_FP8_E4M3;   O: DD_BF16;   q_scale [B*H], k_scale, v_scale [B*Hkv]:
 *   all required; the block's fresh rows Kblk / Vblk use the cache's k_scale / v_scale.
 * Arithmetic: the scores are products of the e4m3 codes of Q and K as stored (fp8 matrix cores, fp32 accumulation;
 * the per-head scales multiply the exponent); V's codes are decoded exactly (e4m3 -> bf16) on their way into LDS and
 * O = P V runs on the bf16 matrix cores with fp32 accumulation, the weights P rounded to bf16; v_scale multiplies
 * the output once.
 * dd_bidir_attention_fp8v needs no workspace; the block call's comes from its own query function.
 * Shapes, alignment and errors as for the calls above (a missing scale: DD_ERR_NULL).
 */
int dd_bidir_attention_fp8v(const void *Q, const void *K, const void *V, void *O,
                            int B, int H, int Hkv, int N, int d,
                            const float *q_scale, const float *k_scale, const float *v_scale, void *stream);
int dd_block_attention_cached_fp8v(const void *Qblk, const void *Kc, const void *Vc, void *O,
                                   int block_start, int block_len,
                                   const void *Kblk, const void *Vblk,
                                   int B, int H, int Hkv, int N, int d,
                                   const float *q_scale, const float *k_scale, const float *v_scale,
                                   void *workspace, size_t workspace_bytes, void *stream);
size_t dd_block_attention_cached_fp8v_workspace_bytes(int block_len, int B, int H, int Hkv, int N, int d);

/*
 * Third precision workload: the verifier's attention on block-scaled ("MX") inputs, the storage of the OCP
 * Microscaling Formats specification v1.0: every 32 consecutive elements of the head dimension share one
 * power-of-two scale, an E8M0 code (real scale 2^(code - 127)); real value = scale x decoded element.  (The paper
 * fixes no storage precision; Sec. 4.1 runs stock models.)  Same formula as dd_bidir_attention (Eq. 3 over all
 * positions, Sec. 2.2):
 *   Q [B,H,N,d], K [B,Hkv,N,d]: e4m3 codes, one byte per element;       Qs [B,H,N,d/32], Ks [B,Hkv,N,d/32]: E8M0
 *   V [B,Hkv,N,d/2]: e2m1 codes (sign, 2 exponent bits with bias 1, 1 mantissa bit: +-{0, 0.5, 1, 1.5, 2, 3, 4, 6}),
 *      two per byte, the element with the even index in the low four bits;   Vs [B,Hkv,N,d/32]: E8M0
 *   O [B,H,N,d]: DD_BF16.   All device pointers, dense, row-major; Q, K, V, O 16-byte aligned, the scale arrays
 *   4-byte aligned.
 * Arithmetic: S = Q K^T runs on the block-scaled matrix instruction (e4m3 operands, both operands' E8M0 scales applied
 * by the hardware, fp32 accumulation); V is decoded, multiplied by its block's scale and held as bf16 on its way into
 * LDS - exact whenever the scaled value is a normal bf16 number or zero, which holds for every scale code in
 * [27, 230] - and O = P V runs on the bf16 matrix cores with the weights rounded to bf16.  Scale codes outside that
 * range and the NaN codes of e4m3 and E8M0 give unspecified results.  No workspace; work is enqueued on `stream`.
 * Errors: DD_ERR_NULL (a missing pointer), DD_ERR_SHAPE (as dd_bidir_attention; d is 64 or 128), DD_ERR_ALIGN,
 * DD_ERR_LAUNCH.
 */
int dd_bidir_attention_mx(const void *Q, const void *Qs, const void *K, const void *Ks, const void *V, const void *Vs,
                          void *O, int B, int H, int Hkv, int N, int d, void *stream);

/*
 * The same call when the block is complete (Sec. 2.3: cached activations are reused across the denoising
 * steps of a block and refreshed at block granularity): the attention exactly as
 * dd_block_attention_cached computes it with Kblk/Vblk given, and in the same call
 *     Kc[b,g,block_start+r,:] <- Kblk[b,g,r,:],   Vc[b,g,block_start+r,:] <- Vblk[b,g,r,:]      0 <= r < block_len
 * (a copy of the stored bytes: with DD_FP8_E4M3 the block's K already uses the cache's k_scale).  Afterwards a
 * call with Kblk == NULL on the same cache returns the same O.  Every other cache row is left untouched.
 * Kblk and Vblk are required and must not overlap Kc / Vc; block_len <= 2^25; everything else (shapes, dtypes, workspace, errors)
 * as for dd_block_attention_cached.  The copy rides on the kernel that merges the key splits (extra workgroups
 * of the same launch), or is one small launch of its own when the key range was not split: no workgroup of the
 * call reads the cache rows it writes.
 */
int dd_block_attention_refresh(const void *Qblk, void *Kc, void *Vc, void *O,
                               int block_start, int block_len,
                               const void *Kblk, const void *Vblk,
                               int B, int H, int Hkv, int N, int d,
                               dd_dtype qk_dtype, dd_dtype v_dtype,
                               const float *q_scale, const float *k_scale,
                               void *workspace, size_t workspace_bytes, void *stream);
size_t dd_block_attention_refresh_workspace_bytes(int block_len, int B, int H, int Hkv, int N, int d,
                                                  dd_dtype qk_dtype, dd_dtype v_dtype);

/*
 * Drafter attention over a local window of the cache (Sec. 2.3 cites dKV-Cache, whose greedy variant restricts
 * the cached context to the positions around the tokens being decoded): as dd_block_attention_cached, but the
 * softmax of Eq. 3 runs over the key rows win_start <= j < win_start + win_len only; every other row of the
 * cache is neither read nor weighted.  The window must contain the block:
 *     0 <= win_start <= block_start,  block_start + block_len <= win_start + win_len <= N.
 * With win_start = 0 and win_len = N the result is that of dd_block_attention_cached (same kernels, same order
 * of operations).  Kc, Vc are the whole cache [B,Hkv,N,d]; the call costs what a cache of win_len rows costs.
 * Workspace from dd_block_attention_window_workspace_bytes; everything else as for dd_block_attention_cached.
 */
int dd_block_attention_window(const void *Qblk, const void *Kc, const void *Vc, void *O,
                              int block_start, int block_len, int win_start, int win_len,
                              const void *Kblk, const void *Vblk,
                              int B, int H, int Hkv, int N, int d,
                              dd_dtype qk_dtype, dd_dtype v_dtype,
                              const float *q_scale, const float *k_scale,
                              void *workspace, size_t workspace_bytes, void *stream);
size_t dd_block_attention_window_workspace_bytes(int block_len, int win_len, int B, int H, int Hkv, int N, int d,
                                                 dd_dtype qk_dtype, dd_dtype v_dtype);

/*
 * Drafter attention for a batch whose sequences stand at different blocks (sequences of a serving batch finish
 * their blocks at different times; Alg. 1 runs per sequence): as dd_block_attention_cached with Kblk/Vblk, but the
 * active block of batch entry b begins at block_starts[b]:
 *     key/value row j of batch b = Kblk/Vblk[b,g,j-block_starts[b],:]  if 0 <= j - block_starts[b] < block_len
 *                                  Kc/Vc[b,g,j,:]                       otherwise.
 *   block_starts [B] i32, DEVICE memory.  The positions are not validated (they live on the device): rows of a
 *   block that would fall outside [0, N) simply replace nothing; no access leaves the tensors for any value.
 *   Kblk and Vblk are required (without them the block position plays no role: use dd_block_attention_cached).
 * Everything else as for dd_block_attention_cached; workspace from dd_block_attention_batched_workspace_bytes.
 */
int dd_block_attention_batched(const void *Qblk, const void *Kc, const void *Vc, void *O,
                               const int32_t *block_starts, int block_len,
                               const void *Kblk, const void *Vblk,
                               int B, int H, int Hkv, int N, int d,
                               dd_dtype qk_dtype, dd_dtype v_dtype,
                               const float *q_scale, const float *k_scale,
                               void *workspace, size_t workspace_bytes, void *stream);
size_t dd_block_attention_batched_workspace_bytes(int block_len, int B, int H, int Hkv, int N, int d,
                                                  dd_dtype qk_dtype, dd_dtype v_dtype);

/*
 * Token-granular cache update.  The cached drafters of Sec. 2.3 differ in when a position's key/value enter
 * the cache (block-wise schemes: when the block is complete; dKV-Cache: one step after the token was decoded);
 * the operation on the cache is the same: rows the drafter computed replace the cache rows of chosen positions:
 *     for b < B, g < Hkv, r < n, with p = positions[b*n + r]:   if 0 <= p < N:
 *         Kc[b,g,p,:] <- Krows[b,g,r,:],   Vc[b,g,p,:] <- Vrows[b,g,r,:]            (stored bytes are copied)
 *
 *   Kc [B,Hkv,N,d] qk_dtype, Vc [B,Hkv,N,d] v_dtype     the cache (modified in place)
 *   Krows [B,Hkv,n,d] qk_dtype, Vrows [B,Hkv,n,d] v_dtype
 *   positions [B*n] i32, DEVICE memory: one list per batch entry, shared by its kv heads; an entry outside
 *       [0, N) (e.g. -1) skips its row; the positions of one batch entry must be distinct (else which row wins
 *       is unspecified)
 * dtypes / d as for dd_bidir_attention (H plays no role); n == 0 is a no-op.  Krows/Vrows must not overlap the cache.
 */
int dd_cache_insert_rows(void *Kc, void *Vc, const void *Krows, const void *Vrows, const int32_t *positions, int n,
                         int B, int Hkv, int N, int d, dd_dtype qk_dtype, dd_dtype v_dtype, void *stream);

/*
 * Verification rule of Sec. 3.2 for P = B*G positions (G verified positions per sequence),
 * softmax at temperature 1 over the whole vocabulary, natural logarithm:
 *     c_V,i  = max_x p_V(x | i)                     (Eq. 7)      t_V,i = lowest x attaining it
 *     KL_i   = sum_x p_D(x|i) (log p_D(x|i) - log p_V(x|i))      (Eq. 5)
 *     score_i = KL_i in the KL modes, c_V,i otherwise
 *     eligible_i = (mask[i] == 0)      -- the rules are stated for decoded positions only
 *     remask_i = eligible_i and
 *         DD_TRUST        false
 *         DD_KL_THRESH    score_i >  threshold       (strict; compared in fp32)
 *         DD_CONF_THRESH  score_i <  threshold       (strict; compared in fp32)
 *         DD_KL_PROB      u_i < max(score_i,0) / sum_{j eligible, same sequence} max(score_j,0)
 *                         (an empty or zero sum remasks nothing)
 *         DD_CONF_PROB    u_i < 1 - score_i
 *         DD_KL_TOPK      fewer than k eligible positions j of the same sequence are worse than i, where
 *         DD_CONF_TOPK    j is worse than i iff its score is larger (KL) / smaller (confidence), or equal
 *                         with j < i; k = floor(threshold), threshold >= 0 and finite (else DD_ERR_SHAPE);
 *                         scores compared in fp32; a sequence with at most k eligible positions
 *                         remasks all of them
 *     u_i = top 24 bits of word 0 of Philox-4x32-10(counter = (i_lo, i_hi, 0, 0),
 *           key = (seed_lo, seed_hi)) times 2^-24, i = global row index b*G+g.
 *
 *   logits_d [P,V] logit_dtype  drafter logits; read only in the KL modes (may be NULL otherwise)
 *   logits_v [P,V] logit_dtype  verifier logits
 *   mask     [P] u8             1 = position still holds [MASK], 0 = decoded
 *   out_mask   [P] u8   = mask[i] | remask_i.  out_mask == mask (update in place) is allowed in DD_TRUST, the
 *                         two threshold modes and DD_CONF_PROB, whose decision for row i reads mask[i] only; in
 *                         DD_KL_PROB and the budgeted modes, which read the whole sequence's mask, and for ranges
 *                         that overlap without being identical, the call returns DD_ERR_SHAPE
 *   out_tokens [P] i32  = t_V,i            (every row, eligible or not, every mode)
 *   out_scores [P] f32  = score_i          (every row)
 * logit_dtype in {DD_F32, DD_BF16}; V >= 1 with V * sizeof(element) a multiple of 16;
 * B, G >= 0 (P == 0 is a no-op returning DD_OK); V < 2^31, P < 2^31.
 * `seed` is ignored by DD_TRUST, the threshold modes and the budgeted modes.
 * Each logit is read from memory exactly once (single pass; rows are split across
 * workgroups and their partial states merged in `workspace`).
 */
int dd_verify_remask(const void *logits_d, const void *logits_v, const uint8_t *mask,
                     dd_mode mode, float threshold, uint64_t seed,
                     uint8_t *out_mask, int32_t *out_tokens, float *out_scores,
                     int B, int G, int V, dd_dtype logit_dtype,
                     void *workspace, size_t workspace_bytes, void *stream);
size_t dd_verify_remask_workspace_bytes(int B, int G, int V, dd_dtype logit_dtype);

/*
 * dd_verify_remask for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without the workspace pair),
 * same kernels, same results bit for bit.  The partial states of a split row live in a file-scope device array
 * inside the library instead: 128 KiB per GPU, held from the time the library's code is loaded on that GPU until
 * the process ends.  The call allocates and frees nothing.
 *   - Limit: dd_verify_remask_workspace_bytes(B, G, V, logit_dtype) <= 131072, else DD_ERR_WORKSPACE and nothing
 *     is launched.  (Today's kernels need at most 191 rows x 16 splits x 32 bytes = 97792 bytes, and none from
 *     192 rows on, so every valid shape fits.)
 *   - The array is looked up once per GPU, at the first call that needs it while that GPU is current (a symbol
 *     look-up, DD_ERR_LAUNCH if it fails): make that first call outside graph capture.  `stream` must belong to
 *     the current device.
 *   - All calls on one GPU share the one array, which keeps the last call's contents (no call depends on them):
 *     two calls of this entry point that overlap in time on one GPU (different streams) race and give wrong
 *     results; calls on one stream, or ordered by events, are fine.  Calls with 192 rows or more use no scratch.
 */
int dd_verify_remask_static(const void *logits_d, const void *logits_v, const uint8_t *mask,
                            dd_mode mode, float threshold, uint64_t seed,
                            uint8_t *out_mask, int32_t *out_tokens, float *out_scores,
                            int B, int G, int V, dd_dtype logit_dtype, void *stream);

typedef enum {
    DD_UNMASK_THRESH = 0,  /* every masked position whose drafter confidence exceeds the threshold */
    DD_UNMASK_TOPK = 1,    /* a fixed number per step: the k = floor(threshold) most confident masked positions */
    DD_UNMASK_MODE_INT_RANGE_LO = -0x7fffffff - 1, DD_UNMASK_MODE_INT_RANGE_HI = 0x7fffffff
} dd_unmask_mode;

/*
 * One drafter unmasking step, x <- Unmask(p_D, x) (Alg. 1, drafting phase): the model's probabilities at the
 * masked positions decide which of them are revealed (Sec. 2.1: the most confident ones);
 * the two selection rules are the ones Sec. 2.3 names: all tokens above a confidence threshold
 * (confidence-aware parallel decoding) or a fixed number per step.  For P = B*G positions, softmax at
 * temperature 1 over the whole vocabulary:
 *     c_D,i = max_x p_D(x | i),  t_D,i = lowest x attaining it
 *     candidate_i = (mask[i] != 0)                        -- only positions that still hold [MASK]
 *     rank_i = number of candidates j of the same sequence with c_D,j > c_D,i, or equal with j < i
 *     select_i = candidate_i and
 *         DD_UNMASK_THRESH   c_D,i > threshold (strict, fp32)  or  rank_i == 0
 *                            (the most confident candidate is always taken, so that every step reveals
 *                             at least one token per unfinished sequence; the paper leaves this open)
 *         DD_UNMASK_TOPK     rank_i < floor(threshold), threshold >= 0 and finite (else DD_ERR_SHAPE)
 *
 *   logits_d [P,V] logit_dtype  drafter logits
 *   mask     [P] u8             1 = position still holds [MASK], 0 = decoded
 *   x_tokens [P] i32, optional  the sequence's token ids: x_tokens[i] = t_D,i is written where select_i,
 *                               every other entry is left as it is (may be NULL)
 *   out_mask   [P] u8   = mask[i] and not select_i
 *   out_tokens [P] i32  = t_D,i     (every row)
 *   out_conf   [P] f32  = c_D,i     (every row)
 * Same shape rules, workspace and single-pass property as dd_verify_remask; out_mask must not overlap mask
 * (DD_ERR_SHAPE).
 */
int dd_unmask(const void *logits_d, const uint8_t *mask, dd_unmask_mode mode, float threshold,
              int32_t *x_tokens, uint8_t *out_mask, int32_t *out_tokens, float *out_conf,
              int B, int G, int V, dd_dtype logit_dtype,
              void *workspace, size_t workspace_bytes, void *stream);
size_t dd_unmask_workspace_bytes(int B, int G, int V, dd_dtype logit_dtype);

/*
 * Every per-position quantity the verification rules of Sec. 3.2 draw on, from one pass over the two logit
 * matrices and with no rule applied: what a caller needs to evaluate several rules A (or the rule ablation of
 * Sec. 4) on the same verifier output without reading the logits once per rule.  For P positions, softmax at
 * temperature 1 over the whole vocabulary:
 *     out_kl[i]     = KL(p_D(.|i) || p_V(.|i))                        (Eq. 5, natural log)
 *     out_conf_v[i] = max_x p_V(x | i),  out_tok_v[i] = lowest x attaining it      (Eq. 7; the token Alg. 1 keeps)
 *     out_conf_d[i] = max_x p_D(x | i),  out_tok_d[i] = lowest x attaining it      (the drafter's proposal)
 *
 *   logits_d, logits_v [P,V] logit_dtype (DD_F32 or DD_BF16), rows dense, V * element size a multiple of 16
 *   out_kl, out_conf_v [P] f32, out_tok_v [P] i32: required;  out_conf_d [P] f32, out_tok_d [P] i32: each may be NULL
 * Workspace, alignment, stream and error behaviour as for dd_verify_remask (P rows, no sequence structure);
 * P == 0 is a no-op.  The numbers are the ones dd_verify_remask reports as out_scores/out_tokens in its KL and
 * confidence modes: the same kernels produce them.
 */
int dd_verify_scores(const void *logits_d, const void *logits_v,
                     float *out_kl, float *out_conf_v, int32_t *out_tok_v, float *out_conf_d, int32_t *out_tok_d,
                     int P, int V, dd_dtype logit_dtype, void *workspace, size_t workspace_bytes, void *stream);
size_t dd_verify_scores_workspace_bytes(int P, int V, dd_dtype logit_dtype);

#ifdef __cplusplus
}
#endif
#endif /* DD_H */
