/*
 * libmulo -- the parallel verification step of Multi-Scale Local Speculative
 * Decoding (MuLo-SD) for autoregressive image generation, for one AMD MI355X
 * (gfx950).  Plain C ABI: no C++ or torch types cross this boundary.
 *
 * One verification step (supplementary Alg. 1, Steps 2-5, with the rejected
 * neighbourhoods re-drawn in one shot):
 *   Step 2  up-sample the low-resolution draft onto the target grid   (Sec. 3.2)
 *   Step 3  one pass of the target decoder over the drafted block against the
 *           KV cache of the prefix                                   (Sec. 3.2)
 *   Step 4  speculative accept test  min(1, p/q)  per position   (Sec. 3.1, Eq. 1;
 *           pooled numerator of Eq. 3 when a neighbour table is given)
 *   Step 5  local expansion: mark the radius-l neighbourhood of every rejected
 *           position, nothing before the first rejection, no raster-order cut
 *                                                              (Sec. 3.3, Eq. 6-7)
 *   then    residual resampling  norm(max(0, p - q))  of the marked positions
 *                                                              (Sec. 3.1, Eq. 2)
 *
 * Conventions that hold for every entry point
 *   - "device pointer" = memory on the GPU the context was created on, owned by
 *     the caller, at least 16-byte aligned, valid until the stream work of the
 *     call has finished.  "host pointer" = ordinary process memory, read during
 *     the call only.
 *   - All work is enqueued on the HIP stream given to mulo_create; nothing
 *     synchronises with the host.  Outputs are valid once the caller has
 *     synchronised that stream.  A context is not thread-safe.
 *   - The compute entry points enqueue kernels only (no allocation, no memset
 *     or copy node, no host synchronisation after mulo_create), so a call may be
 *     recorded into a HIP graph by stream capture on that stream and replayed,
 *     once an ordinary call of the same entry point has run (the first launch of
 *     a kernel configures it).  Host structs are read at record time: a replay
 *     repeats the recorded seed and rng_counter.  Profiling (mulo_profile)
 *     must be off while recording.
 *   - Every argument is checked before anything is launched; on an error
 *     nothing has been written.  No entry point prints, throws or aborts.
 *   - Token grids are raster order: position u of an H x W grid sits at row
 *     u / W, column u % W.  A draft block is L consecutive positions starting at
 *     n0, both whole multiples of W (the drafter proposes whole rows, Sec. 3.2).
 */
#ifndef MULO_H
#define MULO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MULO_API __attribute__((visibility("default")))

typedef struct mulo_ctx mulo_ctx; /* opaque, owned by the library */

typedef enum {
    MULO_OK = 0,
    MULO_ERR_NULL = 1,        /* a required pointer is NULL */
    MULO_ERR_SHAPE = 2,       /* sizes inconsistent with each other or with the context */
    MULO_ERR_RANGE = 3,       /* a scalar outside its allowed range */
    MULO_ERR_ALLOC = 4,       /* device memory for the workspace could not be obtained */
    MULO_ERR_HIP = 5,         /* a HIP call or a launch failed */
    MULO_ERR_UNSUPPORTED = 6  /* valid in principle, not handled by these kernels */
} mulo_status;

typedef enum { MULO_F32 = 0, MULO_BF16 = 1 } mulo_dtype;

/* Decoder dimensions (a pre-norm Llama-style decoder: RMSNorm, rotary multi-head
 * attention with n_heads * head_dim == d_model, SwiGLU feed-forward, no biases).
 * max_block is the largest draft block L, max_batch the largest batch B and
 * max_seq the number of cache rows per sequence (prefix + image tokens).
 * Limits: head_dim 64 or 128 for MULO_BF16; d_model a multiple of 128, d_ffn of 64 (and at least 128),
 * max_seq of 8 and max_block of 4 for MULO_BF16; vocab a multiple of 4 and at most 262144. */
typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int32_t max_batch, max_seq, max_block;
    int32_t dtype;   /* mulo_dtype: type of weights, activations and KV cache */
    float rms_eps;
    /* MULO_BF16 only, 0 or 1.  1: mulo_create makes a second copy of the projection and lm-head weights inside the
     * context's workspace, in the order in which the weight-streaming kernels feed them to the matrix instruction
     * (rows in groups of 16, k in steps of 32, each 1 KB block contiguous), and calls of at most 64 tokens
     * (single-token steps, island passes) read that copy: whole contiguous KB per load and no lane exchange
     * (projections of such calls 8-12 % faster); calls of 65 to 256 tokens (island passes of larger batches) then stream
     * the weights as well instead of running on the tiled kernels.  Costs the size of those weights again (13 GB for a
     * 7B model) plus the partial sums of a 256-token call. */
    int32_t stream_copy;
} mulo_model_cfg;

/* Target weights, device pointers in the model dtype, row-major [out, in]
 * (y = x W^T).  The library keeps these pointers (and, with stream_copy, a re-ordered copy of its own made at
 * mulo_create): they must stay valid and unchanged until mulo_destroy.
 *   embed [vocab, d]   attn_norm, ffn_norm [n_layers, d]   final_norm [d]
 *   wq, wk, wv, wo [n_layers, d, d]   w_gate, w_up [n_layers, f, d]
 *   w_down [n_layers, d, f]   lm_head [vocab, d]
 * rope_cos / rope_sin: float32 [max_seq, head_dim / 2]; row = absolute cache
 * position, column m rotates the pair (2m, 2m+1) of every head. */
typedef struct {
    const void *embed, *attn_norm, *wq, *wk, *wv, *wo, *ffn_norm, *w_gate, *w_up, *w_down,
        *final_norm, *lm_head;
    const float *rope_cos, *rope_sin;
} mulo_weights;

/* KV cache of the target, device memory of the caller in the model dtype.
 *   k: [n_layers, max_batch, n_heads, max_seq, head_dim]   (position-major rows)
 *   v: [n_layers, max_batch, n_heads, head_dim, max_seq]   (stored transposed, so
 *      that the attention kernel reads keys contiguously for its second product)
 * Rows [0, P) must hold the prefix; mulo_verify_forward writes rows [P, P+L). */
typedef struct {
    void *k, *v;
} mulo_kv;

typedef enum { MULO_ACCEPT_RATIO = 0, MULO_ACCEPT_TAU = 1 } mulo_accept_mode;

/* Parameters of the decision stage (host struct).
 *   H, W        target grid; n0 first position of the block; L block length
 *   radius      l of Eq. 6 (>= 0); -1 selects the raster-scan rule of standard
 *               speculative decoding (everything from the first rejection on)
 *   expand      number of dilations by `radius` (1 = Eq. 6-7 as printed,
 *               0 = only the rejected positions themselves)
 *   pool_k,nbr  codebook-neighbour pooling of Eq. 3: nbr is a device pointer to
 *               int32 [vocab, pool_k] with nbr[x][0] == x; pool_k == 1 (nbr may be
 *               NULL) is the plain test of Eq. 1
 *   resample_mode 0: every marked position draws from the residual of Eq. 2;
 *               1: rejected positions draw from the residual, positions marked
 *               only by expansion draw from p; 2: every marked position draws
 *               from p (Alg. 1 Step 6 samples rejected tokens from the target)
 *   accept_mode MULO_ACCEPT_RATIO: speculative test u q < pbar (Eq. 1 / Eq. 3);
 *               MULO_ACCEPT_TAU: the threshold rule of Eq. 5, accept iff
 *               pbar >= tau (float32), no draft probability and no uniform;
 *               with resample_mode 2 the draft distribution is not read at all
 *   tau         threshold of Eq. 5, finite and >= 0 (read in MULO_ACCEPT_TAU only)
 *   cfg_scale   0: off.  s > 0: classifier-free guidance (supplement, "Sampling": s = 4, empty negative
 *               prompt); the target distribution is softmax(z_u + s (z_c - z_u)).  The entry points
 *               then work on 2 B sequences: sequence b is the conditional one, B + b its
 *               unconditional twin (own cache rows, same image tokens, prefix of the same length P);
 *               logits arguments are [2 B, L, vocab] and 2 B <= max_batch
 *   seed, rng_counter  Philox4x32-10 key and per-step counter; position t of
 *               batch element b uses counter words (t, b, counter_lo,
 *               stream << 24 | counter_hi & 0xffffff), stream 0 for the accept
 *               uniform u = (word0 >> 8) * 2^-24 and 1 for the sampler word. */
typedef struct {
    int32_t H, W, n0, L;
    int32_t radius, expand;
    int32_t pool_k;
    const int32_t *nbr;
    int32_t resample_mode;
    uint64_t seed, rng_counter;
    int32_t accept_mode;
    float tau;
    float cfg_scale;
} mulo_step_params;

/* Static description of a status code; never NULL. */
MULO_API const char *mulo_status_string(mulo_status s);

/* Pure host-side checks (no GPU needed), also run by the entry points below.  Among them: a block of more than
 * 131072 positions is MULO_ERR_UNSUPPORTED (the accept flags of a block are staged in the LDS of one workgroup). */
MULO_API mulo_status mulo_check_model_cfg(const mulo_model_cfg *cfg);
MULO_API mulo_status mulo_check_step_params(const mulo_model_cfg *cfg, int32_t B, const mulo_step_params *p);

/* Device bytes mulo_create will allocate for its workspace (0 on a bad cfg). */
MULO_API uint64_t mulo_workspace_bytes(const mulo_model_cfg *cfg);

/* Create a context on the current HIP device.  cfg and w are host structs
 * (copied); w's members are device pointers (kept, see above).  hip_stream is a
 * hipStream_t (NULL = the default stream).  Allocates the workspace once; no
 * later call allocates.  *out is set only on MULO_OK. */
MULO_API mulo_status mulo_create(const mulo_model_cfg *cfg, const mulo_weights *w, void *hip_stream,
                        mulo_ctx **out);
MULO_API void mulo_destroy(mulo_ctx *ctx); /* NULL is allowed */

/* Step 2 (Sec. 3.2; Alg. 1 Step 2).  Weight-free up-sampling by replication:
 * every low-resolution cell (I, J) of the h x w draft grid emits its r x r
 * children on the (r h) x (r w) grid, and a child's draft distribution is its
 * parent's.
 *   draft        device float32 [B, h*w, vocab]: draft logits, or probabilities
 *                when input_is_probs != 0
 *   draft_tokens device int32 [B, h*w]
 *   tokens_hi    device int32 [B, r*h * r*w]        (out)
 *   q_lo         device float32 [B, h*w, vocab]     (out) softmax(draft), or a copy;
 *                may alias `draft` when input_is_probs != 0
 *   q_row        device int32 [r*h * r*w]           (out) parent row of each position
 *   q_hi         device float32 [B, r*h*r*w, vocab] (out) or NULL: materialised rows
 * Errors: NULL -> MULO_ERR_NULL; B, h, w, r < 1 -> MULO_ERR_RANGE. */
MULO_API mulo_status mulo_upsample_draft(mulo_ctx *ctx, int32_t B, int32_t h, int32_t w, int32_t r,
                                const float *draft, int32_t input_is_probs,
                                const int32_t *draft_tokens, int32_t *tokens_hi, float *q_lo,
                                int32_t *q_row, float *q_hi);

/* Step 3 (Sec. 3.2; Alg. 1 Step 3).  One forward pass of the target over L
 * inputs per sequence against cache rows [0, P); logits[b, j, :] is the
 * next-token logit vector AFTER input j.  Writes cache rows [P, P+L).
 *   in_tokens  device int32 [B, L] (ids outside [0, vocab) are clamped to the nearest valid id, silently: the
 *              kernels never fault on a bad id, and no output flags it; the same holds for draft tokens)
 *   in_embeds  device, model dtype [B, L, d], or NULL; when given it replaces
 *              the embedding lookup (conditioning prefixes)
 *   logits     device float32 [B, L, vocab] (out)
 * Errors: B > max_batch, L > max_block, P + L > max_seq -> MULO_ERR_SHAPE. */
MULO_API mulo_status mulo_verify_forward(mulo_ctx *ctx, mulo_kv *kv, int32_t B, int32_t L, int32_t P,
                                const int32_t *in_tokens, const void *in_embeds, float *logits);

/* Steps 4-5 and the re-draw of the marked positions (Sec. 3.1 Eq. 1-3; Sec. 3.3 Eq. 5-7).
 *   logits       device float32 [B, L, vocab]  target logits of the block
 *   q            device float32 draft probabilities; row of position t of batch
 *                b starts at q + b * q_batch_stride + row(t) * vocab, where
 *                row(t) = q_row[t], or t when q_row is NULL; may be NULL when
 *                accept_mode is MULO_ACCEPT_TAU and resample_mode is 2
 *   draft_tokens device int32 [B, L]  x~ on the target grid
 *   tokens_out   device int32 [B, L]  (out) x~ where unmarked, re-drawn where marked
 *   accept, mask device uint8 [B, L]  (out) 1 = accepted / 1 = marked (R_X)
 *   t0           device int32 [B]     (out) first rejected position, L if none
 *   stats        device int32 [B, 4]  (out) accepted, rejected, marked, near ties
 *                (|pbar - u q| < 1e-4 q; threshold rule: |pbar - tau| < 1e-4 tau)
 *   p_probs      device float32 [B, L, vocab] (out) or NULL: softmax(logits) */
MULO_API mulo_status mulo_accept_local_resample(mulo_ctx *ctx, int32_t B, const mulo_step_params *p,
                                       const float *logits, const float *q, const int32_t *q_row,
                                       int64_t q_batch_stride, const int32_t *draft_tokens,
                                       int32_t *tokens_out, uint8_t *accept, uint8_t *mask,
                                       int32_t *t0, int32_t *stats, float *p_probs);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc (mulo_create allocates a workspace, so such a caller may have no context).  The decision
 * stage of mulo_accept_local_resample without a context: same arguments and same results bit for bit, with the
 * vocabulary size and the HIP stream (a hipStream_t, NULL = the default stream) passed directly.  The row
 * statistics that the accept kernel leaves for the re-draw kernel live in a static device array of the library
 * (2 * MULO_STATIC_MAX_ROWS floats = 512 KiB on every GPU the library runs on, held until the process ends).
 * The call allocates and frees nothing and synchronises with nothing; it runs on the current HIP device.
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two threads) race
 * and give undefined decisions; calls on one stream are ordered and safe.  Nothing of an earlier call's contents
 * is read.
 * Errors: as mulo_accept_local_resample, plus B * L > MULO_STATIC_MAX_ROWS -> MULO_ERR_SHAPE; vocab < 4 ->
 * MULO_ERR_RANGE; vocab not a multiple of 4 or > 262144 -> MULO_ERR_UNSUPPORTED; the array's address cannot be
 * obtained -> MULO_ERR_HIP. */
#define MULO_STATIC_MAX_ROWS 65536
MULO_API mulo_status mulo_accept_local_resample_static(void *hip_stream, int32_t vocab, int32_t B,
                                              const mulo_step_params *p, const float *logits, const float *q,
                                              const int32_t *q_row, int64_t q_batch_stride,
                                              const int32_t *draft_tokens, int32_t *tokens_out, uint8_t *accept,
                                              uint8_t *mask, int32_t *t0, int32_t *stats, float *p_probs);

/* The whole step for one block: up-sample the h_blk x w low-resolution rows
 * behind the block (h_blk * r * w * r == L), run the target over the inputs
 * [prev, x~_0 .. x~_{L-2}] so that logit row j is p for draft position j, then
 * decide and re-draw.  Cache rows [P, P+L) are written; rows after the first
 * rejection are stale afterwards and P is never advanced (the caller commits).
 *   draft        device float32 [B, h_blk*w, vocab] logits (or probabilities); may be
 *                NULL when accept_mode is MULO_ACCEPT_TAU and resample_mode is 2
 *   draft_tokens device int32 [B, h_blk*w]
 *   prev_tokens  device int32 [B]  last committed (or last prefix) token (with guidance: also fed
 *                to the unconditional twin)
 *   tokens_hi    device int32 [B, L] (out) or NULL: the up-sampled draft x~
 *   logits       device float32 [B, L, vocab] (out) or NULL
 *   other outputs as in mulo_accept_local_resample. */
MULO_API mulo_status mulo_verify_step(mulo_ctx *ctx, mulo_kv *kv, int32_t B, int32_t P,
                             const mulo_step_params *p, int32_t h_blk, int32_t w, int32_t r,
                             const float *draft, int32_t input_is_probs,
                             const int32_t *draft_tokens, const int32_t *prev_tokens,
                             int32_t *tokens_out, uint8_t *accept, uint8_t *mask, int32_t *t0,
                             int32_t *stats, int32_t *tokens_hi, float *logits);

/* Sequential re-sampling of the marked positions (Alg. 1 Step 6): for u = u_start .. L-1 in order, the
 * target is evaluated on the single input token that precedes position u ([prev, x_0 .. x_{L-2}][u], taken
 * from `tokens` as it stands) against cache rows [0, P+u), cache row P+u is rewritten, and where mask[b,u]
 * is set tokens[b,u] is replaced by a draw from softmax of that logit row (integer inverse CDF, Philox
 * stream 2 at (u, b)); unmarked positions keep their token but their cache row is refreshed, because their
 * context changed.  u_start must be <= the first marked position of every sequence (0 is always valid; the
 * smallest t0 of the parallel step is the useful value).  L - u_start single-token forwards are enqueued.
 *   prev_tokens device int32 [B]; mask device uint8 [B, L]; tokens device int32 [B, L] (in/out)
 *   logits      device float32 [B, L, vocab] (out) or NULL: the logit rows u_start .. L-1 that were used
 * Errors: B > max_batch, P + L > max_seq -> MULO_ERR_SHAPE; u_start outside [0, L] -> MULO_ERR_RANGE. */
MULO_API mulo_status mulo_resample_sequential(mulo_ctx *ctx, mulo_kv *kv, int32_t B, int32_t P, int32_t L,
                                     int32_t u_start, uint64_t seed, uint64_t rng_counter,
                                     const int32_t *prev_tokens, const uint8_t *mask, int32_t *tokens,
                                     float *logits);

/* Rejection islands (Sec. 3.4, Eq. 8): the 8-connected components of the marked set R_X on the 2-D token grid
 * (rows and columns each differ by at most one; columns do not wrap; only positions of the block exist).
 *   mask    device uint8 [B, L]  R_X of the block that starts at grid position n0 (whole rows of W columns)
 *   island  device int32 [B, L]  (out) 0 where unmarked, else 1 + the smallest block position of the island
 *   rank    device int32 [B, L]  (out) -1 where unmarked, else the number of positions of the same island that
 *           precede it in raster order: islands are re-sampled concurrently, pass r takes every rank-r position
 *   counts  device int32 [B, 2]  (out) number of islands, size of the largest (= number of passes)
 * Errors: L not a multiple of W, n0 not on a row start, L > 16384 -> MULO_ERR_SHAPE / MULO_ERR_UNSUPPORTED. */
MULO_API mulo_status mulo_rejection_islands(mulo_ctx *ctx, int32_t B, int32_t W, int32_t n0, int32_t L,
                                   const uint8_t *mask, int32_t *island, int32_t *rank, int32_t *counts);

/* Island-parallel re-sampling (Sec. 3.4, "Parallel resampling via rejection islands"): the islands of R_X are
 * re-sampled concurrently, the positions inside an island one after the other in raster order.  Pass r
 * (r = 0 .. n_passes-1) evaluates the target ONCE on the rank-r position of every island that has one (a batch of
 * single-token queries at scattered cache rows) and replaces tokens[b,u] of each by a draw from softmax of its
 * logit row (integer inverse CDF, Philox stream 2 at (u, b), as in mulo_resample_sequential).  The query at block
 * position u takes the current token at u-1 as input (prev_tokens[b] for u = 0), rewrites cache row P+u in every
 * layer and attends to rows [0, P), to its own row, and to the earlier rows P+v of its block whose position is
 * settled: not marked (the verification pass's row) or re-drawn in an earlier pass.  Marked positions not yet
 * re-drawn are hidden.  (Which context a concurrently evaluated position may use is not spelled out by the paper;
 * this is a reading of Sec. 3.4: only settled positions are context.)  One island that covers everything
 * from its first position on gives exactly mulo_resample_sequential.  The cache rows P .. P+L-1 must hold the
 * verification pass over the block.  bf16 models only.
 * What the cache holds afterwards: row P+v carries the K/V of INPUT v, the token at position v-1.  A pass rewrites
 * only the rows of the positions it evaluates, so when position u is re-drawn and u+1 is not evaluated after it
 * (u+1 is unmarked: the right edge of every island row; or it belongs to another island and was drawn earlier), row
 * P+u+1 keeps the K/V of the draft token that stood at u during verification: later passes attend to that row as
 * it is, and after the call the rows from the first marked position on do not match `tokens`.  As after
 * mulo_verify_step, the caller commits the block (one mulo_verify_forward over the final tokens rewrites rows
 * P .. P+L-1) before the next step; mulo_resample_sequential, by contrast, refreshes every row from u_start on.
 *   n_passes    size of the largest island over the batch, max_islands >= the largest number of islands of a
 *               sequence: both from counts of mulo_rejection_islands (host values; upper bounds are fine);
 *               B * max_islands <= max_batch * max_block
 *   prev_tokens device int32 [B]; mask device uint8 [B, L]; rank device int32 [B, L] (mulo_rejection_islands)
 *   tokens      device int32 [B, L] (in/out)
 *   logits      device float32 [B, L, vocab] (out) or NULL: the logit row of every re-drawn position
 *   overflow    device int32 [1] or NULL: incremented by the number of positions a pass could not place because
 *               max_islands was too small (they are then not re-drawn); the caller zeroes it
 * Nothing synchronises with the host.  Errors: as mulo_resample_sequential; float32 model ->
 * MULO_ERR_UNSUPPORTED; B * max_islands too large -> MULO_ERR_SHAPE. */
MULO_API mulo_status mulo_resample_islands(mulo_ctx *ctx, mulo_kv *kv, int32_t B, int32_t P, int32_t L,
                                  int32_t n_passes, int32_t max_islands, uint64_t seed, uint64_t rng_counter,
                                  const int32_t *prev_tokens, const uint8_t *mask, const int32_t *rank,
                                  int32_t *tokens, float *logits, int32_t *overflow);

/* Test and debugging aid (not part of the method): copies the first `bytes` bytes of one of the context's
 * workspace buffers, as the last mulo_verify_forward (or step) left it, to dst on the context's stream.  With a
 * one-layer model these are that layer's intermediate tensors, which is how the tests compare every stage of a
 * layer with the oracle's.  M = B * L of that call; T = the model dtype.
 *   MULO_WS_RESIDUAL  float32 [M, d]       residual stream after the last layer
 *   MULO_WS_NORMED    T [M, d]             output of the last RMSNorm that ran (the final norm)
 *   MULO_WS_Q         T [B, n_heads, L, head_dim]  rotated queries of the last layer
 *   MULO_WS_ATTN      T [M, d]             attention output of the last layer (input of the out projection)
 *   MULO_WS_FFN       T [M, d_ffn]         silu(gate) * up of the last layer (input of the down projection)
 * After a bf16 call of at most 64 tokens (256 with stream_copy: single-token steps, island passes) NORMED, ATTN and
 * FFN are not row-major: such calls keep the token operand of every projection in the order the matrix instruction reads it
 * (tokens in groups of 16, columns in steps of 32; element (m, k) of a [M, K] operand sits at
 * ((m / 16) * (K / 32) + k / 32) * 512 + ((k % 32) / 8 * 16 + m % 16) * 8 + k % 8).
 *   dst  device pointer, at least `bytes` bytes
 * Errors: unknown buffer -> MULO_ERR_RANGE; bytes not a multiple of 16 or larger than the buffer (sized for
 * max_batch * max_block tokens) -> MULO_ERR_SHAPE. */
enum { MULO_WS_RESIDUAL = 0, MULO_WS_NORMED = 1, MULO_WS_Q = 2, MULO_WS_ATTN = 3, MULO_WS_FFN = 4 };
MULO_API mulo_status mulo_workspace_read(mulo_ctx *ctx, int32_t which, void *dst, uint64_t bytes);

/* Optional per-kernel timing (measurement aid, not part of the method).  While
 * enabled, every kernel launch of the entry points above is bracketed by a pair
 * of HIP events on the context's stream.  mulo_profile_read synchronises the
 * stream, adds up the elapsed time and the launch count per kernel class since
 * the last read, and clears them.  ms and launches are host arrays of
 * MULO_PROF_N entries.  At most 16384 launches are recorded between two reads.
 * enable: 0 = off, 1 = every class, MULO_PROF_ONLY(c) = class c alone (each pair of events
 * costs a few microseconds of stream time, so a benchmark brackets only what it reports). */
#define MULO_PROF_ONLY(c) (0x100 | (c))
enum {
    MULO_PROF_GEMM_QKV = 0,   /* QKV projection + rotary + cache append */
    MULO_PROF_GEMM_OUT = 1,   /* attention output projection + residual */
    MULO_PROF_GEMM_GATE_UP = 2, /* gate|up projection + SwiGLU */
    MULO_PROF_GEMM_DOWN = 3,  /* down projection + residual */
    MULO_PROF_GEMM_LM_HEAD = 4,
    MULO_PROF_ATTENTION = 5,
    MULO_PROF_NORM_EMBED = 6, /* embedding lookup, RMSNorm */
    MULO_PROF_UPSAMPLE = 7,   /* draft softmax (or copy) + token replication */
    MULO_PROF_ACCEPT = 8,     /* target softmax statistics + accept test */
    MULO_PROF_MASK_SAMPLE = 9, /* neighbourhood mask + residual draw */
    MULO_PROF_OTHER = 10,     /* input shift; float32-path helpers */
    MULO_PROF_N = 11
};
MULO_API mulo_status mulo_profile(mulo_ctx *ctx, int32_t enable);
MULO_API mulo_status mulo_profile_read(mulo_ctx *ctx, float *ms, int32_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* MULO_H */
