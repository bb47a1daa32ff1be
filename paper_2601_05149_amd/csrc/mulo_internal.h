// Internal launcher declarations shared by the translation units of libmulo.
// Every launcher only enqueues work on `st`; shapes are validated by the caller
// (mulo_api.hip) before any of them runs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mulo {

// A HIP call made while configuring a kernel (not a launch) failed: the entry point that is running returns
// MULO_ERR_HIP.  The launcher that notes an error does not launch.
void note_hip_error(hipError_t e);
// Raises the dynamic-LDS limit of `kern` to `bytes` once per process (state: 0 = not tried, 1 = done, -1 = failed);
// false, with the error noted, when the runtime refuses.
bool ensure_dynamic_lds(const void* kern, int bytes, int* state);

// Launches of at most STREAM_MAX_TOKENS tokens (single-token decoding of a few sequences, island passes) run every
// bf16 projection in the weight-streaming kernel.  That kernel feeds its MFMA straight from registers, so its token
// operand [M, K] is kept in the order the instruction reads it (FRAGMENT ORDER): tokens in groups of 16, k in steps of
// 32; the 1 KB of (group t, step s) is contiguous, and inside it lane 16 c + r of a wavefront owns 16 bytes: k
// 32 s + 8 c .. + 7 of token 16 t + r.  The kernels that produce such an operand (RMSNorm, attention, the SwiGLU
// epilogue) write it in this order when the launch streams; one load instruction then reads a whole contiguous KB
// and no lane exchange is needed.  Buffers are sized for whole groups of 16 tokens.
constexpr int STREAM_MAX_TOKENS = 64;
inline bool streams_weights(int M) { return M <= STREAM_MAX_TOKENS; }
// With the context's weight copy in fragment order, launches of up to STREAM_MAX_TOKENS_COPY tokens stream: above
// STREAM_SHARED_MIN_TOKENS they run in the kernel that shares the token operand through LDS and splits K over workgroups.
constexpr int STREAM_MAX_TOKENS_COPY = 256;
#ifndef STREAM_SHARED_MIN_TOKENS
#define STREAM_SHARED_MIN_TOKENS 64
#endif
// How a launch of few tokens runs its projections (decided once per forward, the same for every kernel of it):
//   stream  the token operands are in fragment order and the projections run in the weight-streaming kernels
//   w_frag  the weight pointers are the context's copies in fragment order
//   ksums   scratch for the sums of the K slices (stream_ksum_floats) when w_frag, else nullptr
struct StreamMode { bool stream, w_frag; float* ksums; };
// K slices per 128-column group in the LDS-sharing kernel: as many as keep the launch within one round of 256
// workgroups, at most 8, at least 8 k-steps each.  A function of the projection's shape only, so the order of every
// sum is fixed by the model.
inline int stream_ksplit(int ncols, int K) {
    const int groups = (ncols + 127) / 128, steps = K / 32;
    int ks = 256 / groups;
    ks = ks < 1 ? 1 : (ks > 8 ? 8 : ks);
    const int most = steps / 8 > 1 ? steps / 8 : 1;
    return ks > most ? most : ks;
}
// floats of partial sums such a launch of M tokens over `ncols` output columns (gate|up: 2 f, q|k|v: 3 d) needs
inline size_t stream_ksum_floats(int M, int ncols, int K) { return (size_t)stream_ksplit(ncols, K) * M * ncols; }
__host__ __device__ inline int64_t frag_index(int m, int k, int K) {   // in elements; runs of 8 k stay contiguous
    return ((int64_t)(m >> 4) * (K >> 5) + (k >> 5)) * 512 + (((k & 31) >> 3) * 16 + (m & 15)) * 8 + (k & 7);
}

// ---- decision stage (decide.hip) -------------------------------------------
struct DecideArgs {
    int B, L, V;
    int H, W, n0;
    int rho;          // Chebyshev radius expand*radius; -1 = raster-scan rule
    int pool_k;
    const int32_t* nbr;
    int resample_mode;   // 0 residual, 1 residual for rejected / p for expanded, 2 p
    int accept_mode;     // 0: u q < pbar (Eq. 1 / 3), 1: pbar >= tau (Eq. 5)
    float tau;
    uint32_t key0, key1, ctr_lo, ctr_hi24;
    const float* logits;        // [B, L, V]
    const float* logits_u;      // [B, L, V] unconditional logits (classifier-free guidance) or nullptr
    float cfg_scale;
    const float* q;             // rows of V floats
    const int32_t* q_row;       // [L] or nullptr
    int64_t q_batch_stride;
    const int32_t* draft_tokens;  // [B, L]
    int32_t* tokens_out;
    uint8_t* accept;
    uint8_t* mask;
    int32_t* t0;      // [B]
    int32_t* stats;   // [B, 4]
    float* p_probs;   // [B, L, V] or nullptr
    float* rowmax;    // [B*L] workspace
    float* rowinv;    // [B*L] workspace: 1 / sum exp
    // Replication geometry of the draft rows (a verification step): position (r I + a) W + r J + c of the block reads
    // draft row I up_w + J, W = up_r * up_w.  0: unknown (q_row is the caller's).  Only used to place the r * r
    // children of a draft row on one XCD next to each other, so that the row is fetched into one L2 once.
    int up_r, up_w;
};
void launch_softmax_rows(const float* in, float* out, int64_t rows, int V, hipStream_t st);
void launch_copy_rows(const float* in, float* out, int64_t n_floats, hipStream_t st);
// dst[b * dst_stride + c] = src[b * V + c] for B rows of V floats (V a multiple of 4)
void launch_copy_rows_strided(const float* src, float* dst, int B, int V, int64_t dst_stride, hipStream_t st);
void launch_upsample_tokens(const int32_t* draft_tokens, int32_t* tokens_hi, int32_t* q_row, int B,
                            int h, int w, int r, hipStream_t st);
void launch_gather_rows(const float* q_lo, const int32_t* q_row, float* q_hi, int B, int n_lo,
                        int n_hi, int V, hipStream_t st);
void launch_islands(const uint8_t* mask, int32_t* island, int32_t* rank, int32_t* counts, int B, int W, int n0, int L,
                    hipStream_t st);
void launch_seq_input(const int32_t* prev, const int32_t* tokens, int32_t* inp, int B, int L, int u, hipStream_t st);
void launch_seq_draw(const float* logits, const uint8_t* mask, int32_t* tokens, int B, int L, int V, int u,
                     uint64_t seed, uint64_t rng_counter, hipStream_t st);
// island-parallel re-sampling, pass `pass`: slots of the rank-`pass` positions (pos_tab, inputs), the hidden set
// of the pass, and afterwards the draws of the slots from their logit rows
void launch_island_select(const int32_t* prev, const int32_t* tokens, const uint8_t* mask, const int32_t* rank,
                          int32_t* pos_tab, int32_t* inp, uint8_t* hide, int32_t* overflow, int B, int L, int P,
                          int cap, int pass, hipStream_t st);
void launch_island_draw(const float* logits, const int32_t* pos_tab, int32_t* tokens, float* logits_out, int B,
                        int L, int V, int P, int cap, uint64_t seed, uint64_t rng_counter, hipStream_t st);
void launch_accept(const DecideArgs& a, hipStream_t st);         // softmax statistics + accept test
// the accept test from row parts (m, s per 128 columns, float pairs [rows, n_parts]) that the lm-head GEMM left;
// needs pool_k <= 1, no probability output and no guidance
void launch_accept_from_parts(const DecideArgs& a, const float* parts, int n_parts, hipStream_t st);
void launch_decide_finish(const DecideArgs& a, hipStream_t st);  // t0, Eq. 6-7 mask, the step's counters
void launch_mask_sample(const DecideArgs& a, hipStream_t st);    // residual draw of the marked positions
void launch_shift_inputs(const int32_t* prev, const int32_t* tokens_hi, int32_t* inputs, int B,
                         int L, hipStream_t st);

// ---- decoder forward (elementwise.hip, gemm.hip, attention.hip) ------------
struct RopeArgs {
    const float* cos;   // [max_seq, dh/2]
    const float* sin;
    int L, P, n_heads, head_dim, max_seq, max_batch, layer;
    // Scattered single-token queries (island-parallel re-sampling): token m is slot m % L of sequence m / L and
    // sits at cache row pos_tab[m] (< 0: an unused slot, nothing of it is written).  nullptr: token m is position
    // m % L of sequence m / L, at cache row P + m % L.
    const int32_t* pos_tab = nullptr;
};
// x[m, :] = embed[clamp(tok[m])]  (float32 residual stream); T = float or bf16 storage
void launch_embed(const void* embed, int dtype, const int32_t* tok, const void* in_embeds, float* x,
                  int M, int d, int V, hipStream_t st);
// frag: write `out` in fragment order (bf16 launches that stream the weights)
void launch_rmsnorm(const float* x, const void* gain, int dtype, void* out, int M, int d, float eps, bool frag,
                    hipStream_t st);

// bf16 MFMA GEMMs, C = A[M,K] * W[N,K]^T with fused epilogues
void launch_gemm_qkv_bf16(const void* xh, const void* wq, const void* wk, const void* wv, void* q_out,
                          void* k_cache, void* v_cache, int M, int d, const RopeArgs& ra, const StreamMode& sm,
                          hipStream_t st);
void launch_gemm_resid_bf16(const void* a, const void* w, float* x, int M, int N, int K, const StreamMode& sm,
                            hipStream_t st);
void launch_gemm_swiglu_bf16(const void* xh, const void* wg, const void* wu, void* h, int M, int f,
                             int d, const StreamMode& sm, hipStream_t st);
// Copies `layers` bf16 matrices [rows, K] (contiguous, rows % 16 == 0 or layers == 1) into fragment order: rows in
// groups of 16, k in steps of 32, the KB of (group, step) contiguous with lane 16 c + r holding k 8 c .. 8 c + 7 of
// row r; rows past the last are zeros.  dst holds layers * ceil16(rows) * K elements.
void launch_pack_weights(const void* src, void* dst, int layers, int rows, int K, hipStream_t st);
inline size_t packed_weight_elems(int layers, int rows, int K) { return (size_t)layers * ((rows + 15) / 16 * 16) * K; }
// parts: nullptr, or float pairs [M, ceil(V / 128)] that receive the softmax statistics of every 128-column part of
// every row (row_parts.h); returns whether they were written (only the kernels whose wavefront tile is 128 columns
// wide produce them)
bool launch_gemm_logits_bf16(const void* xh, const void* w, float* logits, float* parts, int M, int V, int d,
                             const StreamMode& sm, hipStream_t st);
size_t attention_scratch_bytes(int max_batch, int n_heads, int head_dim);   // partial results of the key split
// frag_out: `out` feeds a weight-streaming projection: written in fragment order
void launch_attention_bf16(const void* q, const void* k_cache, const void* v_cache, void* out, float* scratch,
                           int B, int L, int P, int n_heads, int head_dim, int max_seq, int max_batch,
                           int layer, bool frag_out, hipStream_t st);
// cap single-token queries per sequence at scattered cache rows: slot j of sequence b sits at row
// pos_tab[b * cap + j] (< 0: unused slot, its output row is zeroed) and attends to rows <= its own except the rows
// P0 + t of its sequence with hide[b, t] set (t < Lblk; its own row is never hidden).  Rows are in [P0, P0 + Lblk).
void launch_attention_scattered_bf16(const void* q, const void* k_cache, const void* v_cache, void* out,
                                     float* scratch, int B, const int32_t* pos_tab, int cap, const uint8_t* hide,
                                     int P0, int Lblk, int n_heads, int head_dim, int max_seq, int max_batch,
                                     int layer, bool frag_out, hipStream_t st);

// float32 path (small configurations): plain tiled GEMM + separate elementwise kernels
void launch_gemm_f32(const float* a, const float* w, float* c, int M, int N, int K, int ldc,
                     int accumulate, hipStream_t st);
void launch_rope_append_f32(const float* qkv, float* q_out, float* k_cache, float* v_cache, int M,
                            int d, const RopeArgs& ra, hipStream_t st);
void launch_swiglu_f32(const float* gu, float* h, int M, int f, hipStream_t st);
void launch_attention_f32(const float* q, const float* k_cache, const float* v_cache, float* out,
                          float* scratch, int B, int L, int P, int n_heads, int head_dim,
                          int max_seq, int max_batch, int layer, hipStream_t st);

}  // namespace mulo
