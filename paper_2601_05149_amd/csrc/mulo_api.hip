// C ABI of libmulo (see include/mulo.h): argument validation, the context with
// its workspace, and the order in which the kernels of a verification step are
// enqueued (Alg. 1 Steps 2-5 + residual re-draw).  Nothing here computes.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "../../include/mulo.h"
#include "mulo_internal.h"

using namespace mulo;

// Scratch of mulo_accept_local_resample_static, the entry point for callers that cannot allocate: the row maximum
// and the inverse row sum of the target softmax, MULO_STATIC_MAX_ROWS floats each, which the accept kernel leaves
// for the re-draw kernel.  Every GPU the library runs on holds its own copy at its own address until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress: kernels, copies and memsets get the
// device address that call returns (static_scratch below), never the name.
static __device__ __align__(256) float scratch[2 * MULO_STATIC_MAX_ROWS];

namespace mulo {
namespace {
hipError_t g_config_error = hipSuccess;   // first failed configuration call since the last check_launch()
}
void note_hip_error(hipError_t e) {
    if (e != hipSuccess && g_config_error == hipSuccess) g_config_error = e;
}
bool ensure_dynamic_lds(const void* kern, int bytes, int* state) {
    if (*state == 0) {
        const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        *state = e == hipSuccess ? 1 : -1;
        if (e != hipSuccess) (void)hipGetLastError();
    }
    if (*state < 0) note_hip_error(hipErrorInvalidValue);
    return *state > 0;
}
}  // namespace mulo

struct mulo_ctx {
    mulo_model_cfg cfg;
    mulo_weights w;
    hipStream_t st;
    int64_t maxM;
    size_t esz;  // bytes per element of the model dtype
    // workspace
    float* x;        // [maxM, d] residual stream
    void* xh;        // [maxM, d] normalised activations
    void* qbuf;      // [maxB, nh, maxL, dh]
    void* att;       // [maxM, d]
    void* hmid;      // [maxM, f]
    float* tmp;      // float32 path only: [maxM, max(3d, 2f)]
    float* logits;   // [maxM, V]   (mulo_verify_step)
    float* q_lo;     // [maxM, V]
    float* rowmax;   // [maxM]
    float* rowinv;   // [maxM]
    int32_t* inputs;     // [maxM]
    int32_t* tokens_hi;  // [maxM]
    int32_t* q_row;      // [maxL]
    float* attn_part;    // partial results of the key-split single-token attention
    int32_t* isl_pos;    // [maxM] island-parallel re-sampling: cache row of every slot of a pass
    uint8_t* isl_hide;   // [maxM] positions hidden from the queries of a pass
    float* row_parts;    // [maxM, ceil(V / 128)] float pairs: softmax statistics per 128-column part (lm-head epilogue)
    // cfg.stream_copy: the projection and lm-head weights once more, in the weight-streaming kernels' fragment order
    // (same layer strides as the caller's, the lm-head padded to whole groups of 16 rows); nullptr without the copy
    const char *pk_wq, *pk_wk, *pk_wv, *pk_wo, *pk_gate, *pk_up, *pk_down, *pk_lm;
    float* ksums;        // with the copy: sums of the K slices of a 65..256-token launch's projections
    void* base;      // single allocation
    // optional per-launch timing (mulo_profile)
    bool prof_on = false;
    uint32_t prof_mask = 0;   // classes that are bracketed
    int prof_n = 0;
    std::vector<hipEvent_t> prof_ev;   // 2 events per recorded launch
    std::vector<int> prof_cls;
};

namespace {

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

constexpr int N_BUF = 19;
struct Layout {
    size_t off[N_BUF];
    size_t total;
};

// elements of the fragment-order copy: wq, wk, wv, wo, w_gate, w_up, w_down of every layer, then the lm-head
size_t stream_copy_elems(const mulo_model_cfg& c) {
    const int nl = c.n_layers, d = c.d_model, f = c.d_ffn;
    return 4 * packed_weight_elems(nl, d, d) + 2 * packed_weight_elems(nl, f, d) + packed_weight_elems(nl, d, f) +
           packed_weight_elems(1, c.vocab, d);
}

// the largest partial-sum scratch a projection of this model asks for, at the most tokens that stream (or fit)
size_t ksum_bytes(const mulo_model_cfg& c) {
    const size_t M = (size_t)c.max_batch * c.max_block;
    const int Ms = (int)(M < (size_t)STREAM_MAX_TOKENS_COPY ? M : (size_t)STREAM_MAX_TOKENS_COPY);
    const int d = c.d_model, f = c.d_ffn, V = c.vocab;
    size_t n = stream_ksum_floats(Ms, 3 * d, d);
    const size_t others[4] = {stream_ksum_floats(Ms, d, d), stream_ksum_floats(Ms, 2 * f, d), stream_ksum_floats(Ms, d, f),
                              stream_ksum_floats(Ms, V, d)};
    for (size_t o : others) n = o > n ? o : n;
    return n * sizeof(float);
}

Layout plan(const mulo_model_cfg& c) {
    const size_t M = (size_t)c.max_batch * c.max_block, d = c.d_model, f = c.d_ffn, V = c.vocab;
    const size_t M16 = (M + 15) / 16 * 16;   // the operands of the projections hold whole groups of 16 tokens (fragment order)
    const size_t e = c.dtype == MULO_BF16 ? 2 : 4;
    const size_t tmpw = c.dtype == MULO_F32 ? (3 * d > 2 * f ? 3 * d : 2 * f) : 0;
    const size_t sizes[N_BUF] = {M * d * 4, M16 * d * e, M * d * e, M16 * d * e, M16 * f * e, M * tmpw * 4,
                              M * V * 4, M * V * 4, M * 4, M * 4, M * 4, M * 4, (size_t)c.max_block * 4,
                              c.dtype == MULO_BF16 ? attention_scratch_bytes(c.max_batch, c.n_heads, c.head_dim) : 0,
                              M * 4, M, c.dtype == MULO_BF16 ? M * ((V + 127) / 128) * 8 : 0,
                              c.dtype == MULO_BF16 && c.stream_copy ? stream_copy_elems(c) * 2 : 0,
                              c.dtype == MULO_BF16 && c.stream_copy ? ksum_bytes(c) : 0};
    Layout l{};
    size_t o = 0;
    for (int i = 0; i < N_BUF; ++i) {
        l.off[i] = o;
        o += align_up(sizes[i]);
    }
    l.total = o;
    return l;
}

bool hip_ok(hipError_t e) { return e == hipSuccess; }

constexpr int PROF_MAX = 16384;

// Brackets the launches issued while it is alive with two events on the stream.
struct ProfScope {
    mulo_ctx* c;
    int i;
    ProfScope(mulo_ctx* ctx, int cls) : c(ctx), i(-1) {
        if (!c->prof_on || !((c->prof_mask >> cls) & 1u) || c->prof_n >= PROF_MAX) return;
        i = c->prof_n++;
        c->prof_cls[i] = cls;
        (void)hipEventRecord(c->prof_ev[2 * i], c->st);
    }
    ~ProfScope() {
        if (i >= 0) (void)hipEventRecord(c->prof_ev[2 * i + 1], c->st);
    }
};
#define PROF(cls) ProfScope prof_scope_##__LINE__(c, cls)

mulo_status check_launch() {
    const bool configured = g_config_error == hipSuccess;
    g_config_error = hipSuccess;
    return hip_ok(hipGetLastError()) && configured ? MULO_OK : MULO_ERR_HIP;
}

// Device address of `scratch` on the current device, looked up once per device (with that device current).
constexpr int MAX_DEVICES = 64;
float* static_scratch() {
    static float* per_device[MAX_DEVICES] = {};
    int dev = -1;
    if (!hip_ok(hipGetDevice(&dev)) || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    if (!per_device[dev]) {
        void* p = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)))) {
            (void)hipGetLastError();
            return nullptr;
        }
        per_device[dev] = static_cast<float*>(p);
    }
    return per_device[dev];
}

mulo_status check_forward_args(const mulo_ctx* ctx, const mulo_kv* kv, int B, int L, int P) {
    if (!ctx || !kv || !kv->k || !kv->v) return MULO_ERR_NULL;
    if (B < 1 || L < 1 || P < 0) return MULO_ERR_RANGE;
    if (B > ctx->cfg.max_batch || L > ctx->cfg.max_block || (int64_t)P + L > ctx->cfg.max_seq)
        return MULO_ERR_SHAPE;
    return MULO_OK;
}

// Scattered single-token queries (island-parallel re-sampling): the "block" is L slots per sequence, slot j of
// sequence b sits at cache row pos_tab[b * L + j] (< 0: unused); rows P0 + t of a sequence with hide[b, t] set
// are not attended to.
struct Scatter {
    const int32_t* pos_tab;
    const uint8_t* hide;
    int P0, Lblk;
};

// want_parts: also leave the softmax statistics of every 128-column part of every logit row in c->row_parts
// (returns whether the lm-head kernel that ran produces them)
bool enqueue_forward(mulo_ctx* c, mulo_kv* kv, int B, int L, int P, const int32_t* tok, const void* emb,
                     float* logits, const Scatter* sc = nullptr, bool want_parts = false) {
    const mulo_model_cfg& m = c->cfg;
    const int M = B * L, d = m.d_model, f = m.d_ffn, V = m.vocab, dt = m.dtype;
    const size_t e = c->esz;
    hipStream_t st = c->st;
    // a handful of tokens: every bf16 projection streams its weights and takes its token operand in fragment order
    // with the weight copy up to 256 tokens stream (above 64 in the kernel that shares the token operand through LDS)
    const bool has_copy = c->pk_wq != nullptr;
    const bool frag = dt == MULO_BF16 && M <= (has_copy ? STREAM_MAX_TOKENS_COPY : STREAM_MAX_TOKENS);
    const bool wfrag = frag && has_copy;
    const StreamMode sm{frag, wfrag, wfrag ? c->ksums : nullptr};
    { PROF(MULO_PROF_NORM_EMBED); launch_embed(c->w.embed, dt, tok, emb, c->x, M, d, V, st); }
    for (int l = 0; l < m.n_layers; ++l) {
        RopeArgs ra{c->w.rope_cos, c->w.rope_sin, L, P, m.n_heads, m.head_dim, m.max_seq, m.max_batch, l};
        if (sc) ra.pos_tab = sc->pos_tab;
        // launches that stream the weights read the context's copy in fragment order when it has one (same strides)
        const char* wq = (wfrag ? c->pk_wq : (const char*)c->w.wq) + (size_t)l * d * d * e;
        const char* wk = (wfrag ? c->pk_wk : (const char*)c->w.wk) + (size_t)l * d * d * e;
        const char* wv = (wfrag ? c->pk_wv : (const char*)c->w.wv) + (size_t)l * d * d * e;
        const char* wo = (wfrag ? c->pk_wo : (const char*)c->w.wo) + (size_t)l * d * d * e;
        const char* wg = (wfrag ? c->pk_gate : (const char*)c->w.w_gate) + (size_t)l * f * d * e;
        const char* wu = (wfrag ? c->pk_up : (const char*)c->w.w_up) + (size_t)l * f * d * e;
        const char* wd = (wfrag ? c->pk_down : (const char*)c->w.w_down) + (size_t)l * d * f * e;
        const char* g_attn = (const char*)c->w.attn_norm + (size_t)l * d * e;
        const char* g_ffn = (const char*)c->w.ffn_norm + (size_t)l * d * e;
        { PROF(MULO_PROF_NORM_EMBED); launch_rmsnorm(c->x, g_attn, dt, c->xh, M, d, m.rms_eps, frag, st); }
        if (dt == MULO_BF16) {
            { PROF(MULO_PROF_GEMM_QKV); launch_gemm_qkv_bf16(c->xh, wq, wk, wv, c->qbuf, kv->k, kv->v, M, d, ra, sm, st); }
            { PROF(MULO_PROF_ATTENTION);
              if (sc) launch_attention_scattered_bf16(c->qbuf, kv->k, kv->v, c->att, c->attn_part, B, sc->pos_tab, L, sc->hide,
                                                      sc->P0, sc->Lblk, m.n_heads, m.head_dim, m.max_seq, m.max_batch, l, frag, st);
              else launch_attention_bf16(c->qbuf, kv->k, kv->v, c->att, c->attn_part, B, L, P, m.n_heads, m.head_dim,
                                         m.max_seq, m.max_batch, l, frag, st); }
            { PROF(MULO_PROF_GEMM_OUT); launch_gemm_resid_bf16(c->att, wo, c->x, M, d, d, sm, st); }
            { PROF(MULO_PROF_NORM_EMBED); launch_rmsnorm(c->x, g_ffn, dt, c->xh, M, d, m.rms_eps, frag, st); }
            { PROF(MULO_PROF_GEMM_GATE_UP); launch_gemm_swiglu_bf16(c->xh, wg, wu, c->hmid, M, f, d, sm, st); }
            { PROF(MULO_PROF_GEMM_DOWN); launch_gemm_resid_bf16(c->hmid, wd, c->x, M, d, f, sm, st); }
        } else {
            const float* xh = (const float*)c->xh;
            { PROF(MULO_PROF_GEMM_QKV);
              launch_gemm_f32(xh, (const float*)wq, c->tmp, M, d, d, 3 * d, 0, st);
              launch_gemm_f32(xh, (const float*)wk, c->tmp + d, M, d, d, 3 * d, 0, st);
              launch_gemm_f32(xh, (const float*)wv, c->tmp + 2 * d, M, d, d, 3 * d, 0, st); }
            { PROF(MULO_PROF_OTHER);
              launch_rope_append_f32(c->tmp, (float*)c->qbuf, (float*)kv->k, (float*)kv->v, M, d, ra, st); }
            { PROF(MULO_PROF_ATTENTION);
              launch_attention_f32((const float*)c->qbuf, (const float*)kv->k, (const float*)kv->v, (float*)c->att,
                                   nullptr, B, L, P, m.n_heads, m.head_dim, m.max_seq, m.max_batch, l, st); }
            { PROF(MULO_PROF_GEMM_OUT); launch_gemm_f32((const float*)c->att, (const float*)wo, c->x, M, d, d, d, 1, st); }
            { PROF(MULO_PROF_NORM_EMBED); launch_rmsnorm(c->x, g_ffn, dt, c->xh, M, d, m.rms_eps, frag, st); }
            { PROF(MULO_PROF_GEMM_GATE_UP);
              launch_gemm_f32(xh, (const float*)wg, c->tmp, M, f, d, 2 * f, 0, st);
              launch_gemm_f32(xh, (const float*)wu, c->tmp + f, M, f, d, 2 * f, 0, st); }
            { PROF(MULO_PROF_OTHER); launch_swiglu_f32(c->tmp, (float*)c->hmid, M, f, st); }
            { PROF(MULO_PROF_GEMM_DOWN); launch_gemm_f32((const float*)c->hmid, (const float*)wd, c->x, M, d, f, d, 1, st); }
        }
    }
    { PROF(MULO_PROF_NORM_EMBED); launch_rmsnorm(c->x, c->w.final_norm, dt, c->xh, M, d, m.rms_eps, frag, st); }
    PROF(MULO_PROF_GEMM_LM_HEAD);
    if (dt == MULO_BF16) return launch_gemm_logits_bf16(c->xh, wfrag ? (const void*)c->pk_lm : c->w.lm_head, logits, want_parts ? c->row_parts : nullptr, M, V, d, sm, st);
    launch_gemm_f32((const float*)c->xh, (const float*)c->w.lm_head, logits, M, V, d, V, 0, st);
    return false;
}

void enqueue_upsample(mulo_ctx* c, int B, int h, int w, int r, const float* draft, int input_is_probs,
                      const int32_t* draft_tokens, int32_t* tokens_hi, float* q_lo, int32_t* q_row, float* q_hi) {
    PROF(MULO_PROF_UPSAMPLE);
    const int V = c->cfg.vocab;
    const int64_t rows = (int64_t)B * h * w;
    if (draft) {   // the threshold rule with target re-draws needs no draft distribution
        if (input_is_probs) launch_copy_rows(draft, q_lo, rows * V, c->st);
        else launch_softmax_rows(draft, q_lo, rows, V, c->st);
    }
    launch_upsample_tokens(draft_tokens, tokens_hi, q_row, B, h, w, r, c->st);
    if (q_hi) launch_gather_rows(q_lo, q_row, q_hi, B, h * w, h * r * w * r, V, c->st);
}

void enqueue_decide(mulo_ctx* c, const DecideArgs& a, bool have_parts = false) {
    { PROF(MULO_PROF_ACCEPT);
      if (have_parts) launch_accept_from_parts(a, c->row_parts, (a.V + 127) / 128, c->st);
      else launch_accept(a, c->st); }
    { PROF(MULO_PROF_OTHER); launch_decide_finish(a, c->st); }
    { PROF(MULO_PROF_MASK_SAMPLE); launch_mask_sample(a, c->st); }
}

void fill_decide(DecideArgs& a, int vocab, float* rowmax, float* rowinv, int B, const mulo_step_params* p) {
    a.B = B; a.L = p->L; a.V = vocab;
    a.H = p->H; a.W = p->W; a.n0 = p->n0;
    a.rho = p->radius < 0 ? -1 : p->radius * p->expand;
    a.pool_k = p->pool_k < 1 ? 1 : p->pool_k;
    a.nbr = p->nbr;
    a.resample_mode = p->resample_mode;
    a.accept_mode = p->accept_mode;
    a.tau = p->tau;
    a.cfg_scale = p->cfg_scale;
    a.key0 = (uint32_t)(p->seed & 0xFFFFFFFFu);
    a.key1 = (uint32_t)(p->seed >> 32);
    a.ctr_lo = (uint32_t)(p->rng_counter & 0xFFFFFFFFu);
    a.ctr_hi24 = (uint32_t)((p->rng_counter >> 32) & 0xFFFFFFu);
    a.rowmax = rowmax;
    a.rowinv = rowinv;
}

}  // namespace

extern "C" {

const char* mulo_status_string(mulo_status s) {
    switch (s) {
        case MULO_OK: return "ok";
        case MULO_ERR_NULL: return "a required pointer is NULL";
        case MULO_ERR_SHAPE: return "inconsistent sizes";
        case MULO_ERR_RANGE: return "argument out of range";
        case MULO_ERR_ALLOC: return "device allocation failed";
        case MULO_ERR_HIP: return "HIP call or kernel launch failed";
        case MULO_ERR_UNSUPPORTED: return "configuration not supported by these kernels";
    }
    return "unknown status";
}

mulo_status mulo_check_model_cfg(const mulo_model_cfg* c) {
    if (!c) return MULO_ERR_NULL;
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->head_dim < 2 || c->d_ffn < 1 ||
        c->vocab < 4 || c->max_batch < 1 || c->max_seq < 1 || c->max_block < 1 || !(c->rms_eps >= 0.f))
        return MULO_ERR_RANGE;
    if (c->dtype != MULO_F32 && c->dtype != MULO_BF16) return MULO_ERR_RANGE;
    if ((int64_t)c->n_heads * c->head_dim != c->d_model || (c->head_dim & 1)) return MULO_ERR_SHAPE;
    if (c->max_block > c->max_seq) return MULO_ERR_SHAPE;
    if ((c->vocab & 3) || c->vocab > 262144) return MULO_ERR_UNSUPPORTED;
    if ((int64_t)c->max_batch * c->max_block > (1 << 22)) return MULO_ERR_UNSUPPORTED;
    if (c->stream_copy != 0 && c->stream_copy != 1) return MULO_ERR_RANGE;
    if (c->stream_copy && c->dtype != MULO_BF16) return MULO_ERR_UNSUPPORTED;
    if (c->dtype == MULO_BF16) {
        if (c->head_dim != 64 && c->head_dim != 128) return MULO_ERR_UNSUPPORTED;
        if ((c->d_model % 128) || (c->d_ffn % 64) || c->d_ffn < 128 || (c->max_seq % 8) || (c->max_block % 4))
            return MULO_ERR_UNSUPPORTED;
    } else {
        if (c->max_seq + c->head_dim > 15000) return MULO_ERR_UNSUPPORTED;  // scores of a row live in LDS
    }
    return MULO_OK;
}

namespace {
mulo_status check_step_params_raw(int vocab, int max_batch, int max_block, int32_t B, const mulo_step_params* p);
}

mulo_status mulo_check_step_params(const mulo_model_cfg* c, int32_t B, const mulo_step_params* p) {
    if (!c || !p) return MULO_ERR_NULL;
    return check_step_params_raw(c->vocab, c->max_batch, c->max_block, B, p);
}

namespace {
mulo_status check_step_params_raw(int vocab, int max_batch, int max_block, int32_t B, const mulo_step_params* p) {
    if (B < 1 || p->H < 1 || p->W < 1 || p->L < 1 || p->n0 < 0 || p->radius < -1 || p->expand < 0 ||
        p->pool_k < 1 || p->resample_mode < 0 || p->resample_mode > 2 ||
        (p->accept_mode != MULO_ACCEPT_RATIO && p->accept_mode != MULO_ACCEPT_TAU) ||
        (p->accept_mode == MULO_ACCEPT_TAU && !(p->tau >= 0.f && p->tau <= 3.0e38f)) ||
        !(p->cfg_scale >= 0.f && p->cfg_scale <= 1.0e6f))
        return MULO_ERR_RANGE;
    if ((int64_t)p->radius * p->expand > 4096) return MULO_ERR_RANGE;
    if ((p->cfg_scale > 0.f ? 2 * (int64_t)B : (int64_t)B) > max_batch || p->L > max_block) return MULO_ERR_SHAPE;
    if (p->L > 131072) return MULO_ERR_UNSUPPORTED;   // the accept flags of a block are staged in LDS
    if (p->L % p->W || p->n0 % p->W || (int64_t)p->n0 + p->L > (int64_t)p->H * p->W) return MULO_ERR_SHAPE;
    if (p->pool_k > 1 && !p->nbr) return MULO_ERR_NULL;
    if (p->pool_k > vocab) return MULO_ERR_RANGE;
    return MULO_OK;
}
}  // namespace

uint64_t mulo_workspace_bytes(const mulo_model_cfg* cfg) {
    if (mulo_check_model_cfg(cfg) != MULO_OK) return 0;
    return plan(*cfg).total;
}

mulo_status mulo_create(const mulo_model_cfg* cfg, const mulo_weights* w, void* hip_stream, mulo_ctx** out) {
    if (!cfg || !w || !out) return MULO_ERR_NULL;
    const mulo_status s = mulo_check_model_cfg(cfg);
    if (s != MULO_OK) return s;
    if (!w->embed || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->ffn_norm || !w->w_gate ||
        !w->w_up || !w->w_down || !w->final_norm || !w->lm_head || !w->rope_cos || !w->rope_sin)
        return MULO_ERR_NULL;
    int ndev = 0;
    if (!hip_ok(hipGetDeviceCount(&ndev)) || ndev < 1) return MULO_ERR_HIP;
    mulo_ctx* c = new (std::nothrow) mulo_ctx();
    if (!c) return MULO_ERR_ALLOC;
    c->cfg = *cfg;
    c->w = *w;
    c->st = (hipStream_t)hip_stream;
    c->maxM = (int64_t)cfg->max_batch * cfg->max_block;
    c->esz = cfg->dtype == MULO_BF16 ? 2 : 4;
    const Layout l = plan(*cfg);
    if (!hip_ok(hipMalloc(&c->base, l.total))) {
        (void)hipGetLastError();
        delete c;
        return MULO_ERR_ALLOC;
    }
    char* b = (char*)c->base;
    c->x = (float*)(b + l.off[0]);
    c->xh = b + l.off[1];
    c->qbuf = b + l.off[2];
    c->att = b + l.off[3];
    c->hmid = b + l.off[4];
    c->tmp = (float*)(b + l.off[5]);
    c->logits = (float*)(b + l.off[6]);
    c->q_lo = (float*)(b + l.off[7]);
    c->rowmax = (float*)(b + l.off[8]);
    c->rowinv = (float*)(b + l.off[9]);
    c->inputs = (int32_t*)(b + l.off[10]);
    c->tokens_hi = (int32_t*)(b + l.off[11]);
    c->q_row = (int32_t*)(b + l.off[12]);
    c->attn_part = (float*)(b + l.off[13]);
    c->isl_pos = (int32_t*)(b + l.off[14]);
    c->isl_hide = (uint8_t*)(b + l.off[15]);
    c->row_parts = c->esz == 2 ? (float*)(b + l.off[16]) : nullptr;
    c->pk_wq = c->pk_wk = c->pk_wv = c->pk_wo = c->pk_gate = c->pk_up = c->pk_down = c->pk_lm = nullptr;
    c->ksums = cfg->stream_copy ? (float*)(b + l.off[18]) : nullptr;
    if (cfg->stream_copy) {   // bf16 (checked): the second copy of the weights, made once on the context's stream
        const int nl = cfg->n_layers, d = cfg->d_model, f = cfg->d_ffn;
        char* p = b + l.off[17];
        auto take = [&](const void* src, int layers, int rows, int K) {
            const char* at = p;
            launch_pack_weights(src, p, layers, rows, K, c->st);
            p += packed_weight_elems(layers, rows, K) * 2;
            return at;
        };
        c->pk_wq = take(w->wq, nl, d, d);
        c->pk_wk = take(w->wk, nl, d, d);
        c->pk_wv = take(w->wv, nl, d, d);
        c->pk_wo = take(w->wo, nl, d, d);
        c->pk_gate = take(w->w_gate, nl, f, d);
        c->pk_up = take(w->w_up, nl, f, d);
        c->pk_down = take(w->w_down, nl, d, f);
        c->pk_lm = take(w->lm_head, 1, cfg->vocab, d);
        if (check_launch() != MULO_OK) {
            (void)hipFree(c->base);
            delete c;
            return MULO_ERR_HIP;
        }
    }
    *out = c;
    return MULO_OK;
}

void mulo_destroy(mulo_ctx* ctx) {
    if (!ctx) return;
    (void)hipStreamSynchronize(ctx->st);
    for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
    (void)hipFree(ctx->base);
    delete ctx;
}

mulo_status mulo_workspace_read(mulo_ctx* ctx, int32_t which, void* dst, uint64_t bytes) {
    if (!ctx || !dst) return MULO_ERR_NULL;
    const uint64_t M = (uint64_t)ctx->maxM, d = ctx->cfg.d_model, f = ctx->cfg.d_ffn, e = ctx->esz;
    const void* src = nullptr;
    uint64_t cap = 0;
    switch (which) {
        case MULO_WS_RESIDUAL: src = ctx->x; cap = M * d * 4; break;
        case MULO_WS_NORMED: src = ctx->xh; cap = M * d * e; break;
        case MULO_WS_Q: src = ctx->qbuf; cap = M * d * e; break;
        case MULO_WS_ATTN: src = ctx->att; cap = M * d * e; break;
        case MULO_WS_FFN: src = ctx->hmid; cap = M * f * e; break;
        default: return MULO_ERR_RANGE;
    }
    if ((bytes & 15) || bytes > cap) return MULO_ERR_SHAPE;
    launch_copy_rows((const float*)src, (float*)dst, (int64_t)(bytes / 4), ctx->st);
    return check_launch();
}

mulo_status mulo_profile(mulo_ctx* ctx, int32_t enable) {
    if (!ctx) return MULO_ERR_NULL;
    if (enable && ctx->prof_ev.empty()) {
        ctx->prof_ev.resize(2 * PROF_MAX);
        ctx->prof_cls.resize(PROF_MAX);
        for (auto& e : ctx->prof_ev)
            if (!hip_ok(hipEventCreate(&e))) return MULO_ERR_HIP;
    }
    ctx->prof_on = enable != 0;
    ctx->prof_mask = (enable & 0x100) ? ((enable & 0xff) < MULO_PROF_N ? 1u << (enable & 0xff) : 0u) : 0xFFFFFFFFu;
    return MULO_OK;
}

mulo_status mulo_profile_read(mulo_ctx* ctx, float* ms, int32_t* launches) {
    if (!ctx || !ms || !launches) return MULO_ERR_NULL;
    for (int i = 0; i < MULO_PROF_N; ++i) { ms[i] = 0.f; launches[i] = 0; }
    if (!hip_ok(hipStreamSynchronize(ctx->st))) return MULO_ERR_HIP;
    for (int i = 0; i < ctx->prof_n; ++i) {
        float t = 0.f;
        if (!hip_ok(hipEventElapsedTime(&t, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]))) return MULO_ERR_HIP;
        ms[ctx->prof_cls[i]] += t;
        launches[ctx->prof_cls[i]] += 1;
    }
    ctx->prof_n = 0;
    return MULO_OK;
}

mulo_status mulo_upsample_draft(mulo_ctx* ctx, int32_t B, int32_t h, int32_t w, int32_t r, const float* draft,
                                int32_t input_is_probs, const int32_t* draft_tokens, int32_t* tokens_hi,
                                float* q_lo, int32_t* q_row, float* q_hi) {
    if (!ctx || !draft || !draft_tokens || !tokens_hi || !q_lo || !q_row) return MULO_ERR_NULL;
    if (B < 1 || h < 1 || w < 1 || r < 1) return MULO_ERR_RANGE;
    if ((int64_t)B * h * r * w * r > ((int64_t)1 << 30)) return MULO_ERR_RANGE;
    enqueue_upsample(ctx, B, h, w, r, draft, input_is_probs, draft_tokens, tokens_hi, q_lo, q_row, q_hi);
    return check_launch();
}

mulo_status mulo_verify_forward(mulo_ctx* ctx, mulo_kv* kv, int32_t B, int32_t L, int32_t P,
                                const int32_t* in_tokens, const void* in_embeds, float* logits) {
    const mulo_status s = check_forward_args(ctx, kv, B, L, P);
    if (s != MULO_OK) return s;
    if ((!in_tokens && !in_embeds) || !logits) return MULO_ERR_NULL;
    enqueue_forward(ctx, kv, B, L, P, in_tokens, in_embeds, logits);
    return check_launch();
}

mulo_status mulo_accept_local_resample(mulo_ctx* ctx, int32_t B, const mulo_step_params* p, const float* logits,
                                       const float* q, const int32_t* q_row, int64_t q_batch_stride,
                                       const int32_t* draft_tokens, int32_t* tokens_out, uint8_t* accept,
                                       uint8_t* mask, int32_t* t0, int32_t* stats, float* p_probs) {
    if (!ctx || !p || !logits || !draft_tokens || !tokens_out || !accept || !mask || !t0 || !stats)
        return MULO_ERR_NULL;
    const mulo_status s = mulo_check_step_params(&ctx->cfg, B, p);
    if (s != MULO_OK) return s;
    if (!q && !(p->accept_mode == MULO_ACCEPT_TAU && p->resample_mode == 2)) return MULO_ERR_NULL;
    if (q_batch_stride < 0) return MULO_ERR_RANGE;
    DecideArgs a{};
    fill_decide(a, ctx->cfg.vocab, ctx->rowmax, ctx->rowinv, B, p);
    a.logits = logits; a.q = q; a.q_row = q_row; a.q_batch_stride = q_batch_stride;
    a.logits_u = p->cfg_scale > 0.f ? logits + (int64_t)B * p->L * ctx->cfg.vocab : nullptr;
    a.draft_tokens = draft_tokens; a.tokens_out = tokens_out; a.accept = accept; a.mask = mask;
    a.t0 = t0; a.stats = stats; a.p_probs = p_probs;
    enqueue_decide(ctx, a);
    return check_launch();
}

mulo_status mulo_accept_local_resample_static(void* hip_stream, int32_t vocab, int32_t B, const mulo_step_params* p,
                                              const float* logits, const float* q, const int32_t* q_row,
                                              int64_t q_batch_stride, const int32_t* draft_tokens, int32_t* tokens_out,
                                              uint8_t* accept, uint8_t* mask, int32_t* t0, int32_t* stats,
                                              float* p_probs) {
    if (!p || !logits || !draft_tokens || !tokens_out || !accept || !mask || !t0 || !stats) return MULO_ERR_NULL;
    if (vocab < 4 || B < 1) return MULO_ERR_RANGE;
    if ((vocab & 3) || vocab > 262144) return MULO_ERR_UNSUPPORTED;
    const int64_t seqs = p->cfg_scale > 0.f ? 2 * (int64_t)B : (int64_t)B;
    const mulo_status s = check_step_params_raw(vocab, seqs > 0x7fffffff ? 0x7fffffff : (int)seqs, p->L, B, p);
    if (s != MULO_OK) return s;
    if ((int64_t)B * p->L > MULO_STATIC_MAX_ROWS) return MULO_ERR_SHAPE;   // the row statistics must fit the static scratch
    if (!q && !(p->accept_mode == MULO_ACCEPT_TAU && p->resample_mode == 2)) return MULO_ERR_NULL;
    if (q_batch_stride < 0) return MULO_ERR_RANGE;
    float* const sc = static_scratch();
    if (!sc) return MULO_ERR_HIP;
    DecideArgs a{};
    // both halves are written for every row by the accept kernel before the re-draw reads them: nothing of the
    // last call's contents is used, nothing needs clearing
    fill_decide(a, vocab, sc, sc + MULO_STATIC_MAX_ROWS, B, p);
    a.logits = logits; a.q = q; a.q_row = q_row; a.q_batch_stride = q_batch_stride;
    a.logits_u = p->cfg_scale > 0.f ? logits + (int64_t)B * p->L * vocab : nullptr;
    a.draft_tokens = draft_tokens; a.tokens_out = tokens_out; a.accept = accept; a.mask = mask;
    a.t0 = t0; a.stats = stats; a.p_probs = p_probs;
    hipStream_t st = (hipStream_t)hip_stream;
    launch_accept(a, st);
    launch_decide_finish(a, st);
    launch_mask_sample(a, st);
    return check_launch();
}

mulo_status mulo_verify_step(mulo_ctx* ctx, mulo_kv* kv, int32_t B, int32_t P, const mulo_step_params* p,
                             int32_t h_blk, int32_t w, int32_t r, const float* draft, int32_t input_is_probs,
                             const int32_t* draft_tokens, const int32_t* prev_tokens, int32_t* tokens_out,
                             uint8_t* accept, uint8_t* mask, int32_t* t0, int32_t* stats, int32_t* tokens_hi,
                             float* logits) {
    if (!ctx || !p || !draft_tokens || !prev_tokens || !tokens_out || !accept || !mask || !t0 || !stats)
        return MULO_ERR_NULL;
    mulo_status s = mulo_check_step_params(&ctx->cfg, B, p);
    if (s != MULO_OK) return s;
    const bool need_q = !(p->accept_mode == MULO_ACCEPT_TAU && p->resample_mode == 2);
    if (need_q && !draft) return MULO_ERR_NULL;
    if (h_blk < 1 || w < 1 || r < 1) return MULO_ERR_RANGE;
    if ((int64_t)h_blk * r * w * r != p->L || w * r != p->W) return MULO_ERR_SHAPE;
    const bool cfg_on = p->cfg_scale > 0.f;
    const int B2 = cfg_on ? 2 * B : B;      // guidance: the unconditional twins are sequences B .. 2B-1
    s = check_forward_args(ctx, kv, B2, p->L, P);
    if (s != MULO_OK) return s;

    const int L = p->L, V = ctx->cfg.vocab, n_lo = h_blk * w;
    hipStream_t st = ctx->st;
    int32_t* thi = tokens_hi ? tokens_hi : ctx->tokens_hi;
    float* lg = logits ? logits : ctx->logits;
    // Step 2, the tokens (the draft distributions follow the target pass, see below)
    enqueue_upsample(ctx, B, h_blk, w, r, nullptr, input_is_probs, draft_tokens, thi, ctx->q_lo, ctx->q_row, nullptr);
    // Step 3: inputs [prev, x~_0 .. x~_{L-2}] so that logit row j is p of draft position j
    { mulo_ctx* c = ctx; PROF(MULO_PROF_OTHER); launch_shift_inputs(prev_tokens, thi, ctx->inputs, B, L, st);
      if (cfg_on) launch_shift_inputs(prev_tokens, thi, ctx->inputs + (int64_t)B * L, B, L, st); }
    // the accept test needs only the softmax statistics of a logit row and the draft token's logit: when it is the
    // plain test (no pooling, no guidance) the lm-head's epilogue leaves the statistics and the rows are not re-read
    const bool plain = p->pool_k <= 1 && !cfg_on;
    const bool have_parts = enqueue_forward(ctx, kv, B2, L, P, ctx->inputs, nullptr, lg, nullptr, plain);
    // Step 2, the draft distributions q_lo: only the decision stage reads them, and run here they separate the
    // lm-head's writes of the logits from the re-draw's reads of them (both kernels measured faster in this order)
    if (need_q) { mulo_ctx* c = ctx; PROF(MULO_PROF_UPSAMPLE);
        if (input_is_probs) launch_copy_rows(draft, ctx->q_lo, (int64_t)B * n_lo * V, st);
        else launch_softmax_rows(draft, ctx->q_lo, (int64_t)B * n_lo, V, st); }
    // Steps 4-5 + residual re-draw
    DecideArgs a{};
    fill_decide(a, ctx->cfg.vocab, ctx->rowmax, ctx->rowinv, B, p);
    a.logits = lg; a.q = need_q ? ctx->q_lo : nullptr; a.q_row = ctx->q_row; a.q_batch_stride = (int64_t)n_lo * V;
    a.logits_u = cfg_on ? lg + (int64_t)B * L * V : nullptr;
    a.draft_tokens = thi; a.tokens_out = tokens_out; a.accept = accept; a.mask = mask;
    a.t0 = t0; a.stats = stats; a.p_probs = nullptr;
    if (need_q && r > 1 && L % (r * r) == 0) { a.up_r = r; a.up_w = w; }
    enqueue_decide(ctx, a, have_parts);
    return check_launch();
}

mulo_status mulo_resample_sequential(mulo_ctx* ctx, mulo_kv* kv, int32_t B, int32_t P, int32_t L, int32_t u_start,
                                     uint64_t seed, uint64_t rng_counter, const int32_t* prev_tokens,
                                     const uint8_t* mask, int32_t* tokens, float* logits) {
    if (!ctx || !prev_tokens || !mask || !tokens) return MULO_ERR_NULL;
    if (L < 1 || u_start < 0 || u_start > L) return MULO_ERR_RANGE;
    mulo_status s = check_forward_args(ctx, kv, B, 1, P + L - 1);
    if (s != MULO_OK) return s;
    if (P < 0) return MULO_ERR_RANGE;
    const int V = ctx->cfg.vocab;
    mulo_ctx* c = ctx;
    for (int u = u_start; u < L; ++u) {
        { PROF(MULO_PROF_OTHER); launch_seq_input(prev_tokens, tokens, ctx->inputs, B, L, u, ctx->st); }
        enqueue_forward(ctx, kv, B, 1, P + u, ctx->inputs, nullptr, ctx->logits);
        { PROF(MULO_PROF_MASK_SAMPLE); launch_seq_draw(ctx->logits, mask, tokens, B, L, V, u, seed, rng_counter, ctx->st); }
        if (logits) launch_copy_rows_strided(ctx->logits, logits + (int64_t)u * V, B, V, (int64_t)L * V, ctx->st);
    }
    return check_launch();
}

mulo_status mulo_resample_islands(mulo_ctx* ctx, mulo_kv* kv, int32_t B, int32_t P, int32_t L, int32_t n_passes,
                                  int32_t max_islands, uint64_t seed, uint64_t rng_counter, const int32_t* prev_tokens,
                                  const uint8_t* mask, const int32_t* rank, int32_t* tokens, float* logits,
                                  int32_t* overflow) {
    if (!ctx || !prev_tokens || !mask || !rank || !tokens) return MULO_ERR_NULL;
    if (L < 1 || P < 0 || n_passes < 0 || max_islands < 1) return MULO_ERR_RANGE;
    mulo_status s = check_forward_args(ctx, kv, B, 1, P + L - 1);
    if (s != MULO_OK) return s;
    if (ctx->cfg.dtype != MULO_BF16) return MULO_ERR_UNSUPPORTED;
    const int64_t slots = (int64_t)B * max_islands;
    if (slots > ctx->maxM || L > ctx->cfg.max_block) return MULO_ERR_SHAPE;   // the slots share the step's workspace
    const int V = ctx->cfg.vocab;
    mulo_ctx* c = ctx;
    const Scatter sc{ctx->isl_pos, ctx->isl_hide, P, L};
    for (int r = 0; r < n_passes; ++r) {
        { PROF(MULO_PROF_OTHER);
          launch_island_select(prev_tokens, tokens, mask, rank, ctx->isl_pos, ctx->inputs, ctx->isl_hide, overflow, B, L, P,
                               max_islands, r, ctx->st); }
        enqueue_forward(ctx, kv, B, max_islands, 0, ctx->inputs, nullptr, ctx->logits, &sc);
        { PROF(MULO_PROF_MASK_SAMPLE);
          launch_island_draw(ctx->logits, ctx->isl_pos, tokens, logits, B, L, V, P, max_islands, seed, rng_counter, ctx->st); }
    }
    return check_launch();
}

mulo_status mulo_rejection_islands(mulo_ctx* ctx, int32_t B, int32_t W, int32_t n0, int32_t L, const uint8_t* mask,
                                   int32_t* island, int32_t* rank, int32_t* counts) {
    if (!ctx || !mask || !island || !rank || !counts) return MULO_ERR_NULL;
    if (B < 1 || W < 1 || L < 1 || n0 < 0) return MULO_ERR_RANGE;
    if (L % W != 0 || n0 % W != 0) return MULO_ERR_SHAPE;
    if (L > 16384) return MULO_ERR_UNSUPPORTED;      // labels of a block live in LDS
    mulo_ctx* c = ctx;
    { PROF(MULO_PROF_OTHER); launch_islands(mask, island, rank, counts, B, W, n0, L, ctx->st); }
    return check_launch();
}

}  // extern "C"
