// Decision stage of the verification step: draft up-sampling (Sec. 3.2, Step 2),
// the speculative accept test (Sec. 3.1, Eq. 1 / Eq. 3), local expansion
// (Sec. 3.3, Eq. 6-7) and residual resampling (Sec. 3.1, Eq. 2).
//
// All of it is bound by HBM reads of [rows, V] float32 matrices: one workgroup of
// 256 lanes owns one row, keeps it in registers (V <= 16384) and reduces over the
// codebook with wavefront shuffles, so every logit is read from memory once in
// the accept pass and once more (with the draft row) only for marked positions.
#include "mulo_internal.h"
#include "row_parts.h"

namespace mulo {

namespace {

constexpr int TPB = 256;
constexpr int WAVES = TPB / 64;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float NEAR_TIE = 1e-4f;
constexpr int MAX_CHUNKS = 1024;  // 256 codebook entries per chunk -> V <= 262144

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
// inclusive prefix sum over the 64 lanes of a wavefront
__device__ __forceinline__ unsigned long long wave_scan_u64(unsigned long long v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        unsigned long long n = __shfl_up(v, o);
        if (lane >= o) v += n;
    }
    return v;
}

// Fixed-order block reductions (run-to-run deterministic).
__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) red[wv] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < WAVES; ++i) r = fmaxf(r, red[i]);
    return r;
}
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) red[wv] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < WAVES; ++i) r += red[i];
    return r;
}

// exp(z - m) with one hardware exp2; no contraction so every kernel that
// evaluates it gets the same bits.
__device__ __forceinline__ float expm(float z, float m) { return rowparts::expm(z, m); }
__device__ __forceinline__ float prob(float z, float m, float inv) {
    return __fmul_rn(expm(z, m), inv);
}

// Classifier-free guidance of a target logit: z_u + s (z_c - z_u), every operation rounded on its own so
// that all kernels reproduce the same bits; zu == nullptr (no guidance) returns the logit unchanged.
__device__ __forceinline__ float guide(float zc, float zu, float s) {
    return __fadd_rn(zu, __fmul_rn(s, __fsub_rn(zc, zu)));
}
struct Guided {
    const float* zc;   // row of conditional logits
    const float* zu;   // row of unconditional logits or nullptr
    float s;
    __device__ __forceinline__ float at(int i) const { return zu ? guide(zc[i], zu[i], s) : zc[i]; }
    __device__ __forceinline__ float4 at4(int i4) const {
        const float4 c = reinterpret_cast<const float4*>(zc)[i4];
        if (!zu) return c;
        const float4 u = reinterpret_cast<const float4*>(zu)[i4];
        return make_float4(guide(c.x, u.x, s), guide(c.y, u.y, s), guide(c.z, u.z, s), guide(c.w, u.w, s));
    }
};

// Philox4x32-10 (Salmon et al., SC'11), word 0 of the output block.
__device__ __forceinline__ uint32_t philox_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += W0; k1 += W1;
    }
    return c0;
}

// ---- a row of V floats held by one workgroup -------------------------------
// NV4 > 0: registers (V <= 1024 * NV4); NV4 == 0: re-read from memory (L2) per pass.
template <int NV4>
struct RowRegs {
    float4 v[NV4 > 0 ? NV4 : 1];
};

template <int NV4>
__device__ __forceinline__ void row_stats(const Guided src, int V, RowRegs<NV4>& rr,
                                          float* red, float& m, float& inv) {
    const int nv4 = V >> 2, tid = threadIdx.x;
    const float NEG = -__builtin_huge_valf();
    float mx = NEG;
    if constexpr (NV4 > 0) {
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            const int idx = i * TPB + tid;
            rr.v[i] = idx < nv4 ? src.at4(idx) : make_float4(NEG, NEG, NEG, NEG);
            mx = fmaxf(fmaxf(mx, fmaxf(rr.v[i].x, rr.v[i].y)), fmaxf(rr.v[i].z, rr.v[i].w));
        }
    } else {
        for (int idx = tid; idx < nv4; idx += TPB) {
            const float4 t = src.at4(idx);
            mx = fmaxf(fmaxf(mx, fmaxf(t.x, t.y)), fmaxf(t.z, t.w));
        }
    }
    m = block_max(mx, red);
    float s = 0.f;
    if constexpr (NV4 > 0) {
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            rr.v[i].x = expm(rr.v[i].x, m); rr.v[i].y = expm(rr.v[i].y, m);
            rr.v[i].z = expm(rr.v[i].z, m); rr.v[i].w = expm(rr.v[i].w, m);
            s += (rr.v[i].x + rr.v[i].y) + (rr.v[i].z + rr.v[i].w);
        }
    } else {
        for (int idx = tid; idx < nv4; idx += TPB) {
            const float4 t = src.at4(idx);
            s += (expm(t.x, m) + expm(t.y, m)) + (expm(t.z, m) + expm(t.w, m));
        }
    }
    s = block_sum(s, red);
    inv = 1.0f / s;
}

template <int NV4>
__device__ __forceinline__ void row_write_probs(const Guided src, float* __restrict__ dst,
                                                int V, const RowRegs<NV4>& rr, float m, float inv) {
    const int nv4 = V >> 2, tid = threadIdx.x;
    float4* d4 = reinterpret_cast<float4*>(dst);
    if constexpr (NV4 > 0) {
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            const int idx = i * TPB + tid;
            if (idx < nv4)
                d4[idx] = make_float4(__fmul_rn(rr.v[i].x, inv), __fmul_rn(rr.v[i].y, inv),
                                      __fmul_rn(rr.v[i].z, inv), __fmul_rn(rr.v[i].w, inv));
        }
    } else {
        for (int idx = tid; idx < nv4; idx += TPB) {
            const float4 t = src.at4(idx);
            d4[idx] = make_float4(prob(t.x, m, inv), prob(t.y, m, inv), prob(t.z, m, inv),
                                  prob(t.w, m, inv));
        }
    }
}

// ---- Step 2: softmax of the draft logits, one workgroup per low-res cell ----
template <int NV4>
__global__ __launch_bounds__(TPB) void k_softmax_rows(const float* __restrict__ in,
                                                      float* __restrict__ out, int V) {
    __shared__ float red[WAVES];
    const int64_t row = blockIdx.x;
    RowRegs<NV4> rr;
    float m, inv;
    const Guided src{in + row * V, nullptr, 1.f};
    row_stats<NV4>(src, V, rr, red, m, inv);
    row_write_probs<NV4>(src, out + row * V, V, rr, m, inv);
}

__global__ __launch_bounds__(TPB) void k_copy(const float4* __restrict__ in, float4* __restrict__ out,
                                              int64_t n4) {
    for (int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x; i < n4; i += (int64_t)gridDim.x * TPB)
        out[i] = in[i];
}

// dst[b, :] = src[b, :] for rows of V floats, destination rows dst_stride floats apart
__global__ __launch_bounds__(TPB) void k_copy_rows_strided(const float4* __restrict__ src, float* __restrict__ dst,
                                                           int nv4, int64_t dst_stride) {
    const int b = blockIdx.y;
    float4* d = reinterpret_cast<float4*>(dst + b * dst_stride);
    for (int i = blockIdx.x * TPB + threadIdx.x; i < nv4; i += gridDim.x * TPB) d[i] = src[(int64_t)b * nv4 + i];
}

// x~[b, (rI+a) W + rJ+c] = y~[b, I w + J];  q_row[u] = (i_u / r) w + j_u / r
__global__ __launch_bounds__(TPB) void k_upsample_tokens(const int32_t* __restrict__ lo,
                                                         int32_t* __restrict__ hi,
                                                         int32_t* __restrict__ q_row, int B, int h,
                                                         int w, int r) {
    const int W = w * r, T = h * r * W;
    const int64_t gid = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (gid >= (int64_t)B * T) return;
    const int b = gid / T, u = gid % T;
    const int par = ((u / W) / r) * w + (u % W) / r;
    hi[gid] = lo[(int64_t)b * h * w + par];
    if (b == 0) q_row[u] = par;
}

// q_hi[b, u, :] = q_lo[b, q_row[u], :]
__global__ __launch_bounds__(TPB) void k_gather_rows(const float* __restrict__ q_lo,
                                                     const int32_t* __restrict__ q_row,
                                                     float* __restrict__ q_hi, int n_lo, int n_hi,
                                                     int V) {
    const int u = blockIdx.x, b = blockIdx.y;
    const float4* s = reinterpret_cast<const float4*>(q_lo + ((int64_t)b * n_lo + q_row[u]) * V);
    float4* d = reinterpret_cast<float4*>(q_hi + ((int64_t)b * n_hi + u) * V);
    for (int i = threadIdx.x; i < (V >> 2); i += TPB) d[i] = s[i];
}

__global__ void k_shift_inputs(const int32_t* __restrict__ prev, const int32_t* __restrict__ hi,
                               int32_t* __restrict__ inp, int B, int L) {
    const int64_t gid = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (gid >= (int64_t)B * L) return;
    const int b = gid / L, j = gid % L;
    inp[gid] = j == 0 ? prev[b] : hi[gid - 1];
}

// ---- Step 4: softmax statistics + accept test, one workgroup per position ---
__device__ __forceinline__ int clamp_tok(int t, int V) { return t < 0 ? 0 : (t >= V ? V - 1 : t); }

// The accept test of one position, by one lane: Eq. 1 without the division (u q < pbar), or the threshold rule of
// Eq. 5 (pbar >= tau); leaves the row statistics for the re-draw kernel and parks the near-tie flag in the mask
// array until k_decide_finish has counted it (per-row atomics on the few counters of a sequence cost a quarter of
// the accept kernel's time).
__device__ __forceinline__ void accept_row(const DecideArgs& a, int64_t row, int b, int t, float qt, float pbar,
                                           float m, float inv) {
    const uint32_t w0 = philox_word0((uint32_t)t, (uint32_t)b, a.ctr_lo, a.ctr_hi24, a.key0, a.key1);
    const float u = (float)(w0 >> 8) * 5.9604644775390625e-08f;  // 2^-24, exact
    // the threshold rule is written as "tau' < pbar or equal" through the same comparison with uq := tau
    const bool tau_rule = a.accept_mode == 1;
    const float uq = tau_rule ? a.tau : __fmul_rn(u, qt);
    const bool ok = tau_rule ? pbar >= uq : uq < pbar;
    a.accept[row] = ok ? 1 : 0;
    a.rowmax[row] = m;
    a.rowinv[row] = inv;
    a.mask[row] = fabsf(__fsub_rn(pbar, uq)) < __fmul_rn(NEAR_TIE, tau_rule ? a.tau : qt) ? 1 : 0;
}

constexpr int MAX_PARTS = 2048;   // 128 codebook entries per part -> V <= 262144

// One workgroup per position.  The row is read once: lane `tid` of pass k owns run 256 k + tid (8 consecutive logits),
// so the 16 lanes of a part sit next to each other, the two halves of the part on the even and the odd lanes; the
// part statistics are formed with lane exchanges in the order row_parts.h fixes, left in LDS, and merged by the
// first wavefront.
__global__ __launch_bounds__(TPB) void k_accept(const DecideArgs a) {
    __shared__ float2 parts[MAX_PARTS];
    __shared__ float red[WAVES];
    __shared__ float2 s_stat;
    const int64_t row = blockIdx.x;
    const int b = row / a.L, t = row % a.L, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const Guided z{a.logits + row * a.V, a.logits_u ? a.logits_u + row * a.V : nullptr, a.cfg_scale};
    // the scalar gathers (draft token -> its logit and its draft probability) are issued first, so that
    // their chained latency is hidden behind the streaming of the row
    const int tok = clamp_tok(a.draft_tokens[row], a.V);
    float ztok = 0.f, qt = 0.f;
    if (tid == 0) {
        if (a.accept_mode == 0) {
            const int qr = a.q_row ? a.q_row[t] : t;
            qt = a.q[b * a.q_batch_stride + (int64_t)qr * a.V + tok];
        }
        ztok = z.at(tok);
    }
    const int V = a.V, n_parts = (V + rowparts::PART - 1) / rowparts::PART;
    const float NEG = rowparts::NEG_INF;
    for (int base = 0; base < n_parts * 16; base += TPB) {
        const int R = base + tid;                       // run of 8 logits; V is a multiple of 4
        const int n_valid = V - R * 8 >= 8 ? 8 : (V - R * 8 >= 4 ? 4 : 0);
        float zz[8];
        const float4 lo = n_valid >= 4 ? z.at4(2 * R) : make_float4(NEG, NEG, NEG, NEG);
        const float4 hi = n_valid >= 8 ? z.at4(2 * R + 1) : make_float4(NEG, NEG, NEG, NEG);
        zz[0] = lo.x; zz[1] = lo.y; zz[2] = lo.z; zz[3] = lo.w; zz[4] = hi.x; zz[5] = hi.y; zz[6] = hi.z; zz[7] = hi.w;
        float m = fmaxf(fmaxf(fmaxf(zz[0], zz[1]), fmaxf(zz[2], zz[3])), fmaxf(fmaxf(zz[4], zz[5]), fmaxf(zz[6], zz[7])));
        m = fmaxf(m, __shfl_xor(m, 2));                 // the 8 runs of a half: lanes 2 apart
        m = fmaxf(m, __shfl_xor(m, 4));
        m = fmaxf(m, __shfl_xor(m, 8));
        float s = rowparts::run_sum(zz, m, n_valid);
        s = __fadd_rn(s, __shfl_xor(s, 2));             // ((t0+t1)+(t2+t3))+((t4+t5)+(t6+t7))
        s = __fadd_rn(s, __shfl_xor(s, 4));
        s = __fadd_rn(s, __shfl_xor(s, 8));
        const float2 ps = rowparts::merge_halves(m, s, __shfl_xor(m, 1), __shfl_xor(s, 1));
        if ((tid & 15) == 0 && (R >> 4) < n_parts) parts[R >> 4] = ps;
    }
    __syncthreads();
    if (wv == 0) {
        const float2 st = rowparts::combine_parts(parts, n_parts, lane);
        if (lane == 0) s_stat = st;
    }
    __syncthreads();
    const float m = s_stat.x, inv = 1.0f / s_stat.y;
    if (a.p_probs) {
        RowRegs<0> none;
        row_write_probs<0>(z, a.p_probs + row * a.V, a.V, none, m, inv);
    }
    float pbar;
    if (a.pool_k <= 1) {
        pbar = prob(ztok, m, inv);
    } else {  // Eq. 3: pooled mass over the codebook neighbours of the draft token
        float acc = 0.f;
        for (int i = tid; i < a.pool_k; i += TPB)
            acc += prob(z.at(clamp_tok(a.nbr[(int64_t)tok * a.pool_k + i], a.V)), m, inv);
        pbar = block_sum(acc, red);
    }
    if (tid == 0) accept_row(a, row, b, t, qt, pbar, m, inv);
}

// The same test when the lm-head GEMM has already left the parts of every row (a verification step): one
// wavefront per position merges them and gathers the draft token's logit; the row of logits is not read again.
__global__ __launch_bounds__(TPB) void k_accept_parts(const DecideArgs a, const float2* __restrict__ parts, int n_parts) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * WAVES + wv;
    if (row >= (int64_t)a.B * a.L) return;            // uniform over the wavefront
    const int b = row / a.L, t = row % a.L;
    const int tok = clamp_tok(a.draft_tokens[row], a.V);
    float ztok = 0.f, qt = 0.f;
    if (lane == 0) {
        if (a.accept_mode == 0) {
            const int qr = a.q_row ? a.q_row[t] : t;
            qt = a.q[b * a.q_batch_stride + (int64_t)qr * a.V + tok];
        }
        ztok = a.logits[row * a.V + tok];
    }
    const float2 st = rowparts::combine_parts(parts + row * n_parts, n_parts, lane);
    if (lane == 0) {
        const float m = st.x, inv = 1.0f / st.y;
        accept_row(a, row, b, t, qt, prob(ztok, m, inv), m, inv);
    }
}

// ---- Step 5 (Eq. 6-7) + the step's counters, one workgroup per sequence ----
// From the accept flags of the block (staged in LDS): t0 = first rejected position, the counts of accepted /
// rejected positions and near ties, then R_X: position t is marked when it is at or after t0 and within Chebyshev
// distance rho of some rejected position of the block (rho < 0: the raster rule, everything from t0 on).  Writes
// mask, t0 and stats = (accepted, rejected, marked, near ties); no atomics on global memory anywhere.
__global__ __launch_bounds__(TPB) void k_decide_finish(const DecideArgs a) {
    extern __shared__ uint8_t acc_s[];   // [L]
    __shared__ int red[WAVES][4];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint8_t* acc_g = a.accept + (int64_t)b * a.L;
    uint8_t* mask_g = a.mask + (int64_t)b * a.L;
    int n_acc = 0, n_near = 0, tmin = a.L;
    for (int t = tid; t < a.L; t += TPB) {
        const uint8_t ok = acc_g[t];
        acc_s[t] = ok;
        n_acc += ok;
        n_near += mask_g[t];
        if (!ok && t < tmin) tmin = t;
    }
    auto reduce_counts = [&](int& x, int& y, int& z_min, int& w) {   // sums of x, y, w and the minimum of z_min over the workgroup
        for (int o = 32; o > 0; o >>= 1) {
            x += __shfl_xor(x, o);
            y += __shfl_xor(y, o);
            w += __shfl_xor(w, o);
            const int other = __shfl_xor(z_min, o);
            z_min = other < z_min ? other : z_min;
        }
        __syncthreads();
        if (lane == 0) { red[wv][0] = x; red[wv][1] = y; red[wv][2] = z_min; red[wv][3] = w; }
        __syncthreads();
        x = y = w = 0;
        z_min = a.L;
        for (int i = 0; i < WAVES; ++i) {
            x += red[i][0]; y += red[i][1]; w += red[i][3];
            z_min = red[i][2] < z_min ? red[i][2] : z_min;
        }
    };
    int zero = 0;
    reduce_counts(n_acc, n_near, tmin, zero);   // the barriers inside also publish acc_s and retire the reads of mask_g
    const int t0 = tmin;
    int n_marked = 0;
    for (int t = tid; t < a.L; t += TPB) {
        int marked = 0;
        if (t >= t0) {
            if (a.rho < 0) {
                marked = 1;
            } else {
                // the window, cut to the rows of the block (whole rows of the grid) and to the grid's columns
                const int g = a.n0 + t, gi = g / a.W, gj = g % a.W, r0 = a.n0 / a.W, r1 = (a.n0 + a.L - 1) / a.W;
                const int i_lo = gi - a.rho > r0 ? gi - a.rho : r0, i_hi = gi + a.rho < r1 ? gi + a.rho : r1;
                const int j_lo = gj - a.rho > 0 ? gj - a.rho : 0, j_hi = gj + a.rho < a.W - 1 ? gj + a.rho : a.W - 1;
                for (int ii = i_lo; ii <= i_hi && !marked; ++ii)
                    for (int jj = j_lo; jj <= j_hi; ++jj)
                        if (acc_s[ii * a.W + jj - a.n0] == 0) { marked = 1; break; }
            }
        }
        mask_g[t] = (uint8_t)marked;
        n_marked += marked;
    }
    int d0 = 0, d1 = a.L;
    reduce_counts(n_marked, d0, d1, zero);
    if (tid == 0) {
        a.t0[b] = t0;
        a.stats[b * 4 + 0] = n_acc;
        a.stats[b * 4 + 1] = a.L - n_acc;
        a.stats[b * 4 + 2] = n_marked;
        a.stats[b * 4 + 3] = n_near;
    }
}

// ---- Step 5 + Eq. 2: neighbourhood mask, then the residual draw -------------
__device__ __forceinline__ void weights4(const float4 z, const float4 qv, float m, float inv, bool use_p,
                                         unsigned long long w[4]) {
    const float S = 1099511627776.0f;  // 2^40: w * S is exact in float32
    float p0 = prob(z.x, m, inv), p1 = prob(z.y, m, inv), p2 = prob(z.z, m, inv), p3 = prob(z.w, m, inv);
    if (!use_p) {
        p0 = fmaxf(0.f, __fsub_rn(p0, qv.x)); p1 = fmaxf(0.f, __fsub_rn(p1, qv.y));
        p2 = fmaxf(0.f, __fsub_rn(p2, qv.z)); p3 = fmaxf(0.f, __fsub_rn(p3, qv.w));
    }
    w[0] = (unsigned long long)__fmul_rn(p0, S); w[1] = (unsigned long long)__fmul_rn(p1, S);
    w[2] = (unsigned long long)__fmul_rn(p2, S); w[3] = (unsigned long long)__fmul_rn(p3, S);
}

// Chunk sums of the integer weights of a row (pass 1 of the draw): chunk c covers the 256 codebook entries
// [256 c, 256 c + 256) = 64 lanes x 4 entries.  G float4 per lane are requested together (both rows), and their G
// wavefront sums run side by side, so that neither the memory latency nor the latency of a lane exchange is paid
// once per chunk.  GUIDED: the logits are z_u + s (z_c - z_u); USE_Q: residual weights max(0, p - q), else p.
template <int G, bool GUIDED, bool USE_Q>
__device__ __forceinline__ void chunk_sums(const Guided z, const float4* __restrict__ q4, float m, float inv, int nv4,
                                           int nchunks, unsigned long long* chunk) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float4* zc4 = reinterpret_cast<const float4*>(z.zc);
    const float4* zu4 = reinterpret_cast<const float4*>(z.zu);
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int base = 0; base < nv4; base += TPB * G) {
        float4 zc[G], zu[G], qv[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {       // rows past the end re-read entry 0 and are not counted
            const int idx = base + g * TPB + tid, ci = idx < nv4 ? idx : 0;
            zc[g] = zc4[ci];
            if constexpr (GUIDED) zu[g] = zu4[ci];
            if constexpr (USE_Q) qv[g] = q4[ci];
        }
        unsigned long long sm[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int idx = base + g * TPB + tid;
            float4 zz = zc[g];
            if constexpr (GUIDED)
                zz = make_float4(guide(zz.x, zu[g].x, z.s), guide(zz.y, zu[g].y, z.s), guide(zz.z, zu[g].z, z.s),
                                 guide(zz.w, zu[g].w, z.s));
            unsigned long long w[4];
            weights4(zz, USE_Q ? qv[g] : zero4, m, inv, !USE_Q, w);
            sm[g] = idx < nv4 ? (w[0] + w[1]) + (w[2] + w[3]) : 0ull;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1)
#pragma unroll
            for (int g = 0; g < G; ++g) sm[g] += __shfl_xor(sm[g], o);
        if (lane == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int c = (base >> 6) + g * WAVES + wv;
                if (c < nchunks) chunk[c] = sm[g];
            }
        }
    }
}

// Integer-CDF draw of one row by one workgroup: W(x) = floor(w(x) 2^40) with w = max(0, p - q) (or p when
// use_p), T = (word * tot) >> 32, token = first x whose inclusive prefix exceeds T; an empty residual falls
// back to p.  The token is stored to *out by the lane that finds it.
__device__ __forceinline__ void cdf_draw(const Guided z, const float4* __restrict__ q4, float m,
                                         float inv, bool use_p, uint32_t word, int V, int fallback_tok,
                                         int32_t* out, unsigned long long* chunk, int* s_retry) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int nv4 = V >> 2, nchunks = (nv4 + 63) >> 6;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int attempt = 0; attempt < 2; ++attempt) {
        if (z.zu) {
            if (use_p) chunk_sums<2, true, false>(z, q4, m, inv, nv4, nchunks, chunk);
            else chunk_sums<2, true, true>(z, q4, m, inv, nv4, nchunks, chunk);
        } else {
            if (use_p) chunk_sums<4, false, false>(z, q4, m, inv, nv4, nchunks, chunk);
            else chunk_sums<4, false, true>(z, q4, m, inv, nv4, nchunks, chunk);
        }
        if (tid == 0) *s_retry = 0;
        __syncthreads();
        if (wv == 0) {
            unsigned long long tot = 0;
            for (int c0 = 0; c0 < nchunks; c0 += 64) tot += (c0 + lane < nchunks) ? chunk[c0 + lane] : 0ull;
            tot = wave_sum_u64(tot);
            if (tot == 0) {
                if (lane == 0) *s_retry = 1;  // empty residual: draw from p instead
            } else {
                const unsigned long long T = __umul64hi((unsigned long long)word << 32, tot);
                unsigned long long run = 0, before = 0;
                int cidx = nchunks - 1;
                for (int c0 = 0; c0 < nchunks; c0 += 64) {
                    const unsigned long long v = (c0 + lane < nchunks) ? chunk[c0 + lane] : 0ull;
                    const unsigned long long incl = wave_scan_u64(v, lane) + run;
                    const unsigned long long hit = __ballot(incl > T);
                    if (hit) {
                        const int f = __ffsll((long long)hit) - 1;
                        cidx = c0 + f;
                        before = __shfl(incl - v, f);
                        break;
                    }
                    run = __shfl(incl, 63);
                }
                // inside the chunk: 64 lanes x 4 entries, same weights as above
                const int idx = cidx * 64 + lane;
                unsigned long long w[4] = {0, 0, 0, 0};
                if (idx < nv4) weights4(z.at4(idx), use_p ? zero4 : q4[idx], m, inv, use_p, w);
                const unsigned long long s = (w[0] + w[1]) + (w[2] + w[3]);
                const unsigned long long incl = wave_scan_u64(s, lane) + before;
                const unsigned long long hit = __ballot(incl > T);
                const int f = hit ? __ffsll((long long)hit) - 1 : 63;
                if (lane == f) {
                    unsigned long long cum = incl - s;
                    int tok = fallback_tok;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        cum += w[e];
                        if (cum > T) { tok = idx * 4 + e; break; }
                    }
                    *out = clamp_tok(tok, V);
                }
            }
        }
        __syncthreads();
        if (!*s_retry || use_p) break;
        use_p = true;
        __syncthreads();
    }
}

__global__ __launch_bounds__(TPB) void k_mask_sample(const DecideArgs a) {
    __shared__ unsigned long long chunk[MAX_CHUNKS];
    __shared__ int s_retry;
    // Which position this workgroup handles.  Workgroup ids go round-robin over the 8 XCDs (each with its own L2).
    // When the draft rows are shared by r x r children (replication up-sampling), the children of a draft row are
    // given to consecutive workgroups of ONE XCD, so that the row comes from memory once instead of once per child.
    int64_t row = blockIdx.x;
    if (a.up_r > 1) {
        const int r2 = a.up_r * a.up_r, n_par = a.L / r2;
        const int x = blockIdx.x & 7, k = blockIdx.x >> 3;
        const int64_t pseq = (int64_t)(k / r2) * 8 + x;
        if (pseq >= (int64_t)a.B * n_par) return;      // uniform over the workgroup (the grid is rounded up)
        const int child = k % r2, bb = pseq / n_par, par = pseq % n_par;
        const int I = par / a.up_w, J = par % a.up_w, W = a.up_r * a.up_w;
        row = (int64_t)bb * a.L + (a.up_r * I + child / a.up_r) * W + a.up_r * J + child % a.up_r;
    }
    const int b = row / a.L, t = row % a.L, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;

    // R_X membership of this position (Eq. 6-7) was decided by k_decide_finish
    const int marked = a.mask[row];
    const int draft = clamp_tok(a.draft_tokens[row], a.V);
    if (!marked) {   // uniform over the workgroup
        if (tid == 0) a.tokens_out[row] = draft;
        return;
    }
    // Residual draw through the integer CDF
    const int V = a.V;
    const Guided z{a.logits + row * V, a.logits_u ? a.logits_u + row * V : nullptr, a.cfg_scale};
    const int qr = a.q_row ? a.q_row[t] : t;
    const bool use_p = a.resample_mode == 2 || ((a.resample_mode == 1) && a.accept[row] != 0);
    // the draft row is read only for residual weights (it may be absent when every draw is from p)
    const float4* q4 = reinterpret_cast<const float4*>(a.q ? a.q + b * a.q_batch_stride + (int64_t)qr * V : z.zc);
    const uint32_t word = philox_word0((uint32_t)t, (uint32_t)b, a.ctr_lo, a.ctr_hi24 | (1u << 24),
                                       a.key0, a.key1);
    cdf_draw(z, q4, a.rowmax[row], a.rowinv[row], use_p, word, V, draft, &a.tokens_out[row], chunk, &s_retry);
}

// ---- Alg. 1 Step 6, one position: inputs of the single-token forward, then the draw from p ----
__global__ void k_seq_input(const int32_t* __restrict__ prev, const int32_t* __restrict__ tokens,
                            int32_t* __restrict__ inp, int B, int L, int u) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) inp[b] = u == 0 ? prev[b] : tokens[(int64_t)b * L + u - 1];
}

// one workgroup per sequence: if position u is marked, tokens[b, u] ~ softmax(logits[b, :])
__global__ __launch_bounds__(TPB) void k_seq_draw(const float* __restrict__ logits, const uint8_t* __restrict__ mask,
                                                  int32_t* __restrict__ tokens, int L, int V, int u, uint32_t key0,
                                                  uint32_t key1, uint32_t ctr_lo, uint32_t ctr_hi24) {
    __shared__ unsigned long long chunk[MAX_CHUNKS];
    __shared__ int s_retry;
    __shared__ float red[WAVES];
    const int b = blockIdx.x;
    if (!mask[(int64_t)b * L + u]) return;   // uniform over the workgroup
    const Guided z{logits + (int64_t)b * V, nullptr, 1.f};
    RowRegs<0> none;
    float m, inv;
    row_stats<0>(z, V, none, red, m, inv);
    const uint32_t word = philox_word0((uint32_t)u, (uint32_t)b, ctr_lo, ctr_hi24 | (2u << 24), key0, key1);
    int32_t* out = tokens + (int64_t)b * L + u;
    cdf_draw(z, reinterpret_cast<const float4*>(z.zc), m, inv, true, word, V, *out, out, chunk, &s_retry);
}

// ---- island-parallel re-sampling (Sec. 3.4): one pass handles the rank-`pass` position of every island ----
// One workgroup per sequence.  All threads write the pass's hidden set (marked positions whose rank is >= pass:
// not re-drawn yet); the first wavefront then deals the positions of rank == pass to the sequence's `cap` slots in
// raster order (ballot + prefix count, so the slot of a position does not depend on timing): its cache row, and
// its input token = the current token of the position before it.  Unused slots get row -1.
__global__ __launch_bounds__(TPB) void k_island_select(const int32_t* __restrict__ prev, const int32_t* __restrict__ tokens,
                                                       const uint8_t* __restrict__ mask, const int32_t* __restrict__ rank,
                                                       int32_t* __restrict__ pos_tab, int32_t* __restrict__ inp,
                                                       uint8_t* __restrict__ hide, int32_t* __restrict__ overflow, int L,
                                                       int P, int cap, int pass) {
    const int b = blockIdx.x, tid = threadIdx.x;
    const uint8_t* mk = mask + (int64_t)b * L;
    const int32_t* rk = rank + (int64_t)b * L;
    for (int t = tid; t < L; t += TPB) hide[(int64_t)b * L + t] = mk[t] && rk[t] >= pass;
    if (tid >= 64) return;
    int cnt = 0;
    for (int base = 0; base < L; base += 64) {
        const int t = base + tid;
        const bool sel = t < L && mk[t] && rk[t] == pass;
        const unsigned long long bal = __ballot(sel);
        const int slot = cnt + __popcll(bal & ((1ull << tid) - 1ull));
        if (sel && slot < cap) {
            pos_tab[b * cap + slot] = P + t;
            inp[b * cap + slot] = t == 0 ? prev[b] : tokens[(int64_t)b * L + t - 1];
        }
        cnt += __popcll(bal);
    }
    for (int slot = cnt + tid; slot < cap; slot += 64) {
        pos_tab[b * cap + slot] = -1;
        inp[b * cap + slot] = 0;
    }
    if (tid == 0 && cnt > cap && overflow) atomicAdd(overflow, cnt - cap);   // the caller's bound was too small
}

// one workgroup per slot: tokens[sequence, u] ~ softmax(logits[slot, :]) for the position u the slot holds
__global__ __launch_bounds__(TPB) void k_island_draw(const float* __restrict__ logits, const int32_t* __restrict__ pos_tab,
                                                     int32_t* __restrict__ tokens, float* __restrict__ logits_out, int L,
                                                     int V, int P, int cap, uint32_t key0, uint32_t key1, uint32_t ctr_lo,
                                                     uint32_t ctr_hi24) {
    __shared__ unsigned long long chunk[MAX_CHUNKS];
    __shared__ int s_retry;
    __shared__ float red[WAVES];
    const int v = blockIdx.x, b = v / cap, row = pos_tab[v];
    if (row < 0) return;   // uniform over the workgroup
    const int u = row - P;
    const Guided z{logits + (int64_t)v * V, nullptr, 1.f};
    if (logits_out)
        for (int c = threadIdx.x; c < V; c += TPB) logits_out[((int64_t)b * L + u) * V + c] = z.zc[c];
    RowRegs<0> none;
    float m, inv;
    row_stats<0>(z, V, none, red, m, inv);
    const uint32_t word = philox_word0((uint32_t)u, (uint32_t)b, ctr_lo, ctr_hi24 | (2u << 24), key0, key1);
    int32_t* out = tokens + (int64_t)b * L + u;
    cdf_draw(z, reinterpret_cast<const float4*>(z.zc), m, inv, true, word, V, *out, out, chunk, &s_retry);
}

// ---- rejection islands (Eq. 8): 8-connected components of the marked set, one workgroup per sequence ----
// Labels live in LDS (one int per block position: 0 = unmarked, else 1 + a member's position).  Every round
// a marked position takes the smallest label among itself and its 8 grid neighbours and then jumps to the
// label of the position that label names (pointer jumping), until a round changes nothing: each island ends
// with 1 + its smallest position.  The rank of a position is the number of members of its island before it.
__global__ __launch_bounds__(TPB) void k_islands(const uint8_t* __restrict__ mask, int32_t* __restrict__ island,
                                                 int32_t* __restrict__ rank, int32_t* __restrict__ counts, int W,
                                                 int n0, int L) {
    extern __shared__ int lab[];
    const int b = blockIdx.x, tid = threadIdx.x;
    const uint8_t* mk = mask + (int64_t)b * L;
    for (int t = tid; t < L; t += TPB) lab[t] = mk[t] ? t + 1 : 0;
    __syncthreads();
    while (true) {
        int changed = 0;
        for (int t = tid; t < L; t += TPB) {
            int cur = lab[t];
            if (!cur) continue;
            const int g = n0 + t, i = g / W, j = g % W;
            int best = cur;
#pragma unroll
            for (int di = -1; di <= 1; ++di)
#pragma unroll
                for (int dj = -1; dj <= 1; ++dj) {
                    const int jj = j + dj, u = (i + di) * W + jj - n0;
                    if (jj >= 0 && jj < W && u >= 0 && u < L) {
                        const int v = lab[u];
                        if (v && v < best) best = v;
                    }
                }
            const int hop = lab[best - 1];       // the named position is marked, so its label is > 0
            if (hop < best) best = hop;
            if (best < cur) { atomicMin(&lab[t], best); changed = 1; }
        }
        if (!__syncthreads_or(changed)) break;
    }
    int n_isl = 0, largest = 0;
    for (int t = tid; t < L; t += TPB) {
        const int l = lab[t];
        int r = -1;
        if (l) {
            r = 0;
            for (int u = l - 1; u < t; ++u) r += lab[u] == l;
            if (l == t + 1) {                     // the island's first member counts the island and measures it
                ++n_isl;
                int sz = 0;
                for (int u = t; u < L; ++u) sz += lab[u] == l;
                largest = sz > largest ? sz : largest;
            }
        }
        island[(int64_t)b * L + t] = l;
        rank[(int64_t)b * L + t] = r;
    }
    __shared__ int red_n, red_m;
    if (tid == 0) { red_n = 0; red_m = 0; }
    __syncthreads();
    if (n_isl) atomicAdd(&red_n, n_isl);
    if (largest) atomicMax(&red_m, largest);
    __syncthreads();
    if (tid == 0) { counts[b * 2] = red_n; counts[b * 2 + 1] = red_m; }
}

template <int NV4>
void softmax_rows_inst(const float* in, float* out, int64_t rows, int V, hipStream_t st) {
    hipLaunchKernelGGL(k_softmax_rows<NV4>, dim3((unsigned)rows), dim3(TPB), 0, st, in, out, V);
}
}  // namespace

void launch_softmax_rows(const float* in, float* out, int64_t rows, int V, hipStream_t st) {
    if (rows <= 0) return;
    if (V <= 1024) softmax_rows_inst<1>(in, out, rows, V, st);
    else if (V <= 2048) softmax_rows_inst<2>(in, out, rows, V, st);
    else if (V <= 4096) softmax_rows_inst<4>(in, out, rows, V, st);
    else if (V <= 8192) softmax_rows_inst<8>(in, out, rows, V, st);
    else if (V <= 16384) softmax_rows_inst<16>(in, out, rows, V, st);
    else softmax_rows_inst<0>(in, out, rows, V, st);
}

void launch_copy_rows(const float* in, float* out, int64_t n_floats, hipStream_t st) {
    if (n_floats <= 0 || in == out) return;
    const int64_t n4 = n_floats >> 2;
    const unsigned blocks = (unsigned)((n4 + TPB - 1) / TPB < 65536 ? (n4 + TPB - 1) / TPB : 65536);
    hipLaunchKernelGGL(k_copy, dim3(blocks), dim3(TPB), 0, st, reinterpret_cast<const float4*>(in),
                       reinterpret_cast<float4*>(out), n4);
}

void launch_copy_rows_strided(const float* src, float* dst, int B, int V, int64_t dst_stride, hipStream_t st) {
    if (B <= 0 || V <= 0) return;
    const int nv4 = V >> 2;
    hipLaunchKernelGGL(k_copy_rows_strided, dim3((nv4 + TPB - 1) / TPB < 64 ? (nv4 + TPB - 1) / TPB : 64, B), dim3(TPB), 0, st,
                       reinterpret_cast<const float4*>(src), dst, nv4, dst_stride);
}

void launch_upsample_tokens(const int32_t* draft_tokens, int32_t* tokens_hi, int32_t* q_row, int B,
                            int h, int w, int r, hipStream_t st) {
    const int64_t n = (int64_t)B * h * r * w * r;
    hipLaunchKernelGGL(k_upsample_tokens, dim3((unsigned)((n + TPB - 1) / TPB)), dim3(TPB), 0, st,
                       draft_tokens, tokens_hi, q_row, B, h, w, r);
}

void launch_gather_rows(const float* q_lo, const int32_t* q_row, float* q_hi, int B, int n_lo,
                        int n_hi, int V, hipStream_t st) {
    hipLaunchKernelGGL(k_gather_rows, dim3(n_hi, B), dim3(TPB), 0, st, q_lo, q_row, q_hi, n_lo, n_hi, V);
}

void launch_shift_inputs(const int32_t* prev, const int32_t* tokens_hi, int32_t* inputs, int B,
                         int L, hipStream_t st) {
    const int64_t n = (int64_t)B * L;
    hipLaunchKernelGGL(k_shift_inputs, dim3((unsigned)((n + TPB - 1) / TPB)), dim3(TPB), 0, st, prev,
                       tokens_hi, inputs, B, L);
}

void launch_islands(const uint8_t* mask, int32_t* island, int32_t* rank, int32_t* counts, int B, int W, int n0, int L,
                    hipStream_t st) {   // L <= 16384 (the caller checks): one label per position in LDS
    static int attr_state = 0;
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(k_islands), 16384 * (int)sizeof(int), &attr_state)) return;
    hipLaunchKernelGGL(k_islands, dim3(B), dim3(TPB), (size_t)L * sizeof(int), st, mask, island, rank, counts, W, n0, L);
}

void launch_seq_input(const int32_t* prev, const int32_t* tokens, int32_t* inp, int B, int L, int u, hipStream_t st) {
    hipLaunchKernelGGL(k_seq_input, dim3((B + 63) / 64), dim3(64), 0, st, prev, tokens, inp, B, L, u);
}

void launch_seq_draw(const float* logits, const uint8_t* mask, int32_t* tokens, int B, int L, int V, int u,
                     uint64_t seed, uint64_t rng_counter, hipStream_t st) {
    hipLaunchKernelGGL(k_seq_draw, dim3(B), dim3(TPB), 0, st, logits, mask, tokens, L, V, u,
                       (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32), (uint32_t)(rng_counter & 0xFFFFFFFFu),
                       (uint32_t)((rng_counter >> 32) & 0xFFFFFFu));
}

void launch_island_select(const int32_t* prev, const int32_t* tokens, const uint8_t* mask, const int32_t* rank,
                          int32_t* pos_tab, int32_t* inp, uint8_t* hide, int32_t* overflow, int B, int L, int P,
                          int cap, int pass, hipStream_t st) {
    hipLaunchKernelGGL(k_island_select, dim3(B), dim3(TPB), 0, st, prev, tokens, mask, rank, pos_tab, inp, hide,
                       overflow, L, P, cap, pass);
}

void launch_island_draw(const float* logits, const int32_t* pos_tab, int32_t* tokens, float* logits_out, int B,
                        int L, int V, int P, int cap, uint64_t seed, uint64_t rng_counter, hipStream_t st) {
    hipLaunchKernelGGL(k_island_draw, dim3(B * cap), dim3(TPB), 0, st, logits, pos_tab, tokens, logits_out, L, V, P,
                       cap, (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32),
                       (uint32_t)(rng_counter & 0xFFFFFFFFu), (uint32_t)((rng_counter >> 32) & 0xFFFFFFu));
}

void launch_decide_finish(const DecideArgs& a, hipStream_t st) {   // a.L <= 131072 (the caller checks): flags in LDS
    static int attr_state = 0;
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(k_decide_finish), 131072, &attr_state)) return;
    hipLaunchKernelGGL(k_decide_finish, dim3(a.B), dim3(TPB), (size_t)a.L, st, a);
}

void launch_accept(const DecideArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(k_accept, dim3((unsigned)(a.B * a.L)), dim3(TPB), 0, st, a);
}

void launch_accept_from_parts(const DecideArgs& a, const float* parts, int n_parts, hipStream_t st) {
    const int64_t rows = (int64_t)a.B * a.L;
    hipLaunchKernelGGL(k_accept_parts, dim3((unsigned)((rows + WAVES - 1) / WAVES)), dim3(TPB), 0, st, a,
                       reinterpret_cast<const float2*>(parts), n_parts);
}

void launch_mask_sample(const DecideArgs& a, hipStream_t st) {
    unsigned blocks = (unsigned)(a.B * a.L);
    if (a.up_r > 1) {   // whole groups of 8 draft rows (one per XCD), r * r workgroups each
        const int r2 = a.up_r * a.up_r;
        const int64_t parents = (int64_t)a.B * (a.L / r2);
        blocks = (unsigned)(((parents + 7) / 8) * 8 * r2);
    }
    hipLaunchKernelGGL(k_mask_sample, dim3(blocks), dim3(TPB), 0, st, a);
}

}  // namespace mulo
