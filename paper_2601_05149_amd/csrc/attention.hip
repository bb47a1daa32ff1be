// Causal attention of the drafted block over prefix + block (Alg. 1 Step 3: the
// j-th conditional sees cache rows 0 .. P+j).
//
// bf16 path: flash-style, one workgroup of 8 wavefronts (two per SIMD) per (256
// queries, head, sequence); K and V^T tiles of 128 keys are staged through LDS
// (double buffered, 139 KB) and shared by the 8 wavefronts, so a tile is fetched and
// written to LDS once per 256 queries and the per-tile work (barrier, running
// maximum, rescale test) is spread over 32 MFMAs per product; each wavefront owns
// 32 queries and computes
// S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16, so that a lane
// owns ONE query: the softmax row reductions stay inside the lane (plus one
// cross-half shuffle), and the exponentiated scores are already laid out as the
// B operand of the second product.  The K rows are fetched in a permuted order
// (bits 2 and 3 of the row index swapped) so that a lane's accumulators cover 8
// consecutive keys, which is what lets V^T be read with 16-byte LDS loads.
// float32 path (small configuration): one workgroup per query row.
#include <hip/hip_bf16.h>

#include "mulo_internal.h"

namespace mulo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __hip_bfloat16 bf16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr float LOG2E = 1.4426950408889634f;

struct AttnArgs {
    const bf16* q;    // [B, nh, L, dh]
    const bf16* kc;   // [nl, maxB, nh, S, dh]
    const bf16* vc;   // [nl, maxB, nh, dh, S]
    bf16* out;        // [B*L, nh*dh]
    int frag;         // out is the token operand of a weight-streaming projection: fragment order (frag_index)
    int B, L, P, nh, max_seq, max_batch, layer;
    float scale_log2;  // log2(e) / sqrt(dh)
    int nsplit;        // > 1: the keys are dealt to nsplit workgroups per (sequence, head); one query tile only
    float* part;       // [nsplit, B, nh, L][dh + 2]: unnormalised output of a query, running maximum, running sum (L <= 32)
    // scattered queries (island passes): query j of sequence b (L slots per sequence) sits at cache row
    // pos_tab[b * L + j] in [P0, P0 + Lblk) (< 0: unused slot) and does not see rows P0 + t of its sequence with
    // hide[b, t] set, its own excepted
    const int32_t* pos_tab;
    const uint8_t* hide;   // [B, Lblk]
    int P0, Lblk;
};
constexpr float LAZY_EXP = 8.0f;     // measured at 4 x 1024 queries against 4096 keys: 0 -> 822, 4 -> 843, 8 -> 842 TFLOP/s
constexpr int MAX_SPLIT = 16;
constexpr int NS_TARGET = 512;      // workgroups a key split aims at (measured: 256 -> 1.94, 512 -> 1.78, 1024 -> 1.92, 2048 -> 2.11 ms
                                    // of attention per single-token step at the 7B shape, 4 sequences of 4000 rows)
constexpr int SPLIT_QUERIES = 32;   // a key split serves at most this many queries per (sequence, head)

template <int DH, int BQ, int BKV, int NTH>
__global__ __launch_bounds__(NTH, NTH <= 256 ? 2 : 1) void k_attn_bf16(const AttnArgs a) {
    constexpr int KS = DH + 8;     // K tile row stride (bf16)
    constexpr int VS = BKV + 8;    // V^T tile row stride
    constexpr int NKK = DH / 16;   // k-steps of the first product
    constexpr int NDB = DH / 32;   // 32-row blocks of O^T
    constexpr int LK = BKV * (DH / 8) / NTH, LV = DH * (BKV / 8) / NTH;  // 16-byte chunks per lane

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16* sK = reinterpret_cast<bf16*>(smem);   // [2][BKV][KS]
    bf16* sV = sK + 2 * BKV * KS;               // [2][DH][VS]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;
    // Workgroup id -> (query tile, head).  Consecutive ids go to consecutive XCDs, each with its own L2:
    // all query tiles of one (batch, head) are given to ONE XCD, next to each other in its dispatch
    // order, so that they stream that head's K and V through the same L2 side by side (the cache rows
    // are fetched from memory once per head instead of once per query tile).  Long tiles go first.
    const int qtiles = (a.L + BQ - 1) / BQ, nbh = a.B * a.nh;
    const int split = blockIdx.x / (qtiles * nbh), bid = blockIdx.x % (qtiles * nbh);
    int qt, bh;
    if ((nbh & 7) == 0) {
        const int xcd = bid & 7, s = bid >> 3;
        qt = qtiles - 1 - s % qtiles;
        bh = (s / qtiles) * 8 + xcd;
    } else {
        qt = qtiles - 1 - bid % qtiles;
        bh = bid / qtiles;
    }
    const int j0 = qt * BQ, hd = bh % a.nh, b = bh / a.nh;
    // scattered queries run in the short-block configuration only; the long-block one keeps its registers
    const bool scattered = BQ <= 128 && a.pos_tab != nullptr;
    const int P = a.P;
    const int64_t hb = ((int64_t)a.layer * a.max_batch + b) * a.nh + hd;
    const bf16* kbase = a.kc + hb * a.max_seq * DH;
    const bf16* vbase = a.vc + hb * DH * a.max_seq;

    // this lane's query (clamped for the ragged last tile; such lanes do not store)
    const int jq_raw = j0 + wave * 32 + l32;
    const int jq = jq_raw < a.L ? jq_raw : a.L - 1;
    int qpos = P + jq;
    bool active = true;
    if (scattered) {   // the slot's own cache row; an unused slot computes on row P0 and stores zeros
        const int row = a.pos_tab[(int64_t)b * a.L + jq];
        active = row >= 0;
        qpos = active ? row : a.P0;
    }
    const int wave_jmin = j0 + wave * 32;
    int wave_jmax = wave_jmin + 31;
    wave_jmax = wave_jmax < a.L ? wave_jmax : a.L - 1;
    const bool wave_live = wave_jmin < a.L;

    bf16x8 qf[NKK];
    {
        const bf16* qp = a.q + (((int64_t)b * a.nh + hd) * a.L + jq) * DH + lh * 8;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16);
    }

    int blk_jmax = j0 + BQ - 1;
    blk_jmax = blk_jmax < a.L ? blk_jmax : a.L - 1;
    const int kmax_blk = scattered ? a.P0 + a.Lblk - 1 : P + blk_jmax;   // last key any query of this workgroup may see
    const int n_tiles = kmax_blk / BKV + 1;
    // key split (single-token decoding, island passes: at most 32 queries, one wavefront): this workgroup covers
    // tiles [t_begin, t_end) and leaves its unnormalised partial results (output, running maximum, running sum)
    // for k_attn_combine
    const int tiles_per = (n_tiles + a.nsplit - 1) / a.nsplit;
    const int t_begin = split * tiles_per, t_end = t_begin + tiles_per < n_tiles ? t_begin + tiles_per : n_tiles;
    float* part = a.nsplit > 1 ? a.part + (((int64_t)split * a.B + b) * a.nh + hd) * a.L * (DH + 2) : nullptr;
    if (t_begin >= t_end) {    // uniform over the workgroup, before any barrier: an empty share
        if (part) {
            for (int c = tid; c < a.L * (DH + 2); c += NTH) {
                const int e = c % (DH + 2);
                part[c] = e == DH ? -__builtin_huge_valf() : 0.f;
            }
        }
        return;
    }

    u32x4 rk[LK], rv[LV];
    auto gload = [&](int t) {
        const int kv0 = t * BKV;
#pragma unroll
        for (int i = 0; i < LK; ++i) {
            const int c = tid + i * NTH, row = c / (DH / 8), col = (c % (DH / 8)) * 8;
            int key = kv0 + row;
            key = key < a.max_seq ? key : a.max_seq - 1;
            rk[i] = *reinterpret_cast<const u32x4*>(kbase + (int64_t)key * DH + col);
        }
#pragma unroll
        for (int i = 0; i < LV; ++i) {
            const int c = tid + i * NTH, row = c / (BKV / 8), col = (c % (BKV / 8)) * 8;
            int key = kv0 + col;
            const int kc_ = key + 8 <= a.max_seq ? key : a.max_seq - 8;
            rv[i] = *reinterpret_cast<const u32x4*>(vbase + (int64_t)row * a.max_seq + kc_);
            // cache columns past the last visible key may be uninitialised memory: their
            // probabilities are 0, and 0 * NaN must not reach the accumulators
            if (kv0 + BKV - 1 > kmax_blk) {
                auto keep = [&](int e) -> uint32_t { return key + e <= kmax_blk ? 0xFFFFu : 0u; };
                rv[i].x &= keep(0) | (keep(1) << 16);
                rv[i].y &= keep(2) | (keep(3) << 16);
                rv[i].z &= keep(4) | (keep(5) << 16);
                rv[i].w &= keep(6) | (keep(7) << 16);
            }
        }
    };
    auto sstore = [&](int buf) {
        bf16* k = sK + buf * BKV * KS;
        bf16* v = sV + buf * DH * VS;
#pragma unroll
        for (int i = 0; i < LK; ++i) {
            const int c = tid + i * NTH, row = c / (DH / 8), col = (c % (DH / 8)) * 8;
            *reinterpret_cast<u32x4*>(k + row * KS + col) = rk[i];
        }
#pragma unroll
        for (int i = 0; i < LV; ++i) {
            const int c = tid + i * NTH, row = c / (BKV / 8), col = (c % (BKV / 8)) * 8;
            *reinterpret_cast<u32x4*>(v + row * VS + col) = rv[i];
        }
    };

    f32x16 o[NDB];
#pragma unroll
    for (int i = 0; i < NDB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
    float m_run = -__builtin_huge_valf(), l_run = 0.f;

    // MFMA row rho of a K block is fed key kperm(rho): bits 2 and 3 swapped
    const int kperm = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);

    // Hidden rows (scattered queries): one flag per lane and 64-key tile (lane i: key 64 t + i), requested a tile
    // ahead and turned into a 64-bit mask by a ballot, instead of a byte load per score behind the score product.
    static_assert(BQ > 128 || BKV == 64, "a lane holds the hide flag of one key of a 64-key tile");
    auto hide_flag = [&](int tile) -> uint8_t {
        const int tpos = tile * BKV + lane - a.P0;
        const bool in_block = tpos >= 0 && tpos < a.Lblk;
        const uint8_t f = a.hide[(int64_t)b * a.Lblk + (in_block ? tpos : 0)];
        return in_block ? f : (uint8_t)0;
    };
    unsigned long long hide_cur = 0;
    if constexpr (BQ <= 128) {
        if (a.hide && wave_live) hide_cur = __ballot(hide_flag(t_begin) != 0);
    }
    gload(t_begin);
    sstore(t_begin & 1);
    __syncthreads();
    for (int t = t_begin; t < t_end; ++t) {
        const int kv0 = t * BKV;
        const int t_next = t + 1 < t_end ? t + 1 : t;   // the last tile is fetched twice: no branch in the body
        if (wave_live && (scattered || kv0 <= P + wave_jmax)) {
            gload(t_next);
            uint8_t hide_next = 0;
            if constexpr (BQ <= 128) {
                if (a.hide) hide_next = hide_flag(t_next);
            }
            const bf16* k = sK + (t & 1) * BKV * KS;
            const bf16* v = sV + (t & 1) * DH * VS;
            f32x16 s[BKV / 32];
#pragma unroll
            for (int kb = 0; kb < BKV / 32; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
                const bf16* kr = k + (kb * 32 + kperm) * KS + lh * 8;
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk)
                    s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        *reinterpret_cast<const bf16x8*>(kr + kk * 16), qf[kk], s[kb], 0, 0, 0);
            }
            // accumulator r of block kb holds key kv0 + kb*32 + 16*(r/8) + 8*lh + r%8 for query l32
            const bool need_mask = scattered ? kv0 + BKV > a.P0 : kv0 + BKV - 1 > P + wave_jmin;
            float mx = -__builtin_huge_valf();
            if (need_mask) {
#pragma unroll
                for (int kb = 0; kb < BKV / 32; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = kv0 + kb * 32 + 16 * (r >> 3) + 8 * lh + (r & 7);
                        s[kb][r] = key <= qpos ? s[kb][r] : -__builtin_huge_valf();
                    }
            }
            if constexpr (BQ <= 128) {
                if (a.hide) {   // scattered queries: rows of positions that are not settled yet (the query's own excepted)
                    if (hide_cur != 0) {   // uniform over the wavefront; bits are set for rows of the block only
#pragma unroll
                        for (int kb = 0; kb < BKV / 32; ++kb) {
                            const uint32_t mine = (uint32_t)(hide_cur >> (kb * 32)) >> (8 * lh);   // this lane's keys: bits 16 (r / 8) + r % 8
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int key = kv0 + kb * 32 + 16 * (r >> 3) + 8 * lh + (r & 7);
                                if (((mine >> (16 * (r >> 3) + (r & 7))) & 1u) && key < qpos) s[kb][r] = -__builtin_huge_valf();
                            }
                        }
                    }
                    hide_cur = __ballot(hide_next != 0);   // requested at the top of the iteration, for tile t_next
                }
            }
#pragma unroll
            for (int kb = 0; kb < BKV / 32; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // The exponentials are taken against a reference m_run (exponent units: scores times log2(e) / sqrt(dh);
            // the scale is positive) that follows the running maximum lazily: it moves only when the maximum has
            // outgrown it by more than 2^LAZY_EXP.  Probabilities then stay below that factor, which float32 and
            // bf16 hold with the same relative precision, the normalisation divides it out, and the accumulators
            // are rescaled a few times per query instead of in most tiles.  From -inf the first finite maximum
            // moves it.
            const float mxs = mx * a.scale_log2;
            const float m_new = mxs > m_run + LAZY_EXP ? mxs : m_run;
            // a query that has seen no key yet (every row of its first tiles hidden) keeps -inf as its maximum:
            // exponents are then taken against 0, which makes every term exp2(-inf) = 0 instead of NaN
            const float m_safe = m_new == -__builtin_huge_valf() ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
            m_run = m_new;
            float ps = 0.f;
            bf16x8 pf[BKV / 16];
#pragma unroll
            for (int kb = 0; kb < BKV / 32; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][r], a.scale_log2, -m_safe));
                    ps += p;
                    pf[kb * 2 + (r >> 3)][r & 7] = (__bf16)p;
                }
            l_run = l_run * alpha + ps;
            // the accumulators are rescaled only when some query of the wavefront raised its maximum
            if (!__all(alpha == 1.0f)) {
#pragma unroll
                for (int i = 0; i < NDB; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
            }
            // O^T += V^T P^T : k-step ks covers keys kv0 + 16 ks .. +15
#pragma unroll
            for (int ks = 0; ks < BKV / 16; ++ks) {
#pragma unroll
                for (int i = 0; i < NDB; ++i) {
                    const bf16x8 vf = *reinterpret_cast<const bf16x8*>(v + (i * 32 + l32) * VS + ks * 16 + lh * 8);
                    o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ks], o[i], 0, 0, 0);
                }
            }
            sstore((t + 1) & 1);
        } else {
            gload(t_next);
            sstore((t + 1) & 1);
        }
        __syncthreads();
    }

    l_run += __shfl_xor(l_run, 32);
    if (part) {
        if (wave == 0 && jq_raw < a.L) {     // the tile's queries all belong to the first wavefront
            float* pq = part + (int64_t)jq * (DH + 2);
#pragma unroll
            for (int i = 0; i < NDB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) pq[i * 32 + (r >> 2) * 8 + lh * 4 + (r & 3)] = o[i][r];
            if (lh == 0) { pq[DH] = m_run; pq[DH + 1] = l_run; }
        }
        return;
    }
    if (jq_raw < a.L) {
        const float inv = 1.0f / l_run;
        const int row = b * a.L + jq;
        bf16* op = a.out + (int64_t)row * (a.nh * DH) + hd * DH;
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (__bf16)(active ? o[i][g4 * 4 + e] * inv : 0.f);
                const int c = i * 32 + g4 * 8 + lh * 4;   // 4 | c: the four channels share a run of 8
                *reinterpret_cast<bf16x4*>(a.frag ? a.out + frag_index(row, hd * DH + c, a.nh * DH) : op + c) = w;
            }
    }
}

// float32: one workgroup per (query j, head, sequence); scores live in LDS.
__global__ __launch_bounds__(256) void k_attn_f32(const float* __restrict__ q, const float* __restrict__ kc,
                                                  const float* __restrict__ vc, float* __restrict__ out, int L,
                                                  int P, int nh, int dh, int max_seq, int max_batch, int layer) {
    extern __shared__ float sc[];   // [dh] query, then [P + j + 1] scores
    __shared__ float red[4];
    const int j = blockIdx.x, hd = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int n = P + j + 1;
    float* qs = sc;
    float* s = sc + dh;
    const int64_t hb = ((int64_t)layer * max_batch + b) * nh + hd;
    const float* kb = kc + hb * max_seq * dh;
    const float* vb = vc + hb * dh * max_seq;
    for (int c = tid; c < dh; c += 256) qs[c] = q[(((int64_t)b * nh + hd) * L + j) * dh + c];
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)dh);
    float mx = -__builtin_huge_valf();
    for (int t = tid; t < n; t += 256) {
        float acc = 0.f;
        for (int c = 0; c < dh; ++c) acc += qs[c] * kb[(int64_t)t * dh + c];
        acc *= scale;
        s[t] = acc;
        mx = fmaxf(mx, acc);
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float sum = 0.f;
    for (int t = tid; t < n; t += 256) {
        const float e = expf(s[t] - mx);
        s[t] = e;
        sum += e;
    }
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if ((tid & 63) == 0) red[tid >> 6] = sum;
    __syncthreads();
    sum = (red[0] + red[1]) + (red[2] + red[3]);
    for (int c = tid; c < dh; c += 256) {
        float acc = 0.f;
        for (int t = 0; t < n; ++t) acc += s[t] * vb[(int64_t)c * max_seq + t];
        out[((int64_t)b * L + j) * (nh * dh) + hd * dh + c] = acc / sum;
    }
}

// out[b, hd, :] = sum_s o_s 2^(m_s - M) / sum_s l_s 2^(m_s - M), M = max_s m_s (maxima are in exponent units)
template <int DH>
__global__ __launch_bounds__(DH) void k_attn_combine(const AttnArgs a) {
    const int j = blockIdx.x % a.L, hd = (blockIdx.x / a.L) % a.nh, b = blockIdx.x / (a.L * a.nh), c = threadIdx.x;
    auto share = [&](int s) { return a.part + ((((int64_t)s * a.B + b) * a.nh + hd) * a.L + j) * (DH + 2); };
    float M = -__builtin_huge_valf();
    for (int s = 0; s < a.nsplit; ++s) M = fmaxf(M, share(s)[DH]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < a.nsplit; ++s) {
        const float* p = share(s);
        const float wgt = __builtin_amdgcn_exp2f(p[DH] - M);
        num += p[c] * wgt;
        den += p[DH + 1] * wgt;
    }
    const int row = b * a.L + j;
    a.out[a.frag ? frag_index(row, hd * DH + c, a.nh * DH) : (int64_t)row * (a.nh * DH) + hd * DH + c] =
        __float2bfloat16(den > 0.f ? num / den : 0.f);
}

template <int DH, int BQ, int BKV, int NTH>
void run_attn_cfg(const AttnArgs& a, hipStream_t st) {
    auto kern = k_attn_bf16<DH, BQ, BKV, NTH>;
    const size_t lds = (size_t)2 * (BKV * (DH + 8) + DH * (BKV + 8)) * sizeof(bf16);
    static int attr_state = 0;
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds, &attr_state)) return;
    hipLaunchKernelGGL(kern, dim3(((a.L + BQ - 1) / BQ) * a.nh * a.B * a.nsplit), dim3(NTH), lds, st, a);
    if (a.nsplit > 1) hipLaunchKernelGGL(k_attn_combine<DH>, dim3(a.B * a.nh * a.L), dim3(DH), 0, st, a);
}

// Blocks of more than 128 queries: 256-query workgroups of 8 wavefronts over 128-key tiles (one per CU).  Shorter
// ones (single-token decoding above all): 128-query workgroups of 4 wavefronts over 64-key tiles, two per CU.
constexpr int BKV_SMALL = 64;
template <int DH>
void run_attn(const AttnArgs& a, hipStream_t st) {
    if (a.L > 128) run_attn_cfg<DH, 256, 128, 512>(a, st);
    else run_attn_cfg<DH, 128, BKV_SMALL, 256>(a, st);
}

}  // namespace

size_t attention_scratch_bytes(int max_batch, int n_heads, int head_dim) {
    return (size_t)MAX_SPLIT * max_batch * n_heads * SPLIT_QUERIES * (head_dim + 2) * sizeof(float);
}

void launch_attention_bf16(const void* q, const void* k_cache, const void* v_cache, void* out, float* scratch,
                           int B, int L, int P, int n_heads, int head_dim, int max_seq, int max_batch, int layer,
                           bool frag_out, hipStream_t st) {
    AttnArgs a{};
    a.q = (const bf16*)q; a.kc = (const bf16*)k_cache; a.vc = (const bf16*)v_cache; a.out = (bf16*)out;
    a.B = B; a.L = L; a.P = P; a.nh = n_heads; a.max_seq = max_seq; a.max_batch = max_batch; a.layer = layer;
    a.frag = frag_out ? 1 : 0;   // the out projection of such a launch streams its weights
    a.scale_log2 = LOG2E / sqrtf((float)head_dim);
    // one query per sequence: too few (sequence, head) pairs to fill the chip, so the keys are split as well
    a.nsplit = 1;
    a.part = scratch;
    if (L == 1 && scratch) {
        const int tiles = (P + L - 1) / BKV_SMALL + 1;
        int ns = NS_TARGET / (B * n_heads);
        ns = ns > MAX_SPLIT ? MAX_SPLIT : ns;
        ns = ns > tiles ? tiles : ns;
        a.nsplit = ns < 1 ? 1 : ns;
    }
    if (head_dim == 128) run_attn<128>(a, st);
    else run_attn<64>(a, st);
}

void launch_attention_scattered_bf16(const void* q, const void* k_cache, const void* v_cache, void* out,
                                     float* scratch, int B, const int32_t* pos_tab, int cap, const uint8_t* hide,
                                     int P0, int Lblk, int n_heads, int head_dim, int max_seq, int max_batch,
                                     int layer, bool frag_out, hipStream_t st) {
    AttnArgs a{};
    a.q = (const bf16*)q; a.kc = (const bf16*)k_cache; a.vc = (const bf16*)v_cache; a.out = (bf16*)out;
    a.B = B; a.L = cap; a.P = P0; a.nh = n_heads; a.max_seq = max_seq; a.max_batch = max_batch; a.layer = layer;
    a.frag = frag_out ? 1 : 0;
    a.scale_log2 = LOG2E / sqrtf((float)head_dim);
    a.pos_tab = pos_tab; a.hide = hide; a.P0 = P0; a.Lblk = Lblk;
    // the slots of a sequence are the queries of one workgroup (128 per tile), which streams the sequence's rows
    // once; with few (sequence, head) pairs and at most 32 slots the rows are dealt to several workgroups as well
    a.nsplit = 1;
    a.part = scratch;
    if (scratch && cap <= SPLIT_QUERIES) {
        const int tiles = (P0 + Lblk - 1) / BKV_SMALL + 1;
        int ns = NS_TARGET / (B * n_heads);
        ns = ns > MAX_SPLIT ? MAX_SPLIT : ns;
        ns = ns > tiles ? tiles : ns;
        a.nsplit = ns < 1 ? 1 : ns;
    }
    if (head_dim == 128) run_attn_cfg<128, 128, BKV_SMALL, 256>(a, st);
    else run_attn_cfg<64, 128, BKV_SMALL, 256>(a, st);
}

void launch_attention_f32(const float* q, const float* k_cache, const float* v_cache, float* out,
                          float* scratch, int B, int L, int P, int n_heads, int head_dim, int max_seq,
                          int max_batch, int layer, hipStream_t st) {
    (void)scratch;
    const size_t lds = (size_t)(head_dim + P + L) * sizeof(float);
    hipLaunchKernelGGL(k_attn_f32, dim3(L, n_heads, B), dim3(256), lds, st, q, k_cache, v_cache, out, L, P,
                       n_heads, head_dim, max_seq, max_batch, layer);
}

}  // namespace mulo
