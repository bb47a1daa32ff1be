// Dense projections of the target forward (Alg. 1 Step 3): C = A[M,K] W[N,K]^T.
//
// bf16 path: LDS-staged tiles feeding v_mfma_f32_32x32x16_bf16 (64-lane
// wavefronts; both operands are K-contiguous so every lane fetches its 8-element
// fragment with one 16-byte LDS read), float32 accumulation.  The MFMA operands
// are exchanged (weight rows feed the MFMA rows, tokens run over the lanes) and
// the weight rows are fetched with bits 2-3 of the row index swapped, so a lane
// ends up owning one token and runs of 8 consecutive output columns: every
// epilogue reads and writes 16-byte pieces.  Fused epilogues:
//   Q|K    -> rotary on the adjacent pairs of a run (float4 table reads) + q buffer / K cache rows
//   V      -> operands in order instead: a lane owns 8 consecutive tokens of one
//             column = 16 contiguous bytes of the transposed V cache
//   out, down -> residual add into the float32 stream
//   gate|up   -> silu(gate) * up, gate and up columns interleaved inside a tile so
//                that one lane owns both accumulators of a feed-forward column
//   lm-head   -> float32 logits
// float32 path (small configuration): a plain register-tiled kernel.
#include <hip/hip_bf16.h>

#include <utility>

#include "mulo_internal.h"
#include "row_parts.h"

namespace mulo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __hip_bfloat16 bf16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

enum { EPI_QK = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3, EPI_V = 4,
       EPI_QKV = 5 };   // q | k | v in one launch: the weight-streaming kernel, and tiled launches of a few hundred tokens

struct GemmArgs {
    const bf16* A;        // [M, K]
    const bf16* W0;       // QK: wq | SWIGLU: w_gate | else: W [N, K]
    const bf16* W1;       // QK: wk | SWIGLU: w_up
    const bf16* W2;       // QKV: wv
    int M, N, K;          // N: output columns of the fused problem (QK: 2d, SWIGLU: 2f)
    float* Cf;            // RESID: x [M, N] (+=) | LOGITS: logits [M, N]
    bf16* Cb;             // SWIGLU: h [M, N/2] | QK: q buffer
    bf16* kc;             // QK: K cache
    bf16* vc;             // V: V^T cache
    int d;                // QK: model width (segment size)
    int tiles_n;          // column tiles of the launch (set by the launcher)
    int tile_n0;          // first column tile of the launch (set by the launcher)
    float2* parts;        // LOGITS: softmax statistics per 128-column part of every row [M, n_parts], or nullptr
    int n_parts;
    bool stream;          // A is in fragment order: the launch runs in the weight-streaming kernels
    bool w_frag;          // weight-streaming launches: W0 .. W2 point at copies in fragment order
    float* ksums;         // more than STREAM_SHARED_MIN_TOKENS tokens: sums of the K slices [ksplit, M, columns]
    int ksplit;           // set by the launcher
    RopeArgs ra;
};


// compile-time loop: the body sees its index as a constant, so accumulator arrays
// indexed by it stay in registers whatever the unroller decides
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// g * sigmoid(g) with the hardware reciprocal (1 ulp; the product is rounded to bf16 right after)
__device__ __forceinline__ float silu(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

// Source of weight-tile row nl (fixed over the K loop) for each fused problem: row index, and which of the
// two weight matrices (0: W0, 1: W1) it belongs to.
template <int EPI, int BN, int TN>
__device__ __forceinline__ int b_row_src(const GemmArgs& g, int n0, int tile_n, int nl, int& which) {
    int r;
    if constexpr (EPI == EPI_QK || EPI == EPI_QKV) {
        const int seg = n0 / g.d;
        which = seg;
        r = n0 - seg * g.d + nl;
    } else if constexpr (EPI == EPI_SWIGLU) {
        // tile covers feed-forward columns [f0, f0 + BN/2); the wavefront owning tile columns
        // [w TN, (w+1) TN) gets TN/2 of them: gate rows in its first half, up rows in the second
        const int f = g.N / 2, f0 = tile_n * (BN / 2);
        const int w_ = nl / TN, within = nl % TN;
        r = f0 + w_ * (TN / 2) + (within % (TN / 2));
        r = r < f ? r : f - 1;
        which = within >= TN / 2 ? 1 : 0;
    } else {
        which = 0;
        r = n0 + nl;
        r = r < g.N ? r : g.N - 1;
    }
    return r;
}
template <int EPI, int BN, int TN>
__device__ __forceinline__ const bf16* b_row(const GemmArgs& g, int n0, int tile_n, int nl) {
    int which;
    const int r = b_row_src<EPI, BN, TN>(g, n0, tile_n, nl, which);
    return (which == 0 ? g.W0 : which == 1 ? g.W1 : g.W2) + (int64_t)r * g.K;
}

// Whole-tile launches address their operands through buffer descriptors: the descriptor (matrix base and size)
// and a byte offset of the tile row and K-step live in scalar registers, a lane adds one fixed 32-bit offset
// (its row and 16-byte chunk inside a pass).  No 64-bit lane addresses to keep or to advance.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, int64_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)(bytes < 0x7fffffff ? bytes : 0x7fffffff), 0x00020000);
}
__device__ __forceinline__ u32x4 bload(rsrc_t r, uint32_t lane_off, uint32_t base_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)base_off, 0);
}
// rows of the weight matrices of each fused problem
template <int EPI>
__device__ __forceinline__ int64_t weight_rows(const GemmArgs& g) {
    return (EPI == EPI_QK || EPI == EPI_QKV) ? g.d : EPI == EPI_SWIGLU ? g.N / 2 : g.N;
}

// Which tile row feeds MFMA row rho: bits 2 and 3 exchanged.  With it, accumulator r of a lane
// covers, along the MFMA row axis, index 16*(r/8) + 8*lh + r%8: two runs of 8 consecutive indices
// per 32x32 block, so every lane stores 16-byte (bf16) or 2 x 16-byte (float) pieces.
__device__ __forceinline__ int kperm(int l32) { return (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1); }

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8s;

// Fused epilogues.  acc[i][j] is the 32x32 block (i, j) of the wavefront's TM x TN tile whose corner
// is (m0 + wm TM, n0 + wn TN).  All projections but V run with the MFMA operands exchanged, so a
// lane owns ONE token row (m = ... + l32) and, per block, the column runs [16 g + 8 lh, +8), g = 0, 1
// (accumulators 8 g .. 8 g + 7).  The V projection keeps the operands in order: a lane owns one
// output column and runs of 8 consecutive tokens, which are contiguous in the transposed V cache.
// Where token row m of a projection lives: b, jj index the q buffer [B, nh, L, dh]; bc is its cache sequence and pos
// its cache row (< 0: an unused slot of a scattered launch, nothing of it is written).
struct TokPlace { int b, jj, bc, pos; };
__device__ __forceinline__ TokPlace place(const RopeArgs& ra, int m) {
    const int b = m / ra.L, jj = m % ra.L;
    if (ra.pos_tab) return {b, jj, b, ra.pos_tab[m]};   // scattered queries: slot jj of sequence b (L slots each)
    return {b, jj, b, ra.P + jj};
}

template <int EPI, int BN, int TM, int TN, int MB, int NB>
__device__ __forceinline__ void epilogue(const GemmArgs& g, f32x16 (&acc)[MB][NB], int m0, int n0, int tile_n,
                                         int wm, int wn, int l32, int lh) {
    constexpr int NBE = EPI == EPI_SWIGLU ? NB / 2 : NB;   // gate blocks only: up blocks are consumed with them
    if constexpr (EPI == EPI_RESID) {
        // x += acc.  The compiler cannot tell the stream's loads from its stores, so a plain read-add-write per
        // run is a chain of MB * NB * 2 memory round trips per lane (about a microsecond each: the whole
        // epilogue of a launch with one tile per CU).  All runs of one block row are requested first, then
        // added and written: two round trips per lane.
        static_for<MB>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            const int m = m0 + wm * TM + i * 32 + l32;
            if (m < g.M) {
                float* const row = g.Cf + (int64_t)m * g.N + n0 + wn * TN + lh * 8;
                const int nrow = n0 + wn * TN + lh * 8;
                f32x4 r[NB][2][2];
                static_for<NB>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
#pragma unroll
                    for (int g2 = 0; g2 < 2; ++g2) {
                        const int cl = j * 32 + g2 * 16;
                        if (nrow + cl + 8 <= g.N) {
                            r[j][g2][0] = *reinterpret_cast<const f32x4*>(row + cl);
                            r[j][g2][1] = *reinterpret_cast<const f32x4*>(row + cl + 4);
                        }
                    }
                });
                static_for<NB>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
#pragma unroll
                    for (int g2 = 0; g2 < 2; ++g2) {
                        const int cl = j * 32 + g2 * 16;
                        if (nrow + cl + 8 <= g.N) {
                            f32x4 lo, hi;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                lo[e] = r[j][g2][0][e] + acc[i][j][g2 * 8 + e];
                                hi[e] = r[j][g2][1][e] + acc[i][j][g2 * 8 + 4 + e];
                            }
                            *reinterpret_cast<f32x4*>(row + cl) = lo;
                            *reinterpret_cast<f32x4*>(row + cl + 4) = hi;
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (nrow + cl + e < g.N) row[cl + e] += acc[i][j][g2 * 8 + e];
                        }
                    }
                });
            }
        });
        return;
    }
    if constexpr (EPI == EPI_LOGITS && TN == rowparts::PART) {
        // Softmax statistics of the wavefront tile's 128 columns, per token, for the accept test (Sec. 3.1, Eq. 1):
        // this lane holds half lh of part (tile_n, wn) of token row m, run rr = 2 j + g2 in accumulators
        // 8 g2 .. 8 g2 + 7 of block j; the other half sits in lane + 32.  Whole tiles only (every column exists).
        if (g.parts) {
            static_for<MB>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                const int m = m0 + wm * TM + i * 32 + l32;
                float mx = rowparts::NEG_INF;
                static_for<NB>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[i][j][r]);
                });
                float t[8];
                static_for<NB>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
#pragma unroll
                    for (int g2 = 0; g2 < 2; ++g2) {
                        float zz[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) zz[e] = acc[i][j][g2 * 8 + e];
                        t[j * 2 + g2] = rowparts::run_sum(zz, mx, 8);
                    }
                });
                const float sm = rowparts::tree8(t);
                const float2 ps = rowparts::merge_halves(mx, sm, __shfl_xor(mx, 32), __shfl_xor(sm, 32));
                if (lh == 0 && m < g.M) g.parts[(int64_t)m * g.n_parts + tile_n * (BN / rowparts::PART) + wn] = ps;
            });
        }
    }
    static_for<MB>([&](auto ic) {
        static_for<NBE>([&](auto jc) {
            constexpr int i = decltype(ic)::value, j = decltype(jc)::value;
#pragma unroll
            for (int g2 = 0; g2 < 2; ++g2) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = acc[i][j][g2 * 8 + e];
                if constexpr (EPI == EPI_V) {
                    const int n = n0 + wn * TN + j * 32 + l32;                       // output column (head, cc)
                    const int mb = m0 + wm * TM + i * 32 + g2 * 16 + lh * 8;         // first of 8 tokens
                    if (n < g.N && mb < g.M) {
                        const int dh = g.ra.head_dim, hd = n / dh, cc = n % dh;
                        if (!g.ra.pos_tab && ((g.ra.P | g.ra.L) & 7) == 0) {          // aligned run inside one sequence
                            const int b = mb / g.ra.L, jj = mb % g.ra.L;
                            const int64_t hb = ((int64_t)g.ra.layer * g.ra.max_batch + b) * g.ra.n_heads + hd;
                            bf16* dst = g.vc + (hb * dh + cc) * g.ra.max_seq + g.ra.P + jj;
                            bf16x8s o;
#pragma unroll
                            for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[e];
                            *reinterpret_cast<bf16x8s*>(dst) = o;
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                const int m = mb + e;
                                if (m < g.M) {
                                    const TokPlace pl = place(g.ra, m);
                                    const int64_t hb2 = ((int64_t)g.ra.layer * g.ra.max_batch + pl.bc) * g.ra.n_heads + hd;
                                    if (pl.pos >= 0) g.vc[(hb2 * dh + cc) * g.ra.max_seq + pl.pos] = __float2bfloat16(v[e]);
                                }
                            }
                        }
                    }
                } else {
                    const int m = m0 + wm * TM + i * 32 + l32;                       // token row of this lane
                    const int cl = j * 32 + g2 * 16 + lh * 8;                        // column run inside the wave tile
                    if (m < g.M) {
                        if constexpr (EPI == EPI_RESID || EPI == EPI_LOGITS) {
                            const int n = n0 + wn * TN + cl;
                            float* dst = g.Cf + (int64_t)m * g.N + n;
                            if (n + 8 <= g.N) {
                                f32x4 lo = {v[0], v[1], v[2], v[3]}, hi = {v[4], v[5], v[6], v[7]};
                                if constexpr (EPI == EPI_RESID) {
                                    lo += *reinterpret_cast<const f32x4*>(dst);
                                    hi += *reinterpret_cast<const f32x4*>(dst + 4);
                                }
                                *reinterpret_cast<f32x4*>(dst) = lo;
                                *reinterpret_cast<f32x4*>(dst + 4) = hi;
                            } else {
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    if (n + e < g.N) dst[e] = EPI == EPI_RESID ? dst[e] + v[e] : v[e];
                            }
                        } else if constexpr (EPI == EPI_SWIGLU) {
                            const int f = g.N / 2;
                            const int n = tile_n * (BN / 2) + wn * (TN / 2) + cl;
                            bf16* dst = g.Cb + (int64_t)m * f + n;
                            float h[8];
#pragma unroll
                            for (int e = 0; e < 8; ++e) h[e] = silu(v[e]) * acc[i][j + NB / 2][g2 * 8 + e];
                            if (n + 8 <= f) {
                                bf16x8s o;
#pragma unroll
                                for (int e = 0; e < 8; ++e) o[e] = (__bf16)h[e];
                                *reinterpret_cast<bf16x8s*>(dst) = o;
                            } else {
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    if (n + e < f) dst[e] = __float2bfloat16(h[e]);
                            }
                        } else {  // EPI_QK: rotary on the 4 adjacent pairs of the run, q -> [B, nh, L, dh], k -> cache row
                            const int n = n0 + wn * TN + cl, seg = n / g.d, c = n - seg * g.d;
                            const int dh = g.ra.head_dim, hd = c / dh, cc = c % dh;
                            const TokPlace pl = place(g.ra, m);
                            if (EPI == EPI_QKV && seg == 2) {
                                // V with the operands exchanged: a lane holds 8 consecutive channels of ONE token, the
                                // 32 lanes of a half are 32 consecutive tokens = 64 contiguous bytes of a row of the
                                // transposed cache per store (fine for a few hundred tokens; the large launches keep the
                                // V projection of its own, whose lanes hold 8 consecutive tokens)
                                if (pl.pos >= 0) {
                                    const int64_t hb = ((int64_t)g.ra.layer * g.ra.max_batch + pl.bc) * g.ra.n_heads + hd;
#pragma unroll
                                    for (int e = 0; e < 8; ++e)
                                        g.vc[(hb * dh + cc + e) * g.ra.max_seq + pl.pos] = __float2bfloat16(v[e]);
                                }
                            } else if (pl.pos >= 0) {
                                const int pos = pl.pos;
                                const f32x4 cs = *reinterpret_cast<const f32x4*>(g.ra.cos + (int64_t)pos * (dh / 2) + (cc >> 1));
                                const f32x4 sn = *reinterpret_cast<const f32x4*>(g.ra.sin + (int64_t)pos * (dh / 2) + (cc >> 1));
                                bf16x8s o;
#pragma unroll
                                for (int pr = 0; pr < 4; ++pr) {
                                    o[2 * pr] = (__bf16)(v[2 * pr] * cs[pr] - v[2 * pr + 1] * sn[pr]);
                                    o[2 * pr + 1] = (__bf16)(v[2 * pr] * sn[pr] + v[2 * pr + 1] * cs[pr]);
                                }
                                bf16* dst;
                                if (seg == 0) {
                                    dst = g.Cb + (((int64_t)pl.b * g.ra.n_heads + hd) * g.ra.L + pl.jj) * dh + cc;
                                } else {
                                    const int64_t hb = ((int64_t)g.ra.layer * g.ra.max_batch + pl.bc) * g.ra.n_heads + hd;
                                    dst = g.kc + (hb * g.ra.max_seq + pos) * dh + cc;
                                }
                                *reinterpret_cast<bf16x8s*>(dst) = o;
                            }
                        }
                    }
                }
            }
        });
    });
}

template <bool SWAP>
__device__ __forceinline__ f32x16 mma(const bf16x8& a, const bf16x8& b, const f32x16& c) {
    if constexpr (SWAP)   // D[n][m]: MFMA rows = weight rows (output columns), lanes = tokens
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c, 0, 0, 0);
    else                  // D[m][n]: MFMA rows = tokens, lanes = output columns (V projection)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// ---- BM x BN x 64 tiles, double-buffered LDS, one barrier per K-tile ---------------------------
template <int BM, int BN, int WGM, int WGN, int EPI, int BKT = 64, bool FULL = false>
__global__ __launch_bounds__(WGM* WGN * 64, (WGM * WGN >= 8 || BM * BN >= 65536) ? 1 : 2) void k_gemm_bf16(const GemmArgs g) {
    constexpr int BK = BKT, LDS_STRIDE = BKT + 8, CPR = BKT / 8;   // 16-byte chunks per tile row
    constexpr bool SWAP = EPI != EPI_V;
    constexpr int NT = WGM * WGN * 64;
    constexpr int TM = BM / WGM, TN = BN / WGN, MB = TM / 32, NB = TN / 32;
    constexpr int LA = BM * CPR / NT, LB = BN * CPR / NT;  // 16-byte chunks per lane per stage
    static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "tile/threads");
    static_assert(EPI != EPI_SWIGLU || NB % 2 == 0, "swiglu needs an even number of column blocks");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16* sA = reinterpret_cast<bf16*>(smem);                 // [2][BM][LDS_STRIDE]
    bf16* sB = sA + 2 * BM * LDS_STRIDE;                      // [2][BN][LDS_STRIDE]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN, l32 = lane & 31, lh = lane >> 5;
    const int fra = SWAP ? l32 : kperm(l32), frb = SWAP ? kperm(l32) : l32;   // fragment rows (MFMA-row operand permuted)
    // Persistent workgroups.  Workgroup b runs on XCD b % 8 (round-robin dispatch), and each XCD has
    // its own L2, so the tile sequence is cut into one contiguous chunk per XCD and the sequence
    // itself walks groups of GW column tiles row by row: the workgroups of one XCD then work, at any
    // moment, on a near-square patch of output tiles and share its operand rows through that L2.
    constexpr int GW = 8;
    const int tiles_m = (g.M + BM - 1) / BM, total_tiles = tiles_m * g.tiles_n;
    const int nxcd = (gridDim.x & 7) == 0 ? 8 : 1;
    const int tile_stride = gridDim.x / nxcd, chunk = (total_tiles + nxcd - 1) / nxcd;
    const int chunk_base = (blockIdx.x % nxcd) * chunk;
    const int chunk_len = total_tiles - chunk_base < chunk ? total_tiles - chunk_base : chunk;   // may be <= 0
    int tile = blockIdx.x / nxcd, tile_n = 0, m0 = 0, n0 = 0;
    const int kc8 = (tid % CPR) * 8, trow = tid / CPR;
    // Operand addresses.  General case: one pointer per staged chunk.  FULL (M and N multiples of the
    // tile, the launcher checks): the rows a lane fetches are a fixed stride apart, so a lane keeps
    // ONE 32-bit offset (its row and chunk inside a pass) and everything else is scalar: buffer loads
    // through a descriptor of the whole matrix, with the pass's row and the K-step as scalar offset.
    // No 64-bit lane addresses to keep or to advance (about 25 vector registers fewer).
    constexpr int RP = NT / CPR;   // tile rows per pass
    const bf16* pa[FULL ? 1 : LA];
    const bf16* pb[FULL ? 1 : LB];
    uint32_t sa[FULL ? LA : 1];   // byte offset of pass i's first row in its matrix
    uint32_t sb[FULL ? LB : 1];
    const uint32_t voff = (uint32_t)(trow * g.K + kc8) * 2u;
    const rsrc_t rA = make_rsrc(g.A, (int64_t)g.M * g.K * 2);
    rsrc_t rW[2] = {make_rsrc(g.W0, weight_rows<EPI>(g) * g.K * 2),
                    make_rsrc(EPI == EPI_QK || EPI == EPI_QKV || EPI == EPI_SWIGLU ? g.W1 : g.W0, weight_rows<EPI>(g) * g.K * 2)};
    // which descriptor pass i of the weight tile reads: gate | up alternate inside a tile (compile-time), q | k is per tile
    auto wsel = [&](int i) -> rsrc_t { return rW[EPI == EPI_SWIGLU ? ((i * RP) % TN >= TN / 2 ? 1 : 0) : 0]; };
    auto setup = [&](int local) {   // operand rows of the chunk's tile `local` (fixed over its K loop)
        const int t = chunk_base + local, grp = t / (tiles_m * GW), rem = t - grp * tiles_m * GW;
        const int gw = g.tiles_n - grp * GW < GW ? g.tiles_n - grp * GW : GW;
        tile_n = g.tile_n0 + grp * GW + rem % gw;
        m0 = (rem / gw) * BM;
        n0 = tile_n * BN;
        if constexpr (FULL) {
#pragma unroll
            for (int i = 0; i < LA; ++i) sa[i] = (uint32_t)((m0 + i * RP) * g.K) * 2u;
#pragma unroll
            for (int i = 0; i < LB; ++i) {
                int which;
                sb[i] = (uint32_t)(b_row_src<EPI, BN, TN>(g, n0, tile_n, i * RP, which) * g.K) * 2u;
                if constexpr (EPI == EPI_QK || EPI == EPI_QKV) {
                    if (i == 0) rW[0] = make_rsrc(which == 0 ? g.W0 : which == 1 ? g.W1 : g.W2, weight_rows<EPI>(g) * g.K * 2);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                int r = m0 + trow + i * RP;
                r = r < g.M ? r : g.M - 1;
                pa[i] = g.A + (int64_t)r * g.K + kc8;
            }
#pragma unroll
            for (int i = 0; i < LB; ++i) pb[i] = b_row<EPI, BN, TN>(g, n0, tile_n, trow + i * RP) + kc8;
        }
    };

    f32x16 acc[MB][NB];
    u32x4 ra[LA], rb[LB];
    auto gload = [&](int kt) {
        if constexpr (FULL) {
#pragma unroll
            for (int i = 0; i < LA; ++i) ra[i] = bload(rA, voff, sa[i] + kt * (BK * 2));
#pragma unroll
            for (int i = 0; i < LB; ++i) rb[i] = bload(wsel(i), voff, sb[i] + kt * (BK * 2));
        } else {
#pragma unroll
            for (int i = 0; i < LA; ++i) ra[i] = *reinterpret_cast<const u32x4*>(pa[i] + kt * BK);
#pragma unroll
            for (int i = 0; i < LB; ++i) rb[i] = *reinterpret_cast<const u32x4*>(pb[i] + kt * BK);
        }
    };
    const int nk = g.K / BK;
    auto sstore = [&](int buf) {
        bf16* a = sA + buf * BM * LDS_STRIDE;
        bf16* b = sB + buf * BN * LDS_STRIDE;
#pragma unroll
        for (int i = 0; i < LA; ++i)
            *reinterpret_cast<u32x4*>(a + (trow + i * (NT / CPR)) * LDS_STRIDE + kc8) = ra[i];
#pragma unroll
        for (int i = 0; i < LB; ++i)
            *reinterpret_cast<u32x4*>(b + (trow + i * (NT / CPR)) * LDS_STRIDE + kc8) = rb[i];
    };
    // Fragments of one k-slice, double-buffered in registers.  Inside every 64 consecutive k the index is dealt so
    // that lane half lh owns k in [32 lh, 32 lh + 32) and MFMA slice kk takes its kk-th 8 (both operands alike, so
    // the products are unchanged): the same deal, hence the same summation order, as in the kernels that fetch an
    // operand straight from memory, where it makes a lane's bytes contiguous.  A 128-deep K-step is two such runs of
    // 64 one after the other, so the depth of a step does not show in the sums either.
    bf16x8 af[2][MB], bfr[2][NB];
    auto lfrag = [&](const bf16* a, const bf16* b, int kk, int slot) {
        const int ko = (kk >> 2) * 64 + (kk & 3) * 8;
#pragma unroll
        for (int i = 0; i < MB; ++i)
            af[slot][i] = *reinterpret_cast<const bf16x8*>(a + i * 32 * LDS_STRIDE + ko);
#pragma unroll
        for (int j = 0; j < NB; ++j)
            bfr[slot][j] = *reinterpret_cast<const bf16x8*>(b + j * 32 * LDS_STRIDE + ko);
    };

    // Pipeline over the flattened sequence of K-steps of all this workgroup's tiles.  While step s is
    // multiplied out of LDS buffer s & 1, step s+1 is in flight into the staging registers; spread over
    // the iteration's MFMAs, every staging register is written to the other buffer and requested again
    // at once for step s+2, so each request has a whole iteration to land and the memory pipeline sees
    // one request per few MFMAs instead of a burst.  Near the end of a tile the requests run ahead into
    // the next tile, whose first step is staged while this tile's epilogue runs.  The launcher
    // guarantees nk >= 2.
    if (tile >= chunk_len) return;   // uniform over the workgroup, before any barrier
    setup(tile);
    gload(0);
    sstore(0);
    gload(1);
    __syncthreads();
    constexpr int KS = BK / 16;                      // k-slices (one MFMA deep) per K-step
    constexpr int NMS = MB * NB, NF = MB + NB;       // MFMAs and fragment reads per k-slice
    constexpr int NL = LA + LB;                      // staging registers per lane
    static_assert(KS == 4 || KS == 8, "K-steps are one or two runs of 64");
    auto mm = [&](int slot) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j) acc[i][j] = mma<SWAP>(af[slot][i], bfr[slot][j], acc[i][j]);
    };
    // One K-step, rotated by one k-slice: the step's first fragments are requested right after the barrier and
    // the MFMAs of the PREVIOUS step's last slice (fragments already in registers, slot 1) run while they are on
    // their way, so no wavefront waits for LDS with an empty MFMA queue.  Slice kk lives in slot kk & 1; on return
    // slot 1 holds the step's last slice, not yet multiplied.
    auto step_rot = [&](int step) {
        const bf16* a = sA + (step & 1) * BM * LDS_STRIDE + (wm * TM + fra) * LDS_STRIDE + lh * 32;
        const bf16* b = sB + (step & 1) * BN * LDS_STRIDE + (wn * TN + frb) * LDS_STRIDE + lh * 32;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            lfrag(a, b, kk, kk & 1);
            mm((kk + 1) & 1);
        }
    };
    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    int gs = 0;   // steps done so far: buffer parity
    while (true) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        // nothing is pending at the start of a tile: slot 1 holds zeros, its MFMAs add nothing
#pragma unroll
        for (int i = 0; i < MB; ++i) af[1][i] = zero8;
#pragma unroll
        for (int j = 0; j < NB; ++j) bfr[1][j] = zero8;
        int e_m0 = m0, e_n0 = n0, e_tile_n = tile_n;
        bool more = true;
        int kt = 0;
        // steady state: one scheduling region per K-step.  Fragment reads of slice kk + 1 go in front of the MFMAs
        // of slice kk; over the MFMAs of the step's slices 1 and 2 every staging register is written to LDS as soon
        // as its load (requested one iteration ago) is there and is at once requested again for step kt + 2.
        for (; kt < nk - 2; ++kt, ++gs) {
            const bf16* a = sA + (gs & 1) * BM * LDS_STRIDE + (wm * TM + fra) * LDS_STRIDE + lh * 32;
            const bf16* b = sB + (gs & 1) * BN * LDS_STRIDE + (wn * TN + frb) * LDS_STRIDE + lh * 32;
            bf16* na = sA + ((gs + 1) & 1) * BM * LDS_STRIDE + trow * LDS_STRIDE + kc8;
            bf16* nb = sB + ((gs + 1) & 1) * BN * LDS_STRIDE + trow * LDS_STRIDE + kc8;
            auto stage = [&](auto ic) {   // staging register i: to LDS (step kt + 1), then requested again (step kt + 2)
                constexpr int i = decltype(ic)::value;
                if constexpr (i < LA) {
                    *reinterpret_cast<u32x4*>(na + i * RP * LDS_STRIDE) = ra[i];
                    if constexpr (FULL) ra[i] = bload(rA, voff, sa[i] + (kt + 2) * (BK * 2));
                    else ra[i] = *reinterpret_cast<const u32x4*>(pa[i] + (kt + 2) * BK);
                } else {
                    constexpr int j = i - LA;
                    *reinterpret_cast<u32x4*>(nb + j * RP * LDS_STRIDE) = rb[j];
                    if constexpr (FULL) rb[j] = bload(wsel(j), voff, sb[j] + (kt + 2) * (BK * 2));
                    else rb[j] = *reinterpret_cast<const u32x4*>(pb[j] + (kt + 2) * BK);
                }
            };
            // The NL write + load pairs are dealt evenly over the first SPAN MFMAs of the iteration; the rest run
            // bare, so the last LDS writes have landed when the wavefront reaches the barrier.
            constexpr int SPAN = KS * NMS - NMS / 2;
            auto before = [](int m) constexpr { return m >= SPAN ? NL : m * NL / SPAN; };   // pairs in front of MFMA m
            static_for<KS>([&](auto phc) {   // phase 0 multiplies the previous step's last slice
                constexpr int ph = decltype(phc)::value;
                lfrag(a, b, ph, ph & 1);
                static_for<before((ph + 1) * NMS) - before(ph * NMS)>(
                    [&](auto ic) { stage(std::integral_constant<int, before(ph * NMS) + decltype(ic)::value>{}); });
                mm((ph + 1) & 1);
            });
            static_for<KS>([&](auto phc) {
                constexpr int ph = decltype(phc)::value;
                __builtin_amdgcn_sched_group_barrier(0x100, NF, 0);
                static_for<NMS>([&](auto mc) {
                    constexpr int m = ph * NMS + decltype(mc)::value;
                    static_for<before(m + 1) - before(m)>([&](auto) {
                        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                    });
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                });
            });
            __builtin_amdgcn_sched_barrier(0);   // the bare MFMAs stay in front of the barrier
            __syncthreads();
        }
        for (; kt < nk; ++kt, ++gs) {   // last two steps of the tile: the requests move on to the next tile
            step_rot(gs);
            if (kt == nk - 2) {
                e_m0 = m0; e_n0 = n0; e_tile_n = tile_n;
                tile += tile_stride;
                more = tile < chunk_len;
                if (more) setup(tile);
            }
            if (kt + 1 < nk || more) sstore((gs + 1) & 1);
            if (more) gload(kt + 2 - nk);
            __syncthreads();
        }
        mm(1);   // the tile's last slice
        epilogue<EPI, BN, TM, TN, MB, NB>(g, acc, e_m0, e_n0, e_tile_n, wm, wn, l32, lh);
        if (!more) break;
    }
}


static int cu_count() {
    static int n = 0;
    if (n == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n = prop.multiProcessorCount;
        if (n <= 0) n = 256;
    }
    return n;
}

template <int BM, int BN, int WGM, int WGN, int EPI, int BKT = 64, bool FULL = false>
void run_gemm(GemmArgs g, int tile_n0, int tiles_n, int blocks_per_cu, hipStream_t st) {
    auto kern = k_gemm_bf16<BM, BN, WGM, WGN, EPI, BKT, FULL>;
    const size_t lds = (size_t)2 * (BM + BN) * (BKT + 8) * sizeof(bf16);
    static int attr_state = 0;  // each instantiation is configured once per process
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds, &attr_state)) return;
    const int tiles_m = (g.M + BM - 1) / BM, total = tiles_m * tiles_n;
    const int resident = cu_count() * blocks_per_cu;
    g.tiles_n = tiles_n;
    g.tile_n0 = tile_n0;
    hipLaunchKernelGGL(kern, dim3(total < resident ? total : resident), dim3(WGM * WGN * 64), lds, st, g);
}


// Epilogue of the weight-streaming kernels on two adjacent output columns n, n + 1 of token m (v1: the up sums of
// gate|up).  The same five fused epilogues as the tiled kernels; a bf16 operand of a following projection is written
// in fragment order.
template <int EPI>
__device__ __forceinline__ void stream_epilogue(const GemmArgs& g, int m, int n, const float (&v0)[2], const float (&v1)[2]) {
    if constexpr (EPI == EPI_RESID || EPI == EPI_LOGITS) {
        float* dst = g.Cf + (int64_t)m * g.N + n;
#pragma unroll
        for (int e = 0; e < 2; ++e)
            if (n + e < g.N) dst[e] = EPI == EPI_RESID ? dst[e] + v0[e] : v0[e];
    } else if constexpr (EPI == EPI_SWIGLU) {
        const int f = g.N / 2;
        bf16* dst = g.Cb + frag_index(m, n, f);   // the down projection streams too: its token operand, fragment order
#pragma unroll
        for (int e = 0; e < 2; ++e)
            if (n + e < f) dst[e] = __float2bfloat16(silu(v0[e]) * v1[e]);
    } else {
        const TokPlace pl = place(g.ra, m);
        if (pl.pos < 0) return;   // an unused slot of a scattered launch
        const int dh = g.ra.head_dim, pos = pl.pos;
        if (EPI == EPI_QK || (EPI == EPI_QKV && n < 2 * g.d)) {
            const int seg = n / g.d, c = n - seg * g.d;
            const int hd = c / dh, cc = c % dh;
            const float cs = g.ra.cos[(int64_t)pos * (dh / 2) + (cc >> 1)], sn = g.ra.sin[(int64_t)pos * (dh / 2) + (cc >> 1)];
            bf16* dst;
            if (seg == 0) {
                dst = g.Cb + (((int64_t)pl.b * g.ra.n_heads + hd) * g.ra.L + pl.jj) * dh + cc;
            } else {
                const int64_t hb = ((int64_t)g.ra.layer * g.ra.max_batch + pl.bc) * g.ra.n_heads + hd;
                dst = g.kc + (hb * g.ra.max_seq + pos) * dh + cc;
            }
            dst[0] = __float2bfloat16(v0[0] * cs - v0[1] * sn);
            dst[1] = __float2bfloat16(v0[0] * sn + v0[1] * cs);
        } else {   // V: transposed cache
            const int nv = EPI == EPI_QKV ? n - 2 * g.d : n, nlim = EPI == EPI_QKV ? g.d : g.N;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int hd = (nv + e) / dh, cc = (nv + e) % dh;
                const int64_t hb = ((int64_t)g.ra.layer * g.ra.max_batch + pl.bc) * g.ra.n_heads + hd;
                if (nv + e < nlim) g.vc[(hb * dh + cc) * g.ra.max_seq + pos] = __float2bfloat16(v0[e]);
            }
        }
    }
}

// ---- up to 64 tokens (single-token decoding of a few sequences, island passes): weight-streaming kernel ----
// The work is reading every weight once, so nothing is staged: a workgroup owns 16 output columns (for
// gate|up: 16 feed-forward columns = 16 gate rows + 16 up rows), its 8 wavefronts split K, and every lane
// feeds v_mfma_f32_16x16x32_bf16 from registers loaded straight from global memory.  In that instruction's operand
// layout the four lanes l16, l16 + 16, l16 + 32, l16 + 48 hold 4 x 8 consecutive k of weight row l16, so one load
// instruction of a wavefront reads 64 contiguous bytes of each of 16 rows: whole 64-byte sectors (with the 32-row
// instruction only two lanes share a row, 32 of every 64 bytes fetched per request), and a matrix of N columns
// gives N / 16 workgroups (256 for the 4096-column projections: one per CU).  The tokens are the instruction's
// column dimension (columns m >= M are fed zeros), up to four groups of 16, and arrive in fragment order (the
// producing kernels write them so: one contiguous KB per group and step, no lane exchange); the accumulators come out as
// D[weight row 4 q + i][token l16], q = lane / 16: a lane owns 4 consecutive output columns of one token.  The
// 8 partial sums are added in a fixed order through LDS and the epilogue runs on pairs of adjacent columns.
typedef __attribute__((ext_vector_type(4))) float f32x4v;
template <int EPI, int MT, bool WFRAG>
__global__ __launch_bounds__(512) void k_gemv_bf16(const GemmArgs g) {
    constexpr int NA = EPI == EPI_SWIGLU ? 2 : 1;   // weight matrices (accumulator sets) per column
    // 32-deep k-steps in flight per wavefront: what 16 requests of 16 bytes per lane allow, at least 4 (measured at
    // the 7B shape: 16 -> 181 ms, 24 -> 185, 32 -> 186 for a re-sampling run of 21 island passes)
    constexpr int U = 16 / (NA + MT) < 4 ? 4 : 16 / (NA + MT);
    __shared__ float part[8][NA * MT][4][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, q = lane >> 4;
    // Weight loads use another lane order than the MFMA: lane 4 r + c fetches chunk c (16 bytes) of row r, so that
    // four ADJACENT lanes read 64 contiguous bytes (one access of the vector L1; in the MFMA's own order, lane
    // 16 c + r, adjacent lanes sit in different rows and every lane is an access of its own: the L1 then limits the
    // kernel).  Each fetched register is moved to the MFMA's order by a lane permutation (ds_bpermute: lane 16 c + r
    // takes the value of lane 4 r + c); which k a slot holds is unchanged, hence so is every sum.  The permutations
    // occupy the LDS pipe (measured: about half of the kernel's time with one token group when the token operand was
    // fetched and permuted the same way, 16 of 20 permutations per step with four groups), which is why the token
    // operand arrives in fragment order and needs none.
    const int lrow = lane >> 2, lchunk = lane & 3;
    const int from_lane = (4 * l16 + q) << 2;   // byte address of the source lane for ds_bpermute
    const int n_blk = blockIdx.x * 16;     // first output column (gate|up: first feed-forward column)
    const int steps = g.K / 32, per = (steps + 7) / 8;
    const int s0 = wave * per, s1 = s0 + per < steps ? s0 + per : steps;

    // weight row(s) this lane fetches; with a copy in fragment order (WFRAG) the KB of (16-row block, step) is
    // contiguous in the MFMA's own lane order: lane l owns its bytes [16 l, 16 l + 16), no exchange afterwards
    const bf16* w[NA];
    if constexpr (WFRAG) {
        int blk = blockIdx.x;   // 16-row block inside its matrix
        const bf16* base = g.W0;
        if constexpr (EPI == EPI_QK || EPI == EPI_QKV) {
            const int seg = n_blk / g.d;
            base = seg == 0 ? g.W0 : seg == 1 ? g.W1 : g.W2;
            blk -= seg * (g.d / 16);
        }
        w[0] = base + (int64_t)blk * steps * 512 + lane * 8;
        if constexpr (EPI == EPI_SWIGLU) w[1] = g.W1 + (int64_t)blk * steps * 512 + lane * 8;
    } else {
        int r = n_blk + lrow;
        if constexpr (EPI == EPI_QK || EPI == EPI_QKV) {
            const int seg = n_blk / g.d;                       // a block never straddles q | k | v (d % 16 == 0)
            w[0] = (seg == 0 ? g.W0 : seg == 1 ? g.W1 : g.W2) + (int64_t)(r - seg * g.d) * g.K;
        } else if constexpr (EPI == EPI_SWIGLU) {
            const int f = g.N / 2;
            r = r < f ? r : f - 1;
            w[0] = g.W0 + (int64_t)r * g.K;
            w[1] = g.W1 + (int64_t)r * g.K;
        } else {
            r = r < g.N ? r : g.N - 1;
            w[0] = g.W0 + (int64_t)r * g.K;
        }
    }
    // The token operand is stored in fragment order: the KB of (token group t, step s) is contiguous and lane l owns
    // its bytes [16 l, 16 l + 16) in the MFMA's own order.  Tokens past M are not written by anybody: fed as zeros.
    const bf16* const xg = g.A + lane * 8;
    bool has_x[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) has_x[t] = t * 16 + l16 < g.M;
    if constexpr (!WFRAG) {
#pragma unroll
        for (int i = 0; i < NA; ++i) w[i] += lchunk * 8;
    }
    auto to_mfma_order = [&](u32x4 v) {
        u32x4 r;
        r.x = (uint32_t)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.x);
        r.y = (uint32_t)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.y);
        r.z = (uint32_t)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.z);
        r.w = (uint32_t)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.w);
        return r;
    };

    f32x4v acc[NA][MT];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[i][t] = f32x4v{0.f, 0.f, 0.f, 0.f};
    const u32x4 zero = {0u, 0u, 0u, 0u};
    // U steps in flight per wavefront, all the time: the registers of a step are requested again, for the step U
    // further on, as soon as the step has been multiplied, so the memory pipeline never drains between batches
    // (a batch that is requested, waited for and multiplied as a whole leaves it empty for a memory round trip
    // per batch).  No branch on the step index: steps past the end of the slice re-read the matrix's last step and
    // are multiplied by zeros (a branch there makes the compiler wait for every load in flight).  The last batch
    // requests nothing.
    u32x4 wv[NA][U], xv[MT][U];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int u = 0; u < U; ++u) xv[t][u] = zero;
    auto request = [&](int u, int s) {
        const int sc = s < steps ? s : steps - 1;
#pragma unroll
        for (int i = 0; i < NA; ++i) wv[i][u] = *reinterpret_cast<const u32x4*>(w[i] + sc * (WFRAG ? 512 : 32));
#pragma unroll
        for (int t = 0; t < MT; ++t)   // lanes whose token does not exist request nothing (a 4-token launch reads 4 x 64 bytes of the KB)
            if (has_x[t]) xv[t][u] = *reinterpret_cast<const u32x4*>(xg + ((int64_t)t * steps + sc) * 512);
    };
    auto permute = [&](int u, int s, bf16x8 (&wf)[NA], bf16x8 (&xf)[MT]) {
        const bool in_slice = s < s1;
#pragma unroll
        for (int i = 0; i < NA; ++i) wf[i] = __builtin_bit_cast(bf16x8, WFRAG ? wv[i][u] : to_mfma_order(wv[i][u]));
#pragma unroll
        for (int t = 0; t < MT; ++t) xf[t] = __builtin_bit_cast(bf16x8, (in_slice && has_x[t]) ? xv[t][u] : zero);
    };
    auto multiply = [&](const bf16x8 (&wf)[NA], const bf16x8 (&xf)[MT]) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int i = 0; i < NA; ++i)
                acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], xf[t], acc[i][t], 0, 0, 0);
    };
    if (s0 < s1) {   // uniform over the wavefront
#pragma unroll
        for (int u = 0; u < U; ++u) request(u, s0 + u);
        int sb = s0;
        for (; sb + U < s1; sb += U) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                bf16x8 wf[NA], xf[MT];
                permute(u, sb + u, wf, xf);
                request(u, sb + U + u);
                multiply(wf, xf);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            bf16x8 wf[NA], xf[MT];
            permute(u, sb + u, wf, xf);
            multiply(wf, xf);
        }
    }
    // reduce the K-slices in a fixed order through LDS; thread (pr, t, lane) of the first 2 * MT wavefronts then
    // owns accumulators 2 pr, 2 pr + 1 of token group t = two adjacent columns of token t * 16 + l16
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) part[wave][a * MT + t][r][lane] = acc[a][t][r];
    __syncthreads();
    const int pr = wave & 1, tg = wave >> 1;
    const int m = tg * 16 + l16;
    if (wave >= 2 * MT || m >= g.M) return;
    {
        float v0[2], v1[2] = {0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
            for (int ww = 0; ww < 8; ++ww) {
                sum0 += part[ww][tg][2 * pr + e][lane];
                if constexpr (EPI == EPI_SWIGLU) sum1 += part[ww][MT + tg][2 * pr + e][lane];
            }
            v0[e] = sum0;
            v1[e] = sum1;
        }
        stream_epilogue<EPI>(g, m, n_blk + 4 * q + 2 * pr, v0, v1);
    }
}

// ---- 65 to 256 tokens with the weight copy in fragment order: the token operand goes through LDS ----
// With several token groups the kernel above spends its time on the token operand: every workgroup (16 columns) reads
// all of it through its vector L1, a KB per token group and KB of weights.  Here a workgroup owns 128 columns (a
// wavefront 16 of them) and a slice of K: the slice's token operand, which arrives in fragment order, is copied to LDS
// once per workgroup, 8 k-steps at a time, and every wavefront feeds its MFMAs from there (one 16-byte LDS read per
// lane and token group); only the weights, contiguous KB blocks of the fragment-order copy, come through the memory
// pipeline, 8 steps in flight per wavefront.  K is dealt to `ksplit` workgroups per column group; each leaves its sums
// [M, 128] in `ksums`, and k_stream_finish adds the slices in index order and runs the epilogue (no float atomics:
// the result does not depend on which workgroup finishes first).  Gate|up and q|k|v are concatenations of their weight
// matrices (`seg_rows` rows each) along the column axis.
template <int MTB>
__global__ __launch_bounds__(512) void k_gemv_shared(const GemmArgs g, int ncols, int seg_rows, int ncg) {
    constexpr int CH = 8;                         // k-steps per LDS chunk = weight steps in flight per wavefront
    constexpr int PIECES = CH * MTB * 64 / 512;   // 16-byte pieces of a chunk per thread
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // fragment (group t, step j) at (t CH + j) KB
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, q = lane >> 4;
    const int cg = blockIdx.x % ncg, kw = blockIdx.x / ncg;   // neighbouring workgroups share a K slice of the token operand
    const int n_w = cg * 128 + wave * 16;                     // this wavefront's first column
    const int steps = g.K / 32, per = (steps + g.ksplit - 1) / g.ksplit;
    const int s0 = kw * per, s1 = s0 + per < steps ? s0 + per : steps;
    const int n_groups = (g.M + 15) >> 4;

    const bf16* w;
    {
        const int last = (ncols - 1) / 16 * 16;               // a wavefront past the last column re-reads the last block
        const int n_c = n_w < last ? n_w : last;
        const int seg = n_c / seg_rows;                        // 16 columns never straddle two matrices (seg_rows % 16 == 0)
        w = (seg == 0 ? g.W0 : seg == 1 ? g.W1 : g.W2) + (int64_t)((n_c - seg * seg_rows) / 16) * steps * 512 + lane * 8;
    }
    f32x4v acc[MTB];
#pragma unroll
    for (int t = 0; t < MTB; ++t) acc[t] = f32x4v{0.f, 0.f, 0.f, 0.f};
    const u32x4 zero = {0u, 0u, 0u, 0u};
    u32x4 wv[CH], xr[PIECES];
    auto request = [&](int u, int s) {
        const int sc = s < steps ? s : steps - 1;
        wv[u] = *reinterpret_cast<const u32x4*>(w + (int64_t)sc * 512);
    };
    // chunk of steps [sc0, sc0 + CH): piece p = ((t CH + j) 64 + lane position); steps past the slice and token groups
    // that do not exist are zeros (tokens past M inside the last group are whatever the buffer holds: they only reach
    // accumulator columns that are never stored)
    auto xload = [&](int sc0) {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int p = tid + i * 512, t = p / (CH * 64), j = (p / 64) % CH;
            xr[i] = zero;
            if (t < n_groups && sc0 + j < s1)
                xr[i] = *reinterpret_cast<const u32x4*>(g.A + ((int64_t)t * steps + sc0 + j) * 512 + (p & 63) * 8);
        }
    };
    auto xstore = [&]() {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) *reinterpret_cast<u32x4*>(smem + (size_t)(tid + i * 512) * 16) = xr[i];
    };
    auto chunk = [&](int sc0, auto req) {
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const bf16x8 wf = __builtin_bit_cast(bf16x8, wv[u]);
            if constexpr (decltype(req)::value) request(u, sc0 + CH + u);
#pragma unroll
            for (int t = 0; t < MTB; ++t) {
                const bf16x8 xf = *reinterpret_cast<const bf16x8*>(smem + (size_t)((t * CH + u) * 64 + lane) * 16);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf, acc[t], 0, 0, 0);
            }
        }
    };
    if (s0 < s1) {   // uniform over the workgroup
#pragma unroll
        for (int u = 0; u < CH; ++u) request(u, s0 + u);
        xload(s0);
        xstore();
        __syncthreads();
        int sc0 = s0;
        for (; sc0 + CH < s1; sc0 += CH) {
            xload(sc0 + CH);
            chunk(sc0, std::true_type{});
            __syncthreads();   // every wavefront has read the chunk
            xstore();
            __syncthreads();
        }
        chunk(sc0, std::false_type{});   // the last chunk requests nothing
    }
    // this slice's sums: D[weight row 4 q + i][token l16] -> ksums[kw][m][n_w + 4 q + i]
#pragma unroll
    for (int t = 0; t < MTB; ++t) {
        const int m = t * 16 + l16, n = n_w + 4 * q;
        if (m < g.M && n < ncols) {
            float* dst = g.ksums + ((int64_t)kw * g.M + m) * ncols + n;
            if (n + 4 <= ncols) {
                *reinterpret_cast<f32x4v*>(dst) = acc[t];
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (n + i < ncols) dst[i] = acc[t][i];
            }
        }
    }
}

// adds the K slices of two adjacent columns of a token in index order and runs the projection's epilogue
template <int EPI>
__global__ __launch_bounds__(256) void k_stream_finish(const GemmArgs g, int ncols) {
    const int cols = EPI == EPI_SWIGLU ? ncols / 2 : ncols;   // gate|up: the up sums of column n sit at column f + n
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int pairs = cols / 2;
    const int m = (int)(idx / pairs), n = 2 * (int)(idx % pairs);
    if (m >= g.M) return;
    float v0[2] = {0.f, 0.f}, v1[2] = {0.f, 0.f};
    for (int kw = 0; kw < g.ksplit; ++kw) {
        const float* src = g.ksums + ((int64_t)kw * g.M + m) * ncols + n;
        const float2 a = *reinterpret_cast<const float2*>(src);
        v0[0] += a.x;
        v0[1] += a.y;
        if constexpr (EPI == EPI_SWIGLU) {
            const float2 b = *reinterpret_cast<const float2*>(src + cols);
            v1[0] += b.x;
            v1[1] += b.y;
        }
    }
    stream_epilogue<EPI>(g, m, n, v0, v1);
}

template <int EPI>
void run_gemv_shared(GemmArgs g, hipStream_t st) {
    const int ncols = g.N, seg_rows = (EPI == EPI_QKV || EPI == EPI_QK) ? g.d : EPI == EPI_SWIGLU ? g.N / 2 : g.N;
    const int ncg = (ncols + 127) / 128;
    g.ksplit = stream_ksplit(ncols, g.K);
    const dim3 grid(ncg * g.ksplit);
    auto launch = [&](auto kern, int mtb) {
        static int attr_state = 0;   // one per kernel instantiation (the lambda's call operator is a template)
        if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), mtb * 8 * 1024, &attr_state)) return;
        hipLaunchKernelGGL(kern, grid, dim3(512), (size_t)mtb * 8 * 1024, st, g, ncols, seg_rows, ncg);
    };
    switch ((g.M + 15) / 16) {   // one instantiation per number of token groups: LDS reads and MFMAs follow it
        case 1: case 2: case 3: case 4: launch(k_gemv_shared<4>, 4); break;
        case 5: launch(k_gemv_shared<5>, 5); break;
        case 6: launch(k_gemv_shared<6>, 6); break;
        case 7: launch(k_gemv_shared<7>, 7); break;
        case 8: launch(k_gemv_shared<8>, 8); break;
        case 9: launch(k_gemv_shared<9>, 9); break;
        case 10: launch(k_gemv_shared<10>, 10); break;
        case 11: launch(k_gemv_shared<11>, 11); break;
        case 12: launch(k_gemv_shared<12>, 12); break;
        case 13: launch(k_gemv_shared<13>, 13); break;
        case 14: launch(k_gemv_shared<14>, 14); break;
        case 15: launch(k_gemv_shared<15>, 15); break;
        default: launch(k_gemv_shared<16>, 16); break;
    }
    const int cols = EPI == EPI_SWIGLU ? ncols / 2 : ncols;
    const int64_t threads = (int64_t)g.M * (cols / 2);
    hipLaunchKernelGGL((k_stream_finish<EPI>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, g, ncols);
}

template <int EPI>
void run_gemv(const GemmArgs& g, hipStream_t st) {
    if (g.M > STREAM_SHARED_MIN_TOKENS && g.w_frag && g.ksums) {   // several token groups: the token operand goes through LDS
        run_gemv_shared<EPI>(g, st);
        return;
    }
    if (g.M > STREAM_MAX_TOKENS) {   // the kernel below holds four token groups
        note_hip_error(hipErrorInvalidValue);
        return;
    }
    const int cols = EPI == EPI_SWIGLU ? g.N / 2 : g.N;
    const dim3 grid((cols + 15) / 16);
    if (g.w_frag) {
        if (g.M <= 16) hipLaunchKernelGGL((k_gemv_bf16<EPI, 1, true>), grid, dim3(512), 0, st, g);
        else if (g.M <= 32) hipLaunchKernelGGL((k_gemv_bf16<EPI, 2, true>), grid, dim3(512), 0, st, g);
        else if (g.M <= 48) hipLaunchKernelGGL((k_gemv_bf16<EPI, 3, true>), grid, dim3(512), 0, st, g);
        else hipLaunchKernelGGL((k_gemv_bf16<EPI, 4, true>), grid, dim3(512), 0, st, g);
        return;
    }
    if (g.M <= 16) hipLaunchKernelGGL((k_gemv_bf16<EPI, 1, false>), grid, dim3(512), 0, st, g);
    else if (g.M <= 32) hipLaunchKernelGGL((k_gemv_bf16<EPI, 2, false>), grid, dim3(512), 0, st, g);
    else if (g.M <= 48) hipLaunchKernelGGL((k_gemv_bf16<EPI, 3, false>), grid, dim3(512), 0, st, g);
    else hipLaunchKernelGGL((k_gemv_bf16<EPI, 4, false>), grid, dim3(512), 0, st, g);
}

// one thread per 16-byte piece of the copy: piece p of block (nb, s) is lane p % 64
__global__ __launch_bounds__(256) void k_pack_weights(const bf16* __restrict__ src, bf16* __restrict__ dst, int layers,
                                                      int rows, int K) {
    const int steps = K / 32, nb_per = (rows + 15) / 16;
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x, total = (int64_t)layers * nb_per * steps * 64;
    if (p >= total) return;
    const int lane = (int)(p & 63);
    const int64_t blk = p >> 6;
    const int s = (int)(blk % steps);
    const int64_t nbl = blk / steps;                     // (layer, 16-row block)
    const int layer = (int)(nbl / nb_per), nb = (int)(nbl % nb_per);
    const int row = nb * 16 + (lane & 15), k = s * 32 + (lane >> 4) * 8;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (row < rows) v = *reinterpret_cast<const u32x4*>(src + ((int64_t)layer * rows + row) * K + k);
    *reinterpret_cast<u32x4*>(dst + p * 8) = v;
}

// returns whether the launch ran on the kernels whose wavefront tile is 128 columns wide (whole tiles)
enum { CLS_STREAM, CLS_BIG, CLS_MID, CLS_SMALL };
template <int EPI>
int classify(const GemmArgs& g) {
    if (g.stream) return CLS_STREAM;   // a handful of tokens: stream the weights (A is in fragment order)
    // large problems: 256x256 tiles, 8 wavefronts (4x2, 64x128 each, two per SIMD); small: 128x128, 4 wavefronts
    // (whole tiles only: their operand rows are addressed from scalar bases; a q|k|v tile must not straddle two weights)
    const bool whole_n = g.N % 256 == 0 && ((EPI == EPI_QK || EPI == EPI_QKV) ? g.d % 256 == 0 : true) &&
                         (int64_t)g.K * 256 * 2 < (1ll << 31) && (int64_t)g.M * g.K * 2 < (1ll << 31) &&
                         (int64_t)((EPI == EPI_QK || EPI == EPI_QKV) ? g.d : EPI == EPI_SWIGLU ? g.N / 2 : g.N) * g.K * 2 < (1ll << 31);
    const bool big = whole_n && g.M >= 1024 && g.M % 256 == 0 &&
                     (int64_t)(g.M / 256) * (g.N / 256) * 4 >= 3 * (int64_t)cu_count();   // enough 256x256 tiles to fill the chip
    if (big) return CLS_BIG;
    // a few hundred tokens (any count: rows past M read as zeros through the descriptor and are not stored): the
    // pipelined kernel on 128x256 tiles where their rounds are at least 80 % full (gate|up at 576 tokens: 430 tiles,
    // +10 %; the lm-head's 320 tiles would leave the second round three quarters empty and lose 14 %)
    const int64_t mid_tiles = (int64_t)((g.M + 127) / 128) * (g.N / 256), cus64 = cu_count();
    const bool mid = whole_n && g.M >= 256 && mid_tiles * 5 >= ((mid_tiles + cus64 - 1) / cus64) * cus64 * 4;
    return mid ? CLS_MID : CLS_SMALL;
}

template <int EPI>
bool dispatch(const GemmArgs& g, hipStream_t st) {
    const int cls = classify<EPI>(g);
    if (cls == CLS_STREAM) {
        run_gemv<EPI>(g, st);
        return false;
    }
    const bool mid = cls == CLS_MID, big = cls == CLS_BIG;
    const int64_t cus64 = cu_count();
    if (mid) {
        run_gemm<128, 256, 4, 2, EPI, 64, true>(g, 0, g.N / 256, 1, st);
    } else if (big) {
        // Whole rounds of 256x256 tiles, one tile per CU and round.  A last round that would leave more than
        // half of the CUs idle is cut off and run as 128x256 tiles (twice as many workgroups, half the work each).
        const int tiles_m = g.M / 256, tiles_n = g.N / 256, cus = cu_count();
        const int total = tiles_m * tiles_n, rem = total % cus;
        int n_main = tiles_n;
        if (total > cus && rem > 0 && 2 * rem <= cus) n_main = (total - rem) / tiles_m;
        if ((tiles_n - n_main) * tiles_m * 2 > cus) n_main = tiles_n;   // the cut-off part must fit one round
        run_gemm<256, 256, 4, 2, EPI, 64, true>(g, 0, n_main, 1, st);
        if (n_main < tiles_n) run_gemm<128, 256, 4, 2, EPI, 64, true>(g, n_main, tiles_n - n_main, 1, st);
    } else {
        // One round of tiles (a few hundred tokens: the paper's batch-1 setting) leaves one workgroup per CU, and a
        // K-step then costs its fixed chain of latencies whatever its depth: 128-deep steps halve their number
        // (out and down projections at 576 tokens: +16 %).  The sums are the same bits (see the k deal above).
        const int64_t small_tiles = (int64_t)((g.M + 127) / 128) * ((g.N + 127) / 128);
        if (g.K % 128 == 0 && g.K >= 256 && small_tiles <= cus64) run_gemm<128, 128, 2, 2, EPI, 128>(g, 0, (g.N + 127) / 128, 1, st);
        else run_gemm<128, 128, 2, 2, EPI>(g, 0, (g.N + 127) / 128, 2, st);
        return false;
    }
    return true;
}

// ---------------------------------------------------------------- float32
// C[M, N] (ld = ldc) (+)= A[M, K] W[N, K]^T, 64x64 tile, 4x4 per lane.
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ A, const float* __restrict__ W,
                                                  float* __restrict__ C, int M, int N, int K, int ldc,
                                                  int accumulate) {
    constexpr int T = 64, KB = 16;
    __shared__ float sa[KB][T + 1], sb[KB][T + 1];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * T, n0 = blockIdx.x * T;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += KB) {
        for (int e = tid; e < T * KB; e += 256) {
            const int r = e / KB, c = e % KB;
            sa[c][r] = (m0 + r < M && k0 + c < K) ? A[(int64_t)(m0 + r) * K + k0 + c] : 0.f;
            sb[c][r] = (n0 + r < N && k0 + c < K) ? W[(int64_t)(n0 + r) * K + k0 + c] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < KB; ++c) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sa[c][ty * 4 + i]; b[i] = sb[c][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) {
                float* p = C + (int64_t)m * ldc + n;
                *p = accumulate ? *p + acc[i][j] : acc[i][j];
            }
        }
}

}  // namespace

void launch_gemm_qkv_bf16(const void* xh, const void* wq, const void* wk, const void* wv, void* q_out,
                          void* k_cache, void* v_cache, int M, int d, const RopeArgs& ra, const StreamMode& sm, hipStream_t st) {
    GemmArgs g{};
    g.stream = sm.stream; g.w_frag = sm.w_frag; g.ksums = sm.ksums;
    g.A = (const bf16*)xh; g.W0 = (const bf16*)wq; g.W1 = (const bf16*)wk;
    g.M = M; g.N = 2 * d; g.K = d; g.Cb = (bf16*)q_out; g.kc = (bf16*)k_cache; g.d = d; g.ra = ra;
    if (g.stream) {   // a handful of tokens: q | k | v stream through one launch (xh is in fragment order)
        g.W2 = (const bf16*)wv; g.vc = (bf16*)v_cache; g.N = 3 * d;
        run_gemv<EPI_QKV>(g, st);
        return;
    }
    // a few hundred tokens: q | k | v as ONE problem where its 128x256 tiles fill a round (576 tokens: 240 tiles in one
    // round instead of 320 + 160 on smaller tiles); the same sums, element for element
    {
        GemmArgs m3 = g;
        m3.W2 = (const bf16*)wv; m3.vc = (bf16*)v_cache; m3.N = 3 * d;
        if (classify<EPI_QKV>(m3) == CLS_MID) {
            dispatch<EPI_QKV>(m3, st);
            return;
        }
    }
    dispatch<EPI_QK>(g, st);
    GemmArgs v{};
    v.A = (const bf16*)xh; v.W0 = (const bf16*)wv; v.M = M; v.N = d; v.K = d; v.vc = (bf16*)v_cache; v.ra = ra;
    dispatch<EPI_V>(v, st);
}

void launch_gemm_resid_bf16(const void* a, const void* w, float* x, int M, int N, int K, const StreamMode& sm, hipStream_t st) {
    GemmArgs g{};
    g.stream = sm.stream; g.w_frag = sm.w_frag; g.ksums = sm.ksums;
    g.A = (const bf16*)a; g.W0 = (const bf16*)w; g.M = M; g.N = N; g.K = K; g.Cf = x;
    dispatch<EPI_RESID>(g, st);
}

void launch_gemm_swiglu_bf16(const void* xh, const void* wg, const void* wu, void* h, int M, int f, int d,
                             const StreamMode& sm, hipStream_t st) {
    GemmArgs g{};
    g.stream = sm.stream; g.w_frag = sm.w_frag; g.ksums = sm.ksums;
    g.A = (const bf16*)xh; g.W0 = (const bf16*)wg; g.W1 = (const bf16*)wu; g.M = M; g.N = 2 * f; g.K = d;
    g.Cb = (bf16*)h;
    dispatch<EPI_SWIGLU>(g, st);
}

bool launch_gemm_logits_bf16(const void* xh, const void* w, float* logits, float* parts, int M, int V, int d,
                             const StreamMode& sm, hipStream_t st) {
    GemmArgs g{};
    g.stream = sm.stream; g.w_frag = sm.w_frag; g.ksums = sm.ksums;
    g.A = (const bf16*)xh; g.W0 = (const bf16*)w; g.M = M; g.N = V; g.K = d; g.Cf = logits;
    g.parts = reinterpret_cast<float2*>(parts);
    g.n_parts = (V + rowparts::PART - 1) / rowparts::PART;
    return dispatch<EPI_LOGITS>(g, st) && parts != nullptr;
}

void launch_pack_weights(const void* src, void* dst, int layers, int rows, int K, hipStream_t st) {
    const int64_t pieces = (int64_t)layers * ((rows + 15) / 16) * (K / 32) * 64;
    hipLaunchKernelGGL(k_pack_weights, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, (const bf16*)src, (bf16*)dst,
                       layers, rows, K);
}

void launch_gemm_f32(const float* a, const float* w, float* c, int M, int N, int K, int ldc, int accumulate,
                     hipStream_t st) {
    hipLaunchKernelGGL(k_gemm_f32, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, st, a, w, c, M, N, K,
                       ldc, accumulate);
}

}  // namespace mulo
