// Dense projections of the target forward (Alg. 1 Step 3): C = A[M,K] W[N,K]^T.
//
// bf16 path: LDS-staged tiles feeding v_mfma_f32_32x32x16_bf16 (64-lane
// wavefronts; both operands are K-contiguous so every lane fetches its 8-element
// fragment with one 16-byte LDS read), float32 accumulation, and the element-wise
// neighbours of each projection fused into the epilogue:
//   QKV    -> rotary on adjacent pairs + scatter to q buffer / K cache / V^T cache
//   out, down -> residual add into the float32 stream
//   gate|up   -> silu(gate) * up, gate and up columns interleaved inside a tile so
//                that one lane owns both accumulators of a feed-forward column
//   lm-head   -> float32 logits
// float32 path (small configuration): a plain register-tiled kernel.
#include <hip/hip_bf16.h>

#include <utility>

#include "mulo_internal.h"

namespace mulo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __hip_bfloat16 bf16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

enum { EPI_QK = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3, EPI_V = 4 };

struct GemmArgs {
    const bf16* A;        // [M, K]
    const bf16* W0;       // QK: wq | SWIGLU: w_gate | else: W [N, K]
    const bf16* W1;       // QK: wk | SWIGLU: w_up
    int M, N, K;          // N: output columns of the fused problem (QK: 2d, SWIGLU: 2f)
    float* Cf;            // RESID: x [M, N] (+=) | LOGITS: logits [M, N]
    bf16* Cb;             // SWIGLU: h [M, N/2] | QK: q buffer
    bf16* kc;             // QK: K cache
    bf16* vc;             // V: V^T cache
    int d;                // QK: model width (segment size)
    RopeArgs ra;
};

constexpr int BK = 64;
constexpr int LDS_STRIDE = BK + 8;  // bf16 elements per tile row: 144 B keeps 16-byte reads conflict-free

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

__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM* WGN * 64) void k_gemm_bf16(const GemmArgs g) {
    constexpr bool SWAP = EPI == EPI_V;
    constexpr int NT = WGM * WGN * 64;
    constexpr int TM = BM / WGM, TN = BN / WGN, MB = TM / 32, NB = TN / 32;
    constexpr int LA = BM * 8 / NT, LB = BN * 8 / NT;  // 16-byte chunks per lane per stage
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads");
    static_assert(EPI != EPI_SWIGLU || NB % 2 == 0, "swiglu needs an even number of column blocks");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16* sA = reinterpret_cast<bf16*>(smem);                 // [2][BM][LDS_STRIDE]
    bf16* sB = sA + 2 * BM * LDS_STRIDE;                      // [2][BN][LDS_STRIDE]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN, l32 = lane & 31, lh = lane >> 5;

    const int tiles_m = (g.M + BM - 1) / BM;
    const int tile_m = blockIdx.x % tiles_m, tile_n = blockIdx.x / tiles_m;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;  // first fused output column of this tile

    // per-lane source rows of the two operand tiles (fixed over the K loop)
    const int kc8 = (tid & 7) * 8;
    const bf16* pa[LA];
    const bf16* pb[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        int r = m0 + (tid >> 3) + i * (NT / 8);
        r = r < g.M ? r : g.M - 1;
        pa[i] = g.A + (int64_t)r * g.K + kc8;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int nl = (tid >> 3) + i * (NT / 8);  // row of the B tile
        const bf16* base;
        int r;
        if constexpr (EPI == EPI_QK) {
            const int seg = n0 / g.d;
            base = seg == 0 ? g.W0 : g.W1;
            r = n0 - seg * g.d + nl;
        } else if constexpr (EPI == EPI_SWIGLU) {
            // tile covers feed-forward columns [f0, f0 + BN/2); wave wn owns TN/2 of
            // them, gate rows in its first NB/2 blocks and up rows in the rest
            const int f = g.N / 2, f0 = tile_n * (BN / 2);
            const int w_ = nl / TN, within = nl % TN;
            const bool up = within >= TN / 2;
            r = f0 + w_ * (TN / 2) + (within % (TN / 2));
            r = r < f ? r : f - 1;
            base = up ? g.W1 : g.W0;
        } else {
            base = g.W0;
            r = n0 + nl;
            r = r < g.N ? r : g.N - 1;
        }
        pb[i] = base + (int64_t)r * g.K + kc8;
    }

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    u32x4 ra[LA], rb[LB];
    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < LA; ++i) ra[i] = *reinterpret_cast<const u32x4*>(pa[i] + kt * BK);
#pragma unroll
        for (int i = 0; i < LB; ++i) rb[i] = *reinterpret_cast<const u32x4*>(pb[i] + kt * BK);
    };
    auto sstore = [&](int buf) {
        bf16* a = sA + buf * BM * LDS_STRIDE;
        bf16* b = sB + buf * BN * LDS_STRIDE;
#pragma unroll
        for (int i = 0; i < LA; ++i)
            *reinterpret_cast<u32x4*>(a + ((tid >> 3) + i * (NT / 8)) * LDS_STRIDE + kc8) = ra[i];
#pragma unroll
        for (int i = 0; i < LB; ++i)
            *reinterpret_cast<u32x4*>(b + ((tid >> 3) + i * (NT / 8)) * LDS_STRIDE + kc8) = rb[i];
    };

    // one k-step (16 of the 64 staged columns) of fragments, double-buffered in registers so
    // that the LDS reads of step kk+1 are in flight while the MFMAs of step kk issue
    bf16x8 af[2][MB], bfr[2][NB];
    auto lfrag = [&](const bf16* a, const bf16* b, int kk, int slot) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
            af[slot][i] = *reinterpret_cast<const bf16x8*>(a + i * 32 * LDS_STRIDE + kk * 16);
#pragma unroll
        for (int j = 0; j < NB; ++j)
            bfr[slot][j] = *reinterpret_cast<const bf16x8*>(b + j * 32 * LDS_STRIDE + kk * 16);
    };

    const int nk = g.K / BK;
    gload(0);
    sstore(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) gload(kt + 1);
        const bf16* a = sA + (kt & 1) * BM * LDS_STRIDE + (wm * TM + l32) * LDS_STRIDE + lh * 8;
        const bf16* b = sB + (kt & 1) * BN * LDS_STRIDE + (wn * TN + l32) * LDS_STRIDE + lh * 8;
        lfrag(a, b, 0, 0);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            if (kk + 1 < BK / 16) lfrag(a, b, kk + 1, (kk + 1) & 1);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    if constexpr (SWAP)   // D[n][m]: lanes run over rows of A (tokens)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
                    else                  // D[m][n]: lanes run over rows of W (output columns)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
                }
        }
        if (kt + 1 < nk) sstore((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue.  Accumulator r of a 32x32 block: row (r/4)*8 + lh*4 + r%4, column l32.
    constexpr int NBE = EPI == EPI_SWIGLU ? NB / 2 : NB;   // gate blocks only: up blocks are consumed with them
    static_for<MB>([&](auto ic) {
        static_for<NBE>([&](auto jc) {
            constexpr int i = decltype(ic)::value, j = decltype(jc)::value;
            const int nl = wn * TN + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * TM + i * 32 + (r >> 2) * 8 + lh * 4 + (r & 3);
                const float v = acc[i][j][r];
                if constexpr (EPI == EPI_RESID) {
                    const int n = n0 + nl;
                    if (m < g.M && n < g.N) g.Cf[(int64_t)m * g.N + n] += v;
                } else if constexpr (EPI == EPI_LOGITS) {
                    const int n = n0 + nl;
                    if (m < g.M && n < g.N) g.Cf[(int64_t)m * g.N + n] = v;
                } else if constexpr (EPI == EPI_SWIGLU) {
                    const int f = g.N / 2;
                    const int n = tile_n * (BN / 2) + wn * (TN / 2) + j * 32 + l32;
                    const float u = acc[i][j + NB / 2][r];
                    if (m < g.M && n < f) g.Cb[(int64_t)m * f + n] = __float2bfloat16(silu(v) * u);
                } else if constexpr (EPI == EPI_QK) {
                    // rotary on adjacent column pairs (partner lane), q -> [B, nh, L, dh], k -> cache rows
                    const int n = n0 + nl, seg = n / g.d, c = n - seg * g.d;
                    const int dh = g.ra.head_dim, hd = c / dh, cc = c % dh;
                    const float partner = __shfl_xor(v, 1);
                    if (m < g.M) {
                        const int b = m / g.ra.L, jj = m % g.ra.L, pos = g.ra.P + jj;
                        const float cs = g.ra.cos[(int64_t)pos * (dh / 2) + (cc >> 1)];
                        const float sn = g.ra.sin[(int64_t)pos * (dh / 2) + (cc >> 1)];
                        const bf16 ob = __float2bfloat16((cc & 1) ? partner * sn + v * cs : v * cs - partner * sn);
                        if (seg == 0) {
                            g.Cb[(((int64_t)b * g.ra.n_heads + hd) * g.ra.L + jj) * dh + cc] = ob;
                        } else {
                            const int64_t hb = ((int64_t)g.ra.layer * g.ra.max_batch + b) * g.ra.n_heads + hd;
                            g.kc[(hb * g.ra.max_seq + pos) * dh + cc] = ob;
                        }
                    }
                } else {  // EPI_V: operands swapped, so row index = output column, lane = token:
                          // consecutive lanes write consecutive positions of a V^T cache row
                    const int n = n0 + wn * TN + j * 32 + (r >> 2) * 8 + lh * 4 + (r & 3);
                    const int mm = m0 + wm * TM + i * 32 + l32;
                    if (mm < g.M && n < g.N) {
                        const int dh = g.ra.head_dim, hd = n / dh, cc = n % dh;
                        const int b = mm / g.ra.L, pos = g.ra.P + mm % g.ra.L;
                        const int64_t hb = ((int64_t)g.ra.layer * g.ra.max_batch + b) * g.ra.n_heads + hd;
                        g.vc[(hb * dh + cc) * g.ra.max_seq + pos] = __float2bfloat16(v);
                    }
                }
            }
        });
    });
}

template <int BM, int BN, int WGM, int WGN, int EPI>
void run_gemm(const GemmArgs& g, int tiles_n, hipStream_t st) {
    auto kern = k_gemm_bf16<BM, BN, WGM, WGN, EPI>;
    const size_t lds = (size_t)2 * (BM + BN) * LDS_STRIDE * sizeof(bf16);
    static bool attr_set = false;  // one context per process configures each instantiation once
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const int tiles_m = (g.M + BM - 1) / BM;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(WGM * WGN * 64), lds, st, g);
}

template <int EPI>
void dispatch(const GemmArgs& g, hipStream_t st) {
    // large problems: 256x256 tiles, 8 wavefronts (4x2, 64x128 each: two per SIMD so one can
    // issue MFMAs while the other waits on LDS); small ones: 128x128 tiles, 4 wavefronts
    const bool big = g.M >= 1024 && (EPI == EPI_QK ? g.d % 256 == 0 : true);
    if (big) run_gemm<256, 256, 4, 2, EPI>(g, (g.N + 255) / 256, st);
    else run_gemm<128, 128, 2, 2, EPI>(g, (g.N + 127) / 128, st);
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
                          void* k_cache, void* v_cache, int M, int d, const RopeArgs& ra, hipStream_t st) {
    GemmArgs g{};
    g.A = (const bf16*)xh; g.W0 = (const bf16*)wq; g.W1 = (const bf16*)wk;
    g.M = M; g.N = 2 * d; g.K = d; g.Cb = (bf16*)q_out; g.kc = (bf16*)k_cache; g.d = d; g.ra = ra;
    dispatch<EPI_QK>(g, st);
    GemmArgs v{};
    v.A = (const bf16*)xh; v.W0 = (const bf16*)wv; v.M = M; v.N = d; v.K = d; v.vc = (bf16*)v_cache; v.ra = ra;
    dispatch<EPI_V>(v, st);
}

void launch_gemm_resid_bf16(const void* a, const void* w, float* x, int M, int N, int K, hipStream_t st) {
    GemmArgs g{};
    g.A = (const bf16*)a; g.W0 = (const bf16*)w; g.M = M; g.N = N; g.K = K; g.Cf = x;
    dispatch<EPI_RESID>(g, st);
}

void launch_gemm_swiglu_bf16(const void* xh, const void* wg, const void* wu, void* h, int M, int f, int d,
                             hipStream_t st) {
    GemmArgs g{};
    g.A = (const bf16*)xh; g.W0 = (const bf16*)wg; g.W1 = (const bf16*)wu; g.M = M; g.N = 2 * f; g.K = d;
    g.Cb = (bf16*)h;
    dispatch<EPI_SWIGLU>(g, st);
}

void launch_gemm_logits_bf16(const void* xh, const void* w, float* logits, int M, int V, int d,
                             hipStream_t st) {
    GemmArgs g{};
    g.A = (const bf16*)xh; g.W0 = (const bf16*)w; g.M = M; g.N = V; g.K = d; g.Cf = logits;
    dispatch<EPI_LOGITS>(g, st);
}

void launch_gemm_f32(const float* a, const float* w, float* c, int M, int N, int K, int ldc, int accumulate,
                     hipStream_t st) {
    hipLaunchKernelGGL(k_gemm_f32, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, st, a, w, c, M, N, K,
                       ldc, accumulate);
}

}  // namespace mulo
