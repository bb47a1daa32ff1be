// Row-wise pieces of the target forward (Alg. 1 Step 3): embedding lookup,
// RMSNorm, and -- for the float32 configuration only -- rotary + cache append and
// the SwiGLU product as separate kernels (the bf16 path fuses those into GEMM
// epilogues).  All are HBM-bound streams over [M, d] activations.
#include <hip/hip_bf16.h>

#include "mulo_internal.h"

namespace mulo {
namespace {

constexpr int TPB = 256;

__device__ __forceinline__ float ld(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld(const __hip_bfloat16* p, int64_t i) { return __bfloat162float(p[i]); }
__device__ __forceinline__ void st(float* p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st(__hip_bfloat16* p, int64_t i, float v) { p[i] = __float2bfloat16(v); }

template <typename T>
__global__ __launch_bounds__(TPB) void k_embed(const T* __restrict__ embed, const int32_t* __restrict__ tok,
                                               const T* __restrict__ in_embeds, float* __restrict__ x,
                                               int d, int V) {
    const int64_t m = blockIdx.x;
    const T* src;
    if (in_embeds) {
        src = in_embeds + m * d;
    } else {
        int t = tok[m];
        t = t < 0 ? 0 : (t >= V ? V - 1 : t);
        src = embed + (int64_t)t * d;
    }
    for (int c = threadIdx.x; c < d; c += TPB) x[m * d + c] = ld(src, c);
}

// out = x / sqrt(mean(x^2) + eps) * gain, one workgroup per row, float32 inside.  The row is read
// once with 16-byte loads and kept in registers (d <= 256 * 4 * NV4); NV4 == 0 re-reads it instead.
template <typename T, int NV4>
__global__ __launch_bounds__(TPB) void k_rmsnorm(const float* __restrict__ x, const T* __restrict__ gain,
                                                 T* __restrict__ out, int d, float eps, int frag) {
    __shared__ float red[TPB / 64];
    const int64_t m = blockIdx.x;
    const float* xr = x + m * d;
    const int nv4 = d >> 2, tid = threadIdx.x;
    float4 v[NV4 > 0 ? NV4 : 1];
    float ss = 0.f;
    if constexpr (NV4 > 0) {
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            const int idx = i * TPB + tid;
            v[i] = idx < nv4 ? reinterpret_cast<const float4*>(xr)[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
            ss += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
        }
    } else {
        for (int c = tid; c < d; c += TPB) { const float t = xr[c]; ss += t * t; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    ss = (red[0] + red[1]) + (red[2] + red[3]);
    const float sc = 1.0f / sqrtf(ss / (float)d + eps);
    if constexpr (NV4 > 0) {
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            const int idx = i * TPB + tid;
            if (idx < nv4) {
                const int c = idx * 4;
                const int64_t o = frag ? frag_index((int)m, c, d) : m * d + c;   // 4 | c: one run of 8 either way
                st(out, o, v[i].x * sc * ld(gain, c));
                st(out, o + 1, v[i].y * sc * ld(gain, c + 1));
                st(out, o + 2, v[i].z * sc * ld(gain, c + 2));
                st(out, o + 3, v[i].w * sc * ld(gain, c + 3));
            }
        }
    } else {
        for (int c = tid; c < d; c += TPB) st(out, frag ? frag_index((int)m, c, d) : m * d + c, xr[c] * sc * ld(gain, c));
    }
}

// float32 path: rotary on adjacent pairs of q and k, q -> [B, nh, L, dh],
// k -> cache [.., S, dh], v -> cache transposed [.., dh, S]
__global__ __launch_bounds__(TPB) void k_rope_append_f32(const float* __restrict__ qkv, float* __restrict__ q_out,
                                                         float* __restrict__ kc, float* __restrict__ vc,
                                                         int d, RopeArgs ra) {
    const int64_t m = blockIdx.x;
    const int b = m / ra.L, j = m % ra.L, pos = ra.P + j, dh = ra.head_dim, half = dh / 2;
    const float* row = qkv + m * 3 * d;
    for (int pr = threadIdx.x; pr < d / 2; pr += TPB) {
        const int hd = (2 * pr) / dh, c = (2 * pr) % dh, mm = c / 2;
        const float cs = ra.cos[(int64_t)pos * half + mm], sn = ra.sin[(int64_t)pos * half + mm];
        const float q0 = row[2 * pr], q1 = row[2 * pr + 1];
        const float k0 = row[d + 2 * pr], k1 = row[d + 2 * pr + 1];
        const int64_t qo = (((int64_t)b * ra.n_heads + hd) * ra.L + j) * dh + c;
        q_out[qo] = q0 * cs - q1 * sn;
        q_out[qo + 1] = q0 * sn + q1 * cs;
        const int64_t hb = ((int64_t)ra.layer * ra.max_batch + b) * ra.n_heads + hd;
        const int64_t ko = (hb * ra.max_seq + pos) * dh + c;
        kc[ko] = k0 * cs - k1 * sn;
        kc[ko + 1] = k0 * sn + k1 * cs;
        const int64_t vo = (hb * dh + c) * ra.max_seq + pos;
        vc[vo] = row[2 * d + 2 * pr];
        vc[vo + ra.max_seq] = row[2 * d + 2 * pr + 1];
    }
}

// h = silu(gate) * up from gu = [gate | up] rows of 2f floats
__global__ __launch_bounds__(TPB) void k_swiglu_f32(const float* __restrict__ gu, float* __restrict__ h, int f) {
    const int64_t m = blockIdx.x;
    for (int c = threadIdx.x; c < f; c += TPB) {
        const float g = gu[m * 2 * f + c], u = gu[m * 2 * f + f + c];
        h[m * f + c] = g / (1.0f + expf(-g)) * u;
    }
}

}  // namespace

void launch_embed(const void* embed, int dtype, const int32_t* tok, const void* in_embeds, float* x,
                  int M, int d, int V, hipStream_t s) {
    if (dtype == 1)
        hipLaunchKernelGGL(k_embed<__hip_bfloat16>, dim3(M), dim3(TPB), 0, s, (const __hip_bfloat16*)embed,
                           tok, (const __hip_bfloat16*)in_embeds, x, d, V);
    else
        hipLaunchKernelGGL(k_embed<float>, dim3(M), dim3(TPB), 0, s, (const float*)embed, tok,
                           (const float*)in_embeds, x, d, V);
}

template <typename T>
static void rmsnorm_dispatch(const float* x, const T* gain, T* out, int M, int d, float eps, int frag, hipStream_t s) {
    if ((d & 3) == 0 && d <= 1024) hipLaunchKernelGGL((k_rmsnorm<T, 1>), dim3(M), dim3(TPB), 0, s, x, gain, out, d, eps, frag);
    else if ((d & 3) == 0 && d <= 4096) hipLaunchKernelGGL((k_rmsnorm<T, 4>), dim3(M), dim3(TPB), 0, s, x, gain, out, d, eps, frag);
    else if ((d & 3) == 0 && d <= 8192) hipLaunchKernelGGL((k_rmsnorm<T, 8>), dim3(M), dim3(TPB), 0, s, x, gain, out, d, eps, frag);
    else hipLaunchKernelGGL((k_rmsnorm<T, 0>), dim3(M), dim3(TPB), 0, s, x, gain, out, d, eps, frag);
}

void launch_rmsnorm(const float* x, const void* gain, int dtype, void* out, int M, int d, float eps, bool frag,
                    hipStream_t s) {
    if (dtype == 1) rmsnorm_dispatch(x, (const __hip_bfloat16*)gain, (__hip_bfloat16*)out, M, d, eps, frag ? 1 : 0, s);
    else rmsnorm_dispatch(x, (const float*)gain, (float*)out, M, d, eps, 0, s);
}

void launch_rope_append_f32(const float* qkv, float* q_out, float* k_cache, float* v_cache, int M, int d,
                            const RopeArgs& ra, hipStream_t s) {
    hipLaunchKernelGGL(k_rope_append_f32, dim3(M), dim3(TPB), 0, s, qkv, q_out, k_cache, v_cache, d, ra);
}

void launch_swiglu_f32(const float* gu, float* h, int M, int f, hipStream_t s) {
    hipLaunchKernelGGL(k_swiglu_f32, dim3(M), dim3(TPB), 0, s, gu, h, f);
}

}  // namespace mulo
