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

// out = x / sqrt(mean(x^2) + eps) * gain, one workgroup per row, float32 inside
template <typename T>
__global__ __launch_bounds__(TPB) void k_rmsnorm(const float* __restrict__ x, const T* __restrict__ gain,
                                                 T* __restrict__ out, int d, float eps) {
    __shared__ float red[TPB / 64];
    const int64_t m = blockIdx.x;
    const float* xr = x + m * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += TPB) { const float v = xr[c]; ss += v * v; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = (red[0] + red[1]) + (red[2] + red[3]);
    const float sc = 1.0f / sqrtf(ss / (float)d + eps);
    for (int c = threadIdx.x; c < d; c += TPB) st(out, m * d + c, xr[c] * sc * ld(gain, c));
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

void launch_rmsnorm(const float* x, const void* gain, int dtype, void* out, int M, int d, float eps,
                    hipStream_t s) {
    if (dtype == 1)
        hipLaunchKernelGGL(k_rmsnorm<__hip_bfloat16>, dim3(M), dim3(TPB), 0, s, x,
                           (const __hip_bfloat16*)gain, (__hip_bfloat16*)out, d, eps);
    else
        hipLaunchKernelGGL(k_rmsnorm<float>, dim3(M), dim3(TPB), 0, s, x, (const float*)gain, (float*)out,
                           d, eps);
}

void launch_rope_append_f32(const float* qkv, float* q_out, float* k_cache, float* v_cache, int M, int d,
                            const RopeArgs& ra, hipStream_t s) {
    hipLaunchKernelGGL(k_rope_append_f32, dim3(M), dim3(TPB), 0, s, qkv, q_out, k_cache, v_cache, d, ra);
}

void launch_swiglu_f32(const float* gu, float* h, int M, int f, hipStream_t s) {
    hipLaunchKernelGGL(k_swiglu_f32, dim3(M), dim3(TPB), 0, s, gu, h, f);
}

}  // namespace mulo
