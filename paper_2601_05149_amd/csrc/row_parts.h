// Row statistics of the target softmax (Sec. 3.1, Eq. 1: p = softmax(z)) in ONE fixed summation order that two
// producers share: the lm-head GEMM's epilogue, which has a tile of logits in registers, and the accept kernel, which
// reads a row of logits from memory.  Both must give the same bits, so that a verification step equals the
// composition of its stage entry points.
//
// A row of V logits is cut into parts of 128 columns.  Inside part p, column  p*128 + rr*16 + h*8 + e  belongs to
// half h (0, 1), run rr (0..7), element e (0..7): the layout in which a lane of the GEMM epilogue owns its
// accumulators.  For each half: the maximum m_h of its 64 columns, the sum t_rr of exp(z - m_h) over the 8 elements of
// each run in order, and the runs added as ((t0+t1)+(t2+t3))+((t4+t5)+(t6+t7)).  The halves are merged into the
// part's (m_p, s_p), and the parts into the row's (M, S) by one wavefront: lane l adds the parts l, l+64, ... in
// order, then a butterfly over the lanes.  Every operation is rounded on its own (no contraction).
#pragma once
#include <hip/hip_runtime.h>

namespace mulo {
namespace rowparts {

constexpr int PART = 128;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float NEG_INF = -__builtin_huge_valf();

// exp(z - m) with one hardware exp2, every step rounded on its own
__device__ __forceinline__ float expm(float z, float m) {
    return __builtin_amdgcn_exp2f(__fmul_rn(__fsub_rn(z, m), LOG2E));
}

// sum over the 8 elements of a run, in order; elements e >= n_valid do not exist
__device__ __forceinline__ float run_sum(const float (&z)[8], float m, int n_valid) {
    float t = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < n_valid) t = __fadd_rn(t, expm(z[e], m));
    return m == NEG_INF ? 0.f : t;
}

// the fixed tree over the 8 run sums of a half
__device__ __forceinline__ float tree8(const float (&t)[8]) {
    return __fadd_rn(__fadd_rn(__fadd_rn(t[0], t[1]), __fadd_rn(t[2], t[3])),
                     __fadd_rn(__fadd_rn(t[4], t[5]), __fadd_rn(t[6], t[7])));
}

// merge the two halves of a part; symmetric in its arguments
__device__ __forceinline__ float2 merge_halves(float m_a, float s_a, float m_b, float s_b) {
    const float m = fmaxf(m_a, m_b);
    if (m == NEG_INF) return make_float2(NEG_INF, 0.f);
    return make_float2(m, __fadd_rn(__fmul_rn(s_a, expm(m_a, m)), __fmul_rn(s_b, expm(m_b, m))));
}

// (M, S) of a row from its n_parts parts, by the 64 lanes of one wavefront (all lanes get the result)
__device__ __forceinline__ float2 combine_parts(const float2* parts, int n_parts, int lane) {
    float M = NEG_INF;
    for (int p = lane; p < n_parts; p += 64) M = fmaxf(M, parts[p].x);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
    float a = 0.f;
    for (int p = lane; p < n_parts; p += 64) {
        const float2 q = parts[p];
        a = __fadd_rn(a, __fmul_rn(q.y, expm(q.x, M)));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) a = __fadd_rn(a, __shfl_xor(a, o));
    return make_float2(M, a);
}

}  // namespace rowparts
}  // namespace mulo
