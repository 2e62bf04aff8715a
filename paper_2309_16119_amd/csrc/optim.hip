// AdamW step for the adapter factors (the optimizer named in the paper's Appendix
// hyper-parameter tables): Adam with decoupled weight decay on one flat fp32 buffer that
// holds every trainable A and B back to back, so a whole model's adapters take one launch.
// Purely bandwidth-bound: 16 bytes read and 12 written per element, 16-byte accesses.
#include "launch.h"

namespace mlr {

__device__ __forceinline__ void adamw_one(float &p, float g, float &m, float &v, const AdamWArgs &a) {
    m = __builtin_fmaf(a.one_minus_beta1, g, a.beta1 * m);
    v = __builtin_fmaf(a.one_minus_beta2 * g, g, a.beta2 * v);
    const float denom = __builtin_fmaf(__fsqrt_rn(v), a.inv_sqrt_bc2, a.eps);
    p = __builtin_fmaf(-a.step_size, __fdiv_rn(m, denom), p * a.decay);
}

__global__ __launch_bounds__(256) void adamw_kernel(AdamWArgs a) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= a.n) return;
    if (i + 4 <= a.n) {
        float4 p = *reinterpret_cast<const float4 *>(a.p + i);
        const float4 g = *reinterpret_cast<const float4 *>(a.g + i);
        float4 m = *reinterpret_cast<const float4 *>(a.m + i);
        float4 v = *reinterpret_cast<const float4 *>(a.v + i);
        adamw_one(p.x, g.x, m.x, v.x, a);
        adamw_one(p.y, g.y, m.y, v.y, a);
        adamw_one(p.z, g.z, m.z, v.z, a);
        adamw_one(p.w, g.w, m.w, v.w, a);
        *reinterpret_cast<float4 *>(a.p + i) = p;
        *reinterpret_cast<float4 *>(a.m + i) = m;
        *reinterpret_cast<float4 *>(a.v + i) = v;
        return;
    }
    for (size_t e = i; e < a.n; ++e) {   // ragged end: at most 3 elements
        float p = a.p[e], m = a.m[e], v = a.v[e];
        adamw_one(p, a.g[e], m, v, a);
        a.p[e] = p;
        a.m[e] = m;
        a.v[e] = v;
    }
}

hipError_t launch_adamw(const AdamWArgs &a, hipStream_t stream) {
    const size_t blocks = (a.n + 1023) / 1024;
    launch_kernel("adamw", adamw_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace mlr
