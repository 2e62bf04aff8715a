// Round-to-nearest group quantizer and packer: the quantizer side (the black-box Q of
// ModuLoRA Section 2.2) in its simplest form, the round-to-nearest baseline of the paper's
// quantizer ablation.  W float32 [N][K] -> packed codes, binary16 scales, uint8 zero points in
// the layout the layer kernels read.  Every decision is taken in IEEE float32 (correctly
// rounded subtract / divide, round half to even), so the result is defined bit for bit:
//     lo = min(group, 0), hi = max(group, 0)
//     scale = smallest binary16 >= max((hi - lo) / (2^b - 1), 2^-14)
//     zero  = clamp(rne(-lo / scale), 0, 2^b - 1)
//     q     = clamp(rne(w / scale) + zero, 0, 2^b - 1)
// Two bandwidth-bound passes over W: group statistics (a workgroup per row and run of groups,
// float4 loads along K), then quantize + pack (64 x 64 tiles: loads coalesced along K, codes
// turned through LDS, words stored coalesced along N).
#include <hip/hip_fp16.h>

#include "launch.h"

namespace mlr {

namespace {

__device__ __forceinline__ uint16_t f16_bits_round_up(float x) {
    const __half h = __float2half_rn(x);
    uint16_t bits = __half_as_ushort(h);
    if (__half2float(h) < x) bits += 1;   // positive finite: the next bit pattern is the next value
    return bits;
}

__device__ __forceinline__ float f16_bits_to_float(uint16_t bits) { return __half2float(__ushort_as_half(bits)); }

// ---- pass 1: scales and zero points --------------------------------------------------
// grid (N, runs of groups); a workgroup covers `gpb` whole groups of row n (gpb * g <= 1024
// floats, one float4 per thread) or, for g > 1024, one group in several sweeps.
__global__ __launch_bounds__(256) void rtn_stats_kernel(QuantArgs a, int gpb) {
    __shared__ float mn[256], mx[256];
    const int t = threadIdx.x, n = blockIdx.x;
    const int g = a.group, G = a.K / g;
    const int g_first = blockIdx.y * gpb;
    int ngroups = G - g_first;
    if (ngroups > gpb) ngroups = gpb;
    const int floats = ngroups * g;
    const float *row = a.W + (size_t)n * a.K + (size_t)g_first * g;
    float lo = 0.f, hi = 0.f;            // zero is always inside the range
    for (int i = 4 * t; i < floats; i += 1024) {
        const float4 v = *reinterpret_cast<const float4 *>(row + i);
        lo = fminf(fminf(lo, v.x), fminf(fminf(v.y, v.z), v.w));
        hi = fmaxf(fmaxf(hi, v.x), fmaxf(fmaxf(v.y, v.z), v.w));
    }
    mn[t] = lo;
    mx[t] = hi;
    __syncthreads();
    if (t >= ngroups) return;
    // entries of local group t: one float4 per thread when the run fits one sweep, else all
    int e0 = 0, e1 = 256;
    if (floats <= 1024) { e0 = t * (g / 4); e1 = e0 + g / 4; }
    lo = 0.f; hi = 0.f;
    for (int e = e0; e < e1; ++e) { lo = fminf(lo, mn[e]); hi = fmaxf(hi, mx[e]); }
    const float maxq = (float)((1 << a.bits) - 1);
    const float raw = __fdiv_rn(__fsub_rn(hi, lo), maxq);
    const uint16_t sbits = f16_bits_round_up(fmaxf(raw, 6.103515625e-05f));
    const float s = f16_bits_to_float(sbits);
    const float z = fminf(fmaxf(rintf(__fdiv_rn(-lo, s)), 0.f), maxq);
    const size_t o = (size_t)(g_first + t) * a.N + n;
    a.scales[o] = sbits;
    a.zeros[o] = (uint8_t)z;
}

// ---- pass 2: codes and bitstream -----------------------------------------------------
constexpr int QT = 64;            // tile: 64 output columns x 64 inputs (two 32-code blocks)
constexpr int QROW = QT / 4 + 1;  // LDS row stride in words (4 codes per word), padded

template <int BITS>
__global__ __launch_bounds__(256) void rtn_pack_kernel(QuantArgs a) {
    __shared__ uint32_t codes[QT][QROW];
    const int t = threadIdx.x;
    const int n0 = blockIdx.x * QT, k0 = blockIdx.y * QT;
    const float maxq = (float)((1 << BITS) - 1);
    const int f4 = t & 15, k = k0 + 4 * f4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int nl = (t >> 4) + 16 * i, n = n0 + nl;
        uint32_t packed4 = 0;
        if (n < a.N && k < a.K) {
            const float4 w = *reinterpret_cast<const float4 *>(a.W + (size_t)n * a.K + k);
            const size_t go = (size_t)(k / a.group) * a.N + n;
            const float s = f16_bits_to_float(a.scales[go]);
            const float z = (float)a.zeros[go];
            const float wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float q = fminf(fmaxf(rintf(__fdiv_rn(wv[e], s)) + z, 0.f), maxq);
                packed4 |= (uint32_t)q << (8 * e);
            }
        }
        codes[nl][f4] = packed4;
    }
    __syncthreads();
    if (t >= 2 * QT) return;
    const int nl = t & (QT - 1), blk = t >> 6;    // one 32-code block of one column per thread
    const int n = n0 + nl, kb = k0 + 32 * blk;
    if (n >= a.N || kb >= a.K) return;
    uint32_t out[BITS];
#pragma unroll
    for (int j = 0; j < BITS; ++j) out[j] = 0;
#pragma unroll
    for (int c = 0; c < 32; ++c) {
        const uint32_t q = (codes[nl][blk * 8 + c / 4] >> (8 * (c % 4))) & 0xFFu;
        const int pos = c * BITS, wd = pos >> 5, sh = pos & 31;
        out[wd] |= q << sh;
        if (sh + BITS > 32) out[wd + 1] |= q >> (32 - sh);
    }
    uint32_t *dst = a.qweight + (size_t)(kb / 32) * BITS * a.N + n;
#pragma unroll
    for (int j = 0; j < BITS; ++j) dst[(size_t)j * a.N] = out[j];
}

}  // namespace

hipError_t launch_quantize_rtn(const QuantArgs &a, hipStream_t stream) {
    const int G = a.K / a.group;
    int gpb = 1024 / a.group;
    if (gpb < 1) gpb = 1;
    launch_kernel("rtn_stats", rtn_stats_kernel, dim3(a.N, (G + gpb - 1) / gpb), dim3(256), 0, stream, a, gpb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 grid((a.N + QT - 1) / QT, (a.K + QT - 1) / QT);
    switch (a.bits) {
        case 2: launch_kernel("rtn_pack", rtn_pack_kernel<2>, grid, dim3(256), 0, stream, a); break;
        case 3: launch_kernel("rtn_pack", rtn_pack_kernel<3>, grid, dim3(256), 0, stream, a); break;
        default: launch_kernel("rtn_pack", rtn_pack_kernel<4>, grid, dim3(256), 0, stream, a); break;
    }
    return hipGetLastError();
}

}  // namespace mlr
