// Standalone weight materialization (test-only entry point modulora_dequant):
// the weight materialization step of Figure 1 (LPLinear.forward, before the product),
// written out to HBM as bfloat16 [N][K].  It exists so that unpacking and
// dequantization -- the same device functions the fused kernels use -- can be
// compared with the oracle bit for bit.
#include "device_common.h"
#include "launch.h"

namespace mlr {

// One thread per (column n, 32-code block kb): BITS word loads, coalesced along n,
// then 32 bfloat16 = 64 bytes stored to What[n][32*kb ...].
template <int BITS>
__global__ __launch_bounds__(256) void dequant_kernel(LayerView w, uint16_t *__restrict__ What) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int kb = blockIdx.y;
    if (n >= w.N) return;
    uint32_t words[BITS];
#pragma unroll
    for (int j = 0; j < BITS; ++j) words[j] = w.qweight[(size_t)(kb * BITS + j) * w.N + n];
    const int g = (kb * 32) / w.group;
    const DqConst c = make_dq(w.scales[(size_t)g * w.N + n], w.zeros[(size_t)g * w.N + n]);
    uint4 *dst = reinterpret_cast<uint4 *>(What + (size_t)n * w.K + (size_t)kb * 32);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t o[4];
        dequant_chunk<BITS>(block_chunk<BITS>(words, j), c, o);
        dst[j] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

hipError_t launch_dequant(const LayerView &w, uint16_t *What, hipStream_t stream) {
    dim3 grid((w.N + 255) / 256, w.K / 32);
    switch (w.bits) {
        case 2: launch_kernel("dequant", dequant_kernel<2>, grid, 256, 0, stream, w, What); break;
        case 3: launch_kernel("dequant", dequant_kernel<3>, grid, 256, 0, stream, w, What); break;
        default: launch_kernel("dequant", dequant_kernel<4>, grid, 256, 0, stream, w, What); break;
    }
    return hipGetLastError();
}

}  // namespace mlr
