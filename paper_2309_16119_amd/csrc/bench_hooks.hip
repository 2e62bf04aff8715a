// Benchmark hook: a plain streaming read of a device buffer, the measured ceiling that the
// M <= 16 streaming kernels' packed-weight GB/s is put beside.  No operation of the method.
#include "modulora.h"

#include <hip/hip_runtime.h>

#include "launch.h"

namespace mlr {

typedef uint32_t ru32x4 __attribute__((ext_vector_type(4)));

constexpr int READ_THREADS = 256;
constexpr int READ_UNROLL = 8;      // 16-byte loads in flight per thread

// Every thread reads 16-byte pieces with a grid stride (a wave reads 1 KB of contiguous bytes per
// load, non-temporal like the stream kernels' weight loads) and folds them into one word, so the
// loads cannot be dropped; one word per workgroup is stored.
__global__ __launch_bounds__(READ_THREADS) void bench_read_kernel(const ru32x4 *buf, size_t n16, uint32_t *sink) {
    const size_t stride = (size_t)gridDim.x * READ_THREADS;
    size_t i = (size_t)blockIdx.x * READ_THREADS + threadIdx.x;
    uint32_t acc = 0;
    for (; i + (READ_UNROLL - 1) * stride < n16; i += READ_UNROLL * stride) {
        ru32x4 v[READ_UNROLL];
#pragma unroll
        for (int u = 0; u < READ_UNROLL; ++u) v[u] = __builtin_nontemporal_load(buf + i + u * stride);
#pragma unroll
        for (int u = 0; u < READ_UNROLL; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    for (; i < n16; i += stride) {
        const ru32x4 v = __builtin_nontemporal_load(buf + i);
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_xor(acc, off, 64);
    __shared__ uint32_t part[READ_THREADS / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t a = 0;
        for (int w = 0; w < READ_THREADS / 64; ++w) a ^= part[w];
        sink[blockIdx.x] = a;
    }
}

}  // namespace mlr

extern "C" int modulora_bench_read(const void *buf, size_t bytes, uint32_t *sink, void *stream) {
    if (!buf || !sink) return MODULORA_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(buf) & 15u) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3u) != 0) return MODULORA_ERR_ALIGN;
    if (bytes < 16 || bytes % 16 != 0) return MODULORA_ERR_SHAPE;
    const size_t n16 = bytes / 16;
    // eight workgroups per compute unit, fewer for small buffers (one 16-byte piece per thread at least)
    size_t blocks = (n16 + mlr::READ_THREADS - 1) / mlr::READ_THREADS;
    if (blocks > MODULORA_BENCH_READ_SINK_WORDS) blocks = MODULORA_BENCH_READ_SINK_WORDS;
    mlr::launch_kernel("bench_read", mlr::bench_read_kernel, dim3((unsigned)blocks), dim3(mlr::READ_THREADS), 0,
                       static_cast<hipStream_t>(stream), static_cast<const mlr::ru32x4 *>(buf), n16, sink);
    return hipGetLastError() == hipSuccess ? MODULORA_OK : MODULORA_ERR_HIP;
}
