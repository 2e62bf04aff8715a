// The layer in the paper's own storage convention (Section 2.2 eq. (2), Section 3.2, Figure 1):
//
//     What[n][k] = binary16( fma(q[n][k], scale[g][n], z[g][n]) )        g = k div group
//     Y  = X What^T + bias + s (X A) B            dX = dY What + s (dY B^T) A^T
//
// with a floating (binary16) zero point z that is ADDED, binary16 scales, binary16 activations
// and outputs, an optional binary16 bias, and one (scale, z) pair per group of `group` inputs
// of an output column (group = d_in is the paper's one pair per row).  The packed codes are
// the same LSB-first bitstream as in the bfloat16 path.  What is materialized tile by tile in
// LDS and consumed by v_mfma_f32_32x32x16_f16; it never reaches HBM.
//
// This path has its own, plainer kernels (one tile shape, adapter term in the epilogue):
//   f16_dequant_kernel   test-only materialization of What
//   f16_proj_kernel      P = act F            (X A or dY B^T), fp32
//   f16_gemm_kernel      the two products with What, adapter term and bias in the epilogue
// The adapter gradients reuse lora_grad_partial_kernel with a binary16 element conversion.
#include "device_common.h"
#include "gemm_common.h"
#include "launch.h"

namespace mlr {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

namespace hf {

constexpr int THREADS = 256;
constexpr int MT = 128, CT = 128, RT = 64;     // output tile, contraction elements per step
constexpr int LROW = RT + 8;                   // LDS row stride in elements (144 B: conflict-free 16-byte accesses)
constexpr int TI = 2, TJ = 2;                  // 32 x 32 MFMA tiles of a wave's 64 x 64 tile

// two floats -> two binary16 (round to nearest even), `lo` in bits 0..15
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const _Float16 a = (_Float16)lo, b = (_Float16)hi;
    uint16_t ua, ub;
    __builtin_memcpy(&ua, &a, 2);
    __builtin_memcpy(&ub, &b, 2);
    return (uint32_t)ua | ((uint32_t)ub << 16);
}
__device__ __forceinline__ uint16_t to_bits(float v) { return (uint16_t)(pack2(v, 0.f) & 0xFFFFu); }

// one code: a single rounding to binary32 inside the fma, then one to binary16
__device__ __forceinline__ float affine(uint32_t q, float scale, float z) { return __builtin_fmaf((float)q, scale, z); }

// the 32 codes of a block (BITS words) -> 32 binary16 in 16 registers, code 0 in the low half of out[0]
template <int BITS>
__device__ __forceinline__ void dequant32(const uint32_t *w, float scale, float z, uint32_t out[16]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t chunk = block_chunk<BITS>(w, j);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            out[4 * j + i] = pack2(affine(chunk_code<BITS>(chunk, 2 * i), scale, z), affine(chunk_code<BITS>(chunk, 2 * i + 1), scale, z));
    }
}

}  // namespace hf

// ---------------------------------------------------------------------------------
// test-only materialization: What [N][K] binary16.  One thread per (column, 32-code block).
// ---------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(256) void f16_dequant_kernel(F16Layer w, uint16_t *What) {
    const int n = blockIdx.x * 256 + threadIdx.x, kb = blockIdx.y;
    if (n >= w.N) return;
    uint32_t words[BITS];
#pragma unroll
    for (int q = 0; q < BITS; ++q) words[q] = w.qweight[((size_t)kb * BITS + q) * w.N + n];
    const int g = kb * 32 / w.group;
    const float scale = half_bits_to_float(w.scales[(size_t)g * w.N + n]);
    const float z = half_bits_to_float(w.zeros[(size_t)g * w.N + n]);
    uint32_t o[16];
    hf::dequant32<BITS>(words, scale, z, o);
    uint4 *dst = reinterpret_cast<uint4 *>(What + (size_t)n * w.K + kb * 32);
#pragma unroll
    for (int j = 0; j < 4; ++j) dst[j] = make_uint4(o[4 * j], o[4 * j + 1], o[4 * j + 2], o[4 * j + 3]);
}

hipError_t launch_f16_dequant(const F16Layer &w, uint16_t *What, hipStream_t stream) {
    dim3 grid((w.N + 255) / 256, w.K / 32);
    switch (w.bits) {
        case 2: launch_kernel("f16_dequant", f16_dequant_kernel<2>, grid, 256, 0, stream, w, What); break;
        case 3: launch_kernel("f16_dequant", f16_dequant_kernel<3>, grid, 256, 0, stream, w, What); break;
        default: launch_kernel("f16_dequant", f16_dequant_kernel<4>, grid, 256, 0, stream, w, What); break;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// P[m][j] = sum_c act[m][c] F(c, j):  F = A [C][r] (F_IS_A) or B^T with B [r][C].
// A workgroup owns 4 rows; every thread walks the contraction in chunks of 8 elements
// (16-byte activation loads), keeps 4 x 8 fp32 sums per pass of 8 rank columns, and the 256
// threads' sums meet through wave shuffles and LDS.
// ---------------------------------------------------------------------------------
template <bool F_IS_A>
__global__ __launch_bounds__(256) void f16_proj_kernel(const uint16_t *act, int M, int C, const float *F, int r, float *P) {
    constexpr int RB = 4, RJ = 8;
    __shared__ float red[4][RB * RJ];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.x * RB;
    const uint16_t *rows[RB];
#pragma unroll
    for (int i = 0; i < RB; ++i) rows[i] = act + (size_t)(m0 + i < M ? m0 + i : M - 1) * C;
    for (int j0 = 0; j0 < r; j0 += RJ) {
        float acc[RB][RJ];
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
            for (int j = 0; j < RJ; ++j) acc[i][j] = 0.f;
        for (int c = tid * 8; c < C; c += 256 * 8) {       // C is a multiple of 8
            float x[RB][8];
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const uint4 v = *reinterpret_cast<const uint4 *>(rows[i] + c);
                const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x[i][2 * e] = half_bits_to_float((uint16_t)(wv[e] & 0xFFFFu));
                    x[i][2 * e + 1] = half_bits_to_float((uint16_t)(wv[e] >> 16));
                }
            }
#pragma unroll
            for (int j = 0; j < RJ; ++j) {
                if (j0 + j >= r) break;
                float f[8];
                if (F_IS_A) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[e] = F[(size_t)(c + e) * r + j0 + j];
                } else {
                    const float4 q0 = *reinterpret_cast<const float4 *>(F + (size_t)(j0 + j) * C + c);
                    const float4 q1 = *reinterpret_cast<const float4 *>(F + (size_t)(j0 + j) * C + c + 4);
                    f[0] = q0.x; f[1] = q0.y; f[2] = q0.z; f[3] = q0.w;
                    f[4] = q1.x; f[5] = q1.y; f[6] = q1.z; f[7] = q1.w;
                }
#pragma unroll
                for (int i = 0; i < RB; ++i)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i][j] = __builtin_fmaf(x[i][e], f[e], acc[i][j]);
            }
        }
        // wave sums, then the four waves through LDS
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
            for (int j = 0; j < RJ; ++j) {
                float v = acc[i][j];
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
                if (lane == 0) red[wave][i * RJ + j] = v;
            }
        __syncthreads();
        if (tid < RB * RJ) {
            const int i = tid / RJ, j = tid % RJ;
            if (m0 + i < M && j0 + j < r) P[(size_t)(m0 + i) * r + j0 + j] = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
        }
        __syncthreads();
    }
}

hipError_t launch_f16_proj(const uint16_t *act, int M, int C, const float *F, bool f_is_A, int r, float *P, hipStream_t stream) {
    const int blocks = (M + 3) / 4;
    if (f_is_A) launch_kernel("f16_proj", f16_proj_kernel<true>, blocks, 256, 0, stream, act, M, C, F, r, P);
    else launch_kernel("f16_proj", f16_proj_kernel<false>, blocks, 256, 0, stream, act, M, C, F, r, P);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// out[M][Cout] = act[M][C] (x) What (+ bias) + s P F':
//   forward : C = K, Cout = N, out[m][n] = sum_k act[m][k] What[n][k] + bias[n] + s sum_j P[m][j] B[j][n]
//   backward: C = N, Cout = K, out[m][k] = sum_n act[m][n] What[n][k]           + s sum_j P[m][j] A[k][j]
// 256 threads, 128 x 128 output tile, four waves of 64 x 64; per step of 64 contraction elements
// the activation tile and the dequantized weight tile go through LDS ([row][contraction],
// padded rows); the next step's global data is fetched into registers while the MFMAs of
// the current one run.  Weight staging units, one per thread and step: forward (column, 32-code
// block); backward (n, 32-code block of k), whose 32 values go to 32 LDS rows.
// ---------------------------------------------------------------------------------
struct F16GemmArgs {
    F16Layer w;
    const uint16_t *act;      // binary16 [M][C]
    int M;
    uint16_t *out;            // binary16 [M][Cout]
    const float *P;           // fp32 [M][r] (NULL when r == 0)
    const float *Fm;          // forward: B [r][N]; backward: A [K][r]
    int r;
    float lora_scale;
    int tiles_m, tiles_c;
};

template <int BITS, bool BWD>
__global__ __launch_bounds__(hf::THREADS) void f16_gemm_kernel(F16GemmArgs a) {
    using namespace hf;
    __shared__ __attribute__((aligned(16))) uint16_t smem[(MT + CT) * LROW];   // 36 KB
    uint16_t *As = smem, *Ws = smem + MT * LROW;
    const TileCoord tcoord = tile_of_block(blockIdx.x, a.tiles_m, a.tiles_c);
    if (tcoord.tm < 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const int m0 = tcoord.tm * MT, c0 = tcoord.tc * CT;
    const int K = a.w.K, N = a.w.N;
    const int C = BWD ? N : K, Cout = BWD ? K : N;
    const int n_steps = (C + RT - 1) / RT;

    // activation chunks of this thread: 4 x 16 bytes, chunk idx = tid + 256 i -> row idx / 8, piece idx % 8
    const uint16_t *a_src[4];
    int a_col[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + i * THREADS, row = idx >> 3, ch = idx & 7;
        const int m = m0 + row < a.M ? m0 + row : a.M - 1;
        a_src[i] = a.act + (size_t)m * C + ch * 8;
        a_col[i] = ch * 8;
    }
    // weight unit of this thread
    const int u_lo = BWD ? (tid & 63) : (tid & 127);     // forward: column of the tile; backward: n of the step
    const int u_kb = BWD ? (tid >> 6) : (tid >> 7);      // forward: block of the step (0, 1); backward: k block of the tile (0..3)
    int w_col = 0, kblk = 0, grp_fixed = 0;
    if (!BWD) {
        w_col = c0 + u_lo < N ? c0 + u_lo : N - 1;       // clamped; never stored
    } else {
        const int k = c0 + u_kb * 32 < K ? c0 + u_kb * 32 : K - 32;
        kblk = k >> 5;
        grp_fixed = k / a.w.group;
    }

    uint4 a_reg[4];
    uint32_t w_reg[BITS];
    uint32_t sc_reg = 0, z_reg = 0;
    bool w_ok = false;
    auto fetch = [&](int step) {
        const int r0 = step * RT;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a_reg[i] = make_uint4(0, 0, 0, 0);
            if (r0 + a_col[i] < C) a_reg[i] = *reinterpret_cast<const uint4 *>(a_src[i] + r0);
        }
        if (!BWD) {
            const int k = r0 + u_kb * 32;
            w_ok = k < K;
            const int kb = w_ok ? (k >> 5) : 0;
#pragma unroll
            for (int q = 0; q < BITS; ++q) w_reg[q] = a.w.qweight[((size_t)kb * BITS + q) * N + w_col];
            const int g = (kb * 32) / a.w.group;
            sc_reg = a.w.scales[(size_t)g * N + w_col];
            z_reg = a.w.zeros[(size_t)g * N + w_col];
        } else {
            const int n = r0 + u_lo;
            w_ok = n < N;
            const int nc = w_ok ? n : N - 1;
#pragma unroll
            for (int q = 0; q < BITS; ++q) w_reg[q] = a.w.qweight[((size_t)kblk * BITS + q) * N + nc];
            sc_reg = a.w.scales[(size_t)grp_fixed * N + nc];
            z_reg = a.w.zeros[(size_t)grp_fixed * N + nc];
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + i * THREADS, row = idx >> 3;
            *reinterpret_cast<uint4 *>(As + row * LROW + a_col[i]) = a_reg[i];
        }
        uint32_t o[16];
        dequant32<BITS>(w_reg, half_bits_to_float((uint16_t)sc_reg), half_bits_to_float((uint16_t)z_reg), o);
        if (!w_ok) {
#pragma unroll
            for (int e = 0; e < 16; ++e) o[e] = 0;
        }
        if (!BWD) {
            uint4 *dst = reinterpret_cast<uint4 *>(Ws + u_lo * LROW + u_kb * 32);
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[j] = make_uint4(o[4 * j], o[4 * j + 1], o[4 * j + 2], o[4 * j + 3]);
        } else {
            // value kk of the block belongs to output column (LDS row) 32 u_kb + kk, contraction element u_lo
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                Ws[(u_kb * 32 + 2 * e) * LROW + u_lo] = (uint16_t)(o[e] & 0xFFFFu);
                Ws[(u_kb * 32 + 2 * e + 1) * LROW + u_lo] = (uint16_t)(o[e] >> 16);
            }
        }
    };

    f32x16 acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int wm = wave >> 1, wn = wave & 1;
    const int a_frag = (wm * 64 + (lane & 31)) * LROW + 8 * (lane >> 5);
    const int w_frag = (wn * 64 + (lane & 31)) * LROW + 8 * (lane >> 5);

    fetch(0);
    for (int step = 0; step < n_steps; ++step) {
        stage();
        __syncthreads();
        if (step + 1 < n_steps) fetch(step + 1);
#pragma unroll
        for (int ks = 0; ks < RT / 16; ++ks) {
            f16x8 af[TI], bf[TJ];
#pragma unroll
            for (int i = 0; i < TI; ++i) af[i] = *reinterpret_cast<const f16x8 *>(As + a_frag + i * 32 * LROW + ks * 16);
#pragma unroll
            for (int j = 0; j < TJ; ++j) bf[j] = *reinterpret_cast<const f16x8 *>(Ws + w_frag + j * 32 * LROW + ks * 16);
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // ---- epilogue: adapter term (P tile through LDS), bias, one rounding to binary16 -------------
    static_assert((MT + CT) * LROW * 2 >= MT * 64 * 4, "the P tile fits the tile buffers");
    float *Ps = reinterpret_cast<float *>(smem);         // [MT][r], r <= 64: at most 32 KB of the 36 KB
    const int r = a.r;
    if (r > 0) {
        for (int x = tid; x < MT * r; x += THREADS) {
            const int row = x / r, j = x - row * r;
            const int m = m0 + row < a.M ? m0 + row : a.M - 1;
            Ps[x] = a.P[(size_t)m * r + j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
        const int col = c0 + wn * 64 + j * 32 + (lane & 31);
        const bool col_ok = col < Cout;
        const int cc = col_ok ? col : Cout - 1;
        float lora[TI][16];
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) lora[i][v] = 0.f;
        for (int jj = 0; jj < r; ++jj) {
            const float f = BWD ? a.Fm[(size_t)cc * r + jj] : a.Fm[(size_t)jj * N + cc];
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int prow = wm * 64 + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
                    lora[i][v] = __builtin_fmaf(Ps[prow * r + jj], f, lora[i][v]);
                }
        }
        float bias = 0.f;
        if (!BWD && a.w.bias != nullptr) bias = half_bits_to_float(a.w.bias[cc]);
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
                if (col_ok && m < a.M) a.out[(size_t)m * Cout + col] = to_bits(__builtin_fmaf(a.lora_scale, lora[i][v], acc[i][j][v] + bias));
            }
    }
}

template <int BITS>
static hipError_t launch_f16_gemm_bits(F16GemmArgs &a, bool backward, hipStream_t stream) {
    const int blocks = ((a.tiles_m * a.tiles_c + 7) / 8) * 8;
    if (backward) launch_kernel("f16_gemm_bwd", f16_gemm_kernel<BITS, true>, blocks, hf::THREADS, 0, stream, a);
    else launch_kernel("f16_gemm_fwd", f16_gemm_kernel<BITS, false>, blocks, hf::THREADS, 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_f16_gemm(const F16Layer &w, bool backward, const uint16_t *act, int M, uint16_t *out, const float *P,
                           const float *Fm, int r, float lora_scale, hipStream_t stream) {
    F16GemmArgs a;
    a.w = w; a.act = act; a.M = M; a.out = out; a.P = P; a.Fm = Fm; a.r = r; a.lora_scale = lora_scale;
    const int Cout = backward ? w.K : w.N;
    a.tiles_m = (M + hf::MT - 1) / hf::MT;
    a.tiles_c = (Cout + hf::CT - 1) / hf::CT;
    switch (w.bits) {
        case 2: return launch_f16_gemm_bits<2>(a, backward, stream);
        case 3: return launch_f16_gemm_bits<3>(a, backward, stream);
        default: return launch_f16_gemm_bits<4>(a, backward, stream);
    }
}

}  // namespace mlr
