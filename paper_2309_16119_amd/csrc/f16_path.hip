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
//   f16_gemm_kernel      the two products with What, adapter term and bias in the epilogue
// The projections P = act F (X A or dY B^T) reuse lora_down_kernel, each binary16 activation split
// exactly into two bfloat16 operands; the adapter gradients reuse lora_grad_partial_kernel with a
// binary16 element conversion.
#include "device_common.h"
#include "gemm_common.h"
#include <cstdlib>

#include "launch.h"

namespace mlr {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

namespace hf {

constexpr int THREADS = 256;
constexpr int CT = 128, RT = 64;               // output columns of a tile, contraction elements per step
constexpr int LROW = RT + 8;                   // LDS row stride in elements (144 B: conflict-free 16-byte accesses)

// two floats -> two binary16 (round to nearest even), `lo` in bits 0..15
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f16x2 v = {(_Float16)lo, (_Float16)hi};        // v_fma_mixlo_f16 / v_fma_mixhi_f16 when fed by an fma
    uint32_t u;
    __builtin_memcpy(&u, &v, 4);
    return u;
}
__device__ __forceinline__ uint16_t to_bits(float v) { return (uint16_t)(pack2(v, 0.f) & 0xFFFFu); }

// Loads issued from inline assembly (full per-lane address).  The compiler does not track
// them: a consumer sits behind wait_vm<N>() followed by tie() of every destination register.
// Loads return in order, so waiting until at most N remain outstanding completes everything
// issued before the N most recent ones.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void ld128(u32x4 &dst, const void *p) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void ld32(uint32_t &dst, const void *p) {
    asm volatile("global_load_dword %0, %1, off" : "=v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void ld16(uint32_t &dst, const void *p) {
    asm volatile("global_load_ushort %0, %1, off" : "=v"(dst) : "v"(p) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
template <typename T>
__device__ __forceinline__ void tie(T &x) {
    asm volatile("" : "+v"(x)::"memory");
}

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
// out[M][Cout] = act[M][C] (x) What (+ bias) + s P F':
//   forward : C = K, Cout = N, out[m][n] = sum_k act[m][k] What[n][k] + bias[n] + s sum_j P[m][j] B[j][n]
//   backward: C = N, Cout = K, out[m][k] = sum_n act[m][n] What[n][k]           + s sum_j P[m][j] A[k][j]
// 256 threads, MT x 128 output tile (MT = 128: four waves of 64 x 64; MT = 64, for shapes
// with few tiles: four waves of 64 x 32); per step of 64 contraction elements the activation
// tile and the dequantized weight tile go through LDS ([row][contraction], padded rows, two
// buffers): the next step's global data is fetched into registers before the MFMAs of the
// current step are issued and dequantized into the other buffer behind them, one barrier per step.  Weight staging units, one per thread and step: forward (column, 32-code
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

template <int BITS, bool BWD, int MT>
__global__ __launch_bounds__(hf::THREADS) void f16_gemm_kernel(F16GemmArgs a) {
    using namespace hf;
    constexpr int WAVES_M = MT / 64, WAVES_N = 4 / WAVES_M;        // wave grid over the tile
    constexpr int TI = 2, TJ = CT / WAVES_N / 32;                  // 32 x 32 MFMA tiles of a wave: 2 x 2 or 2 x 1
    constexpr int A_CH = MT * (RT / 8) / THREADS;                  // 16-byte activation chunks per thread
    constexpr int BUF = (MT + CT) * LROW;                          // elements of one buffer (A tile, then W tile)
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];   // two buffers
    const TileCoord tcoord = tile_of_block(blockIdx.x, a.tiles_m, a.tiles_c);
    if (tcoord.tm < 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const int m0 = tcoord.tm * MT, c0 = tcoord.tc * CT;
    const int K = a.w.K, N = a.w.N;
    const int C = BWD ? N : K, Cout = BWD ? K : N;
    const int n_steps = (C + RT - 1) / RT;

    // activation chunks of this thread: A_CH x 16 bytes, chunk idx = tid + 256 i -> row idx / 8, piece idx % 8
    const uint16_t *a_src[A_CH];
    int a_col[A_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int idx = tid + i * THREADS, row = idx >> 3, ch = idx & 7;
        const int m = m0 + row < a.M ? m0 + row : a.M - 1;
        // a chunk past the end of a contraction shorter than one step is never used (a_ok below is
        // false in every step): its loads are pointed at the row's first chunk, inside the matrix
        a_src[i] = a.act + (size_t)m * C + (ch * 8 < C ? ch * 8 : 0);
        a_col[i] = ch * 8;
    }
    // weight unit of this thread
    const int u_lo = BWD ? (tid & 63) : (tid & 127);     // forward: column of the tile; backward: n of the step
    const int u_kb = BWD ? (tid >> 6) : (tid >> 7);      // forward: block of the step (0, 1); backward: k block of the tile (0..3)
    // Running pointers instead of per-step index arithmetic: fetch(step) is called with step =
    // 0, 1, 2, ... in order, and every call advances them by one step.
    const uint32_t *wp;                  // word 0 of this thread's block at the current step
    const uint16_t *sp, *zp;             // its scale and zero point
    int blk_in_group = 0;                // forward: 32-code block index inside the quantization group
    const int bpg = a.w.group / 32;      // blocks per group
    if (!BWD) {
        const int w_col = c0 + u_lo < N ? c0 + u_lo : N - 1;       // clamped; never stored
        // d_in = 32: the second block of a step does not exist in any step (f.ok below is always
        // false for it); its loads are pointed at block 0
        const int kb0 = u_kb * 32 < K ? u_kb : 0;
        wp = a.w.qweight + (size_t)kb0 * BITS * N + w_col;
        const int g0 = (kb0 * 32) / a.w.group;
        blk_in_group = kb0 - g0 * bpg;
        sp = a.w.scales + (size_t)g0 * N + w_col;
        zp = a.w.zeros + (size_t)g0 * N + w_col;
    } else {
        const int k = c0 + u_kb * 32 < K ? c0 + u_kb * 32 : K - 32;
        const int g = k / a.w.group;
        // d_out < 64: lanes whose n lies past the matrix in step 0 lie past it in every step (f.ok
        // below is always false for them); their loads are pointed at the last column
        const int n0 = u_lo < N ? u_lo : N - 1;
        wp = a.w.qweight + (size_t)(k >> 5) * BITS * N + n0;
        sp = a.w.scales + (size_t)g * N + n0;
        zp = a.w.zeros + (size_t)g * N + n0;
    }

    // two register sets: the data of step s + 2 is fetched during step s and staged during step s + 1.
    // Every fetch issues the same LPF loads (addresses past the end are replaced by the step-0
    // ones and the values dropped), so that the waits can count.
    constexpr int LPF = A_CH + BITS + 2;
    struct Fetched {
        u32x4 a[A_CH];
        uint32_t w[BITS];
        uint32_t sc, z;
        bool a_ok[A_CH], ok;
    };
    Fetched R[2];
    const uint32_t *wp0 = wp;
    const uint16_t *sp0 = sp, *zp0 = zp;
    auto fetch = [&](int step, Fetched &f) {
        const int r0 = step * RT;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            f.a_ok[i] = r0 + a_col[i] < C;
            ld128(f.a[i], a_src[i] + (f.a_ok[i] ? r0 : 0));
        }
        // forward: contraction element r0 + 32 u_kb of column w_col; backward: n = r0 + u_lo
        f.ok = (BWD ? r0 + u_lo : r0 + u_kb * 32) < C;
        const uint32_t *wq = f.ok ? wp : wp0;
#pragma unroll
        for (int q = 0; q < BITS; ++q) ld32(f.w[q], wq + (size_t)q * N);
        ld16(f.sc, f.ok ? sp : sp0);
        ld16(f.z, f.ok ? zp : zp0);
        if (!BWD) {
            wp += (size_t)2 * BITS * N;          // two blocks per step
            blk_in_group += 2;
#pragma unroll
            for (int t = 0; t < 2; ++t)
                if (blk_in_group >= bpg) { blk_in_group -= bpg; sp += N; zp += N; }
        } else {
            wp += RT; sp += RT; zp += RT;
        }
    };
    auto landed = [&](Fetched &f) {          // after the wait that covers f's loads
#pragma unroll
        for (int i = 0; i < A_CH; ++i) tie(f.a[i]);
#pragma unroll
        for (int q = 0; q < BITS; ++q) tie(f.w[q]);
        tie(f.sc);
        tie(f.z);
    };
    auto stage = [&](int buf, const Fetched &f) {
        uint16_t *As = smem + buf * BUF, *Ws = As + MT * LROW;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int idx = tid + i * THREADS, row = idx >> 3;
            const bool k = f.a_ok[i];
            *reinterpret_cast<uint4 *>(As + row * LROW + a_col[i]) =
                make_uint4(k ? f.a[i][0] : 0u, k ? f.a[i][1] : 0u, k ? f.a[i][2] : 0u, k ? f.a[i][3] : 0u);
        }
        uint32_t o[16];
        dequant32<BITS>(f.w, half_bits_to_float((uint16_t)f.sc), half_bits_to_float((uint16_t)f.z), o);
        if (!f.ok) {
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
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int a_frag = (wm * 64 + (lane & 31)) * LROW + 8 * (lane >> 5);
    const int w_frag = MT * LROW + (wn * (32 * TJ) + (lane & 31)) * LROW + 8 * (lane >> 5);

    fetch(0, R[0]);
    if (n_steps > 1) {
        fetch(1, R[1]);
        wait_vm<LPF>();
    } else {
        wait_vm<0>();
    }
    landed(R[0]);
    stage(0, R[0]);
    __syncthreads();
    // the loop body for one parity of the step (register sets and LDS buffers alternate)
    auto one_step = [&](int step, Fetched &mine, Fetched &other) {
        const uint16_t *As = smem + (step & 1) * BUF, *Ws = As;     // fragment offsets include the W tile's base
        const bool more = step + 2 < n_steps;
        if (more) fetch(step + 2, mine);                            // `mine` was staged during the previous step
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
        // the other buffer was last read before the previous barrier; the loads of `other` are the
        // ones before this step's fetch
        if (step + 1 < n_steps) {
            if (more) wait_vm<LPF>(); else wait_vm<0>();
            landed(other);
            stage((step + 1) & 1, other);
        }
        __syncthreads();
    };
    for (int step = 0; step < n_steps; step += 2) {
        one_step(step, R[0], R[1]);
        if (step + 1 < n_steps) one_step(step + 1, R[1], R[0]);
    }

    // ---- epilogue: adapter term (P tile through LDS), bias, one rounding to binary16 -------------
    static_assert(2 * BUF * 2 >= MT * 64 * 4, "the P tile fits the tile buffers");
    float *Ps = reinterpret_cast<float *>(smem);         // [MT][r], r <= 64: at most 32 KB
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
        const int col = c0 + wn * (32 * TJ) + j * 32 + (lane & 31);
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

template <int BITS, bool BWD, int MT>
static hipError_t launch_f16_gemm_variant(F16GemmArgs &a, hipStream_t stream) {
    auto kern = f16_gemm_kernel<BITS, BWD, MT>;
    const size_t lds_bytes = 2 * (size_t)(MT + hf::CT) * hf::LROW * 2;
    static bool configured[64] = {};
    const hipError_t e = ensure_lds_limit(reinterpret_cast<const void *>(kern), lds_bytes, configured);
    if (e != hipSuccess) return e;
    const int Cout = BWD ? a.w.K : a.w.N;
    a.tiles_m = (a.M + MT - 1) / MT;
    a.tiles_c = (Cout + hf::CT - 1) / hf::CT;
    const int blocks = ((a.tiles_m * a.tiles_c + 7) / 8) * 8;
    launch_kernel(BWD ? "f16_gemm_bwd" : "f16_gemm_fwd", kern, blocks, hf::THREADS, lds_bytes, stream, a);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_f16_gemm_bits(F16GemmArgs &a, bool backward, hipStream_t stream) {
    // 128-row tiles unless they would leave most of the 256 compute units without one
    const int Cout = backward ? a.w.K : a.w.N;
    const long tiles128 = (long)((a.M + 127) / 128) * ((Cout + hf::CT - 1) / hf::CT);
    const bool small = tiles128 < 256;
    if (backward) return small ? launch_f16_gemm_variant<BITS, true, 64>(a, stream) : launch_f16_gemm_variant<BITS, true, 128>(a, stream);
    return small ? launch_f16_gemm_variant<BITS, false, 64>(a, stream) : launch_f16_gemm_variant<BITS, false, 128>(a, stream);
}

hipError_t launch_f16_gemm(const F16Layer &w, bool backward, const uint16_t *act, int M, uint16_t *out, const float *P,
                           const float *Fm, int r, float lora_scale, float *partials, hipStream_t stream) {
    // About one 128 x 64 tile per compute unit (half a round to a round and a quarter of the 256):
    // the producer / consumer kernel of the bfloat16 path, instantiated for this storage convention
    // (its loads, LDS layout and wave roles are the same; dequantization, MFMA type and epilogue
    // differ).  Measured: 33 against 64-69 us at 512 x 4096 x 4096; with many rounds of such small
    // tiles (4096 x 8192 x 8192) the kernel below is the faster one, 826 against 1197 us.
    {
        const int Cout = backward ? w.K : w.N;
        const long tiles = (long)((M + 127) / 128) * ((Cout + 63) / 64);
        const long tiles256 = (long)((M + 255) / 256) * ((Cout + 255) / 256);
        // a hundred-odd tokens (the last block of 256 rows at most half full) against a large weight: the
        // 256-column kernel with 128-row tiles, as on the bfloat16 path (27 + 7 against 49 us at 128 x 8192 x 8192)
        const bool half_rows = big_plan(M, backward ? w.N : w.K, Cout).mt == 128 && (long)w.K * w.N >= 4096L * 4096L;
        const bool use_mid = !half_rows && tiles >= 128 && tiles <= 320;
        // a few dozen 256 x 256 tiles or more: that kernel (the tiles of a partial last round are cut
        // into slices of the contraction, as on the bfloat16 path)
        const bool use_big = half_rows || (!use_mid && tiles256 >= 24);
        // MODULORA_F16_PLAIN (read once per process) keeps every shape on the plain kernel, for comparisons
        static const bool force_plain = std::getenv("MODULORA_F16_PLAIN") != nullptr;
        if (M > 32 && (use_mid || use_big) && !force_plain) {
            GemmArgs g{};
            g.w.K = w.K; g.w.N = w.N; g.w.bits = w.bits; g.w.group = w.group;
            g.w.qweight = w.qweight; g.w.scales = w.scales; g.w.zeros = nullptr;
            g.backward = backward; g.act = act; g.M = M; g.out = out;
            g.zeros16 = w.zeros; g.bias16 = w.bias;
            g.ep_P = r > 0 ? P : nullptr; g.ep_F = Fm; g.ep_r = r; g.ep_scale = lora_scale;
            g.partials = partials;
            g.partials_bytes = partials ? gemm_partial_bytes(M, w.K, w.N) : 0;
            return use_mid ? launch_gemm_mid_f16(g, stream) : launch_gemm_big_f16(g, stream);
        }
    }
    F16GemmArgs a;
    a.w = w; a.act = act; a.M = M; a.out = out; a.P = P; a.Fm = Fm; a.r = r; a.lora_scale = lora_scale;
    a.tiles_m = a.tiles_c = 0;
    switch (w.bits) {
        case 2: return launch_f16_gemm_bits<2>(a, backward, stream);
        case 3: return launch_f16_gemm_bits<3>(a, backward, stream);
        default: return launch_f16_gemm_bits<4>(a, backward, stream);
    }
}

}  // namespace mlr
