// Small-token-count (M <= 16) kernels: the layer as an HBM stream over the packed codes.
//
// At M <= 16 the layer is bound by one pass over the packed weight (codes + scales +
// zeros), and even the ~3 VALU operations per weight of an exact bfloat16 dequantization
// would cap the stream below the HBM rate.  These kernels therefore take the other route
// the paper names (Section 3.1.2, "Increasing Efficiency Further": row materialization,
// or a direct vector-by-quantized-matrix product with no materialization at all): the
// codes themselves feed the matrix cores and the affine part of eq. (2) is applied to the
// per-group partial sums,
//
//   forward   Y[m][n] = sum_g scale[g][n] * ( sum_{k in g} X[m][k] q[n][k]
//                                            - zero[g][n] * sum_{k in g} X[m][k] )
//
// which is algebraically the same Y = X What^T of eq. (3) with What = (q - zero) * scale,
// minus the intermediate rounding of What to 16 bits (the result is closer to the exact
// product, well inside the layer's tolerance).
//
// How a code becomes an MFMA operand in one instruction: OR-ing a b-bit field into the
// mantissa of bfloat16 128.0 (0x4300) gives exactly 128 + q, so
//     ((word >> s) & 0x000F000F) | 0x43004300
// is two bfloat16 operands (128 + q_a, 128 + q_b) at once.  The +128 is removed with the
// help of one extra MFMA per step against a vector of ones (it yields sum_k X[m][k], which
// the zero point needs anyway).  Which two codes share a register is fixed by the bit
// layout, so the X operand is pre-permuted to the same order by a small prep kernel
// (which also forms the partial sums of X A for the adapter term).  For 3-bit codes a
// field that lands one bit high (128 + 2q) is compensated by halving the matching X
// element -- powers of two, exact.
#include "device_common.h"
#include "launch.h"

namespace mlr {

namespace sm {
constexpr int WG_WAVES = 16, WG_THREADS = WG_WAVES * 64;
constexpr int COLS = 32;               // columns per workgroup (2 per lane of a 16-lane group)
constexpr int PREP_K = 128;            // contraction elements per prep workgroup
constexpr uint32_t MAGIC = 0x43004300u;   // two bfloat16 128.0
constexpr uint32_t ONES = 0x3F803F80u;    // two bfloat16 1.0

__device__ __forceinline__ bf16x8 as_bf16x8(const uint32_t r[4]) {
    bf16x8 v;
    __builtin_memcpy(&v, r, 16);
    return v;
}
__device__ __forceinline__ bf16x8 as_bf16x8(uint4 q) {
    bf16x8 v;
    __builtin_memcpy(&v, &q, 16);
    return v;
}

// chunks (8 codes) per step of a lane group, and codes per wave step
template <int BITS> struct Geo {
    static constexpr int NC = BITS == 4 ? 1 : (BITS == 2 ? 2 : 4);   // MFMA calls per wave step
    static constexpr int WORDS = BITS == 4 ? 1 : (BITS == 2 ? 1 : 3); // packed words per lane-group step
    static constexpr int KSTEP = 32 * NC;                             // codes per wave step
};

// The 8 operand values (4 registers) of call c from the words of one lane-group step.
template <int BITS>
__device__ __forceinline__ void codes_to_operand(const uint32_t *w, int c, uint32_t o[4]) {
    if (BITS == 4) {
        // reg p = (code p, code p+4)
#pragma unroll
        for (int p = 0; p < 4; ++p) o[p] = ((w[0] >> (4 * p)) & 0x000F000Fu) | MAGIC;
    } else if (BITS == 2) {
        // word of 16 codes; call c, reg p = (code 4c+p, code 4c+p+8)
#pragma unroll
        for (int p = 0; p < 4; ++p) o[p] = ((w[0] >> (2 * (4 * c + p))) & 0x00030003u) | MAGIC;
    } else {
        // 24-bit chunk c of the 96-bit block; regs (2*q0, q5) (2*q1, q6) (2*q2, q7) (q3, q4)
        const uint32_t ch = block_chunk<3>(w, c);
        o[0] = ((ch << 1) & 0x0007000Eu) | MAGIC;
        o[1] = ((ch >> 2) & 0x0007000Eu) | MAGIC;
        o[2] = ((ch >> 5) & 0x0007000Eu) | MAGIC;
        const uint32_t t = ch >> 9;                       // code 3 at bits 0-2, code 4 at bits 3-5
        o[3] = (t & 7u) | (((t << 13) & 0x00070000u) | MAGIC);
    }
}

// Source position (inside its permutation unit) and scale of permuted element `pos`.
// Unit = 8 codes (3- and 4-bit) or 16 codes (2-bit).
__device__ __forceinline__ int perm_src(int bits, int pos, float *scale) {
    *scale = 1.0f;
    if (bits == 4) return (pos >> 1) + 4 * (pos & 1);
    if (bits == 2) {
        const int c = pos >> 3, p = (pos >> 1) & 3, h = pos & 1;
        return 4 * c + p + 8 * h;
    }
    // 3-bit: (X0/2, X5, X1/2, X6, X2/2, X7, X3, X4)
    const int src[8] = {0, 5, 1, 6, 2, 7, 3, 4};
    if (pos == 0 || pos == 2 || pos == 4) *scale = 0.5f;
    return src[pos];
}
}  // namespace sm

// ---------------------------------------------------------------------------------
// prep (forward): Xp = X in operand order (rows >= M zero), and per-128-k partial sums of
// XA = X A.  One workgroup per 128 contraction elements; thread (m, chunk of 8).
// ---------------------------------------------------------------------------------
template <int RP>
__global__ __launch_bounds__(256) void smallm_prep_fwd_kernel(const uint16_t *__restrict__ X, int M, int K, int bits,
                                                              const float *__restrict__ A, int r,
                                                              uint16_t *__restrict__ Xp, float *__restrict__ Upart) {
    __shared__ uint16_t Xs[16][sm::PREP_K + 8];
    const int t = threadIdx.x, m = t >> 4, ch = t & 15;
    const int k0 = blockIdx.x * sm::PREP_K;
    const int kc = k0 + ch * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (m < M && kc < K) v = *reinterpret_cast<const uint4 *>(X + (size_t)m * K + kc);
    *reinterpret_cast<uint4 *>(&Xs[m][ch * 8]) = v;

    // adapter partial sums over this thread's 8 elements
    if (r > 0) {
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
        float acc[RP];
#pragma unroll
        for (int j = 0; j < RP; ++j) acc[j] = 0.f;
        if (kc < K) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = (e & 1) ? __uint_as_float(u[e >> 1] & 0xFFFF0000u) : __uint_as_float(u[e >> 1] << 16);
                const float *arow = A + (size_t)(kc + e) * r;
                if (r == RP) {
#pragma unroll
                    for (int j = 0; j < RP; j += 4) {
                        const float4 q = *reinterpret_cast<const float4 *>(arow + j);
                        acc[j] = __builtin_fmaf(x, q.x, acc[j]);
                        acc[j + 1] = __builtin_fmaf(x, q.y, acc[j + 1]);
                        acc[j + 2] = __builtin_fmaf(x, q.z, acc[j + 2]);
                        acc[j + 3] = __builtin_fmaf(x, q.w, acc[j + 3]);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < RP; ++j)
                        if (j < r) acc[j] = __builtin_fmaf(x, arow[j], acc[j]);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            float s = acc[j];
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
            if (ch == 0 && j < r) Upart[((size_t)blockIdx.x * 16 + m) * r + j] = s;
        }
    }
    __syncthreads();
    if (kc >= K) return;
    // permuted (and for 3-bit partly halved) copy of this thread's chunk
    const int unit = bits == 2 ? 16 : 8;
    uint16_t o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int pos = (ch * 8 + e) % unit, ubase = (ch * 8 + e) - pos;
        float sc;
        const int src = sm::perm_src(bits, pos, &sc);
        const uint16_t xb = Xs[m][ubase + src];
        o[e] = sc == 1.0f ? xb : float_to_bf16_bits(bf16_bits_to_float(xb) * sc);
    }
    uint4 ov;
    ov.x = o[0] | ((uint32_t)o[1] << 16);
    ov.y = o[2] | ((uint32_t)o[3] << 16);
    ov.z = o[4] | ((uint32_t)o[5] << 16);
    ov.w = o[6] | ((uint32_t)o[7] << 16);
    *reinterpret_cast<uint4 *>(Xp + (size_t)m * K + kc) = ov;
}

// ---------------------------------------------------------------------------------
// forward stream kernel.  A workgroup owns 32 output columns; its 16 waves split the
// quantization groups along K; each wave keeps a 16 x 32 fp32 partial in registers; the
// partials meet in LDS; the epilogue adds the adapter term and stores bfloat16.
// Inside a wave, lane l = 16 j + i holds columns n0 + 2i, n0 + 2i + 1 (one 8-byte load per
// packed word row) and the k-slice j of each MFMA call.
// ---------------------------------------------------------------------------------
struct SmallFwdDev {
    LayerView w;
    const uint16_t *Xp;     // [16][K] operand order
    const float *Upart;     // [K/128][16][r]
    const float *B;         // [r][N]
    int M, r, n_kparts;
    float lora_scale;
    uint16_t *Y;            // [M][N]
    float *XA;              // [M][r] or NULL
};

template <int BITS>
__global__ __launch_bounds__(sm::WG_THREADS) void smallm_fwd_kernel(SmallFwdDev d) {
    using G = sm::Geo<BITS>;
    __shared__ float red[sm::WG_WAVES][16][sm::COLS + 1];
    __shared__ float Us[16 * 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, j = lane >> 4;
    const int K = d.w.K, N = d.w.N, group = d.w.group;
    const int n0 = blockIdx.x * sm::COLS;
    int n = n0 + 2 * i;
    if (n > N - 2) n = N - 2;                       // clamped pair, masked at the store

    // adapter: XA = sum of the prep kernel's partials, gathered while the stream starts
    const int ur = 16 * d.r;
    for (int t = tid; t < ur; t += sm::WG_THREADS) Us[t] = 0.f;
    __syncthreads();
    if (d.r > 0) {
        const int parts = sm::WG_THREADS / ur > 0 ? sm::WG_THREADS / ur : 1;
        const int mj = tid % ur, part = tid / ur;
        if (part < parts) {
            float s = 0.f;
            for (int kb = part; kb < d.n_kparts; kb += parts) s += d.Upart[(size_t)kb * ur + mj];
            atomicAdd(&Us[mj], s);
        }
    }

    // this wave's share of the quantization groups
    const int n_groups = K / group;
    const int g_begin = (int)((long)n_groups * wave / sm::WG_WAVES);
    const int g_end = (int)((long)n_groups * (wave + 1) / sm::WG_WAVES);
    const int steps_per_group = group / G::KSTEP;

    f32x4 yacc[2];
#pragma unroll
    for (int cs = 0; cs < 2; ++cs)
#pragma unroll
        for (int v = 0; v < 4; ++v) yacc[cs][v] = 0.f;

    const uint32_t ones4[4] = {sm::ONES, sm::ONES, sm::ONES, sm::ONES};
    const uint32_t invf4[4] = {0x3F804000u, 0x3F804000u, 0x3F804000u, sm::ONES};   // (2,1)(2,1)(2,1)(1,1)
    const bf16x8 ones = sm::as_bf16x8(ones4), invf = sm::as_bf16x8(invf4);

    // The wave's work is a run of steps (KSTEP codes each); a group's affine part is
    // applied after its last step.  Loads run DEPTH steps ahead of the MFMAs in a rotating
    // set of register buffers (the loop is unrolled by DEPTH so the buffer index is static).
    constexpr int DEPTH = 4;
    struct Step {
        uint32_t w[2][G::WORDS];
        uint4 xa[G::NC];
        uint32_t sbits, zbits;
    };
    auto load_step = [&](Step &sd, int s) {
        const int g = s / steps_per_group;
        // lane group j takes chunks [cidx, cidx + NC) of 8 codes
        const int cidx = s * (G::KSTEP / 8) + j * G::NC;
        const int row0 = BITS == 4 ? cidx : (BITS == 2 ? cidx / 2 : (cidx / 4) * 3);
#pragma unroll
        for (int q = 0; q < G::WORDS; ++q) {
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            // streamed once: keep the packed words from displacing X and the adapter in cache
            const u32x2 pw = __builtin_nontemporal_load(
                reinterpret_cast<const u32x2 *>(d.w.qweight + (size_t)(row0 + q) * N + n));
            sd.w[0][q] = pw[0];
            sd.w[1][q] = pw[1];
        }
#pragma unroll
        for (int c = 0; c < G::NC; ++c)
            sd.xa[c] = *reinterpret_cast<const uint4 *>(d.Xp + (size_t)i * K + (size_t)(cidx + c) * 8);
        sd.sbits = *reinterpret_cast<const uint32_t *>(d.w.scales + (size_t)g * N + n);
        sd.zbits = *reinterpret_cast<const uint16_t *>(d.w.zeros + (size_t)g * N + n);
    };

    f32x4 tmp[2], s1, s2;
#pragma unroll
    for (int v = 0; v < 4; ++v) { tmp[0][v] = 0.f; tmp[1][v] = 0.f; s1[v] = 0.f; s2[v] = 0.f; }

    auto compute_step = [&](const Step &sd, int s) {
#pragma unroll
        for (int c = 0; c < G::NC; ++c) {
            const bf16x8 a = sm::as_bf16x8(sd.xa[c]);
#pragma unroll
            for (int cs = 0; cs < 2; ++cs) {
                uint32_t o[4];
                sm::codes_to_operand<BITS>(sd.w[cs], c, o);
                tmp[cs] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sm::as_bf16x8(o), tmp[cs], 0, 0, 0);
            }
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ones, s1, 0, 0, 0);
            if (BITS == 3) s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, invf, s2, 0, 0, 0);
        }
        if ((s + 1) % steps_per_group != 0) return;
        // end of a group: tmp = sum a (128 + q/f);  s1 = sum a;  s2 = sum a/f = sum X
        // (f == 1 unless 3-bit)
#pragma unroll
        for (int cs = 0; cs < 2; ++cs) {
            const float scale = half_bits_to_float((uint16_t)(sd.sbits >> (16 * cs)));
            const float zero = (float)((sd.zbits >> (8 * cs)) & 0xFFu);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float xsum = BITS == 3 ? s2[v] : s1[v];
                const float qx = __builtin_fmaf(-128.0f, s1[v], tmp[cs][v]);       // sum X q
                yacc[cs][v] = __builtin_fmaf(scale, __builtin_fmaf(-zero, xsum, qx), yacc[cs][v]);
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) { tmp[0][v] = 0.f; tmp[1][v] = 0.f; s1[v] = 0.f; s2[v] = 0.f; }
    };

    const int s_begin = g_begin * steps_per_group, s_end = g_end * steps_per_group;
    Step buf[DEPTH];
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd)
        if (s_begin + dd < s_end) load_step(buf[dd], s_begin + dd);
    for (int s = s_begin; s < s_end; s += DEPTH) {
#pragma unroll
        for (int dd = 0; dd < DEPTH; ++dd) {
            if (s + dd < s_end) {
                compute_step(buf[dd], s + dd);
                if (s + dd + DEPTH < s_end) load_step(buf[dd], s + dd + DEPTH);
            }
        }
    }

    // meet in LDS: D register v of lane (i, j) is row 4j + v, column i of the call's column set
#pragma unroll
    for (int cs = 0; cs < 2; ++cs)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][4 * j + v][2 * i + cs] = yacc[cs][v];
    __syncthreads();

    if (tid < 16 * sm::COLS) {
        const int m = tid / sm::COLS, c = tid % sm::COLS;
        float y = 0.f;
#pragma unroll
        for (int w = 0; w < sm::WG_WAVES; ++w) y += red[w][m][c];
        const int col = n0 + c;
        if (m < d.M && col < N) {
            float lora = 0.f;
            for (int jj = 0; jj < d.r; ++jj) lora = __builtin_fmaf(Us[m * d.r + jj], d.B[(size_t)jj * N + col], lora);
            d.Y[(size_t)m * N + col] = float_to_bf16_bits(__builtin_fmaf(d.lora_scale, lora, y));
        }
    }
    if (blockIdx.x == 0 && d.XA != nullptr)
        for (int t = tid; t < d.M * d.r; t += sm::WG_THREADS) d.XA[t] = Us[t];
}

bool smallm_fwd_supported(const LayerView &w, int M) {
    if (M > 16) return false;
    const int kstep = w.bits == 4 ? 32 : (w.bits == 2 ? 64 : 128);
    return w.group % kstep == 0 && w.K % sm::PREP_K == 0 && w.N >= 2;
}

size_t smallm_ws_bytes(int K, int N, int r) {
    const size_t kmax = (size_t)(K > N ? K : N);
    const size_t xp = ((size_t)16 * kmax * 2 + 255) & ~(size_t)255;
    const size_t up = (((kmax + sm::PREP_K - 1) / sm::PREP_K) * 16 * (size_t)(r > 0 ? r : 1) * 4 + 255) & ~(size_t)255;
    return xp + up;
}

hipError_t launch_smallm_fwd(const SmallArgs &a, hipStream_t stream) {
    const int K = a.w.K, N = a.w.N;
    uint16_t *Xp = static_cast<uint16_t *>(a.ws);
    const size_t xp_bytes = ((size_t)16 * (K > N ? K : N) * 2 + 255) & ~(size_t)255;
    float *Upart = reinterpret_cast<float *>(static_cast<char *>(a.ws) + xp_bytes);
    const int n_kparts = K / sm::PREP_K;

    prof_before("smallm_prep_fwd", stream);
    if (a.r <= 8)
        smallm_prep_fwd_kernel<8><<<n_kparts, 256, 0, stream>>>(a.act, a.M, K, a.w.bits, a.A, a.r, Xp, Upart);
    else if (a.r <= 16)
        smallm_prep_fwd_kernel<16><<<n_kparts, 256, 0, stream>>>(a.act, a.M, K, a.w.bits, a.A, a.r, Xp, Upart);
    else
        smallm_prep_fwd_kernel<64><<<n_kparts, 256, 0, stream>>>(a.act, a.M, K, a.w.bits, a.A, a.r, Xp, Upart);
    prof_after(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    SmallFwdDev d;
    d.w = a.w;
    d.Xp = Xp;
    d.Upart = Upart;
    d.B = a.B;
    d.M = a.M;
    d.r = a.r;
    d.n_kparts = n_kparts;
    d.lora_scale = a.lora_scale;
    d.Y = a.out;
    d.XA = a.P_out;
    const int blocks = (N + sm::COLS - 1) / sm::COLS;
    prof_before("stream_fwd", stream);
    switch (a.w.bits) {
        case 2: smallm_fwd_kernel<2><<<blocks, sm::WG_THREADS, 0, stream>>>(d); break;
        case 3: smallm_fwd_kernel<3><<<blocks, sm::WG_THREADS, 0, stream>>>(d); break;
        default: smallm_fwd_kernel<4><<<blocks, sm::WG_THREADS, 0, stream>>>(d); break;
    }
    prof_after(stream);
    return hipGetLastError();
}

}  // namespace mlr
