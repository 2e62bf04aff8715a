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
constexpr int WG_WAVES = 4, WG_THREADS = WG_WAVES * 64;
constexpr int COLS = 32;               // columns per workgroup (2 per lane of a 16-lane group)
constexpr int PREP_K = 128;            // contraction elements per prep workgroup
constexpr int MAX_KSPLIT = 8;          // workgroups that may share a column block
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

// (x & mask) | magic.  A VOP3 instruction of this ISA takes no literal, so with literal
// constants the compiler emits v_and + v_or; callers pass mask and magic as opaque
// register values (see opaque_sgpr / opaque_vgpr) and get one v_and_or_b32.  The
// instruction itself is left to the compiler: hand-written VALU assembly next to MFMAs is
// not covered by the compiler's hazard handling.
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic) {
    return (x & mask) | magic;
}
__device__ __forceinline__ uint32_t opaque_sgpr(uint32_t v) {
    asm volatile("" : "+s"(v));
    return v;
}
__device__ __forceinline__ uint32_t opaque_vgpr(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}
struct CodeMasks {
    uint32_t field, top, magic;   // field mask of a register pair, mask of 3-bit code 4, 2 x 128.0
};

// chunks (8 codes) per step of a lane group, and codes per wave step
template <int BITS> struct Geo {
    static constexpr int NC = BITS == 4 ? 1 : (BITS == 2 ? 2 : 4);   // MFMA calls per wave step
    static constexpr int WORDS = BITS == 4 ? 1 : (BITS == 2 ? 1 : 3); // packed words per lane-group step
    static constexpr int KSTEP = 32 * NC;                             // codes per wave step
};

template <int BITS>
__device__ __forceinline__ CodeMasks make_masks() {
    CodeMasks m;
    m.field = opaque_sgpr(BITS == 4 ? 0x000F000Fu : (BITS == 2 ? 0x00030003u : 0x0007000Eu));
    m.top = opaque_sgpr(0x00070000u);
    m.magic = opaque_vgpr(MAGIC);
    return m;
}

// The 8 operand values (4 registers) of call c from the words of one lane-group step.
template <int BITS>
__device__ __forceinline__ void codes_to_operand(const uint32_t *w, int c, const CodeMasks &m, uint32_t o[4]) {
    if (BITS == 4) {
        // reg p = (code p, code p+4)
#pragma unroll
        for (int p = 0; p < 4; ++p) o[p] = and_or(w[0] >> (4 * p), m.field, m.magic);
    } else if (BITS == 2) {
        // word of 16 codes; call c, reg p = (code 4c+p, code 4c+p+8)
#pragma unroll
        for (int p = 0; p < 4; ++p) o[p] = and_or(w[0] >> (2 * (4 * c + p)), m.field, m.magic);
    } else {
        // 24-bit chunk c of the 96-bit block; regs (2*q0, q5) (2*q1, q6) (2*q2, q7) (q3, q4)
        const uint32_t ch = block_chunk<3>(w, c);
        o[0] = and_or(ch << 1, m.field, m.magic);
        o[1] = and_or(ch >> 2, m.field, m.magic);
        o[2] = and_or(ch >> 5, m.field, m.magic);
        // code 3 (bits 9-11) low, code 4 (bits 12-14) high
        o[3] = ((ch >> 9) & 7u) | and_or(ch << 4, m.top, m.magic);
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
// prep (forward): Xp = X in operand order, stored [K/8][16][8] (rows >= M zero), and per-128-k partial sums of
// XA = X A.  One workgroup per 128 contraction elements; thread (m, chunk of 8).
// ---------------------------------------------------------------------------------
template <int RP>
__global__ __launch_bounds__(256) void smallm_prep_fwd_kernel(const uint16_t *__restrict__ X, int M, int K, int bits,
                                                              const float *__restrict__ A, int r,
                                                              uint16_t *__restrict__ Xp, float *__restrict__ Upart,
                                                              int n_kparts) {
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
    // operand layout [chunk of 8][row m][8]: the 16 rows of one chunk are 256 contiguous bytes,
    // which is what the 16 lanes of a lane group fetch together
    *reinterpret_cast<uint4 *>(Xp + ((size_t)(kc >> 3) * 16 + m) * 8) = ov;
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
    const uint16_t *Xp;     // [K/8][16][8] operand order
    const float *Upart;     // [K/128][16][r]
    const float *B;         // [r][N]
    int M, r, n_kparts;
    int ksplit;             // workgroups that share one column block (split of the groups along K)
    float lora_scale;
    uint16_t *Y;            // [M][N]
    float *XA;              // [M][r] or NULL
    float *Yacc;            // [ksplit][16][N] fp32 partial tiles (used when ksplit > 1)
};

// Epilogue shared by the stream kernel (no K split) and the finish kernel: thread tid holds
// outputs tid and tid + WG_THREADS of the 16 x 32 tile of column block cb in y[]; adds the
// adapter term and stores bfloat16.  XA = sum of the prep kernel's partials: element t of the
// 16 x r tile is summed by WG_THREADS / (16 r) threads over interleaved slices of the
// partials, eight independent loads at a time, and the slices meet in LDS (Us, 16 * 64 floats).
__device__ __forceinline__ void smallm_fwd_epilogue(const SmallFwdDev &d, int cb, const float y[2], float *Us) {
    const int tid = threadIdx.x, N = d.w.N, n0 = cb * sm::COLS;
    const int ur = 16 * d.r;
    for (int t = tid; t < ur; t += sm::WG_THREADS) Us[t] = 0.f;
    __syncthreads();
    if (d.r > 0) {
        const int slices = sm::WG_THREADS >= ur ? sm::WG_THREADS / ur : 1;
        for (int t = tid; t < slices * ur; t += sm::WG_THREADS) {
            const int mj = t % ur, slice = t / ur;
            float acc8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            int kb = slice;
            for (; kb + 7 * slices < d.n_kparts; kb += 8 * slices) {
#pragma unroll
                for (int u = 0; u < 8; ++u) acc8[u] += d.Upart[(size_t)(kb + u * slices) * ur + mj];
            }
            for (; kb < d.n_kparts; kb += slices) acc8[0] += d.Upart[(size_t)kb * ur + mj];
            atomicAdd(&Us[mj], ((acc8[0] + acc8[1]) + (acc8[2] + acc8[3])) + ((acc8[4] + acc8[5]) + (acc8[6] + acc8[7])));
        }
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int idx = tid + e * sm::WG_THREADS, m = idx / sm::COLS, col = n0 + idx % sm::COLS;
        if (m < d.M && col < N) {
            float lora = 0.f;
            for (int jj = 0; jj < d.r; ++jj) lora = __builtin_fmaf(Us[m * d.r + jj], d.B[(size_t)jj * N + col], lora);
            d.Y[(size_t)m * N + col] = float_to_bf16_bits(__builtin_fmaf(d.lora_scale, lora, y[e]));
        }
    }
    if (cb == 0 && d.XA != nullptr)
        for (int t = tid; t < d.M * d.r; t += sm::WG_THREADS) d.XA[t] = Us[t];
}

template <int BITS>
__global__ __launch_bounds__(sm::WG_THREADS, 4) void smallm_fwd_kernel(SmallFwdDev d) {
    using G = sm::Geo<BITS>;
    __shared__ float red[sm::WG_WAVES][16][sm::COLS + 1];
    __shared__ float Us[16 * 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, j = lane >> 4;
    const int K = d.w.K, N = d.w.N, group = d.w.group;
    const int cb = blockIdx.x / d.ksplit, ks = blockIdx.x % d.ksplit;   // column block, K split
    const int n0 = cb * sm::COLS;
    int n = n0 + 2 * i;
    if (n > N - 2) n = N - 2;                       // clamped pair, masked at the store

    // this wave's share of the quantization groups
    const int n_groups = K / group;
    const int parts = d.ksplit * sm::WG_WAVES, part = ks * sm::WG_WAVES + wave;
    const int g_begin = (int)((long)n_groups * part / parts);
    const int g_end = (int)((long)n_groups * (part + 1) / parts);
    const int steps_per_group = group / G::KSTEP;

    f32x4 yacc[2];
#pragma unroll
    for (int cs = 0; cs < 2; ++cs)
#pragma unroll
        for (int v = 0; v < 4; ++v) yacc[cs][v] = 0.f;

    const uint32_t ones4[4] = {sm::ONES, sm::ONES, sm::ONES, sm::ONES};
    const uint32_t invf4[4] = {0x3F804000u, 0x3F804000u, 0x3F804000u, sm::ONES};   // (2,1)(2,1)(2,1)(1,1)
    const bf16x8 ones = sm::as_bf16x8(ones4), invf = sm::as_bf16x8(invf4);

    // The wave's work is a run of steps (KSTEP codes each), group after group; a group's
    // affine part is applied after its last step.  Loads run DEPTH steps ahead of the MFMAs
    // in a rotating set of register buffers (the loop is unrolled by DEPTH so the buffer
    // index is static).  Every address is a wave-uniform base plus a per-lane constant.
    // deep enough that a CU keeps ~64-96 KB of packed words in flight (16 waves x DEPTH steps)
    constexpr int DEPTH = BITS == 3 ? 3 : (BITS == 2 ? 6 : 8);
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    struct Step {
        u32x2 w[G::WORDS];
        uint4 xa[G::NC];
        uint32_t sbits;
        uint16_t zbits;
    };
    // lane group j reads packed rows (4 s + j) * WORDS + q, columns n, n + 1
    const uint32_t w_voff = (uint32_t)(((size_t)j * G::WORDS * N + n) * 4);
    // and operand chunks 4 NC s + NC j + c, row i:  element ((chunk) * 16 + i) * 8
    const uint32_t x_voff = (uint32_t)(((j * G::NC) * 16 + i) * 16);
    const uint32_t s_voff = (uint32_t)n * 2u, z_voff = (uint32_t)n;
    auto load_step = [&](Step &sd, int s, int g) {
        const uint32_t *wbase = d.w.qweight + (size_t)s * (4 * G::WORDS) * N;
#pragma unroll
        for (int q = 0; q < G::WORDS; ++q)   // streamed once: non-temporal
            sd.w[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(
                reinterpret_cast<const char *>(wbase + (size_t)q * N) + w_voff));
        const uint16_t *xbase = d.Xp + (size_t)s * (4 * G::NC * 128);
#pragma unroll
        for (int c = 0; c < G::NC; ++c) sd.xa[c] = load_at<uint4>(xbase + c * 128, x_voff);
        sd.sbits = load_at<uint32_t>(d.w.scales + (size_t)g * N, s_voff);
        sd.zbits = load_at<uint16_t>(d.w.zeros + (size_t)g * N, z_voff);
    };

    const sm::CodeMasks masks = sm::make_masks<BITS>();
    f32x4 tmp[2], s1, s2;
#pragma unroll
    for (int v = 0; v < 4; ++v) { tmp[0][v] = 0.f; tmp[1][v] = 0.f; s1[v] = 0.f; s2[v] = 0.f; }

    auto compute_step = [&](const Step &sd, bool group_ends) {
        uint32_t w0[G::WORDS], w1[G::WORDS];
#pragma unroll
        for (int q = 0; q < G::WORDS; ++q) { w0[q] = sd.w[q][0]; w1[q] = sd.w[q][1]; }
#pragma unroll
        for (int c = 0; c < G::NC; ++c) {
            const bf16x8 a = sm::as_bf16x8(sd.xa[c]);
            uint32_t o[4];
            sm::codes_to_operand<BITS>(w0, c, masks, o);
            tmp[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sm::as_bf16x8(o), tmp[0], 0, 0, 0);
            sm::codes_to_operand<BITS>(w1, c, masks, o);
            tmp[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sm::as_bf16x8(o), tmp[1], 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ones, s1, 0, 0, 0);
            if (BITS == 3) s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, invf, s2, 0, 0, 0);
        }
        if (!group_ends) return;
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
    // (step, group, position in group) of the next step to load and of the next to compute
    int ls = s_begin, lg = g_begin, lp = 0;
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd)
        if (ls < s_end) {
            load_step(buf[dd], ls, lg);
            ++ls;
            if (++lp == steps_per_group) { lp = 0; ++lg; }
        }

    int cp = 0;
    for (int s = s_begin; s < s_end; s += DEPTH) {
#pragma unroll
        for (int dd = 0; dd < DEPTH; ++dd) {
            if (s + dd < s_end) {
                const bool ends = ++cp == steps_per_group;
                if (ends) cp = 0;
                compute_step(buf[dd], ends);
                if (ls < s_end) {
                    load_step(buf[dd], ls, lg);
                    ++ls;
                    if (++lp == steps_per_group) { lp = 0; ++lg; }
                }
            }
        }
    }

    // meet in LDS: D register v of lane (i, j) is row 4j + v, column i of the call's column set
#pragma unroll
    for (int cs = 0; cs < 2; ++cs)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][4 * j + v][2 * i + cs] = yacc[cs][v];
    __syncthreads();

    // each thread owns two of the 16 x 32 outputs of the column block
    float y[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int idx = tid + e * sm::WG_THREADS, m = idx / sm::COLS, c = idx % sm::COLS;
        y[e] = 0.f;
#pragma unroll
        for (int w = 0; w < sm::WG_WAVES; ++w) y[e] += red[w][m][c];
    }
    if (d.ksplit > 1) {
        // each K split leaves its fp32 partial tile; the finish kernel (next launch on the
        // stream) adds them up.  No cross-workgroup traffic inside this kernel, hence no fences.
        float *mine = d.Yacc + (size_t)ks * 16 * N;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int idx = tid + e * sm::WG_THREADS, m = idx / sm::COLS, col = n0 + idx % sm::COLS;
            if (col < N) mine[(size_t)m * N + col] = y[e];
        }
        return;
    }
    smallm_fwd_epilogue(d, cb, y, Us);
}

// Sum of the K splits' partial tiles, then the common epilogue.  One workgroup per column block.
__global__ __launch_bounds__(sm::WG_THREADS) void smallm_fwd_finish_kernel(SmallFwdDev d) {
    __shared__ float Us[16 * 64];
    const int tid = threadIdx.x, cb = blockIdx.x, n0 = cb * sm::COLS, N = d.w.N;
    float y[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int idx = tid + e * sm::WG_THREADS, m = idx / sm::COLS, col = n0 + idx % sm::COLS;
        float sum = 0.f;
        if (col < N)
            for (int q = 0; q < d.ksplit; ++q) sum += d.Yacc[((size_t)q * 16 + m) * N + col];
        y[e] = sum;
    }
    smallm_fwd_epilogue(d, cb, y, Us);
}

bool smallm_fwd_supported(const LayerView &w, int M) {
    if (M > 16) return false;
    const int kstep = w.bits == 4 ? 32 : (w.bits == 2 ? 64 : 128);
    return w.group % kstep == 0 && w.K % sm::PREP_K == 0 && w.N >= 2;
}

namespace {
struct SmallWs {
    size_t xp, upart, yacc, total;
};
SmallWs small_ws(int K, int N, int r) {
    const size_t kmax = (size_t)(K > N ? K : N);
    auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
    SmallWs l;
    size_t off = 0;
    l.xp = off;      off += al((size_t)16 * kmax * 2);
    l.upart = off;   off += al(((kmax + sm::PREP_K - 1) / sm::PREP_K) * 16 * (size_t)(r > 0 ? r : 1) * 4);
    l.yacc = off;    off += al((size_t)sm::MAX_KSPLIT * 16 * kmax * 4);
    l.total = off;
    return l;
}
}  // namespace

size_t smallm_ws_bytes(int K, int N, int r) { return small_ws(K, N, r).total; }

hipError_t launch_smallm_fwd(const SmallArgs &a, hipStream_t stream) {
    const int K = a.w.K, N = a.w.N;
    const SmallWs l = small_ws(K, N, a.r);
    char *ws = static_cast<char *>(a.ws);
    uint16_t *Xp = reinterpret_cast<uint16_t *>(ws + l.xp);
    float *Upart = reinterpret_cast<float *>(ws + l.upart);
    float *Yacc = reinterpret_cast<float *>(ws + l.yacc);
    const int n_kparts = K / sm::PREP_K;
    const int col_blocks = (N + sm::COLS - 1) / sm::COLS;

    // enough workgroups (4 waves each) for ~4 per CU; a split never gets less than one group per wave
    int ksplit = (1024 + col_blocks - 1) / col_blocks;
    const int max_split = (K / a.w.group) / sm::WG_WAVES;
    if (ksplit > max_split) ksplit = max_split;
    if (ksplit > sm::MAX_KSPLIT) ksplit = sm::MAX_KSPLIT;
    if (ksplit < 1) ksplit = 1;

    prof_before("smallm_prep_fwd", stream);
    if (a.r <= 8)
        smallm_prep_fwd_kernel<8><<<n_kparts, 256, 0, stream>>>(a.act, a.M, K, a.w.bits, a.A, a.r, Xp, Upart, n_kparts);
    else if (a.r <= 16)
        smallm_prep_fwd_kernel<16><<<n_kparts, 256, 0, stream>>>(a.act, a.M, K, a.w.bits, a.A, a.r, Xp, Upart, n_kparts);
    else
        smallm_prep_fwd_kernel<64><<<n_kparts, 256, 0, stream>>>(a.act, a.M, K, a.w.bits, a.A, a.r, Xp, Upart, n_kparts);
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
    d.ksplit = ksplit;
    d.lora_scale = a.lora_scale;
    d.Y = a.out;
    d.XA = a.P_out;
    d.Yacc = Yacc;
    prof_before("stream_fwd", stream);
    switch (a.w.bits) {
        case 2: smallm_fwd_kernel<2><<<col_blocks * ksplit, sm::WG_THREADS, 0, stream>>>(d); break;
        case 3: smallm_fwd_kernel<3><<<col_blocks * ksplit, sm::WG_THREADS, 0, stream>>>(d); break;
        default: smallm_fwd_kernel<4><<<col_blocks * ksplit, sm::WG_THREADS, 0, stream>>>(d); break;
    }
    prof_after(stream);
    e = hipGetLastError();
    if (e != hipSuccess || ksplit == 1) return e;
    prof_before("stream_fwd_finish", stream);
    smallm_fwd_finish_kernel<<<col_blocks, sm::WG_THREADS, 0, stream>>>(d);
    prof_after(stream);
    return hipGetLastError();
}

}  // namespace mlr
