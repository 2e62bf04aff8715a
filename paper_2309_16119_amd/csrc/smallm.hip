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
// (which also forms the partial sums of X A for the adapter term).  For 3-bit codes the
// low field of a register lands four bits high (128 + 16q), compensated by the matching X
// element divided by 16 -- a power of two, exact.
#include "device_common.h"
#include "gemm_common.h"
#include "launch.h"

namespace mlr {

namespace sm {
constexpr int WG_WAVES = 4, WG_THREADS = WG_WAVES * 64;
constexpr int PREP_K = 128;            // contraction elements per prep workgroup
constexpr int MAX_KSPLIT = 32;         // workgroups that may share a column block
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
    uint32_t field, magic;        // field mask of a register pair, 2 x 128.0
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
    m.field = opaque_sgpr(BITS == 4 ? 0x000F000Fu : (BITS == 2 ? 0x00030003u : 0x00070070u));
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
        // 24-bit chunk c of the 96-bit block (stream bits 24c .. 24c+23); reg p = (16 * code p,
        // code p+4): code p must land at bits 4-6, i.e. the chunk shifted right by 3p - 4, and
        // code p+4 (12 bits further up) then sits at bits 16-18.  The shift is folded into the
        // extraction of the chunk from the words (one funnel shift or plain shift per register).
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int sh = 24 * c + 3 * p - 4;       // stream bit that lands at register bit 0
            uint32_t x;
            if (sh < 0) x = w[0] << (-sh);
            else if ((sh & 31) == 0) x = w[sh >> 5];
            else if ((sh >> 5) == 2) x = w[2] >> (sh & 31);
            else x = __builtin_amdgcn_alignbit(w[(sh >> 5) + 1], w[sh >> 5], sh & 31);
            o[p] = and_or(x, m.field, m.magic);
        }
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
    // 3-bit: (X0/16, X4, X1/16, X5, X2/16, X6, X3/16, X7)
    if ((pos & 1) == 0) *scale = 0.0625f;
    return (pos >> 1) + 4 * (pos & 1);
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
    // permuted (and for 3-bit partly scaled) copy of this thread's chunk
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
// forward stream kernel.  A workgroup of 4 waves owns 256 output columns and one slice of K
// (a run of whole quantization groups); each wave owns 64 of the columns.  The slice of the
// re-ordered activations sits in LDS, shared by the four waves.  Inside a wave, lane
// l = 16 j + i holds columns n0 + 4i .. 4i+3 (one 16-byte load per packed word row, 256
// contiguous bytes per 16-lane group) and the k-slice j of each MFMA call.  Packed words,
// scales and zeros are loaded DEPTH steps ahead by loads issued from assembly and awaited
// with an exact count; loads past the end of the slice are clamped to its last step, so the
// number in flight never changes and the loop needs no predicates.  The 16 x 64 fp32 result
// of a wave is final for the slice and is stored as a partial tile for the finish kernel.
// ---------------------------------------------------------------------------------
struct SmallFwdDev {
    LayerView w;
    const uint16_t *Xp;     // [K/8][16][8] operand order
    const float *Upart;     // [K/128][16][r]
    float *Ufinal;          // [16][r]: XA, summed by the reducer block of the stream kernel
    const float *B;         // [r][N]
    int M, r, n_kparts;
    int ksplit;             // workgroups that share one column block (split of the groups along K)
    float lora_scale;
    uint16_t *Y;            // [M][N]
    float *XA;              // [M][r] or NULL
    float *Yacc;            // [ksplit][16][N] fp32 partial tiles
};

namespace sm {
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void ald(u32x4 &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void ald(u32x2 &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void ald(uint32_t &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base
// wave-uniform, passed in M0); counted in vmcnt like a register load.
__device__ __forceinline__ void ald_lds(const void *gbase_uniform, uint32_t voff_bytes, uint32_t lds_base_uniform) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base_uniform), "v"(voff_bytes), "s"(gbase_uniform)
                 : "memory");
}
// the same with a full per-lane address; earlier LDS reads of the wave are awaited first, so
// that the incoming data cannot overtake a read of the slot it replaces
__device__ __forceinline__ void ald_lds64(const void *gaddr_lane, uint32_t lds_base_uniform) {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_base_uniform), "v"(gaddr_lane)
                 : "memory");
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
constexpr int WCOLS = 64;                 // columns per wave (4 per lane of a 16-lane group)
constexpr int BCOLS = WG_WAVES * WCOLS;   // columns per workgroup
constexpr int MAX_RANGE = 2048;           // contraction elements of one K slice (64 KB of LDS)
}  // namespace sm

// Sum of a prep kernel's partials [n_parts][16][r] into Us (16 x r floats in LDS): element t of the tile
// is summed by WG_THREADS / (16 r) threads over interleaved slices of the partials, eight
// independent loads at a time, and the slices meet through LDS atomics.
__device__ __forceinline__ void smallm_gather_parts(const float *parts, int n_parts, int r, float *Us) {
    const int tid = threadIdx.x;
    const int ur = 16 * r;
    for (int t = tid; t < ur; t += sm::WG_THREADS) Us[t] = 0.f;
    __syncthreads();
    if (r > 0) {
        const int slices = sm::WG_THREADS >= ur ? sm::WG_THREADS / ur : 1;
        for (int t = tid; t < slices * ur; t += sm::WG_THREADS) {
            const int mj = t % ur, slice = t / ur;
            float acc8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            int kb = slice;
            for (; kb + 7 * slices < n_parts; kb += 8 * slices) {
#pragma unroll
                for (int u = 0; u < 8; ++u) acc8[u] += parts[(size_t)(kb + u * slices) * ur + mj];
            }
            for (; kb < n_parts; kb += slices) acc8[0] += parts[(size_t)kb * ur + mj];
            atomicAdd(&Us[mj], ((acc8[0] + acc8[1]) + (acc8[2] + acc8[3])) + ((acc8[4] + acc8[5]) + (acc8[6] + acc8[7])));
        }
    }
    __syncthreads();
}

// Adds the adapter term to the four adjacent outputs y[0..3] of row m, columns col..col+3
// (col a multiple of 4, col + 3 < N) and stores them as bfloat16.
__device__ __forceinline__ void smallm_store4(const SmallFwdDev &d, const float *Us, int m, int col, const float y[4]) {
    float l[4] = {0.f, 0.f, 0.f, 0.f};
    for (int jj = 0; jj < d.r; ++jj) {
        const float u = Us[m * d.r + jj];
        const float4 b = *reinterpret_cast<const float4 *>(d.B + (size_t)jj * d.w.N + col);
        l[0] = __builtin_fmaf(u, b.x, l[0]);
        l[1] = __builtin_fmaf(u, b.y, l[1]);
        l[2] = __builtin_fmaf(u, b.z, l[2]);
        l[3] = __builtin_fmaf(u, b.w, l[3]);
    }
    uint2 o;
    o.x = pack_bf16x2(__builtin_fmaf(d.lora_scale, l[0], y[0]), __builtin_fmaf(d.lora_scale, l[1], y[1]));
    o.y = pack_bf16x2(__builtin_fmaf(d.lora_scale, l[2], y[2]), __builtin_fmaf(d.lora_scale, l[3], y[3]));
    *reinterpret_cast<uint2 *>(d.Y + (size_t)m * d.w.N + col) = o;
}

template <int BITS>
__global__ __launch_bounds__(sm::WG_THREADS, 2) void smallm_fwd_kernel(SmallFwdDev d) {
    using G = sm::Geo<BITS>;
    extern __shared__ __attribute__((aligned(16))) uint4 xs[];   // [chunks of the slice][16 rows]
    __shared__ float Us[16 * 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (blockIdx.x == 0) {
        // reducer block: XA = sum of the prep kernel's partials, for the finish kernel and the
        // caller; it runs beside the streaming blocks, so its latency-bound gather costs nothing
        smallm_gather_parts(d.Upart, d.n_kparts, d.r, Us);
        for (int t = tid; t < 16 * d.r; t += sm::WG_THREADS) d.Ufinal[t] = Us[t];
        if (d.XA != nullptr)
            for (int t = tid; t < d.M * d.r; t += sm::WG_THREADS) d.XA[t] = Us[t];
        return;
    }
    const int bid = blockIdx.x - 1;
    const int i = lane & 15, j = lane >> 4;
    const int N = d.w.N, group = d.w.group;
    const int cb = bid / d.ksplit, ks = bid % d.ksplit;   // column block, K slice
    const int nw = cb * sm::BCOLS + wave * sm::WCOLS;   // first column of the wave
    int n = nw + 4 * i;
    const bool col_ok = n < N;                      // N is a multiple of 8: all four columns or none
    if (n > N - 4) n = N - 4;                       // clamped loads, masked at the store

    // this workgroup's run of quantization groups, as a run of steps (KSTEP codes each)
    const int n_groups = d.w.K / group;
    const int g_begin = (int)((long)n_groups * ks / d.ksplit);
    const int g_end = (int)((long)n_groups * (ks + 1) / d.ksplit);
    const int spg = group / G::KSTEP;               // steps per group
    const int s_begin = g_begin * spg, s_end = g_end * spg;

    constexpr int DEPTH = BITS == 3 ? 4 : 8;
    constexpr int SL = G::WORDS + 2;                // loads per stage
    struct Stage {
        sm::u32x4 w[G::WORDS];
        sm::u32x2 sc;      // 4 binary16 scales
        uint32_t z;        // 4 zero points
    };
    Stage st[DEPTH];
    // lane group j reads packed rows (4 s + j) * WORDS + q, columns n .. n + 3
    const uint32_t w_voff = (uint32_t)(((size_t)j * G::WORDS * N + n) * 4);
    const uint32_t s_voff = (uint32_t)n * 2u, z_voff = (uint32_t)n;
    auto issue = [&](Stage &sd, int s) {            // s: any step of the slice (clamped by the caller)
        const uint32_t *wbase = d.w.qweight + (size_t)s * (4 * G::WORDS) * N;
#pragma unroll
        for (int q = 0; q < G::WORDS; ++q) sm::ald(sd.w[q], wbase + (size_t)q * N, w_voff);
        const int g = s / spg;
        sm::ald(sd.sc, d.w.scales + (size_t)g * N, s_voff);
        sm::ald(sd.z, d.w.zeros + (size_t)g * N, z_voff);
    };
    // The slice of the re-ordered activations, a contiguous run of 16-byte operand rows, goes
    // straight from global memory into LDS: 1 KB per wave and load, the waves take turns.
    // (A slice is a multiple of 32 contraction elements, i.e. of 1 KB.)  These loads are
    // issued first, so they are the oldest ones in flight.
    {
        const char *src = reinterpret_cast<const char *>(d.Xp) + (size_t)s_begin * (G::KSTEP / 8) * 256;
        const int n_kb = (s_end - s_begin) * (G::KSTEP / 8) / 4;          // 1 KB units
        const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)xs;
        for (int u = wave; u < n_kb; u += sm::WG_WAVES) sm::ald_lds(src + (size_t)u * 1024, (uint32_t)lane * 16u, lds0 + (uint32_t)u * 1024u);
    }
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd) issue(st[dd], s_begin + dd < s_end ? s_begin + dd : s_end - 1);
    // everything older than the DEPTH stages has landed: this wave's part of the slice is in LDS
    sm::wait_vm<DEPTH * SL>();
    __syncthreads();

    f32x4 yacc[4], tmp[4], s1, s2;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
#pragma unroll
        for (int cs = 0; cs < 4; ++cs) { yacc[cs][v] = 0.f; tmp[cs][v] = 0.f; }
        s1[v] = 0.f; s2[v] = 0.f;
    }
    const uint32_t ones4[4] = {sm::ONES, sm::ONES, sm::ONES, sm::ONES};
    const uint32_t invf4[4] = {0x3F804180u, 0x3F804180u, 0x3F804180u, 0x3F804180u};   // (16, 1) pairs
    const bf16x8 ones = sm::as_bf16x8(ones4), invf = sm::as_bf16x8(invf4);
    const sm::CodeMasks masks = sm::make_masks<BITS>();

    auto compute = [&](Stage &sd, int srel, bool group_ends) {
        // operand chunks 4 NC srel + NC j + c of the slice, row i
        const uint4 *xrow = xs + ((size_t)srel * 4 * G::NC + G::NC * j) * 16 + i;
        uint4 xa[G::NC];
#pragma unroll
        for (int c = 0; c < G::NC; ++c) xa[c] = xrow[c * 16];
#pragma unroll
        for (int c = 0; c < G::NC; ++c) {
            const bf16x8 a = sm::as_bf16x8(xa[c]);
#pragma unroll
            for (int cs = 0; cs < 4; ++cs) {
                uint32_t wq[G::WORDS], o[4];
#pragma unroll
                for (int q = 0; q < G::WORDS; ++q) wq[q] = sd.w[q][cs];
                sm::codes_to_operand<BITS>(wq, c, masks, o);
                tmp[cs] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sm::as_bf16x8(o), tmp[cs], 0, 0, 0);
            }
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ones, s1, 0, 0, 0);
            if (BITS == 3) s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, invf, s2, 0, 0, 0);
        }
        if (!group_ends) return;
        // end of a group: tmp = sum a (128 + q/f);  s1 = sum a;  s2 = sum a/f = sum X
        // (f == 1 unless 3-bit)
#pragma unroll
        for (int cs = 0; cs < 4; ++cs) {
            const float scale = half_bits_to_float((uint16_t)(sd.sc[cs >> 1] >> (16 * (cs & 1))));
            const float zero = (float)((sd.z >> (8 * cs)) & 0xFFu);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float xsum = BITS == 3 ? s2[v] : s1[v];
                const float qx = __builtin_fmaf(-128.0f, s1[v], tmp[cs][v]);       // sum X q
                yacc[cs][v] = __builtin_fmaf(scale, __builtin_fmaf(-zero, xsum, qx), yacc[cs][v]);
                tmp[cs][v] = 0.f;
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) { s1[v] = 0.f; s2[v] = 0.f; }
    };

    int cp = 0;   // position of the next step inside its group
    for (int s = s_begin; s < s_end; s += DEPTH) {
#pragma unroll
        for (int dd = 0; dd < DEPTH; ++dd) {
            if (s + dd < s_end) {
                // DEPTH - 1 younger stages stay in flight
                sm::wait_vm<(DEPTH - 1) * SL>();
#pragma unroll
                for (int q = 0; q < G::WORDS; ++q) sm::tie(st[dd].w[q]);
                sm::tie(st[dd].sc);
                sm::tie(st[dd].z);
                const bool ends = ++cp == spg;
                if (ends) cp = 0;
                compute(st[dd], s + dd - s_begin, ends);
                const int sn = s + dd + DEPTH;
                issue(st[dd], sn < s_end ? sn : s_end - 1);
            }
        }
    }
    // Loads past the end of the slice are still in flight.  Their destination registers must
    // stay allocated until they have landed: tie every stage after the wait, so that on no path
    // the compiler hands those registers to other values first.
    sm::wait_vm<0>();
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd) {
#pragma unroll
        for (int q = 0; q < G::WORDS; ++q) sm::tie(st[dd].w[q]);
        sm::tie(st[dd].sc);
        sm::tie(st[dd].z);
    }

    // D register v of lane (i, j): row 4j + v, columns n + cs.  The finish kernel (next launch
    // on the stream) adds the slices' partial tiles.
    float *mine = d.Yacc + (size_t)ks * 16 * N;
    if (col_ok) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (4 * j + v < d.M)
                *reinterpret_cast<float4 *>(mine + (size_t)(4 * j + v) * N + n) =
                    make_float4(yacc[0][v], yacc[1][v], yacc[2][v], yacc[3][v]);
    }
}

// Sum of the K slices' partial tiles, then the adapter term and the bfloat16 store.  One
// workgroup per 64 columns: thread t owns row t / 16, columns 4 (t % 16) .. + 3.
__global__ __launch_bounds__(sm::WG_THREADS) void smallm_fwd_finish_kernel(SmallFwdDev d) {
    __shared__ float Us[16 * 64];
    const int tid = threadIdx.x, N = d.w.N;
    const int m = tid >> 4, col = blockIdx.x * 64 + 4 * (tid & 15);
    float y[4] = {0.f, 0.f, 0.f, 0.f};
    if (m < d.M && col < N) {
        for (int q = 0; q < d.ksplit; ++q) {
            const float4 v = *reinterpret_cast<const float4 *>(d.Yacc + ((size_t)q * 16 + m) * N + col);
            y[0] += v.x; y[1] += v.y; y[2] += v.z; y[3] += v.w;
        }
    }
    for (int t = tid; t < 16 * d.r; t += sm::WG_THREADS) Us[t] = d.Ufinal[t];
    __syncthreads();
    if (m < d.M && col < N) smallm_store4(d, Us, m, col, y);
}

// ---------------------------------------------------------------------------------
// Backward (input gradient) at M <= 16:  dX[m][k] = sum_n dY[m][n] What[n][k]  (Figure 1,
// LPLinear.backward, with What never materialized).  With g the group of k,
//
//   dX[m][k] = sum_n (dY[m][n] scale[g][n]) q[n][k]  -  sum_n (dY[m][n] scale[g][n]) zero[g][n]
//
// so a tile of 128 output columns k inside ONE quantization group (group % 128 == 0) is a
// plain product of the scaled activations dYs = bf16(dY * scale[g]) with the codes, minus a
// per-row constant.  Codes enter the matrix cores as 128 + q as in the forward kernel; the
// zero points as exact bfloat16 in one extra MFMA per step, and one more against ones
// removes the 128:  dX = D_codes - 128 * D_ones - D_zeros, applied once at the end.
// Rounding dY * scale to bfloat16 moves the result by at most 2^-9 sum_n |dY| |What|, the
// same size as the rounding of What in the materialized form.
//
// prep: dYp = dY stored [N/8][16][8] (rows >= M zero) and per-128-n partial sums of
// dYBt = dY B^T.  One workgroup per 128 contraction elements; thread (m, chunk of 8).
// ---------------------------------------------------------------------------------
template <int RP>
__global__ __launch_bounds__(256) void smallm_prep_bwd_kernel(const uint16_t *__restrict__ dY, int M, int N,
                                                              const float *__restrict__ B, int r,
                                                              uint16_t *__restrict__ dYp, float *__restrict__ Tpart) {
    const int t = threadIdx.x, m = t >> 4, ch = t & 15;
    const int nc = blockIdx.x * sm::PREP_K + ch * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (m < M) v = *reinterpret_cast<const uint4 *>(dY + (size_t)m * N + nc);
    *reinterpret_cast<uint4 *>(dYp + ((size_t)(nc >> 3) * 16 + m) * 8) = v;
    if (r <= 0) return;
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (e & 1) ? __uint_as_float(u[e >> 1] & 0xFFFF0000u) : __uint_as_float(u[e >> 1] << 16);
#pragma unroll
    for (int jj = 0; jj < RP; ++jj) {
        float s = 0.f;
        if (jj < r) {
            const float4 b0 = *reinterpret_cast<const float4 *>(B + (size_t)jj * N + nc);
            const float4 b1 = *reinterpret_cast<const float4 *>(B + (size_t)jj * N + nc + 4);
            s = x[0] * b0.x + x[1] * b0.y + x[2] * b0.z + x[3] * b0.w + x[4] * b1.x + x[5] * b1.y + x[6] * b1.z + x[7] * b1.w;
        }
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
        if (ch == 0 && jj < r) Tpart[((size_t)blockIdx.x * 16 + m) * r + jj] = s;
    }
}

struct SmallBwdDev {
    LayerView w;
    const uint16_t *dYp;    // [N/8][16][8]
    const float *Tpart;     // [N/128][16][r]
    float *Tfinal;          // [16][r]: dYBt, summed by the reducer block of the stream kernel
    const float *A;         // [K][r]
    int M, r, n_parts;
    int nsplit;             // workgroups that share one 128-column tile (split of N)
    float lora_scale;
    uint16_t *dX;           // [M][K]
    float *T_out;           // dYBt [M][r] or NULL
    float *acc;             // [nsplit][16][K] fp32 partial tiles
    int slice_bytes;        // LDS bytes reserved for the dY slice (and, later, the wave reduction)
};

namespace smb {
constexpr int KT = 128;      // output columns per workgroup: four 32-code blocks
constexpr int NSTEP = 32;    // contraction elements per step (8 per lane group)
constexpr int MAX_STEPS = 32; // steps of one slice of N: 32 KB of dY in LDS
}

// adapter term and bfloat16 store of 8 adjacent outputs dX[m][k0 .. k0+7]
__device__ __forceinline__ void smallm_bwd_store8(const SmallBwdDev &d, const float *Ts, int m, int k0, const float y[8]) {
    float o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        float l = 0.f;
        const float *arow = d.A + (size_t)(k0 + c) * d.r;
        for (int jj = 0; jj < d.r; ++jj) l = __builtin_fmaf(Ts[m * d.r + jj], arow[jj], l);
        o[c] = __builtin_fmaf(d.lora_scale, l, y[c]);
    }
    uint4 v;
    v.x = pack_bf16x2(o[0], o[1]);
    v.y = pack_bf16x2(o[2], o[3]);
    v.z = pack_bf16x2(o[4], o[5]);
    v.w = pack_bf16x2(o[6], o[7]);
    *reinterpret_cast<uint4 *>(d.dX + (size_t)m * d.w.K + k0) = v;
}

// A workgroup owns 128 output columns k (one quantization group's scales and zeros) and a
// slice of N; its four waves split the slice and add their results through LDS.  Lane
// l = 16 j + i: i = 4 u + b picks the 32-code block b of the tile and the 8 codes 8u .. 8u+7
// of it (MFMA call c handles code 8u + c, so the lane's outputs are 8 adjacent k), j picks
// 8 adjacent n of the step.  A lane therefore loads, per step, the packed words that hold
// its 8 codes for 8 adjacent n (32 contiguous bytes per word row).
template <int BITS>
__global__ __launch_bounds__(sm::WG_THREADS, 2) void smallm_bwd_kernel(SmallBwdDev d) {
    extern __shared__ __attribute__((aligned(16))) uint4 ys[];   // [chunks of 8 n of the slice][16 rows]
    __shared__ float Ts[16 * 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (blockIdx.x == 0) {
        // reducer block: dYBt = sum of the prep kernel's partials (see the forward kernel)
        smallm_gather_parts(d.Tpart, d.n_parts, d.r, Ts);
        for (int t = tid; t < 16 * d.r; t += sm::WG_THREADS) d.Tfinal[t] = Ts[t];
        if (d.T_out != nullptr)
            for (int t = tid; t < d.M * d.r; t += sm::WG_THREADS) d.T_out[t] = Ts[t];
        return;
    }
    const int bid = blockIdx.x - 1;
    const int i = lane & 15, j = lane >> 4, b = i & 3, u = i >> 2;
    const int N = d.w.N, K = d.w.K;
    const int kb = bid / d.nsplit, ns = bid % d.nsplit;
    const int kt = kb * smb::KT;
    const int n_steps = N / smb::NSTEP;
    const int S0 = (int)((long)n_steps * ns / d.nsplit), S1 = (int)((long)n_steps * (ns + 1) / d.nsplit);
    const int W0 = S0 + (int)((long)(S1 - S0) * wave / sm::WG_WAVES);
    const int W1 = S0 + (int)((long)(S1 - S0) * (wave + 1) / sm::WG_WAVES);
    const int g = kt / d.w.group;

    // word rows of this lane, relative to the first word row of the tile
    constexpr int NROWS = BITS == 3 ? 2 : 1;
    int row0, row1 = 0;
    uint32_t bitsh = 0;                  // right shift that brings the lane's 8 codes to bit 0
    if (BITS == 4) row0 = b * 4 + u;
    else if (BITS == 2) { row0 = b * 2 + (u >> 1); bitsh = 16u * (u & 1); }
    else {
        const int lo = (24 * u) >> 5;
        row0 = b * 3 + lo;
        row1 = b * 3 + (lo + 1 > 2 ? 2 : lo + 1);
        bitsh = (24u * u) & 31u;
    }
    const uint32_t *wtile = d.w.qweight + (size_t)(kt / 32) * BITS * N;
    const uint16_t *stile = d.w.scales + (size_t)g * N;
    const uint8_t *ztile = d.w.zeros + (size_t)g * N;

    // The packed words, scales and zeros of a step (32 n) travel global -> LDS without passing
    // through registers: every lane moves one 16-byte piece per load, so a whole stage is NI
    // fully coalesced loads (128 contiguous bytes per word row).  Piece p of word row `row` sits
    // at LDS piece p ^ (row & 7) of that row: the later 16-byte reads of 16 different rows then
    // spread over the banks.  Each wave owns DEPTH private stages behind the workgroup's dY slice.
    constexpr int WR = 4 * BITS;                       // word rows of the 128-column tile
    constexpr int W_PIECES = WR * 8, S_PIECE0 = W_PIECES, Z_PIECE0 = W_PIECES + 4, N_PIECES = W_PIECES + 6;
    constexpr int NI = (N_PIECES + 63) / 64;           // loads per stage
    constexpr int STAGE_BYTES = NI * 1024;
    constexpr int DEPTH = 4;
    const char *gaddr[NI];                             // this lane's piece of load q, at step 0 of the matrix
    uint32_t gstr[NI];                                 // ... and its advance per step
#pragma unroll
    for (int q = 0; q < NI; ++q) {
        const int pc = q * 64 + lane;                  // lanes past N_PIECES sit out the last load
        if (pc < W_PIECES) {
            const int row = pc >> 3, pp = (pc & 7) ^ (row & 7);
            gaddr[q] = reinterpret_cast<const char *>(wtile) + ((size_t)row * N + pp * 4) * 4;
            gstr[q] = smb::NSTEP * 4;
        } else if (pc < Z_PIECE0) {
            gaddr[q] = reinterpret_cast<const char *>(stile) + (pc - S_PIECE0) * 16;
            gstr[q] = smb::NSTEP * 2;
        } else {
            gaddr[q] = reinterpret_cast<const char *>(ztile) + (pc < N_PIECES ? pc - Z_PIECE0 : 0) * 16;
            gstr[q] = smb::NSTEP;
        }
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)ys;
    const uint32_t stage0 = (uint32_t)d.slice_bytes + (uint32_t)wave * (DEPTH * STAGE_BYTES);   // offset of the wave's stages
    auto issue = [&](int slot, int step) {             // step: any step of the workgroup's slice
#pragma unroll
        for (int q = 0; q < NI; ++q) {
            if ((q + 1) * 64 <= N_PIECES || q * 64 + lane < N_PIECES)
                sm::ald_lds64(gaddr[q] + (size_t)step * gstr[q], lds0 + stage0 + (uint32_t)slot * STAGE_BYTES + q * 1024);
        }
    };
    auto clamp_step = [&](int s) { return s < S1 ? s : S1 - 1; };

    // the slice of dY goes straight into LDS, 1 KB (one step) per wave and load
    {
        const char *src = reinterpret_cast<const char *>(d.dYp) + (size_t)S0 * 1024;
        for (int q = wave; q < S1 - S0; q += sm::WG_WAVES) sm::ald_lds(src + (size_t)q * 1024, (uint32_t)lane * 16u, lds0 + (uint32_t)q * 1024u);
    }
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd) issue(dd, clamp_step(W0 + dd));
    sm::wait_vm<DEPTH * NI>();
    __syncthreads();

    f32x4 acc[8], accz, accs;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c][v] = 0.f;
        accz[v] = 0.f;
        accs[v] = 0.f;
    }
    const uint32_t ones4[4] = {sm::ONES, sm::ONES, sm::ONES, sm::ONES};
    const bf16x8 ones = sm::as_bf16x8(ones4);
    const uint32_t fmask = sm::opaque_sgpr(BITS == 4 ? 0x000F000Fu : (BITS == 2 ? 0x00030003u : 0x00070007u));
    const uint32_t magic = sm::opaque_vgpr(sm::MAGIC);

    struct Stage {
        sm::u32x4 w[NROWS][2];   // 8 adjacent n of each word row
        sm::u32x4 sc;            // 8 binary16 scales
        sm::u32x2 z;             // 8 zero points
    };
    auto compute = [&](int slot, int srel) {        // srel: step relative to S0
        const unsigned char *sb = reinterpret_cast<const unsigned char *>(ys) + stage0 + slot * STAGE_BYTES;
        Stage sd;
        sd.w[0][0] = *reinterpret_cast<const sm::u32x4 *>(sb + row0 * 128 + (((2 * j) ^ (row0 & 7)) << 4));
        sd.w[0][1] = *reinterpret_cast<const sm::u32x4 *>(sb + row0 * 128 + (((2 * j + 1) ^ (row0 & 7)) << 4));
        if (NROWS == 2) {
            sd.w[NROWS - 1][0] = *reinterpret_cast<const sm::u32x4 *>(sb + row1 * 128 + (((2 * j) ^ (row1 & 7)) << 4));
            sd.w[NROWS - 1][1] = *reinterpret_cast<const sm::u32x4 *>(sb + row1 * 128 + (((2 * j + 1) ^ (row1 & 7)) << 4));
        }
        sd.sc = *reinterpret_cast<const sm::u32x4 *>(sb + S_PIECE0 * 16 + 16 * j);
        sd.z = *reinterpret_cast<const sm::u32x2 *>(sb + Z_PIECE0 * 16 + 8 * j);
        // A operand: dY[i][8 n] * scale[g][8 n], rounded to bfloat16
        const uint4 yv = ys[((size_t)srel * 4 + j) * 16 + i];
        const uint32_t yw[4] = {yv.x, yv.y, yv.z, yv.w};
        uint32_t areg[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const float y0 = __uint_as_float(yw[p] << 16), y1 = __uint_as_float(yw[p] & 0xFFFF0000u);
            const float s0 = half_bits_to_float((uint16_t)(sd.sc[p] & 0xFFFFu)), s1 = half_bits_to_float((uint16_t)(sd.sc[p] >> 16));
            areg[p] = pack_bf16x2(y0 * s0, y1 * s1);
        }
        const bf16x8 a = sm::as_bf16x8(areg);
        // the lane's 8 codes of each of its 8 n, at bit 0 of ch[e]
        uint32_t ch[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t lo = sd.w[0][e >> 2][e & 3];
            if (BITS == 4) ch[e] = lo;
            else if (BITS == 2) ch[e] = lo >> bitsh;
            else ch[e] = __builtin_amdgcn_alignbit(sd.w[NROWS - 1][e >> 2][e & 3], lo, bitsh);
        }
        // pairs of n side by side: low halves (bits 0-15) and, where codes reach further, a second view
        uint32_t plo[4], phi[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            plo[p] = __builtin_amdgcn_perm(ch[2 * p + 1], ch[2 * p], 0x05040100u);
            if (BITS == 4) phi[p] = __builtin_amdgcn_perm(ch[2 * p + 1], ch[2 * p], 0x07060302u);        // bits 16-31
            else if (BITS == 3) phi[p] = __builtin_amdgcn_perm(ch[2 * p + 1], ch[2 * p], 0x06050201u);   // bits 8-23
            else phi[p] = 0;
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            uint32_t o[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                uint32_t x;
                if (BITS == 4) x = c < 4 ? plo[p] >> (4 * c) : phi[p] >> (4 * (c - 4));
                else if (BITS == 2) x = plo[p] >> (2 * c);
                else x = c < 5 ? plo[p] >> (3 * c) : phi[p] >> (3 * c - 8);
                o[p] = sm::and_or(x, fmask, magic);
            }
            acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sm::as_bf16x8(o), acc[c], 0, 0, 0);
        }
        // zero points as exact bfloat16
        uint32_t zo[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t zw = sd.z[p >> 1] >> (16 * (p & 1));
            zo[p] = pack_bf16x2((float)(zw & 0xFFu), (float)((zw >> 8) & 0xFFu));
        }
        accz = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sm::as_bf16x8(zo), accz, 0, 0, 0);
        accs = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ones, accs, 0, 0, 0);
    };

    for (int s = W0; s < W1; s += DEPTH) {
#pragma unroll
        for (int dd = 0; dd < DEPTH; ++dd) {
            if (s + dd < W1) {
                sm::wait_vm<(DEPTH - 1) * NI>();     // this wave's stage dd has landed; DEPTH - 1 younger ones in flight
                compute(dd, s + dd - S0);
                issue(dd, clamp_step(s + dd + DEPTH));
            }
        }
    }
    // loads past the end of the slice are still in flight towards this workgroup's LDS
    sm::wait_vm<0>();
    __syncthreads();                                 // every wave is done with the dY slice

    // the four waves' tiles meet in LDS: red[wave][c * 4 + v][lane]
    float *red = reinterpret_cast<float *>(ys);
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            red[(wave * 32 + c * 4 + v) * 64 + lane] = acc[c][v] - 128.0f * accs[v] - accz[v];
    __syncthreads();
    // thread (wave, lane) finishes D register v = wave of lane's position: row 4j + wave, 8 adjacent k
    float y[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        float sum = 0.f;
#pragma unroll
        for (int wv = 0; wv < sm::WG_WAVES; ++wv) sum += red[(wv * 32 + c * 4 + wave) * 64 + lane];
        y[c] = sum;
    }
    const int m = 4 * j + wave, k0 = kt + 32 * b + 8 * u;
    if (m < d.M) {
        float *dst = d.acc + ((size_t)ns * 16 + m) * K + k0;
        *reinterpret_cast<float4 *>(dst) = make_float4(y[0], y[1], y[2], y[3]);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(y[4], y[5], y[6], y[7]);
    }
}

// Sum of the N slices' partial tiles, adapter term, bfloat16 store.  One workgroup per 128
// columns: thread t owns row t / 16, columns 8 (t % 16) .. + 7.
__global__ __launch_bounds__(sm::WG_THREADS) void smallm_bwd_finish_kernel(SmallBwdDev d) {
    __shared__ float Ts[16 * 64];
    const int tid = threadIdx.x, K = d.w.K;
    const int m = tid >> 4, k0 = blockIdx.x * 128 + 8 * (tid & 15);
    float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (m < d.M) {
        for (int q = 0; q < d.nsplit; ++q) {
            const float *src = d.acc + ((size_t)q * 16 + m) * K + k0;
            const float4 v0 = *reinterpret_cast<const float4 *>(src), v1 = *reinterpret_cast<const float4 *>(src + 4);
            y[0] += v0.x; y[1] += v0.y; y[2] += v0.z; y[3] += v0.w;
            y[4] += v1.x; y[5] += v1.y; y[6] += v1.z; y[7] += v1.w;
        }
    }
    for (int t = tid; t < 16 * d.r; t += sm::WG_THREADS) Ts[t] = d.Tfinal[t];
    __syncthreads();
    if (m < d.M) smallm_bwd_store8(d, Ts, m, k0, y);
}

namespace {
// K slices for a product with contraction length Kc (groups of `group`) and Nout outputs:
// enough workgroups to fill the chip, slices of whole groups that fit the LDS, at most
// MAX_KSPLIT.  Returns 0 when no such split exists.
int pick_ksplit(int Kc, int Nout, int group) {
    if (group > sm::MAX_RANGE) return 0;
    const int n_groups = Kc / group;
    const int gmax = sm::MAX_RANGE / group;                    // groups per slice that fit the LDS
    const int need = (n_groups + gmax - 1) / gmax;
    const int col_blocks = (Nout + sm::BCOLS - 1) / sm::BCOLS;
    int ksplit = (512 + col_blocks - 1) / col_blocks;
    if (ksplit < need) ksplit = need;
    if (ksplit > n_groups) ksplit = n_groups;
    if (ksplit > sm::MAX_KSPLIT) ksplit = sm::MAX_KSPLIT;
    if (ksplit < need) return 0;
    // every slice holds at most ceil(n_groups / ksplit) groups
    if ((long)((n_groups + ksplit - 1) / ksplit) * group > sm::MAX_RANGE) return 0;
    return ksplit;
}
// upper bound of pick_ksplit over all group sizes (for the workspace query)
int ksplit_bound(int Kc, int Nout) {
    const int col_blocks = (Nout + sm::BCOLS - 1) / sm::BCOLS;
    int b = (512 + col_blocks - 1) / col_blocks;
    const int need = (Kc + 1023) / 1024;
    if (b < need) b = need;
    if (b > sm::MAX_KSPLIT) b = sm::MAX_KSPLIT;
    return b;
}
// N slices of the backward product (contraction length N, K outputs in tiles of 128)
int pick_nsplit(int N, int K) {
    const int n_steps = N / smb::NSTEP;
    const int k_blocks = K / smb::KT;
    const int max_steps = smb::MAX_STEPS;                      // steps of one slice that fit the LDS
    const int need = (n_steps + max_steps - 1) / max_steps;
    int nsplit = (512 + k_blocks - 1) / k_blocks;
    if (nsplit < need) nsplit = need;
    if (nsplit > n_steps) nsplit = n_steps;
    if (nsplit > sm::MAX_KSPLIT) nsplit = sm::MAX_KSPLIT;
    if (nsplit < need || nsplit < 1) return 0;
    return nsplit;
}
}  // namespace

bool smallm_bwd_supported(const LayerView &w, int M) {
    if (M > 16) return false;
    return w.group % smb::KT == 0 && w.N % sm::PREP_K == 0 && pick_nsplit(w.N, w.K) > 0;
}

bool smallm_fwd_supported(const LayerView &w, int M) {
    if (M > 16) return false;
    const int kstep = w.bits == 4 ? 32 : (w.bits == 2 ? 64 : 128);
    return w.group % kstep == 0 && w.K % sm::PREP_K == 0 && pick_ksplit(w.K, w.N, w.group) > 0;
}

namespace {
struct SmallWs {
    size_t xp, upart, ufinal, yacc, total;
};
SmallWs small_ws(int K, int N, int r) {
    const size_t kmax = (size_t)(K > N ? K : N);
    auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
    SmallWs l;
    size_t off = 0;
    l.xp = off;      off += al((size_t)16 * kmax * 2);
    l.upart = off;   off += al(((kmax + sm::PREP_K - 1) / sm::PREP_K) * 16 * (size_t)(r > 0 ? r : 1) * 4);
    l.ufinal = off;  off += al((size_t)16 * 64 * 4);
    const size_t yf = (size_t)ksplit_bound(K, N) * 16 * N, yb = (size_t)sm::MAX_KSPLIT * 16 * K;
    l.yacc = off;    off += al((yf > yb ? yf : yb) * 4);
    l.total = off;
    return l;
}
}  // namespace

size_t smallm_ws_bytes(int K, int N, int r) { return small_ws(K, N, r).total; }

template <int BITS>
static hipError_t launch_fwd_bits(const SmallFwdDev &d, int col_blocks, size_t lds_bytes, hipStream_t stream) {
    auto kern = smallm_fwd_kernel<BITS>;
    static bool configured[64] = {};
    const hipError_t e = ensure_lds_limit(reinterpret_cast<const void *>(kern), (size_t)sm::MAX_RANGE * 32, configured);
    if (e != hipSuccess) return e;
    launch_kernel("stream_fwd", kern, col_blocks * d.ksplit + 1, sm::WG_THREADS, lds_bytes, stream, d);   // + the reducer block
    return hipGetLastError();
}

hipError_t launch_smallm_fwd(const SmallArgs &a, hipStream_t stream) {
    const int K = a.w.K, N = a.w.N;
    const SmallWs l = small_ws(K, N, a.r);
    char *ws = static_cast<char *>(a.ws);
    uint16_t *Xp = reinterpret_cast<uint16_t *>(ws + l.xp);
    float *Upart = reinterpret_cast<float *>(ws + l.upart);
    float *Yacc = reinterpret_cast<float *>(ws + l.yacc);
    const int n_kparts = K / sm::PREP_K;
    const int col_blocks = (N + sm::BCOLS - 1) / sm::BCOLS;
    const int ksplit = pick_ksplit(K, N, a.w.group);
    if (ksplit < 1) return hipErrorInvalidValue;     // callers check smallm_fwd_supported first

    auto prep = a.r <= 8 ? smallm_prep_fwd_kernel<8> : (a.r <= 16 ? smallm_prep_fwd_kernel<16> : smallm_prep_fwd_kernel<64>);
    launch_kernel("smallm_prep_fwd", prep, n_kparts, 256, 0, stream, a.act, a.M, K, a.w.bits, a.A, a.r, Xp, Upart, n_kparts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    SmallFwdDev d;
    d.w = a.w;
    d.Xp = Xp;
    d.Upart = Upart;
    d.Ufinal = reinterpret_cast<float *>(ws + l.ufinal);
    d.B = a.B;
    d.M = a.M;
    d.r = a.r;
    d.n_kparts = n_kparts;
    d.ksplit = ksplit;
    d.lora_scale = a.lora_scale;
    d.Y = a.out;
    d.XA = a.P_out;
    d.Yacc = Yacc;
    // LDS for the largest slice: ceil(groups / ksplit) groups of 32 bytes per contraction element
    const int n_groups = K / a.w.group;
    const size_t lds_bytes = (size_t)((n_groups + ksplit - 1) / ksplit) * a.w.group * 32;
    switch (a.w.bits) {
        case 2: e = launch_fwd_bits<2>(d, col_blocks, lds_bytes, stream); break;
        case 3: e = launch_fwd_bits<3>(d, col_blocks, lds_bytes, stream); break;
        default: e = launch_fwd_bits<4>(d, col_blocks, lds_bytes, stream); break;
    }
    if (e != hipSuccess) return e;
    launch_kernel("stream_fwd_finish", smallm_fwd_finish_kernel, (N + 63) / 64, sm::WG_THREADS, 0, stream, d);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_bwd_bits(const SmallBwdDev &d, int k_blocks, size_t lds_bytes, hipStream_t stream) {
    auto kern = smallm_bwd_kernel<BITS>;
    static bool configured[64] = {};
    const hipError_t e = ensure_lds_limit(reinterpret_cast<const void *>(kern), (size_t)80 * 1024, configured);
    if (e != hipSuccess) return e;
    launch_kernel("stream_bwd", kern, k_blocks * d.nsplit + 1, sm::WG_THREADS, lds_bytes, stream, d);   // + the reducer block
    return hipGetLastError();
}

hipError_t launch_smallm_bwd(const SmallArgs &a, hipStream_t stream) {
    const int K = a.w.K, N = a.w.N;
    const SmallWs l = small_ws(K, N, a.r);
    char *ws = static_cast<char *>(a.ws);
    uint16_t *dYp = reinterpret_cast<uint16_t *>(ws + l.xp);
    float *Tpart = reinterpret_cast<float *>(ws + l.upart);
    const int n_parts = N / sm::PREP_K;
    const int k_blocks = K / smb::KT;
    const int nsplit = pick_nsplit(N, K);
    if (nsplit < 1) return hipErrorInvalidValue;     // callers check smallm_bwd_supported first

    auto prep = a.r <= 8 ? smallm_prep_bwd_kernel<8> : (a.r <= 16 ? smallm_prep_bwd_kernel<16> : smallm_prep_bwd_kernel<64>);
    launch_kernel("smallm_prep_bwd", prep, n_parts, 256, 0, stream, a.act, a.M, N, a.B, a.r, dYp, Tpart);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    SmallBwdDev d;
    d.w = a.w;
    d.dYp = dYp;
    d.Tpart = Tpart;
    d.Tfinal = reinterpret_cast<float *>(ws + l.ufinal);
    d.A = a.A;
    d.M = a.M;
    d.r = a.r;
    d.n_parts = n_parts;
    d.nsplit = nsplit;
    d.lora_scale = a.lora_scale;
    d.dX = a.out;
    d.T_out = a.P_out;
    d.acc = reinterpret_cast<float *>(ws + l.yacc);
    // LDS: the largest slice of dY (1 KB per step; at least the 32 KB of the wave reduction), then
    // 4 waves x 4 stages of packed words (3 KB per stage for 4-bit, 2 KB otherwise)
    d.slice_bytes = 32 * 1024;
    const size_t lds_bytes = (size_t)d.slice_bytes + 16 * (size_t)(a.w.bits == 4 ? 3072 : 2048);
    switch (a.w.bits) {
        case 2: e = launch_bwd_bits<2>(d, k_blocks, lds_bytes, stream); break;
        case 3: e = launch_bwd_bits<3>(d, k_blocks, lds_bytes, stream); break;
        default: e = launch_bwd_bits<4>(d, k_blocks, lds_bytes, stream); break;
    }
    if (e != hipSuccess) return e;
    launch_kernel("stream_bwd_finish", smallm_bwd_finish_kernel, k_blocks, sm::WG_THREADS, 0, stream, d);
    return hipGetLastError();
}

}  // namespace mlr
