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
// help of an MFMA against a vector of ones (it yields sum_k X[m][k], which the zero point
// needs anyway); these sums depend on the activations only, so a workgroup computes them once
// per quantization group of its slice, and every product starts from minus the offsets'
// share instead of zero.  Which two codes share a register is fixed by the bit
// layout, so every workgroup re-orders its slice of X to the same order on its way into LDS.
// For 3-bit codes the
// low field of a register lands four bits high; there the field is OR-ed into bfloat16 8.0
// (0x4100) instead, whose mantissa bit 4 has weight one: 8 + q.  The offsets (8 or 128 times
// X) are removed by one MFMA against the vector of the offsets themselves.
#include "device_common.h"
#include "gemm_common.h"
#include "launch.h"

namespace mlr {

namespace sm {
constexpr int WG_WAVES = 4, WG_THREADS = WG_WAVES * 64;      // backward stream and finish kernels
constexpr int FWD_WAVES = 8, FWD_THREADS = FWD_WAVES * 64;  // forward stream kernel: one workgroup per compute unit
constexpr int PREP_K = 128;            // the contraction length must be a multiple of this
constexpr int MAX_KSPLIT = 32;         // workgroups that may share a column block
// Number format of the activations and of the operands built from the codes: bfloat16, or binary16
// for the layer in the paper's own storage convention (F16).  A b-bit field OR-ed into the mantissa
// of a power of two whose unit in the last place is one gives that power of two plus the code:
// bfloat16 128.0 (7 mantissa bits), binary16 1024.0 (10 mantissa bits); with the field four bits up,
// bfloat16 8.0 or binary16 64.0.
template <bool F16> struct Num {
    static constexpr uint32_t MAGIC = F16 ? 0x64006400u : 0x43004300u;    // two 1024.0 / two 128.0
    static constexpr uint32_t MAGIC3 = F16 ? 0x64005400u : 0x43004100u;   // (64.0, 1024.0) / (8.0, 128.0): 3-bit forward, low field at bits 4-6
    static constexpr uint32_t ONES = F16 ? 0x3C003C00u : 0x3F803F80u;     // two 1.0
    static constexpr float OFFSET = F16 ? 1024.0f : 128.0f;
};
constexpr uint32_t MAGIC = Num<false>::MAGIC;
constexpr uint32_t MAGIC3 = Num<false>::MAGIC3;
constexpr uint32_t ONES = Num<false>::ONES;
typedef _Float16 half16x8 __attribute__((ext_vector_type(8)));

// D = A B + C on a 16 x 16 x 32 tile, operands given as four registers of 16-bit pairs
template <bool F16>
__device__ __forceinline__ f32x4 mma(const bf16x8 &a, const bf16x8 &b, const f32x4 &c) {
    if (F16) {
        half16x8 x, y;
        __builtin_memcpy(&x, &a, 16);
        __builtin_memcpy(&y, &b, 16);
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(x, y, c, 0, 0, 0);
    }
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// two fp32 -> a pair of 16-bit floats (round to nearest even), `lo` in the low half
template <bool F16>
__device__ __forceinline__ uint32_t pack16(float lo, float hi) {
    return pack_pair<F16>(lo, hi);
}
// a stored 16-bit float -> fp32 (exact)
template <bool F16>
__device__ __forceinline__ float widen16(uint32_t bits16) {
    return F16 ? half_bits_to_float((uint16_t)bits16) : __uint_as_float(bits16 << 16);
}

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

template <int BITS, bool F16>
__device__ __forceinline__ CodeMasks make_masks() {
    CodeMasks m;
    m.field = opaque_sgpr(BITS == 4 ? 0x000F000Fu : (BITS == 2 ? 0x00030003u : 0x00070070u));
    m.magic = opaque_vgpr(BITS == 3 ? Num<F16>::MAGIC3 : Num<F16>::MAGIC);
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
        // 24-bit chunk c of the 96-bit block (stream bits 24c .. 24c+23); reg p = (code p,
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

}  // namespace sm

// ---------------------------------------------------------------------------------
// The rank-r projection of the (at most 16) activation rows, XA = X A or dYBt = dY B^T, for
// the adapter term: done by the first `nblk` workgroups of a stream kernel beside the
// streaming ones, on the matrix cores (16x16x32 bf16 MFMA; the fp32 factor split exactly
// into three bfloat16 terms).  The waves of those workgroups split the contraction; each
// workgroup leaves one partial [16][r] and the finish kernel adds the nblk of them.
// Lane l = 16 cs + i: activation row i (rows >= M repeat row M - 1; their results are never
// used), factor column 16 g + i, contraction elements 8 cs .. 8 cs + 7 of a step of 32.
// ---------------------------------------------------------------------------------
template <bool F_IS_A, int NWAVES>
__device__ __forceinline__ void smallm_project(const uint16_t *act, int M, int C, const float *F, int r, int blk,
                                               int nblk, float *parts, float *red /* LDS, NWAVES * 4 * 256 floats */) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, cs = lane >> 4;
    const uint16_t *arow = act + (size_t)(i < M ? i : M - 1) * C;
    const int steps = C / 32;
    const long part = (long)blk * NWAVES + wave, nparts = (long)nblk * NWAVES;
    const int s0 = (int)(steps * part / nparts), s1 = (int)(steps * (part + 1) / nparts);
    const int RG = (r + 15) >> 4;
    f32x4 acc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int st = s0; st < s1; st += 2) {
        uint4 av[2];
        bool ok[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            ok[q] = st + q < s1;
            av[q] = make_uint4(0, 0, 0, 0);
            if (ok[q]) av[q] = *reinterpret_cast<const uint4 *>(arow + (st + q) * 32 + cs * 8);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (g >= RG) break;
            const int j = g * 16 + i;
            float f[2][8];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int c = (st + q) * 32 + cs * 8;
#pragma unroll
                for (int e = 0; e < 8; ++e) f[q][e] = 0.f;
                if (ok[q] && j < r) {
                    if (F_IS_A) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) f[q][e] = F[(size_t)(c + e) * r + j];
                    } else {
                        const float4 q0 = *reinterpret_cast<const float4 *>(F + (size_t)j * C + c);
                        const float4 q1 = *reinterpret_cast<const float4 *>(F + (size_t)j * C + c + 4);
                        f[q][0] = q0.x; f[q][1] = q0.y; f[q][2] = q0.z; f[q][3] = q0.w;
                        f[q][4] = q1.x; f[q][5] = q1.y; f[q][6] = q1.z; f[q][7] = q1.w;
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                uint32_t hi[4], mid[4], lo[4];
                split3(f[q], hi, mid, lo);
                const bf16x8 a = sm::as_bf16x8(av[q]);
                acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sm::as_bf16x8(hi), acc[g], 0, 0, 0);
                acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sm::as_bf16x8(mid), acc[g], 0, 0, 0);
                acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sm::as_bf16x8(lo), acc[g], 0, 0, 0);
            }
        }
    }
    // D register v of lane (i, cs): row 4 cs + v, column 16 g + i
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[((wave * 4 + g) * 4 + v) * 64 + lane] = acc[g][v];
    __syncthreads();
    float *mine = parts + (size_t)blk * 16 * r;
    for (int x = tid; x < RG * 256; x += NWAVES * 64) {
        const int g = x >> 8, v = (x >> 6) & 3, l = x & 63;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) sum += red[((w * 4 + g) * 4 + v) * 64 + l];
        const int prow = 4 * (l >> 4) + v, j = g * 16 + (l & 15);
        if (j < r) mine[prow * r + j] = sum;
    }
}

// The same projection for binary16 activations (the layer in the paper's own storage convention),
// in plain fp32 on the vector ALUs: a binary16 activation does not fit a bfloat16 operand, and at
// most 16 rows by a few thousand contraction elements per workgroup are too little work to matter.
// Thread t: row t % 16, chunks of 8 contraction elements (t / 16) + k * (threads / 16) of the
// workgroup's range (one 16-byte activation load per chunk, and every factor load of the chunk in
// flight with it); eight rank columns per pass; the threads' sums meet in LDS.  Same partial layout
// as above: one [16][r] per workgroup.
template <bool F_IS_A, int NWAVES>
__device__ __forceinline__ void smallm_project_f16(const uint16_t *act, int M, int C, const float *F, int r, int blk,
                                                   int nblk, float *parts, float *red /* LDS, NWAVES * 64 * 8 floats */) {
    constexpr int NT = NWAVES * 64, KL = NT / 16;
    const int tid = threadIdx.x, m = tid & 15, kl = tid >> 4;
    const int chunks = C >> 3;
    const int ch0 = (int)((long)chunks * blk / nblk), ch1 = (int)((long)chunks * (blk + 1) / nblk);
    const uint16_t *arow = act + (size_t)(m < M ? m : M - 1) * C;
    float *mine = parts + (size_t)blk * 16 * r;
    for (int j0 = 0; j0 < r; j0 += 8) {
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        for (int ch = ch0 + kl; ch < ch1; ch += KL) {
            const int c = ch << 3;
            const uint4 xv = *reinterpret_cast<const uint4 *>(arow + c);
            const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = half_bits_to_float((uint16_t)(xw[e >> 1] >> (16 * (e & 1))));
            float f[8][8];       // [rank column][contraction element]
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool ok = j0 + j < r;
                if (F_IS_A) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[j][e] = ok ? F[(size_t)(c + e) * r + j0 + j] : 0.f;
                } else {
                    const float *src = F + (size_t)(ok ? j0 + j : 0) * C + c;     // 32-byte aligned: C is a multiple of 8
                    const float4 q0 = *reinterpret_cast<const float4 *>(src), q1 = *reinterpret_cast<const float4 *>(src + 4);
                    f[j][0] = q0.x; f[j][1] = q0.y; f[j][2] = q0.z; f[j][3] = q0.w;
                    f[j][4] = q1.x; f[j][5] = q1.y; f[j][6] = q1.z; f[j][7] = q1.w;
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[j] = __builtin_fmaf(x[e], f[j][e], acc[j]);
        }
        __syncthreads();                         // the previous pass has been read
#pragma unroll
        for (int j = 0; j < 8; ++j) red[(kl * 16 + m) * 8 + j] = acc[j];
        __syncthreads();
        if (tid < 128) {                         // (row, column) = (tid / 8, tid % 8)
            float sum = 0.f;
            for (int q = 0; q < KL; ++q) sum += red[(q * 16 + (tid >> 3)) * 8 + (tid & 7)];
            if (j0 + (tid & 7) < r) mine[(tid >> 3) * r + j0 + (tid & 7)] = sum;
        }
    }
}

// Sum of the projection workgroups' partials into Us (16 x r floats in LDS).
template <int EPT>
__device__ __forceinline__ void smallm_sum_parts(const float *parts, int n_parts, int r, float *Us) {
    // EPT elements per thread and up to sixteen workgroups' partials of each in flight together
    // (n_parts <= 32), so that a small workgroup and a large rank still wait for few round trips
    const int n = 16 * r, stride = blockDim.x;
    for (int t0 = threadIdx.x; t0 < n; t0 += EPT * stride) {
        float sum[EPT];
#pragma unroll
        for (int q = 0; q < EPT; ++q) sum[q] = 0.f;
        for (int b0 = 0; b0 < n_parts; b0 += 16) {
            float v[EPT][16];
#pragma unroll
            for (int q = 0; q < EPT; ++q) {
                const int t = t0 + q * stride;
#pragma unroll
                for (int b = 0; b < 16; ++b) {     // clamped, not predicated: past the end the last one is re-read and not added
                    const int bb = b0 + b < n_parts ? b0 + b : n_parts - 1;
                    v[q][b] = parts[(size_t)bb * n + (t < n ? t : n - 1)];
                }
            }
#pragma unroll
            for (int q = 0; q < EPT; ++q)
#pragma unroll
                for (int b = 0; b < 16; ++b) sum[q] += b0 + b < n_parts ? v[q][b] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < EPT; ++q)
            if (t0 + q * stride < n) Us[t0 + q * stride] = sum[q];
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------
// forward stream kernel.  A workgroup of 8 waves owns 512 output columns and one slice of K
// (a run of whole quantization groups); each wave owns 64 of the columns.  The slice of the
// re-ordered activations sits in LDS, shared by the eight waves (one workgroup per compute
// unit: all its waves get their activations, and start on the weights, together).  Inside a wave, lane
// l = 16 j + i holds columns n0 + 4i .. 4i+3 (one 16-byte load per packed word row, 256
// contiguous bytes per 16-lane group) and the k-slice j of each MFMA call.  Packed words,
// scales and zeros are loaded DEPTH steps ahead by loads issued from assembly and awaited
// with an exact count; loads past the end of the slice are clamped to its last step, so the
// number in flight never changes and the loop needs no predicates.  The 16 x 64 fp32 result
// of a wave is final for the slice and is stored as a partial tile for the finish kernel.
// ---------------------------------------------------------------------------------
struct SmallFwdDev {
    LayerView w;
    const uint16_t *X;      // [M][K]
    const float *A;         // [K][r]
    float *Upart;           // [n_proj][16][r]: partials of XA = X A, left by the projection workgroups
    const float *B;         // [r][N]
    int M, r, n_proj;       // n_proj: workgroups of the stream kernel that do the projection
    int ksplit;             // workgroups that share one column block (split of the groups along K)
    float lora_scale;
    uint16_t *Y;            // [M][N]
    float *XA;              // [M][r] or NULL
    float *Yacc;            // [ksplit][16][N] fp32 partial tiles
    // the layer in the paper's own storage convention (F16 kernels only; w.zeros unused there)
    const uint16_t *zeros16;   // binary16 [K/group][N], added
    const uint16_t *bias16;    // binary16 [N] or NULL
};

namespace sm {
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void ald(u32x4 &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
// the same without the non-temporal hint, for data that other workgroups read again
__device__ __forceinline__ void ald_cached(u32x4 &dst, const void *gaddr_lane) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(gaddr_lane) : "memory");
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
// that the incoming data cannot overtake a read of the slot it replaces.  STREAM: data that is
// read once (non-temporal hint).
template <bool STREAM>
__device__ __forceinline__ void ald_lds64(const void *gaddr_lane, uint32_t lds_base_uniform) {
    if (STREAM)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                     :
                     : "s"(lds_base_uniform), "v"(gaddr_lane)
                     : "memory");
    else
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
// wait_vm<BASE + extra>() for 0 <= extra < 16 known after unrolling
template <int BASE>
__device__ __forceinline__ void wait_vm_plus(int extra) {
    switch (extra) {
        case 0: wait_vm<BASE>(); break;
        case 1: wait_vm<BASE + 1>(); break;
        case 2: wait_vm<BASE + 2>(); break;
        case 3: wait_vm<BASE + 3>(); break;
        case 4: wait_vm<BASE + 4>(); break;
        case 5: wait_vm<BASE + 5>(); break;
        case 6: wait_vm<BASE + 6>(); break;
        case 7: wait_vm<BASE + 7>(); break;
        case 8: wait_vm<BASE + 8>(); break;
        case 9: wait_vm<BASE + 9>(); break;
        case 10: wait_vm<BASE + 10>(); break;
        case 11: wait_vm<BASE + 11>(); break;
        case 12: wait_vm<BASE + 12>(); break;
        case 13: wait_vm<BASE + 13>(); break;
        case 14: wait_vm<BASE + 14>(); break;
        default: wait_vm<BASE + 15>(); break;
    }
}
// 16-byte store of a partial tile: written once, read once by the next launch (non-temporal,
// so the lines leave the L2 as they fill instead of waiting for the end-of-kernel write-back)
typedef float f32x4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_stream(float *dst, float a, float b, float c, float d) {
    f32x4v v = {a, b, c, d};
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4v *>(dst));
}
template <typename T>
__device__ __forceinline__ void tie(T &x) {
    asm volatile("" : "+v"(x)::"memory");
}
constexpr int WCOLS = 64;                 // columns per wave (4 per lane of a 16-lane group)
constexpr int BCOLS = FWD_WAVES * WCOLS;  // columns per workgroup
constexpr int MAX_RANGE = 2048;           // contraction elements of one K slice (64 KB of LDS)
}  // namespace sm

// The eight rows jj0 .. jj0 + 7 of B at columns col .. col + 7, all loads issued together (rows
// past r come back as zeros).
constexpr int FIN_BROWS = 8;
__device__ __forceinline__ void smallm_load_b8x8(const SmallFwdDev &d, int jj0, int col, float4 b[FIN_BROWS][2]) {
#pragma unroll
    for (int q = 0; q < FIN_BROWS; ++q) {
        b[q][0] = make_float4(0.f, 0.f, 0.f, 0.f);
        b[q][1] = b[q][0];
        if (jj0 + q < d.r) {
            const float *src = d.B + (size_t)(jj0 + q) * d.w.N + col;
            b[q][0] = *reinterpret_cast<const float4 *>(src);
            b[q][1] = *reinterpret_cast<const float4 *>(src + 4);
        }
    }
}

// Adds the adapter term (and, F16, the bias) to the eight adjacent outputs y[0..7] of row m, columns
// col .. col + 7 (col a multiple of 8, col + 7 < N) and stores them as 16-bit floats.  `b0`: rows
// 0 .. 7 of B for these columns, loaded by the caller ahead of time.
template <bool F16>
__device__ __forceinline__ void smallm_fwd_store8(const SmallFwdDev &d, const float *Us, int m, int col, const float y[8], const float4 b0[FIN_BROWS][2]) {
    float l[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int jj0 = 0; jj0 < d.r; jj0 += FIN_BROWS) {
        float4 b[FIN_BROWS][2];
        if (jj0 == 0) {
#pragma unroll
            for (int q = 0; q < FIN_BROWS; ++q) { b[q][0] = b0[q][0]; b[q][1] = b0[q][1]; }
        } else {
            smallm_load_b8x8(d, jj0, col, b);
        }
#pragma unroll
        for (int q = 0; q < FIN_BROWS; ++q) {
            const float u = jj0 + q < d.r ? Us[m * d.r + jj0 + q] : 0.f;
            l[0] = __builtin_fmaf(u, b[q][0].x, l[0]); l[1] = __builtin_fmaf(u, b[q][0].y, l[1]);
            l[2] = __builtin_fmaf(u, b[q][0].z, l[2]); l[3] = __builtin_fmaf(u, b[q][0].w, l[3]);
            l[4] = __builtin_fmaf(u, b[q][1].x, l[4]); l[5] = __builtin_fmaf(u, b[q][1].y, l[5]);
            l[6] = __builtin_fmaf(u, b[q][1].z, l[6]); l[7] = __builtin_fmaf(u, b[q][1].w, l[7]);
        }
    }
    float bias[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (F16 && d.bias16 != nullptr) {          // the bias of Figure 1 / eq. (3): part of the frozen layer
        const uint4 bw = *reinterpret_cast<const uint4 *>(d.bias16 + col);
        const uint32_t w4[4] = {bw.x, bw.y, bw.z, bw.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bias[2 * q] = half_bits_to_float((uint16_t)(w4[q] & 0xFFFFu));
            bias[2 * q + 1] = half_bits_to_float((uint16_t)(w4[q] >> 16));
        }
    }
    float o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = __builtin_fmaf(d.lora_scale, l[c], y[c] + bias[c]);
    uint4 v;
    v.x = sm::pack16<F16>(o[0], o[1]);
    v.y = sm::pack16<F16>(o[2], o[3]);
    v.z = sm::pack16<F16>(o[4], o[5]);
    v.w = sm::pack16<F16>(o[6], o[7]);
    *reinterpret_cast<uint4 *>(d.Y + (size_t)m * d.w.N + col) = v;
}

// SPG1: a quantization group is exactly one step (KSTEP codes), so every step starts its
// sums from zero (the first MFMA of a step takes a zero C operand) and ends with the affine part.
template <int BITS, bool SPG1, bool F16>
__global__ __launch_bounds__(sm::FWD_THREADS, 4) void smallm_fwd_kernel(SmallFwdDev d) {
    using G = sm::Geo<BITS>;
    extern __shared__ __attribute__((aligned(16))) uint4 xs[];   // [chunks of the slice][16 rows]
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if ((int)blockIdx.x < d.n_proj) {
        // projection workgroups: partials of XA = X A for the finish kernel; they run beside the
        // streaming ones and are done long before them
        if (F16) smallm_project_f16<true, sm::FWD_WAVES>(d.X, d.M, d.w.K, d.A, d.r, blockIdx.x, d.n_proj, d.Upart, reinterpret_cast<float *>(xs));
        else smallm_project<true, sm::FWD_WAVES>(d.X, d.M, d.w.K, d.A, d.r, blockIdx.x, d.n_proj, d.Upart, reinterpret_cast<float *>(xs));
        return;
    }
    const int bid = blockIdx.x - d.n_proj;
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

    // stages in flight (the binary16 zero points take one more register per stage: one stage fewer,
    // so that the kernel stays within 128 registers)
    constexpr int DEPTH = BITS == 3 ? 3 : (F16 ? 7 : 8);
    constexpr int SL = G::WORDS + 2;                // loads per stage
    struct Stage {
        sm::u32x4 w[G::WORDS];
        sm::u32x2 sc;      // 4 binary16 scales
        uint32_t z;        // 4 integer zero points (bfloat16 layer)
        sm::u32x2 z16;     // 4 binary16 zero points (F16)
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
        if (F16) sm::ald(sd.z16, d.zeros16 + (size_t)g * N, s_voff);
        else sm::ald(sd.z, d.w.zeros + (size_t)g * N, z_voff);
    };
    // The workgroup's slice of X goes into LDS in operand order: chunk c of 8 contraction
    // elements, row m at xs[16 c + m].  Inside a chunk the elements are re-ordered to the pairing
    // the code registers have (4- and 3-bit: (0,4,1,5,2,6,3,7); 2-bit: over two chunks,
    // (0,8,1,9,2,10,3,11) and (4,12,5,13,6,14,7,15)).  Thread t takes row t % 16 of chunk
    // t / 16 (+ 16 per pass): 64 contiguous bytes per row and wave, conflict-free 16-byte LDS
    // stores.  Rows >= M are zero.
    // The loads of the whole slice (at most MAX_RANGE contraction elements) are issued from
    // assembly BEFORE the weight stages, so they return first and the re-ordering runs while the
    // weights are in flight; every lane issues all of them (clamped addresses, masked
    // afterwards), which keeps the load count the waits rely on.
    {
        const int k_begin = s_begin * G::KSTEP, n_chunks = (s_end - s_begin) * (G::KSTEP / 8);
        const int m = tid & 15;
        const uint16_t *xrow = d.X + (size_t)(m < d.M ? m : 0) * d.w.K + k_begin;
        constexpr int CPP = sm::FWD_THREADS / 16;         // chunks per pass of the workgroup
        constexpr int BATCH = sm::MAX_RANGE / 8 / CPP;
        static_assert(DEPTH * SL + BATCH - 1 < 64, "vmcnt is a 6-bit counter");
        sm::u32x4 first[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int c = (tid >> 4) + CPP * u;
            sm::ald_cached(first[u], xrow + 8 * (c < n_chunks ? c : n_chunks - 1));
        }
#pragma unroll
        for (int dd = 0; dd < DEPTH; ++dd) issue(st[dd], s_begin + dd < s_end ? s_begin + dd : s_end - 1);
        // re-order one chunk (all lanes of the wave call this together) and store it
        auto reorder_store = [&](const uint4 &raw, int c) {
            uint32_t ow[4];
            if (BITS == 2) {
                // the partner chunk c ^ 1 is held by lane ^ 16 (n_chunks is even: both or neither in range)
                uint4 pr;
                pr.x = __shfl_xor(raw.x, 16, 64);
                pr.y = __shfl_xor(raw.y, 16, 64);
                pr.z = __shfl_xor(raw.z, 16, 64);
                pr.w = __shfl_xor(raw.w, 16, 64);
                const bool odd = (c & 1) != 0;
                const uint32_t a0 = odd ? pr.z : raw.x, a1 = odd ? pr.w : raw.y;      // elements 4h .. 4h+3 of the unit
                const uint32_t b0 = odd ? raw.z : pr.x, b1 = odd ? raw.w : pr.y;      // elements 8 + 4h .. 8 + 4h+3
                ow[0] = __builtin_amdgcn_perm(b0, a0, 0x05040100u);
                ow[1] = __builtin_amdgcn_perm(b0, a0, 0x07060302u);
                ow[2] = __builtin_amdgcn_perm(b1, a1, 0x05040100u);
                ow[3] = __builtin_amdgcn_perm(b1, a1, 0x07060302u);
            } else {
                ow[0] = __builtin_amdgcn_perm(raw.z, raw.x, 0x05040100u);   // (x0, x4)
                ow[1] = __builtin_amdgcn_perm(raw.z, raw.x, 0x07060302u);   // (x1, x5)
                ow[2] = __builtin_amdgcn_perm(raw.w, raw.y, 0x05040100u);   // (x2, x6)
                ow[3] = __builtin_amdgcn_perm(raw.w, raw.y, 0x07060302u);   // (x3, x7)
            }
            if (c < n_chunks) xs[(size_t)c * 16 + m] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        };
        // every thread waits for and ties every one of its loads, in range or not; chunks past the
        // end of the slice (n_chunks is a multiple of 16 and a wave's four chunks lie inside one
        // block of 16: the same answer for all lanes of a wave) are skipped
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int c = (tid >> 4) + CPP * u;
            // the weight stages and the BATCH - 1 - u younger loads of this pass stay in flight
            sm::wait_vm_plus<DEPTH * SL>(BATCH - 1 - u);
            sm::tie(first[u]);
            if (4 * wave + CPP * u < n_chunks) {
                const bool in = m < d.M;
                reorder_store(make_uint4(in ? first[u][0] : 0u, in ? first[u][1] : 0u, in ? first[u][2] : 0u, in ? first[u][3] : 0u), c);
            }
        }
    }
    __syncthreads();

    using NF = sm::Num<F16>;
    const uint32_t ones4[4] = {NF::ONES, NF::ONES, NF::ONES, NF::ONES};
    const uint32_t offs4[4] = {NF::MAGIC3, NF::MAGIC3, NF::MAGIC3, NF::MAGIC3};   // 3-bit: the two offsets themselves
    const bf16x8 ones = sm::as_bf16x8(ones4), offs = sm::as_bf16x8(offs4);
    const sm::CodeMasks masks = sm::make_masks<BITS, F16>();

    // What the affine part of eq. (2) needs of the activations alone, once per workgroup instead of
    // in every wave's loop: for each quantization group of the slice and each row,
    //   gs[g][0][m] = -sum_k offset_k X[m][k]   (what the operands' offsets 8 / 128 / 1024 add to the product)
    //   gs[g][1][m] =  sum_k X[m][k]            (the zero point's factor)
    // by the same MFMAs against constant vectors; wave w takes groups w, w + 8, ...  Behind the
    // slice in LDS.
    float *gs = reinterpret_cast<float *>(xs + (size_t)(s_end - s_begin) * (G::KSTEP / 8) * 16);
    for (int g = wave; g < g_end - g_begin; g += sm::FWD_WAVES) {
        f32x4 a1 = {0.f, 0.f, 0.f, 0.f}, a2 = {0.f, 0.f, 0.f, 0.f};
        for (int srel = g * spg; srel < (g + 1) * spg; ++srel) {
            const uint4 *xrow = xs + ((size_t)srel * 4 * G::NC + G::NC * j) * 16 + i;
#pragma unroll
            for (int c = 0; c < G::NC; ++c) {
                const bf16x8 a = sm::as_bf16x8(xrow[c * 16]);
                a1 = sm::mma<F16>(a, BITS == 3 ? offs : ones, a1);
                if (BITS == 3) a2 = sm::mma<F16>(a, ones, a2);
            }
        }
        // D register v of lane (i, j): row 4 j + v, the same value in every column i
        if (i == 0) {
            const f32x4 neg = BITS == 3 ? f32x4{-a1[0], -a1[1], -a1[2], -a1[3]}
                                        : f32x4{-NF::OFFSET * a1[0], -NF::OFFSET * a1[1], -NF::OFFSET * a1[2], -NF::OFFSET * a1[3]};
            *reinterpret_cast<f32x4 *>(gs + (g * 2 + 0) * 16 + 4 * j) = neg;
            *reinterpret_cast<f32x4 *>(gs + (g * 2 + 1) * 16 + 4 * j) = BITS == 3 ? a2 : a1;
        }
    }
    __syncthreads();

    f32x4 yacc[4], tmp[4], xsum;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
#pragma unroll
        for (int cs = 0; cs < 4; ++cs) { yacc[cs][v] = 0.f; tmp[cs][v] = 0.f; }
        xsum[v] = 0.f;
    }

    // grel: the step's quantization group inside the slice; group_begins / group_ends: first / last step of it
    auto compute = [&](Stage &sd, int srel, int grel, bool group_begins, bool group_ends) {
        // operand chunks 4 NC srel + NC j + c of the slice, row i
        const uint4 *xrow = xs + ((size_t)srel * 4 * G::NC + G::NC * j) * 16 + i;
        uint4 xa[G::NC];
#pragma unroll
        for (int c = 0; c < G::NC; ++c) xa[c] = xrow[c * 16];
        // the products start from minus the offsets' share, so that they end at sum X q
        f32x4 start = {0.f, 0.f, 0.f, 0.f};
        if (SPG1 || group_begins) {
            start = *reinterpret_cast<const f32x4 *>(gs + (grel * 2 + 0) * 16 + 4 * j);
            xsum = *reinterpret_cast<const f32x4 *>(gs + (grel * 2 + 1) * 16 + 4 * j);
            if (!SPG1) {
#pragma unroll
                for (int cs = 0; cs < 4; ++cs) tmp[cs] = start;
            }
        }
#pragma unroll
        for (int c = 0; c < G::NC; ++c) {
            const bf16x8 a = sm::as_bf16x8(xa[c]);
            const bool fresh = SPG1 && c == 0;       // first call of a one-step group
#pragma unroll
            for (int cs = 0; cs < 4; ++cs) {
                uint32_t wq[G::WORDS], o[4];
#pragma unroll
                for (int q = 0; q < G::WORDS; ++q) wq[q] = sd.w[q][cs];
                sm::codes_to_operand<BITS>(wq, c, masks, o);
                tmp[cs] = sm::mma<F16>(a, sm::as_bf16x8(o), fresh ? start : tmp[cs]);
            }
        }
        if (!SPG1 && !group_ends) return;
        // end of a group: tmp = sum X q (the offsets' share was taken off at the start); apply zero point and scale
#pragma unroll
        for (int cs = 0; cs < 4; ++cs) {
            const float scale = half_bits_to_float((uint16_t)(sd.sc[cs >> 1] >> (16 * (cs & 1))));
            // integer zero point: w = (q - zero) scale; binary16 zero point: w = q scale + z (eq. (2) as printed)
            const float zero = F16 ? half_bits_to_float((uint16_t)(sd.z16[cs >> 1] >> (16 * (cs & 1)))) : (float)((sd.z >> (8 * cs)) & 0xFFu);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float qx = tmp[cs][v];                                                             // sum X q
                if (F16) yacc[cs][v] = __builtin_fmaf(scale, qx, __builtin_fmaf(zero, xsum[v], yacc[cs][v]));
                else yacc[cs][v] = __builtin_fmaf(scale, __builtin_fmaf(-zero, xsum[v], qx), yacc[cs][v]);
            }
        }
    };

    int cp = 0, grel = 0;   // position of the next step inside its group; that group's index inside the slice
    for (int s = s_begin; s < s_end; s += DEPTH) {
#pragma unroll
        for (int dd = 0; dd < DEPTH; ++dd) {
            if (s + dd < s_end) {
                // DEPTH - 1 younger stages stay in flight
                sm::wait_vm<(DEPTH - 1) * SL>();
#pragma unroll
                for (int q = 0; q < G::WORDS; ++q) sm::tie(st[dd].w[q]);
                sm::tie(st[dd].sc);
                if (F16) sm::tie(st[dd].z16); else sm::tie(st[dd].z);
                const bool begins = cp == 0;
                const bool ends = ++cp == spg;
                compute(st[dd], s + dd - s_begin, grel, begins, ends);
                if (ends) { cp = 0; ++grel; }
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
        if (F16) sm::tie(st[dd].z16); else sm::tie(st[dd].z);
    }

    // D register v of lane (i, j): row 4j + v, columns n + cs.  The finish kernel (next launch
    // on the stream) adds the slices' partial tiles.
    float *mine = d.Yacc + (size_t)ks * 16 * N;
    if (col_ok) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (4 * j + v < d.M)
                sm::store_stream(mine + (size_t)(4 * j + v) * N + n, yacc[0][v], yacc[1][v], yacc[2][v], yacc[3][v]);
    }
}

// Sum of the K slices' partial tiles, then the adapter term and the 16-bit store.  One single-wave
// workgroup per 32 columns (whole-chip parallelism also for a narrow output): lane l owns row
// l / 4, columns 8 (l % 4) .. + 7.  The kernel is a chain of memory round trips; everything that
// does not depend on another load is issued first and consumed last: the first sixteen slices'
// tiles, the first rows of B, and (inside smallm_sum_parts) the projection partials.
constexpr int FIN_COLS = 32, FIN_SLICES = 16;
template <bool F16>
__global__ __launch_bounds__(64) void smallm_fwd_finish_kernel(SmallFwdDev d) {
    __shared__ float Us[16 * 64];
    const int tid = threadIdx.x, N = d.w.N;
    const int m = tid >> 2, col = blockIdx.x * FIN_COLS + 8 * (tid & 3);
    const bool mine = m < d.M && col < N;          // N is a multiple of 8: all eight columns or none
    float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float4 b0[FIN_BROWS][2];
#pragma unroll
    for (int q = 0; q < FIN_BROWS; ++q) { b0[q][0] = make_float4(0.f, 0.f, 0.f, 0.f); b0[q][1] = b0[q][0]; }
    if (mine) smallm_load_b8x8(d, 0, col, b0);
    // (lanes with nothing to do read row 0, columns 0 .. 7; slices past the last one re-read the last
    // and are not added: no predicate per load)
    const float *base = d.Yacc + (mine ? (size_t)m * N + col : (size_t)0);
    // (the stride lives in a vector register: with scalar address arithmetic the sixteen slice
    // addresses of a batch are all formed up front and overflow the scalar registers)
    const uint32_t slice_stride = sm::opaque_vgpr((uint32_t)16 * (uint32_t)N);      // floats; < 2^32 bytes checked by the launcher
    float4 v0[FIN_SLICES], v1[FIN_SLICES];
    // A batch is four sets of four slices; a set is skipped as a whole (one scalar branch) when it
    // lies past the last slice, and inside a set a slice past the end re-reads the last one and is
    // added with weight 0 (weights 1 / 0 from a vector compare: a scalar condition per slice, all
    // held at once, overflows the scalar registers).
    auto load_slices = [&](int q0) {
#pragma unroll
        for (int set = 0; set < FIN_SLICES / 4; ++set) {
            if (q0 + 4 * set < d.ksplit) {
                const float *src = base + (size_t)(q0 + 4 * set) * slice_stride;
#pragma unroll
                for (int u = 4 * set; u < 4 * set + 4; ++u) {
                    v0[u] = *reinterpret_cast<const float4 *>(src);
                    v1[u] = *reinterpret_cast<const float4 *>(src + 4);
                    src += q0 + u + 1 < d.ksplit ? slice_stride : 0u;
                }
            }
        }
    };
    auto add_slices = [&](int q0) {
        const int left = (int)sm::opaque_vgpr((uint32_t)(d.ksplit - q0));
#pragma unroll
        for (int set = 0; set < FIN_SLICES / 4; ++set) {
            if (q0 + 4 * set < d.ksplit) {
#pragma unroll
                for (int u = 4 * set; u < 4 * set + 4; ++u) {
                    const float w = u < left ? 1.f : 0.f;
                    y[0] = __builtin_fmaf(w, v0[u].x, y[0]); y[1] = __builtin_fmaf(w, v0[u].y, y[1]);
                    y[2] = __builtin_fmaf(w, v0[u].z, y[2]); y[3] = __builtin_fmaf(w, v0[u].w, y[3]);
                    y[4] = __builtin_fmaf(w, v1[u].x, y[4]); y[5] = __builtin_fmaf(w, v1[u].y, y[5]);
                    y[6] = __builtin_fmaf(w, v1[u].z, y[6]); y[7] = __builtin_fmaf(w, v1[u].w, y[7]);
                }
            }
        }
    };
    load_slices(0);
    if (d.r <= 8) smallm_sum_parts<2>(d.Upart, d.n_proj, d.r, Us);     // 16 r elements over 64 lanes: no more loads than needed
    else smallm_sum_parts<4>(d.Upart, d.n_proj, d.r, Us);
    add_slices(0);
    for (int q0 = FIN_SLICES; q0 < d.ksplit; q0 += FIN_SLICES) { load_slices(q0); add_slices(q0); }
    if (blockIdx.x == 0 && d.XA != nullptr)
        for (int t = tid; t < d.M * d.r; t += 64) d.XA[t] = Us[t];
    if (mine) smallm_fwd_store8<F16>(d, Us, m, col, y, b0);
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
// Nothing of dY is staged per workgroup: the 16 x 32 piece of dY that a step needs travels with
// the step's packed words (1 KB, 64 contiguous bytes per row), so a workgroup's slice of N can
// be of any length and the grid is sized to the chip, not to the LDS.
// ---------------------------------------------------------------------------------
struct SmallBwdDev {
    LayerView w;
    const uint16_t *dY;     // [M][N]
    const float *B;         // [r][N]
    float *Tpart;           // [n_proj][16][r]: partials of dYBt = dY B^T, left by the projection workgroups
    const float *A;         // [K][r]
    int M, r, n_proj;       // n_proj: workgroups of the stream kernel that do the projection
    int nsplit;             // workgroups that share one 128-column tile (split of N)
    float lora_scale;
    uint16_t *dX;           // [M][K]
    float *T_out;           // dYBt [M][r] or NULL
    float *acc;             // [nsplit][16][K] fp32 partial tiles
    const uint16_t *zeros16;   // F16 kernels only: binary16 zero points [K/group][N], added (w.zeros unused there)
};

namespace smb {
constexpr int KT = 128;      // output columns per workgroup: four 32-code blocks
constexpr int NSTEP = 32;    // contraction elements per step (8 per lane group)
constexpr int RED_BYTES = sm::WG_WAVES * 32 * 64 * 4;   // the waves' tiles meeting in LDS
}

// A[k0 + c][jj0 .. jj0 + 7] for the eight adjacent rows c, all loads issued together (columns past
// r come back as zeros): 16-byte loads when the rows are 16-byte aligned (r a multiple of 4).
__device__ __forceinline__ void smallm_load_a8(const SmallBwdDev &d, int k0, int jj0, float4 a[8][2]) {
    const int r = d.r;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float *src = d.A + (size_t)(k0 + c) * r + jj0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            a[c][h] = make_float4(0.f, 0.f, 0.f, 0.f);
            const int j = jj0 + 4 * h;
            if ((r & 3) == 0) {
                if (j < r) a[c][h] = *reinterpret_cast<const float4 *>(src + 4 * h);
            } else {
                if (j < r) a[c][h].x = src[4 * h];
                if (j + 1 < r) a[c][h].y = src[4 * h + 1];
                if (j + 2 < r) a[c][h].z = src[4 * h + 2];
                if (j + 3 < r) a[c][h].w = src[4 * h + 3];
            }
        }
    }
}

// Adapter term and 16-bit store of 8 adjacent outputs dX[m][k0 .. k0+7].  `a0`: columns 0 .. 7 of
// the eight rows of A, loaded by the caller ahead of time.
template <bool F16>
__device__ __forceinline__ void smallm_bwd_store8(const SmallBwdDev &d, const float *Ts, int m, int k0, const float y[8], const float4 a0[8][2]) {
    float l[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int jj0 = 0; jj0 < d.r; jj0 += 8) {
        float4 a[8][2];
        if (jj0 == 0) {
#pragma unroll
            for (int c = 0; c < 8; ++c) { a[c][0] = a0[c][0]; a[c][1] = a0[c][1]; }
        } else {
            smallm_load_a8(d, k0, jj0, a);
        }
        float t[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) t[q] = jj0 + q < d.r ? Ts[m * d.r + jj0 + q] : 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            l[c] = __builtin_fmaf(t[0], a[c][0].x, l[c]);
            l[c] = __builtin_fmaf(t[1], a[c][0].y, l[c]);
            l[c] = __builtin_fmaf(t[2], a[c][0].z, l[c]);
            l[c] = __builtin_fmaf(t[3], a[c][0].w, l[c]);
            l[c] = __builtin_fmaf(t[4], a[c][1].x, l[c]);
            l[c] = __builtin_fmaf(t[5], a[c][1].y, l[c]);
            l[c] = __builtin_fmaf(t[6], a[c][1].z, l[c]);
            l[c] = __builtin_fmaf(t[7], a[c][1].w, l[c]);
        }
    }
    float o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = __builtin_fmaf(d.lora_scale, l[c], y[c]);
    uint4 v;
    v.x = sm::pack16<F16>(o[0], o[1]);
    v.y = sm::pack16<F16>(o[2], o[3]);
    v.z = sm::pack16<F16>(o[4], o[5]);
    v.w = sm::pack16<F16>(o[6], o[7]);
    *reinterpret_cast<uint4 *>(d.dX + (size_t)m * d.w.K + k0) = v;
}

// A workgroup owns 128 output columns k (one quantization group's scales and zeros) and a
// slice of N; its four waves take the steps of the slice in turn (wave w: steps w, w + 4, ...,
// so the workgroup reads 512 contiguous bytes of every word row at a time) and add their
// results through LDS at the end.  Lane l = 16 j + i: i = 4 u + b picks the 32-code block b of
// the tile and the 8 codes 8u .. 8u+7 of it (MFMA call c handles code 8u + c, so the lane's
// outputs are 8 adjacent k), j picks 8 adjacent n of the step.
// GPT: quantization groups per 128-column tile (1: group a multiple of 128; 2: group 64).
template <int BITS, bool F16 = false, int GPT = 1>
struct BwdGeo {
    static constexpr int WR = 4 * BITS;                // word rows of the 128-column tile
    // 16-byte pieces of one stage: word rows (8 per row), per group of the tile scales (4) and zeros
    // (2 of uint8, or 4 of binary16), dY (16 rows x 4)
    static constexpr int Z_PER_GROUP = F16 ? 4 : 2;
    static constexpr int W_PIECES = WR * 8, S_PIECE0 = W_PIECES, Z_PIECE0 = S_PIECE0 + 4 * GPT, Y_PIECE0 = Z_PIECE0 + Z_PER_GROUP * GPT;
    static constexpr int N_PIECES = Y_PIECE0 + 64;
    static constexpr int NI = (N_PIECES + 63) / 64;    // loads per stage
    static constexpr int STAGE_BYTES = NI * 1024;
    static constexpr int DEPTH = 4;                    // stages per wave (even: two register sets alternate)
    static constexpr int LDS_BYTES = sm::WG_WAVES * DEPTH * STAGE_BYTES;
    static_assert(LDS_BYTES >= smb::RED_BYTES, "the wave reduction re-uses the stages");
    static_assert(DEPTH * NI < 64, "vmcnt is a 6-bit counter");
    // mantissa bit at which code c of a lane's 8 codes is left by the shifted view it is taken from
    __host__ __device__ static constexpr int field_pos(int c) {
        return BITS == 4 ? 0 : (BITS == 2 ? 2 * (c % 3) : (c < 5 ? 3 * (c % 2) : (c == 6 ? 3 : 0)));
    }
    // XOR swizzle of a word row's eight 16-byte pieces.  Eight consecutive lanes read one piece
    // each of up to eight different rows at a time (lane 4u + b: 4-bit row 4b + u; 3-bit rows
    // 3b + {0,0,1,2}[u] and 3b + {1,1,2,2}[u]; 2-bit row 2b + u / 2, u in {0,1} or {2,3}); the
    // rows that meet must get different values.
    __device__ static __forceinline__ int swz(int row) {
        if (BITS == 4) return (row >> 2) | ((row & 1) << 2);
        if (BITS == 2) return row & 7;
        return row < 8 ? row : ((0x6310 >> (4 * (row - 8))) & 7);     // rows 8..11 -> 0, 1, 3, 6
    }
};

template <int BITS, bool F16, int GPT>
__global__ __launch_bounds__(sm::WG_THREADS, 2) void smallm_bwd_kernel(SmallBwdDev d) {
    using BG = BwdGeo<BITS, F16, GPT>;
    using NF = sm::Num<F16>;
    extern __shared__ __attribute__((aligned(16))) uint4 ys[];   // [wave][stage] private stages, later the reduction
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if ((int)blockIdx.x < d.n_proj) {
        // projection workgroups: partials of dYBt = dY B^T (see the forward kernel)
        if (F16) smallm_project_f16<false, sm::WG_WAVES>(d.dY, d.M, d.w.N, d.B, d.r, blockIdx.x, d.n_proj, d.Tpart, reinterpret_cast<float *>(ys));
        else smallm_project<false, sm::WG_WAVES>(d.dY, d.M, d.w.N, d.B, d.r, blockIdx.x, d.n_proj, d.Tpart, reinterpret_cast<float *>(ys));
        return;
    }
    const int bid = blockIdx.x - d.n_proj;
    const int i = lane & 15, j = lane >> 4, b = i & 3, u = i >> 2;
    const int N = d.w.N, K = d.w.K;
    const int kb = bid / d.nsplit, ns = bid % d.nsplit;
    const int kt = kb * smb::KT;
    const int n_steps = N / smb::NSTEP;
    const int S0 = (int)((long)n_steps * ns / d.nsplit), S1 = (int)((long)n_steps * (ns + 1) / d.nsplit);
    // this wave's steps: S0 + wave + 4 t, t = 0 .. nw - 1
    const int nw = S1 - S0 > wave ? (S1 - S0 - wave + sm::WG_WAVES - 1) / sm::WG_WAVES : 0;
    const int g = kt / d.w.group;        // first of the tile's GPT quantization groups

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
    // zero points of the group: one byte each, or (F16) one binary16 each
    const char *ztile = F16 ? reinterpret_cast<const char *>(d.zeros16 + (size_t)g * N) : reinterpret_cast<const char *>(d.w.zeros + (size_t)g * N);

    // The packed words, scales, zeros and the dY piece of a step (32 n) travel global -> LDS
    // without passing through registers: every lane moves one 16-byte piece per load, so a whole
    // stage is NI fully coalesced loads (128 contiguous bytes per word row, 64 per dY row).  Piece p
    // of word row `row` sits at LDS piece p ^ swz(row) of that row: the later 16-byte reads of 16
    // different rows then spread over the banks.  dY piece 16 c + m is row m (rows >= M repeat row
    // M - 1; their results are never stored), elements 8 c .. 8 c + 7 of the step.
    constexpr int NI = BG::NI, DEPTH = BG::DEPTH, STAGE_BYTES = BG::STAGE_BYTES;
    const char *gaddr[NI];                             // this lane's piece of load q, at step 0 of the matrix
    uint32_t gstr[NI];                                 // ... and its advance per step
#pragma unroll
    for (int q = 0; q < NI; ++q) {
        const int pc = q * 64 + lane;                  // lanes past N_PIECES sit out the last load
        if (pc < BG::W_PIECES) {
            const int row = pc >> 3, pp = (pc & 7) ^ BG::swz(row);
            gaddr[q] = reinterpret_cast<const char *>(wtile) + ((size_t)row * N + pp * 4) * 4;
            gstr[q] = smb::NSTEP * 4;
        } else if (pc < BG::Z_PIECE0) {
            const int sp = pc - BG::S_PIECE0;          // group sp / 4 of the tile, piece sp % 4 of its 64 bytes
            gaddr[q] = reinterpret_cast<const char *>(stile) + (size_t)(sp >> 2) * N * 2 + (sp & 3) * 16;
            gstr[q] = smb::NSTEP * 2;
        } else if (pc < BG::Y_PIECE0) {
            const int zp = pc - BG::Z_PIECE0;
            gaddr[q] = ztile + (size_t)(zp / BG::Z_PER_GROUP) * N * (F16 ? 2 : 1) + (zp % BG::Z_PER_GROUP) * 16;
            gstr[q] = smb::NSTEP * (F16 ? 2 : 1);
        } else {
            const int yp = pc < BG::N_PIECES ? pc - BG::Y_PIECE0 : 0;
            const int m = (yp & 15) < d.M ? (yp & 15) : d.M - 1;
            gaddr[q] = reinterpret_cast<const char *>(d.dY + (size_t)m * N + (yp >> 4) * 8);
            gstr[q] = smb::NSTEP * 2;
        }
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)ys;
    const uint32_t stage0 = (uint32_t)wave * (DEPTH * STAGE_BYTES);   // offset of the wave's stages
    auto issue = [&](int slot, int step) {             // step: any step of the workgroup's slice
#pragma unroll
        for (int q = 0; q < NI; ++q) {
            // loads made of packed words only are read once: non-temporal
            if ((q + 1) * 64 <= BG::W_PIECES)
                sm::ald_lds64<true>(gaddr[q] + (size_t)step * gstr[q], lds0 + stage0 + (uint32_t)slot * STAGE_BYTES + q * 1024);
            else if ((q + 1) * 64 <= BG::N_PIECES || q * 64 + lane < BG::N_PIECES)
                sm::ald_lds64<false>(gaddr[q] + (size_t)step * gstr[q], lds0 + stage0 + (uint32_t)slot * STAGE_BYTES + q * 1024);
        }
    };
    // step t of this wave, clamped into the slice (a clamped stage is loaded and never used)
    auto wave_step = [&](int t) { const int st = S0 + wave + sm::WG_WAVES * t; return st < S1 ? st : S1 - 1; };
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd) issue(dd, wave_step(dd));

    // per quantization group of the tile: the scaled activations differ, so each group has its own
    // products (a lane keeps the ones of the group its output columns lie in)
    f32x4 acc[GPT][8], accz[GPT], accs[GPT];
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[gi][c][v] = 0.f;
            accz[gi][v] = 0.f;
            accs[gi][v] = 0.f;
        }
    const uint32_t ones4[4] = {NF::ONES, NF::ONES, NF::ONES, NF::ONES};
    const bf16x8 ones = sm::as_bf16x8(ones4);
    // field masks at the positions field_pos() can return (multiples of BITS)
    constexpr uint32_t FM = BITS == 4 ? 0x000F000Fu : (BITS == 2 ? 0x00030003u : 0x00070007u);
    const uint32_t fmask[3] = {sm::opaque_sgpr(FM), sm::opaque_sgpr(FM << BITS), sm::opaque_sgpr(FM << (2 * BITS))};
    const uint32_t magic = sm::opaque_vgpr(NF::MAGIC);

    struct Stage {
        sm::u32x4 w[NROWS][2];   // 8 adjacent n of each word row
        sm::u32x4 sc[GPT];       // 8 binary16 scales per group
        sm::u32x2 z[GPT];        // 8 integer zero points (bfloat16 layer)
        sm::u32x4 z16[GPT];      // 8 binary16 zero points (F16)
        sm::u32x4 y;             // dY[i][8 n]
    };
    // marks a register set as complete (call after a wait for the LDS reads that fill it), so
    // that the compiler does not add a wait of its own that would also cover younger reads
    auto settled = [&](Stage &sd) {
        sm::tie(sd.w[0][0]);
        sm::tie(sd.w[0][1]);
        if (NROWS == 2) {
            sm::tie(sd.w[NROWS - 1][0]);
            sm::tie(sd.w[NROWS - 1][1]);
        }
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            sm::tie(sd.sc[gi]);
            if (F16) sm::tie(sd.z16[gi]); else sm::tie(sd.z[gi]);
        }
        sm::tie(sd.y);
    };
    // a landed stage, LDS -> registers
    auto fetch = [&](Stage &sd, int slot) {
        const unsigned char *sb = reinterpret_cast<const unsigned char *>(ys) + stage0 + slot * STAGE_BYTES;
        sd.w[0][0] = *reinterpret_cast<const sm::u32x4 *>(sb + row0 * 128 + (((2 * j) ^ BG::swz(row0)) << 4));
        sd.w[0][1] = *reinterpret_cast<const sm::u32x4 *>(sb + row0 * 128 + (((2 * j + 1) ^ BG::swz(row0)) << 4));
        if (NROWS == 2) {
            sd.w[NROWS - 1][0] = *reinterpret_cast<const sm::u32x4 *>(sb + row1 * 128 + (((2 * j) ^ BG::swz(row1)) << 4));
            sd.w[NROWS - 1][1] = *reinterpret_cast<const sm::u32x4 *>(sb + row1 * 128 + (((2 * j + 1) ^ BG::swz(row1)) << 4));
        }
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            sd.sc[gi] = *reinterpret_cast<const sm::u32x4 *>(sb + (BG::S_PIECE0 + 4 * gi) * 16 + 16 * j);
            if (F16) sd.z16[gi] = *reinterpret_cast<const sm::u32x4 *>(sb + (BG::Z_PIECE0 + 4 * gi) * 16 + 16 * j);
            else sd.z[gi] = *reinterpret_cast<const sm::u32x2 *>(sb + (BG::Z_PIECE0 + 2 * gi) * 16 + 8 * j);
        }
        sd.y = *reinterpret_cast<const sm::u32x4 *>(sb + (BG::Y_PIECE0 + 16 * j + i) * 16);
    };
    auto compute = [&](const Stage &sd) {
        // A operands: dY[i][8 n] * scale[group][8 n], rounded to the activations' 16-bit format
        const uint32_t yw[4] = {sd.y[0], sd.y[1], sd.y[2], sd.y[3]};
        bf16x8 a[GPT];
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            uint32_t areg[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const float y0 = sm::widen16<F16>(yw[p] & 0xFFFFu), y1 = sm::widen16<F16>(yw[p] >> 16);
                const float s0 = half_bits_to_float((uint16_t)(sd.sc[gi][p] & 0xFFFFu)), s1 = half_bits_to_float((uint16_t)(sd.sc[gi][p] >> 16));
                areg[p] = sm::pack16<F16>(y0 * s0, y1 * s1);
            }
            a[gi] = sm::as_bf16x8(areg);
        }
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
        // Code c of a pair register: shifted views put 3- and 2-bit fields at mantissa bit 0, 3
        // (3-bit) or 0, 2, 4 (2-bit); a field at bit s enters the product as 128 + 2^s q, and the
        // column's factor 2^s is divided out when the tile is finished.
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            uint32_t o[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                uint32_t x;
                if (BITS == 4) x = c < 4 ? plo[p] >> (4 * c) : phi[p] >> (4 * (c - 4));
                else if (BITS == 2) x = plo[p] >> (6 * (c / 3));
                else x = c < 5 ? plo[p] >> (6 * (c / 2)) : phi[p] >> (c < 7 ? 7 : 13);
                o[p] = sm::and_or(x, fmask[BG::field_pos(c) / BITS], magic);
            }
            const bf16x8 ob = sm::as_bf16x8(o);
#pragma unroll
            for (int gi = 0; gi < GPT; ++gi) acc[gi][c] = sm::mma<F16>(a[gi], ob, acc[gi][c]);
        }
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            if (F16) {
                // the added zero point: sum_n dY[m][n] z[group][n], with the unscaled dY and z as stored
                const uint32_t zo[4] = {sd.z16[gi][0], sd.z16[gi][1], sd.z16[gi][2], sd.z16[gi][3]};
                accz[gi] = sm::mma<F16>(sm::as_bf16x8(yw), sm::as_bf16x8(zo), accz[gi]);
            } else {
                // integer zero points as exact bfloat16: sum_n (dY scale)[m][n] zero[group][n]
                uint32_t zo[4];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const uint32_t zw = sd.z[gi][p >> 1] >> (16 * (p & 1));
                    zo[p] = pack_bf16x2((float)(zw & 0xFFu), (float)((zw >> 8) & 0xFFu));
                }
                accz[gi] = sm::mma<F16>(a[gi], sm::as_bf16x8(zo), accz[gi]);
            }
            accs[gi] = sm::mma<F16>(a[gi], ones, accs[gi]);
        }
    };

    // Two workgroups share a compute unit and the instruction arbiter favours the older wave, so
    // one would run ahead and leave the other to finish alone on a half-empty SIMD.  A wave's
    // priority falls with its progress (3 in the first quarter of its steps ... 0 in the last), which
    // lets the wave that lags behind issue first.
    const int q1 = nw / 4, q2 = nw / 2, q3 = nw - nw / 4;
    __builtin_amdgcn_s_setprio(3);
    // Step t: its stage is already in registers (read from LDS during step t - 1); refill the
    // slot for step t + DEPTH, read stage t + 1 into the other register set, then compute -- the
    // LDS reads of the next step run under the arithmetic of this one.
    Stage regs[2];
    sm::wait_vm<(DEPTH - 1) * NI>();                 // stage 0 has landed
    fetch(regs[0], 0);
    for (int t = 0; t < nw; t += DEPTH) {
#pragma unroll
        for (int dd = 0; dd < DEPTH; ++dd) {
            if (t + dd < nw) {
                if (t + dd == q3) __builtin_amdgcn_s_setprio(0);
                else if (t + dd == q2) __builtin_amdgcn_s_setprio(1);
                else if (t + dd == q1) __builtin_amdgcn_s_setprio(2);
                issue(dd, wave_step(t + dd + DEPTH));   // waits for the LDS reads of slot dd first
                settled(regs[dd & 1]);
                sm::wait_vm<(DEPTH - 1) * NI>();     // the next stage has landed; DEPTH - 1 younger ones in flight
                fetch(regs[(dd + 1) & 1], (dd + 1) % DEPTH);
                __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads ahead of the arithmetic
                compute(regs[dd & 1]);
            }
        }
    }
    __builtin_amdgcn_s_setprio(0);
    // loads past the end of the slice are still in flight towards this workgroup's LDS
    sm::wait_vm<0>();
    __syncthreads();                                 // every wave is done with its stages

    // the four waves' tiles meet in LDS: red[wave][c * 4 + v][lane]
    float *red = reinterpret_cast<float *>(ys);
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int v = 0; v < 4; ++v)
        {
            // the lane's output columns lie in 32-code block b of the tile: group b * GPT / 4
            float av = acc[0][c][v], sv = accs[0][v], zv = accz[0][v];
            if (GPT == 2 && b >= 2) { av = acc[GPT - 1][c][v]; sv = accs[GPT - 1][v]; zv = accz[GPT - 1][v]; }
            red[(wave * 32 + c * 4 + v) * 64 + lane] =
                (av - NF::OFFSET * sv) * (1.0f / (float)(1 << BG::field_pos(c))) + (F16 ? zv : -zv);
        }
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
        sm::store_stream(dst, y[0], y[1], y[2], y[3]);
        sm::store_stream(dst + 4, y[4], y[5], y[6], y[7]);
    }
}

// Sum of the N slices' partial tiles, adapter term, 16-bit store.  One single-wave workgroup per 32
// columns (a few dozen 256-thread workgroups left most of the chip idle while each waited for its
// chain of loads): lane l owns row l / 4, columns 8 (l % 4) .. + 7.
template <bool F16>
__global__ __launch_bounds__(64) void smallm_bwd_finish_kernel(SmallBwdDev d) {
    __shared__ float Ts[16 * 64];
    const int tid = threadIdx.x, K = d.w.K;
    const int m = tid >> 2, k0 = blockIdx.x * FIN_COLS + 8 * (tid & 3);
    float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // the first columns of the eight rows of A are fetched ahead of everything that waits
    float4 a0[8][2];
#pragma unroll
    for (int c = 0; c < 8; ++c) { a0[c][0] = make_float4(0.f, 0.f, 0.f, 0.f); a0[c][1] = a0[c][0]; }
    if (m < d.M && d.r > 0) smallm_load_a8(d, k0, 0, a0);
    // sixteen slices' loads (two 16-byte loads each) in flight at a time; the first sixteen are issued
    // before the projection partials are summed and consumed after
    constexpr int SB = FIN_SLICES;
    float4 v0[SB], v1[SB];
    // (slices past the last one re-read the last and are not added: one predicate for all the loads
    // of a batch instead of one per slice keeps the scalar registers within bounds)
    const float *mine = d.acc + (size_t)(m < d.M ? m : 0) * K + k0;
    const uint32_t slice_stride = sm::opaque_vgpr((uint32_t)16 * (uint32_t)K);      // floats, in a vector register (see the forward kernel)
    // four sets of four slices, as in the forward finish kernel
    auto load_slices = [&](int q0) {
#pragma unroll
        for (int set = 0; set < SB / 4; ++set) {
            if (q0 + 4 * set < d.nsplit) {
                const float *src = mine + (size_t)(q0 + 4 * set) * slice_stride;
#pragma unroll
                for (int u = 4 * set; u < 4 * set + 4; ++u) {
                    v0[u] = *reinterpret_cast<const float4 *>(src);
                    v1[u] = *reinterpret_cast<const float4 *>(src + 4);
                    src += q0 + u + 1 < d.nsplit ? slice_stride : 0u;
                }
            }
        }
    };
    auto add_slices = [&](int q0) {
        const int left = (int)sm::opaque_vgpr((uint32_t)(d.nsplit - q0));
#pragma unroll
        for (int set = 0; set < SB / 4; ++set) {
            if (q0 + 4 * set < d.nsplit) {
#pragma unroll
                for (int u = 4 * set; u < 4 * set + 4; ++u) {
                    const float w = u < left ? 1.f : 0.f;
                    y[0] = __builtin_fmaf(w, v0[u].x, y[0]); y[1] = __builtin_fmaf(w, v0[u].y, y[1]);
                    y[2] = __builtin_fmaf(w, v0[u].z, y[2]); y[3] = __builtin_fmaf(w, v0[u].w, y[3]);
                    y[4] = __builtin_fmaf(w, v1[u].x, y[4]); y[5] = __builtin_fmaf(w, v1[u].y, y[5]);
                    y[6] = __builtin_fmaf(w, v1[u].z, y[6]); y[7] = __builtin_fmaf(w, v1[u].w, y[7]);
                }
            }
        }
    };
    load_slices(0);
    if (d.r <= 8) smallm_sum_parts<2>(d.Tpart, d.n_proj, d.r, Ts);     // 16 r elements over 64 lanes: no more loads than needed
    else smallm_sum_parts<4>(d.Tpart, d.n_proj, d.r, Ts);
    add_slices(0);
    for (int q0 = SB; q0 < d.nsplit; q0 += SB) { load_slices(q0); add_slices(q0); }
    if (blockIdx.x == 0 && d.T_out != nullptr)
        for (int t = tid; t < d.M * d.r; t += 64) d.T_out[t] = Ts[t];
    if (m < d.M) smallm_bwd_store8<F16>(d, Ts, m, k0, y, a0);
}

namespace {
// K slices for a product with contraction length Kc (groups of `group`) and Nout outputs:
// slices of whole groups that fit the LDS, at most MAX_KSPLIT, about one (8-wave) workgroup
// per compute unit.  The stream is bound by instruction issue, so the time is set by the
// fullest unit: workgroups per unit x groups per slice; a grid a little over 256 workgroups
// (43 column blocks x 6 = 258) would leave a few units with two.  Returns 0 when no split exists.
int pick_ksplit(int Kc, int Nout, int group) {
    if (group > sm::MAX_RANGE) return 0;
    const int n_groups = Kc / group;
    const int gmax = sm::MAX_RANGE / group;                    // groups per slice that fit the LDS
    const int need = (n_groups + gmax - 1) / gmax;
    const int col_blocks = (Nout + sm::BCOLS - 1) / sm::BCOLS;
    const int cap = n_groups < sm::MAX_KSPLIT ? n_groups : sm::MAX_KSPLIT;
    if (need > cap) return 0;
    int lo = (192 + col_blocks - 1) / col_blocks;
    if (lo < need) lo = need;
    if (lo > cap) lo = cap;
    int best = 0;
    double best_cost = 1e30;
    for (int ks = lo; ks <= cap; ++ks) {
        const int gps = (n_groups + ks - 1) / ks;              // groups of the longest slice
        if ((long)gps * group > sm::MAX_RANGE) continue;
        const int wgs = col_blocks * ks, per_cu = (wgs + 255) / 256;
        const double cost = (double)per_cu * gps + (wgs > 256 ? 3.0 : 0.0) + 0.1 * ks;
        if (cost < best_cost) { best_cost = cost; best = ks; }
    }
    return best;
}
// upper bound of pick_ksplit over all group sizes (for the workspace query)
int ksplit_bound(int, int) { return sm::MAX_KSPLIT; }
// N slices of the backward product (contraction length N, K outputs in tiles of 128).  Every
// workgroup of the grid is resident at once (up to 3 per compute unit); the time is set by the
// fullest unit, rounds x slice length, so take the split that makes that product smallest, and
// among equals the smallest one (fewer partial tiles).  A wave keeps at least two steps.
int pick_nsplit(int N, int K) {
    const int n_steps = N / smb::NSTEP;
    const int k_blocks = K / smb::KT;
    if (n_steps < 1 || k_blocks < 1) return 0;
    // largest admissible split: two steps per wave, at most 768 workgroups
    int cap = 1;
    while (cap < sm::MAX_KSPLIT && n_steps / (cap + 1) >= 2 * sm::WG_WAVES && (long)k_blocks * (cap + 1) <= 768) ++cap;
    // two workgroups per compute unit where the shape allows (a second wave per SIMD hides the
    // first one's waits)
    int lo = (512 + k_blocks - 1) / k_blocks;
    if (lo > cap) lo = cap;
    int best = lo;
    double best_cost = 1e30;
    for (int ns = lo; ns <= cap; ++ns) {
        const int per_cu = (k_blocks * ns + 255) / 256;
        // steps the fullest unit runs, a fixed cost per workgroup, the partial tiles
        const double cost = (double)per_cu * ((n_steps + ns - 1) / ns) + 8.0 * per_cu + 0.5 * ns;
        if (cost < best_cost) { best_cost = cost; best = ns; }
    }
    return best;
}
}  // namespace

// More than one pass (M > SMALLM_ROWS) only over a weight of at least 4 MB of codes: below that a
// pass is all launch latency and the tile kernels are as fast.
static bool smallm_rows_ok(const LayerView &w, int M) {
    if (M <= SMALLM_ROWS) return true;
    return M <= SMALLM_MAX_M && (size_t)w.K * w.N * w.bits / 8 >= ((size_t)4 << 20);
}

bool smallm_bwd_supported(const LayerView &w, int M) {
    if (!smallm_rows_ok(w, M)) return false;
    // a 128-column tile lies inside one quantization group, or covers exactly two
    const bool group_ok = w.group % smb::KT == 0 || w.group == smb::KT / 2;
    return group_ok && w.K % smb::KT == 0 && w.N % sm::PREP_K == 0 && pick_nsplit(w.N, w.K) > 0;
}

bool smallm_fwd_supported(const LayerView &w, int M) {
    if (!smallm_rows_ok(w, M)) return false;
    const int kstep = w.bits == 4 ? 32 : (w.bits == 2 ? 64 : 128);
    return w.group % kstep == 0 && w.K % sm::PREP_K == 0 && pick_ksplit(w.K, w.N, w.group) > 0;
}

namespace {
struct SmallWs {
    size_t upart, yacc, total;
};
// workgroups that do the rank-r projection beside the streaming ones: one per 512 contraction
// elements (four steps of 32 per wave), at most 16 -- or, for the binary16 layer, whose projection
// runs on the vector ALUs with one 8-element chunk per thread and pass, at most 32
constexpr int MAX_PROJ_BLOCKS = 32;
int n_proj_blocks(int C, int r, bool f16) {
    if (r <= 0) return 0;
    const int cap = f16 ? MAX_PROJ_BLOCKS : 16;
    int n = C / 512;
    return n < 1 ? 1 : (n > cap ? cap : n);
}
SmallWs small_ws(int K, int N, int r) {
    const size_t kmax = (size_t)(K > N ? K : N);
    auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
    SmallWs l;
    size_t off = 0;
    (void)kmax;
    l.upart = off;   off += al((size_t)MAX_PROJ_BLOCKS * 16 * (size_t)(r > 0 ? r : 1) * 4);
    const size_t yf = (size_t)ksplit_bound(K, N) * 16 * N, yb = (size_t)sm::MAX_KSPLIT * 16 * K;
    l.yacc = off;    off += al((yf > yb ? yf : yb) * 4);
    l.total = off;
    return l;
}
}  // namespace

size_t smallm_ws_bytes(int K, int N, int r) { return small_ws(K, N, r).total; }

size_t smallm_fwd_ws_bytes(const LayerView &w, int r) {
    const int ksplit = pick_ksplit(w.K, w.N, w.group);
    if (ksplit < 1) return 0;
    // the projection partials, then ksplit partial tiles [16][N]
    return small_ws(w.K, w.N, r).yacc + (((size_t)ksplit * 16 * w.N * 4 + 255) & ~(size_t)255);
}

template <int BITS, bool SPG1, bool F16>
static hipError_t launch_fwd_bits(const SmallFwdDev &d, int col_blocks, size_t lds_bytes, hipStream_t stream) {
    auto kern = smallm_fwd_kernel<BITS, SPG1, F16>;
    static bool configured[64] = {};
    // the largest slice plus its per-group sums (groups of at least 32 codes)
    const hipError_t e = ensure_lds_limit(reinterpret_cast<const void *>(kern), (size_t)sm::MAX_RANGE * 32 + (sm::MAX_RANGE / 32) * 128, configured);
    if (e != hipSuccess) return e;
    launch_kernel(F16 ? "f16_stream_fwd" : "stream_fwd", kern, col_blocks * d.ksplit + d.n_proj, sm::FWD_THREADS, lds_bytes, stream, d);
    return hipGetLastError();
}
template <bool F16>
static hipError_t launch_fwd_any(const SmallFwdDev &d, int bits, bool spg1, int col_blocks, size_t lds_bytes, hipStream_t stream) {
    switch (bits) {
        case 2: return spg1 ? launch_fwd_bits<2, true, F16>(d, col_blocks, lds_bytes, stream) : launch_fwd_bits<2, false, F16>(d, col_blocks, lds_bytes, stream);
        case 3: return spg1 ? launch_fwd_bits<3, true, F16>(d, col_blocks, lds_bytes, stream) : launch_fwd_bits<3, false, F16>(d, col_blocks, lds_bytes, stream);
        default: return spg1 ? launch_fwd_bits<4, true, F16>(d, col_blocks, lds_bytes, stream) : launch_fwd_bits<4, false, F16>(d, col_blocks, lds_bytes, stream);
    }
}

// The rows beyond the first SMALLM_ROWS of a call: the same arguments, advanced by that many rows
// of the input (row length C), the output (row length Cout) and the projection hand-off.
static SmallArgs rows_after_first_pass(const SmallArgs &a, int C, int Cout) {
    SmallArgs b = a;
    b.act = a.act + (size_t)SMALLM_ROWS * C;
    b.out = a.out + (size_t)SMALLM_ROWS * Cout;
    if (a.P_out) b.P_out = a.P_out + (size_t)SMALLM_ROWS * a.r;
    b.M = a.M - SMALLM_ROWS;
    return b;
}

hipError_t launch_smallm_fwd(const SmallArgs &a, hipStream_t stream) {
    if (a.M > SMALLM_ROWS) {
        SmallArgs first = a;
        first.M = SMALLM_ROWS;
        const hipError_t e1 = launch_smallm_fwd(first, stream);
        if (e1 != hipSuccess) return e1;
        return launch_smallm_fwd(rows_after_first_pass(a, a.w.K, a.w.N), stream);
    }
    const int K = a.w.K, N = a.w.N;
    const SmallWs l = small_ws(K, N, a.r);
    char *ws = static_cast<char *>(a.ws);
    float *Upart = reinterpret_cast<float *>(ws + l.upart);
    float *Yacc = reinterpret_cast<float *>(ws + l.yacc);
    const int col_blocks = (N + sm::BCOLS - 1) / sm::BCOLS;
    const int ksplit = pick_ksplit(K, N, a.w.group);
    if (ksplit < 1) return hipErrorInvalidValue;     // callers check smallm_fwd_supported first

    hipError_t e;
    SmallFwdDev d;
    d.w = a.w;
    d.X = a.act;
    d.A = a.A;
    d.Upart = Upart;
    d.B = a.B;
    d.M = a.M;
    d.r = a.r;
    d.n_proj = n_proj_blocks(K, a.r, a.f16);
    d.ksplit = ksplit;
    d.lora_scale = a.lora_scale;
    d.Y = a.out;
    d.XA = a.P_out;
    d.Yacc = Yacc;
    d.zeros16 = a.zeros16;
    d.bias16 = a.bias16;
    // LDS for the largest slice: ceil(groups / ksplit) groups of 32 bytes per contraction element
    const int n_groups = K / a.w.group;
    // ... plus the per-group sums behind the slice: 2 x 16 floats per group
    const size_t groups_per_slice = (size_t)((n_groups + ksplit - 1) / ksplit);
    size_t lds_bytes = groups_per_slice * a.w.group * 32 + groups_per_slice * 128;
    if (lds_bytes < 32 * 1024) lds_bytes = 32 * 1024;      // the projection workgroups' wave reduction
    const int kstep = a.w.bits == 4 ? 32 : (a.w.bits == 2 ? 64 : 128);
    const bool spg1 = a.w.group == kstep;             // one step per quantization group
    e = a.f16 ? launch_fwd_any<true>(d, a.w.bits, spg1, col_blocks, lds_bytes, stream)
              : launch_fwd_any<false>(d, a.w.bits, spg1, col_blocks, lds_bytes, stream);
    if (e != hipSuccess) return e;
    if (a.f16) launch_kernel("f16_stream_fwd_finish", smallm_fwd_finish_kernel<true>, (N + FIN_COLS - 1) / FIN_COLS, 64, 0, stream, d);
    else launch_kernel("stream_fwd_finish", smallm_fwd_finish_kernel<false>, (N + FIN_COLS - 1) / FIN_COLS, 64, 0, stream, d);
    return hipGetLastError();
}

template <int BITS, bool F16, int GPT>
static hipError_t launch_bwd_bits(const SmallBwdDev &d, int k_blocks, hipStream_t stream) {
    auto kern = smallm_bwd_kernel<BITS, F16, GPT>;
    static bool configured[64] = {};
    constexpr size_t LDS = (size_t)BwdGeo<BITS, F16, GPT>::LDS_BYTES;
    const hipError_t e = ensure_lds_limit(reinterpret_cast<const void *>(kern), LDS, configured);
    if (e != hipSuccess) return e;
    launch_kernel(F16 ? "f16_stream_bwd" : "stream_bwd", kern, k_blocks * d.nsplit + d.n_proj, sm::WG_THREADS, LDS, stream, d);
    return hipGetLastError();
}
template <bool F16>
static hipError_t launch_bwd_any(const SmallBwdDev &d, int bits, int k_blocks, hipStream_t stream) {
    const bool two = d.w.group == smb::KT / 2;      // two quantization groups per 128-column tile
    switch (bits) {
        case 2: return two ? launch_bwd_bits<2, F16, 2>(d, k_blocks, stream) : launch_bwd_bits<2, F16, 1>(d, k_blocks, stream);
        case 3: return two ? launch_bwd_bits<3, F16, 2>(d, k_blocks, stream) : launch_bwd_bits<3, F16, 1>(d, k_blocks, stream);
        default: return two ? launch_bwd_bits<4, F16, 2>(d, k_blocks, stream) : launch_bwd_bits<4, F16, 1>(d, k_blocks, stream);
    }
}

hipError_t launch_smallm_bwd(const SmallArgs &a, hipStream_t stream) {
    if (a.M > SMALLM_ROWS) {
        SmallArgs first = a;
        first.M = SMALLM_ROWS;
        const hipError_t e1 = launch_smallm_bwd(first, stream);
        if (e1 != hipSuccess) return e1;
        return launch_smallm_bwd(rows_after_first_pass(a, a.w.N, a.w.K), stream);
    }
    const int K = a.w.K, N = a.w.N;
    const SmallWs l = small_ws(K, N, a.r);
    char *ws = static_cast<char *>(a.ws);
    float *Tpart = reinterpret_cast<float *>(ws + l.upart);
    const int k_blocks = K / smb::KT;
    const int nsplit = pick_nsplit(N, K);
    if (nsplit < 1) return hipErrorInvalidValue;     // callers check smallm_bwd_supported first

    hipError_t e;
    SmallBwdDev d;
    d.w = a.w;
    d.dY = a.act;
    d.B = a.B;
    d.Tpart = Tpart;
    d.A = a.A;
    d.M = a.M;
    d.r = a.r;
    d.n_proj = n_proj_blocks(N, a.r, a.f16);
    d.nsplit = nsplit;
    d.lora_scale = a.lora_scale;
    d.dX = a.out;
    d.T_out = a.P_out;
    d.acc = reinterpret_cast<float *>(ws + l.yacc);
    d.zeros16 = a.zeros16;
    e = a.f16 ? launch_bwd_any<true>(d, a.w.bits, k_blocks, stream) : launch_bwd_any<false>(d, a.w.bits, k_blocks, stream);
    if (e != hipSuccess) return e;
    if (a.f16) launch_kernel("f16_stream_bwd_finish", smallm_bwd_finish_kernel<true>, K / FIN_COLS, 64, 0, stream, d);
    else launch_kernel("stream_bwd_finish", smallm_bwd_finish_kernel<false>, K / FIN_COLS, 64, 0, stream, d);
    return hipGetLastError();
}

}  // namespace mlr
