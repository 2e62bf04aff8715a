// The rank-r adapter side of the layer (Section 3.1 eq. (3) and Section 3.1.1 of the
// ModuLoRA paper): the skinny projections  XA = X A  and  dYBt = dY B^T, the adapter
// gradients  dA = s X^T dYBt  and  dB = s XA^T dY, and the preparation of the
// "extended contraction" operands with which the tile GEMM adds the adapter term
// s (X A) B inside its MFMA loop.
//
// All of these are bound by one streaming pass over X or dY.  The projections run on the
// matrix cores (the fp32 factor split into three bfloat16 terms); the gradients are plain
// fp32 FMA with coalesced 4-byte loads per lane.
#include "device_common.h"
#include "launch.h"

namespace mlr {

// value of extended-operand element e (0 <= e < RE) given the fp32 source values:
// segments [0,r) [r,2r) [2r,3r) hold (hi,hi,lo) for the activation side and
// (hi,lo,hi) for the weight side, so that the dot product over the three segments
// is  hi*hi + hi*lo + lo*hi  ~=  (hi+lo)*(hi+lo)  to about 2^-16 relative.
__device__ __forceinline__ uint16_t split_part(float v, bool want_lo) {
    const uint16_t hi = float_to_bf16_bits(v);
    if (!want_lo) return hi;
    return float_to_bf16_bits(v - bf16_bits_to_float(hi));
}

// ---------------------------------------------------------------------------
// Projection: P[m][j] = sum_c act[m][c] F(c, j) on the matrix cores.  A workgroup owns 16 rows;
// its waves split the contraction and meet in LDS.  act is bfloat16 already; the fp32 factor is
// split on the fly into three bfloat16 terms (hi + mid + lo carry all 24 significand bits), so
// three 16x16x32 MFMAs per step give the fp32-exact products, accumulated in fp32.
// Lane l = 16 cs + i: activation row i / factor column i, contraction elements 8 cs .. 8 cs + 7
// of the step.  Extra workgroups (blockIdx.x >= row blocks) write the weight-side extension.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bf16x8 regs_to_bf16x8(const uint32_t r[4]) {
    bf16x8 v;
    __builtin_memcpy(&v, r, 16);
    return v;
}

// Eight consecutive elements (one 16-byte store) of the weight-side extension w_ext [Cw][RE]:
// row c holds the segments (hi, lo, hi) of the r factor values of that row and zero padding.
// Unit u = c * (RE / 8) + chunk, consecutive threads take consecutive units: the stores are
// contiguous, and the loads of a wave touch a few dozen adjacent rows c (from B [r][Cw]: runs of
// adjacent floats in up to eight rows j; from A [Cw][r]: adjacent floats of a row).
__device__ __forceinline__ void write_w_ext_unit(const DownArgs &a, size_t u) {
    const int r = a.r, per_row = a.RE >> 3;
    const int c = (int)(u / per_row), e0 = (int)(u % per_row) * 8;
    float src[8];
    int seg[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int e = e0 + q;
        seg[q] = e / r;
        const int j = e - seg[q] * r;
        src[q] = seg[q] < 3 ? (a.w_from_A ? a.Wsrc[(size_t)c * r + j] : a.Wsrc[(size_t)j * a.Cw + c]) : 0.f;
    }
    uint32_t o[4];
#pragma unroll
    for (int q = 0; q < 8; q += 2) {
        const uint32_t lo16 = seg[q] < 3 ? split_part(src[q], seg[q] == 1) : 0u;
        const uint32_t hi16 = seg[q + 1] < 3 ? split_part(src[q + 1], seg[q + 1] == 1) : 0u;
        o[q >> 1] = lo16 | (hi16 << 16);
    }
    *reinterpret_cast<uint4 *>(a.w_ext + u * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

// ROWT: 16-row tiles per workgroup (they share every factor operand); UNR: steps whose loads
// are issued together before any of them is used.
// ACT_F16: the activations are binary16; each operand is split exactly into two bfloat16 ones.
template <int RG, int ROWT, bool F_IS_A, bool ACT_F16>
__global__ __launch_bounds__(1024) void lora_down_kernel(DownArgs a, int row_blocks, int split) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];   // [waves][ROWT][RG][256] partial tiles, then Ps
    constexpr int UNR = ROWT > 1 ? 2 : (RG == 1 ? 4 : (RG == 2 ? 2 : 1));
    constexpr int ROWS = 16 * ROWT;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int r = a.r;

    if ((int)blockIdx.x >= row_blocks) {
        if (blockIdx.y != 0) return;
        // weight-side extension, one 16-byte unit per thread
        const size_t u = (size_t)(blockIdx.x - row_blocks) * nthreads + tid;
        if (u < (size_t)a.Cw * (a.RE >> 3)) write_w_ext_unit(a, u);
        return;
    }

    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthreads >> 6;
    const int i = lane & 15, cs = lane >> 4;
    const int m0 = blockIdx.x * ROWS;
    const uint16_t *arow[ROWT];
#pragma unroll
    for (int t = 0; t < ROWT; ++t) {
        int row = m0 + 16 * t + i;
        if (row > a.M - 1) row = a.M - 1;
        arow[t] = a.act + (size_t)row * a.C;
    }
    // the contraction is cut over (blockIdx.y, wave)
    const int steps = (a.C + 31) / 32;
    const long part = (long)blockIdx.y * nwaves + wave, parts = (long)split * nwaves;
    const int s_begin = (int)(steps * part / parts), s_end = (int)(steps * (part + 1) / parts);

    f32x4 acc[ROWT][RG];
#pragma unroll
    for (int t = 0; t < ROWT; ++t)
#pragma unroll
        for (int g = 0; g < RG; ++g) acc[t][g] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int st = s_begin; st < s_end; st += UNR) {
        uint4 av[UNR][ROWT];
        float f[UNR][RG][8];
        // all loads of UNR steps first
#pragma unroll
        for (int q = 0; q < UNR; ++q) {
            const int c = (st + q) * 32 + cs * 8;       // C is a multiple of 8: the chunk is all in or all out
            const bool c_ok = st + q < s_end && c < a.C;
#pragma unroll
            for (int t = 0; t < ROWT; ++t) {
                av[q][t] = make_uint4(0, 0, 0, 0);
                if (c_ok) av[q][t] = *reinterpret_cast<const uint4 *>(arow[t] + c);
            }
#pragma unroll
            for (int g = 0; g < RG; ++g) {
                const int j = g * 16 + i;
#pragma unroll
                for (int e = 0; e < 8; ++e) f[q][g][e] = 0.f;
                if (c_ok && j < r) {
                    if (F_IS_A) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) f[q][g][e] = a.Fm[(size_t)(c + e) * r + j];
                    } else {
                        const float4 q0 = *reinterpret_cast<const float4 *>(a.Fm + (size_t)j * a.C + c);
                        const float4 q1 = *reinterpret_cast<const float4 *>(a.Fm + (size_t)j * a.C + c + 4);
                        f[q][g][0] = q0.x; f[q][g][1] = q0.y; f[q][g][2] = q0.z; f[q][g][3] = q0.w;
                        f[q][g][4] = q1.x; f[q][g][5] = q1.y; f[q][g][6] = q1.z; f[q][g][7] = q1.w;
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < UNR; ++q)
#pragma unroll
            for (int g = 0; g < RG; ++g) {
                uint32_t hi[4], mid[4], lo[4];
                split3(f[q][g], hi, mid, lo);
                const bf16x8 bh = regs_to_bf16x8(hi), bm = regs_to_bf16x8(mid), bl = regs_to_bf16x8(lo);
#pragma unroll
                for (int t = 0; t < ROWT; ++t) {
                    const uint32_t ar[4] = {av[q][t].x, av[q][t].y, av[q][t].z, av[q][t].w};
                    if (ACT_F16) {
                        uint32_t ah[4], al[4];
                        split_f16x8(ar, ah, al);
                        const bf16x8 aop = regs_to_bf16x8(ah), aop2 = regs_to_bf16x8(al);
                        acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bh, acc[t][g], 0, 0, 0);
                        acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bm, acc[t][g], 0, 0, 0);
                        acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bl, acc[t][g], 0, 0, 0);
                        acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop2, bh, acc[t][g], 0, 0, 0);
                        acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop2, bm, acc[t][g], 0, 0, 0);
                        acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop2, bl, acc[t][g], 0, 0, 0);
                    } else {
                        const bf16x8 aop = regs_to_bf16x8(ar);
                        acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bh, acc[t][g], 0, 0, 0);
                        acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bm, acc[t][g], 0, 0, 0);
                        acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bl, acc[t][g], 0, 0, 0);
                    }
                }
            }
    }

    // D register v of lane (i, cs): row 4 cs + v, column i.  Partial tiles -> LDS -> sum over the waves.
    constexpr int TILES = ROWT * RG;
#pragma unroll
    for (int t = 0; t < ROWT; ++t)
#pragma unroll
        for (int g = 0; g < RG; ++g)
#pragma unroll
            for (int v = 0; v < 4; ++v) lds_f[((wave * TILES + t * RG + g) * 4 + v) * 64 + lane] = acc[t][g][v];
    __syncthreads();
    float *Ps = lds_f + nwaves * TILES * 256;               // [ROWS][16 * RG]
    for (int x = tid; x < TILES * 256; x += nthreads) {
        const int tile = x >> 8, v = (x >> 6) & 3, l = x & 63;
        float sum = 0.f;
        for (int w = 0; w < nwaves; ++w) sum += lds_f[((w * TILES + tile) * 4 + v) * 64 + l];
        const int prow = 16 * (tile / RG) + 4 * (l >> 4) + v, j = (tile % RG) * 16 + (l & 15);
        Ps[prow * (16 * RG) + j] = sum;
        if (split > 1)   // a slice of the contraction: leave the tile for lora_down_finish_kernel
            a.partials[((size_t)blockIdx.y * row_blocks + blockIdx.x) * (TILES * 256) + prow * (16 * RG) + j] = sum;
        else if (m0 + prow < a.M && j < r)
            a.P[(size_t)(m0 + prow) * r + j] = sum;
    }
    if (a.act_ext == nullptr || split > 1) return;
    __syncthreads();
    for (int x = tid; x < ROWS * a.RE; x += nthreads) {
        const int pr = x / a.RE, e = x % a.RE;
        if (m0 + pr >= a.M) continue;
        uint16_t v = 0;
        if (e < 3 * r) {
            const int seg = e / r, j = e % r;
            v = split_part(a.lora_scale * Ps[pr * (16 * RG) + j], seg == 2);
        }
        a.act_ext[(size_t)(m0 + pr) * a.RE + e] = v;
    }
}

// Second stage when the contraction was split over workgroups: add the slices' tiles of 16 rows
// in slice order, write P and the activation-side extension.  One workgroup per 16 rows; the
// partials of a first-stage workgroup hold its ROWT tiles one after the other.
template <int RG>
__global__ __launch_bounds__(256) void lora_down_finish_kernel(DownArgs a, int row_blocks, int split, int rowt) {
    __shared__ float Ps[16 * 16 * RG];
    const int tid = threadIdx.x, r = a.r, m0 = blockIdx.x * 16;
    const int rb = blockIdx.x / rowt, tile = blockIdx.x % rowt;
    const size_t wg_floats = (size_t)rowt * 256 * RG;
    for (int x = tid; x < 256 * RG; x += 256) {
        const float *src = a.partials + (size_t)rb * wg_floats + (size_t)tile * (256 * RG) + x;
        float sum = 0.f;
        int y = 0;
        for (; y + 4 <= split; y += 4) {      // four slices' loads in flight
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = src[(size_t)(y + u) * row_blocks * wg_floats];
            sum += v[0]; sum += v[1]; sum += v[2]; sum += v[3];
        }
        for (; y < split; ++y) sum += src[(size_t)y * row_blocks * wg_floats];
        Ps[x] = sum;
        const int prow = x / (16 * RG), j = x % (16 * RG);
        if (m0 + prow < a.M && j < r) a.P[(size_t)(m0 + prow) * r + j] = sum;
    }
    if (a.act_ext == nullptr) return;
    __syncthreads();
    for (int x = tid; x < 16 * a.RE; x += 256) {
        const int pr = x / a.RE, e = x % a.RE;
        if (m0 + pr >= a.M) continue;
        uint16_t v = 0;
        if (e < 3 * r) {
            const int seg = e / r, j = e % r;
            v = split_part(a.lora_scale * Ps[pr * (16 * RG) + j], seg == 2);
        }
        a.act_ext[(size_t)(m0 + pr) * a.RE + e] = v;
    }
}

template <int RG, int ROWT>
static hipError_t launch_down_rg(const DownArgs &a, const DownPlan &plan, hipStream_t stream) {
    constexpr int ROWS = 16 * ROWT;
    const int row_blocks = (a.M + ROWS - 1) / ROWS;
    const int nwaves = plan.nwaves, nthreads = nwaves * 64, split = plan.split;
    const int w_blocks = a.w_ext ? (int)(((size_t)a.Cw * (a.RE / 8) + nthreads - 1) / nthreads) : 0;
    const size_t lds = (size_t)(nwaves * RG * ROWT * 256 + ROWS * 16 * RG) * sizeof(float);
    const dim3 grid(row_blocks + w_blocks, split);
    if (a.act_f16) {
        if (a.f_is_A)
            launch_kernel("lora_down", lora_down_kernel<RG, ROWT, true, true>, grid, nthreads, lds, stream, a, row_blocks, split);
        else
            launch_kernel("lora_down", lora_down_kernel<RG, ROWT, false, true>, grid, nthreads, lds, stream, a, row_blocks, split);
    } else if (a.f_is_A) {
        launch_kernel("lora_down", lora_down_kernel<RG, ROWT, true, false>, grid, nthreads, lds, stream, a, row_blocks, split);
    } else {
        launch_kernel("lora_down", lora_down_kernel<RG, ROWT, false, false>, grid, nthreads, lds, stream, a, row_blocks, split);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split <= 1) return e;
    launch_kernel("lora_down_finish", lora_down_finish_kernel<RG>, (a.M + 15) / 16, 256, 0, stream, a, row_blocks, split, ROWT);
    return hipGetLastError();
}

hipError_t launch_lora_down(const DownArgs &a, hipStream_t stream) {
    const DownPlan plan = lora_down_plan(a.M, a.C, a.r);
    if (plan.rowt == 4) {
        if (a.r <= 16) return launch_down_rg<1, 4>(a, plan, stream);
        return launch_down_rg<2, 4>(a, plan, stream);
    }
    if (a.r <= 16) return launch_down_rg<1, 1>(a, plan, stream);
    if (a.r <= 32) return launch_down_rg<2, 1>(a, plan, stream);
    if (a.r <= 48) return launch_down_rg<3, 1>(a, plan, stream);
    return launch_down_rg<4, 1>(a, plan, stream);
}

// ---------------------------------------------------------------------------
// Adapter gradients (Section 3.1.1), both in one launch plus one reduction launch:
//   dA[k][j] = s * sum_m X[m][k]  dYBt[m][j]      dB[j][n] = s * sum_m XA[m][j] dY[m][n]
// Stage 1: a workgroup owns 128 or 256 columns of X (or dY) and a chunk of rows; each lane owns 2
// or 4 adjacent columns (one 4- or 8-byte load per row), the 4 waves take rows round-robin, P[m][:] is
// wave-uniform.  The 4 waves' sums meet in LDS and go out as one partial per row chunk, laid
// out like the outputs ([chunk][dA | dB]).  Stage 2 adds the chunks, applies s and the
// accumulate flag.  No atomics (device-scope fp32 atomics bypass the per-XCD L2 and are slow)
// and no zero-fill of the outputs.
// ---------------------------------------------------------------------------
// Up to this many rows go in one chunk (measured per call: 5.9 - 6.5 against 7.9 - 8.1 us at 33 - 64
// rows; at 128 rows the single launch is no quicker than the pair).
constexpr int GRAD_ONE_CHUNK_ROWS = 64;
GradGeom grad_geom(int M, int K, int N, int r) {
    GradGeom g;
    g.cpl = r <= 16 ? 4 : 2;                        // columns per lane (8- or 4-byte loads)
    const int wcols = 64 * g.cpl;                   // columns per workgroup
    g.cols_a = (K + wcols - 1) / wcols;
    g.cols_b = (N + wcols - 1) / wcols;
    const int col_blocks = g.cols_a + g.cols_b;
    // enough row chunks to give the chip ~1024 workgroups, at least 32 rows each
    int chunks = (1024 + col_blocks - 1) / col_blocks;
    const int max_chunks = (M + 31) / 32;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    if (M <= GRAD_ONE_CHUNK_ROWS) chunks = 1;       // few rows: one launch, no reduction launch behind it
    int rows = (M + chunks - 1) / chunks;
    rows = (rows + 3) / 4 * 4;
    g.rows_per_block = rows;
    g.chunks = (M + rows - 1) / rows;
    g.passes = r > 32 ? 2 : 1;
    g.partial_floats = (size_t)g.chunks * (size_t)(K + N) * (size_t)(r > 0 ? r : 0);
    return g;
}

// F16: the activations are binary16 (paper-literal path) instead of bfloat16.
template <int RP, int CPL, bool F16>
__global__ __launch_bounds__(256) void lora_grad_partial_kernel(GradPairArgs a, GradGeom g) {
    // one LDS buffer, used first for pieces of P and then for the waves' sums
    constexpr int PROWS = 128, RED_ROW = CPL * RP + 1;
    constexpr int LDS_FLOATS = 3 * 64 * RED_ROW > PROWS * RP ? 3 * 64 * RED_ROW : PROWS * RP;
    __shared__ __attribute__((aligned(16))) float lds_buf[LDS_FLOATS];
    float (*red)[64][RED_ROW] = reinterpret_cast<float (*)[64][RED_ROW]>(lds_buf);
    float (*Ps)[RP] = reinterpret_cast<float (*)[RP]>(lds_buf);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool is_a = (int)blockIdx.x < g.cols_a;
    const uint16_t *__restrict__ act = is_a ? a.X : a.dY;
    const float *__restrict__ P = is_a ? a.dYBt : a.XA;   // [M][r]: a row is the same for every lane (scalar loads)
    const int C = is_a ? a.K : a.N;
    const int c = (is_a ? blockIdx.x : blockIdx.x - g.cols_a) * (64 * CPL) + CPL * lane;
    const int r = a.r, j0 = blockIdx.z * RP;
    const int m_begin = blockIdx.y * g.rows_per_block;
    int m_end = m_begin + g.rows_per_block;
    if (m_end > a.M) m_end = a.M;
    const bool col_ok = c < C;   // C is a multiple of 8 >= CPL, so c + CPL - 1 < C too

    float acc[CPL][RP];
#pragma unroll
    for (int t = 0; t < CPL; ++t)
#pragma unroll
        for (int j = 0; j < RP; ++j) acc[t][j] = 0.f;

    // The rows of P that the workgroup needs pass through LDS, a piece of PROWS rows at a time:
    // every lane of a wave needs the same RP values of a row, and reading them from LDS (one
    // address for the whole wave: a broadcast) costs RP / 4 instructions per row, where loads from
    // global memory with a wave-uniform address would cost RP.
    typedef uint32_t words_t __attribute__((ext_vector_type(CPL / 2)));
    auto row_fma = [&](words_t v, int prow) {
        float x[CPL];
#pragma unroll
        for (int q = 0; q < CPL / 2; ++q) {
            uint32_t wq;
            wq = v[q];
            x[2 * q] = F16 ? half_bits_to_float((uint16_t)(wq & 0xFFFFu)) : __uint_as_float(wq << 16);
            x[2 * q + 1] = F16 ? half_bits_to_float((uint16_t)(wq >> 16)) : __uint_as_float(wq & 0xFFFF0000u);
        }
#pragma unroll
        for (int j = 0; j < RP; j += 4) {
            const float4 pj = *reinterpret_cast<const float4 *>(&Ps[prow][j]);
            const float pv[4] = {pj.x, pj.y, pj.z, pj.w};
#pragma unroll
            for (int z = 0; z < 4; ++z)
#pragma unroll
                for (int t = 0; t < CPL; ++t) acc[t][j + z] = __builtin_fmaf(x[t], pv[z], acc[t][j + z]);
        }
    };
    const uint16_t *col = act + (col_ok ? c : 0);
    for (int mb = m_begin; mb < m_end; mb += PROWS) {
        const int me = mb + PROWS < m_end ? mb + PROWS : m_end;
        __syncthreads();                              // the previous piece has been consumed
        for (int x = threadIdx.x; x < (me - mb) * RP; x += 256) {
            const int prow = x / RP, j = x % RP;
            Ps[prow][j] = j0 + j < r ? P[(size_t)(mb + prow) * r + j0 + j] : 0.f;
        }
        __syncthreads();
        // groups of four rows per wave (rows m, m + 4, m + 8, m + 12); the loads of the next group
        // are issued before the arithmetic of the current one, so a wave always has a group in flight
        int m = mb + wave;
        bool have = m + 12 < me;
        words_t cur[4];
        if (have) {
#pragma unroll
            for (int u = 0; u < 4; ++u) cur[u] = *reinterpret_cast<const words_t *>(col + (size_t)(m + 4 * u) * C);
        }
        while (have) {
            const int mn = m + 16;
            const bool have_next = mn + 12 < me;
            words_t nxt[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) nxt[u] = cur[u];
            if (have_next) {
#pragma unroll
                for (int u = 0; u < 4; ++u) nxt[u] = *reinterpret_cast<const words_t *>(col + (size_t)(mn + 4 * u) * C);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) row_fma(cur[u], m + 4 * u - mb);
#pragma unroll
            for (int u = 0; u < 4; ++u) cur[u] = nxt[u];
            m = mn;
            have = have_next;
        }
        for (; m < me; m += 4) row_fma(*reinterpret_cast<const words_t *>(col + (size_t)m * C), m - mb);
    }
    __syncthreads();                                  // every wave is done with the last piece of P

    if (wave > 0) {
#pragma unroll
        for (int t = 0; t < CPL; ++t)
#pragma unroll
            for (int j = 0; j < RP; ++j) red[wave - 1][lane][t * RP + j] = acc[t][j];
    }
    __syncthreads();
    if (wave != 0 || !col_ok) return;
    // a single row chunk is the whole sum: finish here (scale, accumulate flag) in the outputs
    // themselves, which have the layout of a partial, and skip stage 2
    const bool direct = g.chunks == 1;
    float *part = a.partials + (size_t)blockIdx.y * ((size_t)(a.K + a.N) * r);
    float *base_a = direct ? a.dA : part;
    float *base_b = direct ? a.dB : part + (size_t)a.K * r;
    const bool add_old = direct && a.accumulate;
#pragma unroll
    for (int t = 0; t < CPL; ++t) {
        float v[RP];
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            v[j] = acc[t][j] + red[0][lane][t * RP + j] + red[1][lane][t * RP + j] + red[2][lane][t * RP + j];
            if (direct) v[j] *= a.lora_scale;
        }
        if (is_a) {
            float *dst = base_a + (size_t)(c + t) * r + j0;
            if ((r & 3) == 0) {
#pragma unroll
                for (int j = 0; j < RP; j += 4)
                    if (j0 + j < r) {
                        float4 o = make_float4(v[j], v[j + 1], v[j + 2], v[j + 3]);
                        if (add_old) {
                            const float4 old = *reinterpret_cast<const float4 *>(dst + j);
                            o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
                        }
                        *reinterpret_cast<float4 *>(dst + j) = o;
                    }
            } else {
#pragma unroll
                for (int j = 0; j < RP; ++j)
                    if (j0 + j < r) dst[j] = add_old ? dst[j] + v[j] : v[j];
            }
        } else {
            float *dst = base_b + (size_t)j0 * a.N + (c + t);
#pragma unroll
            for (int j = 0; j < RP; ++j)
                if (j0 + j < r) dst[(size_t)j * a.N] = add_old ? dst[(size_t)j * a.N] + v[j] : v[j];
        }
    }
}

// out = (accumulate ? out : 0) + s * sum over chunks; 4 consecutive elements per thread.
__global__ __launch_bounds__(256) void lora_grad_reduce_kernel(GradPairArgs a, int chunks) {
    const size_t n_a = (size_t)a.K * a.r, n = n_a + (size_t)a.N * a.r;
    const size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= n) return;
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    const float *p = a.partials + e;
    int q = 0;
    for (; q + 4 <= chunks; q += 4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4 *>(p + (size_t)(q + u) * n);
#pragma unroll
        for (int u = 0; u < 4; ++u) { sum.x += v[u].x; sum.y += v[u].y; sum.z += v[u].z; sum.w += v[u].w; }
    }
    for (; q < chunks; ++q) {
        const float4 v = *reinterpret_cast<const float4 *>(p + (size_t)q * n);
        sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    float4 *dst = reinterpret_cast<float4 *>(e < n_a ? a.dA + e : a.dB + (e - n_a));
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    if (a.accumulate) o = *dst;
    o.x = __builtin_fmaf(a.lora_scale, sum.x, o.x);
    o.y = __builtin_fmaf(a.lora_scale, sum.y, o.y);
    o.z = __builtin_fmaf(a.lora_scale, sum.z, o.z);
    o.w = __builtin_fmaf(a.lora_scale, sum.w, o.w);
    *dst = o;
}

hipError_t launch_lora_grad_pair(const GradPairArgs &a, hipStream_t stream) {
    const GradGeom g = grad_geom(a.M, a.K, a.N, a.r);
    dim3 grid(g.cols_a + g.cols_b, g.chunks, g.passes);
    if (a.f16) {
        if (a.r <= 8) launch_kernel("lora_grad", lora_grad_partial_kernel<8, 4, true>, grid, 256, 0, stream, a, g);
        else if (a.r <= 16) launch_kernel("lora_grad", lora_grad_partial_kernel<16, 4, true>, grid, 256, 0, stream, a, g);
        else launch_kernel("lora_grad", lora_grad_partial_kernel<32, 2, true>, grid, 256, 0, stream, a, g);
    } else {
        if (a.r <= 8) launch_kernel("lora_grad", lora_grad_partial_kernel<8, 4, false>, grid, 256, 0, stream, a, g);
        else if (a.r <= 16) launch_kernel("lora_grad", lora_grad_partial_kernel<16, 4, false>, grid, 256, 0, stream, a, g);
        else launch_kernel("lora_grad", lora_grad_partial_kernel<32, 2, false>, grid, 256, 0, stream, a, g);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || g.chunks == 1) return e;
    const size_t n = (size_t)(a.K + a.N) * a.r;
    launch_kernel("lora_grad_reduce", lora_grad_reduce_kernel, (unsigned)((n / 4 + 255) / 256), 256, 0, stream, a, g.chunks);
    return hipGetLastError();
}

}  // namespace mlr
