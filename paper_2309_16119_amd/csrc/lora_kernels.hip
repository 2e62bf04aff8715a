// The rank-r adapter side of the layer (Section 3.1 eq. (3) and Section 3.1.1 of the
// ModuLoRA paper): the skinny projections  XA = X A  and  dYBt = dY B^T, the adapter
// gradients  dA = s X^T dYBt  and  dB = s XA^T dY, and the preparation of the
// "extended contraction" operands with which the tile GEMM adds the adapter term
// s (X A) B inside its MFMA loop.
//
// All of these are bound by one streaming pass over X or dY; the arithmetic is plain
// fp32 FMA with coalesced 16-byte (projection) or 4-byte (gradient) loads per lane.
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
// Projection: P[m][j] = sum_c act[m][c] F(c, j); one workgroup owns ROWS rows and
// walks the whole contraction; lanes own 8-column chunks (16-byte loads).
// Extra workgroups (blockIdx.x >= row blocks) write the weight-side extension.
// ---------------------------------------------------------------------------
template <int RP, int ROWS, bool F_IS_A>
__global__ __launch_bounds__(256) void lora_down_kernel(DownArgs a, int row_blocks) {
    __shared__ float red[4][ROWS * RP];
    __shared__ float Ps[ROWS * RP];
    const int tid = threadIdx.x;
    const int r = a.r;

    if ((int)blockIdx.x >= row_blocks) {
        // weight-side extension: w_ext[c][e]
        const size_t total = (size_t)a.Cw * a.RE;
        size_t idx = (size_t)(blockIdx.x - row_blocks) * 256 + tid;
        const size_t stride = (size_t)(gridDim.x - row_blocks) * 256;
        for (; idx < total; idx += stride) {
            const int c = (int)(idx / a.RE), e = (int)(idx % a.RE);
            uint16_t v = 0;
            if (e < 3 * r) {
                const int seg = e / r, j = e % r;
                const float src = a.w_from_A ? a.Wsrc[(size_t)c * r + j] : a.Wsrc[(size_t)j * a.Cw + c];
                v = split_part(src, seg == 1);
            }
            a.w_ext[idx] = v;
        }
        return;
    }

    const int m0 = blockIdx.x * ROWS;
    float acc[ROWS][RP];
#pragma unroll
    for (int i = 0; i < ROWS; ++i)
#pragma unroll
        for (int j = 0; j < RP; ++j) acc[i][j] = 0.f;

    for (int c = tid * 8; c < a.C; c += 256 * 8) {
        float x[ROWS][8];
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (m0 + i < a.M) v = *reinterpret_cast<const uint4 *>(a.act + (size_t)(m0 + i) * a.C + c);
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                x[i][2 * t] = __uint_as_float(u[t] << 16);
                x[i][2 * t + 1] = __uint_as_float(u[t] & 0xFFFF0000u);
            }
        }
        if (F_IS_A) {
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) {
                float f[RP];
                const float *src = a.Fm + (size_t)(c + cc) * r;
                if (r == RP) {
#pragma unroll
                    for (int j = 0; j < RP; j += 4) {
                        const float4 q = *reinterpret_cast<const float4 *>(src + j);
                        f[j] = q.x; f[j + 1] = q.y; f[j + 2] = q.z; f[j + 3] = q.w;
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < RP; ++j) f[j] = j < r ? src[j] : 0.f;
                }
#pragma unroll
                for (int i = 0; i < ROWS; ++i)
#pragma unroll
                    for (int j = 0; j < RP; ++j) acc[i][j] = __builtin_fmaf(x[i][cc], f[j], acc[i][j]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < RP; ++j) {
                float f[8];
                if (j < r) {
                    const float4 q0 = *reinterpret_cast<const float4 *>(a.Fm + (size_t)j * a.C + c);
                    const float4 q1 = *reinterpret_cast<const float4 *>(a.Fm + (size_t)j * a.C + c + 4);
                    f[0] = q0.x; f[1] = q0.y; f[2] = q0.z; f[3] = q0.w;
                    f[4] = q1.x; f[5] = q1.y; f[6] = q1.z; f[7] = q1.w;
                } else {
#pragma unroll
                    for (int cc = 0; cc < 8; ++cc) f[cc] = 0.f;
                }
#pragma unroll
                for (int i = 0; i < ROWS; ++i)
#pragma unroll
                    for (int cc = 0; cc < 8; ++cc) acc[i][j] = __builtin_fmaf(x[i][cc], f[cc], acc[i][j]);
            }
        }
    }

    // reduce over the 64 lanes of each wave, then over the 4 waves through LDS
#pragma unroll
    for (int i = 0; i < ROWS; ++i)
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            float v = acc[i][j];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
            acc[i][j] = v;
        }
    const int wave = tid >> 6, lane = tid & 63;
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < ROWS; ++i)
#pragma unroll
            for (int j = 0; j < RP; ++j) red[wave][i * RP + j] = acc[i][j];
    }
    __syncthreads();
    for (int t = tid; t < ROWS * RP; t += 256) {
        const float v = red[0][t] + red[1][t] + red[2][t] + red[3][t];
        Ps[t] = v;
        const int i = t / RP, j = t % RP;
        if (m0 + i < a.M && j < r) a.P[(size_t)(m0 + i) * r + j] = v;
    }
    if (a.act_ext == nullptr) return;
    __syncthreads();
    for (int t = tid; t < ROWS * a.RE; t += 256) {
        const int i = t / a.RE, e = t % a.RE;
        if (m0 + i >= a.M) continue;
        uint16_t v = 0;
        if (e < 3 * r) {
            const int seg = e / r, j = e % r;
            v = split_part(a.lora_scale * Ps[i * RP + j], seg == 2);
        }
        a.act_ext[(size_t)(m0 + i) * a.RE + e] = v;
    }
}

template <int RP, int ROWS>
static hipError_t launch_down_rp(const DownArgs &a, hipStream_t stream) {
    const int row_blocks = (a.M + ROWS - 1) / ROWS;
    int w_blocks = 0;
    if (a.w_ext) {
        const size_t total = (size_t)a.Cw * a.RE;
        w_blocks = (int)((total + 256 * 8 - 1) / (256 * 8));
        if (w_blocks > 512) w_blocks = 512;
        if (w_blocks < 1) w_blocks = 1;
    }
    prof_before("lora_down", stream);
    if (a.f_is_A)
        lora_down_kernel<RP, ROWS, true><<<row_blocks + w_blocks, 256, 0, stream>>>(a, row_blocks);
    else
        lora_down_kernel<RP, ROWS, false><<<row_blocks + w_blocks, 256, 0, stream>>>(a, row_blocks);
    prof_after(stream);
    return hipGetLastError();
}

hipError_t launch_lora_down(const DownArgs &a, hipStream_t stream) {
    if (a.r <= 8) return launch_down_rp<8, 4>(a, stream);
    if (a.r <= 16) return launch_down_rp<16, 4>(a, stream);
    if (a.r <= 32) return launch_down_rp<32, 2>(a, stream);
    return launch_down_rp<64, 1>(a, stream);
}

// ---------------------------------------------------------------------------
// Adapter gradients (Section 3.1.1), both in one launch plus one reduction launch:
//   dA[k][j] = s * sum_m X[m][k]  dYBt[m][j]      dB[j][n] = s * sum_m XA[m][j] dY[m][n]
// Stage 1: a workgroup owns 128 columns of X (or dY) and a chunk of rows; each lane owns 2
// adjacent columns (one 4-byte load per row), the 4 waves take rows round-robin, P[m][:] is
// wave-uniform.  The 4 waves' sums meet in LDS and go out as one partial per row chunk, laid
// out like the outputs ([chunk][dA | dB]).  Stage 2 adds the chunks, applies s and the
// accumulate flag.  No atomics (device-scope fp32 atomics bypass the per-XCD L2 and are slow)
// and no zero-fill of the outputs.
// ---------------------------------------------------------------------------
GradGeom grad_geom(int M, int K, int N, int r) {
    GradGeom g;
    g.cols_a = (K + 127) / 128;
    g.cols_b = (N + 127) / 128;
    const int col_blocks = g.cols_a + g.cols_b;
    // enough row chunks to give the chip ~1024 workgroups, at least 32 rows each
    int chunks = (1024 + col_blocks - 1) / col_blocks;
    const int max_chunks = (M + 31) / 32;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    int rows = (M + chunks - 1) / chunks;
    rows = (rows + 3) / 4 * 4;
    g.rows_per_block = rows;
    g.chunks = (M + rows - 1) / rows;
    g.passes = r > 32 ? 2 : 1;
    g.partial_floats = (size_t)g.chunks * (size_t)(K + N) * (size_t)(r > 0 ? r : 0);
    return g;
}

template <int RP>
__global__ __launch_bounds__(256) void lora_grad_partial_kernel(GradPairArgs a, GradGeom g) {
    __shared__ float red[3][64][2 * RP + 1];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool is_a = (int)blockIdx.x < g.cols_a;
    const uint16_t *act = is_a ? a.X : a.dY;
    const float *P = is_a ? a.dYBt : a.XA;
    const int C = is_a ? a.K : a.N;
    const int c = (is_a ? blockIdx.x : blockIdx.x - g.cols_a) * 128 + 2 * lane;
    const int r = a.r, j0 = blockIdx.z * RP;
    const int m_begin = blockIdx.y * g.rows_per_block;
    int m_end = m_begin + g.rows_per_block;
    if (m_end > a.M) m_end = a.M;
    const bool col_ok = c < C;   // C is even, so c + 1 < C too

    float acc[2][RP];
#pragma unroll
    for (int j = 0; j < RP; ++j) acc[0][j] = acc[1][j] = 0.f;

    auto row_fma = [&](uint32_t v, int m) {
        const float x0 = __uint_as_float(v << 16), x1 = __uint_as_float(v & 0xFFFF0000u);
        const float *p = P + (size_t)m * r + j0;
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            const float pj = j0 + j < r ? p[j] : 0.f;
            acc[0][j] = __builtin_fmaf(x0, pj, acc[0][j]);
            acc[1][j] = __builtin_fmaf(x1, pj, acc[1][j]);
        }
    };
    const uint16_t *col = act + (col_ok ? c : 0);
    int m = m_begin + wave;
    for (; m + 12 < m_end; m += 16) {     // four rows in flight per wave
        uint32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const uint32_t *>(col + (size_t)(m + 4 * u) * C);
#pragma unroll
        for (int u = 0; u < 4; ++u) row_fma(v[u], m + 4 * u);
    }
    for (; m < m_end; m += 4) row_fma(*reinterpret_cast<const uint32_t *>(col + (size_t)m * C), m);

    if (wave > 0) {
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            red[wave - 1][lane][j] = acc[0][j];
            red[wave - 1][lane][RP + j] = acc[1][j];
        }
    }
    __syncthreads();
    if (wave != 0 || !col_ok) return;
    float *part = a.partials + (size_t)blockIdx.y * ((size_t)(a.K + a.N) * r);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        float v[RP];
#pragma unroll
        for (int j = 0; j < RP; ++j)
            v[j] = acc[t][j] + red[0][lane][t * RP + j] + red[1][lane][t * RP + j] + red[2][lane][t * RP + j];
        if (is_a) {
            float *dst = part + (size_t)(c + t) * r + j0;
            if ((r & 3) == 0) {
#pragma unroll
                for (int j = 0; j < RP; j += 4)
                    if (j0 + j < r) *reinterpret_cast<float4 *>(dst + j) = make_float4(v[j], v[j + 1], v[j + 2], v[j + 3]);
            } else {
#pragma unroll
                for (int j = 0; j < RP; ++j)
                    if (j0 + j < r) dst[j] = v[j];
            }
        } else {
            float *dst = part + (size_t)a.K * r + (size_t)j0 * a.N + (c + t);
#pragma unroll
            for (int j = 0; j < RP; ++j)
                if (j0 + j < r) dst[(size_t)j * a.N] = v[j];
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
    prof_before("lora_grad", stream);
    if (a.r <= 8) lora_grad_partial_kernel<8><<<grid, 256, 0, stream>>>(a, g);
    else if (a.r <= 16) lora_grad_partial_kernel<16><<<grid, 256, 0, stream>>>(a, g);
    else lora_grad_partial_kernel<32><<<grid, 256, 0, stream>>>(a, g);
    prof_after(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t n = (size_t)(a.K + a.N) * a.r;
    prof_before("lora_grad_reduce", stream);
    lora_grad_reduce_kernel<<<(unsigned)((n / 4 + 255) / 256), 256, 0, stream>>>(a, g.chunks);
    prof_after(stream);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *dst, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) dst[i] = 0.f;
}

hipError_t launch_fill_zero(float *dst, size_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    prof_before("fill_zero", stream);
    fill_zero_kernel<<<(unsigned)blocks, 256, 0, stream>>>(dst, n);
    prof_after(stream);
    return hipGetLastError();
}

}  // namespace mlr
