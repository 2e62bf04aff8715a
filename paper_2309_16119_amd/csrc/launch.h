// Internal host-side interface between the C-ABI layer (api.hip) and the kernel
// translation units.  Not installed; nothing outside csrc/ includes it.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace mlr {

// The frozen quantized weight (same fields as modulora_qweight, device pointers).
struct LayerView {
    int K, N, bits, group;
    const uint32_t *qweight;
    const uint16_t *scales;
    const uint8_t *zeros;
};

// Length of the extended contraction that carries the rank-r adapter through the
// MFMA pipeline: three bfloat16 segments of r (hi*hi, hi*lo, lo*hi), padded to
// the MFMA K-step of 16.
inline int lora_ext_len(int r) { return r > 0 ? ((3 * r + 15) / 16) * 16 : 0; }

// ---- kernel launches and the profiling hook (api.hip owns the state) ---------------
// While modulora_profile_begin() is active, prof_events() hands out a fresh pair of events
// for one launch and returns true.
bool prof_events(const char *kernel_name, hipEvent_t *start, hipEvent_t *stop);

// Every kernel launch of the library goes through here.  Normally a plain launch; while
// profiling, the two events are attached to the dispatch itself, so they time the kernel
// alone (not the launch path around it).
template <typename... KArgs, typename... Args>
inline void launch_kernel(const char *name, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes,
                          hipStream_t stream, Args... args) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (prof_events(name, &e0, &e1))
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, stream, e0, e1, 0u, static_cast<KArgs>(args)...);
    else
        hipLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, stream, static_cast<KArgs>(args)...);
}

// ---- dequant_kernel.hip ------------------------------------------------------
hipError_t launch_dequant(const LayerView &w, uint16_t *What, hipStream_t stream);

// ---- gemm_tile.hip -----------------------------------------------------------
// out[M][Cout] = act[M][C] (x) What  (+ act_ext[M][RE] . w_ext[Cout][RE]^T)
//   forward : C = K, Cout = N, out[m][n] = sum_k act[m][k] What[n][k]
//   backward: C = N, Cout = K, out[m][k] = sum_n act[m][n] What[n][k]
struct GemmArgs {
    LayerView w;
    bool backward;
    const uint16_t *act;      // bf16 [M][C]
    int M;
    uint16_t *out;            // bf16 [M][Cout]
    const uint16_t *act_ext;  // bf16 [M][RE]    (NULL when RE == 0)
    const uint16_t *w_ext;    // bf16 [Cout][RE] (NULL when RE == 0)
    int RE;                   // multiple of 16
    float *partials;          // scratch for the partial tiles of a split contraction, or NULL
    size_t partials_bytes;    // its size: a plan that needs more runs whole tiles only
    // The layer in the paper's own storage convention (launch_gemm_mid_f16 only): binary16
    // activations and outputs, binary16 zero points that are added (w.zeros unused), an optional
    // binary16 bias (forward), and the adapter term s P F in the epilogue instead of the extended
    // contraction (act_ext, w_ext, RE unused).
    const uint16_t *zeros16;  // binary16 [K/group][N]
    const uint16_t *bias16;   // binary16 [N] or NULL
    const float *ep_P;        // fp32 [M][ep_r] or NULL
    const float *ep_F;        // forward B [r][N], backward A [K][r]
    int ep_r;
    float ep_scale;
};
hipError_t launch_gemm(const GemmArgs &a, hipStream_t stream);
// gemm_mid.hip, binary16 instantiation: the 128 x 64 producer / consumer kernel for the layer in
// the paper's own storage convention (GemmArgs::zeros16, bias16, ep_*).
hipError_t launch_gemm_mid_f16(const GemmArgs &a, hipStream_t stream);
// gemm_big.hip, binary16 instantiation: the 256 x 256 kernel (whole tiles only when GemmArgs::partials is NULL).
hipError_t launch_gemm_big_f16(const GemmArgs &a, hipStream_t stream);

// How the 256 x 256 kernel fills 256 compute units when the tile count is not a multiple of
// 256: the first `full` tiles run whole; each of the `tail` remaining ones is cut into
// `split` slices of the contraction, one workgroup each, which leave fp32 partial tiles
// that a second small kernel adds up.  split == 1: nothing is cut.  `mt`: rows of a tile,
// 256 or (the kernel's second instantiation) 128.
struct BigPlan {
    int full, tail, split, mt;
    size_t partial_bytes() const { return split > 1 ? (size_t)tail * split * ((size_t)mt * 256u * 4u) : 0; }
};
inline BigPlan big_plan_rows(int M, int C, int Cout, int mt) {
    BigPlan p;
    p.mt = mt;
    const long tiles = (long)((M + mt - 1) / mt) * ((Cout + 255) / 256);
    p.full = (int)(tiles / 256 * 256);
    p.tail = (int)(tiles - p.full);
    p.split = 1;
    if (p.tail > 0) {
        int s = 256 / p.tail;                 // slices that still fit one round
        const int by_depth = (C / 64) / 8;    // at least 8 steps of 64 per slice
        if (s > by_depth) s = by_depth;
        if (s > 8) s = 8;
        if (s > 1) p.split = s;
    }
    return p;
}
// 128-row tiles where the last block of 256 rows would be at most half full and the row blocks
// are few: a step of the 128-row kernel takes 0.55 of a 256-row step, so an odd number n of
// 128-row blocks costs 0.55 n against (n + 1) / 2.
inline BigPlan big_plan(int M, int C, int Cout) {
    const int n128 = (M + 127) / 128;
    const bool half_rows = (n128 & 1) != 0 && n128 <= 5;
    return big_plan_rows(M, C, Cout, half_rows ? 128 : 256);
}
// Scratch for the partial tiles of either direction.
inline size_t gemm_partial_bytes(int M, int K, int N) {
    const size_t f = big_plan(M, K, N).partial_bytes(), b = big_plan(M, N, K).partial_bytes();
    return f > b ? f : b;
}

// ---- lora_kernels.hip ----------------------------------------------------------
// P[m][j] = sum_c act[m][c] * F(c, j)  and the extended operands for launch_gemm.
//   f_is_A: F(c, j) = Fm[c * r + j]  (A [K][r], projection of X)
//   else  : F(c, j) = Fm[j * C + c]  (B [r][N], projection of dY onto B^T)
// Writes P (fp32 [M][r]); if act_ext != NULL also the split of lora_scale * P into
// act_ext [M][RE]; if w_ext != NULL also w_ext [Cw][RE] from Wsrc:
//   w_from_A: w_ext[c][.] from Wsrc[c * r + j] (A, for the backward pass)
//   else    : w_ext[c][.] from Wsrc[j * Cw + c] (B, for the forward pass)
struct DownArgs {
    const uint16_t *act;  // bf16 [M][C] (binary16 when act_f16)
    bool act_f16;         // the layer in the paper's own storage convention: binary16 activations, P only
    int M, C, r;
    const float *Fm;
    bool f_is_A;
    float *P;             // fp32 [M][r]
    float lora_scale;
    uint16_t *act_ext;    // may be NULL
    int RE;
    uint16_t *w_ext;      // may be NULL
    const float *Wsrc;
    bool w_from_A;
    int Cw;
    float *partials;      // scratch of lora_down_partial_bytes() bytes (split contraction)
};
// How launch_lora_down covers act [M][C]: a workgroup of `nwaves` waves owns `rowt` tiles of 16 rows
// (they share every factor operand: the fp32 factor is fetched and split once per workgroup and
// step, not once per 16 rows) and one of `split` slices of the contraction, which its waves
// divide again.  With split > 1 the slices leave partial tiles that a second small kernel adds.
// Many tokens take rowt = 4 and as many slices as give the chip about two workgroups per compute
// unit; few tokens keep one tile per workgroup and split only a deep contraction.
struct DownPlan {
    int rowt, nwaves, split;
};
inline DownPlan lora_down_plan(int M, int C, int r) {
    DownPlan p;
    const int rg = (r + 15) / 16;
    const int tiles16 = (M + 15) / 16;
    // (a contraction under ~6000 is too short to split further: there one tile per workgroup and no
    // second launch is quicker)
    p.rowt = (tiles16 >= 64 && rg <= 2 && C >= 6144) ? 4 : 1;
    const int row_blocks = (tiles16 + p.rowt - 1) / p.rowt;
    const int steps = (C + 31) / 32;
    if (p.rowt == 4) {
        p.nwaves = rg == 1 ? 8 : 4;                      // at most 32 partial tiles meet in a workgroup's LDS
        int split = (512 + row_blocks - 1) / row_blocks;
        const int by_depth = steps / (2 * p.nwaves);     // at least 2 steps of 32 per wave
        if (split > by_depth) split = by_depth;
        if (split > 16) split = 16;
        p.split = split < 2 ? 1 : split;
        return p;
    }
    int nwaves = 4;
    while (nwaves < 16 && row_blocks * nwaves < 2048 && nwaves * 2 * rg <= 32) nwaves *= 2;
    p.nwaves = nwaves;
    p.split = 1;
    if (row_blocks * 16 < 1024) {                        // 16 waves per workgroup do not fill the chip yet
        int split = (2048 + row_blocks * 16 - 1) / (row_blocks * 16);
        const int by_depth = C / (32 * 16 * 2);
        if (split > by_depth) split = by_depth;
        if (split > 16) split = 16;
        // (measured at 512 tokens x 4096: one launch with 8 steps per wave takes 10-11 us, the split
        // launch plus its finish kernel 5-6 + 4-5 us, and the whole call 3 us less)
        if (split >= 2) p.split = split;
    }
    return p;
}
inline size_t lora_down_partial_bytes(int M, int K, int N, int r) {
    if (r <= 0) return 0;
    size_t most = 0;
    for (int C : {K, N}) {
        const DownPlan p = lora_down_plan(M, C, r);
        if (p.split <= 1) continue;
        const size_t rg = (size_t)(r + 15) / 16;
        const size_t row_blocks = (size_t)(((M + 15) / 16) + p.rowt - 1) / p.rowt;
        const size_t b = (size_t)p.split * row_blocks * (size_t)p.rowt * 256u * rg * sizeof(float);
        if (b > most) most = b;
    }
    return most;
}
hipError_t launch_lora_down(const DownArgs &a, hipStream_t stream);

// dA[k][j] (+)= lora_scale * sum_m X[m][k] dYBt[m][j]   and
// dB[j][n] (+)= lora_scale * sum_m XA[m][j] dY[m][n],  in two launches (partials, reduce).
struct GradPairArgs {
    const uint16_t *X, *dY;      // bf16 [M][K], [M][N]
    int M, K, N, r;              // r >= 1
    const float *XA, *dYBt;      // fp32 [M][r]
    float lora_scale;
    float *dA, *dB;              // fp32 [K][r], [r][N]
    int accumulate;              // 0: overwrite, 1: add onto the outputs
    float *partials;             // scratch, grad_geom().partial_floats floats
    int f16;                     // X, dY are binary16 instead of bfloat16 (the paper-literal path)
};
struct GradGeom {
    int cpl;                     // columns per lane (2 or 4)
    int cols_a, cols_b;          // column blocks (64 * cpl columns) of X and of dY
    int chunks, rows_per_block;  // row chunks (one partial each)
    int passes;                  // rank passes of 32 (r > 32)
    size_t partial_floats;
};
GradGeom grad_geom(int M, int K, int N, int r);
hipError_t launch_lora_grad_pair(const GradPairArgs &a, hipStream_t stream);

// ---- f16_path.hip: the layer in the paper's own storage convention ---------------------
// (float zero point that is added, binary16 scales / zero points / activations / outputs, bias)
struct F16Layer {
    int K, N, bits, group;
    const uint32_t *qweight;
    const uint16_t *scales;   // binary16 [K/group][N]
    const uint16_t *zeros;    // binary16 [K/group][N], added
    const uint16_t *bias;     // binary16 [N] or NULL
};
hipError_t launch_f16_dequant(const F16Layer &w, uint16_t *What, hipStream_t stream);
// P[M][r] = act[M][C] F, F = A [C][r] (f_is_A) or B^T with B [r][C]
// forward: out[M][N] = act What^T + bias + s P B; backward: out[M][K] = act What + s P A^T
// partials: scratch of gemm_partial_bytes(M, K, N) bytes for the 256 x 256 kernel's split contraction, or NULL
hipError_t launch_f16_gemm(const F16Layer &w, bool backward, const uint16_t *act, int M, uint16_t *out, const float *P,
                           const float *Fm, int r, float lora_scale, float *partials, hipStream_t stream);

// ---- quantize.hip: round-to-nearest group quantizer + packer -------------------------
struct QuantArgs {
    const float *W;       // fp32 [N][K]
    int K, N, bits, group;
    uint32_t *qweight;    // [K*bits/32][N]
    uint16_t *scales;     // binary16 [K/group][N]
    uint8_t *zeros;       // [K/group][N]
};
hipError_t launch_quantize_rtn(const QuantArgs &a, hipStream_t stream);

// ---- optim.hip: AdamW on a flat fp32 buffer ---------------------------------------
struct AdamWArgs {
    float *p, *m, *v;
    const float *g;
    size_t n;
    float beta1, beta2, one_minus_beta1, one_minus_beta2;
    float decay;          // 1 - lr * weight_decay
    float step_size;      // lr / (1 - beta1^step)
    float inv_sqrt_bc2;   // 1 / sqrt(1 - beta2^step)
    float eps;
};
hipError_t launch_adamw(const AdamWArgs &a, hipStream_t stream);

// ---- smallm.hip: streaming kernels for a handful of tokens ------------------------
// A launch of the kernels handles at most SMALLM_ROWS token rows (one MFMA tile); the launchers take
// up to SMALLM_MAX_M rows and run that many passes over the packed weight, one after the other on
// the stream (sharing the scratch): two passes over a weight of some megabytes still cost a
// fraction of what a tile kernel needs for so few rows.
constexpr int SMALLM_ROWS = 16, SMALLM_MAX_M = 32;
struct SmallArgs {
    LayerView w;
    const uint16_t *act;  // bf16 [M][K] (forward) or [M][N] (backward)
    int M;
    uint16_t *out;        // bf16 [M][N] (forward) or [M][K] (backward)
    const float *A, *B;   // adapter factors (ignored when r == 0)
    int r;
    float lora_scale;
    float *P_out;         // XA / dYBt hand-off [M][r], may be NULL
    void *ws;             // at least smallm_ws_bytes() bytes
    // The layer in the paper's own storage convention: binary16 activations and outputs, binary16
    // zero points [K/group][N] that are added (w.zeros unused), optional binary16 bias [N] (forward).
    bool f16;
    const uint16_t *zeros16;
    const uint16_t *bias16;
};
bool smallm_fwd_supported(const LayerView &w, int M);
bool smallm_bwd_supported(const LayerView &w, int M);
size_t smallm_ws_bytes(int K, int N, int r);              // enough for both passes of any layer of this shape
size_t smallm_fwd_ws_bytes(const LayerView &w, int r);    // what launch_smallm_fwd touches for this layer
hipError_t launch_smallm_fwd(const SmallArgs &a, hipStream_t stream);
hipError_t launch_smallm_bwd(const SmallArgs &a, hipStream_t stream);

}  // namespace mlr
