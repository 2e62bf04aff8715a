// Fused dequantize + bf16 MFMA tile kernel for the two products with the frozen
// low-precision weight (ModuLoRA Figure 1):
//   forward   out[m][n] = sum_k act[m][k] What[n][k]      (LPLinear.forward)
//   backward  out[m][k] = sum_n act[m][n] What[n][k]      (LPLinear.backward, with
//                                                          What re-materialized)
// What is produced tile by tile from the packed codes straight into LDS (Section 3.1.2:
// materialize only what is needed, when it is needed) and never reaches HBM.  The
// rank-r adapter term of eq. (3) rides along as a short "extended contraction" of
// bfloat16 hi/lo splits prepared by lora_down_kernel.
//
// Layout facts used below (gfx950, wave64):
//   v_mfma_f32_32x32x16_bf16: lane l gives A[row l%32][8 consecutive k at 8*(l/32)]
//   and B[8 consecutive k at 8*(l/32)][col l%32]; accumulator register v of lane l is
//   D[row 8*(v/4) + 4*(l/32) + v%4][col l%32].
//   Both operands therefore want the contraction index contiguous per lane, so both
//   LDS tiles are stored [row or col][contraction], 16-byte reads per lane.
//   - forward: one packed word holds codes along k for one column n -> a lane that
//     loads the words of column n writes 8 consecutive k of row n of the W tile.
//   - backward: the contraction runs over n, and qweight is n-contiguous, so a lane
//     that loads the words of 8 adjacent columns holds, for each k of the chunk, the
//     8 consecutive n the MFMA operand wants; no transpose through LDS is needed.
#include "device_common.h"
#include "launch.h"

namespace mlr {

constexpr int RT = 64;         // contraction elements per LDS tile
constexpr int LDS_PAD = 8;     // bf16 elements of row padding (row stride 144 B: conflict-free 16-B accesses)
constexpr int LROW = RT + LDS_PAD;
constexpr int THREADS = 256;

struct TileCoord {
    int tm, tc;
};

// XCD-aware tile order: consecutive workgroup ids go round-robin over the 8 XCDs, so
// give each XCD a contiguous run of tiles, and walk tiles column-major inside a run
// so that neighbours on one XCD share the weight tile (and its L2 lines).
__device__ __forceinline__ TileCoord tile_of_block(int bid, int tiles_m, int tiles_c) {
    const int total = tiles_m * tiles_c;
    const int per_xcd = (total + 7) / 8;
    int t = (bid % 8) * per_xcd + bid / 8;
    TileCoord tc;
    if (t >= total) { tc.tm = -1; tc.tc = -1; return tc; }
    tc.tc = t / tiles_m;
    tc.tm = t % tiles_m;
    return tc;
}

template <int BITS, bool BWD, int MT, int CT, int WM, int WN>
__global__ __launch_bounds__(THREADS) void gemm_tile_kernel(GemmArgs a, int tiles_m, int tiles_c) {
    static_assert((MT / WM) * (CT / WN) == THREADS / 64, "4 waves");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 MFMA tiles");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t *As = lds;                 // [MT][LROW]
    uint16_t *Ws = lds + MT * LROW;     // [CT][LROW]

    // grid is padded up to a multiple of 8 blocks; surplus blocks leave here
    const TileCoord tcoord = tile_of_block(blockIdx.x, tiles_m, tiles_c);
    if (tcoord.tm < 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = tcoord.tm * MT, c0 = tcoord.tc * CT;
    const int K = a.w.K, N = a.w.N;
    const int C = BWD ? N : K;          // contraction length
    const int Cout = BWD ? K : N;       // output columns
    const int n_main = (C + RT - 1) / RT;
    const int n_ext = (a.RE + RT - 1) / RT;
    const int n_tiles = n_main + n_ext;

    // ---- register staging for one tile -------------------------------------
    constexpr int A_CH = MT * (RT / 8) / THREADS;            // 16-byte activation chunks per thread
    constexpr int FW_UNITS = CT * (RT / 32) / THREADS;       // forward: (column, 32-code block) units
    constexpr int BW_UNITS = (CT / 8) * (RT / 8) / THREADS;  // backward: (8 columns n, 8 codes k) units
    static_assert(A_CH >= 1 && (MT * (RT / 8)) % THREADS == 0, "activation tile divides");
    static_assert(CT * (RT / 32) % THREADS == 0 && FW_UNITS >= 1, "forward units divide");
    static_assert(BWD ? ((CT / 8) * (RT / 8) % THREADS == 0 && BW_UNITS >= 1) : true, "backward units divide");
    constexpr int W_CH = CT * (RT / 8) / THREADS;             // 16-byte chunks of an extension W tile

    uint4 a_reg[A_CH];
    uint32_t fw_words[BWD ? 1 : FW_UNITS][BITS];
    DqConst fw_dq[BWD ? 1 : FW_UNITS];
    uint32_t bw_lo[BWD ? BW_UNITS : 1][8], bw_hi[BWD ? BW_UNITS : 1][8];
    uint32_t bw_scale[BWD ? BW_UNITS : 1][4];   // 8 binary16
    uint32_t bw_zero[BWD ? BW_UNITS : 1][2];    // 8 uint8
    int bw_shift[BWD ? BW_UNITS : 1];
    uint4 w_reg[W_CH];                           // extension tiles only

    auto load_tile = [&](int t) {
        const bool ext = t >= n_main;
        const int r0 = ext ? (t - n_main) * RT : t * RT;       // first contraction index
        const uint16_t *src = ext ? a.act_ext : a.act;
        const int ld = ext ? a.RE : C;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int idx = tid + i * THREADS;
            const int row = idx / (RT / 8), ch = idx % (RT / 8);
            const int m = m0 + row, cc = r0 + ch * 8;
            a_reg[i] = make_uint4(0, 0, 0, 0);
            if (m < a.M && cc < ld) a_reg[i] = *reinterpret_cast<const uint4 *>(src + (size_t)m * ld + cc);
        }
        if (ext) {
#pragma unroll
            for (int i = 0; i < W_CH; ++i) {
                const int idx = tid + i * THREADS;
                const int row = idx / (RT / 8), ch = idx % (RT / 8);
                const int c = c0 + row, cc = r0 + ch * 8;
                w_reg[i] = make_uint4(0, 0, 0, 0);
                if (c < Cout && cc < a.RE) w_reg[i] = *reinterpret_cast<const uint4 *>(a.w_ext + (size_t)c * a.RE + cc);
            }
            return;
        }
        if (!BWD) {
#pragma unroll
            for (int u = 0; u < FW_UNITS; ++u) {
                const int idx = tid + u * THREADS;
                const int nl = idx % CT, kb = idx / CT;
                const int n = c0 + nl, k = r0 + kb * 32;
                const bool ok = n < N && k < K;
#pragma unroll
                for (int j = 0; j < BITS; ++j)
                    fw_words[u][j] = ok ? a.w.qweight[(size_t)((k / 32) * BITS + j) * N + n] : 0u;
                if (ok) {
                    const size_t gi = (size_t)(k / a.w.group) * N + n;
                    fw_dq[u] = make_dq(a.w.scales[gi], a.w.zeros[gi]);
                } else {
                    fw_dq[u].scale = 0.f;
                    fw_dq[u].bias = 0.f;
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                const int idx = tid + u * THREADS;
                const int no = idx % (RT / 8), ko = idx / (RT / 8);
                const int n = r0 + no * 8, k = c0 + ko * 8;
                const bool ok = n < N && k < K;
                const int bit = k * BITS;                 // first stream bit of the 8-code chunk
                const int row = bit >> 5;
                bw_shift[u] = bit & 31;
                const int last_row = K * BITS / 32 - 1;
                const int row_hi = row + 1 > last_row ? last_row : row + 1;
                if (ok) {
                    const uint4 *p = reinterpret_cast<const uint4 *>(a.w.qweight + (size_t)row * N + n);
                    const uint4 l0 = p[0], l1 = p[1];
                    bw_lo[u][0] = l0.x; bw_lo[u][1] = l0.y; bw_lo[u][2] = l0.z; bw_lo[u][3] = l0.w;
                    bw_lo[u][4] = l1.x; bw_lo[u][5] = l1.y; bw_lo[u][6] = l1.z; bw_lo[u][7] = l1.w;
                    if (BITS == 3) {
                        const uint4 *ph = reinterpret_cast<const uint4 *>(a.w.qweight + (size_t)row_hi * N + n);
                        const uint4 h0 = ph[0], h1 = ph[1];
                        bw_hi[u][0] = h0.x; bw_hi[u][1] = h0.y; bw_hi[u][2] = h0.z; bw_hi[u][3] = h0.w;
                        bw_hi[u][4] = h1.x; bw_hi[u][5] = h1.y; bw_hi[u][6] = h1.z; bw_hi[u][7] = h1.w;
                    }
                    const size_t gi = (size_t)(k / a.w.group) * N + n;
                    const uint4 sc = *reinterpret_cast<const uint4 *>(a.w.scales + gi);
                    bw_scale[u][0] = sc.x; bw_scale[u][1] = sc.y; bw_scale[u][2] = sc.z; bw_scale[u][3] = sc.w;
                    const uint2 zz = *reinterpret_cast<const uint2 *>(a.w.zeros + gi);
                    bw_zero[u][0] = zz.x; bw_zero[u][1] = zz.y;
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) { bw_lo[u][i] = 0; bw_hi[u][i] = 0; }
#pragma unroll
                    for (int i = 0; i < 4; ++i) bw_scale[u][i] = 0;   // scale 0 -> weight 0
                    bw_zero[u][0] = bw_zero[u][1] = 0;
                }
            }
        }
    };

    auto store_tile = [&](int t) {
        const bool ext = t >= n_main;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int idx = tid + i * THREADS;
            const int row = idx / (RT / 8), ch = idx % (RT / 8);
            *reinterpret_cast<uint4 *>(As + row * LROW + ch * 8) = a_reg[i];
        }
        if (ext) {
#pragma unroll
            for (int i = 0; i < W_CH; ++i) {
                const int idx = tid + i * THREADS;
                const int row = idx / (RT / 8), ch = idx % (RT / 8);
                *reinterpret_cast<uint4 *>(Ws + row * LROW + ch * 8) = w_reg[i];
            }
            return;
        }
        if (!BWD) {
#pragma unroll
            for (int u = 0; u < FW_UNITS; ++u) {
                const int idx = tid + u * THREADS;
                const int nl = idx % CT, kb = idx / CT;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t o[4];
                    dequant_chunk<BITS>(block_chunk<BITS>(fw_words[u], j), fw_dq[u], o);
                    *reinterpret_cast<uint4 *>(Ws + nl * LROW + kb * 32 + j * 8) = make_uint4(o[0], o[1], o[2], o[3]);
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                const int idx = tid + u * THREADS;
                const int no = idx % (RT / 8), ko = idx / (RT / 8);
                uint32_t chunk[8];
                DqConst dq[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (BITS == 3)
                        chunk[i] = __builtin_amdgcn_alignbit(bw_hi[u][i], bw_lo[u][i], bw_shift[u]);
                    else
                        chunk[i] = bw_lo[u][i] >> bw_shift[u];
                    const uint16_t sb = (uint16_t)(bw_scale[u][i >> 1] >> ((i & 1) * 16));
                    const uint8_t zb = (uint8_t)(bw_zero[u][i >> 2] >> ((i & 3) * 8));
                    dq[i] = make_dq(sb, zb);
                }
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    uint32_t o[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        o[i] = pack_bf16x2(dq_value(chunk_code<BITS>(chunk[2 * i], kk), dq[2 * i]),
                                           dq_value(chunk_code<BITS>(chunk[2 * i + 1], kk), dq[2 * i + 1]));
                    *reinterpret_cast<uint4 *>(Ws + (ko * 8 + kk) * LROW + no * 8) = make_uint4(o[0], o[1], o[2], o[3]);
                }
            }
        }
    };

    // ---- accumulators ---------------------------------------------------------
    constexpr int TI = WM / 32, TJ = WN / 32;
    f32x16 acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int wm = wave / (CT / WN), wn = wave % (CT / WN);
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;

    load_tile(0);
    for (int t = 0; t < n_tiles; ++t) {
        store_tile(t);
        __syncthreads();
        if (t + 1 < n_tiles) load_tile(t + 1);
        int ksteps = RT / 16;
        if (t >= n_main) {
            const int left = a.RE - (t - n_main) * RT;
            if (left < RT) ksteps = left / 16;
        }
        for (int ks = 0; ks < ksteps; ++ks) {
            bf16x8 af[TI], bf[TJ];
#pragma unroll
            for (int i = 0; i < TI; ++i)
                af[i] = *reinterpret_cast<const bf16x8 *>(As + (wm * WM + i * 32 + frag_row) * LROW + ks * 16 + frag_k);
#pragma unroll
            for (int j = 0; j < TJ; ++j)
                bf[j] = *reinterpret_cast<const bf16x8 *>(Ws + (wn * WN + j * 32 + frag_row) * LROW + ks * 16 + frag_k);
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // ---- epilogue: one RNE to bfloat16, guarded stores --------------------------
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const int col = c0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * WM + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
                if (row < a.M && col < Cout) a.out[(size_t)row * Cout + col] = float_to_bf16_bits(acc[i][j][v]);
            }
        }
}

template <int BITS, bool BWD, int MT, int CT, int WM, int WN>
static hipError_t launch_variant(const GemmArgs &a, const char *name, hipStream_t stream) {
    const int Cout = BWD ? a.w.K : a.w.N;
    const int tiles_m = (a.M + MT - 1) / MT, tiles_c = (Cout + CT - 1) / CT;
    const int blocks = (tiles_m * tiles_c + 7) / 8 * 8;
    const size_t lds_bytes = (size_t)(MT + CT) * LROW * sizeof(uint16_t);
    auto kern = gemm_tile_kernel<BITS, BWD, MT, CT, WM, WN>;
    // raise the dynamic-LDS limit once per variant and device (not a stream operation,
    // but keep it out of the steady state and out of graph captures after the first call)
    static bool configured[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64 || !configured[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) configured[dev] = true;
    }
    prof_before(name, stream);
    kern<<<blocks, THREADS, lds_bytes, stream>>>(a, tiles_m, tiles_c);
    prof_after(stream);
    return hipGetLastError();
}

template <int BITS, bool BWD>
static hipError_t launch_bits_dir(const GemmArgs &a, hipStream_t stream) {
    const int Cout = BWD ? a.w.K : a.w.N;
    const long tiles_large = (long)((a.M + 255) / 256) * ((Cout + 255) / 256);
    if (a.M <= 32)
        return launch_variant<BITS, BWD, 32, 256, 32, 64>(a, BWD ? "gemm_bwd_32x256" : "gemm_fwd_32x256", stream);
    if (a.M <= 128 || tiles_large < 192)
        return launch_variant<BITS, BWD, 128, 256, 64, 128>(a, BWD ? "gemm_bwd_128x256" : "gemm_fwd_128x256", stream);
    return launch_variant<BITS, BWD, 256, 256, 128, 128>(a, BWD ? "gemm_bwd_256x256" : "gemm_fwd_256x256", stream);
}

hipError_t launch_gemm(const GemmArgs &a, hipStream_t stream) {
    switch (a.w.bits) {
        case 2: return a.backward ? launch_bits_dir<2, true>(a, stream) : launch_bits_dir<2, false>(a, stream);
        case 3: return a.backward ? launch_bits_dir<3, true>(a, stream) : launch_bits_dir<3, false>(a, stream);
        default: return a.backward ? launch_bits_dir<4, true>(a, stream) : launch_bits_dir<4, false>(a, stream);
    }
}

}  // namespace mlr
