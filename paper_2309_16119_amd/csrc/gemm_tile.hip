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
//     that loads the words of 4 adjacent columns holds, for each k of the chunk, 4
//     consecutive n of the MFMA operand; no transpose through LDS is needed.
//
// Scheduling.  One VALU instruction costs a SIMD 4 cycles and one 32x32x16 MFMA 32;
// they overlap when they come from different waves of the same SIMD.  The large
// variant therefore runs 8 waves (2 per SIMD) on a double-buffered LDS tile pair and
// lets the two waves of a SIMD take the two halves of a step in opposite order: one
// issues the MFMAs of tile t while the other dequantizes tile t+1, then they swap.
// The mid variant runs 4 waves with one LDS buffer and relies on two workgroups per
// CU to fill each other's gaps.
//
// The steady-state loop is branch-free: rows past M and columns past the matrix are
// clamped to valid addresses (their results are never stored), uniform address parts
// live in scalar registers, and only a ragged last contraction tile and the adapter
// extension take the predicated path.
#include <cstdlib>
#include <cstring>

#include "gemm_common.h"

namespace mlr {

constexpr int RT = 64;         // contraction elements per LDS tile
constexpr int LDS_PAD = 8;     // bf16 elements of row padding (row stride 144 B: conflict-free 16-B accesses)
constexpr int LROW = RT + LDS_PAD;

template <int BITS, bool BWD, int THREADS, int MT, int CT, int WM, int WN, int OCC>
__global__ __launch_bounds__(THREADS, OCC) void gemm_tile_kernel(GemmDev d) {
    constexpr int NWAVES = THREADS / 64;
    static_assert((MT / WM) * (CT / WN) == NWAVES, "wave grid covers the tile");
    static_assert(WM % 32 == 0 && WN == 64, "wave tile: rows in 32s, two 32-column MFMA tiles");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

    const GemmArgs &a = d.a;
    // grid is padded up to a multiple of 8 blocks; surplus blocks leave here
    const TileCoord tcoord = tile_of_block(blockIdx.x, d.tiles_m, d.tiles_c);
    if (tcoord.tm < 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const int m0 = tcoord.tm * MT, c0 = tcoord.tc * CT;
    const int K = a.w.K, N = a.w.N;
    const int C = BWD ? N : K;          // contraction length
    const int Cout = BWD ? K : N;       // output columns
    const int n_full = C / RT;          // tiles that need no predicate
    const int n_main = (C + RT - 1) / RT;
    const int n_ext = (a.RE + RT - 1) / RT;
    const int n_tiles = n_main + n_ext;

    // ---- per-thread constants of the staging pattern ---------------------------
    constexpr int A_CH = MT * (RT / 8) / THREADS;            // 16-byte activation chunks per thread
    constexpr int FW_UNITS = CT * (RT / 32) / THREADS;       // forward: (column, 32-code block) units
    constexpr int BW_UNITS = (CT / 8) * (RT / 4) / THREADS;  // backward: (4 columns n, 8 codes k) units
    constexpr int W_CH = CT * (RT / 8) / THREADS;            // 16-byte chunks of an extension W tile
    static_assert(A_CH >= 1 && (MT * (RT / 8)) % THREADS == 0, "activation tile divides");
    static_assert(FW_UNITS >= 1 && (CT * (RT / 32)) % THREADS == 0, "forward units divide");
    static_assert(BW_UNITS >= 1 && ((CT / 8) * (RT / 4)) % THREADS == 0, "backward units divide");
    static_assert(W_CH >= 1, "extension tile divides");
    static_assert(THREADS % CT == 0 || CT % THREADS == 0, "forward unit -> k-block is wave-uniform");

    // activations: uniform base (row block, tile) + per-thread byte offset
    uint32_t a_off[A_CH];       // bytes from act + m0*C: clamped row * C + chunk
    int a_col[A_CH];            // contraction offset of the chunk inside the tile
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int idx = tid + i * THREADS;
        const int row = idx / (RT / 8), ch = idx % (RT / 8);
        int m = m0 + row;
        if (m > a.M - 1) m = a.M - 1;
        a_off[i] = (uint32_t)(((size_t)(m - m0) * C + ch * 8) * 2);
        a_col[i] = ch * 8;
    }
    const uint16_t *act_rowblock = a.act + (size_t)m0 * C;

    // forward weight units
    uint32_t fw_off[BWD ? 1 : FW_UNITS];   // bytes: clamped column * 4
    uint32_t fw_n[BWD ? 1 : FW_UNITS];     // clamped column
    int fw_kb[BWD ? 1 : FW_UNITS];         // 32-code block inside the tile (wave-uniform)
    // backward weight units
    uint32_t bw_off[BWD ? BW_UNITS : 1];   // bytes from qweight row of c0: (drow * N + no*4) * 4
    uint32_t bw_offhi[BWD ? BW_UNITS : 1];
    uint32_t bw_soff[BWD ? BW_UNITS : 1];  // elements from scales/zeros row of c0's group: dgroup * N + no*4
    int bw_shift[BWD ? BW_UNITS : 1];
    bool bw_kok[BWD ? BW_UNITS : 1];
    int bw_row0 = 0, bw_g0 = 0;
    if (!BWD) {
#pragma unroll
        for (int u = 0; u < FW_UNITS; ++u) {
            const int idx = tid + u * THREADS;
            int n = c0 + idx % CT;
            if (n > N - 1) n = N - 1;
            fw_n[u] = (uint32_t)n;
            fw_off[u] = (uint32_t)n * 4u;
            fw_kb[u] = uniform(idx / CT);
        }
    } else {
        bw_row0 = (c0 * BITS) >> 5;
        bw_g0 = (int)d.group_of_block((uint32_t)(c0 >> 5));
        const int last_row = K * BITS / 32 - 1;
#pragma unroll
        for (int u = 0; u < BW_UNITS; ++u) {
            const int idx = tid + u * THREADS;
            const int no = idx % (RT / 4), ko = idx / (RT / 4);
            int k = c0 + ko * 8;
            bw_kok[u] = k < K;
            if (k > K - 8) k = K - 8;
            const int bit = k * BITS;
            const int row = bit >> 5;
            const int row_hi = row + 1 > last_row ? last_row : row + 1;
            bw_shift[u] = bit & 31;
            bw_off[u] = (uint32_t)(((size_t)(row - bw_row0) * N + no * 4) * 4);
            bw_offhi[u] = (uint32_t)(((size_t)(row_hi - bw_row0) * N + no * 4) * 4);
            const int g = (int)d.group_of_block((uint32_t)(k >> 5));
            bw_soff[u] = (uint32_t)((size_t)(g - bw_g0) * N + no * 4);
        }
    }

    // ---- register staging for one tile -------------------------------------
    uint4 a_reg[A_CH];
    uint32_t fw_words[BWD ? 1 : FW_UNITS][BITS];
    uint16_t fw_scale[BWD ? 1 : FW_UNITS];       // binary16 bits (0: block dequantizes to +0)
    uint8_t fw_zero[BWD ? 1 : FW_UNITS];
    uint4 bw_lo[BWD ? BW_UNITS : 1], bw_hi[BWD ? BW_UNITS : 1];
    uint2 bw_scale[BWD ? BW_UNITS : 1];          // 4 binary16
    uint32_t bw_zero[BWD ? BW_UNITS : 1];        // 4 uint8
    uint4 w_reg[W_CH];                           // extension tiles only

    // full main tile t: no predicates at all
    auto load_main = [&](int t) {
        const uint16_t *abase = act_rowblock + (size_t)t * RT;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) a_reg[i] = load_at<uint4>(abase, a_off[i]);
        if (!BWD) {
#pragma unroll
            for (int u = 0; u < FW_UNITS; ++u) {
                const int blk = t * (RT / 32) + fw_kb[u];
                const uint32_t *wbase = a.w.qweight + (size_t)blk * BITS * N;
#pragma unroll
                for (int j = 0; j < BITS; ++j) fw_words[u][j] = load_at<uint32_t>(wbase + (size_t)j * N, fw_off[u]);
                const size_t grow = (size_t)d.group_of_block((uint32_t)blk) * N;
                fw_scale[u] = load_at<uint16_t>(a.w.scales + grow, fw_n[u] * 2);
                fw_zero[u] = load_at<uint8_t>(a.w.zeros + grow, fw_n[u]);
            }
        } else {
            const uint32_t *wbase = a.w.qweight + (size_t)bw_row0 * N + (size_t)t * RT;
            const uint16_t *sbase = a.w.scales + (size_t)bw_g0 * N + (size_t)t * RT;
            const uint8_t *zbase = a.w.zeros + (size_t)bw_g0 * N + (size_t)t * RT;
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                bw_lo[u] = load_at<uint4>(wbase, bw_off[u]);
                if (BITS == 3) bw_hi[u] = load_at<uint4>(wbase, bw_offhi[u]);
                bw_scale[u] = load_at<uint2>(sbase, bw_soff[u] * 2);
                bw_zero[u] = load_at<uint32_t>(zbase, bw_soff[u]);
            }
        }
    };

    // ragged last main tile (C % 64 != 0) and extension tiles: predicated
    auto load_edge = [&](int t) {
        const bool ext = t >= n_main;
        const int r0 = ext ? (t - n_main) * RT : t * RT;
        const int ld = ext ? a.RE : C;
        const uint16_t *abase = (ext ? a.act_ext + (size_t)m0 * ld : act_rowblock) + r0;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int idx = tid + i * THREADS;
            const int row = idx / (RT / 8);
            int m = m0 + row;
            if (m > a.M - 1) m = a.M - 1;
            a_reg[i] = make_uint4(0, 0, 0, 0);
            if (r0 + a_col[i] < ld) a_reg[i] = load_at<uint4>(abase, (uint32_t)(((size_t)(m - m0) * ld + a_col[i]) * 2));
        }
        if (ext) {
#pragma unroll
            for (int i = 0; i < W_CH; ++i) {
                const int idx = tid + i * THREADS;
                const int row = idx / (RT / 8), ch = idx % (RT / 8);
                int c = c0 + row;
                if (c > Cout - 1) c = Cout - 1;
                const int cc = r0 + ch * 8;
                w_reg[i] = make_uint4(0, 0, 0, 0);
                if (cc < a.RE) w_reg[i] = *reinterpret_cast<const uint4 *>(a.w_ext + (size_t)c * a.RE + cc);
            }
            return;
        }
        if (!BWD) {
#pragma unroll
            for (int u = 0; u < FW_UNITS; ++u) {
                const int blk = t * (RT / 32) + fw_kb[u];
                const bool ok = blk * 32 < K;
                const int blk_c = ok ? blk : 0;
                const uint32_t *wbase = a.w.qweight + (size_t)blk_c * BITS * N;
#pragma unroll
                for (int j = 0; j < BITS; ++j) fw_words[u][j] = load_at<uint32_t>(wbase + (size_t)j * N, fw_off[u]);
                const size_t grow = (size_t)d.group_of_block((uint32_t)blk_c) * N;
                // scale bits 0 -> every weight of the block dequantizes to +0
                fw_scale[u] = ok ? load_at<uint16_t>(a.w.scales + grow, fw_n[u] * 2) : (uint16_t)0;
                fw_zero[u] = load_at<uint8_t>(a.w.zeros + grow, fw_n[u]);
            }
        } else {
            const uint32_t *wbase = a.w.qweight + (size_t)bw_row0 * N + r0;
            const uint16_t *sbase = a.w.scales + (size_t)bw_g0 * N + r0;
            const uint8_t *zbase = a.w.zeros + (size_t)bw_g0 * N + r0;
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                const int idx = tid + u * THREADS;
                const int no = idx % (RT / 4);
                const bool ok = r0 + no * 4 < N;
                bw_lo[u] = make_uint4(0, 0, 0, 0);
                bw_hi[u] = make_uint4(0, 0, 0, 0);
                bw_scale[u] = make_uint2(0, 0);
                bw_zero[u] = 0;
                if (ok) {
                    bw_lo[u] = load_at<uint4>(wbase, bw_off[u]);
                    if (BITS == 3) bw_hi[u] = load_at<uint4>(wbase, bw_offhi[u]);
                    bw_scale[u] = load_at<uint2>(sbase, bw_soff[u] * 2);
                    bw_zero[u] = load_at<uint32_t>(zbase, bw_soff[u]);
                }
            }
        }
    };

    auto store_tile = [&](bool ext, uint16_t *As, uint16_t *Ws) {
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
                const int nl = idx % CT;
                const DqConst dq = make_dq(fw_scale[u], fw_zero[u]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t o[4];
                    dequant_chunk<BITS>(block_chunk<BITS>(fw_words[u], j), dq, o);
                    *reinterpret_cast<uint4 *>(Ws + nl * LROW + fw_kb[u] * 32 + j * 8) = make_uint4(o[0], o[1], o[2], o[3]);
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                const int idx = tid + u * THREADS;
                const int no = idx % (RT / 4), ko = idx / (RT / 4);
                const uint32_t lo[4] = {bw_lo[u].x, bw_lo[u].y, bw_lo[u].z, bw_lo[u].w};
                const uint32_t hi[4] = {bw_hi[u].x, bw_hi[u].y, bw_hi[u].z, bw_hi[u].w};
                const uint32_t sc[2] = {bw_scale[u].x, bw_scale[u].y};
                uint32_t chunk[4];
                DqConst dq[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (BITS == 3)
                        chunk[i] = __builtin_amdgcn_alignbit(hi[i], lo[i], bw_shift[u]);
                    else
                        chunk[i] = lo[i] >> bw_shift[u];
                    const uint16_t sb = bw_kok[u] ? (uint16_t)(sc[i >> 1] >> ((i & 1) * 16)) : (uint16_t)0;
                    const uint8_t zb = (uint8_t)(bw_zero[u] >> (i * 8));
                    dq[i] = make_dq(sb, zb);
                }
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    uint32_t o[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        o[i] = pack_bf16x2(dq_value(chunk_code<BITS>(chunk[2 * i], kk), dq[2 * i]),
                                           dq_value(chunk_code<BITS>(chunk[2 * i + 1], kk), dq[2 * i + 1]));
                    *reinterpret_cast<uint2 *>(Ws + (ko * 8 + kk) * LROW + no * 4) = make_uint2(o[0], o[1]);
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
    const int a_frag_off = (wm * WM + frag_row) * LROW + frag_k;
    const int w_frag_off = (wn * WN + frag_row) * LROW + frag_k;

    struct Frags {
        bf16x8 af[TI], bf[TJ];
    };
    auto load_frags = [&](Frags &f, const uint16_t *As, const uint16_t *Ws, int ks) {
#pragma unroll
        for (int i = 0; i < TI; ++i)
            f.af[i] = *reinterpret_cast<const bf16x8 *>(As + a_frag_off + i * 32 * LROW + ks * 16);
#pragma unroll
        for (int j = 0; j < TJ; ++j)
            f.bf[j] = *reinterpret_cast<const bf16x8 *>(Ws + w_frag_off + j * 32 * LROW + ks * 16);
    };
    auto mfma_frags = [&](const Frags &f) {
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int j = 0; j < TJ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.af[i], f.bf[j], acc[i][j], 0, 0, 0);
    };

    // a full 64-deep tile.  Fragments are fetched per 16-deep step; the second wave of
    // the SIMD covers the LDS latency, and keeping one set of fragments live (instead of
    // prefetching the next) keeps the kernel under 256 registers without live-range splits.
    auto mfma_full = [&](const uint16_t *As, const uint16_t *Ws) {
#pragma unroll
        for (int ks = 0; ks < RT / 16; ++ks) {
            Frags f;
            load_frags(f, As, Ws, ks);
            mfma_frags(f);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- steady state: full main tiles only, no predicates -----------------------
    uint16_t *const As0 = lds, *const Ws0 = lds + MT * LROW;
    if (n_full > 0) {
        load_main(0);
        for (int t = 0; t < n_full; ++t) {
            store_tile(false, As0, Ws0);
            __syncthreads();
            load_main(t + 1 < n_full ? t + 1 : n_full - 1);
            mfma_full(As0, Ws0);
            __syncthreads();
        }
    }

    // ---- tail: a ragged last main tile and the adapter extension, one at a time ----
    for (int t = n_full; t < n_tiles; ++t) {
        const bool ext = t >= n_main;
        load_edge(t);
        store_tile(ext, As0, Ws0);
        __syncthreads();
        int ksteps = RT / 16;
        if (ext) {
            ksteps = (a.RE - (t - n_main) * RT) / 16;
            if (ksteps > RT / 16) ksteps = RT / 16;
        }
        for (int ks = 0; ks < ksteps; ++ks) {
            Frags f;
            load_frags(f, As0, Ws0, ks);
            mfma_frags(f);
        }
        __syncthreads();
    }

    // ---- epilogue: one RNE to bfloat16; 32x64 patches go through LDS so that the
    // global stores are 16 bytes per lane and 128 contiguous bytes per row ----------
    uint16_t *patch = lds + wave * (32 * LROW);        // per-wave [32][LROW]
#pragma unroll
    for (int i = 0; i < TI; ++i) {
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int prow = 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
                patch[prow * LROW + j * 32 + (lane & 31)] = float_to_bf16_bits(acc[i][j][v]);
            }
        // the patch is private to the wave: a wave-level wait is enough
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int idx = lane + q * 64;            // 256 chunks of 16 bytes: 32 rows x 8
            const int prow = idx / 8, ch = idx % 8;
            const uint4 v = *reinterpret_cast<const uint4 *>(patch + prow * LROW + ch * 8);
            const int row = m0 + wm * WM + i * 32 + prow;
            const int col = c0 + wn * WN + ch * 8;
            if (row < a.M && col < Cout) *reinterpret_cast<uint4 *>(a.out + (size_t)row * Cout + col) = v;
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_wave_barrier();
    }
}

template <int BITS, bool BWD, int THREADS, int MT, int CT, int WM, int WN, int OCC>
static hipError_t launch_variant(const GemmArgs &a, const char *name, hipStream_t stream) {
    const GemmDev d = make_gemm_dev(a, MT, CT);
    const int blocks = (d.tiles_m * d.tiles_c + 7) / 8 * 8;
    const size_t lds_bytes = (size_t)(MT + CT) * LROW * sizeof(uint16_t);
    static_assert((size_t)(MT + CT) >= (size_t)(THREADS / 64) * 32, "epilogue patches fit");
    auto kern = gemm_tile_kernel<BITS, BWD, THREADS, MT, CT, WM, WN, OCC>;
    static bool configured[64] = {};
    const hipError_t e = ensure_lds_limit(reinterpret_cast<const void *>(kern), lds_bytes, configured);
    if (e != hipSuccess) return e;
    prof_before(name, stream);
    kern<<<blocks, THREADS, lds_bytes, stream>>>(d);
    prof_after(stream);
    return hipGetLastError();
}

// Tile variants.  `pick` may be forced with the environment variable MODULORA_TILE
// (big | mid | small), a tuning knob for benchmarks.
enum TilePick { PICK_AUTO = 0, PICK_BIG, PICK_MID, PICK_SMALL };

static TilePick forced_pick() {
    static int cached = -1;
    if (cached < 0) {
        const char *e = std::getenv("MODULORA_TILE");
        cached = PICK_AUTO;
        if (e) {
            if (!std::strcmp(e, "big")) cached = PICK_BIG;
            else if (!std::strcmp(e, "mid")) cached = PICK_MID;
            else if (!std::strcmp(e, "small")) cached = PICK_SMALL;
        }
    }
    return (TilePick)cached;
}

template <int BITS, bool BWD>
static hipError_t launch_bits_dir(const GemmArgs &a, hipStream_t stream) {
    const int Cout = BWD ? a.w.K : a.w.N;
    TilePick pick = forced_pick();
    if (pick == PICK_AUTO) {
        const long tiles_big = (long)((a.M + 255) / 256) * ((Cout + 255) / 256);
        const long tiles_mid = (long)((a.M + 255) / 256) * ((Cout + 127) / 128);
        if (a.M <= 32) pick = PICK_SMALL;
        else {
            // rounds of 256 CUs; a mid tile costs about half a big one
            const double cost_big = (double)((tiles_big + 255) / 256);
            const double cost_mid = 0.5 * (double)((tiles_mid + 255) / 256) * 1.1;
            pick = cost_big <= cost_mid ? PICK_BIG : PICK_MID;
        }
    }
    switch (pick) {
        case PICK_SMALL:
            return launch_variant<BITS, BWD, 256, 32, 256, 32, 64, 1>(
                a, BWD ? "gemm_bwd_32x256" : "gemm_fwd_32x256", stream);
        case PICK_MID:
            return launch_variant<BITS, BWD, 256, 256, 128, 128, 64, 2>(
                a, BWD ? "gemm_bwd_256x128" : "gemm_fwd_256x128", stream);
        default:
            return launch_gemm_big(a, stream);
    }
}

hipError_t launch_gemm(const GemmArgs &a, hipStream_t stream) {
    switch (a.w.bits) {
        case 2: return a.backward ? launch_bits_dir<2, true>(a, stream) : launch_bits_dir<2, false>(a, stream);
        case 3: return a.backward ? launch_bits_dir<3, true>(a, stream) : launch_bits_dir<3, false>(a, stream);
        default: return a.backward ? launch_bits_dir<4, true>(a, stream) : launch_bits_dir<4, false>(a, stream);
    }
}

}  // namespace mlr
