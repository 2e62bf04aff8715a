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
// Scheduling.  One VALU instruction costs a SIMD about 4 cycles and one 32x32x16 MFMA 32;
// they overlap when they come from different waves of the same SIMD, or when a wave issues
// independent VALU work after an MFMA.  The 256x256 variant lives in gemm_big.hip.  The
// variants of this file are: a single-buffered one (256x128 with two workgroups per CU
// filling each other's gaps) and pipelined ones for grids of
// about one tile per CU, where nothing else hides latency: register stages filled several
// tiles ahead, two LDS buffers with one barrier per tile, the dequantization of the next
// tile issued between the MFMA steps of the current one, and optionally 8 waves that split
// the 16-deep steps of each tile between k-groups (two waves per SIMD on a small tile).
//
// The steady-state loop is branch-free: rows past M and columns past the matrix are
// clamped to valid addresses (their results are never stored), uniform address parts
// live in scalar registers, and only a ragged last contraction tile and the adapter
// extension take the predicated path.
#include <cstdlib>
#include <cstring>

#include "gemm_common.h"

namespace mlr {

constexpr int LDS_PAD = 8;     // bf16 elements of row padding (row stride 144 or 272 B: conflict-free 16-B accesses)

typedef uint32_t tu32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t tu32x4 __attribute__((ext_vector_type(4)));

// Loads issued from inline assembly (wave-uniform base + per-lane byte offset) for the
// pipelined variants.  The compiler does not track them: a consumer must sit behind
// wait_vm<N>() followed by tie() of every destination register.  Loads return in order,
// so waiting until at most N remain outstanding completes everything issued before the
// N most recent ones.
namespace tl {
__device__ __forceinline__ void ld(uint32_t &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void ld_u16(uint32_t &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_ushort %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void ld_u8(uint32_t &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_ubyte %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void ld(tu32x2 &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void ld(tu32x4 &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
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
}  // namespace tl

// RT: contraction elements per LDS tile (64 or 128).  KG: wave groups that split the 16-deep
// steps of every tile between them (their accumulators are added through LDS at the end).
template <int BITS, bool BWD, int THREADS, int MT, int CT, int WM, int WN, int OCC, int PF, int RT, int KG>
__global__ __launch_bounds__(THREADS, OCC) void gemm_tile_kernel(GemmDev d) {
    constexpr int LROW = RT + LDS_PAD;
    constexpr int NWAVES = THREADS / 64;
    constexpr int GWAVES = NWAVES / KG;      // waves of one k-group: they tile the MT x CT output
    static_assert((MT / WM) * (CT / WN) == GWAVES && GWAVES * KG == NWAVES, "wave grid covers the tile");
    constexpr int KS_LOCAL = (RT / 16) / KG;   // 16-deep steps of a tile that one wave takes: ks = i * KG + kg
    static_assert((KG == 1 || KG == 2) && (RT / 16) % KG == 0 && (KS_LOCAL == 2 || KS_LOCAL == 4 || KS_LOCAL == 8),
                  "k-steps divide between the groups");
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
    // Weight staging units of a tile: forward (column, 32-code block), backward (4 columns n,
    // 8 codes k).  With fewer units than threads only the first FW_N (BW_N) threads dequantize
    // and store; the others issue the same loads again (so that every wave has the same
    // number of loads in flight) and drop them.
    constexpr int FW_N = CT * (RT / 32), BW_N = (CT / 8) * (RT / 4);
    constexpr int FW_UNITS = FW_N >= THREADS ? FW_N / THREADS : 1;
    constexpr int BW_UNITS = BW_N >= THREADS ? BW_N / THREADS : 1;
    const bool w_active = tid < (BWD ? BW_N : FW_N);
    constexpr int W_CH = CT * (RT / 8) / THREADS;            // 16-byte chunks of an extension W tile
    static_assert(A_CH >= 1 && (MT * (RT / 8)) % THREADS == 0, "activation tile divides");
    static_assert(FW_N % THREADS == 0 || THREADS % FW_N == 0, "forward units divide");
    static_assert(BW_N % THREADS == 0 || THREADS % BW_N == 0, "backward units divide");
    static_assert(FW_N % 64 == 0 && BW_N % 64 == 0, "the staging threads are whole waves");
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
            const int idx = (tid + u * THREADS) % FW_N;
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
            const int idx = (tid + u * THREADS) % BW_N;
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
    struct Stage {
        tu32x4 a_reg[A_CH];
        uint32_t fw_words[BWD ? 1 : FW_UNITS][BITS];
        uint32_t fw_scale[BWD ? 1 : FW_UNITS];       // binary16 bits (0: block dequantizes to +0)
        uint32_t fw_zero[BWD ? 1 : FW_UNITS];
        tu32x4 bw_lo[BWD ? BW_UNITS : 1], bw_hi[BWD ? BW_UNITS : 1];
        tu32x2 bw_scale[BWD ? BW_UNITS : 1];         // 4 binary16
        uint32_t bw_zero[BWD ? BW_UNITS : 1];        // 4 uint8
    };
    // load instructions one stage issues through load_main_async
    constexpr int STAGE_LOADS = A_CH + (BWD ? BW_UNITS * (BITS == 3 ? 4 : 3) : FW_UNITS * (BITS + 2));
    uint4 w_reg[W_CH];                               // extension tiles only

    // full main tile t: no predicates at all
    auto load_main = [&](Stage &st, int t) {
        const uint16_t *abase = act_rowblock + (size_t)t * RT;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) st.a_reg[i] = load_at<tu32x4>(abase, a_off[i]);
        if (!BWD) {
#pragma unroll
            for (int u = 0; u < FW_UNITS; ++u) {
                const int blk = t * (RT / 32) + fw_kb[u];
                const uint32_t *wbase = a.w.qweight + (size_t)blk * BITS * N;
#pragma unroll
                for (int j = 0; j < BITS; ++j) st.fw_words[u][j] = load_at<uint32_t>(wbase + (size_t)j * N, fw_off[u]);
                const size_t grow = (size_t)d.group_of_block((uint32_t)blk) * N;
                st.fw_scale[u] = load_at<uint16_t>(a.w.scales + grow, fw_n[u] * 2);
                st.fw_zero[u] = load_at<uint8_t>(a.w.zeros + grow, fw_n[u]);
            }
        } else {
            const uint32_t *wbase = a.w.qweight + (size_t)bw_row0 * N + (size_t)t * RT;
            const uint16_t *sbase = a.w.scales + (size_t)bw_g0 * N + (size_t)t * RT;
            const uint8_t *zbase = a.w.zeros + (size_t)bw_g0 * N + (size_t)t * RT;
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                st.bw_lo[u] = load_at<tu32x4>(wbase, bw_off[u]);
                if (BITS == 3) st.bw_hi[u] = load_at<tu32x4>(wbase, bw_offhi[u]);
                st.bw_scale[u] = load_at<tu32x2>(sbase, bw_soff[u] * 2);
                st.bw_zero[u] = load_at<uint32_t>(zbase, bw_soff[u]);
            }
        }
    };

    // the same loads, issued from assembly (exactly STAGE_LOADS instructions) and left in flight
    auto load_main_async = [&](Stage &st, int t) {
        const uint16_t *abase = act_rowblock + (size_t)t * RT;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) tl::ld(st.a_reg[i], abase, a_off[i]);
        if (!BWD) {
#pragma unroll
            for (int u = 0; u < FW_UNITS; ++u) {
                const int blk = t * (RT / 32) + fw_kb[u];
                const uint32_t *wbase = a.w.qweight + (size_t)blk * BITS * N;
#pragma unroll
                for (int j = 0; j < BITS; ++j) tl::ld(st.fw_words[u][j], wbase + (size_t)j * N, fw_off[u]);
                const size_t grow = (size_t)d.group_of_block((uint32_t)blk) * N;
                tl::ld_u16(st.fw_scale[u], a.w.scales + grow, fw_n[u] * 2);
                tl::ld_u8(st.fw_zero[u], a.w.zeros + grow, fw_n[u]);
            }
        } else {
            const uint32_t *wbase = a.w.qweight + (size_t)bw_row0 * N + (size_t)t * RT;
            const uint16_t *sbase = a.w.scales + (size_t)bw_g0 * N + (size_t)t * RT;
            const uint8_t *zbase = a.w.zeros + (size_t)bw_g0 * N + (size_t)t * RT;
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                tl::ld(st.bw_lo[u], wbase, bw_off[u]);
                if (BITS == 3) tl::ld(st.bw_hi[u], wbase, bw_offhi[u]);
                tl::ld(st.bw_scale[u], sbase, bw_soff[u] * 2);
                tl::ld(st.bw_zero[u], zbase, bw_soff[u]);
            }
        }
    };
    // make every register of a stage depend on the wait that precedes this call
    auto tie_stage = [&](Stage &st) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) tl::tie(st.a_reg[i]);
        if (!BWD) {
#pragma unroll
            for (int u = 0; u < FW_UNITS; ++u) {
#pragma unroll
                for (int j = 0; j < BITS; ++j) tl::tie(st.fw_words[u][j]);
                tl::tie(st.fw_scale[u]);
                tl::tie(st.fw_zero[u]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                tl::tie(st.bw_lo[u]);
                if (BITS == 3) tl::tie(st.bw_hi[u]);
                tl::tie(st.bw_scale[u]);
                tl::tie(st.bw_zero[u]);
            }
        }
    };

    // ragged last main tile (C % 64 != 0) and extension tiles: predicated
    auto load_edge = [&](Stage &st, int t) {
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
            st.a_reg[i] = tu32x4{0, 0, 0, 0};
            if (r0 + a_col[i] < ld) st.a_reg[i] = load_at<tu32x4>(abase, (uint32_t)(((size_t)(m - m0) * ld + a_col[i]) * 2));
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
                for (int j = 0; j < BITS; ++j) st.fw_words[u][j] = load_at<uint32_t>(wbase + (size_t)j * N, fw_off[u]);
                const size_t grow = (size_t)d.group_of_block((uint32_t)blk_c) * N;
                // scale bits 0 -> every weight of the block dequantizes to +0
                st.fw_scale[u] = ok ? (uint32_t)load_at<uint16_t>(a.w.scales + grow, fw_n[u] * 2) : 0u;
                st.fw_zero[u] = load_at<uint8_t>(a.w.zeros + grow, fw_n[u]);
            }
        } else {
            const uint32_t *wbase = a.w.qweight + (size_t)bw_row0 * N + r0;
            const uint16_t *sbase = a.w.scales + (size_t)bw_g0 * N + r0;
            const uint8_t *zbase = a.w.zeros + (size_t)bw_g0 * N + r0;
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                const int idx = (tid + u * THREADS) % BW_N;
                const int no = idx % (RT / 4);
                const bool ok = r0 + no * 4 < N;
                st.bw_lo[u] = tu32x4{0, 0, 0, 0};
                st.bw_hi[u] = tu32x4{0, 0, 0, 0};
                st.bw_scale[u] = tu32x2{0, 0};
                st.bw_zero[u] = 0;
                if (ok) {
                    st.bw_lo[u] = load_at<tu32x4>(wbase, bw_off[u]);
                    if (BITS == 3) st.bw_hi[u] = load_at<tu32x4>(wbase, bw_offhi[u]);
                    st.bw_scale[u] = load_at<tu32x2>(sbase, bw_soff[u] * 2);
                    st.bw_zero[u] = load_at<uint32_t>(zbase, bw_soff[u]);
                }
            }
        }
    };

    // Store one staged tile into LDS in four parts (part 0..3), so that the parts can be
    // interleaved with the MFMA steps of the tile before it.  part < 0 stores everything.
    auto store_tile = [&](const Stage &st, bool ext, uint16_t *As, uint16_t *Ws, int part) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            if (part >= 0 && (A_CH >= 4 ? i / (A_CH / 4) : (i == 0 ? 0 : 2 * i)) != part) continue;
            const int idx = tid + i * THREADS;
            const int row = idx / (RT / 8), ch = idx % (RT / 8);
            *reinterpret_cast<tu32x4 *>(As + row * LROW + ch * 8) = st.a_reg[i];
        }
        if (ext) {
            if (part > 0) return;
#pragma unroll
            for (int i = 0; i < W_CH; ++i) {
                const int idx = tid + i * THREADS;
                const int row = idx / (RT / 8), ch = idx % (RT / 8);
                *reinterpret_cast<uint4 *>(Ws + row * LROW + ch * 8) = w_reg[i];
            }
            return;
        }
        if (!w_active) return;
        if (!BWD) {
#pragma unroll
            for (int u = 0; u < FW_UNITS; ++u) {
                const int idx = (tid + u * THREADS) % FW_N;
                const int nl = idx % CT;
                const DqConst dq = make_dq((uint16_t)st.fw_scale[u], (uint8_t)st.fw_zero[u]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (part >= 0 && j != part) continue;
                    uint32_t o[4];
                    dequant_chunk<BITS>(block_chunk<BITS>(st.fw_words[u], j), dq, o);
                    *reinterpret_cast<uint4 *>(Ws + nl * LROW + fw_kb[u] * 32 + j * 8) = make_uint4(o[0], o[1], o[2], o[3]);
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < BW_UNITS; ++u) {
                const int idx = (tid + u * THREADS) % BW_N;
                const int no = idx % (RT / 4), ko = idx / (RT / 4);
                const uint32_t lo[4] = {st.bw_lo[u][0], st.bw_lo[u][1], st.bw_lo[u][2], st.bw_lo[u][3]};
                const uint32_t hi[4] = {st.bw_hi[u][0], st.bw_hi[u][1], st.bw_hi[u][2], st.bw_hi[u][3]};
                const uint32_t sc[2] = {st.bw_scale[u][0], st.bw_scale[u][1]};
                uint32_t chunk[4];
                DqConst dq[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (BITS == 3)
                        chunk[i] = __builtin_amdgcn_alignbit(hi[i], lo[i], bw_shift[u]);
                    else
                        chunk[i] = lo[i] >> bw_shift[u];
                    const uint16_t sb = bw_kok[u] ? (uint16_t)(sc[i >> 1] >> ((i & 1) * 16)) : (uint16_t)0;
                    const uint8_t zb = (uint8_t)(st.bw_zero[u] >> (i * 8));
                    dq[i] = make_dq(sb, zb);
                }
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    if (part >= 0 && kk / 2 != part) continue;
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

    const int kg = wave / GWAVES, gw = wave % GWAVES;   // k-group, wave inside the group
    const int wm = gw / (CT / WN), wn = gw % (CT / WN);
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
        for (int i = 0; i < KS_LOCAL; ++i) {
            Frags f;
            load_frags(f, As, Ws, i * KG + kg);
            mfma_frags(f);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- steady state: full main tiles only, no predicates -----------------------
    uint16_t *const As0 = lds, *const Ws0 = lds + MT * LROW;
    constexpr int NST = PF > 0 ? PF : 1;
    Stage stg[NST];
    if (PF == 0) {
        // single LDS buffer, loads one tile ahead
        if (n_full > 0) {
            load_main(stg[0], 0);
            for (int t = 0; t < n_full; ++t) {
                store_tile(stg[0], false, As0, Ws0, -1);
                __syncthreads();
                load_main(stg[0], t + 1 < n_full ? t + 1 : n_full - 1);
                mfma_full(As0, Ws0);
                __syncthreads();
            }
        }
    } else if (n_full > 0) {
        // Two LDS buffers and PF register stages: global loads run PF tiles ahead (issued from
        // assembly, awaited with exact counts), and the dequantization of tile t+1 into the
        // other LDS buffer is issued in four parts between the MFMA steps of tile t (the matrix
        // cores work while the wave issues VALU work).  One barrier per tile: before it,
        // everyone has read buffer t&1 and written the other.
        static_assert(PF == 0 || (PF >= 2 && PF <= 4), "pipelined variants keep 2..4 stages");
        constexpr int BUF = (MT + CT) * LROW;
        constexpr int SL = STAGE_LOADS;
        // wait until the stage that was followed by `later` younger stages has landed
        auto wait_stage = [&](Stage &st, int later) {
            if (NST >= 4 && later >= 3) tl::wait_vm<(3 * SL < 64 ? 3 * SL : 0)>();
            else if (NST >= 3 && later == 2) tl::wait_vm<(2 * SL < 64 ? 2 * SL : 0)>();
            else if (later == 1) tl::wait_vm<(SL < 64 ? SL : 0)>();
            else tl::wait_vm<0>();
            tie_stage(st);
        };
#pragma unroll
        for (int dd = 0; dd < NST; ++dd)
            if (dd < n_full) load_main_async(stg[dd], dd);
        wait_stage(stg[0], n_full - 1 < NST - 1 ? n_full - 1 : NST - 1);
        store_tile(stg[0], false, As0, Ws0, -1);
        __syncthreads();
        for (int t = 0; t < n_full; t += NST) {
#pragma unroll
            for (int dd = 0; dd < NST; ++dd) {
                const int tt = t + dd;
                if (tt < n_full) {
                    const uint16_t *Ac = As0 + (tt & 1) * BUF, *Wc = Ws0 + (tt & 1) * BUF;
                    uint16_t *An = As0 + ((tt + 1) & 1) * BUF, *Wn = Ws0 + ((tt + 1) & 1) * BUF;
                    const bool has_next = tt + 1 < n_full;
                    // tile tt already sits in LDS: its stage takes the loads of tile tt + PF
                    if (tt + NST < n_full) load_main_async(stg[dd], tt + NST);
                    Frags f[2];
                    load_frags(f[0], Ac, Wc, kg);
#pragma unroll
                    for (int i = 0; i < KS_LOCAL; ++i) {
                        if (i + 1 < KS_LOCAL) load_frags(f[(i + 1) & 1], Ac, Wc, (i + 1) * KG + kg);
                        mfma_frags(f[i & 1]);
                        if (has_next) {
                            Stage &nx = stg[(dd + 1) % NST];
                            if (i == 0) {
                                const int younger = n_full - tt - 2;   // stages issued after nx
                                wait_stage(nx, younger < NST - 1 ? younger : NST - 1);
                            }
                            // the four parts of the next tile, spread over this wave's steps
                            if (KS_LOCAL >= 4) {
                                if (i % (KS_LOCAL / 4) == 0) store_tile(nx, false, An, Wn, i / (KS_LOCAL / 4));
                            } else {
#pragma unroll
                                for (int pp = 0; pp < 4 / KS_LOCAL; ++pp) store_tile(nx, false, An, Wn, i * (4 / KS_LOCAL) + pp);
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    __syncthreads();
                }
            }
        }
    }

    // ---- tail: a ragged last main tile and the adapter extension, one at a time ----
    for (int t = n_full; t < n_tiles; ++t) {
        const bool ext = t >= n_main;
        load_edge(stg[0], t);
        store_tile(stg[0], ext, As0, Ws0, -1);
        __syncthreads();
        int ksteps = RT / 16;
        if (ext) {
            ksteps = (a.RE - (t - n_main) * RT) / 16;
            if (ksteps > RT / 16) ksteps = RT / 16;
        }
        for (int ks = kg; ks < ksteps; ks += KG) {
            Frags f;
            load_frags(f, As0, Ws0, ks);
            mfma_frags(f);
        }
        __syncthreads();
    }

    // ---- the k-groups' accumulators meet in LDS; group 0 carries on alone -------------
    if (KG > 1) {
        float *redbuf = reinterpret_cast<float *>(lds);      // [kg - 1][gw][i][j][v][lane]
        constexpr int GROUP_FLOATS = GWAVES * TI * TJ * 16 * 64;   // = MT * CT
        if (kg > 0) {
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        redbuf[(kg - 1) * GROUP_FLOATS + (((gw * TI + i) * TJ + j) * 16 + v) * 64 + lane] = acc[i][j][v];
        }
        __syncthreads();
        if (kg != 0) return;
#pragma unroll
        for (int g = 0; g < KG - 1; ++g)
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[i][j][v] += redbuf[g * GROUP_FLOATS + (((gw * TI + i) * TJ + j) * 16 + v) * 64 + lane];
        // group 0's waves now reuse the same LDS for their patches: wait for each other's reads
        __syncthreads();
    }

    // ---- epilogue: one RNE to bfloat16; 32x64 patches go through LDS so that the
    // global stores are 16 bytes per lane and 128 contiguous bytes per row ----------
    uint16_t *patch = lds + gw * (32 * LROW);          // per-wave [32][LROW]
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

template <int BITS, bool BWD, int THREADS, int MT, int CT, int WM, int WN, int OCC, int PF, int RT = 64, int KG = 1>
static hipError_t launch_variant(const GemmArgs &a, const char *name, hipStream_t stream) {
    constexpr int LROW = RT + LDS_PAD;
    static_assert(KG == 1 || (size_t)(KG - 1) * MT * CT * 4 <= (size_t)(PF > 0 ? 2 : 1) * (MT + CT) * LROW * 2, "k-group partials fit");
    const GemmDev d = make_gemm_dev(a, MT, CT);
    const int blocks = (d.tiles_m * d.tiles_c + 7) / 8 * 8;
    size_t lds_bytes = (size_t)(PF > 0 ? 2 : 1) * (MT + CT) * LROW * sizeof(uint16_t);
    // With no more workgroups than CUs, ask for more than half of a CU's 160 KB of LDS: the
    // dispatcher then cannot put two workgroups on one CU while another CU stays empty.
    if (blocks <= 256 && lds_bytes < 81 * 1024) lds_bytes = 81 * 1024;
    static_assert((size_t)(MT + CT) >= (size_t)(THREADS / 64 / KG) * 32, "epilogue patches fit");
    auto kern = gemm_tile_kernel<BITS, BWD, THREADS, MT, CT, WM, WN, OCC, PF, RT, KG>;
    static bool configured[64] = {};
    const hipError_t e = ensure_lds_limit(reinterpret_cast<const void *>(kern), lds_bytes, configured);
    if (e != hipSuccess) return e;
    launch_kernel(name, kern, blocks, THREADS, lds_bytes, stream, d);
    return hipGetLastError();
}

// Tile variants.  `pick` may be forced with the environment variable MODULORA_TILE
// (big | mid | m128 | m64 | m64k | t128s), a tuning knob for benchmarks.  Every variant
// listed is one the automatic choice below can reach.
enum TilePick { PICK_AUTO = 0, PICK_BIG, PICK_MID, PICK_M128, PICK_M64, PICK_M64K, PICK_T128S };

static TilePick forced_pick() {
    static int cached = -1;
    if (cached < 0) {
        const char *e = std::getenv("MODULORA_TILE");
        cached = PICK_AUTO;
        if (e) {
            if (!std::strcmp(e, "big")) cached = PICK_BIG;
            else if (!std::strcmp(e, "mid")) cached = PICK_MID;
            else if (!std::strcmp(e, "m128")) cached = PICK_M128;
            else if (!std::strcmp(e, "m64")) cached = PICK_M64;
            else if (!std::strcmp(e, "m64k")) cached = PICK_M64K;
            else if (!std::strcmp(e, "t128s")) cached = PICK_T128S;
        }
    }
    return (TilePick)cached;
}

template <int BITS, bool BWD>
static hipError_t launch_bits_dir(const GemmArgs &a, hipStream_t stream) {
    const int Cout = BWD ? a.w.K : a.w.N;
    TilePick pick = forced_pick();
    if (pick == PICK_AUTO) {
        {   // (any token count: a 32-row tile kernel for M <= 32 measured 1.2 us per step, more than any of these)
            // Estimated time of the whole grid in microseconds, from measured times of one 64-deep
            // contraction step of each variant: alone on a CU (t1) and sharing it with a second
            // workgroup (t2), times how often the 256 CUs (x occupancy) are refilled.  The 256 x 256
            // kernel cuts the tiles of its last, partial round into slices of the contraction
            // (BigPlan); that round then costs 1/split of a round plus the traffic of the partial
            // tiles (written once, read once) and one more launch.
            struct Variant { TilePick pick; int mt, ct, occ; double t1, t2; };
            const Variant vs[5] = {{PICK_MID, 256, 128, 2, 1.46, 1.95},
                                   {PICK_M128, 128, 128, 2, 0.97, 1.40},
                                   {PICK_M64, 64, 128, 2, 0.75, 1.10},
                                   {PICK_M64K, 64, 128, 1, 0.62, 0.62},
                                   {PICK_T128S, 128, 64, 1, 0.48, 0.48}};   // gemm_mid.hip
            const int C = BWD ? a.w.N : a.w.K;
            const double steps = (double)C / 64.0;
            const BigPlan bp = big_plan(a.M, C, Cout);
            double best = ((double)(bp.full / 256) + (bp.tail ? 1.0 / bp.split : 0.0)) * (bp.mt == 128 ? 1.0 : 1.83) * steps;
            if (bp.split > 1) best += (bp.mt == 128 ? 12.0 : 9.0) + (double)bp.partial_bytes() / 4.0e6;
            pick = PICK_BIG;
            for (const Variant &v : vs) {
                const long tiles = (long)((a.M + v.mt - 1) / v.mt) * ((Cout + v.ct - 1) / v.ct);
                const double cost = steps * (tiles <= 256 ? v.t1 : (double)((tiles + 256 * v.occ - 1) / (256 * v.occ)) * v.t2);
                if (cost < best) { best = cost; pick = v.pick; }
            }
        }
    }
    switch (pick) {
        case PICK_MID:
            return launch_variant<BITS, BWD, 256, 256, 128, 128, 64, 2, 0>(
                a, BWD ? "gemm_bwd_256x128" : "gemm_fwd_256x128", stream);
        case PICK_M128:
            return launch_variant<BITS, BWD, 256, 128, 128, 64, 64, 2, 2>(
                a, BWD ? "gemm_bwd_128x128" : "gemm_fwd_128x128", stream);
        case PICK_M64:
            return launch_variant<BITS, BWD, 256, 64, 128, 32, 64, 2, 3>(
                a, BWD ? "gemm_bwd_64x128" : "gemm_fwd_64x128", stream);
        case PICK_M64K:   // 8 waves: two k-groups of 4 share every 128-deep tile
            return launch_variant<BITS, BWD, 512, 64, 128, 32, 64, 1, 3, 128, 2>(
                a, BWD ? "gemm_bwd_64x128k" : "gemm_fwd_64x128k", stream);
        case PICK_T128S:  // 8 waves: four consumers (k-groups of one 128x64 wave tile) and four producers
            return launch_gemm_mid(a, stream);
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
