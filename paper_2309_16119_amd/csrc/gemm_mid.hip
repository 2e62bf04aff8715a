// The fused dequantize + bf16 MFMA tile kernel for grids of about one 128 x 64 tile per
// compute unit (a few hundred tokens against a 4096-wide layer).  Same mathematics as
// gemm_tile.hip (ModuLoRA Figure 1: forward X What^T and backward dY What with What
// re-materialized from the packed codes, plus the adapter term of eq. (3) as an extended
// contraction).  A second instantiation (F16) serves the layer in the paper's own storage
// convention: binary16 activations and outputs, What = binary16(fma(q, scale, z)) with a binary16
// zero point that is added, f16 MFMAs, and the adapter term and the bias added in the epilogue.
//
// With one small tile per CU every 128-deep step holds only 16 MFMAs per SIMD, and in a
// kernel where every wave fetches, dequantizes, stores, synchronizes and multiplies in
// turn the costs of a step add up instead of overlapping (measured on the 8-wave k-group
// variant of gemm_tile.hip: taking out the activation stores, the dequantization or the
// loads each shortened the kernel by its own share, taking out the MFMAs changed nothing).
// Here the waves are specialized instead (12 waves, three per SIMD, one of each kind):
//
//   - waves 0-3 are consumers: each owns half of the tile's rows (64 x 64) for half of every
//     128-deep step (four 16-deep MFMA steps); they read fragments and issue MFMAs, nothing
//     else.  The two halves of the contraction are added through LDS at the end.
//   - waves 4-7 dequantize: a thread fetches the packed words, scale and zero point of one
//     32-code unit four steps ahead into registers (three sets) and writes the unit's 32
//     bfloat16 into the weight tile of the next step.
//   - waves 8-11 only send the direct global->LDS loads of the activation tile, three steps
//     ahead into a ring of four tiles.  A step is shorter than a trip to memory, hence the
//     distances.
//   - one barrier per step hands the buffers over.  LDS rows are 256 bytes (one line of the
//     64 banks) with the 16-byte chunk index XOR-ed with row & 15: fragment reads, weight
//     stores and direct loads are all conflict-free.
//   - measured with stamps from instrumented builds: a consumer needs ~900 cycles per step (300
//     until its fragments are there, 560 for 16 MFMAs), a dequantizing wave ~900 (120 VALU
//     instructions, 4 LDS stores) plus ~250 to get its five loads accepted; loads issued right
//     after the barrier, ahead of other work of the same wave, held that wave up for 600 cycles.
//     Fetching the raw weight data with a handful of wide direct loads into an LDS staging ring
//     (instead of 20 narrow register loads per step) was slower, not faster: the dequantization
//     then starts with a round trip to LDS after every barrier.
//   - what bounds a step now is LDS store bandwidth: stores reach LDS at ~80 bytes per clock and
//     CU whatever their width (direct loads included; reads get ~240), and a step stores 48 KB
//     and reads 64 KB.  Issuing every direct load twice lengthened the kernel by exactly what
//     removing them saves.  Loading the activation fragments from global memory straight into
//     MFMA registers (16x16x32, 64-byte pieces of a row per four lanes) avoided those stores and
//     was a third slower.
#include <type_traits>

#include "gemm_common.h"

namespace mlr {

namespace mid {
typedef _Float16 half16x8 __attribute__((ext_vector_type(8)));
constexpr int THREADS = 768, CWAVES = 4, PTHREADS = 512;
constexpr int MT = 128, CT = 64, RT = 128;
constexpr int TI = 2, TJ = CT / 32;               // a consumer's wave tile: 64 x 64
constexpr int KS = RT / 16 / 2;                   // 16-deep steps of a consumer per tile = 4
constexpr int ROW_BYTES = RT * 2;                 // 256
constexpr int A_BYTES = MT * ROW_BYTES;           // 32 KB
constexpr int W_BYTES = CT * ROW_BYTES;           // 16 KB
constexpr int A_SLOTS = 4, W_SLOTS = 2;
constexpr int W_BASE = A_SLOTS * A_BYTES;         // 128 KB
constexpr int LDS_BYTES = W_BASE + W_SLOTS * W_BYTES;   // 160 KB, all of a CU's LDS
constexpr int W_SETS = 3;                         // staged register sets of packed words
constexpr int A_CH = MT * 16 / 256;               // direct loads per loader thread and tile = 8
constexpr int PATCH_ROW = 72;                     // epilogue patch row stride (elements)
static_assert(A_SLOTS == 4 && W_SETS == 3, "the steady state below fetches three and four tiles ahead");

__device__ __forceinline__ int swz(int row) { return row & 15; }
// byte offset of logical 16-byte chunk `c` (0..15) of row `row` inside a tile
__device__ __forceinline__ int tile_off(int row, int c) { return row * ROW_BYTES + ((c ^ swz(row)) << 4); }
}  // namespace mid

template <int BITS, bool BWD, bool F16>
__global__ __launch_bounds__(mid::THREADS, 3) void gemm_mid_kernel(GemmDev d) {
    using namespace mid;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const GemmArgs &a = d.a;
    const TileCoord tco = tile_of_block(blockIdx.x, d.tiles_m, d.tiles_c);
    if (tco.tm < 0) return;   // grid padded to a multiple of 8
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const bool producer = wave >= CWAVES;
    // waves 4-7 dequantize (thread -> weight unit 0..255), waves 8-11 only send direct loads
    const int ptid = (tid - CWAVES * 64) & (PTHREADS - 1), pwave = (wave - CWAVES) & 7;
    const bool loader = pwave >= 4;
    const int unit = ptid & 255, ukb = uniform(pwave & 3);
    const int m0 = tco.tm * MT, c0 = tco.tc * CT;
    const int K = a.w.K, N = a.w.N;
    const int C = BWD ? N : K;
    const int Cout = BWD ? K : N;
    const int n_full = C / RT;
    const int n_main = (C + RT - 1) / RT;
    const int n_ext = (a.RE + RT - 1) / RT;
    const int n_tiles = n_main + n_ext;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const uint16_t *act_rowblock = a.act + (size_t)m0 * C;

    // ---- producers: activation tile by direct loads --------------------------------
    // chunk idx = i*256 + unit sits at byte 16*idx of the tile: row idx/16, physical chunk
    // idx%16, which holds logical chunk (idx%16) ^ swz(row).
    uint32_t a_voff[A_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int idx = i * 256 + unit;
        const int row = idx >> 4, lc = (idx & 15) ^ swz(row);
        int m = m0 + row;
        if (m > a.M - 1) m = a.M - 1;
        a_voff[i] = (uint32_t)(((size_t)(m - m0) * C + lc * 8) * 2);
    }
    auto issue_a_part = [&](int t, int a_slot, int i) {
        load_to_lds_16(act_rowblock + (size_t)t * RT, a_voff[i], lds0 + a_slot + i * (256 * 16) + ukb * 1024);
    };

    // ---- producers: weight units ------------------------------------------------------
    // forward: one (column, 32-code block) per thread; backward: one (4 n, 8 k) unit per thread
    uint32_t fw_off = 0, fw_n = 0;
    uint32_t bw_off = 0, bw_offhi = 0, bw_soff = 0;
    int bw_shift = 0, bw_row0 = 0, bw_g0 = 0;
    bool bw_kok = true;
    if (!BWD) {
        int n = c0 + (unit & (CT - 1));
        if (n > N - 1) n = N - 1;
        fw_n = (uint32_t)n;
        fw_off = (uint32_t)n * 4u;
    } else {
        bw_row0 = (c0 * BITS) >> 5;
        bw_g0 = (int)d.group_of_block((uint32_t)(c0 >> 5));
        const int last_row = K * BITS / 32 - 1;
        const int no = unit & 31, ko = unit >> 5;
        int k = c0 + ko * 8;
        bw_kok = k < K;
        if (k > K - 8) k = K - 8;
        const int bit = k * BITS, row = bit >> 5;
        const int row_hi = row + 1 > last_row ? last_row : row + 1;
        bw_shift = bit & 31;
        bw_off = (uint32_t)(((size_t)(row - bw_row0) * N + no * 4) * 4);
        bw_offhi = (uint32_t)(((size_t)(row_hi - bw_row0) * N + no * 4) * 4);
        bw_soff = (uint32_t)((size_t)((int)d.group_of_block((uint32_t)(k >> 5)) - bw_g0) * N + no * 4);
    }

    // staging registers of the asm loads: three sets, main tile i goes through set i % 3
    struct WStage {
        uint32_t fw_words[BITS];
        uint32_t fw_scale, fw_zero;
        u32x4 bw_lo, bw_hi;
        u32x2 bw_scale;
        uint32_t bw_zero;     // four 8-bit zero points
        u32x2 bw_zero16;      // F16: four binary16 zero points
    };
    WStage wst[W_SETS];
#pragma unroll
    for (int i = 0; i < W_SETS; ++i) {
#pragma unroll
        for (int j = 0; j < BITS; ++j) wst[i].fw_words[j] = 0;
        wst[i].fw_scale = wst[i].fw_zero = wst[i].bw_zero = 0;
        wst[i].bw_lo = wst[i].bw_hi = u32x4{0, 0, 0, 0};
        wst[i].bw_scale = wst[i].bw_zero16 = u32x2{0, 0};
    }
    auto load_w = [&](WStage &st, int t) {     // raw words, scales and zeros of full main tile t -> registers (async)
        if (!BWD) {
            const int blk = t * (RT / 32) + ukb;
            const uint32_t *wbase = a.w.qweight + (size_t)blk * BITS * N;
#pragma unroll
            for (int j = 0; j < BITS; ++j) aload_b32(st.fw_words[j], wbase + (size_t)j * N, fw_off);
            const size_t grow = (size_t)d.group_of_block((uint32_t)blk) * N;
            aload_u16(st.fw_scale, a.w.scales + grow, fw_n * 2);
            if (F16) aload_u16(st.fw_zero, a.zeros16 + grow, fw_n * 2);
            else aload_u8(st.fw_zero, a.w.zeros + grow, fw_n);
        } else {
            const uint32_t *wbase = a.w.qweight + (size_t)bw_row0 * N + (size_t)t * RT;
            aload_b128(st.bw_lo, wbase, bw_off);
            if (BITS == 3) aload_b128(st.bw_hi, wbase, bw_offhi);
            aload_b64(st.bw_scale, a.w.scales + (size_t)bw_g0 * N + (size_t)t * RT, bw_soff * 2);
            if (F16) aload_b64(st.bw_zero16, a.zeros16 + (size_t)bw_g0 * N + (size_t)t * RT, bw_soff * 2);
            else aload_b32(st.bw_zero, a.w.zeros + (size_t)bw_g0 * N + (size_t)t * RT, bw_soff);
        }
    };
    // Loads return in order: waiting until at most KEEP remain outstanding completes everything
    // issued before the KEEP most recent ones.  The staged registers of the set are pinned behind
    // the wait.
    auto wait_loads = [&](WStage &st, auto keep) {
        constexpr int KEEP = decltype(keep)::value;
        if (!BWD) {
            if (BITS == 2)
                asm volatile("s_waitcnt vmcnt(%4)" : "+v"(st.fw_words[0]), "+v"(st.fw_words[1]), "+v"(st.fw_scale), "+v"(st.fw_zero) : "n"(KEEP) : "memory");
            else if (BITS == 3)
                asm volatile("s_waitcnt vmcnt(%5)" : "+v"(st.fw_words[0]), "+v"(st.fw_words[1]), "+v"(st.fw_words[2 % BITS]), "+v"(st.fw_scale), "+v"(st.fw_zero) : "n"(KEEP) : "memory");
            else
                asm volatile("s_waitcnt vmcnt(%6)" : "+v"(st.fw_words[0]), "+v"(st.fw_words[1]), "+v"(st.fw_words[2 % BITS]), "+v"(st.fw_words[3 % BITS]), "+v"(st.fw_scale), "+v"(st.fw_zero) : "n"(KEEP) : "memory");
        } else {
            if (BITS == 3) {
                asm volatile("s_waitcnt vmcnt(%4)" : "+v"(st.bw_lo), "+v"(st.bw_hi), "+v"(st.bw_scale), "+v"(st.bw_zero) : "n"(KEEP) : "memory");
                // the 8-code chunks straddle two words: join them now
#pragma unroll
                for (int i = 0; i < 4; ++i) st.bw_lo[i] = __builtin_amdgcn_alignbit(st.bw_hi[i], st.bw_lo[i], bw_shift);
            } else {
                asm volatile("s_waitcnt vmcnt(%3)" : "+v"(st.bw_lo), "+v"(st.bw_scale), "+v"(st.bw_zero) : "n"(KEEP) : "memory");
            }
            if (F16) asm volatile("" : "+v"(st.bw_zero16)::"memory");   // stays behind the wait: volatile asms keep their order
        }
    };
    // w = fma(q, scale, bias): bias = -zero * scale for an integer zero point, or the binary16 zero
    // point itself where it is one that is added (Section 2.2 eq. (2) as printed)
    auto dq_of = [](uint16_t scale_bits, uint32_t zero_bits) {
        if (!F16) return make_dq(scale_bits, (uint8_t)zero_bits);
        DqConst c;
        c.scale = half_bits_to_float(scale_bits);
        c.bias = half_bits_to_float((uint16_t)zero_bits);
        return c;
    };
    // dequantize quarter `part` (0..3) of the unit whose words are staged in `st` into weight tile `buf`
    auto store_w = [&](int buf, const WStage &st, int part) {
        unsigned char *Ws = smem + W_BASE + buf * W_BYTES;
        if (!BWD) {
            const int nl = unit & (CT - 1);
            const DqConst dq = dq_of((uint16_t)st.fw_scale, st.fw_zero);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (j != part) continue;
                uint32_t o[4];
                dequant_quarter<BITS, F16>(st.fw_words, j, dq, o);
                *reinterpret_cast<uint4 *>(Ws + tile_off(nl, ukb * 4 + j)) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        } else {
            const int no = unit & 31, ko = unit >> 5;
            const uint32_t sc[2] = {st.bw_scale[0], st.bw_scale[1]};
            uint32_t chunk[4];
            DqConst dq[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                chunk[i] = BITS == 3 ? st.bw_lo[i] : st.bw_lo[i] >> bw_shift;   // 3-bit: joined by wait_loads()
                const uint16_t sb = bw_kok ? (uint16_t)(sc[i >> 1] >> ((i & 1) * 16)) : (uint16_t)0;
                const uint32_t zb = F16 ? (bw_kok ? (st.bw_zero16[i >> 1] >> ((i & 1) * 16)) & 0xFFFFu : 0u) : (st.bw_zero >> (i * 8)) & 0xFFu;
                dq[i] = dq_of(sb, zb);
            }
            // 32 lanes fill one whole row per store
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                if (kk / 2 != part) continue;
                uint32_t o[2];
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    o[i] = pack_pair<F16>(dq_value(chunk_code<BITS>(chunk[2 * i], kk), dq[2 * i]),
                                          dq_value(chunk_code<BITS>(chunk[2 * i + 1], kk), dq[2 * i + 1]));
                *reinterpret_cast<uint2 *>(Ws + tile_off(ko * 8 + kk, no >> 1) + (no & 1) * 8) = make_uint2(o[0], o[1]);
            }
        }
    };

    // ---- tail tiles (ragged last main tile, adapter extension): staged one at a time through
    // registers into slot 0 / weight tile 0 by all waves (predicated; a handful of tiles at most)
    auto tail_geometry = [&](int t, bool &ext, int &r0, int &ksteps) {
        ext = t >= n_main;
        r0 = ext ? (t - n_main) * RT : t * RT;
        ksteps = RT / 16;
        if (ext) {
            ksteps = (a.RE - r0) / 16;
            if (ksteps > RT / 16) ksteps = RT / 16;
        }
    };
    auto stage_tail_tile = [&](int t, bool is_producer) {
        bool ext;
        int r0, ksteps;
        tail_geometry(t, ext, r0, ksteps);
        const int ld = ext ? a.RE : C;
        const uint16_t *abase = (ext ? a.act_ext + (size_t)m0 * ld : act_rowblock) + r0;
        unsigned char *As = smem, *Ws = smem + W_BASE;
#pragma unroll
        for (int i = 0; i < (MT * 16 + THREADS - 1) / THREADS; ++i) {
            const int idx = i * THREADS + tid;
            if (idx < MT * 16) {
                const int row = idx >> 4, ch = idx & 15;
                int m = m0 + row;
                if (m > a.M - 1) m = a.M - 1;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (r0 + ch * 8 < ld) v = load_at<uint4>(abase, (uint32_t)(((size_t)(m - m0) * ld + ch * 8) * 2));
                *reinterpret_cast<uint4 *>(As + tile_off(row, ch)) = v;
            }
        }
        if (ext) {
#pragma unroll
            for (int i = 0; i < (CT * 16 + THREADS - 1) / THREADS; ++i) {
                const int idx = i * THREADS + tid;
                if (idx < CT * 16) {
                    const int row = idx >> 4, ch = idx & 15;
                    int c = c0 + row;
                    if (c > Cout - 1) c = Cout - 1;
                    uint4 v = make_uint4(0, 0, 0, 0);
                    if (r0 + ch * 8 < a.RE) v = *reinterpret_cast<const uint4 *>(a.w_ext + (size_t)c * a.RE + r0 + ch * 8);
                    *reinterpret_cast<uint4 *>(Ws + tile_off(row, ch)) = v;
                }
            }
        } else if (is_producer && !loader) {
            WStage &st = wst[0];
            if (!BWD) {
                const int blk = t * (RT / 32) + ukb;
                const bool ok = blk * 32 < K;
                const int blk_c = ok ? blk : 0;
                const uint32_t *wbase = a.w.qweight + (size_t)blk_c * BITS * N;
#pragma unroll
                for (int j = 0; j < BITS; ++j) st.fw_words[j] = load_at<uint32_t>(wbase + (size_t)j * N, fw_off);
                const size_t grow = (size_t)d.group_of_block((uint32_t)blk_c) * N;
                st.fw_scale = ok ? (uint32_t)load_at<uint16_t>(a.w.scales + grow, fw_n * 2) : 0u;   // 0 -> weights +0
                if (F16) st.fw_zero = ok ? (uint32_t)load_at<uint16_t>(a.zeros16 + grow, fw_n * 2) : 0u;
                else st.fw_zero = load_at<uint8_t>(a.w.zeros + grow, fw_n);
            } else {
                const bool ok = r0 + (unit & 31) * 4 < N;
                st.bw_lo = u32x4{0, 0, 0, 0};
                st.bw_hi = u32x4{0, 0, 0, 0};
                st.bw_scale = st.bw_zero16 = u32x2{0, 0};
                st.bw_zero = 0;
                if (ok) {
                    const uint32_t *wbase = a.w.qweight + (size_t)bw_row0 * N + r0;
                    st.bw_lo = load_at<u32x4>(wbase, bw_off);
                    if (BITS == 3) {
                        st.bw_hi = load_at<u32x4>(wbase, bw_offhi);
#pragma unroll
                        for (int i = 0; i < 4; ++i) st.bw_lo[i] = __builtin_amdgcn_alignbit(st.bw_hi[i], st.bw_lo[i], bw_shift);
                    }
                    st.bw_scale = load_at<u32x2>(a.w.scales + (size_t)bw_g0 * N + r0, bw_soff * 2);
                    if (F16) st.bw_zero16 = load_at<u32x2>(a.zeros16 + (size_t)bw_g0 * N + r0, bw_soff * 2);
                    else st.bw_zero = load_at<uint32_t>(a.w.zeros + (size_t)bw_g0 * N + r0, bw_soff);
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) store_w(0, st, q);
        }
    };

    // Producers and consumers run separate loops that meet at the same barriers (every wave of the
    // workgroup executes the same number of them).
    //
    // Step i of the steady state (full main tiles): consumers work on activation slot i % 4 and
    // weight tile i & 1.  Producers dequantize weight tile i + 1 from staged set (i + 1) % 3, send
    // the direct loads of activation tile i + 3 into the slot the consumers left at the last
    // barrier and refill the set with the words of tile i + 4.  Loads return in order, so "at most
    // n still in flight" completes all but the n most recent: the wait that ends step i asks for
    // the words of tile i + 2 (needed when step i + 1 opens), which also completes the direct
    // loads of tile i + 1 issued before them, and leaves in flight the direct loads of tiles
    // i + 2 and i + 3 and the words of tiles i + 3 and i + 4.
    constexpr int W_LOADS = BWD ? (BITS == 3 ? 4 : 3) : BITS + 2;   // load instructions of one load_w()
    const int last = n_full - 1;   // past the last tile the fetches repeat it; what they bring is never consumed
    if (producer) {
        if (n_full > 0 && loader) {
            // activation tiles three steps ahead; the wait leaves the loads of two steps in flight
#pragma unroll
            for (int sl = 0; sl < 3; ++sl)
#pragma unroll
                for (int i = 0; i < A_CH; ++i) issue_a_part(last < sl ? last : sl, sl * A_BYTES, i);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            int a_fill = 3 * A_BYTES;   // ring slot being filled (byte offset, wave-uniform)
            for (int tt = 0; tt < n_full; ++tt) {
                const int ta = tt + 3 < n_full ? tt + 3 : last;
#pragma unroll
                for (int i = 0; i < A_CH; ++i) issue_a_part(ta, a_fill, i);
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * A_CH) : "memory");
                __syncthreads();
                a_fill = a_fill == 3 * A_BYTES ? 0 : a_fill + A_BYTES;
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        } else if (n_full > 0) {
            load_w(wst[0], 0);
            load_w(wst[1], last < 1 ? last : 1);
            load_w(wst[2], last < 2 ? last : 2);
            // everything has landed after the first wait; set 2 is pinned (and, for 3-bit backward,
            // joined) by the wait that opens step 1, the only one it passes through
            wait_loads(wst[0], std::integral_constant<int, 0>());
            wait_loads(wst[1], std::integral_constant<int, 0>());
#pragma unroll
            for (int q = 0; q < 4; ++q) store_w(0, wst[0], q);
            load_w(wst[0], last < 3 ? last : 3);
            __syncthreads();
            for (int t = 0; t < n_full; t += 3) {
#pragma unroll
                for (int u = 0; u < 3; ++u) {
                    const int tt = t + u;
                    if (tt < n_full) {
                        WStage &st = wst[(u + 1) % 3];          // words of tile tt + 1
                        const int wbuf = (tt + 1) & 1;
                        // in flight at most: the words of tiles tt + 2 and tt + 3
                        if (tt > 0) wait_loads(st, std::integral_constant<int, 2 * W_LOADS>());
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            store_w(wbuf, st, q);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        load_w(st, tt + 4 < n_full ? tt + 4 : last);
                        __syncthreads();
                    }
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
        for (int t = n_full; t < n_tiles; ++t) {
            stage_tail_tile(t, true);
            __syncthreads();
            __syncthreads();
        }
        __syncthreads();   // the consumers' two barriers around their sum
        __syncthreads();
        return;
    }

    // ---- consumers ------------------------------------------------------------------------
    const int wm = wave & 1, kg = wave >> 1;   // row half of the tile, half of each 128-deep step
    f32x16 acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // the consumer's 16-deep step s (0..3) of a tile is step 4 kg + s: logical chunks
    // 8 kg + 2 s + h for lane half h.  +32 rows leaves the swizzle unchanged, and s only flips
    // bits 5-6 of the offset.
    const int offA0 = tile_off(wm * 64 + (lane & 31), 8 * kg + (lane >> 5));
    const int offW0 = W_BASE + tile_off(lane & 31, 8 * kg + (lane >> 5));
    struct Frags {
        bf16x8 af[TI], bf[TJ];
    };
    auto load_frags = [&](Frags &f, int a_slot, int wbuf, int sidx) {
#pragma unroll
        for (int i = 0; i < TI; ++i)
            f.af[i] = *reinterpret_cast<const bf16x8 *>(smem + a_slot + (offA0 ^ (sidx << 5)) + i * 32 * ROW_BYTES);
#pragma unroll
        for (int j = 0; j < TJ; ++j)
            f.bf[j] = *reinterpret_cast<const bf16x8 *>(smem + wbuf * W_BYTES + (offW0 ^ (sidx << 5)) + j * 32 * ROW_BYTES);
    };
    auto mfma_frags = [&](const Frags &f) {
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int j = 0; j < TJ; ++j)
                if (F16) {
                    half16x8 x, y;
                    __builtin_memcpy(&x, &f.af[i], sizeof x);
                    __builtin_memcpy(&y, &f.bf[j], sizeof y);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x, y, acc[i][j], 0, 0, 0);
                } else {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.af[i], f.bf[j], acc[i][j], 0, 0, 0);
                }
    };

    if (n_full > 0) {
        __syncthreads();
        int a_cur = 0;
        for (int t = 0; t < n_full; t += 2) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (t + u < n_full) {
                    Frags f[KS];
#pragma unroll
                    for (int sidx = 0; sidx < KS; ++sidx) load_frags(f[sidx], a_cur, u, sidx);
#pragma unroll
                    for (int sidx = 0; sidx < KS; ++sidx) mfma_frags(f[sidx]);
                    __syncthreads();
                    a_cur = a_cur == 3 * A_BYTES ? 0 : a_cur + A_BYTES;
                }
            }
        }
        __syncthreads();
    }
    for (int t = n_full; t < n_tiles; ++t) {
        bool ext;
        int r0, ksteps;
        tail_geometry(t, ext, r0, ksteps);
        stage_tail_tile(t, false);
        __syncthreads();
#pragma unroll
        for (int sidx = 0; sidx < KS; ++sidx) {
            if (KS * kg + sidx < ksteps) {
                Frags f;
                load_frags(f, 0, 0, sidx);
                mfma_frags(f);
            }
        }
        __syncthreads();
    }

    // ---- the two halves of the contraction meet in LDS: of its 64 rows a consumer keeps block kg
    // (32 rows) and hands the other block to its partner
    float *red = reinterpret_cast<float *>(smem);   // [receiving wave][j][v][lane]
    {
        const int partner = wave ^ 2;
#pragma unroll
        for (int i = 0; i < TI; ++i) {
            if (i == kg) continue;
#pragma unroll
            for (int j = 0; j < TJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[((partner * TJ + j) * 16 + v) * 64 + lane] = acc[i][j][v];
        }
    }
    __syncthreads();
    f32x16 fin[TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i) {
        if (i != kg) continue;
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                fin[j][v] = acc[i][j][v] + red[((wave * TJ + j) * 16 + v) * 64 + lane];
            }
    }
    __syncthreads();

    // ---- F16: the adapter term s P F and the bias join here, before the one rounding
    // (Figure 1 / eq. (3); the bias belongs to the frozen layer and enters the forward pass only) ----
    if (F16) {
        const int r = a.ep_r;
        float *Ps = reinterpret_cast<float *>(smem + 32768) + wave * (32 * 64);   // this wave's 32 rows of P, [jj][32 rows]
        int cc[TJ];
        float lora[TJ][16];
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const int col = c0 + j * 32 + (lane & 31);
            cc[j] = col < Cout ? col : Cout - 1;
        }
        adapter_term_32rows<TJ>(a.ep_P, a.ep_F, r, N, BWD, m0 + wm * 64 + kg * 32, a.M, cc, Ps, lane, lora);
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            float bias = 0.f;
            if (!BWD && a.bias16 != nullptr) bias = half_bits_to_float(a.bias16[cc[j]]);
#pragma unroll
            for (int v = 0; v < 16; ++v) fin[j][v] = __builtin_fmaf(a.ep_scale, lora[j][v], fin[j][v] + bias);
        }
    }

    // ---- epilogue of a consumer: its 32 x 64 block, one RNE to bfloat16 (binary16), through an LDS
    // patch so that the global stores are 16 bytes per lane and 128 contiguous bytes per row ------
    uint16_t *patch = reinterpret_cast<uint16_t *>(smem) + wave * (32 * PATCH_ROW);
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int prow = 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
            patch[prow * PATCH_ROW + j * 32 + (lane & 31)] = (uint16_t)(pack_pair<F16>(fin[j][v], 0.f) & 0xFFFFu);
        }
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the patch is private to the wave
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int idx = lane + q * 64;    // 256 chunks of 16 bytes: 32 rows x 8
        const int prow = idx / 8, ch = idx % 8;
        const uint4 v = *reinterpret_cast<const uint4 *>(patch + prow * PATCH_ROW + ch * 8);
        const int row = m0 + wm * 64 + kg * 32 + prow;
        const int col = c0 + ch * 8;
        if (row < a.M && col < Cout) *reinterpret_cast<uint4 *>(a.out + (size_t)row * Cout + col) = v;
    }
}

template <int BITS, bool BWD, bool F16 = false>
static hipError_t launch_mid(const GemmArgs &a, hipStream_t stream) {
    const GemmDev d = make_gemm_dev(a, mid::MT, mid::CT);
    const int blocks = (d.tiles_m * d.tiles_c + 7) / 8 * 8;
    auto kern = gemm_mid_kernel<BITS, BWD, F16>;
    static bool configured[64] = {};
    const hipError_t e = ensure_lds_limit(reinterpret_cast<const void *>(kern), mid::LDS_BYTES, configured);
    if (e != hipSuccess) return e;
    launch_kernel(F16 ? (BWD ? "f16_gemm_bwd" : "f16_gemm_fwd") : (BWD ? "gemm_bwd_128x64s" : "gemm_fwd_128x64s"), kern,
                  blocks, mid::THREADS, mid::LDS_BYTES, stream, d);
    return hipGetLastError();
}

hipError_t launch_gemm_mid(const GemmArgs &a, hipStream_t stream) {
    switch (a.w.bits) {
        case 2: return a.backward ? launch_mid<2, true>(a, stream) : launch_mid<2, false>(a, stream);
        case 3: return a.backward ? launch_mid<3, true>(a, stream) : launch_mid<3, false>(a, stream);
        default: return a.backward ? launch_mid<4, true>(a, stream) : launch_mid<4, false>(a, stream);
    }
}

hipError_t launch_gemm_mid_f16(const GemmArgs &a, hipStream_t stream) {
    switch (a.w.bits) {
        case 2: return a.backward ? launch_mid<2, true, true>(a, stream) : launch_mid<2, false, true>(a, stream);
        case 3: return a.backward ? launch_mid<3, true, true>(a, stream) : launch_mid<3, false, true>(a, stream);
        default: return a.backward ? launch_mid<4, true, true>(a, stream) : launch_mid<4, false, true>(a, stream);
    }
}

}  // namespace mlr
