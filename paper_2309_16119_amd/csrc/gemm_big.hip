// The large-M variant of the fused dequantize + bf16 MFMA tile kernel: a 256 x 256
// output tile per workgroup, 8 waves (two per SIMD) of 128 x 64 each, 64-deep steps.
// (A second instantiation with 128-row tiles, waves of 64 x 64, serves token counts whose last
// block of 256 rows would be at most half full -- a hundred-odd tokens above all; both exist for
// either storage convention.)
// Same mathematics as gemm_tile.hip (ModuLoRA Figure 1: forward X What^T and backward
// dY What with What re-materialized from the packed codes, plus the adapter term of eq. (3)
// as an extended contraction); what differs is the data path, chosen from what was measured
// on MI355X:
//
//   - LDS stores from registers (ds_write_b128) sustain only ~70 B/clk per CU while
//     LDS reads sustain ~200: the activation tile therefore never passes through
//     registers -- it is fetched with direct global->LDS loads (16 B per lane), and only
//     the dequantized weight tile is written with ds_write.
//   - Direct loads place lane i's 16 bytes at LDS base + 16 i, so rows cannot be padded.
//     Rows are 128 B and the 16-byte chunk index is XOR-swizzled with (row >> 1) & 7.  The
//     LDS has 64 banks, so two rows share a bank line: 16 consecutive rows at one logical
//     chunk (a quarter of a 16-byte fragment read, or of a forward weight-tile store) then
//     cover all 16 bank groups.  SQ_LDS_BANK_CONFLICT of the backward kernel fell from 40 % of
//     its active LDS cycles (with row & 7) to nothing.
//   - All of a CU's 160 KB of LDS: a ring of three activation tiles and two weight tiles.
//     Every wave runs the same step: the MFMAs of tile t with, between them, its share of
//     the dequantization of weight tile t + 1 (from registers staged a step earlier) and the
//     fetches of what comes after -- the packed words of tile t + 2 and, a quarter per
//     16-deep step, the direct loads of activation tile t + 2.  Stamps written by an
//     instrumented build showed why: with all fetches at the top of a step the eight waves
//     queue at the memory pipeline for 500-800 cycles while the matrix cores idle, and loads
//     issued one step ahead arrive ~300 cycles after the step's MFMAs are done.
//   - The loads are issued from inline assembly and awaited with an explicit s_waitcnt vmcnt
//     that leaves exactly the step's four direct loads in flight (loads return in order).
//   - 256 x 256 tiles rarely come in multiples of the 256 compute units.  The tiles beyond
//     the last full round are cut into slices of the contraction (BigPlan): every slice is
//     a workgroup that leaves its fp32 accumulators, in register order, in a scratch buffer,
//     and gemm_big_fixup_kernel adds the slices of a tile in a fixed order and runs the same
//     epilogue.  No atomics and no fences, so results do not depend on timing.
#include <type_traits>

#include "gemm_common.h"

namespace mlr {

namespace big {
typedef _Float16 half16x8 __attribute__((ext_vector_type(8)));
constexpr int THREADS = 512, NWAVES = 8;
constexpr int BAND = 4;                  // row blocks per band of the tile walk (2 measures the same, 8 is 1-2 % slower)
constexpr int CT = 256, WN = 64, RT = 64;
constexpr int TJ = WN / 32;
constexpr int ROW_BYTES = RT * 2;                 // 128
constexpr int W_BYTES = CT * ROW_BYTES;           // 32 KB: one weight tile
constexpr int A_SLOTS = 3, W_SLOTS = 2;           // activation ring (filled two steps ahead), weight tiles
constexpr int W_CH = CT * 8 / THREADS;            // 16-byte chunks of an extension W tile per thread
constexpr int FW_UNITS = CT * 2 / THREADS;        // (column, 32-code block) units per thread = 1
constexpr int BW_UNITS = (CT / 8) * (RT / 4) / THREADS;   // (4 n, 8 k) units per thread = 1
constexpr int PATCH_ROW = 72;                     // epilogue patch row stride (elements)
// What depends on the rows of a tile (MT = 256 or 128; two rows of four waves either way).
template <int MT_>
struct Geo {
    static constexpr int MT = MT_, WM = MT / 2, TI = WM / 32;
    static constexpr int A_BYTES = MT * ROW_BYTES;            // 32 / 16 KB: one activation tile
    static constexpr int W_BASE = A_SLOTS * A_BYTES;
    static constexpr int LDS_BYTES = A_SLOTS * A_BYTES + W_SLOTS * W_BYTES;   // 160 KB (all of a CU's LDS) / 112 KB
    static constexpr int A_CH = MT * 8 / THREADS;             // 16-byte activation chunks per thread: 4 / 2
    static constexpr int A_EVERY = (RT / 16) / A_CH;          // one of them every so many 16-deep steps
    static constexpr int PART_F4 = THREADS * (MT / 8);        // float4 of one partial tile
    static_assert(A_CH * A_EVERY == RT / 16, "the activation tile's chunks spread evenly over the 16-deep steps");
};

// XOR swizzle of a row's eight 16-byte chunks.  Rows are 128 bytes and the LDS has 64 banks
// (256 bytes per cycle, 16 lanes of a 16-byte access), so two rows share a bank line: the even
// rows of 16 consecutive ones need eight different values, and so do the odd ones.
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }
// byte offset of logical 16-byte chunk `c` of row `row` inside a tile
__device__ __forceinline__ int tile_off(int row, int c) { return row * ROW_BYTES + ((c ^ swz(row)) << 4); }
}  // namespace big

// What a workgroup works on: a whole tile (slice < 0) or slice `slice` of `split` of a tile.
// Workgroup ids go round-robin over the 8 XCDs; every XCD gets a contiguous run of the whole
// tiles first (walked in bands of BAND row blocks, see banded_tile()) and then a contiguous
// run of the slices.
struct BigItem {
    int tile, slice;
};
__device__ __forceinline__ BigItem big_item_of_block(int bid, const BigPlan &p) {
    BigItem it;
    const int x = bid & 7, q = bid >> 3;
    const int whole = p.split > 1 ? p.full : p.full + p.tail;
    const int whole_per_xcd = (whole + 7) >> 3;
    it.slice = -1;
    if (q < whole_per_xcd) {
        it.tile = x * whole_per_xcd + q;
        if (it.tile >= whole) it.tile = -1;
        return it;
    }
    const int slices = p.split > 1 ? p.tail * p.split : 0;
    const int slices_per_xcd = (slices + 7) >> 3;
    const int j = x * slices_per_xcd + (q - whole_per_xcd);
    if (q - whole_per_xcd >= slices_per_xcd || j >= slices) {
        it.tile = -1;
        return it;
    }
    it.tile = p.full + j / p.split;
    it.slice = j % p.split;
    return it;
}

// Epilogue of one wave for its i-th block of 32 rows: one RNE to bfloat16 (binary16); the
// 32 x 64 patch goes through LDS so that the global stores are 16 bytes per lane and 128
// contiguous bytes per row.  F16 (the layer in the paper's own storage convention): the adapter
// term s P F and the bias join here, before the rounding (Figure 1 / eq. (3); the bias belongs
// to the frozen layer and enters the forward pass only); P's 32 rows pass through LDS behind
// the patches.
// `slot`: which of the per-wave LDS areas (patch, rows of P) this wave uses.
template <bool F16, int WM>
__device__ __forceinline__ void big_epilogue_rows(f32x16 (&acc_i)[big::TJ], int i, unsigned char *smem, const GemmArgs &a, int Cout,
                                                  int m0, int c0, int wave, int lane, int slot) {
    using namespace big;
    const int wm = wave >> 2, wn = wave & 3;
    uint16_t *out = a.out;
    const int M = a.M;
    if (F16) {
        const int r = a.ep_r, N = a.w.N;
        const bool bwd = a.backward;
        float *Ps = reinterpret_cast<float *>(smem + 40960) + slot * (32 * 64);   // [jj][32 rows]
        int cc[TJ];
        float lora[TJ][16];
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const int col = c0 + wn * WN + j * 32 + (lane & 31);
            cc[j] = col < Cout ? col : Cout - 1;
        }
        adapter_term_32rows<TJ>(a.ep_P, a.ep_F, r, N, bwd, m0 + wm * WM + i * 32, M, cc, Ps, lane, lora);
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            float bias = 0.f;
            if (!bwd && a.bias16 != nullptr) bias = half_bits_to_float(a.bias16[cc[j]]);
#pragma unroll
            for (int v = 0; v < 16; ++v) acc_i[j][v] = __builtin_fmaf(a.ep_scale, lora[j][v], acc_i[j][v] + bias);
        }
    }
    uint16_t *patch = reinterpret_cast<uint16_t *>(smem) + slot * (32 * PATCH_ROW);
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int prow = 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
            patch[prow * PATCH_ROW + j * 32 + (lane & 31)] = (uint16_t)(pack_pair<F16>(acc_i[j][v], 0.f) & 0xFFFFu);
        }
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the patch is private to the wave
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int idx = lane + q * 64;    // 256 chunks of 16 bytes: 32 rows x 8
        const int prow = idx / 8, ch = idx % 8;
        const uint4 v = *reinterpret_cast<const uint4 *>(patch + prow * PATCH_ROW + ch * 8);
        const int row = m0 + wm * WM + i * 32 + prow;
        const int col = c0 + wn * WN + ch * 8;
        if (row < M && col < Cout) *reinterpret_cast<uint4 *>(out + (size_t)row * Cout + col) = v;
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
}

// Partial tiles: slice j of the plan owns MT x 256 floats, stored as MT / 8 float4 per thread
// in register order ([float4 index][thread]), so writes and reads are fully coalesced.
template <int MT>
__device__ __forceinline__ float4 *big_partial_of(float *partials, int tail_tile, int slice, int split) {
    return reinterpret_cast<float4 *>(partials) + ((size_t)tail_tile * split + slice) * (size_t)big::Geo<MT>::PART_F4;
}

template <int BITS, bool BWD, bool F16, int MT>
__global__ __launch_bounds__(big::THREADS, 2) void gemm_big_kernel(GemmDev d, BigPlan plan) {
    using namespace big;
    using G = Geo<MT>;
    constexpr int WM = G::WM, TI = G::TI, A_BYTES = G::A_BYTES, W_BASE = G::W_BASE, A_CH = G::A_CH;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const GemmArgs &a = d.a;
    const BigItem item = big_item_of_block(blockIdx.x, plan);
    if (item.tile < 0) return;   // grid padded to a multiple of 8
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const TileCoord tco = banded_tile<big::BAND>(item.tile, d.tiles_m, d.tiles_c);
    const int m0 = tco.tm * MT, c0 = tco.tc * CT;
    const int K = a.w.K, N = a.w.N;
    const int C = BWD ? N : K;
    const int Cout = BWD ? K : N;
    const int n_full = C / RT;
    const int n_main = (C + RT - 1) / RT;
    const int n_ext = (a.RE + RT - 1) / RT;
    const int n_tiles = n_main + n_ext;
    // this workgroup's share of the full main tiles; the last slice also takes the ragged
    // tile and the adapter extension
    const int t0 = item.slice < 0 ? 0 : (int)((long)n_full * item.slice / plan.split);
    const int t1 = item.slice < 0 ? n_full : (int)((long)n_full * (item.slice + 1) / plan.split);
    const bool takes_tail = item.slice < 0 || item.slice == plan.split - 1;
    // LDS byte address of the dynamic segment (what M0 wants)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;

    // ---- activation tile: direct loads ------------------------------------------
    // chunk idx = i*512 + tid sits at byte 16*idx of the tile: row idx/8, physical chunk
    // idx%8, which holds logical chunk (idx%8) ^ swz(row).
    uint32_t a_voff[A_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int idx = i * THREADS + tid;
        const int row = idx >> 3, lc = (idx & 7) ^ swz(idx >> 3);
        int m = m0 + row;
        if (m > a.M - 1) m = a.M - 1;
        a_voff[i] = (uint32_t)(((size_t)(m - m0) * C + lc * 8) * 2);
    }
    const uint16_t *act_rowblock = a.act + (size_t)m0 * C;
    // quarter i of activation tile t -> ring slot at byte a_slot (wave-uniform)
    auto issue_a_part = [&](int t, int a_slot, int i) {
        load_to_lds_16(act_rowblock + (size_t)t * RT, a_voff[i], lds0 + a_slot + i * (THREADS * 16) + wave * 1024);
    };
    auto issue_a = [&](int t, int a_slot) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) issue_a_part(t, a_slot, i);
    };

    // ---- weight units -------------------------------------------------------------
    uint32_t fw_off = 0, fw_n = 0;
    int fw_kb = 0;
    uint32_t bw_off = 0, bw_offhi = 0, bw_soff = 0;
    int bw_shift = 0, bw_row0 = 0, bw_g0 = 0;
    bool bw_kok = true;
    if (!BWD) {
        int n = c0 + (tid & (CT - 1));
        if (n > N - 1) n = N - 1;
        fw_n = (uint32_t)n;
        fw_off = (uint32_t)n * 4u;
        fw_kb = uniform(tid >> 8);
    } else {
        bw_row0 = (c0 * BITS) >> 5;
        bw_g0 = (int)d.group_of_block((uint32_t)(c0 >> 5));
        const int last_row = K * BITS / 32 - 1;
        const int no = tid & 15, ko = tid >> 4;
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

    // staging registers of the asm loads: two sets, tile t0 + i goes through set i & 1
    struct WStage {
        uint32_t fw_words[BITS];
        uint32_t fw_scale, fw_zero;
        u32x4 bw_lo, bw_hi;
        u32x2 bw_scale;
        uint32_t bw_zero;     // four 8-bit zero points
        u32x2 bw_zero16;      // F16: four binary16 zero points
    };
    WStage wst[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < BITS; ++j) wst[i].fw_words[j] = 0;
        wst[i].fw_scale = wst[i].fw_zero = wst[i].bw_zero = 0;
        wst[i].bw_lo = wst[i].bw_hi = u32x4{0, 0, 0, 0};
        wst[i].bw_scale = wst[i].bw_zero16 = u32x2{0, 0};
    }

    auto load_w = [&](WStage &st, int t) {     // raw words, scales and zeros of full main tile t -> registers (async)
        if (!BWD) {
            const int blk = t * 2 + fw_kb;
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
    // wait for every outstanding load of this wave (direct and staged) and pin the staged
    // registers of one set behind the wait
    // Loads return in order: waiting until at most KEEP remain outstanding completes everything
    // issued before the KEEP most recent ones.
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
                // the 8-code chunks straddle two words: join them now, so that a landed set is 4 registers
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
    // dequantize the staged words of one set into the W tile of buffer buf: quarter `part`
    // (0..3) of the thread's share, or all of it (part < 0)
    auto store_w = [&](int buf, const WStage &st, int part) {
        unsigned char *Ws = smem + W_BASE + buf * W_BYTES;
        if (!BWD) {
            const int nl = tid & (CT - 1);
            const DqConst dq = dq_of((uint16_t)st.fw_scale, st.fw_zero);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (part >= 0 && j != part) continue;
                uint32_t o[4];
                dequant_quarter<BITS, F16>(st.fw_words, j, dq, o);
                *reinterpret_cast<uint4 *>(Ws + tile_off(nl, fw_kb * 4 + j)) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        } else {
            const int no = tid & 15, ko = tid >> 4;
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
            // a 16-lane group fills one row per store; neighbouring groups take their eight rows in
            // opposite order of parity, so that the two rows of a 32-lane store fall into different
            // halves of the banks
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                if (part >= 0 && kk / 2 != part) continue;
                const int kq = kk ^ (ko & 1);
                uint32_t o[2];
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    o[i] = pack_pair<F16>(dq_value(chunk_code<BITS>(chunk[2 * i], kq), dq[2 * i]),
                                          dq_value(chunk_code<BITS>(chunk[2 * i + 1], kq), dq[2 * i + 1]));
                *reinterpret_cast<uint2 *>(Ws + tile_off(ko * 8 + kq, no >> 1) + (no & 1) * 8) = make_uint2(o[0], o[1]);
            }
        }
    };

    // ---- accumulators and fragment addressing ------------------------------------
    f32x16 acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int wm = wave >> 2, wn = wave & 3;
    const int rowA = wm * WM + (lane & 31), rowW = wn * WN + (lane & 31);
    // +32 rows leaves the swizzle unchanged, so one offset serves all i / j; 16-deep step ks reads
    // logical chunks 2 ks and 2 ks + 1, and (2 ks + h) ^ z = (2 ks) ^ (h ^ z): its offset is that of
    // step 0 with ks XOR-ed into bits 5-6 (one VALU operation instead of a register per step)
    const int offA0 = tile_off(rowA, lane >> 5);
    const int offW0 = W_BASE + tile_off(rowW, lane >> 5);

    struct Frags {
        bf16x8 af[TI], bf[TJ];
    };
    // oa: offA0 plus the ring slot's byte offset; wbuf: which weight tile
    auto load_frags = [&](Frags &f, int oa, int wbuf, int ks) {
#pragma unroll
        for (int i = 0; i < TI; ++i)
            f.af[i] = *reinterpret_cast<const bf16x8 *>(smem + (oa ^ (ks << 5)) + i * 32 * ROW_BYTES);
#pragma unroll
        for (int j = 0; j < TJ; ++j)
            f.bf[j] = *reinterpret_cast<const bf16x8 *>(smem + (offW0 ^ (ks << 5)) + wbuf * W_BYTES + j * 32 * ROW_BYTES);
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
    // ---- steady state: full main tiles -------------------------------------------
    // Step i works on tile t0 + i: activations in ring slot i % 3, weights in tile buffer i & 1.
    // Between its MFMAs a wave dequantizes its share of weight tile i + 1 (staged set (i + 1) & 1,
    // landed before the barrier that ended step i - 1) into the other tile buffer, and issues what
    // comes later: the words of tile i + 2 into set i & 1 and, one quarter per 16-deep step so that
    // the waves of a CU do not queue at the memory pipeline all at once, the direct loads of
    // activation tile i + 2 into the slot that every wave left at the last barrier.  The wait that
    // ends a step leaves exactly those four direct loads in flight: they have a whole further step
    // to land.
    if (t1 > t0) {
        const int last = t1 - 1;   // past the last tile the fetches repeat it; what they bring is never consumed
        issue_a(t0, 0);
        issue_a(t0 + 1 < t1 ? t0 + 1 : last, A_BYTES);
        load_w(wst[0], t0);
        wait_loads(wst[0], std::integral_constant<int, 0>());
        store_w(0, wst[0], -1);
        load_w(wst[1], t0 + 1 < t1 ? t0 + 1 : last);
        wait_loads(wst[1], std::integral_constant<int, 0>());
        __syncthreads();
        int a_cur = 0, a_nxt = A_BYTES, a_fill = 2 * A_BYTES;   // ring slots (byte offsets, wave-uniform)
        for (int t = t0; t < t1; t += 2) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int tt = t + u;
                if (tt < t1) {
                    const int ta = tt + 2 < t1 ? tt + 2 : last;
                    const int oa = offA0 + a_cur;
                    Frags f[2];
                    load_frags(f[0], oa, u, 0);
                    load_w(wst[u], ta);
#pragma unroll
                    for (int ks = 0; ks < RT / 16; ++ks) {
                        if (ks % G::A_EVERY == 0) issue_a_part(ta, a_fill, ks / G::A_EVERY);
                        if (ks + 1 < RT / 16) load_frags(f[(ks + 1) & 1], oa, u, ks + 1);
                        mfma_frags(f[ks & 1]);
                        store_w(u ^ 1, wst[u ^ 1], ks);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    wait_loads(wst[u], std::integral_constant<int, A_CH>());
                    __syncthreads();
                    const int freed = a_cur;
                    a_cur = a_nxt;
                    a_nxt = a_fill;
                    a_fill = freed;
                }
            }
        }
        // the repeated fetches of the last steps still write into the ring
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }

    // ---- tail: ragged last main tile and the adapter extension, one at a time, through
    // registers into buffer 0 (predicated; a handful of tiles at most) ---------------
    for (int t = takes_tail ? n_full : n_tiles; t < n_tiles; ++t) {
        const bool ext = t >= n_main;
        const int r0 = ext ? (t - n_main) * RT : t * RT;
        const int ld = ext ? a.RE : C;
        const uint16_t *abase = (ext ? a.act_ext + (size_t)m0 * ld : act_rowblock) + r0;
        unsigned char *As = smem, *Ws = smem + W_BASE;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int idx = i * THREADS + tid;
            const int row = idx >> 3, ch = idx & 7;
            int m = m0 + row;
            if (m > a.M - 1) m = a.M - 1;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (r0 + ch * 8 < ld) v = load_at<uint4>(abase, (uint32_t)(((size_t)(m - m0) * ld + ch * 8) * 2));
            *reinterpret_cast<uint4 *>(As + tile_off(row, ch)) = v;
        }
        if (ext) {
#pragma unroll
            for (int i = 0; i < W_CH; ++i) {
                const int idx = i * THREADS + tid;
                const int row = idx >> 3, ch = idx & 7;
                int c = c0 + row;
                if (c > Cout - 1) c = Cout - 1;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (r0 + ch * 8 < a.RE) v = *reinterpret_cast<const uint4 *>(a.w_ext + (size_t)c * a.RE + r0 + ch * 8);
                *reinterpret_cast<uint4 *>(Ws + tile_off(row, ch)) = v;
            }
        } else if (!BWD) {
            const int blk = t * 2 + fw_kb;
            const bool ok = blk * 32 < K;
            const int blk_c = ok ? blk : 0;
            const uint32_t *wbase = a.w.qweight + (size_t)blk_c * BITS * N;
#pragma unroll
            for (int j = 0; j < BITS; ++j) wst[0].fw_words[j] = load_at<uint32_t>(wbase + (size_t)j * N, fw_off);
            const size_t grow = (size_t)d.group_of_block((uint32_t)blk_c) * N;
            wst[0].fw_scale = ok ? (uint32_t)load_at<uint16_t>(a.w.scales + grow, fw_n * 2) : 0u;   // 0 -> weights +0
            if (F16) wst[0].fw_zero = ok ? (uint32_t)load_at<uint16_t>(a.zeros16 + grow, fw_n * 2) : 0u;
            else wst[0].fw_zero = load_at<uint8_t>(a.w.zeros + grow, fw_n);
            store_w(0, wst[0], -1);
        } else {
            const bool ok = r0 + (tid & 15) * 4 < N;
            WStage &st = wst[0];
            st.bw_lo = u32x4{0, 0, 0, 0};
            st.bw_hi = u32x4{0, 0, 0, 0};
            st.bw_scale = u32x2{0, 0};
            st.bw_zero = 0;
            st.bw_zero16 = u32x2{0, 0};
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
            store_w(0, st, -1);
        }
        __syncthreads();
        int ksteps = RT / 16;
        if (ext) {
            ksteps = (a.RE - r0) / 16;
            if (ksteps > RT / 16) ksteps = RT / 16;
        }
        for (int ks = 0; ks < ksteps; ++ks) {
            Frags f;
            load_frags(f, offA0, 0, ks);
            mfma_frags(f);
        }
        __syncthreads();
    }

    if (item.slice >= 0) {
        // a slice: leave the raw accumulators for gemm_big_fixup_kernel
        float4 *part = big_partial_of<MT>(a.partials, item.tile - plan.full, item.slice, plan.split) + tid;
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int j = 0; j < TJ; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    part[(size_t)(((i * TJ + j) * 4 + q) * THREADS)] =
                        make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        return;
    }
#pragma unroll
    for (int i = 0; i < TI; ++i) big_epilogue_rows<F16, WM>(acc[i], i, smem, a, Cout, m0, c0, wave, lane, wave);
}

// 8 TI single-wave workgroups per split tile (workgroup (y, z) stands in for wave z of the tile's
// workgroup and takes that wave's y-th block of 32 rows; whole-chip parallelism even for a few
// deeply split tiles): add the slices in slice order, then the common epilogue.
template <bool F16, int MT>
__global__ __launch_bounds__(64) void gemm_big_fixup_kernel(GemmDev d, BigPlan plan) {
    using namespace big;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // FIXUP_LDS bytes
    const int lane = threadIdx.x, wave = blockIdx.z, tid = wave * 64 + lane;
    const int tile = plan.full + blockIdx.x, i = blockIdx.y;
    const TileCoord tco = banded_tile<big::BAND>(tile, d.tiles_m, d.tiles_c);
    const int m0 = tco.tm * MT, c0 = tco.tc * CT;
    const int Cout = d.a.backward ? d.a.w.K : d.a.w.N;
    f32x16 acc[TJ];
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    // four slices' loads in flight at a time (a slice per round trip leaves the few workgroups of
    // a deep split waiting on memory latency), added in slice order
    constexpr int SB = 4;
    for (int sl0 = 0; sl0 < plan.split; sl0 += SB) {
        float4 v[SB][TJ * 4];
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (sl0 + u < plan.split) {
                const float4 *part = big_partial_of<MT>(d.a.partials, blockIdx.x, sl0 + u, plan.split) + tid;
#pragma unroll
                for (int e = 0; e < TJ * 4; ++e) v[u][e] = part[(size_t)((i * TJ * 4 + e) * THREADS)];
            }
        }
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            if (sl0 + u < plan.split) {
#pragma unroll
                for (int e = 0; e < TJ * 4; ++e) {
                    acc[e / 4][4 * (e % 4)] += v[u][e].x;
                    acc[e / 4][4 * (e % 4) + 1] += v[u][e].y;
                    acc[e / 4][4 * (e % 4) + 2] += v[u][e].z;
                    acc[e / 4][4 * (e % 4) + 3] += v[u][e].w;
                }
            }
        }
    }
    big_epilogue_rows<F16, MT / 2>(acc, i, smem, d.a, Cout, m0, c0, wave, lane, 0);
}

template <int BITS, bool BWD, bool F16, int MT>
static hipError_t launch_big_mt(const GemmArgs &a, BigPlan plan, hipStream_t stream) {
    const GemmDev d = make_gemm_dev(a, MT, big::CT);
    // no (or too little) scratch for partial tiles: whole tiles only
    if (a.partials == nullptr || a.partials_bytes < plan.partial_bytes()) plan.split = 1;
    const int whole = plan.split > 1 ? plan.full : plan.full + plan.tail;
    const int slices = plan.split > 1 ? plan.tail * plan.split : 0;
    const int blocks = ((whole + 7) / 8 + (slices + 7) / 8) * 8;
    const size_t lds_bytes = big::Geo<MT>::LDS_BYTES;
    auto kern = gemm_big_kernel<BITS, BWD, F16, MT>;
    static bool configured[64] = {};
    const hipError_t e = ensure_lds_limit(reinterpret_cast<const void *>(kern), lds_bytes, configured);
    if (e != hipSuccess) return e;
    const char *name = F16 ? (BWD ? "f16_gemm_bwd" : "f16_gemm_fwd")
                           : MT == 256 ? (BWD ? "gemm_bwd_256x256" : "gemm_fwd_256x256") : (BWD ? "gemm_bwd_128x256" : "gemm_fwd_128x256");
    launch_kernel(name, kern, blocks, big::THREADS, lds_bytes, stream, d, plan);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || plan.split <= 1) return err;
    // one wave's patch, and (F16, at the offset the epilogue expects) its 32 rows of P
    constexpr size_t FIXUP_LDS = F16 ? 40960 + 32 * 64 * 4 : 32 * big::PATCH_ROW * 2;
    auto fix = gemm_big_fixup_kernel<F16, MT>;
    static bool fix_configured[64] = {};
    const hipError_t e2 = ensure_lds_limit(reinterpret_cast<const void *>(fix), FIXUP_LDS, fix_configured);
    if (e2 != hipSuccess) return e2;
    const char *fix_name = F16 ? (BWD ? "f16_gemm_bwd_fixup" : "f16_gemm_fwd_fixup")
                               : MT == 256 ? (BWD ? "gemm_bwd_256x256_fixup" : "gemm_fwd_256x256_fixup")
                                           : (BWD ? "gemm_bwd_128x256_fixup" : "gemm_fwd_128x256_fixup");
    launch_kernel(fix_name, fix, dim3(plan.tail, big::Geo<MT>::TI, big::NWAVES), 64, FIXUP_LDS, stream, d, plan);
    return hipGetLastError();
}

template <int BITS, bool BWD, bool F16 = false>
static hipError_t launch_big(const GemmArgs &a, hipStream_t stream) {
    const int C = BWD ? a.w.N : a.w.K, Cout = BWD ? a.w.K : a.w.N;
    const BigPlan plan = big_plan(a.M, C, Cout);
    if (plan.mt == 128) return launch_big_mt<BITS, BWD, F16, 128>(a, plan, stream);
    return launch_big_mt<BITS, BWD, F16, 256>(a, plan, stream);
}

hipError_t launch_gemm_big(const GemmArgs &a, hipStream_t stream) {
    switch (a.w.bits) {
        case 2: return a.backward ? launch_big<2, true>(a, stream) : launch_big<2, false>(a, stream);
        case 3: return a.backward ? launch_big<3, true>(a, stream) : launch_big<3, false>(a, stream);
        default: return a.backward ? launch_big<4, true>(a, stream) : launch_big<4, false>(a, stream);
    }
}

hipError_t launch_gemm_big_f16(const GemmArgs &a, hipStream_t stream) {
    switch (a.w.bits) {
        case 2: return a.backward ? launch_big<2, true, true>(a, stream) : launch_big<2, false, true>(a, stream);
        case 3: return a.backward ? launch_big<3, true, true>(a, stream) : launch_big<3, false, true>(a, stream);
        default: return a.backward ? launch_big<4, true, true>(a, stream) : launch_big<4, false, true>(a, stream);
    }
}

}  // namespace mlr
