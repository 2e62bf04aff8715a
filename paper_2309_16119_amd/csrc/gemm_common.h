// Pieces shared by the tile GEMM kernels: tile order, the per-launch device
// arguments and small address helpers.
#pragma once
#include "device_common.h"
#include "launch.h"

namespace mlr {

struct TileCoord {
    int tm, tc;
};

// XCD-aware tile order: consecutive workgroup ids go round-robin over the 8 XCDs, so
// give each XCD a contiguous run of tiles, and walk tiles row-block-fastest inside a
// run so that neighbours on one XCD share the weight tile (and its L2 lines).
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

// Row block and column block of a linear tile index when the tiles are walked in bands of
// BAND row blocks, row-block-fastest inside a band: the ~32 tiles of consecutive index that
// one XCD runs at a time then span BAND activation panels and 32 / BAND weight panels.  An
// activation panel is 16 / bits times the bytes of a weight panel, so few rows and many
// columns keep the bytes that XCD pulls through its L2 lowest (2 rows: about a third of what
// a whole column of 16 row blocks costs).
template <int BAND>
__device__ __forceinline__ TileCoord banded_tile(int tile, int tiles_m, int tiles_c) {
    const int full = (tiles_m / BAND) * BAND * tiles_c;     // tiles in whole bands
    TileCoord tc;
    if (tile < full) {
        const int band = tile / (BAND * tiles_c), r = tile - band * (BAND * tiles_c);
        tc.tc = r / BAND;
        tc.tm = band * BAND + r % BAND;
    } else {
        const int rows = tiles_m % BAND, r = tile - full;   // the last, narrower band
        tc.tc = r / rows;
        tc.tm = (tiles_m / BAND) * BAND + r % rows;
    }
    return tc;
}

struct GemmDev {
    GemmArgs a;
    int tiles_m, tiles_c;
    // group index of a 32-code block: blk / (group/32), as one multiply-high with
    // magic = floor(2^32 / d) + 1 (exact for blk, d < 2^15); d == 1 is passed through
    uint32_t blocks_per_group, blocks_per_group_magic;
    __device__ __forceinline__ uint32_t group_of_block(uint32_t blk) const {
        return blocks_per_group == 1 ? blk : __umulhi(blk, blocks_per_group_magic);
    }
};



inline GemmDev make_gemm_dev(const GemmArgs &a, int MT, int CT) {
    const int Cout = a.backward ? a.w.K : a.w.N;
    GemmDev d;
    d.a = a;
    d.tiles_m = (a.M + MT - 1) / MT;
    d.tiles_c = (Cout + CT - 1) / CT;
    d.blocks_per_group = (uint32_t)(a.w.group / 32);
    d.blocks_per_group_magic = d.blocks_per_group > 1 ? (uint32_t)((1ull << 32) / d.blocks_per_group) + 1u : 0u;
    return d;
}

// Raise the dynamic-LDS limit of a kernel once per device (not a stream operation, but
// keep it out of the steady state and out of graph captures after the first call).
inline hipError_t ensure_lds_limit(const void *kernel, size_t lds_bytes, bool *configured /*[64]*/) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64 || !configured[dev]) {
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) configured[dev] = true;
    }
    return hipSuccess;
}

// One direct global->LDS load of 16 bytes per lane: lane i's data lands at
// lds_base + 16 i (lds_base wave-uniform, in M0).
__device__ __forceinline__ void load_to_lds_16(const void *gbase_uniform, uint32_t voff_bytes, uint32_t lds_base_uniform) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base_uniform), "v"(voff_bytes), "s"(gbase_uniform)
                 : "memory");
}

// Register loads issued from inline assembly (uniform base + per-lane byte offset).  The
// compiler does not know that they are in flight: every consumer must sit behind
// wait_loads(), which also ties the destination registers so that no use can be moved
// ahead of the wait.  This keeps the compiler from sprinkling conservative vmcnt waits
// (which would also wait for the direct loads) through the MFMA phase.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void aload_b32(uint32_t &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void aload_u16(uint32_t &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_ushort %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void aload_u8(uint32_t &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_ubyte %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void aload_b64(u32x2 &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}
__device__ __forceinline__ void aload_b128(u32x4 &dst, const void *base, uint32_t voff) {
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(base) : "memory");
}

// Two fp32 values rounded to nearest even into a pair of 16-bit floats, `lo` in the low half:
// bfloat16, or binary16 for the layer in the paper's own storage convention.
typedef _Float16 half16x2 __attribute__((ext_vector_type(2)));
template <bool F16>
__device__ __forceinline__ uint32_t pack_pair(float lo, float hi) {
    if (!F16) return pack_bf16x2(lo, hi);
    const half16x2 v = {(_Float16)lo, (_Float16)hi};
    uint32_t u;
    __builtin_memcpy(&u, &v, sizeof u);
    return u;
}

// Quarter j (0..3) of a 32-code block held in BITS words: its 8 codes dequantized with one
// (scale, bias) into 8 bfloat16 (or binary16), code 8 j in the low half of out[0].
template <int BITS, bool F16 = false>
__device__ __forceinline__ void dequant_quarter(const uint32_t *w, int j, const DqConst &c, uint32_t out[4]) {
    if (BITS == 4) {
        const uint32_t lo = w[j] & 0x0F0F0F0Fu, hi = (w[j] >> 4) & 0x0F0F0F0Fu;
#pragma unroll
        for (int i = 0; i < 4; ++i)   // codes 2i (byte i of lo) and 2i+1 (byte i of hi)
            out[i] = pack_pair<F16>(dq_value((lo >> (8 * i)) & 0xFFu, c), dq_value((hi >> (8 * i)) & 0xFFu, c));
    } else if (BITS == 2) {
        const uint32_t h = w[j >> 1] >> (16 * (j & 1));   // 8 codes in the low 16 bits
        const uint32_t even = h & 0x3333u, odd = (h >> 2) & 0x3333u;   // nibble n: code 2n / 2n+1
#pragma unroll
        for (int i = 0; i < 4; ++i)
            out[i] = pack_pair<F16>(dq_value((even >> (4 * i)) & 0xFu, c), dq_value((odd >> (4 * i)) & 0xFu, c));
    } else {
        const uint32_t chunk = block_chunk<BITS>(w, j);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            out[i] = pack_pair<F16>(dq_value(chunk_code<BITS>(chunk, 2 * i), c), dq_value(chunk_code<BITS>(chunk, 2 * i + 1), c));
    }
}

// gemm_big.hip: the 256x256 8-wave variant
hipError_t launch_gemm_big(const GemmArgs &a, hipStream_t stream);
// gemm_mid.hip: 128x64 tiles for grids of about one tile per CU, producer and consumer waves
hipError_t launch_gemm_mid(const GemmArgs &a, hipStream_t stream);

// The adapter term of a wave's block of 32 rows x (TJ x 32) columns in the epilogue (the layer in
// the paper's own storage convention adds s P F there, before the one rounding):
//   lora[j][v] = sum_jj P[row(v)][jj] F(jj, cc[j]),   row(v) = 8 (v / 4) + 4 (lane / 32) + v % 4,
// P fp32 [M][r] (rows first_row .. first_row + 31, clamped to M - 1), F = B [r][N] (forward) or A [K][r]
// (backward: F(jj, c) = A[c][jj]).  The block's rows of P pass through LDS (Ps: 32 x 64 floats,
// private to the wave), [jj][32 rows].  Loads go out eight at a time before anything waits for
// them: one round trip per eight rank columns instead of one per column.
template <int TJ>
__device__ __forceinline__ void adapter_term_32rows(const float *P, const float *F, int r, int N, bool bwd, int first_row, int M,
                                                    const int (&cc)[TJ], float *Ps, int lane, float (&lora)[TJ][16]) {
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) lora[j][v] = 0.f;
    if (r <= 0) return;
    for (int x0 = lane; x0 < 32 * r; x0 += 8 * 64) {
        float pv[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int x = x0 + 64 * t;
            const int prow = x & 31, jj = x >> 5;
            int m = first_row + prow;
            if (m > M - 1) m = M - 1;
            pv[t] = x < 32 * r ? P[(size_t)m * r + jj] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < 8; ++t)
            if (x0 + 64 * t < 32 * r) Ps[x0 + 64 * t] = pv[t];
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
    for (int jj0 = 0; jj0 < r; jj0 += 8) {
        float f[8][TJ];
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                const int jj = jj0 + q;
                f[q][j] = jj < r ? (bwd ? F[(size_t)cc[j] * r + jj] : F[(size_t)jj * N + cc[j]]) : 0.f;
            }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            if (jj0 + q < r) {
                // accumulator register v belongs to row 8 (v / 4) + 4 (lane / 32) + v % 4: four float4
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const float4 p = *reinterpret_cast<const float4 *>(Ps + (jj0 + q) * 32 + 8 * qq + 4 * (lane >> 5));
                    const float p4[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
                    for (int z = 0; z < 4; ++z)
#pragma unroll
                        for (int j = 0; j < TJ; ++j) lora[j][4 * qq + z] = __builtin_fmaf(p4[z], f[q][j], lora[j][4 * qq + z]);
                }
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);   // the next block of rows overwrites Ps
    __builtin_amdgcn_wave_barrier();
}

}  // namespace mlr
