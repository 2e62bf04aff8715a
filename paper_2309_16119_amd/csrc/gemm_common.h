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

// gemm_big.hip: the 256x256 double-buffered 8-wave variant
hipError_t launch_gemm_big(const GemmArgs &a, hipStream_t stream);

}  // namespace mlr
