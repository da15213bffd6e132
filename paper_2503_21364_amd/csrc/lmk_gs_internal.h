// Internal declarations shared by the translation units of liblmk_gs.so.
// Not part of the public ABI (include/lmk_gs.h is).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lmk_gs.h"

namespace lmk {

typedef uint64_t u64;
typedef uint32_t u32;

constexpr u32 kWave = 64;               // CDNA wavefront width
constexpr u32 kPreBlock = 256;          // primitives per preprocess / emit workgroup
constexpr u32 kSortThreads = 256;       // radix sort workgroup
constexpr u32 kSortItems = 16;          // keys per thread
constexpr u32 kSortTile = kSortThreads * kSortItems;   // 4096 pairs per workgroup pass
constexpr u32 kRadixBits = 8;
constexpr u32 kRadix = 1u << kRadixBits;
constexpr u32 kMaxPasses = 8;

// Header at the start of the scratch buffer.
struct ScratchHeader {
    u64 dup_count;      // D = sum of tiles_touched
    int32_t status;     // sticky LMK_GS_* code set by kernels
    int32_t pad;
};

// Carving of the caller's scratch buffer (all offsets multiples of 256 bytes).
struct ScratchLayout {
    size_t header;        // ScratchHeader
    size_t block_sums;    // u32 [pre_blocks]      tile counts per preprocess workgroup
    size_t block_offsets; // u64 [pre_blocks + 1]  their exclusive prefix sum
    size_t digit_totals;  // u64 [kMaxPasses][256] global digit histograms of each pass
    size_t table;         // u64 [256][sort_tiles] per-(digit, sort tile) counts, then offsets
    size_t total;
    u32 pre_blocks;
    u64 sort_tiles;       // ceil(capacity / kSortTile), row stride of `table`
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline ScratchLayout scratch_layout(u32 n, u64 capacity)
{
    ScratchLayout L;
    L.pre_blocks = (n + kPreBlock - 1) / kPreBlock;
    L.sort_tiles = (capacity + kSortTile - 1) / kSortTile;
    if (L.sort_tiles == 0) L.sort_tiles = 1;
    size_t o = 0;
    L.header = o;        o += align256(sizeof(ScratchHeader));
    L.block_sums = o;    o += align256(sizeof(u32) * (size_t)(L.pre_blocks + 1));
    L.block_offsets = o; o += align256(sizeof(u64) * ((size_t)L.pre_blocks + 1));
    L.digit_totals = o;  o += align256(sizeof(u64) * kMaxPasses * kRadix);
    L.table = o;         o += align256(sizeof(u64) * kRadix * (size_t)L.sort_tiles);
    L.total = o;
    return L;
}

// Number of 8-bit passes for keys of 32 depth bits + ceil(log2(tiles)) tile bits.
inline u32 sort_passes(u32 tiles)
{
    u32 tile_bits = 0;
    while ((1ull << tile_bits) < (u64)tiles) ++tile_bits;
    u32 bits = 32 + tile_bits;
    return (bits + kRadixBits - 1) / kRadixBits;
}

// Camera-derived kernel arguments (host-computed, passed by value).
struct ProjParams {
    lmk_gs_camera cam;
    float lim_x, lim_y;   // guard band on x/z, y/z for the EWA Jacobian
    u32 tiles_x, tiles_y;
};

// Launchers (each returns the hipError_t of its launches).
hipError_t launch_preprocess(const lmk_gs_gaussians &g, const ProjParams &pp, const lmk_gs_projected &out,
                             char *scratch, const ScratchLayout &L, hipStream_t stream);
hipError_t launch_bin_sort(const lmk_gs_projected &proj, u32 n, const ProjParams &pp, const lmk_gs_binned &out,
                           char *scratch, const ScratchLayout &L, hipStream_t stream);
hipError_t launch_render(const lmk_gs_projected &proj, const lmk_gs_binned &binned, const ProjParams &pp,
                         float *out_rgb, float *out_T, hipStream_t stream);

}  // namespace lmk
