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
constexpr u32 kPreBlock = LMK_GS_PRE_BLOCK;   // primitives per preprocess / emit workgroup
constexpr u32 kSortThreads = 256;       // radix sort workgroup
// Keys per thread of the partition kernels, so 2048 or 4096 pairs per sort tile.  With few sort
// tiles a pass is bound by the latency of one workgroup and smaller tiles spread better over
// the chip; with very many it is bound by HBM and the longer runs of a larger tile fill the
// lines they write.  The host picks from the capacity, which it knows (D it does not).
constexpr u32 kSortItemsFew = 8, kSortItemsMany = 16;
constexpr u64 kManyPairs = 64ull << 20;
inline u32 sort_items(u64 capacity) { return capacity > kManyPairs ? kSortItemsMany : kSortItemsFew; }
inline u32 sort_tile_pairs(u64 capacity) { return kSortThreads * sort_items(capacity); }
constexpr u32 kMaxRadixBits = 8;         // digits are at most 8 bits wide, chosen per frame
constexpr u32 kMaxRadix = 1u << kMaxRadixBits;
constexpr u32 kMaxPasses = 8;
constexpr u32 kScanGroup = 256;         // preprocess workgroups per group of the two-level prefix sum
constexpr u32 kTotalCopies = 4;         // copies of each pass's digit totals, to spread the atomics

// Header at the start of the scratch buffer.
struct ScratchHeader {
    u64 dup_count;      // D = sum of tiles_touched
    int32_t status;     // sticky LMK_GS_* code set by kernels
    int32_t pad;
    u32 big_count;      // emit stage: deferred primitives expanded one wavefront each (front of the list)
    u32 giant_count;    // ... and one workgroup each (back of the list)
};

// Carving of the caller's scratch buffer (all offsets multiples of 256 bytes).
struct ScratchLayout {
    size_t header;        // ScratchHeader
    size_t block_sums;    // u32 [pre_blocks]      tile counts per preprocess workgroup
    size_t block_offsets; // u64 [pre_blocks + 1]  their exclusive prefix sum within groups of kScanGroup
    size_t group_totals;  // u64 [groups]          total of each group
    size_t voxel_flags;   // u8  [n]               voxel filter: 1 = the voxel may reach the image (at most n voxels)
    size_t tile_masks;    // u32 [n]               binning rule 1: kept tiles of rectangles of up to 32 tiles
    size_t digit_totals;  // u64 [kMaxPasses][kTotalCopies][kMaxRadix] digit totals of each pass
    size_t table;         // u32 [512][sort_tiles] per-(digit, sort tile) counts of the running pass
    size_t offsets;       // u64 [512][sort_tiles] their output offsets
    size_t order;         // u32 [tiles]     tile ids by descending list length
    size_t classes;       // u32 [8]         tiles per size class of the per-tile sort (see tile_order_kernel)
    size_t chunk_list;    // uint2 [capacity / 2048 + 2]  (tile, chunk) of every chunk of the lists sorted in chunks
    size_t big_idx;       // u32 [n]         primitives whose rectangles are expanded one wavefront each
    size_t big_off;       // u64 [n]         and where their pairs start
    size_t total;
    u32 pre_blocks;
    u64 sort_tiles;       // ceil(capacity / sort_tile_pairs(capacity))
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline ScratchLayout scratch_layout(u32 n, u64 capacity, u32 tiles)
{
    ScratchLayout L;
    L.pre_blocks = (n + kPreBlock - 1) / kPreBlock;
    L.sort_tiles = (capacity + sort_tile_pairs(capacity) - 1) / sort_tile_pairs(capacity);
    if (L.sort_tiles == 0) L.sort_tiles = 1;
    size_t o = 0;
    L.header = o;        o += align256(sizeof(ScratchHeader));
    L.block_sums = o;    o += align256(sizeof(u32) * (size_t)(L.pre_blocks + 1));
    L.block_offsets = o; o += align256(sizeof(u64) * ((size_t)L.pre_blocks + 1));
    L.group_totals = o;  o += align256(sizeof(u64) * ((size_t)L.pre_blocks / kScanGroup + 2));
    L.voxel_flags = o;   o += align256((size_t)n + 1);
    L.tile_masks = o;    o += align256(sizeof(u32) * ((size_t)n + 1));
    L.digit_totals = o;  o += align256(sizeof(u64) * kMaxPasses * kTotalCopies * kMaxRadix);
    L.table = o;         o += align256(sizeof(u32) * kMaxRadix * (size_t)L.sort_tiles);
    L.offsets = o;       o += align256(sizeof(u64) * kMaxRadix * (size_t)L.sort_tiles);
    L.order = o;         o += align256(sizeof(u32) * (size_t)(tiles + 1));
    L.classes = o;       o += align256(sizeof(u32) * 8);
    L.chunk_list = o;    o += align256(sizeof(u32) * 2 * (size_t)(capacity / 2048 + 2));
    L.big_idx = o;       o += align256(sizeof(u32) * ((size_t)n + 1));
    L.big_off = o;       o += align256(sizeof(u64) * ((size_t)n + 1));
    L.total = o;
    return L;
}

// The pairs are first partitioned by tile id with a stable LSD radix sort over the tile bits
// only (digits of at most 8 bits: 7 + 6 at 1080p, 8 + 7 at 2160p, one pass at 256 x 256),
// then every tile's list is sorted by (depth, index) on its own.
constexpr u32 kChunk = 4096;             // pairs sorted in LDS by one workgroup

struct SortPlan {
    u32 passes;
    u32 shift[kMaxPasses];
    u32 bits[kMaxPasses];
};

inline SortPlan sort_plan(u32 tiles)
{
    u32 tile_bits = 0;
    while ((1ull << tile_bits) < (u64)tiles) ++tile_bits;
    SortPlan P;
    P.passes = (tile_bits + kMaxRadixBits - 1) / kMaxRadixBits;
    const u32 base = P.passes ? tile_bits / P.passes : 0, extra = P.passes ? tile_bits % P.passes : 0;
    u32 at = 32;
    for (u32 p = 0; p < kMaxPasses; ++p) {
        P.shift[p] = at;
        P.bits[p] = p < P.passes ? base + (p < extra ? 1u : 0u) : 0u;
        at += P.bits[p];
    }
    return P;
}

// Camera-derived kernel arguments (host-computed, passed by value).
struct ProjParams {
    lmk_gs_camera cam;
    float lim_x, lim_y;   // guard band on x/z, y/z for the EWA Jacobian
    u32 tiles_x, tiles_y;
    float tau_tab[8];     // binning rule 1: 2 (ln 255 + ln(1 + (k+1)/8)) + 0.01, k = top 3 mantissa bits of opacity
};

// Launchers (each returns the hipError_t of its launches).
// index == nullptr: every primitive is processed; else the voxel filter runs first and the
// per-workgroup decisions are also written to block_visible when that is not nullptr
hipError_t launch_preprocess(const lmk_gs_gaussians &g, const lmk_gs_voxel_index *index, uint8_t *block_visible,
                             const ProjParams &pp, const lmk_gs_projected &out,
                             char *scratch, const ScratchLayout &L, hipStream_t stream);
// the scratch contents lmk_gs_bin_sort expects from lmk_gs_preprocess, recomputed from proj alone
hipError_t launch_rebuild_handover(const lmk_gs_projected &proj, u32 n, const ProjParams &pp,
                                   char *scratch, const ScratchLayout &L, hipStream_t stream);
// out[0] = D, out[1] = status (sign-extended) from the scratch header
hipError_t launch_copy_status(const char *scratch, const ScratchLayout &L, u64 *out, hipStream_t stream);
hipError_t launch_build_cov3d(const lmk_gs_gaussians &g, float *cov3d, hipStream_t stream);
hipError_t launch_bin_sort(const lmk_gs_projected &proj, u32 n, const ProjParams &pp, const lmk_gs_binned &out,
                           char *scratch, const ScratchLayout &L, hipStream_t stream);
hipError_t launch_render(const lmk_gs_projected &proj, const lmk_gs_binned &binned, const ProjParams &pp,
                         float *out_rgb, float *out_T, hipStream_t stream);
hipError_t launch_render_backward(const lmk_gs_projected &proj, u32 n, const lmk_gs_binned &binned,
                                  const ProjParams &pp, const float *grad_rgb, const float *grad_T,
                                  float *grad_feat, hipStream_t stream);
hipError_t launch_preprocess_backward(const lmk_gs_gaussians &g, const ProjParams &pp,
                                      const lmk_gs_projected &proj, const float *grad_feat,
                                      const lmk_gs_gaussian_grads &out, hipStream_t stream);
hipError_t launch_anchor_decode(const lmk_gs_anchors &anchors, const lmk_gs_anchor_decoder &decoder,
                                const float *cam_pos, const u32 *visible, u32 v, const uint8_t *anchor_visible,
                                const lmk_gs_decoded &out, hipStream_t stream);
// visible[i] = the box (lo, hi, reach of the scales) passes the frustum test of the voxel filter
hipError_t launch_box_flags(const float *box, u32 count, const ProjParams &pp, uint8_t *visible, hipStream_t stream);

}  // namespace lmk
