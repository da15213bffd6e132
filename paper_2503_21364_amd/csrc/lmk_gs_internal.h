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
constexpr u32 kPreBlock = LMK_GS_PRE_BLOCK;   // primitives per preprocess workgroup
constexpr u32 kBinBlock = 2048;         // primitives per workgroup of the counting and emit kernels of stage 2
constexpr u32 kScanGroup = 256;         // preprocess workgroups per group of the two-level prefix sum
static_assert(kScanGroup % (kBinBlock / kPreBlock) == 0, "the blocks of one counting workgroup lie in one group");
// The counting and emit kernels keep one counter per tile in LDS: up to 8192 tiles (1080p has
// 8160) in 32 KB, up to 32768 (2160p has 32400) in 128 KB.  Larger images take the route of the
// large rectangles for every primitive: one global atomic per pair.
constexpr u32 kLdsTilesSmall = 8192, kLdsTilesLarge = 32768;
constexpr u32 kChunk = 4096;            // pairs sorted in LDS by one workgroup of the per-tile sort

// Header at the start of the scratch buffer.
struct ScratchHeader {
    u64 dup_count;      // D = pairs of the frame = sum of tiles_touched (known when lmk_gs_preprocess is done)
    int32_t status;     // LMK_GS_* code of the frame's latest stage 2 (LMK_GS_OK after stage 1)
    int32_t pad;
    u32 big_count;      // stage 2: primitives on the deferred list, from the front (one wavefront each)
    u32 giant_count;    // ... and from the back (one workgroup each)
    u32 pad2[2];
};

// Carving of the caller's scratch buffer (all offsets multiples of 256 bytes).  The part up to
// `bin_count` is what lmk_gs_preprocess touches; it depends on n and the image size only.
struct ScratchLayout {
    size_t header;        // ScratchHeader
    size_t tile_count;    // u32 [2][tiles + 1]  pairs per tile in the counting workgroups' runs / of the listed primitives:
                          //                     zero between frames, accumulated by the counting kernels
    size_t block_sums;    // u32 [pre_blocks]      tile counts per preprocess workgroup (256 primitives)
    size_t block_offsets; // u64 [pre_blocks + 1]  their exclusive prefix sum within groups of kScanGroup
    size_t group_totals;  // u64 [groups]          total of each group
    size_t voxel_flags;   // u8  [n]           voxel filter: 1 = the voxel may reach the image (at most n voxels)
    size_t tile_masks;    // u32 [n]           binning rule 1: kept tiles of rectangles of up to 32 tiles
    size_t bin_count;     // u32 [bin_blocks]  entries in each counting workgroup's list of (tile, start of its run)
    size_t tile_cursor;   // u32 [tiles + 1] running position of the listed primitives' pairs inside every tile's slice
    size_t big_idx;       // u32 [n]         deferred list: primitives whose rectangles are walked by wavefronts of their own
    size_t order;         // u32 [tiles]     tile ids by descending list length
    size_t classes;       // u32 [8]         tiles per size class of the per-tile sort (see tile_scan_kernel)
    size_t chunk_list;    // uint2 [capacity / 2048 + 2]  (tile, chunk) of every chunk of the lists sorted in chunks
    size_t total;
    u32 pre_blocks;       // ceil(n / kPreBlock)
    u32 bin_blocks;       // ceil(n / kBinBlock)
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline ScratchLayout scratch_layout(u32 n, u64 capacity, u32 tiles)
{
    ScratchLayout L;
    L.pre_blocks = (n + kPreBlock - 1) / kPreBlock;
    L.bin_blocks = (n + kBinBlock - 1) / kBinBlock;
    size_t o = 0;
    L.header = o;        o += align256(sizeof(ScratchHeader));
    L.tile_count = o;    o += align256(sizeof(u32) * 2 * ((size_t)tiles + 1));
    L.block_sums = o;    o += align256(sizeof(u32) * (size_t)(L.pre_blocks + 1));
    L.block_offsets = o; o += align256(sizeof(u64) * ((size_t)L.pre_blocks + 1));
    L.group_totals = o;  o += align256(sizeof(u64) * ((size_t)L.pre_blocks / kScanGroup + 2));
    L.voxel_flags = o;   o += align256((size_t)n + 1);
    L.tile_masks = o;    o += align256(sizeof(u32) * ((size_t)n + 1));
    L.bin_count = o;     o += align256(sizeof(u32) * ((size_t)L.bin_blocks + 1));
    L.tile_cursor = o;   o += align256(sizeof(u32) * ((size_t)tiles + 1));
    L.big_idx = o;       o += align256(sizeof(u32) * ((size_t)n + 1));
    L.order = o;         o += align256(sizeof(u32) * (size_t)(tiles + 1));
    L.classes = o;       o += align256(sizeof(u32) * 8);
    L.chunk_list = o;    o += align256(sizeof(u32) * 2 * (size_t)(capacity / 2048 + 2));
    L.total = o;
    return L;
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
