// Offline voxel reordering of a scene (host code only; Sec. 4.2.2, frustum-based dynamic
// loading).  Once, before any frame, the primitives are sorted by the cell of a regular grid that
// holds their centre, so that a voxel is a run of consecutive primitives; per frame the voxels,
// not the primitives, are then tested against the view frustum.
#include "lmk_gs_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

namespace {

// interleave the low 21 bits of x, y, z: bit b of x lands at 3b, of y at 3b + 1, of z at 3b + 2
uint64_t spread3(uint64_t v)
{
    v &= 0x1fffffull;
    v = (v | (v << 32)) & 0x001f00000000ffffull;
    v = (v | (v << 16)) & 0x001f0000ff0000ffull;
    v = (v | (v << 8)) & 0x100f00f00f00f00full;
    v = (v | (v << 4)) & 0x10c30c30c30c30c3ull;
    v = (v | (v << 2)) & 0x1249249249249249ull;
    return v;
}

}  // namespace

extern "C" int32_t lmk_gs_index_build(const float *mean, const float *scale, uint32_t n, float voxel_size,
                                      uint32_t *perm, uint32_t *first, float *box, uint32_t *block_range,
                                      uint32_t *num_voxels)
{
    if (!num_voxels) return LMK_GS_ERR_INVALID;
    *num_voxels = 0;
    if (!(voxel_size > 0.0f) || !std::isfinite(voxel_size)) return LMK_GS_ERR_INVALID;
    if (n == 0) { if (first) first[0] = 0; return LMK_GS_OK; }
    if (!mean || !scale || !perm || !first || !box || !block_range) return LMK_GS_ERR_INVALID;
    const size_t N = n;

    // cell coordinates, relative to the smallest cell on each axis
    std::vector<int64_t> cell(3 * N);
    int64_t lo[3], hi[3];
    for (int a = 0; a < 3; ++a) {
        lo[a] = std::numeric_limits<int64_t>::max();
        hi[a] = std::numeric_limits<int64_t>::min();
        for (size_t i = 0; i < N; ++i) {
            const float m = mean[a * N + i];
            if (!std::isfinite(m)) return LMK_GS_ERR_INVALID;
            const float q = m / voxel_size;                      // one fp32 rounding, then floor
            if (!(std::fabs(q) < 9.0e15f)) return LMK_GS_ERR_UNSUPPORTED;
            const int64_t c = (int64_t)std::floor(q);
            cell[a * N + i] = c;
            lo[a] = std::min(lo[a], c);
            hi[a] = std::max(hi[a], c);
        }
        if (hi[a] - lo[a] >= (int64_t)1 << 21) return LMK_GS_ERR_UNSUPPORTED;
    }
    std::vector<uint64_t> key(N);
    for (size_t i = 0; i < N; ++i)
        key[i] = spread3((uint64_t)(cell[i] - lo[0])) | (spread3((uint64_t)(cell[N + i] - lo[1])) << 1) |
                 (spread3((uint64_t)(cell[2 * N + i] - lo[2])) << 2);
    for (uint32_t i = 0; i < n; ++i) perm[i] = i;
    std::sort(perm, perm + n, [&](uint32_t a, uint32_t b) { return key[a] != key[b] ? key[a] < key[b] : a < b; });

    // voxels = runs of equal key; their boxes, reach and the voxel range of every group of primitives
    uint32_t nv = 0;
    for (uint32_t k = 0; k < n; ++k) {
        const uint32_t i = perm[k];
        if (k == 0 || key[i] != key[perm[k - 1]]) {
            first[nv] = k;
            float *b = box + 8 * (size_t)nv;
            b[0] = b[3] = mean[i]; b[1] = b[4] = mean[N + i]; b[2] = b[5] = mean[2 * N + i];
            b[6] = 0.0f; b[7] = 0.0f;
            ++nv;
        }
        float *b = box + 8 * (size_t)(nv - 1);
        for (int a = 0; a < 3; ++a) {
            const float m = mean[a * N + i];
            b[a] = std::min(b[a], m);
            b[3 + a] = std::max(b[3 + a], m);
            b[6] = std::max(b[6], std::fabs(scale[a * N + i]));
        }
        if (k % LMK_GS_PRE_BLOCK == 0) block_range[2 * (size_t)(k / LMK_GS_PRE_BLOCK)] = nv - 1;
        if (k % LMK_GS_PRE_BLOCK == LMK_GS_PRE_BLOCK - 1 || k == n - 1)
            block_range[2 * (size_t)(k / LMK_GS_PRE_BLOCK) + 1] = nv - 1;
    }
    first[nv] = n;
    *num_voxels = nv;
    return LMK_GS_OK;
}

extern "C" int32_t lmk_gs_anchor_index_build(const float *position, const float *extent, const float *offsets,
                                             uint32_t a, uint32_t k, float *box, uint32_t *block_range)
{
    if (k == 0) return LMK_GS_ERR_INVALID;
    if ((uint64_t)a * k >= (1ull << 32)) return LMK_GS_ERR_INVALID;
    if (a == 0) return LMK_GS_OK;
    if (!position || !extent || !offsets || !box || !block_range) return LMK_GS_ERR_INVALID;
    const size_t A = a;
    for (size_t i = 0; i < A; ++i) {
        float reach[3] = {0.0f, 0.0f, 0.0f};
        for (uint32_t j = 0; j < k; ++j)
            for (int c = 0; c < 3; ++c) {
                const float r = std::fabs(offsets[(i * k + j) * 3 + c]) * extent[c * A + i];
                // a NaN reach must not be lost in the comparison
                if (!(r <= reach[c])) reach[c] = r;
            }
        float *b = box + 8 * i;
        for (int c = 0; c < 3; ++c) {
            const float centre = position[c * A + i];
            b[c] = centre - reach[c];
            b[3 + c] = centre + reach[c];
        }
        float smax = extent[3 * A + i];
        for (int c = 4; c < 6; ++c)
            if (!(extent[c * A + i] <= smax)) smax = extent[c * A + i];
        b[6] = smax;
        b[7] = 0.0f;
    }
    const uint64_t n = (uint64_t)a * k;
    const uint64_t groups = (n + LMK_GS_PRE_BLOCK - 1) / LMK_GS_PRE_BLOCK;
    for (uint64_t g = 0; g < groups; ++g) {
        const uint64_t s0 = g * LMK_GS_PRE_BLOCK;
        const uint64_t s1 = s0 + LMK_GS_PRE_BLOCK - 1 < n - 1 ? s0 + LMK_GS_PRE_BLOCK - 1 : n - 1;
        block_range[2 * g] = (uint32_t)(s0 / k);
        block_range[2 * g + 1] = (uint32_t)(s1 / k);
    }
    return LMK_GS_OK;
}
