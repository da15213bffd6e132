// Stage 3: per-tile front-to-back alpha compositing (Sec. 2.2 Eq. 9-10; the
// blend kernel whose share of render time Sec. 4.2.1 reports).
//
// One workgroup of 256 threads (4 wavefronts) per 16x16 tile, one pixel per
// lane; wavefront w owns rows 4w..4w+3 of the tile.  The tile's sorted list is
// consumed in batches of 256 entries: each thread fetches one entry's feature
// record (48 bytes, three 16-byte loads) and stages it in LDS with the conic
// pre-multiplied by -0.5*log2(e), so the inner loop is a handful of FMAs and
// one v_exp_f32 per (pixel, entry).  A wavefront whose 64 pixels have all
// stopped skips the rest of a batch; the tile leaves when all four have.
// Bound by FP32 VALU issue; LDS reads are wavefront-wide broadcasts.
#include "lmk_gs_internal.h"

namespace lmk {

constexpr u32 kBlendThreads = 256;
constexpr u32 kBatch = 256;
constexpr u32 kXcds = 8;     // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

struct BlendParams {
    u32 width, height, tiles_x, num_tiles, tiles_per_xcd;
    float bg0, bg1, bg2;
};

__global__ __launch_bounds__(kBlendThreads) void blend_kernel(
    const u64 *__restrict__ tile_offsets, const u32 *__restrict__ vals,
    const float4 *__restrict__ feat, BlendParams bp,
    float *__restrict__ out_rgb, float *__restrict__ out_T)
{
    __shared__ float4 s_geo[kBatch];    // u, v, A', B'   (A' = -0.5*log2e*A, B' = -log2e*B)
    __shared__ float4 s_col[kBatch];    // C', opacity, r, g
    __shared__ float s_blue[kBatch];

    // consecutive workgroup ids land on different XCDs; give each XCD one
    // contiguous band of tiles so neighbouring tiles share that XCD's L2
    const u32 tile = (blockIdx.x % kXcds) * bp.tiles_per_xcd + blockIdx.x / kXcds;
    if (blockIdx.x / kXcds >= bp.tiles_per_xcd || tile >= bp.num_tiles) return;

    const u32 tid = threadIdx.x;
    const u32 tx = tile % bp.tiles_x, ty = tile / bp.tiles_x;
    const u32 pxi = tx * LMK_GS_TILE + (tid & 15u), pyi = ty * LMK_GS_TILE + (tid >> 4);
    const bool inside = pxi < bp.width && pyi < bp.height;
    const float px = (float)pxi + 0.5f, py = (float)pyi + 0.5f;

    const u64 start = tile_offsets[tile], end = tile_offsets[tile + 1];
    float T = 1.0f, cr = 0.0f, cg = 0.0f, cb = 0.0f;
    bool done = !inside;
    const float kL2E = 1.4426950408889634f;

    for (u64 base = start; base < end; base += kBatch) {
        if (__syncthreads_and(done)) break;
        const u32 cnt = (u32)((end - base) < (u64)kBatch ? (end - base) : (u64)kBatch);
        if (tid < cnt) {
            const u32 g = vals[base + tid];
            const float4 *f = feat + (size_t)g * (LMK_GS_FEAT_STRIDE / 4);
            const float4 f0 = f[0], f1 = f[1], f2 = f[2];
            s_geo[tid] = make_float4(f0.x, f0.y, -0.5f * kL2E * f0.z, -kL2E * f0.w);
            s_col[tid] = make_float4(-0.5f * kL2E * f1.x, f1.y, f1.z, f1.w);
            s_blue[tid] = f2.x;
        }
        __syncthreads();
        for (u32 j = 0; j < cnt; ++j) {
            // wavefront-wide vote at a uniform point: leave the batch once all 64 pixels stopped
            if (__ballot(!done) == 0ull) break;
            const float4 ge = s_geo[j];
            const float4 co = s_col[j];
            const float dx = ge.x - px, dy = ge.y - py;
            // log2 of the Gaussian falloff: A' dx^2 + B' dx dy + C' dy^2  (<= 0 up to rounding)
            float p = dx * (ge.z * dx + ge.w * dy) + co.x * dy * dy;
            p = fminf(p, 0.0f);
            const float alpha = fminf(0.99f, co.y * __builtin_amdgcn_exp2f(p));
            const float Tn = T * (1.0f - alpha);
            const bool hit = !done && !(alpha < 1.0f / 255.0f);
            const bool stop = hit && Tn < 1e-4f;
            done = done || stop;
            if (hit && !stop) {
                const float w = alpha * T;
                cr += co.z * w; cg += co.w * w; cb += s_blue[j] * w;
                T = Tn;
            }
        }
    }
    if (inside) {
        const size_t plane = (size_t)bp.width * bp.height;
        const size_t p = (size_t)pyi * bp.width + pxi;
        out_rgb[p] = cr + T * bp.bg0;
        out_rgb[plane + p] = cg + T * bp.bg1;
        out_rgb[2 * plane + p] = cb + T * bp.bg2;
        out_T[p] = T;
    }
}

hipError_t launch_render(const lmk_gs_projected &proj, const lmk_gs_binned &binned, const ProjParams &pp,
                         float *out_rgb, float *out_T, hipStream_t stream)
{
    BlendParams bp;
    bp.width = pp.cam.width; bp.height = pp.cam.height;
    bp.tiles_x = pp.tiles_x; bp.num_tiles = pp.tiles_x * pp.tiles_y;
    bp.tiles_per_xcd = (bp.num_tiles + kXcds - 1) / kXcds;
    bp.bg0 = pp.cam.bg[0]; bp.bg1 = pp.cam.bg[1]; bp.bg2 = pp.cam.bg[2];
    hipLaunchKernelGGL(blend_kernel, dim3(bp.tiles_per_xcd * kXcds), dim3(kBlendThreads), 0, stream,
                       binned.tile_offsets, binned.vals, reinterpret_cast<const float4 *>(proj.feat), bp,
                       out_rgb, out_T);
    return hipGetLastError();
}

}  // namespace lmk
