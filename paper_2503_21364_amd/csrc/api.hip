// extern "C" entry points of liblmk_gs.so: argument validation on the host,
// then kernel launches on the caller's stream.  See include/lmk_gs.h for the
// contract of each call.
#include "lmk_gs_internal.h"

#include <atomic>
#include <cmath>
#include <mutex>

using namespace lmk;

namespace {

std::atomic<int32_t> g_last_hip_error{0};

int32_t hip_fail(hipError_t e)
{
    g_last_hip_error.store((int32_t)e);
    return LMK_GS_ERR_HIP;
}

bool finite_all(const float *p, int n)
{
    for (int i = 0; i < n; ++i)
        if (!std::isfinite(p[i])) return false;
    return true;
}

constexpr uint32_t kMaxTilesPerAxis = 4096;      // 65536 pixels per axis
constexpr uint32_t kMaxTiles = 1u << 22;         // keeps a workgroup's tile count inside 32 bits

int32_t check_camera(const lmk_gs_camera *cam, ProjParams *pp)
{
    if (!cam) return LMK_GS_ERR_INVALID;
    if (cam->tile != LMK_GS_TILE) return LMK_GS_ERR_UNSUPPORTED;
    if (cam->width == 0 || cam->height == 0) return LMK_GS_ERR_INVALID;
    if (!finite_all(cam->view, 12) || !finite_all(cam->cam_pos, 3) || !finite_all(cam->bg, 3) ||
        !finite_all(&cam->fx, 4) || !std::isfinite(cam->near_z) || !std::isfinite(cam->lowpass))
        return LMK_GS_ERR_INVALID;
    if (!(cam->fx > 0.0f) || !(cam->fy > 0.0f) || !(cam->near_z > 0.0f) || !(cam->lowpass >= 0.0f))
        return LMK_GS_ERR_INVALID;
    const uint32_t tx = (cam->width + LMK_GS_TILE - 1) / LMK_GS_TILE;
    const uint32_t ty = (cam->height + LMK_GS_TILE - 1) / LMK_GS_TILE;
    if (tx > kMaxTilesPerAxis || ty > kMaxTilesPerAxis || (uint64_t)tx * ty > kMaxTiles)
        return LMK_GS_ERR_UNSUPPORTED;
    pp->cam = *cam;
    // guard band of the EWA Jacobian: 1.3 x the half-frustum tangent
    pp->lim_x = 1.3f * ((0.5f * (float)cam->width) / cam->fx);
    pp->lim_y = 1.3f * ((0.5f * (float)cam->height) / cam->fy);
    pp->tiles_x = tx;
    pp->tiles_y = ty;
    if (cam->binning > 1u) return LMK_GS_ERR_INVALID;
    for (int k = 0; k < 8; ++k)
        pp->tau_tab[k] = (float)(2.0 * (std::log(255.0) + std::log(1.0 + (k + 1) / 8.0)) + 0.01);
    return LMK_GS_OK;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// ---- the scratch of lmk_gs_bin_sort_static: one array per GPU, part of the loaded code object.
// `static_scratch` is only a host-side handle of the symbol; the device address comes from
// hipGetSymbolAddress, once per device, and only that address is ever handed to a kernel.
constexpr uint32_t kStaticMaxN = LMK_GS_STATIC_MAX_N;
constexpr uint64_t kStaticMaxCapacity = LMK_GS_STATIC_MAX_CAPACITY;
constexpr uint32_t kStaticMaxTiles = LMK_GS_STATIC_MAX_TILES;
constexpr size_t kStaticBytes = 96u << 20;
static __device__ __align__(256) unsigned char static_scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
char *g_static_ptr[kMaxDevices] = {};

// device address of this GPU's copy of the array (the current device's), or nullptr with *err set
char *static_scratch_ptr(hipError_t *err)
{
    int dev = 0;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch));
        if (*err != hipSuccess) return nullptr;
        g_static_ptr[dev] = static_cast<char *>(p);
    }
    return g_static_ptr[dev];
}

}  // namespace

extern "C" {

int32_t lmk_gs_workspace_bytes(uint32_t n, uint32_t width, uint32_t height, uint64_t capacity,
                               size_t *scratch_bytes)
{
    if (!scratch_bytes || width == 0 || height == 0) return LMK_GS_ERR_INVALID;
    const uint32_t tx = (width + LMK_GS_TILE - 1) / LMK_GS_TILE;
    const uint32_t ty = (height + LMK_GS_TILE - 1) / LMK_GS_TILE;
    if (tx > kMaxTilesPerAxis || ty > kMaxTilesPerAxis || (uint64_t)tx * ty > kMaxTiles)
        return LMK_GS_ERR_UNSUPPORTED;
    *scratch_bytes = scratch_layout(n, capacity, tx * ty).total;
    return LMK_GS_OK;
}

static int32_t preprocess_common(const lmk_gs_gaussians *g, const lmk_gs_voxel_index *index, uint8_t *block_visible,
                                 const lmk_gs_camera *cam, const lmk_gs_projected *out,
                                 void *scratch, size_t scratch_bytes, void *stream)
{
    ProjParams pp;
    const int32_t rc = check_camera(cam, &pp);
    if (rc != LMK_GS_OK) return rc;
    if (!g || !out || !scratch) return LMK_GS_ERR_INVALID;
    if (g->sh_degree > 3) return LMK_GS_ERR_INVALID;
    if (g->n > 0) {
        if (!g->mean || !g->opacity || !g->sh) return LMK_GS_ERR_INVALID;
        if (!g->cov3d && (!g->scale || !g->rot)) return LMK_GS_ERR_INVALID;
        if (!out->depth || !out->tiles_touched || !out->rect || !out->feat) return LMK_GS_ERR_INVALID;
        if (!aligned(out->feat, 16) || !aligned(out->rect, 8) || !aligned(g->sh, 16)) return LMK_GS_ERR_INVALID;
        if (index) {
            if (!index->box || !index->block_range || index->num_voxels == 0 || index->num_voxels > g->n)
                return LMK_GS_ERR_INVALID;
            if (!aligned(index->box, 16) || !aligned(index->block_range, 8)) return LMK_GS_ERR_INVALID;
            // the bound on a splat's support assumes a rigid camera: rows of the 3x3 part orthonormal
            const float *V = cam->view;
            for (int r = 0; r < 3; ++r)
                for (int c = r; c < 3; ++c) {
                    const double d = (double)V[4 * r] * V[4 * c] + (double)V[4 * r + 1] * V[4 * c + 1] +
                                     (double)V[4 * r + 2] * V[4 * c + 2];
                    if (std::fabs(d - (r == c ? 1.0 : 0.0)) > 1e-3) return LMK_GS_ERR_UNSUPPORTED;
                }
        }
    }
    if (!aligned(scratch, 256)) return LMK_GS_ERR_INVALID;
    // the part of the scratch this call touches does not depend on the pair capacity
    const ScratchLayout L = scratch_layout(g->n, 0, pp.tiles_x * pp.tiles_y);
    if (scratch_bytes < L.bin_count) return LMK_GS_ERR_CAPACITY;
    const hipError_t e = launch_preprocess(*g, g->n > 0 ? index : nullptr, block_visible, pp, *out,
                                           static_cast<char *>(scratch), L, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LMK_GS_OK : hip_fail(e);
}

int32_t lmk_gs_preprocess(const lmk_gs_gaussians *g, const lmk_gs_camera *cam,
                          const lmk_gs_projected *out, void *scratch, size_t scratch_bytes,
                          void *stream)
{
    return preprocess_common(g, nullptr, nullptr, cam, out, scratch, scratch_bytes, stream);
}

int32_t lmk_gs_build_cov3d(const lmk_gs_gaussians *g, float *cov3d, void *stream)
{
    if (!g) return LMK_GS_ERR_INVALID;
    if (g->n > 0 && (!g->scale || !g->rot || !cov3d)) return LMK_GS_ERR_INVALID;
    const hipError_t e = launch_build_cov3d(*g, cov3d, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LMK_GS_OK : hip_fail(e);
}

int32_t lmk_gs_preprocess_culled(const lmk_gs_gaussians *g, const lmk_gs_voxel_index *index,
                                 const lmk_gs_camera *cam, const lmk_gs_projected *out,
                                 uint8_t *block_visible,
                                 void *scratch, size_t scratch_bytes, void *stream)
{
    if (!index) return LMK_GS_ERR_INVALID;
    return preprocess_common(g, index, block_visible, cam, out, scratch, scratch_bytes, stream);
}

int32_t lmk_gs_bin_sort(const lmk_gs_projected *proj, uint32_t n, const lmk_gs_camera *cam,
                        const lmk_gs_binned *out, void *scratch, size_t scratch_bytes, void *stream)
{
    ProjParams pp;
    const int32_t rc = check_camera(cam, &pp);
    if (rc != LMK_GS_OK) return rc;
    if (!proj || !out || !scratch) return LMK_GS_ERR_INVALID;
    if (n > 0 && (!proj->depth || !proj->tiles_touched || !proj->rect)) return LMK_GS_ERR_INVALID;
    if (n > 0 && cam->binning == 1u && (!proj->feat || !aligned(proj->feat, 16))) return LMK_GS_ERR_INVALID;
    if (!out->tile_offsets) return LMK_GS_ERR_INVALID;
    if (out->capacity > 0 && (!out->keys || !out->vals || !out->keys_alt || !out->vals_alt))
        return LMK_GS_ERR_INVALID;
    if (!aligned(scratch, 256) || !aligned(proj->rect, 8)) return LMK_GS_ERR_INVALID;
    const ScratchLayout L = scratch_layout(n, out->capacity, pp.tiles_x * pp.tiles_y);
    if (scratch_bytes < L.total) return LMK_GS_ERR_CAPACITY;
    const hipError_t e = launch_bin_sort(*proj, n, pp, *out, static_cast<char *>(scratch), L,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LMK_GS_OK : hip_fail(e);
}

int32_t lmk_gs_bin_sort_static(const lmk_gs_projected *proj, uint32_t n, const lmk_gs_camera *cam,
                               const lmk_gs_binned *out, uint64_t *count_status, void *stream)
{
    ProjParams pp;
    const int32_t rc = check_camera(cam, &pp);
    if (rc != LMK_GS_OK) return rc;
    if (!proj || !out) return LMK_GS_ERR_INVALID;
    if (n > 0 && (!proj->depth || !proj->tiles_touched || !proj->rect)) return LMK_GS_ERR_INVALID;
    if (n > 0 && cam->binning == 1u && (!proj->feat || !aligned(proj->feat, 16))) return LMK_GS_ERR_INVALID;
    if (!out->tile_offsets) return LMK_GS_ERR_INVALID;
    if (out->capacity > 0 && (!out->keys || !out->vals || !out->keys_alt || !out->vals_alt))
        return LMK_GS_ERR_INVALID;
    if (!aligned(proj->rect, 8) || !aligned(count_status, 8)) return LMK_GS_ERR_INVALID;
    // the fixed array bounds what fits: sizes beyond it are refused before anything is enqueued
    if (n > kStaticMaxN || out->capacity > kStaticMaxCapacity || pp.tiles_x * pp.tiles_y > kStaticMaxTiles)
        return LMK_GS_ERR_CAPACITY;
    const ScratchLayout L = scratch_layout(n, out->capacity, pp.tiles_x * pp.tiles_y);
    if (L.total > kStaticBytes) return LMK_GS_ERR_CAPACITY;
    hipError_t e = hipSuccess;
    char *scratch = static_scratch_ptr(&e);
    if (!scratch) return hip_fail(e);
    hipStream_t s = static_cast<hipStream_t>(stream);
    e = launch_rebuild_handover(*proj, n, pp, scratch, L, s);
    if (e == hipSuccess) e = launch_bin_sort(*proj, n, pp, *out, scratch, L, s);
    if (e == hipSuccess && count_status) e = launch_copy_status(scratch, L, count_status, s);
    return e == hipSuccess ? LMK_GS_OK : hip_fail(e);
}

int32_t lmk_gs_render(const lmk_gs_projected *proj, const lmk_gs_binned *binned,
                      const lmk_gs_camera *cam, float *out_rgb, float *out_transmittance,
                      void *stream)
{
    ProjParams pp;
    const int32_t rc = check_camera(cam, &pp);
    if (rc != LMK_GS_OK) return rc;
    if (!proj || !binned || !out_rgb || !out_transmittance) return LMK_GS_ERR_INVALID;
    if (!binned->tile_offsets) return LMK_GS_ERR_INVALID;
    if (binned->capacity > 0 && (!binned->vals || !proj->feat)) return LMK_GS_ERR_INVALID;
    if (!aligned(proj->feat, 16)) return LMK_GS_ERR_INVALID;
    const hipError_t e = launch_render(*proj, *binned, pp, out_rgb, out_transmittance,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LMK_GS_OK : hip_fail(e);
}

int32_t lmk_gs_render_backward(const lmk_gs_projected *proj, uint32_t n, const lmk_gs_binned *binned,
                               const lmk_gs_camera *cam, const float *grad_rgb,
                               const float *grad_transmittance, float *grad_feat, void *stream)
{
    ProjParams pp;
    const int32_t rc = check_camera(cam, &pp);
    if (rc != LMK_GS_OK) return rc;
    if (!proj || !binned || !grad_rgb) return LMK_GS_ERR_INVALID;
    if (n > 0 && (!grad_feat || !proj->feat)) return LMK_GS_ERR_INVALID;
    if (!binned->tile_offsets) return LMK_GS_ERR_INVALID;
    if (binned->capacity > 0 && !binned->vals) return LMK_GS_ERR_INVALID;
    if (!aligned(proj->feat, 16) || !aligned(grad_feat, 16)) return LMK_GS_ERR_INVALID;
    const hipError_t e = launch_render_backward(*proj, n, *binned, pp, grad_rgb, grad_transmittance,
                                                grad_feat, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LMK_GS_OK : hip_fail(e);
}

int32_t lmk_gs_preprocess_backward(const lmk_gs_gaussians *g, const lmk_gs_camera *cam,
                                   const lmk_gs_projected *proj, const float *grad_feat,
                                   const lmk_gs_gaussian_grads *out, void *stream)
{
    ProjParams pp;
    const int32_t rc = check_camera(cam, &pp);
    if (rc != LMK_GS_OK) return rc;
    if (!g || !proj || !out) return LMK_GS_ERR_INVALID;
    if (g->sh_degree > 3) return LMK_GS_ERR_INVALID;
    if (g->n > 0) {
        if (!g->mean || !g->scale || !g->rot || !g->sh || !proj->tiles_touched || !grad_feat)
            return LMK_GS_ERR_INVALID;
        if (!out->mean || !out->scale || !out->rot || !out->opacity || !out->sh) return LMK_GS_ERR_INVALID;
        if (!aligned(g->sh, 16) || !aligned(out->sh, 16) || !aligned(grad_feat, 16)) return LMK_GS_ERR_INVALID;
    }
    const hipError_t e = launch_preprocess_backward(*g, pp, *proj, grad_feat, *out,
                                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LMK_GS_OK : hip_fail(e);
}

// Host-side checks shared by the two decode calls: v anchors are going to be decoded.
static int32_t check_decode_args(const lmk_gs_anchors *anchors, const lmk_gs_anchor_decoder *decoder,
                                 const float *cam_pos, const uint32_t *visible, uint32_t v,
                                 const lmk_gs_decoded *out)
{
    if (!anchors || !decoder || !cam_pos || !out) return LMK_GS_ERR_INVALID;
    if (anchors->k != 10u && anchors->k != 4u) return LMK_GS_ERR_UNSUPPORTED;
    if ((uint64_t)v * anchors->k >= (1ull << 32)) return LMK_GS_ERR_INVALID;
    if (!visible && v > anchors->a) return LMK_GS_ERR_INVALID;
    for (int i = 0; i < 3; ++i)
        if (!std::isfinite(cam_pos[i])) return LMK_GS_ERR_INVALID;
    if (v == 0) return LMK_GS_OK;
    if (anchors->a > 0 && (!anchors->position || !anchors->feature || !anchors->extent || !anchors->offsets))
        return LMK_GS_ERR_INVALID;
    if (!aligned(anchors->feature, 16) || !aligned(anchors->offsets, 8)) return LMK_GS_ERR_INVALID;
    const lmk_gs_perceptron *nets[3] = {&decoder->opacity, &decoder->colour, &decoder->cov};
    for (const lmk_gs_perceptron *p : nets)
        if (!p->w1 || !p->b1 || !p->w2t || !p->b2 || !aligned(p->w1, 4) || !aligned(p->w2t, 4))
            return LMK_GS_ERR_INVALID;
    if (!out->mean || !out->scale || !out->rot || !out->opacity || !out->sh) return LMK_GS_ERR_INVALID;
    if (!aligned(out->sh, 16)) return LMK_GS_ERR_INVALID;
    return LMK_GS_OK;
}

int32_t lmk_gs_anchor_decode(const lmk_gs_anchors *anchors, const lmk_gs_anchor_decoder *decoder,
                             const float *cam_pos, const uint32_t *visible, uint32_t v,
                             const lmk_gs_decoded *out, void *stream)
{
    const int32_t rc = check_decode_args(anchors, decoder, cam_pos, visible, v, out);
    if (rc != LMK_GS_OK) return rc;
    const hipError_t e = launch_anchor_decode(*anchors, *decoder, cam_pos, visible, v, nullptr, *out,
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LMK_GS_OK : hip_fail(e);
}

int32_t lmk_gs_anchor_decode_culled(const lmk_gs_anchors *anchors, const lmk_gs_anchor_decoder *decoder,
                                    const lmk_gs_camera *cam, const float *box, uint8_t *anchor_visible,
                                    const lmk_gs_decoded *out, void *stream)
{
    ProjParams pp;
    const int32_t rc = check_camera(cam, &pp);
    if (rc != LMK_GS_OK) return rc;
    if (!anchors) return LMK_GS_ERR_INVALID;
    const int32_t rc2 = check_decode_args(anchors, decoder, cam->cam_pos, nullptr, anchors->a, out);
    if (rc2 != LMK_GS_OK) return rc2;
    if (anchors->a == 0) return LMK_GS_OK;
    if (!box || !anchor_visible || !aligned(box, 16)) return LMK_GS_ERR_INVALID;
    hipError_t e = launch_box_flags(box, anchors->a, pp, anchor_visible, static_cast<hipStream_t>(stream));
    if (e == hipSuccess)
        e = launch_anchor_decode(*anchors, *decoder, cam->cam_pos, nullptr, anchors->a, anchor_visible, *out,
                                 static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LMK_GS_OK : hip_fail(e);
}

int32_t lmk_gs_read_status(const void *scratch, uint64_t *dup_count, int32_t *status, void *stream)
{
    if (!scratch) return LMK_GS_ERR_INVALID;
    ScratchHeader h;
    hipError_t e = hipMemcpyAsync(&h, scratch, sizeof(h), hipMemcpyDeviceToHost,
                                  static_cast<hipStream_t>(stream));
    if (e == hipSuccess) e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    if (dup_count) *dup_count = h.dup_count;
    if (status) *status = h.status;
    return LMK_GS_OK;
}

const char *lmk_gs_strerror(int32_t code)
{
    switch (code) {
    case LMK_GS_OK: return "ok";
    case LMK_GS_ERR_INVALID: return "invalid argument";
    case LMK_GS_ERR_CAPACITY: return "capacity exceeded";
    case LMK_GS_ERR_HIP: return "HIP runtime error";
    case LMK_GS_ERR_UNSUPPORTED: return "unsupported configuration";
    default: return "unknown error code";
    }
}

int32_t lmk_gs_last_hip_error(void) { return g_last_hip_error.load(); }

// 0.2.0: the gradient calls and the anchor decoder joined the three forward calls
uint32_t lmk_gs_version(void) { return 300; }

}  // extern "C"
