/* Runs the host-side code of liblmk_gs once for a build with AddressSanitizer and
 * UndefinedBehaviorSanitizer on the host pass (tests/test_sanitizers_cpu.py): the two index
 * builders on exactly sized arrays, the size arithmetic of lmk_gs_workspace_bytes up to the
 * largest arguments, and the argument checks of every device entry point.  Every call to a device
 * entry point here is one its checks must refuse, so no kernel is launched and no GPU is needed. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "lmk_gs.h"

static uint32_t rng_state = 88172645u;
static float uni(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return (float)(rng_state >> 8) / 16777216.0f;
}

static int failures = 0;
#define EXPECT(call, code) do { const int32_t rc_ = (call); if (rc_ != (code)) { \
    fprintf(stderr, "%s:%d: %s returned %d (%s), expected %d\n", __FILE__, __LINE__, #call, (int)rc_, \
            lmk_gs_strerror(rc_), (int)(code)); ++failures; } } while (0)
#define NEW(type, count) ((type *)calloc((size_t)(count) ? (size_t)(count) : 1, sizeof(type)))

static lmk_gs_camera good_camera(void)
{
    lmk_gs_camera cam;
    memset(&cam, 0, sizeof cam);
    cam.view[0] = cam.view[5] = cam.view[10] = 1.0f;
    cam.fx = cam.fy = 500.0f; cam.cx = 320.0f; cam.cy = 240.0f;
    cam.width = 640; cam.height = 480; cam.tile = LMK_GS_TILE; cam.near_z = 0.2f; cam.lowpass = 0.3f;
    return cam;
}

static void index_builders(uint32_t n, float voxel_size)
{
    float *mean = NEW(float, 3 * (size_t)n), *scale = NEW(float, 3 * (size_t)n);
    for (size_t i = 0; i < 3 * (size_t)n; ++i) { mean[i] = 8.0f * uni() - 4.0f; scale[i] = 0.01f + 0.3f * uni(); }
    const uint32_t groups = (n + LMK_GS_PRE_BLOCK - 1) / LMK_GS_PRE_BLOCK;
    uint32_t *perm = NEW(uint32_t, n), *first = NEW(uint32_t, (size_t)n + 1), *range = NEW(uint32_t, 2 * (size_t)groups);
    float *box = NEW(float, 8 * (size_t)n);
    uint32_t nv = 0;
    EXPECT(lmk_gs_index_build(mean, scale, n, voxel_size, perm, first, box, range, &nv), LMK_GS_OK);
    if (nv > n || (n > 0 && nv == 0)) { fprintf(stderr, "index_build: %u voxels for %u primitives\n", nv, n); ++failures; }
    /* refused inputs */
    const uint32_t found = nv;
    if (n > 0) EXPECT(lmk_gs_index_build(NULL, scale, n, voxel_size, perm, first, box, range, &nv), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_index_build(mean, scale, n, 0.0f, perm, first, box, range, &nv), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_index_build(mean, scale, n, -1.0f, perm, first, box, range, &nv), LMK_GS_ERR_INVALID);
    if (n > 0) {
        const float keep = mean[n / 2];
        mean[n / 2] = NAN;
        EXPECT(lmk_gs_index_build(mean, scale, n, voxel_size, perm, first, box, range, &nv), LMK_GS_ERR_INVALID);
        mean[n / 2] = 3.0e9f;       /* more than 2^21 cells between the two ends of an axis */
        if (n > 1) EXPECT(lmk_gs_index_build(mean, scale, n, 1.0f, perm, first, box, range, &nv), LMK_GS_ERR_UNSUPPORTED);
        mean[n / 2] = keep;
    }
    free(mean); free(scale); free(perm); free(first); free(range); free(box);
    printf("index_build: n %u, voxel %.2f -> %u voxels\n", n, (double)voxel_size, found);
}

static void anchor_index(uint32_t a, uint32_t k)
{
    float *pos = NEW(float, 3 * (size_t)a), *ext = NEW(float, 6 * (size_t)a), *off = NEW(float, 3 * (size_t)a * k);
    for (size_t i = 0; i < 3 * (size_t)a; ++i) pos[i] = 30.0f * uni() - 15.0f;
    for (size_t i = 0; i < 6 * (size_t)a; ++i) ext[i] = 0.05f + uni();
    for (size_t i = 0; i < 3 * (size_t)a * k; ++i) off[i] = 2.0f * uni() - 1.0f;
    const uint32_t groups = (uint32_t)(((uint64_t)a * k + LMK_GS_PRE_BLOCK - 1) / LMK_GS_PRE_BLOCK);
    float *box = NEW(float, 8 * (size_t)a);
    uint32_t *range = NEW(uint32_t, 2 * (size_t)groups);
    EXPECT(lmk_gs_anchor_index_build(pos, ext, off, a, k, box, range), LMK_GS_OK);
    EXPECT(lmk_gs_anchor_index_build(pos, ext, off, a, 0, box, range), LMK_GS_ERR_INVALID);
    if (a > 0) EXPECT(lmk_gs_anchor_index_build(NULL, ext, off, a, k, box, range), LMK_GS_ERR_INVALID);
    free(pos); free(ext); free(off); free(box); free(range);
    printf("anchor_index_build: a %u, k %u\n", a, k);
}

static void workspace_sizes(void)
{
    size_t bytes = 0;
    EXPECT(lmk_gs_workspace_bytes(0, 16, 16, 0, &bytes), LMK_GS_OK);
    EXPECT(lmk_gs_workspace_bytes(1000000, 1920, 1080, 20000000ull, &bytes), LMK_GS_OK);
    printf("workspace_bytes(1e6, 1920x1080, 2e7) = %zu\n", bytes);
    EXPECT(lmk_gs_workspace_bytes(1000, 0, 1080, 10, &bytes), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_workspace_bytes(1000, 1920, 1080, 10, NULL), LMK_GS_ERR_INVALID);
    /* the largest arguments: either a size or a refusal, never an overflowed size */
    const uint32_t big[] = { 0xffffffffu, 0x80000000u, 65536u * 16u, 65535u * 16u };
    for (unsigned i = 0; i < 4; ++i)
        for (unsigned j = 0; j < 4; ++j) {
            const int32_t rc = lmk_gs_workspace_bytes(big[i], big[j], big[(i + j) % 4], ~0ull >> (i * 8), &bytes);
            if (rc != LMK_GS_OK && rc != LMK_GS_ERR_UNSUPPORTED && rc != LMK_GS_ERR_INVALID && rc != LMK_GS_ERR_CAPACITY) {
                fprintf(stderr, "workspace_bytes: unexpected code %d\n", (int)rc); ++failures;
            }
        }
}

static void refused_calls(void)
{
    lmk_gs_camera cam = good_camera(), bad;
    static float __attribute__((aligned(256))) buf[4096];      /* never dereferenced by a refused call */
    lmk_gs_gaussians g;
    memset(&g, 0, sizeof g);
    g.mean = g.scale = g.rot = g.opacity = g.sh = buf; g.n = 64; g.sh_degree = 3;
    lmk_gs_projected proj;
    memset(&proj, 0, sizeof proj);
    lmk_gs_binned binned;
    memset(&binned, 0, sizeof binned);

    EXPECT(lmk_gs_preprocess(NULL, &cam, &proj, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_preprocess(&g, NULL, &proj, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_preprocess(&g, &cam, &proj, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);   /* no outputs */
    bad = cam; bad.tile = 8;
    EXPECT(lmk_gs_preprocess(&g, &bad, &proj, buf, sizeof buf, NULL), LMK_GS_ERR_UNSUPPORTED);
    bad = cam; bad.fx = NAN;
    EXPECT(lmk_gs_preprocess(&g, &bad, &proj, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    bad = cam; bad.near_z = 0.0f;
    EXPECT(lmk_gs_preprocess(&g, &bad, &proj, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    bad = cam; bad.binning = 2;
    EXPECT(lmk_gs_preprocess(&g, &bad, &proj, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    bad = cam; bad.width = 0;
    EXPECT(lmk_gs_preprocess(&g, &bad, &proj, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    g.sh_degree = 4;
    EXPECT(lmk_gs_preprocess(&g, &cam, &proj, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    g.sh_degree = 3;
    EXPECT(lmk_gs_preprocess_culled(&g, NULL, &cam, &proj, NULL, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_build_cov3d(NULL, buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_build_cov3d(&g, NULL, NULL), LMK_GS_ERR_INVALID);

    EXPECT(lmk_gs_bin_sort(NULL, 64, &cam, &binned, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_bin_sort(&proj, 64, &cam, NULL, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_bin_sort(&proj, 64, &cam, &binned, NULL, 0, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_bin_sort(&proj, 64, &cam, &binned, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);    /* no inputs */
    EXPECT(lmk_gs_bin_sort(&proj, 0, &cam, &binned, buf, sizeof buf, NULL), LMK_GS_ERR_INVALID);     /* no tile_offsets */
    EXPECT(lmk_gs_bin_sort_static(NULL, 64, &cam, &binned, (uint64_t *)buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_bin_sort_static(&proj, 64, &cam, &binned, (uint64_t *)buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_bin_sort_static(&proj, 0, &cam, &binned, (uint64_t *)buf, NULL), LMK_GS_ERR_INVALID);

    EXPECT(lmk_gs_render(NULL, &binned, &cam, buf, buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_render(&proj, &binned, &cam, NULL, buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_render(&proj, &binned, &cam, buf, buf, NULL), LMK_GS_ERR_INVALID);                 /* no tile_offsets */
    EXPECT(lmk_gs_render_backward(NULL, 64, &binned, &cam, buf, buf, buf, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_render_backward(&proj, 64, &binned, &cam, buf, buf, NULL, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_preprocess_backward(NULL, &cam, &proj, buf, NULL, NULL), LMK_GS_ERR_INVALID);

    lmk_gs_anchors anchors;
    memset(&anchors, 0, sizeof anchors);
    anchors.a = 8; anchors.k = 7;
    lmk_gs_anchor_decoder dec;
    memset(&dec, 0, sizeof dec);
    lmk_gs_decoded out;
    memset(&out, 0, sizeof out);
    EXPECT(lmk_gs_anchor_decode(NULL, &dec, cam.cam_pos, NULL, 8, &out, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_anchor_decode(&anchors, &dec, cam.cam_pos, NULL, 8, &out, NULL), LMK_GS_ERR_UNSUPPORTED);   /* k = 7 */
    anchors.k = 10;
    EXPECT(lmk_gs_anchor_decode(&anchors, &dec, cam.cam_pos, NULL, 9, &out, NULL), LMK_GS_ERR_INVALID);       /* v > a */
    EXPECT(lmk_gs_anchor_decode(&anchors, &dec, cam.cam_pos, NULL, 8, &out, NULL), LMK_GS_ERR_INVALID);       /* no arrays */
    EXPECT(lmk_gs_anchor_decode_culled(NULL, &dec, &cam, buf, (uint8_t *)buf, &out, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_anchor_decode_culled(&anchors, &dec, &cam, NULL, (uint8_t *)buf, &out, NULL), LMK_GS_ERR_INVALID);
    EXPECT(lmk_gs_read_status(NULL, NULL, NULL, NULL), LMK_GS_ERR_INVALID);

    for (int32_t code = -6; code <= 1; ++code)
        if (!lmk_gs_strerror(code) || !lmk_gs_strerror(code)[0]) { fprintf(stderr, "strerror(%d) empty\n", (int)code); ++failures; }
    printf("version %u, last hip error %d\n", lmk_gs_version(), (int)lmk_gs_last_hip_error());
}

int main(void)
{
    index_builders(5000, 1.0f);
    index_builders(777, 0.37f);       /* a ragged last group */
    index_builders(1, 5.0f);
    index_builders(0, 1.0f);
    anchor_index(300, 10);
    anchor_index(77, 4);
    anchor_index(0, 10);
    workspace_sizes();
    refused_calls();
    if (failures) { fprintf(stderr, "%d unexpected return codes\n", failures); return 1; }
    puts("host driver done");
    return 0;
}
