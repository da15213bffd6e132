/* Runs every entry point of oracle/lmk_ref.c once on a small synthetic frame, for a build with
 * AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_sanitizers_cpu.py compiles this file
 * together with the oracle and fails on any report).  All sizes are exact: a read or write past the
 * end of any array is a report.  No result is checked here -- the pins of the oracle live in the
 * other CPU tests. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    float view[12]; float cam_pos[3]; float fx, fy, cx, cy;
    uint32_t width, height, tile; float near_z; float lowpass; float bg[3]; uint32_t binning;
} ref_camera;

float lmk_ref_opacity_tau(float o);
int lmk_ref_tile_kept(float, float, float, float, float, float, uint32_t, uint32_t, uint32_t);
void lmk_ref_covariance3d(const float q[4], const float s[3], float out9[9]);
void lmk_ref_sh_basis(const double d[3], double Y[16]);
void lmk_ref_preprocess(uint32_t, const float *, const float *, const float *, const float *, const float *,
                        uint32_t, const ref_camera *, uint8_t *, float *, float *, float *, float *,
                        uint16_t *, uint32_t *, double *);
uint64_t lmk_ref_scan(uint32_t, const uint32_t *, uint64_t *);
void lmk_ref_emit(uint32_t, const uint32_t *, const uint16_t *, const float *, const uint64_t *, uint32_t,
                  uint32_t, uint32_t, const float *, const float *, const float *, uint64_t *, uint32_t *);
void lmk_ref_sort(uint64_t, uint64_t *, uint32_t *);
void lmk_ref_ranges(uint64_t, const uint64_t *, uint32_t, uint64_t *);
void lmk_ref_render(uint32_t, const uint8_t *, const float *, const float *, const float *, const double *,
                    const uint32_t *, const uint64_t *, const ref_camera *, double *, double *, uint32_t *,
                    uint32_t *, double *, double *, uint32_t *);
uint32_t lmk_ref_depth_order(uint32_t, const uint8_t *, const float *, uint32_t *);
void lmk_ref_render_pixels_brute(uint32_t, const uint8_t *, const float *, const float *, const float *,
                                 const double *, const uint32_t *, uint32_t, const ref_camera *, uint32_t,
                                 const uint32_t *, const uint32_t *, double *, double *, uint32_t *, double *,
                                 double *, uint32_t *);
uint64_t lmk_ref_tile_list(uint32_t, const uint32_t *, const uint16_t *, const float *, uint32_t, uint32_t,
                           uint32_t, uint32_t, const float *, const float *, const float *, uint32_t *, uint64_t);
uint64_t lmk_ref_band_lists(uint32_t, const uint32_t *, const uint16_t *, const uint32_t *, uint32_t, uint32_t,
                            uint32_t, uint32_t, uint32_t, uint32_t, const float *, const float *, const float *,
                            uint64_t *, uint32_t *, uint64_t);
void lmk_ref_render_band(uint32_t, const uint8_t *, const float *, const float *, const float *, const double *,
                         const uint32_t *, const uint64_t *, const ref_camera *, uint32_t, uint32_t, double *,
                         double *, uint32_t *, uint32_t *, double *, double *, uint32_t *);
void lmk_ref_render_pixels_list(uint32_t, const uint8_t *, const float *, const float *, const float *,
                                const double *, const uint32_t *, uint64_t, const ref_camera *, uint32_t,
                                const uint32_t *, const uint32_t *, double *, double *, uint32_t *, uint32_t *,
                                double *, double *, uint32_t *);
uint32_t lmk_ref_trace_pixel(uint32_t, const float *, const float *, const float *, const double *,
                             const uint32_t *, uint64_t, uint32_t, uint32_t, double *, uint32_t);
int lmk_ref_voxel_visible(const ref_camera *, const float lo[3], const float hi[3], float);
void lmk_ref_voxels_visible(const ref_camera *, uint32_t, const float *, const float *, const float *, uint8_t *);
void lmk_ref_render_backward(uint32_t, const float *, const float *, const float *, const double *,
                             const uint32_t *, const uint64_t *, const ref_camera *, const double *,
                             const double *, double *, double *, double *, double *, double *, double *,
                             uint32_t *, double *);
void lmk_ref_preprocess_backward(uint32_t, const float *, const float *, const float *, const float *, uint32_t,
                                 const ref_camera *, const uint8_t *, const double *, double *, double *,
                                 double *, double *, double *);

static uint32_t rng_state = 2463534242u;
static float uni(void)                   /* [0,1) */
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return (float)(rng_state >> 8) / 16777216.0f;
}

#define NEW(type, count) ((type *)calloc((size_t)(count) ? (size_t)(count) : 1, sizeof(type)))

static void run(uint32_t n, uint32_t W, uint32_t H, uint32_t binning, uint32_t sh_degree)
{
    const uint32_t ts = 16, tx = (W + ts - 1) / ts, ty = (H + ts - 1) / ts, T = tx * ty;
    const uint32_t ncoef = (sh_degree + 1) * (sh_degree + 1);
    ref_camera cam;
    memset(&cam, 0, sizeof cam);
    cam.view[0] = cam.view[5] = cam.view[10] = 1.0f;
    cam.view[11] = 4.0f;                       /* camera 4 units behind the origin, looking along +z */
    cam.cam_pos[2] = -4.0f;
    cam.fx = cam.fy = 0.8f * (float)W; cam.cx = 0.5f * (float)W; cam.cy = 0.5f * (float)H;
    cam.width = W; cam.height = H; cam.tile = ts; cam.near_z = 0.2f; cam.lowpass = 0.3f;
    cam.bg[0] = 0.1f; cam.bg[1] = 0.2f; cam.bg[2] = 0.3f; cam.binning = binning;

    float *mean = NEW(float, 3 * n), *scale = NEW(float, 3 * n), *rot = NEW(float, 4 * n);
    float *opacity = NEW(float, n), *sh = NEW(float, (size_t)n * ncoef * 3);
    for (uint32_t i = 0; i < n; ++i) {
        for (int c = 0; c < 3; ++c) {
            mean[3 * i + c] = 6.0f * uni() - 3.0f;       /* some behind the camera, some off screen */
            scale[3 * i + c] = 0.02f + 0.5f * uni() * uni();
        }
        mean[3 * i + 2] = 12.0f * uni() - 6.0f;
        float q[4], len = 0.0f;
        for (int c = 0; c < 4; ++c) { q[c] = 2.0f * uni() - 1.0f; len += q[c] * q[c]; }
        len = sqrtf(len) + 1e-6f;
        for (int c = 0; c < 4; ++c) rot[4 * i + c] = q[c] / len;
        opacity[i] = uni() < 0.1f ? 0.002f : 0.05f + 0.95f * uni();
        for (uint32_t c = 0; c < ncoef * 3; ++c) sh[(size_t)i * ncoef * 3 + c] = 1.2f * uni() - 0.4f;
    }

    uint8_t *stage = NEW(uint8_t, n);
    float *depth = NEW(float, n), *mean2d = NEW(float, 2 * n), *cov2d = NEW(float, 3 * n), *conic = NEW(float, 3 * n);
    uint16_t *rect = NEW(uint16_t, 4 * n);
    uint32_t *touched = NEW(uint32_t, n);
    double *rgb = NEW(double, 3 * n);
    lmk_ref_preprocess(n, mean, scale, rot, opacity, sh, sh_degree, &cam, stage, depth, mean2d, cov2d, conic,
                       rect, touched, rgb);

    uint64_t *offsets = NEW(uint64_t, n + 1);
    const uint64_t D = lmk_ref_scan(n, touched, offsets);
    uint64_t *keys = NEW(uint64_t, D);
    uint32_t *vals = NEW(uint32_t, D);
    lmk_ref_emit(n, touched, rect, depth, offsets, tx, binning, ts, mean2d, conic, opacity, keys, vals);
    lmk_ref_sort(D, keys, vals);
    uint64_t *tile_offsets = NEW(uint64_t, T + 1);
    lmk_ref_ranges(D, keys, T, tile_offsets);

    const size_t P = (size_t)W * H;
    double *out_rgb = NEW(double, 3 * P), *out_T = NEW(double, P), *beta = NEW(double, P), *beta_T = NEW(double, P);
    uint32_t *E = NEW(uint32_t, P), *C = NEW(uint32_t, P), *amb = NEW(uint32_t, P);
    lmk_ref_render(n, stage, mean2d, conic, opacity, rgb, vals, tile_offsets, &cam, out_rgb, out_T, E, C, beta,
                   beta_T, amb);

    uint32_t *order = NEW(uint32_t, n);
    const uint32_t m = lmk_ref_depth_order(n, stage, depth, order);

    /* per-tile lists, one tile at its exact length, and the banded path over the whole frame */
    for (uint32_t t = 0; t < T; t += (T > 7 ? T / 7 : 1)) {
        const uint64_t len = tile_offsets[t + 1] - tile_offsets[t];
        uint32_t *lst = NEW(uint32_t, len);
        const uint64_t got = lmk_ref_tile_list(n, touched, rect, depth, t % tx, t / tx, binning, ts, mean2d, conic,
                                               opacity, lst, len);
        if (got != len) { fprintf(stderr, "tile_list length %llu != %llu\n", (unsigned long long)got, (unsigned long long)len); exit(3); }
        free(lst);
    }
    for (uint32_t a = 0; a < ty; a += 2) {
        const uint32_t b = a + 2 < ty ? a + 2 : ty;
        const uint64_t len = tile_offsets[b * tx] - tile_offsets[a * tx];
        uint64_t *boff = NEW(uint64_t, (b - a) * tx + 1);
        uint32_t *bval = NEW(uint32_t, len);
        const uint64_t got = lmk_ref_band_lists(n, touched, rect, order, m, binning, ts, tx, a, b, mean2d, conic,
                                                opacity, boff, bval, len);
        if (got != len) { fprintf(stderr, "band_lists length mismatch\n"); exit(3); }
        const uint32_t y0 = a * ts, y1 = b * ts < H ? b * ts : H;
        const size_t bp = (size_t)(y1 - y0) * W;
        double *br = NEW(double, 3 * bp), *bT = NEW(double, bp), *bb = NEW(double, bp), *bbT = NEW(double, bp);
        uint32_t *bE = NEW(uint32_t, bp), *bC = NEW(uint32_t, bp), *ba = NEW(uint32_t, bp);
        lmk_ref_render_band(n, stage, mean2d, conic, opacity, rgb, bval, boff, &cam, a, b, br, bT, bE, bC, bb, bbT, ba);
        free(boff); free(bval); free(br); free(bT); free(bb); free(bbT); free(bE); free(bC); free(ba);
    }

    /* sampled pixels: brute force over the depth order, and through one tile's list */
    enum { NP = 5 };
    uint32_t xs[NP], ys[NP];
    for (int k = 0; k < NP; ++k) { xs[k] = (uint32_t)(uni() * (float)W) % W; ys[k] = (uint32_t)(uni() * (float)H) % H; }
    xs[0] = W - 1; ys[0] = H - 1;
    double p_rgb[3 * NP], p_T[NP], p_b[NP], p_bT[NP];
    uint32_t p_E[NP], p_C[NP], p_a[NP];
    lmk_ref_render_pixels_brute(n, stage, mean2d, conic, opacity, rgb, order, m, &cam, NP, xs, ys, p_rgb, p_T, p_C,
                                p_b, p_bT, p_a);
    {
        const uint32_t t = (ys[0] / ts) * tx + xs[0] / ts;
        const uint64_t beg = tile_offsets[t], len = tile_offsets[t + 1] - beg;
        lmk_ref_render_pixels_list(n, stage, mean2d, conic, opacity, rgb, vals + beg, len, &cam, 1, xs, ys, p_rgb,
                                   p_T, p_E, p_C, p_b, p_bT, p_a);
        const uint32_t cap = (uint32_t)len;
        double *trace = NEW(double, 4 * (size_t)cap);
        lmk_ref_trace_pixel(n, mean2d, conic, opacity, rgb, vals + beg, len, xs[0], ys[0], trace, cap);
        free(trace);
    }

    /* backward of the compositing and of the projection */
    double *g_img = NEW(double, 3 * P), *g_T = NEW(double, P);
    for (size_t k = 0; k < 3 * P; ++k) g_img[k] = (double)uni() - 0.5;
    for (size_t k = 0; k < P; ++k) g_T[k] = (double)uni() - 0.5;
    double *g_m2 = NEW(double, 2 * n), *g_con = NEW(double, 3 * n), *g_op = NEW(double, n), *g_rgb = NEW(double, 3 * n);
    double *g_abs = NEW(double, 9 * n);
    lmk_ref_render_backward(n, mean2d, conic, opacity, rgb, vals, tile_offsets, &cam, g_img, g_T, g_m2, g_con, g_op,
                            g_rgb, out_rgb, out_T, amb, g_abs);
    double *g_feat = NEW(double, 9 * n);   /* planes u, v, A, B, C, o, r, g, b of n each */
    const size_t N = n;
    memcpy(g_feat, g_m2, sizeof(double) * 2 * N);
    memcpy(g_feat + 2 * N, g_con, sizeof(double) * 3 * N);
    memcpy(g_feat + 5 * N, g_op, sizeof(double) * N);
    memcpy(g_feat + 6 * N, g_rgb, sizeof(double) * 3 * N);
    double *g_mean = NEW(double, 3 * n), *g_scale = NEW(double, 3 * n), *g_rot = NEW(double, 4 * n);
    double *g_opac = NEW(double, n), *g_sh = NEW(double, (size_t)n * ncoef * 3);
    lmk_ref_preprocess_backward(n, mean, scale, rot, sh, sh_degree, &cam, stage, g_feat, g_mean, g_scale, g_rot,
                                g_opac, g_sh);

    /* small helpers and the box test */
    const float q1[4] = { 0.5f, -0.5f, 0.5f, 0.5f }, s1[3] = { 0.1f, 0.2f, 0.3f };
    float cov9[9]; lmk_ref_covariance3d(q1, s1, cov9);
    double dir[3] = { 0.6, 0.0, 0.8 }, Y[16]; lmk_ref_sh_basis(dir, Y);
    (void)lmk_ref_opacity_tau(0.5f);
    (void)lmk_ref_tile_kept(20.0f, 20.0f, 0.1f, 0.0f, 0.1f, 0.5f, 1, 1, ts);
    const uint32_t nv = 9;
    float lo[3 * 9], hi[3 * 9], smax[9]; uint8_t vis[9];
    for (uint32_t v = 0; v < nv; ++v)
        for (int c = 0; c < 3; ++c) { lo[3 * v + c] = 16.0f * uni() - 8.0f; hi[3 * v + c] = lo[3 * v + c] + uni(); smax[v] = 0.3f * uni(); }
    lmk_ref_voxels_visible(&cam, nv, lo, hi, smax, vis);
    (void)lmk_ref_voxel_visible(&cam, lo, hi, smax[0]);

    printf("n %u, %ux%u, rule %u, degree %u: D %llu, depth order %u\n", n, W, H, binning, sh_degree,
           (unsigned long long)D, m);
    free(mean); free(scale); free(rot); free(opacity); free(sh); free(stage); free(depth); free(mean2d); free(cov2d);
    free(conic); free(rect); free(touched); free(rgb); free(offsets); free(keys); free(vals); free(tile_offsets);
    free(out_rgb); free(out_T); free(beta); free(beta_T); free(E); free(C); free(amb); free(order);
    free(g_img); free(g_T); free(g_m2); free(g_con); free(g_op); free(g_rgb); free(g_abs); free(g_feat);
    free(g_mean); free(g_scale); free(g_rot); free(g_opac); free(g_sh);
}

int main(void)
{
    run(2500, 100, 70, 0, 3);     /* ragged right and bottom tiles */
    run(2500, 100, 70, 1, 2);
    run(1, 16, 16, 1, 0);
    run(0, 33, 17, 0, 1);         /* empty scene */
    puts("oracle driver done");
    return 0;
}
