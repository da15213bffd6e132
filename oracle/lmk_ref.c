/*
 * lmk_ref.c -- CPU oracle for tile-based 3D Gaussian splatting (forward, and the
 * gradient through the compositing).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU renderer is checked against.  It shares no code, header, table or
 * constant generator with the HIP library, and nothing in the product path may
 * import, link or call it.
 *
 * What it follows (LandMarkSystem technical report):
 *   Sec. 2.2 Eq. 7   the 3D Gaussian primitive G(x)
 *   Sec. 2.2 Eq. 8   covariance from rotation and scale, Sigma = R S S^T R^T
 *   Sec. 2.2 (text)  SH colour + opacity per primitive; EWA projection to a 2D
 *                    Gaussian ("splatting"); depth sort; blending per screen tile
 *   Sec. 2.2 Eq. 9-10  front-to-back compositing with sigma_i = alpha_i G'_i(x')
 *   Sec. 2.2 (text)  the rasteriser is differentiable: gradient of a loss through Eq. 9-10
 *                    with respect to each primitive's 2D mean, conic, opacity and colour, and
 *                    from there through the projection to mean, scale, rotation, opacity, SH
 *   Sec. 4.2.1       the rasteriser stages named there: per-primitive projection,
 *                    duplication into (tile, depth) keys, sort, per-tile blend;
 *                    the per-tile intersection test (binning rule 1)
 *   Sec. 4.2.2       view-frustum filtering of voxels of a reordered scene
 *
 * The report prints no constants (tile size, thresholds, SH basis, pixel
 * centres, key layout).  The readings taken here are listed at each step and
 * marked [reading].
 *
 * Precision.  Everything that decides an integer (depth bits in the sort key,
 * the tile rectangle, every cull) is evaluated in IEEE fp32, one rounding per
 * written operation, left to right, no fused multiply-add (compile with
 * -ffp-contract=off).  The GPU side evaluates the same formulas in the same
 * precision, so keys and rectangles are unique.  Everything else (SH colour,
 * the blend) is evaluated in fp64 from those fp32 inputs; the two blend
 * decisions (alpha below 1/255, transmittance below 1e-4) are taken on the
 * value rounded to fp32, the precision the kernel decides in.
 *
 * Pins (tests/test_oracle_*.py): closed-form isotropic footprint, single and
 * double splat closed forms, SH orthonormality and addition theorem against a
 * library routine, brute-force per-pixel compositing over all primitives,
 * tile-size independence, transmittance monotonicity, sort/CSR invariants;
 * the tile intersection test of binning rule 1 against dense sampling and
 * against the unchanged image; the voxel visibility test against brute-force
 * conservativeness, closed cases and a planted mistake; the culls of
 * degenerate attribute values; the gradients through the compositing and through
 * the projection against central differences of the forward functions, one- and
 * two-splat closed forms, the partition of unity of the weights, and the
 * invariances of the projection.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef M_PI
#define M_PI 3.14159265358979323846
#endif

typedef struct {
    float view[12];   /* row-major 3x4 world->camera [R|t]; +x right, +y down, +z forward */
    float cam_pos[3]; /* camera centre in world space */
    float fx, fy, cx, cy;
    uint32_t width, height, tile;
    float near_z;
    float lowpass;    /* h: added to the diagonal of the 2D covariance, px^2 */
    float bg[3];
    uint32_t binning; /* 0: every tile of the support rectangle; 1: only tiles the splat can reach */
} ref_camera;

/* cull stage recorded per primitive */
enum { REF_VISIBLE = 0, REF_CULL_NEAR = 1, REF_CULL_DET = 2, REF_CULL_OPACITY = 3, REF_CULL_OFFSCREEN = 4 };

#define REF_TAU 11.09f            /* [reading] support: q <= tau, a hair above 2 ln 255 */
#define REF_ALPHA_MIN (1.0f / 255.0f)
#define REF_ALPHA_MAX 0.99f
#define REF_T_MIN 1e-4f

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* ------------------------------------------------------------------ */
/* Binning rule 1 ("intersection operations for each tile", Sec. 4.2.1) [reading]:
 * a tile of the support rectangle is kept only if the splat can reach alpha >=
 * 1/255 somewhere on the square spanned by the tile's pixel centres.
 *
 * q(d) = d^T conic d is convex, so its minimum over the square sits at the splat
 * centre if that is inside, else on an edge facing it: clamp one coordinate into
 * the square, minimise along that line (clamped), and take the better of the
 * two choices.  A pair contributes only if q <= 2 ln(255 o); tau bounds that from
 * above using only the exponent and the top three mantissa bits of o
 * (o < (1 + (k+1)/8) 2^E), so that no logarithm of a run-time value is needed
 * and the decision is reproducible bit for bit.  All fp32, one rounding per
 * operation.  The 0.01 added to tau and the 4e-6 m subtracted from q keep the
 * rule conservative under rounding (m = A ex^2 + C ey^2 bounds the magnitude
 * of every term of q). */
static float tau_table[8];
static int tau_table_ready = 0;

static void init_tau_table(void)
{
    if (tau_table_ready) return;
    for (int k = 0; k < 8; ++k)
        tau_table[k] = (float)(2.0 * (log(255.0) + log(1.0 + (k + 1) / 8.0)) + 0.01);
    tau_table_ready = 1;
}

static float opacity_tau(float o)
{
    uint32_t bits; memcpy(&bits, &o, 4);
    const int E = (int)((bits >> 23) & 0xffu) - 127;
    const uint32_t k = (bits >> 20) & 7u;
    return tau_table[k] + (float)E * 1.3862944f;
}

static float clampf(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

static float quad_adj(float A, float B, float C, float ex, float ey)
{
    const float m = A * ex * ex + C * ey * ey;
    const float q = m + 2.0f * B * ex * ey;
    return q - 4e-6f * m;
}

static int tile_kept(float u, float v, float A, float B, float C, float tau,
                     uint32_t tx, uint32_t ty, uint32_t ts)
{
    const float h = 0.5f * (float)ts - 0.5f;                       /* 7.5 for 16-pixel tiles */
    const float xs = u - ((float)(tx * ts) + 0.5f * (float)ts);    /* splat centre in square coordinates */
    const float ys = v - ((float)(ty * ts) + 0.5f * (float)ts);
    const float ex1 = clampf(xs, -h, h) - xs;
    const float ey1 = clampf(ys + (-B / C) * ex1, -h, h) - ys;
    const float ey2 = clampf(ys, -h, h) - ys;
    const float ex2 = clampf(xs + (-B / A) * ey2, -h, h) - xs;
    const float q1 = quad_adj(A, B, C, ex1, ey1);
    const float q2 = quad_adj(A, B, C, ex2, ey2);
    const float qmin = q1 < q2 ? q1 : q2;
    return qmin <= tau;
}

/* exported for the pins */
float lmk_ref_opacity_tau(float o) { init_tau_table(); return opacity_tau(o); }
int lmk_ref_tile_kept(float u, float v, float A, float B, float C, float o,
                      uint32_t tx, uint32_t ty, uint32_t ts)
{
    init_tau_table();
    return tile_kept(u, v, A, B, C, opacity_tau(o), tx, ty, ts);
}

/* clamp that sends NaN to lo */
static float clampf_lo(float v, float lo, float hi) { return !(v > lo) ? lo : (v > hi ? hi : v); }

/* ------------------------------------------------------------------ */
/* Sec. 2.2 Eq. 8: rotation matrix from a (w,x,y,z) quaternion [reading: order] */
static void quat_to_rot(const float q[4], float R[3][3])
{
    float n = sqrtf(q[0] * q[0] + q[1] * q[1] + q[2] * q[2] + q[3] * q[3]);
    float w = q[0] / n, x = q[1] / n, y = q[2] / n, z = q[3] / n;
    R[0][0] = 1.0f - 2.0f * (y * y + z * z);
    R[0][1] = 2.0f * (x * y - w * z);
    R[0][2] = 2.0f * (x * z + w * y);
    R[1][0] = 2.0f * (x * y + w * z);
    R[1][1] = 1.0f - 2.0f * (x * x + z * z);
    R[1][2] = 2.0f * (y * z - w * x);
    R[2][0] = 2.0f * (x * z - w * y);
    R[2][1] = 2.0f * (y * z + w * x);
    R[2][2] = 1.0f - 2.0f * (x * x + y * y);
}

/* Sec. 2.2 Eq. 8: Sigma = (R S)(R S)^T, S = diag(s) */
static void covariance3d(const float q[4], const float s[3], float Sigma[3][3])
{
    float R[3][3], M[3][3];
    quat_to_rot(q, R);
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j)
            M[i][j] = R[i][j] * s[j];
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j)
            Sigma[i][j] = M[i][0] * M[j][0] + M[i][1] * M[j][1] + M[i][2] * M[j][2];
}

/* exported for the pins */
void lmk_ref_covariance3d(const float q[4], const float s[3], float out9[9])
{
    float S[3][3];
    covariance3d(q, s, S);
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j)
            out9[3 * i + j] = S[i][j];
}

/* ------------------------------------------------------------------ */
/* Real spherical harmonics up to degree 3 at unit direction d.
 * [reading] order and signs: within each degree, m = -l..l, with the sign
 * (-1)^m of the usual real basis dropped on odd m (the convention in common
 * use for splat colours).  Constants come from their closed forms. */
void lmk_ref_sh_basis(const double d[3], double Y[16])
{
    const double x = d[0], y = d[1], z = d[2];
    const double xx = x * x, yy = y * y, zz = z * z;
    const double k0 = 0.5 * sqrt(1.0 / M_PI);
    const double k1 = sqrt(3.0 / (4.0 * M_PI));
    const double k2 = 0.5 * sqrt(15.0 / M_PI);
    const double k20 = 0.25 * sqrt(5.0 / M_PI);
    const double k33 = 0.25 * sqrt(35.0 / (2.0 * M_PI));
    const double k32 = 0.5 * sqrt(105.0 / M_PI);
    const double k31 = 0.25 * sqrt(21.0 / (2.0 * M_PI));
    const double k30 = 0.25 * sqrt(7.0 / M_PI);
    const double k32b = 0.25 * sqrt(105.0 / M_PI);
    Y[0] = k0;
    Y[1] = -k1 * y;
    Y[2] = k1 * z;
    Y[3] = -k1 * x;
    Y[4] = k2 * x * y;
    Y[5] = -k2 * y * z;
    Y[6] = k20 * (2.0 * zz - xx - yy);
    Y[7] = -k2 * x * z;
    Y[8] = 0.5 * k2 * (xx - yy);
    Y[9] = -k33 * y * (3.0 * xx - yy);
    Y[10] = k32 * x * y * z;
    Y[11] = -k31 * y * (4.0 * zz - xx - yy);
    Y[12] = k30 * z * (2.0 * zz - 3.0 * xx - 3.0 * yy);
    Y[13] = -k31 * x * (4.0 * zz - xx - yy);
    Y[14] = k32b * z * (xx - yy);
    Y[15] = -k33 * x * (xx - 3.0 * yy);
}

/* ------------------------------------------------------------------ */
/* Per-primitive projection (Sec. 2.2 text: EWA splatting; Sec. 4.2.1 first stage).
 *
 * Inputs are structure-of-arrays, each plane n floats: mean[3], scale[3]
 * (linear, > 0), rot[4] (w,x,y,z, any norm), opacity in [0,1], sh laid out
 * [(deg+1)^2][3][n].
 * Outputs, all length n (planes where several): stage (see enum), depth,
 * mean2d u/v, cov2d a/b/c (with low-pass), conic A/B/C, rect (x0,y0,x1,y1
 * interleaved, tile units, half-open), tiles_touched, rgb (3 planes, fp64).
 * For stage 1..3 only `stage` and tiles_touched (=0) are meaningful.
 */
void lmk_ref_preprocess(uint32_t n,
                        const float *mean, const float *scale, const float *rot,
                        const float *opacity, const float *sh, uint32_t sh_degree,
                        const ref_camera *cam,
                        uint8_t *stage, float *depth, float *mean2d, float *cov2d,
                        float *conic, uint16_t *rect, uint32_t *tiles_touched, double *rgb)
{
    const size_t N = n;
    const float TS = (float)cam->tile;
    const uint32_t TX = (cam->width + cam->tile - 1) / cam->tile;
    const uint32_t TY = (cam->height + cam->tile - 1) / cam->tile;
    const float lim_x = 1.3f * ((0.5f * (float)cam->width) / cam->fx);
    const float lim_y = 1.3f * ((0.5f * (float)cam->height) / cam->fy);
    const float *V = cam->view;
    const uint32_t ncoef = (sh_degree + 1) * (sh_degree + 1);
    init_tau_table();

#pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)n; ++ii) {
        const size_t i = (size_t)ii;
        tiles_touched[i] = 0;
        depth[i] = 0.0f;
        mean2d[i] = mean2d[N + i] = 0.0f;
        cov2d[i] = cov2d[N + i] = cov2d[2 * N + i] = 0.0f;
        conic[i] = conic[N + i] = conic[2 * N + i] = 0.0f;
        rect[4 * i] = rect[4 * i + 1] = rect[4 * i + 2] = rect[4 * i + 3] = 0;
        rgb[i] = rgb[N + i] = rgb[2 * N + i] = 0.0;

        /* 1. camera-space position; cull unless z > near [reading] */
        const float mx = mean[i], my = mean[N + i], mz = mean[2 * N + i];
        const float px = V[0] * mx + V[1] * my + V[2] * mz + V[3];
        const float py = V[4] * mx + V[5] * my + V[6] * mz + V[7];
        const float pz = V[8] * mx + V[9] * my + V[10] * mz + V[11];
        if (!(pz > cam->near_z)) { stage[i] = REF_CULL_NEAR; continue; }

        /* 2. Sigma = R S S^T R^T (Eq. 8) */
        const float q[4] = { rot[i], rot[N + i], rot[2 * N + i], rot[3 * N + i] };
        const float s[3] = { scale[i], scale[N + i], scale[2 * N + i] };
        float Sigma[3][3];
        covariance3d(q, s, Sigma);

        /* 3. EWA: local affine approximation of the perspective map at the
         * (guard-band clamped) camera-space mean [reading: formula not printed];
         * Sigma' = (J W) Sigma (J W)^T + h I */
        const float txz = clampf_lo(px / pz, -lim_x, lim_x) * pz;
        const float tyz = clampf_lo(py / pz, -lim_y, lim_y) * pz;
        float J[2][3];
        J[0][0] = cam->fx / pz; J[0][1] = 0.0f;        J[0][2] = -(cam->fx * txz) / (pz * pz);
        J[1][0] = 0.0f;        J[1][1] = cam->fy / pz; J[1][2] = -(cam->fy * tyz) / (pz * pz);
        float Tm[2][3], U[2][3];
        for (int r = 0; r < 2; ++r)
            for (int c = 0; c < 3; ++c)
                Tm[r][c] = J[r][0] * V[c] + J[r][1] * V[4 + c] + J[r][2] * V[8 + c];
        for (int r = 0; r < 2; ++r)
            for (int c = 0; c < 3; ++c)
                U[r][c] = Tm[r][0] * Sigma[0][c] + Tm[r][1] * Sigma[1][c] + Tm[r][2] * Sigma[2][c];
        const float a = (U[0][0] * Tm[0][0] + U[0][1] * Tm[0][1] + U[0][2] * Tm[0][2]) + cam->lowpass;
        const float b = U[0][0] * Tm[1][0] + U[0][1] * Tm[1][1] + U[0][2] * Tm[1][2];
        const float c = (U[1][0] * Tm[1][0] + U[1][1] * Tm[1][1] + U[1][2] * Tm[1][2]) + cam->lowpass;

        /* 4. invert; cull unless det > 0 (also rejects NaN) */
        const float det = a * c - b * b;
        if (!(det > 0.0f)) { stage[i] = REF_CULL_DET; continue; }
        const float cA = c / det, cB = -b / det, cC = a / det;

        /* 5. centre in pixels; pixel (i,j) has centre (i+0.5, j+0.5) [reading] */
        const float u = (cam->fx * px) / pz + cam->cx;
        const float v = (cam->fy * py) / pz + cam->cy;

        /* 6. can never reach alpha >= 1/255 [reading] */
        const float o = opacity[i];
        if (o < REF_ALPHA_MIN) { stage[i] = REF_CULL_OPACITY; continue; }

        /* 7. axis-aligned bounding box of the ellipse q <= tau [reading] */
        const float hx = sqrtf(REF_TAU * a);
        const float hy = sqrtf(REF_TAU * c);

        /* 8. tile rectangle, clamped in float before conversion */
        const float fTX = (float)TX, fTY = (float)TY;
        const uint32_t x0 = (uint32_t)clampf_lo(floorf((u - hx) / TS), 0.0f, fTX);
        const uint32_t x1 = (uint32_t)clampf_lo(floorf((u + hx) / TS) + 1.0f, 0.0f, fTX);
        const uint32_t y0 = (uint32_t)clampf_lo(floorf((v - hy) / TS), 0.0f, fTY);
        const uint32_t y1 = (uint32_t)clampf_lo(floorf((v + hy) / TS) + 1.0f, 0.0f, fTY);
        uint32_t cnt = (x1 > x0 && y1 > y0) ? (x1 - x0) * (y1 - y0) : 0u;
        if (cnt && cam->binning == 1) {
            const float tau = opacity_tau(o);
            cnt = 0;
            for (uint32_t ty = y0; ty < y1; ++ty)
                for (uint32_t tx = x0; tx < x1; ++tx)
                    cnt += (uint32_t)tile_kept(u, v, cA, cB, cC, tau, tx, ty, cam->tile);
        }

        depth[i] = pz;
        mean2d[i] = u; mean2d[N + i] = v;
        cov2d[i] = a; cov2d[N + i] = b; cov2d[2 * N + i] = c;
        conic[i] = cA; conic[N + i] = cB; conic[2 * N + i] = cC;

        /* 9. view-dependent colour from SH, fp64:
         * rgb = max(0, 0.5 + sum_k Y_k(dir) sh_k) [reading: offset and clamp] */
        double dir[3] = { (double)mx - (double)cam->cam_pos[0],
                          (double)my - (double)cam->cam_pos[1],
                          (double)mz - (double)cam->cam_pos[2] };
        const double len = sqrt(dir[0] * dir[0] + dir[1] * dir[1] + dir[2] * dir[2]);
        dir[0] /= len; dir[1] /= len; dir[2] /= len;
        double Y[16];
        lmk_ref_sh_basis(dir, Y);
        for (int ch = 0; ch < 3; ++ch) {
            double acc = 0.5;
            for (uint32_t k = 0; k < ncoef; ++k)
                acc += Y[k] * (double)sh[((size_t)k * 3 + ch) * N + i];
            rgb[ch * N + i] = acc > 0.0 ? acc : 0.0;
        }

        if (cnt == 0) { stage[i] = REF_CULL_OFFSCREEN; continue; }
        stage[i] = REF_VISIBLE;
        rect[4 * i] = (uint16_t)x0; rect[4 * i + 1] = (uint16_t)y0;
        rect[4 * i + 2] = (uint16_t)x1; rect[4 * i + 3] = (uint16_t)y1;
        tiles_touched[i] = cnt;
    }
}

/* ------------------------------------------------------------------ */
/* Exclusive prefix sum of tiles_touched; offsets has n+1 entries; returns D. */
uint64_t lmk_ref_scan(uint32_t n, const uint32_t *tiles_touched, uint64_t *offsets)
{
    uint64_t run = 0;
    for (uint32_t i = 0; i < n; ++i) { offsets[i] = run; run += tiles_touched[i]; }
    offsets[n] = run;
    return run;
}

/* One (key,value) per (primitive, kept tile of its rectangle), rectangle walked
 * row-major, primitives in index order.  Under binning rule 0 every tile of the
 * rectangle is kept; under rule 1 only those passing tile_kept().
 * [reading] key = tile_id << 32 | bits(depth); value = primitive index. */
void lmk_ref_emit(uint32_t n, const uint32_t *tiles_touched, const uint16_t *rect,
                  const float *depth, const uint64_t *offsets, uint32_t tiles_x,
                  uint32_t binning, uint32_t ts, const float *mean2d, const float *conic,
                  const float *opacity, uint64_t *keys, uint32_t *vals)
{
    const size_t N = n;
    init_tau_table();
    for (uint32_t i = 0; i < n; ++i) {
        if (tiles_touched[i] == 0) continue;
        uint64_t o = offsets[i];
        const float tau = binning == 1 ? opacity_tau(opacity[i]) : 0.0f;
        for (uint32_t ty = rect[4 * i + 1]; ty < rect[4 * i + 3]; ++ty)
            for (uint32_t tx = rect[4 * i]; tx < rect[4 * i + 2]; ++tx) {
                if (binning == 1 && !tile_kept(mean2d[i], mean2d[N + i], conic[i], conic[N + i],
                                               conic[2 * N + i], tau, tx, ty, ts))
                    continue;
                keys[o] = ((uint64_t)(ty * tiles_x + tx) << 32) | f32_bits(depth[i]);
                vals[o] = i;
                ++o;
            }
    }
}

typedef struct { uint64_t key; uint32_t val; } ref_pair;

static int pair_cmp(const void *pa, const void *pb)
{
    const ref_pair *a = (const ref_pair *)pa, *b = (const ref_pair *)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    if (a->val != b->val) return a->val < b->val ? -1 : 1;
    return 0;
}

/* Sort ascending by (tile, depth bits, primitive index) [reading: index as the
 * tie-break, which makes the order unique].  In place. */
void lmk_ref_sort(uint64_t count, uint64_t *keys, uint32_t *vals)
{
    ref_pair *p = (ref_pair *)malloc((size_t)(count ? count : 1) * sizeof(ref_pair));
    for (uint64_t i = 0; i < count; ++i) { p[i].key = keys[i]; p[i].val = vals[i]; }
    qsort(p, (size_t)count, sizeof(ref_pair), pair_cmp);
    for (uint64_t i = 0; i < count; ++i) { keys[i] = p[i].key; vals[i] = p[i].val; }
    free(p);
}

/* tile_offsets[t] = number of sorted pairs whose tile id is < t, t = 0..T
 * [reading: an empty tile has start == end]. */
void lmk_ref_ranges(uint64_t count, const uint64_t *keys, uint32_t num_tiles, uint64_t *tile_offsets)
{
    for (uint32_t t = 0; t <= num_tiles; ++t) tile_offsets[t] = 0;
    for (uint64_t i = 0; i < count; ++i) {
        uint64_t t = keys[i] >> 32;
        if (t + 1 <= num_tiles) tile_offsets[t + 1] += 1;
    }
    for (uint32_t t = 0; t < num_tiles; ++t) tile_offsets[t + 1] += tile_offsets[t];
}

/* ------------------------------------------------------------------ */
/* Eq. 9-10 for one pixel: walk `count` primitives (indices in list, already in
 * front-to-back order) and composite.
 *   q = A dx^2 + 2 B dx dy + C dy^2, dx = u - px, dy = v - py
 *   alpha = min(0.99, o exp(min(0, -q/2)))            [reading: both clamps]
 *   skip when alpha < 1/255                            [reading]
 *   stop, without compositing, when T (1-alpha) < 1e-4 [reading]
 * Also counts E (entries visited, including the one that stopped the walk) and
 * C (entries composited), and the pixel's error budget for an fp32 renderer
 * (image tolerance rule):
 *   - rounding: an fp32 evaluation of q carries an absolute error of up to
 *     about 8 * 2^-24 * (|A| dx^2 + 2 |B dx dy| + |C| dy^2), which matters when
 *     the terms are large and cancel (long thin splats far from their centre);
 *     it is propagated to first order through alpha and T;
 *   - ambiguity: a pair whose alpha (or whose T') is within that rounding of
 *     its threshold may be decided the other way, which moves the pixel by the
 *     pair's whole contribution.  `amb` counts such decisions.
 * beta bounds the colour error from both, beta_T the transmittance error.
 */
typedef struct {
    double rgb[3]; double T; uint32_t E, C, amb; double beta, beta_T;
} ref_pixel;

static void composite_pixel(double pxc, double pyc, const uint32_t *list, uint64_t count,
                            size_t N, const float *mean2d, const float *conic,
                            const float *opacity, const double *rgb, double cmax,
                            const float bg[3], ref_pixel *out, double *trace, uint32_t trace_cap)
{
    double T = 1.0, acc[3] = { 0.0, 0.0, 0.0 };
    uint32_t E = 0, C = 0;
    uint32_t amb = 0;
    double beta = 0.0, beta_T = 0.0;
    double relT = 0.0;                 /* first-order bound on the relative error of an fp32 T */
    const double EPS = 1.0 / 16777216.0;   /* 2^-24 */
    for (uint64_t k = 0; k < count; ++k) {
        const size_t g = list[k];
        ++E;
        const double dx = (double)mean2d[g] - pxc;
        const double dy = (double)mean2d[N + g] - pyc;
        const double A = conic[g], B = conic[N + g], Cc = conic[2 * N + g];
        const double q = A * dx * dx + 2.0 * B * dx * dy + Cc * dy * dy;
        double power = -0.5 * q;
        if (power > 0.0) power = 0.0;
        const double raw = (double)opacity[g] * exp(power);
        double alpha = raw;
        if (alpha > (double)REF_ALPHA_MAX) alpha = (double)REF_ALPHA_MAX;
        /* error budget of this pair */
        const double mag = fabs(A) * dx * dx + 2.0 * fabs(B * dx * dy) + fabs(Cc) * dy * dy;
        const double dalpha = 0.5 * 8.0 * EPS * mag + 8.0 * EPS;   /* relative error of an fp32 alpha */
        if (fabs(log(255.0 * raw)) <= dalpha + 1e-6) {
            ++amb; beta += 2.0 * alpha * T * cmax; beta_T += alpha * T;
        }
        if ((float)alpha < REF_ALPHA_MIN) {
            if (trace && E <= trace_cap) trace[E - 1] = T;
            continue;
        }
        const double Tn = T * (1.0 - alpha);
        const double relTn = relT + alpha * dalpha / (1.0 - alpha) + 2.0 * EPS;
        if (fabs(Tn / (double)REF_T_MIN - 1.0) <= relTn + 1e-6) {
            ++amb; beta += (alpha * T + Tn) * cmax; beta_T += T;
        }
        if ((float)Tn < REF_T_MIN) {
            if (trace && E <= trace_cap) trace[E - 1] = T;
            break;
        }
        const double w = alpha * T;
        acc[0] += rgb[g] * w;
        acc[1] += rgb[N + g] * w;
        acc[2] += rgb[2 * N + g] * w;
        double cg = rgb[g];
        if (rgb[N + g] > cg) cg = rgb[N + g];
        if (rgb[2 * N + g] > cg) cg = rgb[2 * N + g];
        beta += w * cg * (dalpha + relT + 4.0 * EPS);
        T = Tn;
        relT = relTn;
        ++C;
        if (trace && E <= trace_cap) trace[E - 1] = T;
    }
    beta += T * relT * cmax;           /* cmax >= 1 >= |bg| is assumed by the tests */
    beta_T += T * relT;
    out->rgb[0] = acc[0] + T * (double)bg[0];
    out->rgb[1] = acc[1] + T * (double)bg[1];
    out->rgb[2] = acc[2] + T * (double)bg[2];
    out->T = T; out->E = E; out->C = C; out->amb = amb; out->beta = beta; out->beta_T = beta_T;
}

static double max_rgb(uint32_t n, const uint8_t *stage, const double *rgb)
{
    double m = 1.0;
    for (size_t i = 0; i < (size_t)n; ++i)
        if (stage[i] == REF_VISIBLE || stage[i] == REF_CULL_OFFSCREEN)
            for (int ch = 0; ch < 3; ++ch)
                if (rgb[ch * (size_t)n + i] > m) m = rgb[ch * (size_t)n + i];
    return m;
}

/* Tile pipeline render: every pixel walks the sorted slice of its tile.
 * out_rgb [3][H][W], out_T [H][W], out_E/out_C [H][W], beta/beta_T/amb [H][W]. */
void lmk_ref_render(uint32_t n, const uint8_t *stage, const float *mean2d, const float *conic,
                    const float *opacity, const double *rgb,
                    const uint32_t *sorted_vals, const uint64_t *tile_offsets,
                    const ref_camera *cam,
                    double *out_rgb, double *out_T, uint32_t *out_E, uint32_t *out_C,
                    double *out_beta, double *out_beta_T, uint32_t *out_amb)
{
    const uint32_t W = cam->width, H = cam->height, TS = cam->tile;
    const uint32_t TX = (W + TS - 1) / TS;
    const double cmax = max_rgb(n, stage, rgb);
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t jj = 0; jj < (int64_t)H; ++jj) {
        const uint32_t j = (uint32_t)jj;
        for (uint32_t i = 0; i < W; ++i) {
            const uint32_t t = (j / TS) * TX + (i / TS);
            ref_pixel r;
            composite_pixel((double)i + 0.5, (double)j + 0.5,
                            sorted_vals + tile_offsets[t], tile_offsets[t + 1] - tile_offsets[t],
                            n, mean2d, conic, opacity, rgb, cmax, cam->bg, &r, NULL, 0);
            const size_t p = (size_t)j * W + i;
            for (int ch = 0; ch < 3; ++ch) out_rgb[(size_t)ch * H * W + p] = r.rgb[ch];
            out_T[p] = r.T; out_E[p] = r.E; out_C[p] = r.C;
            out_beta[p] = r.beta; out_beta_T[p] = r.beta_T; out_amb[p] = r.amb;
        }
    }
}

/* ------------------------------------------------------------------ */
/* The definition the tile pipeline must reach: front-to-back order of ALL
 * primitives that pass the per-primitive culls 1, 4 and 6 (their rectangle is
 * ignored, so off-screen ones are included), by (depth bits, index).
 * Writes the order to `order` (capacity n) and returns its length. */
typedef struct { uint32_t bits, idx; } ref_di;
static int di_cmp(const void *pa, const void *pb)
{
    const ref_di *a = (const ref_di *)pa, *b = (const ref_di *)pb;
    if (a->bits != b->bits) return a->bits < b->bits ? -1 : 1;
    if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;
    return 0;
}

uint32_t lmk_ref_depth_order(uint32_t n, const uint8_t *stage, const float *depth, uint32_t *order)
{
    ref_di *p = (ref_di *)malloc(((size_t)n + 1) * sizeof(ref_di));
    uint32_t m = 0;
    for (uint32_t i = 0; i < n; ++i)
        if (stage[i] == REF_VISIBLE || stage[i] == REF_CULL_OFFSCREEN) {
            p[m].bits = f32_bits(depth[i]); p[m].idx = i; ++m;
        }
    qsort(p, m, sizeof(ref_di), di_cmp);
    for (uint32_t k = 0; k < m; ++k) order[k] = p[k].idx;
    free(p);
    return m;
}

/* Brute force at chosen pixels: each walks the whole depth order.
 * xs, ys: integer pixel coordinates; outputs are per sample:
 * out_rgb [npix][3], out_T, out_C, out_beta, out_beta_T, out_amb [npix]. */
void lmk_ref_render_pixels_brute(uint32_t n, const uint8_t *stage, const float *mean2d,
                                 const float *conic, const float *opacity, const double *rgb,
                                 const uint32_t *order, uint32_t order_len, const ref_camera *cam,
                                 uint32_t npix, const uint32_t *xs, const uint32_t *ys,
                                 double *out_rgb, double *out_T, uint32_t *out_C,
                                 double *out_beta, double *out_beta_T, uint32_t *out_amb)
{
    const double cmax = max_rgb(n, stage, rgb);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t kk = 0; kk < (int64_t)npix; ++kk) {
        const size_t k = (size_t)kk;
        ref_pixel r;
        composite_pixel((double)xs[k] + 0.5, (double)ys[k] + 0.5, order, order_len,
                        n, mean2d, conic, opacity, rgb, cmax, cam->bg, &r, NULL, 0);
        for (int ch = 0; ch < 3; ++ch) out_rgb[3 * k + ch] = r.rgb[ch];
        out_T[k] = r.T; out_C[k] = r.C; out_beta[k] = r.beta; out_beta_T[k] = r.beta_T; out_amb[k] = r.amb;
    }
}

/* The sorted list of one tile, straight from the definition: every primitive
 * whose rectangle contains the tile, ordered by (depth bits, index).
 * out_vals has capacity cap; returns the list length (which may exceed cap,
 * in which case only cap entries were written). */
uint64_t lmk_ref_tile_list(uint32_t n, const uint32_t *tiles_touched, const uint16_t *rect,
                           const float *depth, uint32_t tile_x, uint32_t tile_y,
                           uint32_t binning, uint32_t ts, const float *mean2d, const float *conic,
                           const float *opacity, uint32_t *out_vals, uint64_t cap)
{
    const size_t N = n;
    init_tau_table();
    ref_di *p = NULL;
    uint64_t m = 0, have = 0;
    for (int pass = 0; pass < 2; ++pass) {
        uint64_t k = 0;
        for (uint32_t i = 0; i < n; ++i) {
            if (!(tiles_touched[i] && rect[4 * i] <= tile_x && tile_x < rect[4 * i + 2] &&
                  rect[4 * i + 1] <= tile_y && tile_y < rect[4 * i + 3]))
                continue;
            if (binning == 1 && !tile_kept(mean2d[i], mean2d[N + i], conic[i], conic[N + i],
                                           conic[2 * N + i], opacity_tau(opacity[i]), tile_x, tile_y, ts))
                continue;
            if (pass == 1) { p[k].bits = f32_bits(depth[i]); p[k].idx = i; }
            ++k;
        }
        if (pass == 0) { m = k; p = (ref_di *)malloc((size_t)(m + 1) * sizeof(ref_di)); }
        else have = k;
    }
    (void)have;
    qsort(p, (size_t)m, sizeof(ref_di), di_cmp);
    for (uint64_t j = 0; j < m && j < cap; ++j) out_vals[j] = p[j].idx;
    free(p);
    return m;
}

/* The sorted lists of every tile of a band of tile rows [ty0, ty1), for frames too large to bin
 * whole on the host.  The primitives are visited in front-to-back order (`order`, from
 * lmk_ref_depth_order), and a primitive is appended to the list of every tile of the band that its
 * rectangle contains (binning rule 1: and on which tile_kept holds): the lists are born in
 * (depth bits, index) order, which is the sorted order of step 12 restricted to one tile.
 * out_offsets[k], k = 0 .. (ty1 - ty0) * tiles_x: start of the list of tile (ty0 * tiles_x + k) inside
 * out_vals; out_vals has capacity cap.  Returns the number of pairs of the band; if that exceeds
 * cap only out_offsets is complete and nothing is written to out_vals. */
uint64_t lmk_ref_band_lists(uint32_t n, const uint32_t *tiles_touched, const uint16_t *rect,
                            const uint32_t *order, uint32_t order_len,
                            uint32_t binning, uint32_t ts, uint32_t tiles_x, uint32_t ty0, uint32_t ty1,
                            const float *mean2d, const float *conic, const float *opacity,
                            uint64_t *out_offsets, uint32_t *out_vals, uint64_t cap)
{
    const size_t N = n;
    const uint32_t rows = ty1 - ty0;
    const size_t nt = (size_t)rows * tiles_x;
    init_tau_table();
    uint64_t *count = (uint64_t *)calloc(nt + 1, sizeof(uint64_t));
    for (int pass = 0; pass < 2; ++pass) {
        /* one tile row at a time; rows are independent */
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t rr = 0; rr < (int64_t)rows; ++rr) {
            const uint32_t ty = ty0 + (uint32_t)rr;
            uint64_t *cur = (uint64_t *)malloc((size_t)tiles_x * sizeof(uint64_t));
            for (uint32_t tx = 0; tx < tiles_x; ++tx)
                cur[tx] = pass ? out_offsets[(size_t)rr * tiles_x + tx] : 0;
            for (uint32_t k = 0; k < order_len; ++k) {
                const uint32_t i = order[k];
                if (!tiles_touched[i] || !(rect[4 * i + 1] <= ty && ty < rect[4 * i + 3])) continue;
                for (uint32_t tx = rect[4 * i]; tx < rect[4 * i + 2] && tx < tiles_x; ++tx) {
                    if (binning == 1 && !tile_kept(mean2d[i], mean2d[N + i], conic[i], conic[N + i],
                                                   conic[2 * N + i], opacity_tau(opacity[i]), tx, ty, ts))
                        continue;
                    if (pass) out_vals[cur[tx]] = i;
                    ++cur[tx];
                }
            }
            if (!pass)
                for (uint32_t tx = 0; tx < tiles_x; ++tx) count[(size_t)rr * tiles_x + tx] = cur[tx];
            free(cur);
        }
        if (!pass) {
            uint64_t run = 0;
            for (size_t t = 0; t < nt; ++t) { out_offsets[t] = run; run += count[t]; }
            out_offsets[nt] = run;
            if (run > cap) { free(count); return run; }
        }
    }
    free(count);
    return out_offsets[nt];
}

/* Step 14 for the pixel rows of a band of tile rows [ty0, ty1) through the lists of
 * lmk_ref_band_lists: outputs are [rows_px][W] (rgb: [3][rows_px][W]), rows_px = the band's
 * pixel rows inside the image. */
void lmk_ref_render_band(uint32_t n, const uint8_t *stage, const float *mean2d, const float *conic,
                         const float *opacity, const double *rgb,
                         const uint32_t *band_vals, const uint64_t *band_offsets,
                         const ref_camera *cam, uint32_t ty0, uint32_t ty1,
                         double *out_rgb, double *out_T, uint32_t *out_E, uint32_t *out_C,
                         double *out_beta, double *out_beta_T, uint32_t *out_amb)
{
    const uint32_t W = cam->width, H = cam->height, TS = cam->tile;
    const uint32_t TX = (W + TS - 1) / TS;
    const uint32_t y0 = ty0 * TS, y1 = ty1 * TS < H ? ty1 * TS : H;
    const size_t rows = y1 > y0 ? y1 - y0 : 0;
    const double cmax = max_rgb(n, stage, rgb);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t jj = 0; jj < (int64_t)rows; ++jj) {
        const uint32_t j = y0 + (uint32_t)jj;
        for (uint32_t i = 0; i < W; ++i) {
            const size_t t = (size_t)(j / TS - ty0) * TX + (i / TS);
            ref_pixel r;
            composite_pixel((double)i + 0.5, (double)j + 0.5,
                            band_vals + band_offsets[t], band_offsets[t + 1] - band_offsets[t],
                            n, mean2d, conic, opacity, rgb, cmax, cam->bg, &r, NULL, 0);
            const size_t p = (size_t)jj * W + i;
            for (int ch = 0; ch < 3; ++ch) out_rgb[(size_t)ch * rows * W + p] = r.rgb[ch];
            out_T[p] = r.T; out_E[p] = r.E; out_C[p] = r.C;
            out_beta[p] = r.beta; out_beta_T[p] = r.beta_T; out_amb[p] = r.amb;
        }
    }
}

/* Walk an explicit list at chosen pixels (used with lmk_ref_tile_list to check
 * tiles of a frame too large to bin whole on the host). */
void lmk_ref_render_pixels_list(uint32_t n, const uint8_t *stage, const float *mean2d,
                                const float *conic, const float *opacity, const double *rgb,
                                const uint32_t *list, uint64_t list_len, const ref_camera *cam,
                                uint32_t npix, const uint32_t *xs, const uint32_t *ys,
                                double *out_rgb, double *out_T, uint32_t *out_E, uint32_t *out_C,
                                double *out_beta, double *out_beta_T, uint32_t *out_amb)
{
    const double cmax = max_rgb(n, stage, rgb);
    for (size_t k = 0; k < (size_t)npix; ++k) {
        ref_pixel r;
        composite_pixel((double)xs[k] + 0.5, (double)ys[k] + 0.5, list, list_len,
                        n, mean2d, conic, opacity, rgb, cmax, cam->bg, &r, NULL, 0);
        for (int ch = 0; ch < 3; ++ch) out_rgb[3 * k + ch] = r.rgb[ch];
        out_T[k] = r.T; out_E[k] = r.E; out_C[k] = r.C;
        out_beta[k] = r.beta; out_beta_T[k] = r.beta_T; out_amb[k] = r.amb;
    }
}

/* Transmittance after each visited entry of one pixel's walk over `list`
 * (for the monotonicity pin); returns the number of entries visited. */
uint32_t lmk_ref_trace_pixel(uint32_t n, const float *mean2d, const float *conic,
                             const float *opacity, const double *rgb,
                             const uint32_t *list, uint64_t count,
                             uint32_t x, uint32_t y, double *trace, uint32_t cap)
{
    const float bg[3] = { 0.0f, 0.0f, 0.0f };
    ref_pixel r;
    composite_pixel((double)x + 0.5, (double)y + 0.5, list, count, n, mean2d, conic,
                    opacity, rgb, 1.0, bg, &r, trace, cap);
    return r.E;
}


/* ------------------------------------------------------------------------
 * View-frustum filtering of a voxel grid (Sec. 4.2.2, frustum-based dynamic loading:
 * primitives are reordered offline into voxels, and per frame the voxels are
 * filtered against the view frustum instead of the primitives).  [reading: the
 * report gives no formula.]  A voxel is described by the bounding box of the
 * means of its primitives and by smax, the largest scale component among them.
 * It may be skipped only if every primitive in it is certain to be culled by
 * steps 1 and 8 of lmk_ref_preprocess:
 *  - near: every point of the box has camera z <= near;
 *  - sides: for a primitive at camera-space (x, y, z), z > 0, the half-width of
 *    its support in pixels is at most fx R / z + r0, with
 *    R = sqrt(tau) sqrt(1 + lim_x^2) smax  (row norm of the clamped Jacobian
 *    times the largest eigenvalue of Sigma) and r0 = sqrt(tau h); so it is off
 *    the left edge if fx x + (cx + r0) z < -fx R, a linear inequality, and a
 *    linear function over a box takes its extremes at the corners.  Likewise
 *    for the other three edges (the right and bottom edges are those of the
 *    tile grid, 16 TX and 16 TY).
 * All of it in fp32 like the other key-path steps, with a relative slack so
 * that rounding can only keep a voxel too many.  Assumes the 3x3 part of the
 * view matrix is a rotation.
 */
int lmk_ref_voxel_visible(const ref_camera *cam, const float lo[3], const float hi[3], float smax)
{
    const float *V = cam->view;
    const uint32_t TX = (cam->width + cam->tile - 1) / cam->tile;
    const uint32_t TY = (cam->height + cam->tile - 1) / cam->tile;
    const float XW = (float)(TX * cam->tile), YH = (float)(TY * cam->tile);
    const float lim_x = 1.3f * ((0.5f * (float)cam->width) / cam->fx);
    const float lim_y = 1.3f * ((0.5f * (float)cam->height) / cam->fy);
    const float st = sqrtf(REF_TAU);
    const float Rx = (st * sqrtf(1.0f + lim_x * lim_x)) * smax;
    const float Ry = (st * sqrtf(1.0f + lim_y * lim_y)) * smax;
    const float r0 = sqrtf(REF_TAU * cam->lowpass);
    const float cl = cam->cx + r0, cr = (cam->cx - r0) - XW;
    const float ct = cam->cy + r0, cb = (cam->cy - r0) - YH;
    float zmax = 0.0f, maxL = 0.0f, minR = 0.0f, maxT = 0.0f, minB = 0.0f, mag = 0.0f;
    for (int k = 0; k < 8; ++k) {
        const float wx = (k & 1) ? hi[0] : lo[0], wy = (k & 2) ? hi[1] : lo[1], wz = (k & 4) ? hi[2] : lo[2];
        const float x = V[0] * wx + V[1] * wy + V[2] * wz + V[3];
        const float y = V[4] * wx + V[5] * wy + V[6] * wz + V[7];
        const float z = V[8] * wx + V[9] * wy + V[10] * wz + V[11];
        const float L = cam->fx * x + cl * z, R = cam->fx * x + cr * z;
        const float T = cam->fy * y + ct * z, B = cam->fy * y + cb * z;
        const float m = (cam->fx * fabsf(x) + cam->fy * fabsf(y)) + ((XW + YH) + (fabsf(cam->cx) + fabsf(cam->cy))) * fabsf(z);
        if (k == 0) { zmax = z; maxL = L; minR = R; maxT = T; minB = B; mag = m; }
        else {
            zmax = z > zmax ? z : zmax; maxL = L > maxL ? L : maxL; minR = R < minR ? R : minR;
            maxT = T > maxT ? T : maxT; minB = B < minB ? B : minB; mag = m > mag ? m : mag;
        }
    }
    const float slack = 1e-5f * mag;
    const float bx = (cam->fx * Rx) * 1.004f, by = (cam->fy * Ry) * 1.004f;
    if (zmax + 1e-5f * fabsf(zmax) < cam->near_z) return 0;         /* behind the near plane */
    if (maxL + slack < -bx) return 0;                               /* off the left edge */
    if (minR - slack > bx) return 0;                                /* off the right edge */
    if (maxT + slack < -by) return 0;                               /* above the top edge */
    if (minB - slack > by) return 0;                                /* below the bottom edge */
    return 1;
}

void lmk_ref_voxels_visible(const ref_camera *cam, uint32_t num_voxels, const float *box_lo,
                            const float *box_hi, const float *smax, uint8_t *visible)
{
    for (uint32_t v = 0; v < num_voxels; ++v)
        visible[v] = (uint8_t)lmk_ref_voxel_visible(cam, box_lo + 3 * (size_t)v, box_hi + 3 * (size_t)v, smax[v]);
}


/* ------------------------------------------------------------------------
 * Gradient of a scalar loss through the compositing of Eq. 9-10 (Sec. 2.2: the
 * rasteriser is differentiable, and all parameters of the primitives are optimised
 * through the rendering process).  Given dL/dC_hat(x') (three channels) and
 * dL/dT_end(x') for every pixel, the gradient with respect to what the compositing
 * reads of every primitive: its 2D mean (u, v), its conic (A, B, C), its opacity o and
 * its colour c.  The chain from there back to the 3D parameters is not part of this
 * function.
 *
 * For one pixel with composited entries i = 1..m in front-to-back order,
 *   T_1 = 1, T_{i+1} = T_i (1 - alpha_i), w_i = alpha_i T_i,
 *   C_hat = sum_i c_i w_i + bg T_{m+1},   T_end = T_{m+1},
 * so, with S_i = sum_{j>i} c_j w_j + bg T_end (what lies behind entry i),
 *   dL/dc_i     = w_i dL/dC_hat
 *   dL/dalpha_i = dL/dC_hat . (T_i c_i - S_i / (1 - alpha_i)) - dL/dT_end T_end / (1 - alpha_i)
 * and alpha_i = o_i exp(-q_i / 2), q = A dx^2 + 2 B dx dy + C dy^2, dx = u - px, dy = v - py:
 *   dalpha/do = exp(-q/2),  dalpha/dq = -alpha / 2,
 *   dq/dA = dx^2, dq/dB = 2 dx dy, dq/dC = dy^2, dq/du = 2 (A dx + B dy), dq/dv = 2 (B dx + C dy).
 * [reading] The thresholds of the forward walk are constants of the derivative: an entry
 * that was skipped (alpha < 1/255), the entry that stopped the walk and everything after it
 * get no gradient; where alpha was clamped to 0.99 it does not depend on o or q; where the
 * exponent was clamped to 0 (q < 0) alpha does not depend on q.
 * The forward walk here takes the same steps and the same decisions as composite_pixel
 * (a test compares the two images bit for bit); it also reports the pixels that hold a
 * decision within rounding of its threshold (amb), whose gradients an fp32 renderer may
 * legitimately compute from the other decision.
 * Outputs are accumulated over all pixels in fp64: g_mean2d [2][n], g_conic [3][n],
 * g_opacity [n], g_rgb [3][n] (overwritten).  out_rgb/out_T (may be NULL): the forward image.
 * g_abs (may be NULL) [9][n], rows u, v, A, B, C, o, r, g, b: the same sums with every term
 * replaced by its magnitude (|dL/dC| . (T_i |c_i| + |S_i| / (1 - alpha_i)) + |dL/dT_end| T_end /
 * (1 - alpha_i) in place of dL/dalpha_i), the scale against which an fp32 evaluation's rounding is
 * measured.
 */
typedef struct { uint32_t g; double alpha, gauss, dx, dy, T; int clamped_alpha, clamped_power; } ref_entry;

void lmk_ref_render_backward(uint32_t n, const float *mean2d, const float *conic,
                             const float *opacity, const double *rgb,
                             const uint32_t *sorted_vals, const uint64_t *tile_offsets,
                             const ref_camera *cam, const double *grad_rgb, const double *grad_T,
                             double *g_mean2d, double *g_conic, double *g_opacity, double *g_rgb,
                             double *out_rgb, double *out_T, uint32_t *out_amb, double *g_abs)
{
    const uint32_t W = cam->width, H = cam->height, TS = cam->tile;
    const uint32_t TX = (W + TS - 1) / TS;
    const size_t N = n, HW = (size_t)H * W;
    const double EPS = 1.0 / 16777216.0;
    memset(g_mean2d, 0, sizeof(double) * 2 * N);
    memset(g_conic, 0, sizeof(double) * 3 * N);
    memset(g_opacity, 0, sizeof(double) * N);
    memset(g_rgb, 0, sizeof(double) * 3 * N);
    if (g_abs) memset(g_abs, 0, sizeof(double) * 9 * N);
#pragma omp parallel
    {
        ref_entry *rec = NULL;
        size_t rec_cap = 0;
#pragma omp for schedule(dynamic, 4)
        for (int64_t jj = 0; jj < (int64_t)H; ++jj) {
            const uint32_t j = (uint32_t)jj;
            for (uint32_t i = 0; i < W; ++i) {
                const uint32_t t = (j / TS) * TX + (i / TS);
                const uint32_t *list = sorted_vals + tile_offsets[t];
                const uint64_t count = tile_offsets[t + 1] - tile_offsets[t];
                if (count > rec_cap) {
                    free(rec);
                    rec_cap = (size_t)count + 64;
                    rec = (ref_entry *)malloc(sizeof(ref_entry) * rec_cap);
                }
                const double pxc = (double)i + 0.5, pyc = (double)j + 0.5;
                const size_t p = (size_t)j * W + i;
                /* forward walk, recording the composited entries */
                double T = 1.0, acc[3] = { 0.0, 0.0, 0.0 }, relT = 0.0;
                uint32_t m = 0, amb = 0;
                for (uint64_t k = 0; k < count; ++k) {
                    const size_t g = list[k];
                    const double dx = (double)mean2d[g] - pxc;
                    const double dy = (double)mean2d[N + g] - pyc;
                    const double A = conic[g], B = conic[N + g], Cc = conic[2 * N + g];
                    const double q = A * dx * dx + 2.0 * B * dx * dy + Cc * dy * dy;
                    double power = -0.5 * q;
                    const int cp = power > 0.0;
                    if (cp) power = 0.0;
                    const double gauss = exp(power);
                    const double raw = (double)opacity[g] * gauss;
                    double alpha = raw;
                    const int ca = alpha > (double)REF_ALPHA_MAX;
                    if (ca) alpha = (double)REF_ALPHA_MAX;
                    const double mag = fabs(A) * dx * dx + 2.0 * fabs(B * dx * dy) + fabs(Cc) * dy * dy;
                    const double dalpha = 0.5 * 8.0 * EPS * mag + 8.0 * EPS;
                    if (fabs(log(255.0 * raw)) <= dalpha + 1e-6) ++amb;
                    if (fabs(raw / (double)REF_ALPHA_MAX - 1.0) <= dalpha + 1e-6) ++amb;   /* at the 0.99 clamp */
                    if ((float)alpha < REF_ALPHA_MIN) continue;
                    const double Tn = T * (1.0 - alpha);
                    const double relTn = relT + alpha * dalpha / (1.0 - alpha) + 2.0 * EPS;
                    if (fabs(Tn / (double)REF_T_MIN - 1.0) <= relTn + 1e-6) ++amb;
                    if ((float)Tn < REF_T_MIN) break;
                    const double w = alpha * T;
                    acc[0] += rgb[g] * w; acc[1] += rgb[N + g] * w; acc[2] += rgb[2 * N + g] * w;
                    rec[m].g = (uint32_t)g; rec[m].alpha = alpha; rec[m].gauss = gauss;
                    rec[m].dx = dx; rec[m].dy = dy; rec[m].T = T;
                    rec[m].clamped_alpha = ca; rec[m].clamped_power = cp;
                    ++m;
                    T = Tn; relT = relTn;
                }
                if (out_rgb)
                    for (int ch = 0; ch < 3; ++ch) out_rgb[(size_t)ch * HW + p] = acc[ch] + T * (double)cam->bg[ch];
                if (out_T) out_T[p] = T;
                if (out_amb) out_amb[p] = amb;
                /* back to front */
                const double Gc[3] = { grad_rgb[p], grad_rgb[HW + p], grad_rgb[2 * HW + p] };
                const double GT = grad_T ? grad_T[p] : 0.0;
                const double Tend = T;
                double S[3] = { (double)cam->bg[0] * Tend, (double)cam->bg[1] * Tend, (double)cam->bg[2] * Tend };
                double Sabs[3] = { fabs(S[0]), fabs(S[1]), fabs(S[2]) };
                for (uint32_t e = m; e-- > 0;) {
                    const ref_entry *r = &rec[e];
                    const size_t g = r->g;
                    const double c[3] = { rgb[g], rgb[N + g], rgb[2 * N + g] };
                    const double w = r->alpha * r->T;
                    const double inv = 1.0 / (1.0 - r->alpha);
                    double dLda = -GT * Tend * inv;
                    for (int ch = 0; ch < 3; ++ch) dLda += Gc[ch] * (r->T * c[ch] - S[ch] * inv);
                    double mag = fabs(GT) * Tend * inv;
                    for (int ch = 0; ch < 3; ++ch) mag += fabs(Gc[ch]) * (r->T * fabs(c[ch]) + Sabs[ch] * inv);
                    for (int ch = 0; ch < 3; ++ch) {
#pragma omp atomic
                        g_rgb[(size_t)ch * N + g] += w * Gc[ch];
                        if (g_abs) {
#pragma omp atomic
                            g_abs[(size_t)(6 + ch) * N + g] += w * fabs(Gc[ch]);
                        }
                        S[ch] += c[ch] * w;
                        Sabs[ch] += fabs(c[ch]) * w;
                    }
                    if (g_abs && !r->clamped_alpha) {
                        const double mq = r->clamped_power ? 0.0 : mag * 0.5 * r->alpha;
                        const double Aa = fabs((double)conic[g]), Ba = fabs((double)conic[N + g]), Ca = fabs((double)conic[2 * N + g]);
                        const double ax = fabs(r->dx), ay = fabs(r->dy);
#pragma omp atomic
                        g_abs[0 * N + g] += mq * 2.0 * (Aa * ax + Ba * ay);
#pragma omp atomic
                        g_abs[1 * N + g] += mq * 2.0 * (Ba * ax + Ca * ay);
#pragma omp atomic
                        g_abs[2 * N + g] += mq * ax * ax;
#pragma omp atomic
                        g_abs[3 * N + g] += mq * 2.0 * ax * ay;
#pragma omp atomic
                        g_abs[4 * N + g] += mq * ay * ay;
#pragma omp atomic
                        g_abs[5 * N + g] += mag * r->gauss;
                    }
                    if (r->clamped_alpha) continue;
                    const double dLdo = dLda * r->gauss;
#pragma omp atomic
                    g_opacity[g] += dLdo;
                    if (r->clamped_power) continue;
                    const double dLdq = dLda * (-0.5 * r->alpha);
                    const double A = conic[g], B = conic[N + g], Cc = conic[2 * N + g];
#pragma omp atomic
                    g_conic[g] += dLdq * r->dx * r->dx;
#pragma omp atomic
                    g_conic[N + g] += dLdq * 2.0 * r->dx * r->dy;
#pragma omp atomic
                    g_conic[2 * N + g] += dLdq * r->dy * r->dy;
#pragma omp atomic
                    g_mean2d[g] += dLdq * 2.0 * (A * r->dx + B * r->dy);
#pragma omp atomic
                    g_mean2d[N + g] += dLdq * 2.0 * (B * r->dx + Cc * r->dy);
                }
            }
        }
        free(rec);
    }
}


/* ------------------------------------------------------------------------
 * Gradient of a scalar loss through the per-primitive projection (the chain behind
 * lmk_ref_render_backward: Sec. 2.2 says every parameter of the primitives is optimised through
 * the rendering process).  Given, for each primitive, dL/d{u, v, A, B, C, o, r, g, b} -- the
 * quantities lmk_ref_preprocess hands to the compositing -- the gradient with respect to its
 * mean, scale, rotation quaternion (as stored, any norm), opacity and SH coefficients.
 * Each step of lmk_ref_preprocess is differentiated in reverse order, in fp64, from the fp32
 * inputs:
 *   conic = inverse of [[a, b], [b, c]];  a, b, c = rows of T = J W applied to Sigma (+ h on the
 *   diagonal);  J from the camera-space position p (with the guard-band clamp: where p_x / p_z is
 *   clamped, J's third column depends on p_z only);  u, v from p;  p = W mean + t;
 *   Sigma = M M^T, M = R(q / |q|) diag(s);  colour = max(0, 0.5 + sum_k Y_k(d) sh_k) with
 *   d = (mean - camera centre) / |.|.
 * [reading] Culls and clamps are constants of the derivative: a primitive that lmk_ref_preprocess
 * did not bin (stage != visible) gets zero; a colour channel clamped at 0 passes nothing on.  B is
 * the single off-diagonal value that q = A dx^2 + 2 B dx dy + C dy^2 uses.
 * Outputs (overwritten), same layouts as the inputs: g_mean [3][n], g_scale [3][n], g_rot [4][n],
 * g_opacity [n], g_sh [ncoef][3][n].  g_feat: [9][n] planes u, v, A, B, C, o, r, g, b.
 */
static void sh_basis_grad(const double d[3], double dY[16][3])
{
    const double x = d[0], y = d[1], z = d[2];
    const double xx = x * x, yy = y * y, zz = z * z;
    const double k1 = sqrt(3.0 / (4.0 * M_PI));
    const double k2 = 0.5 * sqrt(15.0 / M_PI);
    const double k20 = 0.25 * sqrt(5.0 / M_PI);
    const double k33 = 0.25 * sqrt(35.0 / (2.0 * M_PI));
    const double k32 = 0.5 * sqrt(105.0 / M_PI);
    const double k31 = 0.25 * sqrt(21.0 / (2.0 * M_PI));
    const double k30 = 0.25 * sqrt(7.0 / M_PI);
    const double k32b = 0.25 * sqrt(105.0 / M_PI);
    memset(dY, 0, sizeof(double) * 16 * 3);
    dY[1][1] = -k1;
    dY[2][2] = k1;
    dY[3][0] = -k1;
    dY[4][0] = k2 * y;            dY[4][1] = k2 * x;
    dY[5][1] = -k2 * z;           dY[5][2] = -k2 * y;
    dY[6][0] = -2.0 * k20 * x;    dY[6][1] = -2.0 * k20 * y;   dY[6][2] = 4.0 * k20 * z;
    dY[7][0] = -k2 * z;           dY[7][2] = -k2 * x;
    dY[8][0] = k2 * x;            dY[8][1] = -k2 * y;
    dY[9][0] = -k33 * 6.0 * x * y;                 dY[9][1] = -k33 * (3.0 * xx - 3.0 * yy);
    dY[10][0] = k32 * y * z;      dY[10][1] = k32 * x * z;     dY[10][2] = k32 * x * y;
    dY[11][0] = k31 * 2.0 * x * y;
    dY[11][1] = -k31 * (4.0 * zz - xx - 3.0 * yy);
    dY[11][2] = -k31 * 8.0 * y * z;
    dY[12][0] = -k30 * 6.0 * x * z;
    dY[12][1] = -k30 * 6.0 * y * z;
    dY[12][2] = k30 * (6.0 * zz - 3.0 * xx - 3.0 * yy);
    dY[13][0] = -k31 * (4.0 * zz - 3.0 * xx - yy);
    dY[13][1] = k31 * 2.0 * x * y;
    dY[13][2] = -k31 * 8.0 * x * z;
    dY[14][0] = k32b * 2.0 * x * z;
    dY[14][1] = -k32b * 2.0 * y * z;
    dY[14][2] = k32b * (xx - yy);
    dY[15][0] = -k33 * (3.0 * xx - 3.0 * yy);
    dY[15][1] = k33 * 6.0 * x * y;
}

void lmk_ref_preprocess_backward(uint32_t n, const float *mean, const float *scale, const float *rot,
                                 const float *sh, uint32_t sh_degree,
                                 const ref_camera *cam, const uint8_t *stage, const double *g_feat,
                                 double *g_mean, double *g_scale, double *g_rot, double *g_opacity,
                                 double *g_sh)
{
    const size_t N = n;
    const uint32_t ncoef = (sh_degree + 1) * (sh_degree + 1);
    const double lim_x = (double)(1.3f * ((0.5f * (float)cam->width) / cam->fx));
    const double lim_y = (double)(1.3f * ((0.5f * (float)cam->height) / cam->fy));
    const float *V = cam->view;
    const double fx = cam->fx, fy = cam->fy;
    memset(g_mean, 0, sizeof(double) * 3 * N);
    memset(g_scale, 0, sizeof(double) * 3 * N);
    memset(g_rot, 0, sizeof(double) * 4 * N);
    memset(g_opacity, 0, sizeof(double) * N);
    memset(g_sh, 0, sizeof(double) * (size_t)ncoef * 3 * N);
#pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)n; ++ii) {
        const size_t i = (size_t)ii;
        if (stage[i] != REF_VISIBLE) continue;
        const double gu = g_feat[i], gv = g_feat[N + i];
        const double gA = g_feat[2 * N + i], gB = g_feat[3 * N + i], gC = g_feat[4 * N + i];
        const double gcol[3] = { g_feat[6 * N + i], g_feat[7 * N + i], g_feat[8 * N + i] };
        g_opacity[i] = g_feat[5 * N + i];

        /* forward quantities, fp64 from the fp32 inputs */
        const double m[3] = { mean[i], mean[N + i], mean[2 * N + i] };
        double W[3][3], p[3];
        for (int r = 0; r < 3; ++r) {
            for (int c = 0; c < 3; ++c) W[r][c] = V[4 * r + c];
            p[r] = W[r][0] * m[0] + W[r][1] * m[1] + W[r][2] * m[2] + (double)V[4 * r + 3];
        }
        const double qr[4] = { rot[i], rot[N + i], rot[2 * N + i], rot[3 * N + i] };
        const double qn = sqrt(qr[0] * qr[0] + qr[1] * qr[1] + qr[2] * qr[2] + qr[3] * qr[3]);
        const double w = qr[0] / qn, x = qr[1] / qn, y = qr[2] / qn, z = qr[3] / qn;
        double R[3][3];
        R[0][0] = 1.0 - 2.0 * (y * y + z * z); R[0][1] = 2.0 * (x * y - w * z); R[0][2] = 2.0 * (x * z + w * y);
        R[1][0] = 2.0 * (x * y + w * z); R[1][1] = 1.0 - 2.0 * (x * x + z * z); R[1][2] = 2.0 * (y * z - w * x);
        R[2][0] = 2.0 * (x * z - w * y); R[2][1] = 2.0 * (y * z + w * x); R[2][2] = 1.0 - 2.0 * (x * x + y * y);
        const double s[3] = { scale[i], scale[N + i], scale[2 * N + i] };
        double M[3][3], Sg[3][3];
        for (int r = 0; r < 3; ++r) for (int c = 0; c < 3; ++c) M[r][c] = R[r][c] * s[c];
        for (int r = 0; r < 3; ++r)
            for (int c = 0; c < 3; ++c) Sg[r][c] = M[r][0] * M[c][0] + M[r][1] * M[c][1] + M[r][2] * M[c][2];
        const double rx = p[0] / p[2], ry = p[1] / p[2];
        const int clx = !(rx > -lim_x) || rx > lim_x, cly = !(ry > -lim_y) || ry > lim_y;
        const double cxr = !(rx > -lim_x) ? -lim_x : (rx > lim_x ? lim_x : rx);
        const double cyr = !(ry > -lim_y) ? -lim_y : (ry > lim_y ? lim_y : ry);
        double J[2][3] = { { fx / p[2], 0.0, -fx * cxr / p[2] }, { 0.0, fy / p[2], -fy * cyr / p[2] } };
        double T[2][3];
        for (int r = 0; r < 2; ++r)
            for (int c = 0; c < 3; ++c) T[r][c] = J[r][0] * W[0][c] + J[r][1] * W[1][c] + J[r][2] * W[2][c];
        double ST[2][3];                       /* Sigma T_r^T */
        for (int r = 0; r < 2; ++r)
            for (int c = 0; c < 3; ++c) ST[r][c] = Sg[c][0] * T[r][0] + Sg[c][1] * T[r][1] + Sg[c][2] * T[r][2];
        const double a = T[0][0] * ST[0][0] + T[0][1] * ST[0][1] + T[0][2] * ST[0][2] + (double)cam->lowpass;
        const double b = T[0][0] * ST[1][0] + T[0][1] * ST[1][1] + T[0][2] * ST[1][2];
        const double c = T[1][0] * ST[1][0] + T[1][1] * ST[1][1] + T[1][2] * ST[1][2] + (double)cam->lowpass;
        const double det = a * c - b * b, id2 = 1.0 / (det * det);

        /* conic (A, B, C) = (c, -b, a) / det  ->  a, b, c */
        const double ga = gA * (-c * c * id2) + gB * (b * c * id2) + gC * (-b * b * id2);
        const double gb = gA * (2.0 * b * c * id2) + gB * (-(a * c + b * b) * id2) + gC * (2.0 * a * b * id2);
        const double gc = gA * (-b * b * id2) + gB * (a * b * id2) + gC * (-a * a * id2);

        /* a = T0 Sigma T0^T + h, b = T0 Sigma T1^T, c = T1 Sigma T1^T + h  ->  Sigma (all nine entries), T */
        double gS[3][3], gT[2][3];
        for (int r = 0; r < 3; ++r)
            for (int k = 0; k < 3; ++k)
                gS[r][k] = ga * T[0][r] * T[0][k] + gb * T[0][r] * T[1][k] + gc * T[1][r] * T[1][k];
        for (int k = 0; k < 3; ++k) {
            gT[0][k] = 2.0 * ga * ST[0][k] + gb * ST[1][k];
            gT[1][k] = 2.0 * gc * ST[1][k] + gb * ST[0][k];
        }
        /* T = J W  ->  J */
        double gJ[2][3];
        for (int r = 0; r < 2; ++r)
            for (int k = 0; k < 3; ++k) gJ[r][k] = gT[r][0] * W[k][0] + gT[r][1] * W[k][1] + gT[r][2] * W[k][2];
        /* J and (u, v)  ->  p */
        double gp[3] = { 0.0, 0.0, 0.0 };
        const double iz = 1.0 / p[2], iz2 = iz * iz;
        gp[2] += gJ[0][0] * (-fx * iz2) + gJ[1][1] * (-fy * iz2);
        if (clx) gp[2] += gJ[0][2] * (fx * cxr * iz2);
        else { gp[0] += gJ[0][2] * (-fx * iz2); gp[2] += gJ[0][2] * (2.0 * fx * p[0] * iz2 * iz); }
        if (cly) gp[2] += gJ[1][2] * (fy * cyr * iz2);
        else { gp[1] += gJ[1][2] * (-fy * iz2); gp[2] += gJ[1][2] * (2.0 * fy * p[1] * iz2 * iz); }
        gp[0] += gu * fx * iz;  gp[2] += gu * (-fx * p[0] * iz2);
        gp[1] += gv * fy * iz;  gp[2] += gv * (-fy * p[1] * iz2);
        double gm[3];
        for (int k = 0; k < 3; ++k) gm[k] = W[0][k] * gp[0] + W[1][k] * gp[1] + W[2][k] * gp[2];

        /* Sigma = M M^T  ->  M  ->  s, R */
        double gM[3][3], gR[3][3];
        for (int r = 0; r < 3; ++r)
            for (int k = 0; k < 3; ++k)
                gM[r][k] = (gS[r][0] + gS[0][r]) * M[0][k] + (gS[r][1] + gS[1][r]) * M[1][k] + (gS[r][2] + gS[2][r]) * M[2][k];
        for (int k = 0; k < 3; ++k) {
            g_scale[(size_t)k * N + i] = gM[0][k] * R[0][k] + gM[1][k] * R[1][k] + gM[2][k] * R[2][k];
            for (int r = 0; r < 3; ++r) gR[r][k] = gM[r][k] * s[k];
        }
        /* R(w, x, y, z)  ->  unit quaternion  ->  stored quaternion */
        double gq[4];
        gq[0] = 2.0 * (-z * gR[0][1] + y * gR[0][2] + z * gR[1][0] - x * gR[1][2] - y * gR[2][0] + x * gR[2][1]);
        gq[1] = 2.0 * (y * gR[0][1] + z * gR[0][2] + y * gR[1][0] - 2.0 * x * gR[1][1] - w * gR[1][2]
                       + z * gR[2][0] + w * gR[2][1] - 2.0 * x * gR[2][2]);
        gq[2] = 2.0 * (-2.0 * y * gR[0][0] + x * gR[0][1] + w * gR[0][2] + x * gR[1][0] + z * gR[1][2]
                       - w * gR[2][0] + z * gR[2][1] - 2.0 * y * gR[2][2]);
        gq[3] = 2.0 * (-2.0 * z * gR[0][0] - w * gR[0][1] + x * gR[0][2] + w * gR[1][0] - 2.0 * z * gR[1][1]
                       + y * gR[1][2] + x * gR[2][0] + y * gR[2][1]);
        const double qh[4] = { w, x, y, z };
        const double dot = gq[0] * w + gq[1] * x + gq[2] * y + gq[3] * z;
        for (int k = 0; k < 4; ++k) g_rot[(size_t)k * N + i] = (gq[k] - qh[k] * dot) / qn;

        /* colour = max(0, 0.5 + sum_k Y_k(d) sh_k), d = (mean - camera centre) / |.| */
        double dv[3] = { m[0] - (double)cam->cam_pos[0], m[1] - (double)cam->cam_pos[1], m[2] - (double)cam->cam_pos[2] };
        const double len = sqrt(dv[0] * dv[0] + dv[1] * dv[1] + dv[2] * dv[2]);
        const double d[3] = { dv[0] / len, dv[1] / len, dv[2] / len };
        double Y[16], dY[16][3];
        lmk_ref_sh_basis(d, Y);
        sh_basis_grad(d, dY);
        double gd[3] = { 0.0, 0.0, 0.0 };
        for (int ch = 0; ch < 3; ++ch) {
            double acc = 0.5;
            for (uint32_t k = 0; k < ncoef; ++k) acc += Y[k] * (double)sh[((size_t)k * 3 + ch) * N + i];
            if (!(acc > 0.0)) continue;                      /* clamped at 0 */
            for (uint32_t k = 0; k < ncoef; ++k) {
                const double c_k = (double)sh[((size_t)k * 3 + ch) * N + i];
                g_sh[((size_t)k * 3 + ch) * N + i] = Y[k] * gcol[ch];
                for (int t = 0; t < 3; ++t) gd[t] += gcol[ch] * c_k * dY[k][t];
            }
        }
        const double dd = gd[0] * d[0] + gd[1] * d[1] + gd[2] * d[2];
        for (int k = 0; k < 3; ++k) gm[k] += (gd[k] - d[k] * dd) / len;
        for (int k = 0; k < 3; ++k) g_mean[(size_t)k * N + i] = gm[k];
    }
}
