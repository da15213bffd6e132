/*
 * lmk_gs.h -- C ABI of the MI355X (gfx950) tile-based Gaussian-splatting
 * forward rasteriser.
 *
 * The path is the rasteriser of the LandMarkSystem report: primitives defined
 * by Sec. 2.2 Eq. 7-8 (mean, rotation, scale, SH colour, opacity) are projected
 * to 2D Gaussians (EWA splatting, Sec. 2.2), duplicated into (tile | depth)
 * keys and depth-sorted per screen tile (Sec. 2.2; Sec. 4.2.1 names the stages),
 * then composited front to back per pixel (Sec. 2.2 Eq. 9-10).
 *
 * General rules
 *  - Every pointer inside the structs below is a DEVICE pointer owned by the
 *    caller.  The library allocates and frees nothing and keeps no state
 *    between calls apart from the last HIP error code.
 *  - All work is enqueued on the caller's HIP stream (`stream`, a hipStream_t
 *    passed as void*; NULL is the default stream).  No call synchronises except
 *    lmk_gs_read_status.  Buffers must stay valid until the stream has drained.
 *  - Arguments are validated on the host before the first HIP call; a
 *    validation failure enqueues nothing.
 *  - Return value: LMK_GS_OK or a negative LMK_GS_ERR_* code.
 *  - Geometry inputs are structure-of-arrays: an attribute with k components
 *    is k consecutive planes of n floats (component-major, plane stride n).
 *    The SH coefficients are one record per primitive (only primitives that
 *    survive culling need theirs, and a record is then two cache lines).
 */
#ifndef LMK_GS_H
#define LMK_GS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LMK_GS_OK 0
#define LMK_GS_ERR_INVALID (-1)     /* NULL pointer, bad size, unsupported tile, non-finite camera */
#define LMK_GS_ERR_CAPACITY (-2)    /* more (primitive, tile) pairs than `capacity`, or scratch too small */
#define LMK_GS_ERR_HIP (-3)         /* a HIP call failed; see lmk_gs_last_hip_error */
#define LMK_GS_ERR_UNSUPPORTED (-4)

#define LMK_GS_TILE 16u             /* pixels per tile edge; the only supported value */
#define LMK_GS_FEAT_STRIDE 12u      /* floats per primitive in lmk_gs_projected.feat */
/* floats per primitive in lmk_gs_gaussians.sh: 3 (deg+1)^2 rounded up to whole 16-byte vectors (4, 12, 28, 48) */
#define LMK_GS_SH_STRIDE(deg) ((3u * ((deg) + 1u) * ((deg) + 1u) + 3u) & ~3u)

/* The scene (Sec. 2.2 Eq. 7-8 and the text after Eq. 8). */
typedef struct lmk_gs_gaussians {
    const float *mean;     /* [3][n]  world-space centre mu                         */
    const float *scale;    /* [3][n]  diagonal of S, linear and > 0                 */
    const float *rot;      /* [4][n]  quaternion (w,x,y,z) of R, any non-zero norm  */
    const float *opacity;  /* [n]     alpha in [0,1]                                */
    const float *sh;       /* [n][LMK_GS_SH_STRIDE(sh_degree)] real SH colour coefficients, one 16-byte
                              aligned record per primitive: coefficient k of channel c at [3k + c],
                              the tail of the record unused                          */
    uint32_t n;            /* number of primitives (0 is allowed)                   */
    uint32_t sh_degree;    /* 0..3                                                  */
    const float *cov3d;    /* optional [6][n]: Sigma = R S S^T R^T of every primitive (xx, xy, xz,
                              yy, yz, zz) as written by lmk_gs_build_cov3d -- the view-independent
                              "inference parameter cache" of Sec. 5.2.2.  When not NULL,
                              lmk_gs_preprocess reads it instead of rot and scale (which may then
                              be NULL); the results are the same bit for bit             */
} lmk_gs_gaussians;

/* Pinhole camera.  Passed by value to the kernels (kernel arguments live in
 * scalar registers on CDNA, the counterpart of the constant-memory argument
 * passing listed in Sec. 4.2.1). */
typedef struct lmk_gs_camera {
    float view[12];        /* row-major 3x4 world->camera [R|t]; +x right, +y down, +z forward */
    float cam_pos[3];      /* camera centre in world space (for the SH view direction) */
    float fx, fy, cx, cy;  /* focal lengths and principal point in pixels; pixel (i,j) has centre (i+.5, j+.5) */
    uint32_t width, height;
    uint32_t tile;         /* must equal LMK_GS_TILE */
    float near_z;          /* primitives with camera z <= near_z are culled; must be > 0 */
    float lowpass;         /* added to the diagonal of the 2D covariance (px^2), >= 0 */
    float bg[3];           /* background colour composited behind everything */
    uint32_t binning;      /* which tiles of a primitive's support rectangle get a (key, value) pair:
                              0 = all of them;
                              1 = only tiles on whose pixel-centre square the splat can reach
                                  alpha >= 1/255 (the per-tile intersection test of Sec. 4.2.1):
                                  min over the square of d^T conic d, in closed form, against an
                                  upper bound of 2 ln(255 opacity) taken from the exponent and the
                                  top three mantissa bits of the opacity.  The image is the same
                                  under both rules; only pairs that can never contribute are dropped. */
} lmk_gs_camera;

/* Voxel index of a scene whose primitives were reordered offline into a voxel grid, for the
 * view-frustum filtering of voxels of Sec. 4.2.2 (frustum-based dynamic loading): per frame the
 * voxels, not the primitives, are tested against the view frustum, and primitives of voxels
 * that cannot reach the image are neither read nor projected.  Built by lmk_gs_index_build;
 * the pointers below are DEVICE copies of its outputs. */
#define LMK_GS_PRE_BLOCK 256u       /* primitives per group in lmk_gs_voxel_index.block_range */
typedef struct lmk_gs_voxel_index {
    const float *box;             /* [num_voxels][8] per voxel: bounding box of its primitives' means
                                     (lo x,y,z, hi x,y,z), largest scale component among them, 0;
                                     16-byte aligned                                               */
    const uint32_t *block_range;  /* [ceil(n / LMK_GS_PRE_BLOCK)][2] first and last voxel holding a
                                     primitive of each group of LMK_GS_PRE_BLOCK consecutive primitives */
    uint32_t num_voxels;
    const uint8_t *visible;       /* optional [num_voxels]: this frame's result of the box test for every voxel,
                                     already on the device (lmk_gs_anchor_decode_culled leaves it in
                                     anchor_visible, for the same camera); NULL = lmk_gs_preprocess_culled
                                     computes it                                                    */
} lmk_gs_voxel_index;

/* Per-primitive results of lmk_gs_preprocess.  For a primitive with
 * tiles_touched == 0 (culled) the other arrays hold unspecified values. */
typedef struct lmk_gs_projected {
    float *depth;             /* [n]     camera-space z                                       */
    uint32_t *tiles_touched;  /* [n]     tiles of the support rectangle that get a pair (see
                                         lmk_gs_camera.binning); 0 = culled                    */
    uint16_t *rect;           /* [n][4]  x0,y0,x1,y1 in tile units, half-open                  */
    float *feat;              /* [n][12] u, v, conic A, B, C, opacity, r, g, b, 0, 0, 0;
                                         16-byte aligned                                       */
    uint64_t *offsets;        /* [n+1]   exclusive prefix sum of tiles_touched; optional (may be
                                         NULL), written by lmk_gs_bin_sort when present        */
} lmk_gs_projected;

/* Results of lmk_gs_bin_sort. */
typedef struct lmk_gs_binned {
    uint64_t *keys;           /* [capacity] sorted keys: tile id << 32 | bits of depth          */
    uint32_t *vals;           /* [capacity] primitive index of each sorted key                  */
    uint64_t *keys_alt;       /* [capacity] ping-pong buffer, contents unspecified on return    */
    uint32_t *vals_alt;       /* [capacity] ping-pong buffer                                    */
    uint64_t capacity;        /* pairs each buffer can hold                                     */
    uint64_t *tile_offsets;   /* [tiles+1]  CSR: pairs of tile t are [tile_offsets[t], tile_offsets[t+1]) */
    uint32_t *tile_order;     /* [tiles]    optional (may be NULL): tile ids by descending list length,
                                            a scheduling hint that lmk_gs_render uses to start the
                                            longest lists first; ties in unspecified order        */
} lmk_gs_binned;

/* Bytes of device scratch the three calls need for n primitives, a
 * width x height image and `capacity` pairs.  The same scratch buffer
 * (256-byte aligned) must be passed to preprocess and bin_sort of one frame:
 * it carries the pair count, the per-group tile counts with their prefix sum and,
 * under binning rule 1, the masks of kept tiles from the one to the other.  Its
 * contents need no initialisation.  Its first 16 bytes are {uint64 pair count D,
 * int32 status, int32 pad}; D is final when lmk_gs_preprocess has completed. */
int32_t lmk_gs_workspace_bytes(uint32_t n, uint32_t width, uint32_t height,
                               uint64_t capacity, size_t *scratch_bytes);

/* Stage 1 (Sec. 2.2 Eq. 8 + EWA projection + SH colour; the per-primitive
 * kernel of Sec. 4.2.1).  For each primitive: camera-space position and
 * near-plane cull; Sigma = R S S^T R^T; Sigma' = J W Sigma W^T J^T + lowpass*I;
 * conic = Sigma'^-1 (culled unless det > 0); pixel centre; cull if opacity <
 * 1/255; support rectangle of the ellipse d^T conic d <= 11.09 in tiles,
 * clamped to the grid (empty = culled); rgb = max(0, 0.5 + SH(dir)).
 * Also accumulates per-block tile counts into scratch and clears the status
 * word.  Writes every array of `out` except `offsets`. */
int32_t lmk_gs_preprocess(const lmk_gs_gaussians *g, const lmk_gs_camera *cam,
                          const lmk_gs_projected *out,
                          void *scratch, size_t scratch_bytes, void *stream);

/* Fills the parameter cache lmk_gs_gaussians.cov3d (device array [6][n]) from g->rot and
 * g->scale with the arithmetic lmk_gs_preprocess uses (Sec. 2.2 Eq. 8), once per scene.
 * g->cov3d is ignored.  Asynchronous on `stream`. */
int32_t lmk_gs_build_cov3d(const lmk_gs_gaussians *g, float *cov3d, void *stream);

/* Offline step of Sec. 4.2.2, on the HOST (all pointers are host pointers, nothing touches the
 * GPU): assigns every primitive to the voxel floor(mean / voxel_size) (per axis, in fp32), orders
 * the occupied voxels along a Morton curve and the primitives of a voxel by their original index.
 *   perm[k]        original index of the primitive that comes k-th in the new order   [n]
 *   first[v]       new index of the first primitive of voxel v; first[num_voxels] = n [up to n + 1]
 *   box            as lmk_gs_voxel_index.box                                           [up to n][8]
 *   block_range    as lmk_gs_voxel_index.block_range         [ceil(n / LMK_GS_PRE_BLOCK)][2]
 * The caller permutes its scene arrays with perm, uploads them and the index arrays, and from
 * then on uses the new primitive indices everywhere.  scale may be linear scales of any sign
 * (absolute values are used).  LMK_GS_ERR_INVALID for NULL pointers, voxel_size <= 0 or
 * non-finite means; LMK_GS_ERR_UNSUPPORTED if the grid needs more than 2^21 cells along an axis. */
int32_t lmk_gs_index_build(const float *mean, const float *scale, uint32_t n, float voxel_size,
                           uint32_t *perm, uint32_t *first, float *box, uint32_t *block_range,
                           uint32_t *num_voxels);

/* lmk_gs_preprocess with the view-frustum filtering of voxels in front (Sec. 4.2.2): a group of
 * LMK_GS_PRE_BLOCK consecutive primitives is skipped -- tiles_touched = 0, nothing else read or
 * written -- when none of its voxels can reach the image.  A voxel is skipped only if, by a bound
 * on the support of its largest splat, every primitive in it is certain to be culled by the
 * near plane or to have an empty support rectangle, so every output is identical to
 * lmk_gs_preprocess on the same (reordered) scene.  `g` must be the scene in the order of the
 * index.  The 3x3 part of cam->view must be a rotation (LMK_GS_ERR_UNSUPPORTED otherwise).
 * block_visible: optional device array [ceil(n / LMK_GS_PRE_BLOCK)] receiving 1 for every group
 * that was processed, 0 for every group skipped (NULL: not reported). */
int32_t lmk_gs_preprocess_culled(const lmk_gs_gaussians *g, const lmk_gs_voxel_index *index,
                                 const lmk_gs_camera *cam, const lmk_gs_projected *out,
                                 uint8_t *block_visible,
                                 void *scratch, size_t scratch_bytes, void *stream);

/* Stage 2 (duplication into keys, depth sort at tile granularity, Sec. 2.2 and
 * Sec. 4.2.1).  One (key, value) pair per (primitive, tile that lmk_gs_camera.binning
 * keeps); on return all pairs are in keys/vals in ascending (tile, depth bits,
 * primitive index) order, which is unique, together with the per-tile ranges.
 * How: that order has no ties, so the order in which a tile's pairs arrive in the
 * tile's slice is free -- the pairs are counted per tile, the counts are scanned into
 * the ranges, every pair is written straight into its tile's slice, and each slice
 * is sorted on its own.  proj->offsets, when present, receives the exclusive prefix
 * sum of tiles_touched.  keys_alt/vals_alt are working space.
 * If the pair count D exceeds `capacity`, nothing is emitted: the status word
 * becomes LMK_GS_ERR_CAPACITY, every tile range is empty (lmk_gs_render then gives
 * the background), keys/vals are left as they were, and D (lmk_gs_read_status) tells
 * how much room a retry needs.  The call may be repeated for the same frame -- same
 * proj and scratch, no lmk_gs_preprocess in between, e.g. with larger buffers after an
 * overflow (the scratch must have been sized for the larger capacity): the status
 * word is that of the latest call. */
int32_t lmk_gs_bin_sort(const lmk_gs_projected *proj, uint32_t n, const lmk_gs_camera *cam,
                        const lmk_gs_binned *out,
                        void *scratch, size_t scratch_bytes, void *stream);

/* lmk_gs_bin_sort for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with
 * the scratch in a fixed array that is part of the library's code object (96 MiB on every GPU the
 * library runs on, held until the process ends).  The call allocates and frees nothing.  What
 * lmk_gs_preprocess would have left in a caller's scratch is recomputed from `proj` (tiles_touched,
 * rect, and under binning rule 1 the feature records), so `proj` may come from lmk_gs_preprocess on
 * any scratch buffer; keys, vals, tile_offsets and tile_order are the same as lmk_gs_bin_sort's,
 * bit for bit (proj->offsets, when present, too).
 * count_status: optional device array of two 64-bit words receiving {pair count D, status (0 or
 * LMK_GS_ERR_CAPACITY, sign-extended)} when the work completes -- this call has no scratch to hand
 * to lmk_gs_read_status.
 * Limits: n <= LMK_GS_STATIC_MAX_N, out->capacity <= LMK_GS_STATIC_MAX_CAPACITY, at most
 * LMK_GS_STATIC_MAX_TILES tiles; beyond them LMK_GS_ERR_CAPACITY is returned and nothing is
 * enqueued.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (different streams, or different host threads) race and give undefined results; calls on one
 * stream, or otherwise ordered, are safe, and nothing needs clearing between them. */
#define LMK_GS_STATIC_MAX_N (4u << 20)
#define LMK_GS_STATIC_MAX_CAPACITY (16ull << 20)
#define LMK_GS_STATIC_MAX_TILES 16384u
int32_t lmk_gs_bin_sort_static(const lmk_gs_projected *proj, uint32_t n, const lmk_gs_camera *cam,
                               const lmk_gs_binned *out, uint64_t *count_status, void *stream);

/* Stage 3 (Sec. 2.2 Eq. 9-10).  Each pixel walks its tile's list front to back:
 * alpha = min(0.99, o * exp(-q/2)), pairs with alpha < 1/255 are skipped, the
 * walk stops before the pair that would take T below 1e-4.
 * out_rgb is [3][height][width] (planar), out_transmittance [height][width]:
 * rgb = sum c_i alpha_i T_i + T_final * bg. */
int32_t lmk_gs_render(const lmk_gs_projected *proj, const lmk_gs_binned *binned,
                      const lmk_gs_camera *cam,
                      float *out_rgb, float *out_transmittance, void *stream);

/* Gradient of a scalar loss L through stage 3 (Sec. 2.2: the rasteriser is differentiable and
 * the parameters of the primitives are optimised through the rendering process).  Inputs:
 * the frame as lmk_gs_render read it (proj->feat, the sorted lists and tile ranges, the
 * camera), grad_rgb [3][height][width] = dL/d out_rgb and grad_transmittance [height][width]
 * = dL/d out_transmittance (NULL: zero), all device pointers.  Output: grad_feat
 * [n][LMK_GS_FEAT_STRIDE] (device, 16-byte aligned), laid out like the feature record:
 * dL/d{u, v, A, B, C, opacity, r, g, b}, then three zeros; it is overwritten (cleared by the
 * call, then accumulated with float atomics whose order is not fixed, so two runs agree to
 * fp32 rounding, not bit for bit).  The thresholds of the forward walk are constants of the
 * derivative: a skipped pair (alpha < 1/255), the pair that stopped a pixel's walk and every
 * pair behind it get nothing, and where alpha was clamped to 0.99 it depends on neither the
 * opacity nor the conic.  The chain from the feature record back to the 3D parameters is not
 * part of this call.  Errors as lmk_gs_render. */
int32_t lmk_gs_render_backward(const lmk_gs_projected *proj, uint32_t n, const lmk_gs_binned *binned,
                               const lmk_gs_camera *cam,
                               const float *grad_rgb, const float *grad_transmittance,
                               float *grad_feat, void *stream);

/* Where lmk_gs_preprocess_backward writes; device pointers, same layouts as lmk_gs_gaussians. */
typedef struct lmk_gs_gaussian_grads {
    float *mean;      /* [3][n] */
    float *scale;     /* [3][n] */
    float *rot;       /* [4][n] with respect to the quaternion as stored (any norm) */
    float *opacity;   /* [n]    */
    float *sh;        /* [n][LMK_GS_SH_STRIDE(sh_degree)], 16-byte aligned; padding entries get 0 */
} lmk_gs_gaussian_grads;

/* Gradient of a scalar loss through stage 1 (Sec. 2.2: every parameter of the primitives is
 * optimised through the rendering process): from grad_feat [n][LMK_GS_FEAT_STRIDE], the
 * output of lmk_gs_render_backward, to the gradient with respect to mean, scale, rotation,
 * opacity and SH coefficients of every primitive.  g: the scene as lmk_gs_preprocess read it
 * (scale and rot are required even when a covariance cache is present); proj->tiles_touched
 * from that call tells which primitives were binned.  Culls and clamps are constants of the
 * derivative: a primitive that was not binned gets zeros, a colour channel clamped at 0 passes
 * nothing on.  Every output element is written.  Asynchronous on `stream`; errors as
 * lmk_gs_preprocess. */
int32_t lmk_gs_preprocess_backward(const lmk_gs_gaussians *g, const lmk_gs_camera *cam,
                                   const lmk_gs_projected *proj, const float *grad_feat,
                                   const lmk_gs_gaussian_grads *out, void *stream);

/* ---- AnchorDecoder (Sec. 3.1: the Decoder component of the anchor-based Gaussian models; Sec. 4.2.1:
 * its steps -- the mask of the anchors to decode, the collation of an anchor's feature with the view
 * without the distance, three dual-layer perceptrons for covariance, colour and neural opacity, the
 * combination with the anchor's own tensors, post-processing -- fused here into one kernel).  The
 * report gives no formula for the steps; what each computes follows the anchor-based method that its
 * ScaffoldGSEncoding / OctreeGSEncoding implement. */
#define LMK_GS_ANCHOR_FEAT 32u      /* feature values per anchor = hidden width of the perceptrons */

/* The anchors of a scene; device pointers, read only. */
typedef struct lmk_gs_anchors {
    const float *position;  /* [3][a]     anchor centres                                              */
    const float *feature;   /* [a][LMK_GS_ANCHOR_FEAT]  one 128-byte record per anchor, 16-byte aligned */
    const float *extent;    /* [6][a]     linear, > 0: rows 0-2 scale the offsets, rows 3-5 bound the scales */
    const float *offsets;   /* [a][k][3]  offsets of the k primitives of an anchor, in units of extent 0-2, 8-byte aligned */
    uint32_t a;             /* number of anchors (0 is allowed)                                       */
    uint32_t k;             /* primitives per anchor: 10 or 4                                         */
} lmk_gs_anchors;

/* One perceptron y = W2 relu(W1 x + b1) + b2 with x = [feature, dir] (LMK_GS_ANCHOR_FEAT + 3 inputs),
 * hidden width LMK_GS_ANCHOR_FEAT; device pointers, read only. */
typedef struct lmk_gs_perceptron {
    const float *w1;    /* [LMK_GS_ANCHOR_FEAT][LMK_GS_ANCHOR_FEAT + 3]  (hidden unit, input)       */
    const float *b1;    /* [LMK_GS_ANCHOR_FEAT]                                                     */
    const float *w2t;   /* [LMK_GS_ANCHOR_FEAT][outputs]                 (hidden unit, output)      */
    const float *b2;    /* [outputs]                                                                */
} lmk_gs_perceptron;

/* outputs: opacity k (unit j = primitive j), colour 3k (units 3j..3j+2), cov 7k (units 7j..7j+2 the
 * scales, 7j+3..7j+6 the quaternion). */
typedef struct lmk_gs_anchor_decoder {
    lmk_gs_perceptron opacity, colour, cov;
} lmk_gs_anchor_decoder;

/* Where lmk_gs_anchor_decode writes: the arrays of an lmk_gs_gaussians of n = v * k primitives with
 * sh_degree 0, device pointers.  Slot v' * k + j holds primitive j of the anchor listed v'-th. */
typedef struct lmk_gs_decoded {
    float *mean;      /* [3][n] */
    float *scale;     /* [3][n] */
    float *rot;       /* [4][n] unnormalised quaternion (w, x, y, z) */
    float *opacity;   /* [n]    */
    float *sh;        /* [n][4] degree-0 coefficient per channel, then 0; 16-byte aligned */
} lmk_gs_decoded;

/* Decodes the anchors listed in `visible` (device array of v anchor indices computed beforehand, the
 * pre-computed mask indices of Sec. 4.2.1; NULL = anchors 0..v-1, then v <= a) as seen from cam_pos
 * (host pointer, 3 floats).  Per listed anchor: dir = (position - cam_pos) / |.| (0 if the two
 * coincide); the three perceptrons on [feature, dir]; per primitive j: opacity = tanh(y) if y > 0,
 * else exactly 0 (lmk_gs_preprocess culls such a primitive); colour = logistic(y), stored as the
 * degree-0 SH coefficient (colour - 0.5) / Y_00; scale = extent[3..5] * logistic(y);
 * rotation = the four quaternion units as they are; centre = position + offsets[j] * extent[0..2].
 * All in fp32.  A listed index >= a gives k primitives of opacity 0 (all other values 0).  Every
 * element of the n slots of `out` is written; `out` feeds lmk_gs_preprocess directly.
 * Asynchronous on `stream`.  LMK_GS_ERR_INVALID: NULL or misaligned pointer, v * k >= 2^32, visible
 * NULL with v > a; LMK_GS_ERR_UNSUPPORTED: k other than 10 or 4. */
int32_t lmk_gs_anchor_decode(const lmk_gs_anchors *anchors, const lmk_gs_anchor_decoder *decoder,
                             const float *cam_pos, const uint32_t *visible, uint32_t v,
                             const lmk_gs_decoded *out, void *stream);

/* Offline step of the anchors' view-frustum mask, on the HOST (host pointers, nothing touches the GPU;
 * layouts as in lmk_gs_anchors).  Per anchor: the box that holds every centre its primitives can take,
 * position -+ max_j |offsets[j]| * extent[0..2] per axis, and the largest scale they can take,
 * max(extent[3..5]); and, for the decoded scene of a * k slots, the anchors spanned by every group of
 * LMK_GS_PRE_BLOCK consecutive slots.
 *   box          [a][8]  lo x,y,z, hi x,y,z, scale bound, 0      (as lmk_gs_voxel_index.box)
 *   block_range  [ceil(a k / LMK_GS_PRE_BLOCK)][2]               (as lmk_gs_voxel_index.block_range)
 * Uploaded, {box, block_range, num_voxels = a} is the lmk_gs_voxel_index with which
 * lmk_gs_preprocess_culled skips the slots of anchors outside the view, and box is what
 * lmk_gs_anchor_decode_culled reads.  LMK_GS_ERR_INVALID: NULL pointer, k = 0, a k >= 2^32. */
int32_t lmk_gs_anchor_index_build(const float *position, const float *extent, const float *offsets,
                                  uint32_t a, uint32_t k, float *box, uint32_t *block_range);

/* lmk_gs_anchor_decode of all a anchors in their order (slot i k + j = primitive j of anchor i), with
 * the mask computation of Sec. 4.2.1 in front: an anchor is decoded only if its box (device array
 * [a][8] from lmk_gs_anchor_index_build, 16-byte aligned) passes the conservative box-against-frustum
 * test of Sec. 4.2.2 that lmk_gs_preprocess_culled applies to voxels -- a box that fails holds no
 * primitive that can be binned, so the image is unchanged.  anchor_visible (device, [a] bytes) receives
 * the mask.  The k slots of an anchor that fails get opacity 0; their other elements are zero or left
 * untouched (a tile of 32 consecutive anchors none of which passes is neither read nor decoded).
 * Errors as lmk_gs_anchor_decode and lmk_gs_preprocess (camera). */
int32_t lmk_gs_anchor_decode_culled(const lmk_gs_anchors *anchors, const lmk_gs_anchor_decoder *decoder,
                                    const lmk_gs_camera *cam, const float *box, uint8_t *anchor_visible,
                                    const lmk_gs_decoded *out, void *stream);

/* Copies {pair count D, status} of the frame from scratch to the host.
 * Synchronises `stream`.  Either output pointer may be NULL. */
int32_t lmk_gs_read_status(const void *scratch, uint64_t *dup_count, int32_t *status, void *stream);

/* Text for an LMK_GS_* code; never NULL. */
const char *lmk_gs_strerror(int32_t code);

/* The hipError_t value of the last failed HIP call in this process (0 if none). */
int32_t lmk_gs_last_hip_error(void);

/* Library version, major*10000 + minor*100 + patch. */
uint32_t lmk_gs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LMK_GS_H */
