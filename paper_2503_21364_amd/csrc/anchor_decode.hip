// AnchorDecoder (Sec. 3.1, Sec. 4.2.1): anchors + viewing position -> Gaussian primitives, one kernel.
//
// The steps the report times separately -- collating feature and view, three dual-layer
// perceptrons, combining their outputs with the anchor's tensors, post-processing -- run in one
// pass over the listed anchors with nothing written in between.  The perceptrons are dense
// products of the anchors' inputs with weights shared by all anchors, so they run on the matrix
// cores (fp32 in, fp32 accumulate).
//
// A tile of 32 listed anchors goes through a perceptron as two chained products, both written
// transposed so that the anchors stay on the 32 columns of v_mfma_f32_32x32x2_f32
// (column = lane % 32):
//     H^T (32 hidden x 32 anchors) = W1 (32 x 36) . X^T (36 x 32)      18 instructions
//     Y^T (32 outputs x 32 anchors) = W2 (32 x 32) . relu(H^T)         16 per tile of 32 outputs
// In this form the result registers of the first product are, as they are, the B operand of the
// second: lane (column j, half hi) holds rows 8g + 4hi + r (g, r < 4) of H^T, and a K step of
// the second product may pair any row of the lower half-lanes with any row of the upper ones as
// long as the weights are arranged to match -- step (g, r) takes row 8g + r from hi = 0 and row
// 8g + 4 + r from hi = 1.  Nothing is transposed or moved between the layers.  The same freedom
// orders the 36 inputs of the first product by how a lane loads them: the lower half-lane of an
// anchor holds features 0-17, the upper one features 18-31, the direction, and the constant 1
// whose weights are the first layer's biases.  The weights, arranged once per workgroup in LDS in
// the order the lanes consume them (one conflict-free 4-byte read per lane and instruction), are
// the A operands.  Each wavefront takes tiles in a strided loop, reading the next tile's inputs
// while it works on the current one; per tile 54 + 16 x (output tiles) matrix instructions
// (134 for k = 10).
//
// Outputs are structure-of-arrays over slots (listed anchor, primitive); the 32 anchors of a
// tile own 32 k consecutive slots of every plane.  A lane's results are scattered over those
// slots, so each wavefront stages its planes in LDS and writes them back as runs of consecutive
// floats.
#include "lmk_gs_internal.h"

namespace lmk {

namespace {

constexpr u32 kFeat = LMK_GS_ANCHOR_FEAT;
constexpr u32 kIn = kFeat + 3;
constexpr float kInvY00 = 3.5449077018110318f;      // 1 / (0.5 sqrt(1/pi))

__device__ __forceinline__ float logistic(float y) { return __builtin_amdgcn_rcpf(1.0f + __expf(-y)); }

// tanh for y > 0 from e = exp(-2y) in (0, 1): (1 - e) / (1 + e)
__device__ __forceinline__ float tanh_pos(float y)
{
    const float e = __expf(-2.0f * y);
    return (1.0f - e) * __builtin_amdgcn_rcpf(1.0f + e);
}

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr u32 kTile = 32;                 // anchors per matrix tile
constexpr u32 kMaxDecodeBlocks = 512;     // two workgroups of four wavefronts per compute unit
constexpr u32 kSteps1 = (kIn + 1) / 2;    // K steps of the first product (36 inputs, two per step)
constexpr u32 kSteps2 = kFeat / 2;        // K steps of the second product
constexpr int kPadInput = -1;

// which input a lane of half `hi` feeds to K step t of the first product
__host__ __device__ constexpr int input_of_step(u32 t, u32 hi)
{
    if (hi == 0) return (int)t;                       // features 0..17
    if (t < 12) return 20 + (int)t;                   // features 20..31
    if (t < 15) return (int)kFeat + (int)(t - 12);    // direction x, y, z
    if (t == 15) return kPadInput;                    // the constant 1 (bias)
    return 18 + (int)(t - 16);                        // features 18, 19
}
// which row of a 32-row result tile register v of a lane of half `hi` holds
__host__ __device__ constexpr u32 row_of_reg(u32 v, u32 hi) { return 8 * (v / 4) + 4 * hi + (v % 4); }

template <u32 K> struct DecodeLayout {
    static_assert(K % 2 == 0, "the two half-lanes of an anchor split its primitives");
    static constexpr u32 outs(u32 m) { return m == 0 ? K : (m == 1 ? 3 * K : 7 * K); }
    static constexpr u32 tiles(u32 m) { return (outs(m) + kTile - 1) / kTile; }
    static constexpr u32 tiles_before(u32 m) { return m == 0 ? 0 : tiles(m - 1) + tiles_before(m - 1); }
    static constexpr u32 kTiles = tiles_before(3);
    static constexpr u32 kFrag1 = 3 * kSteps1;                 // fragments (64 floats each) of the first layers
    static constexpr u32 kFrags = kFrag1 + kTiles * kSteps2;
    static constexpr u32 kBias2 = kFrags * kWave;              // float offset of the output biases in the staged weights
    static constexpr u32 kWeightFloats = kBias2 + kTiles * kTile;
    static constexpr u32 kPlane = kTile * K;                   // slots of a tile
    static constexpr u32 kStage = 8 * kPlane;                  // floats staged per wavefront (opacity, centres, SH records)
};

// PLANES staged planes of MAX floats each (s[c * MAX ..]) go to dst[c * plane_stride ..], `count`
// floats of each.  All LDS reads are issued before the first store, so their latency is paid once.
template <u32 MAX, u32 PLANES>
__device__ __forceinline__ void write_planes(float *__restrict__ dst, size_t plane_stride, const float *s,
                                             u32 count, u32 lane)
{
    static_assert(MAX % kWave == 0, "whole wavefront steps");
    float vals[PLANES][MAX / kWave];
#pragma unroll
    for (u32 c = 0; c < PLANES; ++c)
#pragma unroll
        for (u32 q = 0; q < MAX / kWave; ++q) vals[c][q] = s[c * MAX + q * kWave + lane];
#pragma unroll
    for (u32 c = 0; c < PLANES; ++c)
#pragma unroll
        for (u32 q = 0; q < MAX / kWave; ++q)
            if (q * kWave + lane < count) dst[c * plane_stride + q * kWave + lane] = vals[c][q];
}

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- the pieces of a tile's work, as functions of compile-time (perceptron M, output tile T)

// First layer of perceptron M: 18 accumulations from zero (the bias rides on the constant input), ReLU.
template <u32 K, u32 M>
__device__ __forceinline__ f32x16 first_layer(const float *s_w, const float (&xf)[kSteps1], u32 lane)
{
    f32x16 h = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (u32 t = 0; t < kSteps1; ++t)
        h = __builtin_amdgcn_mfma_f32_32x32x2f32(s_w[(M * kSteps1 + t) * kWave + lane], xf[t], h, 0, 0, 0);
    return h;
}

__device__ __forceinline__ void relu16(f32x16 &h)
{
#pragma unroll
    for (u32 r = 0; r < 16; ++r) h[r] = fmaxf(h[r], 0.0f);
}

// Output tile T of the second layer of perceptron M, without its bias.
template <u32 K, u32 M, u32 T>
__device__ __forceinline__ f32x16 second_layer(const float *s_w, const f32x16 &h, u32 lane)
{
    using L = DecodeLayout<K>;
    f32x16 y = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (u32 st = 0; st < kSteps2; ++st)
        y = __builtin_amdgcn_mfma_f32_32x32x2f32(
            s_w[(L::kFrag1 + (L::tiles_before(M) + T) * kSteps2 + st) * kWave + lane], h[st], y, 0, 0, 0);
    return y;
}

// Reads out output tile T of perceptron M: bias, activation, and the value into its slot of the
// wavefront's stage `s` (first half: opacity | centres x 3 | SH records; second half: the seven
// covariance planes and an eighth, never read).  No control flow: a register that holds no output
// (rows of a padded tile) writes to a slot that is overwritten later (opacity: the centres' planes;
// colour: the padding word of a record) or never read.
template <u32 K, u32 M, u32 T>
__device__ __forceinline__ void read_out(const f32x16 &y, float *s, const float *s_w, u32 j, u32 hi, u32 lane,
                                         bool live, float ex3, float ex4, float ex5)
{
    using L = DecodeLayout<K>;
    constexpr u32 outs = L::outs(M);
    float *s_sh = s + 4 * L::kPlane;
#pragma unroll
    for (u32 r = 0; r < 16; ++r) {
        if (kTile * T + row_of_reg(r, 0) >= outs) continue;              // neither half-lane holds an output here
        const u32 o = kTile * T + row_of_reg(r, 0) + 4 * hi;               // output unit of this register
        const float yr = y[r] + s_w[L::kBias2 + (L::tiles_before(M) + T) * kTile + row_of_reg(r, 0) + 4 * hi];
        const bool valid = o < outs;
        if (M == 0) {
            s[valid ? j * K + o : L::kPlane + lane] = (live && yr > 0.0f) ? tanh_pos(yr) : 0.0f;
        } else if (M == 1) {
            const u32 p = o / 3, c = o - 3 * p;
            s_sh[valid ? 4 * (j * K + p) + c : 4 * (j * K) + 3] = live ? (logistic(yr) - 0.5f) * kInvY00 : 0.0f;
        } else {
            const u32 p = o / 7, c = o - 7 * p;
            // a scale (c < 3) or a quaternion component; which, depends on the half-lane only
            const u32 o0 = kTile * T + row_of_reg(r, 0), o1 = o0 + 4;     // folded: the loop is unrolled
            const bool scale0 = o0 % 7 < 3, scale1 = o1 % 7 < 3;
            float val = yr;
            if (scale0 || scale1) {
                float bound = ex5;
                bound = c == 1 ? ex4 : bound;
                bound = c == 0 ? ex3 : bound;
                const float sc = bound * logistic(yr);
                // bitwise select: both arms are computed, no branch around the exponential
                const u32 pick = c < 3 ? ~0u : 0u;
                val = __uint_as_float((__float_as_uint(sc) & pick) | (__float_as_uint(yr) & ~pick));
            }
            s[valid ? c * L::kPlane + j * K + p : 7 * L::kPlane + lane] = live ? val : 0.0f;
        }
    }
}

template <u32 K>
__global__ __launch_bounds__(256, 2) void anchor_decode_kernel(
    const float *__restrict__ position, const float *__restrict__ feature, const float *__restrict__ extent,
    const float *__restrict__ offsets, u32 a, const u32 *__restrict__ visible, u32 v,
    const unsigned char *__restrict__ anchor_visible,
    const float *__restrict__ op_w1, const float *__restrict__ op_b1, const float *__restrict__ op_w2t,
    const float *__restrict__ op_b2,
    const float *__restrict__ col_w1, const float *__restrict__ col_b1, const float *__restrict__ col_w2t,
    const float *__restrict__ col_b2,
    const float *__restrict__ cov_w1, const float *__restrict__ cov_b1, const float *__restrict__ cov_w2t,
    const float *__restrict__ cov_b2,
    float cam_x, float cam_y, float cam_z,
    float *__restrict__ mean, float *__restrict__ scale, float *__restrict__ rot,
    float *__restrict__ opacity, float *__restrict__ sh)
{
    using L = DecodeLayout<K>;
    constexpr u32 kWaves = 256 / kWave;
    __shared__ float s_w[L::kWeightFloats];
    __shared__ __align__(16) float s_stage[kWaves][L::kStage];
    const u32 lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const u32 j = lane & (kTile - 1), hi = lane / kTile;

    // ---- the weights, in consumption order
    const float *w1s[3] = {op_w1, col_w1, cov_w1}, *b1s[3] = {op_b1, col_b1, cov_b1};
    const float *w2s[3] = {op_w2t, col_w2t, cov_w2t}, *b2s[3] = {op_b2, col_b2, cov_b2};
#pragma unroll
    for (u32 m = 0; m < 3; ++m) {
        for (u32 t = wv; t < kSteps1; t += kWaves) {
            const int in = hi == 0 ? input_of_step(t, 0) : input_of_step(t, 1);
            // the 36th input is the constant 1 and its weight the bias of the hidden unit
            s_w[(m * kSteps1 + t) * kWave + lane] = in == kPadInput ? b1s[m][j] : w1s[m][j * kIn + (u32)in];
        }
        const u32 outs = L::outs(m);
        for (u32 f = wv; f < L::tiles(m) * kSteps2; f += kWaves) {
            const u32 T = f / kSteps2, st = f % kSteps2;
            const u32 o = kTile * T + j, k = row_of_reg(st, hi);
            s_w[(L::kFrag1 + L::tiles_before(m) * kSteps2 + f) * kWave + lane] = o < outs ? w2s[m][k * outs + o] : 0.0f;
        }
        for (u32 r = threadIdx.x; r < L::tiles(m) * kTile; r += 256)
            s_w[L::kBias2 + L::tiles_before(m) * kTile + r] = r < outs ? b2s[m][r] : 0.0f;
    }
    __syncthreads();

    float *s = s_stage[wv];
    const size_t A = a, n = (size_t)v * K;
    const u32 num_tiles = (v + kTile - 1) / kTile;
    const u32 stride = gridDim.x * kWaves;

    // What a half-lane reads of its anchor: 18 inputs (the upper half's direction is computed from
    // the centre when the tile is processed), centre, extents, its half of the offsets.
    struct TileIn {
        float4 q0, q1, q2, q3;
        float p2x, p2y;
        float pos[3], ex[6], off[3 * K / 2];
        bool live;
    };
    auto list_entry = [&](u32 tile) -> u32 {            // anchor index of this lane in `tile`; ~0u if none
        const u32 item = tile * kTile + j;
        if (tile >= num_tiles || item >= v) return ~0u;
        return visible ? visible[item] : item;
    };
    // Only issues loads: nothing here waits for them (but for the mask bit, requested a tile earlier).
    // A lane without an anchor reads anchor 0 (its results are replaced by zeros when they are
    // staged), so the loads of a tile are unconditional.
    auto mask_entry = [&](u32 idx_or_none) -> u32 {      // the anchor's bit of the frustum mask (1 without a mask)
        return (anchor_visible && idx_or_none < a) ? (u32)anchor_visible[idx_or_none] : 1u;
    };
    auto load_tile = [&](u32 idx_or_none, u32 mask_bit) -> TileIn {
        TileIn in;
        in.live = idx_or_none < a && mask_bit != 0u;
        const u32 idx = in.live ? idx_or_none : 0u;
        // a tile none of whose anchors is decoded reads nothing
        if (a > 0 && __builtin_amdgcn_ballot_w64(in.live) != 0ull) {          // uniform
            const float *rec = feature + (size_t)idx * kFeat;
            const float4 *r4 = reinterpret_cast<const float4 *>(rec + (hi ? 20 : 0));
            in.q0 = r4[0]; in.q1 = r4[1]; in.q2 = r4[2];
            in.q3 = reinterpret_cast<const float4 *>(rec)[3];      // the upper half overwrites it with the direction
            in.p2x = rec[16 + 2 * hi]; in.p2y = rec[17 + 2 * hi];
            in.pos[0] = position[idx]; in.pos[1] = position[A + idx]; in.pos[2] = position[2 * A + idx];
#pragma unroll
            for (u32 m = 0; m < 6; ++m) in.ex[m] = extent[m * A + idx];
            const float *orec = offsets + (size_t)idx * (3 * K) + hi * (3 * K / 2);
#pragma unroll
            for (u32 q = 0; q < 3 * K / 2; ++q) in.off[q] = orec[q];
        } else {
            in.q0 = in.q1 = in.q2 = in.q3 = float4{0.f, 0.f, 0.f, 0.f};
            in.p2x = in.p2y = 0.0f;
#pragma unroll
            for (u32 m = 0; m < 3; ++m) in.pos[m] = 0.0f;
#pragma unroll
            for (u32 m = 0; m < 6; ++m) in.ex[m] = 0.0f;
#pragma unroll
            for (u32 q = 0; q < 3 * K / 2; ++q) in.off[q] = 0.0f;
        }
        return in;
    };

    // Every wavefront takes tiles in a strided loop (no workgroup barrier inside: trip counts
    // differ).  The loads run two tiles ahead for the list entry and the mask bit and one tile
    // ahead for the anchor's data, so a tile's arithmetic covers the next tile's memory latency.
    const u32 first = blockIdx.x * kWaves + wv;
    const u32 first_idx = list_entry(first);
    TileIn next_in = load_tile(first_idx, mask_entry(first_idx));
    u32 next_idx = list_entry(first + stride);
    u32 next_bit = mask_entry(next_idx);
    for (u32 tile = first; tile < num_tiles; tile += stride) {
        const TileIn in = next_in;
        next_in = load_tile(next_idx, next_bit);
        next_idx = list_entry(tile + 2 * stride);
        next_bit = mask_entry(next_idx);

        const u32 tile_items = v - tile * kTile < kTile ? v - tile * kTile : kTile;
        const u32 count = tile_items * K;
        const size_t slot0 = (size_t)tile * L::kPlane;
        const bool live = in.live;
        if (anchor_visible && __builtin_amdgcn_ballot_w64(live) == 0ull) {
            // nothing of this tile is in view: its slots get opacity 0 and nothing else
            for (u32 t = lane; t < count; t += kWave) opacity[slot0 + t] = 0.0f;
            continue;
        }
        float xf[kSteps1];
        float pos[3], ex[6], off[3 * K / 2];
#pragma unroll
        for (u32 m = 0; m < 3; ++m) pos[m] = in.pos[m];
#pragma unroll
        for (u32 m = 0; m < 6; ++m) ex[m] = in.ex[m];
#pragma unroll
        for (u32 q = 0; q < 3 * K / 2; ++q) off[q] = in.off[q];
        {
            float4 q3 = in.q3;
            if (hi != 0) {
                const float dx = pos[0] - cam_x, dy = pos[1] - cam_y, dz = pos[2] - cam_z;
                const float d2 = dx * dx + dy * dy + dz * dz;
                const float inv = d2 > 0.0f ? __builtin_amdgcn_rsqf(d2) : 0.0f;
                q3 = float4{dx * inv, dy * inv, dz * inv, 1.0f};        // .w: the constant input that carries the bias
            }
            xf[0] = in.q0.x; xf[1] = in.q0.y; xf[2] = in.q0.z; xf[3] = in.q0.w;
            xf[4] = in.q1.x; xf[5] = in.q1.y; xf[6] = in.q1.z; xf[7] = in.q1.w;
            xf[8] = in.q2.x; xf[9] = in.q2.y; xf[10] = in.q2.z; xf[11] = in.q2.w;
            xf[12] = q3.x; xf[13] = q3.y; xf[14] = q3.z; xf[15] = q3.w;
            xf[16] = in.p2x; xf[17] = in.p2y;
        }

        // The tile's products in order; the read-out of an output tile follows the issue of the next product.
        float *s_op = s, *s_mean = s + L::kPlane, *s_sh = s + 4 * L::kPlane;
        f32x16 h = first_layer<K, 0>(s_w, xf, lane);
        relu16(h);
        const f32x16 y_op = second_layer<K, 0, 0>(s_w, h, lane);
        h = first_layer<K, 1>(s_w, xf, lane);
        read_out<K, 0, 0>(y_op, s, s_w, j, hi, lane, live, ex[3], ex[4], ex[5]);
        relu16(h);
        const f32x16 y_col = second_layer<K, 1, 0>(s_w, h, lane);
        h = first_layer<K, 2>(s_w, xf, lane);
        read_out<K, 1, 0>(y_col, s, s_w, j, hi, lane, live, ex[3], ex[4], ex[5]);
        relu16(h);
        const f32x16 y_cov0 = second_layer<K, 2, 0>(s_w, h, lane);

        // the first half leaves the stage: opacity, centres, SH records
#pragma unroll
        for (u32 pp = 0; pp < K / 2; ++pp) {
            const u32 p = hi * (K / 2) + pp;
#pragma unroll
            for (u32 c = 0; c < 3; ++c)
                s_mean[c * L::kPlane + j * K + p] = live ? fmaf(off[3 * pp + c], ex[c], pos[c]) : 0.0f;
        }
#pragma unroll
        for (u32 q = 0; q < L::kPlane / kWave; ++q) s_sh[4 * (q * kWave + lane) + 3] = 0.0f;
        wave_sync();
        write_planes<L::kPlane, 1>(opacity + slot0, 0, s_op, count, lane);
        write_planes<L::kPlane, 3>(mean + slot0, n, s_mean, count, lane);
        {
            const float4 *s4 = reinterpret_cast<const float4 *>(s_sh);
            float4 *dst = reinterpret_cast<float4 *>(sh) + slot0;
            float4 recs[L::kPlane / kWave];
#pragma unroll
            for (u32 q = 0; q < L::kPlane / kWave; ++q) recs[q] = s4[q * kWave + lane];
#pragma unroll
            for (u32 q = 0; q < L::kPlane / kWave; ++q)
                if (q * kWave + lane < count) dst[q * kWave + lane] = recs[q];
        }
        wave_sync();

        // second half: the seven covariance planes
        if constexpr (L::tiles(2) == 3) {
            const f32x16 y_cov1 = second_layer<K, 2, 1>(s_w, h, lane);
            read_out<K, 2, 0>(y_cov0, s, s_w, j, hi, lane, live, ex[3], ex[4], ex[5]);
            const f32x16 y_cov2 = second_layer<K, 2, 2>(s_w, h, lane);
            read_out<K, 2, 1>(y_cov1, s, s_w, j, hi, lane, live, ex[3], ex[4], ex[5]);
            read_out<K, 2, 2>(y_cov2, s, s_w, j, hi, lane, live, ex[3], ex[4], ex[5]);
        } else {
            static_assert(L::tiles(2) == 1 || L::tiles(2) == 3, "7 k outputs in one or three tiles");
            read_out<K, 2, 0>(y_cov0, s, s_w, j, hi, lane, live, ex[3], ex[4], ex[5]);
        }
        wave_sync();
        write_planes<L::kPlane, 3>(scale + slot0, n, s, count, lane);
        write_planes<L::kPlane, 4>(rot + slot0, n, s + 3 * L::kPlane, count, lane);
        wave_sync();
    }
}

template <u32 K>
hipError_t launch_k(const lmk_gs_anchors &an, const lmk_gs_anchor_decoder &d, const float *cam,
                    const u32 *visible, u32 v, const uint8_t *anchor_visible, const lmk_gs_decoded &out,
                    hipStream_t stream)
{
    const u32 num_tiles = (v + kTile - 1) / kTile;
    const u32 want = (num_tiles + 3) / 4;
    const u32 blocks = want < kMaxDecodeBlocks ? want : kMaxDecodeBlocks;
    hipLaunchKernelGGL(anchor_decode_kernel<K>, dim3(blocks), dim3(256), 0, stream,
                       an.position, an.feature, an.extent, an.offsets, an.a, visible, v, anchor_visible,
                       d.opacity.w1, d.opacity.b1, d.opacity.w2t, d.opacity.b2,
                       d.colour.w1, d.colour.b1, d.colour.w2t, d.colour.b2,
                       d.cov.w1, d.cov.b1, d.cov.w2t, d.cov.b2,
                       cam[0], cam[1], cam[2], out.mean, out.scale, out.rot, out.opacity, out.sh);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_anchor_decode(const lmk_gs_anchors &anchors, const lmk_gs_anchor_decoder &decoder,
                                const float *cam_pos, const u32 *visible, u32 v, const uint8_t *anchor_visible,
                                const lmk_gs_decoded &out, hipStream_t stream)
{
    if (v == 0) return hipSuccess;
    if (anchors.k == 10) return launch_k<10>(anchors, decoder, cam_pos, visible, v, anchor_visible, out, stream);
    return launch_k<4>(anchors, decoder, cam_pos, visible, v, anchor_visible, out, stream);
}

}  // namespace lmk
