// AnchorDecoder (Sec. 3.1, Sec. 4.2.1): anchors + viewing position -> Gaussian primitives, one kernel.
//
// The steps the report times separately -- collating feature and view, three dual-layer
// perceptrons, combining their outputs with the anchor's tensors, post-processing -- run in one
// pass over the listed anchors with nothing written in between: an anchor's 35 inputs, one
// perceptron's outputs and one hidden unit at a time live in registers.
//
// One lane per anchor.  The weights are the same for every lane, so each weight is a scalar
// operand of the multiply-add that uses it: the loops below index the weight arrays with
// wave-uniform indices only, which lets the compiler fetch them with scalar loads (whole rows at
// a time) and spend vector instructions on arithmetic alone -- 35 + outputs multiply-adds per
// hidden unit, 6 880 per anchor for k = 10.
//
// Outputs are structure-of-arrays over slots (listed anchor, primitive); the 64 anchors of a
// wavefront own 64 k consecutive slots of every plane.  A lane's k values of a plane are k
// consecutive floats, so stores straight from registers would be 64 scattered 4-byte writes per
// instruction; instead each wavefront stages up to four planes in LDS and writes them back as
// runs of consecutive floats.
#include "lmk_gs_internal.h"

namespace lmk {

namespace {

constexpr u32 kFeat = LMK_GS_ANCHOR_FEAT;
constexpr u32 kIn = kFeat + 3;
constexpr u32 kDecBlock = 64;           // one wavefront per workgroup: nothing is shared between wavefronts
constexpr float kInvY00 = 3.5449077018110318f;      // 1 / (0.5 sqrt(1/pi))

// y = W2 relu(W1 x + b1) + b2.  w1 [kFeat][kIn], w2t [kFeat][OUTS]; every index is wave-uniform.
template <u32 OUTS>
__device__ __forceinline__ void perceptron(const float (&x)[kIn], const float *__restrict__ w1,
                                           const float *__restrict__ b1, const float *__restrict__ w2t,
                                           const float *__restrict__ b2, float (&y)[OUTS])
{
#pragma unroll
    for (u32 u = 0; u < OUTS; ++u) y[u] = b2[u];
#pragma unroll 1
    for (u32 h = 0; h < kFeat; ++h) {
        const float *row1 = w1 + h * kIn;
        float acc = b1[h];
#pragma unroll
        for (u32 i = 0; i < kIn; ++i) acc = fmaf(row1[i], x[i], acc);
        acc = fmaxf(acc, 0.0f);
        const float *row2 = w2t + h * OUTS;
#pragma unroll
        for (u32 u = 0; u < OUTS; ++u) y[u] = fmaf(row2[u], acc, y[u]);
    }
}

__device__ __forceinline__ float logistic(float y) { return __builtin_amdgcn_rcpf(1.0f + __expf(-y)); }

// tanh for y > 0 from e = exp(-2y) in (0, 1): (1 - e) / (1 + e)
__device__ __forceinline__ float tanh_pos(float y)
{
    const float e = __expf(-2.0f * y);
    return (1.0f - e) * __builtin_amdgcn_rcpf(1.0f + e);
}

// The wavefront's `count` floats staged at s[0..count) go to dst[0..count).
__device__ __forceinline__ void write_run(float *__restrict__ dst, const float *s, u32 count, u32 lane)
{
    for (u32 t = lane; t < count; t += kWave) dst[t] = s[t];
}

template <u32 K>
__global__ __launch_bounds__(kDecBlock) void anchor_decode_kernel(
    const float *__restrict__ position, const float *__restrict__ feature, const float *__restrict__ extent,
    const float *__restrict__ offsets, u32 a, const u32 *__restrict__ visible, u32 v,
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
    constexpr u32 kRun = kWave * K;                         // slots of a wavefront
    __shared__ __align__(16) float s_stage[kDecBlock / kWave][4 * kRun];
    const u32 lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    float *s = s_stage[wv];
    const u32 item = blockIdx.x * kDecBlock + threadIdx.x;  // position in the list
    const u32 wave_first = item - lane;
    const u32 wave_items = wave_first < v ? (v - wave_first < kWave ? v - wave_first : kWave) : 0u;
    const u32 count = wave_items * K;                       // slots this wavefront writes
    const size_t slot0 = (size_t)wave_first * K;
    const size_t n = (size_t)v * K;

    // the anchor of this lane; an index beyond the scene decodes to nothing
    u32 idx = 0;
    bool live = false;
    if (item < v) {
        idx = visible ? visible[item] : item;
        live = idx < a;
        if (!live) idx = 0;
    }
    const size_t A = a;

    float x[kIn];
    float px = 0.f, py = 0.f, pz = 0.f;
    if (live) {
        const float4 *rec = reinterpret_cast<const float4 *>(feature) + (size_t)idx * (kFeat / 4);
#pragma unroll
        for (u32 q = 0; q < kFeat / 4; ++q) {
            const float4 f = rec[q];
            x[4 * q] = f.x; x[4 * q + 1] = f.y; x[4 * q + 2] = f.z; x[4 * q + 3] = f.w;
        }
        px = position[idx]; py = position[A + idx]; pz = position[2 * A + idx];
        const float dx = px - cam_x, dy = py - cam_y, dz = pz - cam_z;
        const float d2 = dx * dx + dy * dy + dz * dz;
        const float inv = d2 > 0.0f ? 1.0f / sqrtf(d2) : 0.0f;
        x[kFeat] = dx * inv; x[kFeat + 1] = dy * inv; x[kFeat + 2] = dz * inv;
    } else {
#pragma unroll
        for (u32 i = 0; i < kIn; ++i) x[i] = 0.0f;
    }

    // neural opacity: kept where the raw output is positive
    {
        float y[K];
        perceptron<K>(x, op_w1, op_b1, op_w2t, op_b2, y);
#pragma unroll
        for (u32 j = 0; j < K; ++j) s[lane * K + j] = (live && y[j] > 0.0f) ? tanh_pos(y[j]) : 0.0f;
    }
    __syncthreads();
    write_run(opacity + slot0, s, count, lane);
    __syncthreads();

    // colour, as the degree-0 SH coefficient of a 16-byte record
    {
        float y[3 * K];
        perceptron<3 * K>(x, col_w1, col_b1, col_w2t, col_b2, y);
        float4 *s4 = reinterpret_cast<float4 *>(s);
#pragma unroll
        for (u32 j = 0; j < K; ++j) {
            float4 r = {0.f, 0.f, 0.f, 0.f};
            if (live) {
                r.x = (logistic(y[3 * j]) - 0.5f) * kInvY00;
                r.y = (logistic(y[3 * j + 1]) - 0.5f) * kInvY00;
                r.z = (logistic(y[3 * j + 2]) - 0.5f) * kInvY00;
            }
            s4[lane * K + j] = r;
        }
    }
    __syncthreads();
    {
        const float4 *s4 = reinterpret_cast<const float4 *>(s);
        float4 *dst = reinterpret_cast<float4 *>(sh) + slot0;
        for (u32 t = lane; t < count; t += kWave) dst[t] = s4[t];
    }
    __syncthreads();

    // covariance: three scales bounded by the anchor's extent, four quaternion components
    float ex[6];
#pragma unroll
    for (u32 m = 0; m < 6; ++m) ex[m] = live ? extent[m * A + idx] : 0.0f;
    {
        float y[7 * K];
        perceptron<7 * K>(x, cov_w1, cov_b1, cov_w2t, cov_b2, y);
        // planes scale 0-2 and rot 0
#pragma unroll
        for (u32 j = 0; j < K; ++j) {
#pragma unroll
            for (u32 m = 0; m < 3; ++m) s[m * kRun + lane * K + j] = live ? ex[3 + m] * logistic(y[7 * j + m]) : 0.0f;
            s[3 * kRun + lane * K + j] = live ? y[7 * j + 3] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (u32 m = 0; m < 3; ++m) write_run(scale + m * n + slot0, s + m * kRun, count, lane);
        write_run(rot + slot0, s + 3 * kRun, count, lane);
        __syncthreads();
        // planes rot 1-3
#pragma unroll
        for (u32 j = 0; j < K; ++j)
#pragma unroll
            for (u32 m = 0; m < 3; ++m) s[m * kRun + lane * K + j] = live ? y[7 * j + 4 + m] : 0.0f;
    }
    // centres: anchor + offset * reach, into the fourth staged plane onwards
    float off[3 * K];
    if (live) {
        const float2 *rec = reinterpret_cast<const float2 *>(offsets + (size_t)idx * (3 * K));
#pragma unroll
        for (u32 q = 0; q < 3 * K / 2; ++q) {
            const float2 f = rec[q];
            off[2 * q] = f.x; off[2 * q + 1] = f.y;
        }
        if constexpr ((3 * K) % 2 == 1) off[3 * K - 1] = offsets[(size_t)idx * (3 * K) + 3 * K - 1];
    } else {
#pragma unroll
        for (u32 q = 0; q < 3 * K; ++q) off[q] = 0.0f;
    }
#pragma unroll
    for (u32 j = 0; j < K; ++j) s[3 * kRun + lane * K + j] = fmaf(off[3 * j], ex[0], px);
    __syncthreads();
#pragma unroll
    for (u32 m = 0; m < 3; ++m) write_run(rot + (1 + m) * n + slot0, s + m * kRun, count, lane);
    write_run(mean + slot0, s + 3 * kRun, count, lane);
    __syncthreads();
#pragma unroll
    for (u32 j = 0; j < K; ++j) {
        s[lane * K + j] = fmaf(off[3 * j + 1], ex[1], py);
        s[kRun + lane * K + j] = fmaf(off[3 * j + 2], ex[2], pz);
    }
    __syncthreads();
    write_run(mean + n + slot0, s, count, lane);
    write_run(mean + 2 * n + slot0, s + kRun, count, lane);
}

template <u32 K>
hipError_t launch_k(const lmk_gs_anchors &an, const lmk_gs_anchor_decoder &d, const float *cam,
                    const u32 *visible, u32 v, const lmk_gs_decoded &out, hipStream_t stream)
{
    const u32 blocks = (v + kDecBlock - 1) / kDecBlock;
    hipLaunchKernelGGL(anchor_decode_kernel<K>, dim3(blocks), dim3(kDecBlock), 0, stream,
                       an.position, an.feature, an.extent, an.offsets, an.a, visible, v,
                       d.opacity.w1, d.opacity.b1, d.opacity.w2t, d.opacity.b2,
                       d.colour.w1, d.colour.b1, d.colour.w2t, d.colour.b2,
                       d.cov.w1, d.cov.b1, d.cov.w2t, d.cov.b2,
                       cam[0], cam[1], cam[2], out.mean, out.scale, out.rot, out.opacity, out.sh);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_anchor_decode(const lmk_gs_anchors &anchors, const lmk_gs_anchor_decoder &decoder,
                                const float *cam_pos, const u32 *visible, u32 v,
                                const lmk_gs_decoded &out, hipStream_t stream)
{
    if (v == 0) return hipSuccess;
    if (anchors.k == 10) return launch_k<10>(anchors, decoder, cam_pos, visible, v, out, stream);
    return launch_k<4>(anchors, decoder, cam_pos, visible, v, out, stream);
}

}  // namespace lmk
