// Stage 1: per-primitive projection, culling, support rectangle and SH colour
// (Sec. 2.2 Eq. 8, the EWA projection and SH colour of Sec. 2.2; the
// per-primitive kernel named in Sec. 4.2.1).
//
// This translation unit is compiled with -ffp-contract=off and correctly
// rounded fp32 divide/sqrt: everything that decides an integer (depth bits,
// rectangle, culls) is evaluated one IEEE fp32 operation at a time in the
// written order, so those outputs are unique.
//
// HBM-bound: one thread per primitive, every load/store is a plane access
// that is contiguous across the wavefront.  The SH planes (192 of the 240
// bytes a visible primitive needs) are read only by lanes that survive the
// culls.
#include "lmk_gs_internal.h"
#include "tile_test.h"

#include <cmath>

namespace lmk {

struct ShConsts { float k0, k1, k2, k20, k33, k32, k31, k30, k32b; };

static ShConsts make_sh_consts()
{
    const double pi = 3.14159265358979323846;
    ShConsts k;
    k.k0 = (float)(0.5 * std::sqrt(1.0 / pi));
    k.k1 = (float)std::sqrt(3.0 / (4.0 * pi));
    k.k2 = (float)(0.5 * std::sqrt(15.0 / pi));
    k.k20 = (float)(0.25 * std::sqrt(5.0 / pi));
    k.k33 = (float)(0.25 * std::sqrt(35.0 / (2.0 * pi)));
    k.k32 = (float)(0.5 * std::sqrt(105.0 / pi));
    k.k31 = (float)(0.25 * std::sqrt(21.0 / (2.0 * pi)));
    k.k30 = (float)(0.25 * std::sqrt(7.0 / pi));
    k.k32b = (float)(0.25 * std::sqrt(105.0 / pi));
    return k;
}

__device__ __forceinline__ float clamp_nan_lo(float v, float lo, float hi)
{
    return !(v > lo) ? lo : (v > hi ? hi : v);
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------- voxel filter (Sec. 4.2.2)
// Can any primitive of a voxel (bounding box of the means, largest scale component smax) be
// binned?  Not if the whole box is behind the near plane, or beyond one image edge by more
// than the largest support a primitive of the voxel can have there: for a primitive at
// camera-space (x, y, z), z > 0, the half-width of its support is at most fx R / z + r0 pixels,
// R = sqrt(11.09) sqrt(1 + lim_x^2) smax (row norm of the clamped EWA Jacobian times the largest
// eigenvalue of Sigma), r0 = sqrt(11.09 lowpass); "off the left edge" then reads
// fx x + (cx + r0) z < -fx R, linear in the position, so the box corners decide.  Evaluated in
// fp32 without contraction like every step that decides an integer; the slack terms make
// rounding keep a voxel rather than drop it.
__device__ __forceinline__ bool voxel_visible(const ProjParams &pp, const float4 b0, const float4 b1)
{
    const float *V = pp.cam.view;
    const float lo[3] = { b0.x, b0.y, b0.z }, hi[3] = { b0.w, b1.x, b1.y };
    const float smax = b1.z;
    const float XW = (float)(pp.tiles_x * LMK_GS_TILE), YH = (float)(pp.tiles_y * LMK_GS_TILE);
    const float st = sqrtf(11.09f);
    const float Rx = (st * sqrtf(1.0f + pp.lim_x * pp.lim_x)) * smax;
    const float Ry = (st * sqrtf(1.0f + pp.lim_y * pp.lim_y)) * smax;
    const float r0 = sqrtf(11.09f * pp.cam.lowpass);
    const float cl = pp.cam.cx + r0, cr = (pp.cam.cx - r0) - XW;
    const float ct = pp.cam.cy + r0, cb = (pp.cam.cy - r0) - YH;
    const float cm = (XW + YH) + (fabsf(pp.cam.cx) + fabsf(pp.cam.cy));
    float zmax = 0.f, maxL = 0.f, minR = 0.f, maxT = 0.f, minB = 0.f, mag = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float wx = (k & 1) ? hi[0] : lo[0], wy = (k & 2) ? hi[1] : lo[1], wz = (k & 4) ? hi[2] : lo[2];
        const float x = V[0] * wx + V[1] * wy + V[2] * wz + V[3];
        const float y = V[4] * wx + V[5] * wy + V[6] * wz + V[7];
        const float z = V[8] * wx + V[9] * wy + V[10] * wz + V[11];
        const float L = pp.cam.fx * x + cl * z, R = pp.cam.fx * x + cr * z;
        const float T = pp.cam.fy * y + ct * z, B = pp.cam.fy * y + cb * z;
        const float m = (pp.cam.fx * fabsf(x) + pp.cam.fy * fabsf(y)) + cm * fabsf(z);
        if (k == 0) { zmax = z; maxL = L; minR = R; maxT = T; minB = B; mag = m; }
        else {
            zmax = z > zmax ? z : zmax; maxL = L > maxL ? L : maxL; minR = R < minR ? R : minR;
            maxT = T > maxT ? T : maxT; minB = B < minB ? B : minB; mag = m > mag ? m : mag;
        }
    }
    const float slack = 1e-5f * mag;
    const float bx = (pp.cam.fx * Rx) * 1.004f, by = (pp.cam.fy * Ry) * 1.004f;
    if (zmax + 1e-5f * fabsf(zmax) < pp.cam.near_z) return false;
    if (maxL + slack < -bx) return false;
    if (minR - slack > bx) return false;
    if (maxT + slack < -by) return false;
    if (minB - slack > by) return false;
    return true;
}

// One thread per voxel.
__global__ __launch_bounds__(256) void voxel_flags_kernel(
    const float4 *__restrict__ box, u32 num_voxels, ProjParams pp, unsigned char *__restrict__ voxel_flags)
{
    const u32 v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= num_voxels) return;
    voxel_flags[v] = voxel_visible(pp, box[2 * (size_t)v], box[2 * (size_t)v + 1]) ? 1 : 0;
}

// Sigma = (R S)(R S)^T from an unnormalised quaternion (w, x, y, z) and the scales (Sec. 2.2 Eq. 8)
__device__ __forceinline__ void covariance3d(float qw0, float qx0, float qy0, float qz0, float s0, float s1, float s2,
                                             float &S00, float &S01, float &S02, float &S11, float &S12, float &S22)
{
    const float qn = sqrtf(qw0 * qw0 + qx0 * qx0 + qy0 * qy0 + qz0 * qz0);
    const float w = qw0 / qn, x = qx0 / qn, y = qy0 / qn, z = qz0 / qn;
    const float M00 = (1.0f - 2.0f * (y * y + z * z)) * s0;
    const float M01 = (2.0f * (x * y - w * z)) * s1;
    const float M02 = (2.0f * (x * z + w * y)) * s2;
    const float M10 = (2.0f * (x * y + w * z)) * s0;
    const float M11 = (1.0f - 2.0f * (x * x + z * z)) * s1;
    const float M12 = (2.0f * (y * z - w * x)) * s2;
    const float M20 = (2.0f * (x * z - w * y)) * s0;
    const float M21 = (2.0f * (y * z + w * x)) * s1;
    const float M22 = (1.0f - 2.0f * (x * x + y * y)) * s2;
    S00 = M00 * M00 + M01 * M01 + M02 * M02;
    S01 = M00 * M10 + M01 * M11 + M02 * M12;
    S02 = M00 * M20 + M01 * M21 + M02 * M22;
    S11 = M10 * M10 + M11 * M11 + M12 * M12;
    S12 = M10 * M20 + M11 * M21 + M12 * M22;
    S22 = M20 * M20 + M21 * M21 + M22 * M22;
}

// The view-independent part of the projection, once per scene (parameter cache, Sec. 5.2.2).
__global__ __launch_bounds__(256) void build_cov3d_kernel(
    const float *__restrict__ scale, const float *__restrict__ rot, u32 n, float *__restrict__ cov3d)
{
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const size_t N = n;
    float S00, S01, S02, S11, S12, S22;
    covariance3d(rot[i], rot[N + i], rot[2 * N + i], rot[3 * N + i], scale[i], scale[N + i], scale[2 * N + i],
                 S00, S01, S02, S11, S12, S22);
    cov3d[i] = S00; cov3d[N + i] = S01; cov3d[2 * N + i] = S02;
    cov3d[3 * N + i] = S11; cov3d[4 * N + i] = S12; cov3d[5 * N + i] = S22;
}

hipError_t launch_build_cov3d(const lmk_gs_gaussians &g, float *cov3d, hipStream_t stream)
{
    if (g.n == 0) return hipSuccess;
    hipLaunchKernelGGL(build_cov3d_kernel, dim3((g.n + 255) / 256), dim3(256), 0, stream, g.scale, g.rot, g.n, cov3d);
    return hipGetLastError();
}

// A new frame starts from a clean header and zeroed per-tile pair counters (stage 2 accumulates
// into them with atomics, and leaves them zero again).  Called by every thread of a grid of
// `threads` threads, `g` = global thread id.
__device__ __forceinline__ void reset_frame_state(ScratchHeader *header, u32 *__restrict__ tile_count,
                                                  u32 num_tiles, u32 g, u32 threads)
{
    if (g == 0) {
        header->dup_count = 0;
        header->status = LMK_GS_OK;
        header->pad = 0;
        header->big_count = 0;
        header->giant_count = 0;
        header->pad2[0] = header->pad2[1] = 0;
    }
    for (u32 t = g; t < 2u * (num_tiles + 1u); t += threads) tile_count[t] = 0;    // both halves: runs, listed primitives
}

// an empty scene: no projection kernel runs, the frame state is reset by this one
__global__ __launch_bounds__(256) void reset_frame_kernel(ScratchHeader *header, u32 *tile_count, u32 num_tiles)
{
    reset_frame_state(header, tile_count, num_tiles, blockIdx.x * blockDim.x + threadIdx.x, gridDim.x * blockDim.x);
}

// tile count of a workgroup of kPreBlock primitives (input of the prefix sum that fixes D and
// gives stage 2 a place for each workgroup's list); called by the whole workgroup
__device__ __forceinline__ void block_total(u32 cnt, u32 *s_part, u32 *__restrict__ block_sums)
{
    u32 v = cnt;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        u32 t = 0;
#pragma unroll
        for (u32 k = 0; k < kPreBlock / kWave; ++k) t += s_part[k];
        block_sums[blockIdx.x] = t;
    }
}

template <u32 DEG>
__global__ __launch_bounds__(kPreBlock) void preprocess_kernel(
    const float *__restrict__ mean, const float *__restrict__ scale, const float *__restrict__ rot,
    const float *__restrict__ opacity, const float *__restrict__ sh, const float *__restrict__ cov3d, u32 n,
    ProjParams pp, ShConsts kc,
    float *__restrict__ depth, u32 *__restrict__ tiles_touched, ushort4 *__restrict__ rect,
    float4 *__restrict__ feat, u32 *__restrict__ tile_masks,
    const unsigned char *__restrict__ voxel_flags, const uint2 *__restrict__ block_range, u32 num_voxels,
    unsigned char *__restrict__ block_visible, ScratchHeader *__restrict__ header,
    u32 *__restrict__ tile_count, u32 num_tiles, u32 *__restrict__ block_sums)
{
    __shared__ u32 s_part[kPreBlock / kWave];
    const u32 i = blockIdx.x * kPreBlock + threadIdx.x;
    reset_frame_state(header, tile_count, num_tiles, i, gridDim.x * kPreBlock);
    if (voxel_flags) {
        // voxel filter: does any voxel holding one of this workgroup's primitives pass?
        const uint2 r = block_range[blockIdx.x];
        // a corrupt range can only cost time, never an out-of-bounds read
        const u32 last = r.y < num_voxels ? r.y : num_voxels - 1;
        int mine = 0;
        for (u32 v = r.x + threadIdx.x; v <= last; v += kPreBlock) mine |= voxel_flags[v];
        const int any = __syncthreads_or(mine);
        if (block_visible && threadIdx.x == 0) block_visible[blockIdx.x] = any ? 1 : 0;
        if (!any) {
            // nothing of this workgroup can be binned: no input is read
            if (i < n) tiles_touched[i] = 0;
            if (threadIdx.x == 0) block_sums[blockIdx.x] = 0;
            return;
        }
    }
    const size_t N = n;
    u32 cnt = 0;            // tiles of the support rectangle (then: tiles kept)
    u32 kept_mask = 0;      // binning rule 1: bit s = slot s (row-major) of the rectangle is kept, for the first 32 slots
    float mx = 0.f, my = 0.f, mz = 0.f, pz = 0.f, o = 0.f;
    float u = 0.f, v = 0.f, cA = 1.f, cB = 0.f, cC = 1.f;
    u32 x0 = 0, y0 = 0, x1 = 0, y1 = 0;

    if (i < n) {
        const float *V = pp.cam.view;
        // inputs are read exactly once per frame: stream them past the caches.  All eleven
        // geometry planes are requested before the first use: primitives are culled in no
        // particular index order, so the cache lines of a plane are needed whatever this lane
        // decides, and one round trip to memory replaces three dependent ones.
        mx = __builtin_nontemporal_load(mean + i); my = __builtin_nontemporal_load(mean + N + i);
        mz = __builtin_nontemporal_load(mean + 2 * N + i);
        // Sigma: from the parameter cache when the caller built one, else from rotation and scale
        float S00, S01, S02, S11, S12, S22;
        float qw0 = 1.f, qx0 = 0.f, qy0 = 0.f, qz0 = 0.f, s0 = 0.f, s1 = 0.f, s2 = 0.f;
        if (cov3d) {
            S00 = __builtin_nontemporal_load(cov3d + i); S01 = __builtin_nontemporal_load(cov3d + N + i);
            S02 = __builtin_nontemporal_load(cov3d + 2 * N + i); S11 = __builtin_nontemporal_load(cov3d + 3 * N + i);
            S12 = __builtin_nontemporal_load(cov3d + 4 * N + i); S22 = __builtin_nontemporal_load(cov3d + 5 * N + i);
        } else {
            qw0 = __builtin_nontemporal_load(rot + i); qx0 = __builtin_nontemporal_load(rot + N + i);
            qy0 = __builtin_nontemporal_load(rot + 2 * N + i); qz0 = __builtin_nontemporal_load(rot + 3 * N + i);
            s0 = __builtin_nontemporal_load(scale + i); s1 = __builtin_nontemporal_load(scale + N + i);
            s2 = __builtin_nontemporal_load(scale + 2 * N + i);
        }
        const float o_in = __builtin_nontemporal_load(opacity + i);
        const float px = V[0] * mx + V[1] * my + V[2] * mz + V[3];
        const float py = V[4] * mx + V[5] * my + V[6] * mz + V[7];
        pz = V[8] * mx + V[9] * my + V[10] * mz + V[11];
        if (pz > pp.cam.near_z) {
            if (!cov3d) covariance3d(qw0, qx0, qy0, qz0, s0, s1, s2, S00, S01, S02, S11, S12, S22);

            // EWA: Jacobian of the pinhole map at the guard-band clamped mean, times W
            const float txz = clamp_nan_lo(px / pz, -pp.lim_x, pp.lim_x) * pz;
            const float tyz = clamp_nan_lo(py / pz, -pp.lim_y, pp.lim_y) * pz;
            const float J00 = pp.cam.fx / pz, J02 = -(pp.cam.fx * txz) / (pz * pz);
            const float J11 = pp.cam.fy / pz, J12 = -(pp.cam.fy * tyz) / (pz * pz);
            // the zero entries of J are kept as written products so that every
            // sum has the same terms (and zero signs) as the plain 2x3 * 3x3 product
            const float T00 = J00 * V[0] + 0.0f * V[4] + J02 * V[8];
            const float T01 = J00 * V[1] + 0.0f * V[5] + J02 * V[9];
            const float T02 = J00 * V[2] + 0.0f * V[6] + J02 * V[10];
            const float T10 = 0.0f * V[0] + J11 * V[4] + J12 * V[8];
            const float T11 = 0.0f * V[1] + J11 * V[5] + J12 * V[9];
            const float T12 = 0.0f * V[2] + J11 * V[6] + J12 * V[10];
            const float U00 = T00 * S00 + T01 * S01 + T02 * S02;
            const float U01 = T00 * S01 + T01 * S11 + T02 * S12;
            const float U02 = T00 * S02 + T01 * S12 + T02 * S22;
            const float U10 = T10 * S00 + T11 * S01 + T12 * S02;
            const float U11 = T10 * S01 + T11 * S11 + T12 * S12;
            const float U12 = T10 * S02 + T11 * S12 + T12 * S22;
            const float a = (U00 * T00 + U01 * T01 + U02 * T02) + pp.cam.lowpass;
            const float b = U00 * T10 + U01 * T11 + U02 * T12;
            const float c = (U10 * T10 + U11 * T11 + U12 * T12) + pp.cam.lowpass;

            const float det = a * c - b * b;
            o = o_in;
            if (det > 0.0f && !(o < 1.0f / 255.0f)) {
                cA = c / det; cB = -b / det; cC = a / det;
                u = (pp.cam.fx * px) / pz + pp.cam.cx;
                v = (pp.cam.fy * py) / pz + pp.cam.cy;
                const float hx = sqrtf(11.09f * a);
                const float hy = sqrtf(11.09f * c);
                const float TS = (float)LMK_GS_TILE;
                const float fTX = (float)pp.tiles_x, fTY = (float)pp.tiles_y;
                x0 = (u32)clamp_nan_lo(floorf((u - hx) / TS), 0.0f, fTX);
                x1 = (u32)clamp_nan_lo(floorf((u + hx) / TS) + 1.0f, 0.0f, fTX);
                y0 = (u32)clamp_nan_lo(floorf((v - hy) / TS), 0.0f, fTY);
                y1 = (u32)clamp_nan_lo(floorf((v + hy) / TS) + 1.0f, 0.0f, fTY);
                cnt = (x1 > x0 && y1 > y0) ? (x1 - x0) * (y1 - y0) : 0u;
            }
        }
    }

    // SH records (see below): a wavefront most of whose primitives are still alive requests its
    // whole block of records now, so that the loads are in flight during the tile counting
    constexpr u32 kVec = LMK_GS_SH_STRIDE(DEG) / 4;         // 16-byte vectors per record
    constexpr u32 kCoef = (DEG + 1) * (DEG + 1);
    constexpr u32 kPart = kVec > 7 ? kVec / 2 : kVec;       // vectors of a record staged at a time
    constexpr u32 kParts = kVec / kPart;
    constexpr u32 kSlot = kPart + 1;                        // padded record stride in LDS (bank spread)
    constexpr u32 kDirectMax = 40;                          // survivors per wavefront served by direct loads
    static_assert(kPart * kParts == kVec, "records are staged in equal parts");
    __shared__ f32x4 s_sh[kPreBlock / kWave][kWave * kSlot];
    const u32 sh_lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const bool staged = (u32)__builtin_popcountll(__builtin_amdgcn_ballot_w64(cnt > 0)) > kDirectMax;   // wave-uniform
    const u32 first = blockIdx.x * kPreBlock + wv * kWave;  // first primitive of this wavefront
    const u32 recs = first < n ? (n - first < kWave ? n - first : kWave) : 0u;
    f32x4 buf[kVec];
    if (staged) {
        // every load instruction covers 1 KiB of consecutive addresses, all of them in flight together
        const f32x4 *src = reinterpret_cast<const f32x4 *>(sh) + (size_t)first * kVec;
#pragma unroll
        for (u32 j = 0; j < kVec; ++j) {
            const u32 idx = j * kWave + sh_lane;
            buf[j] = idx < recs * kVec ? src[idx] : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }

    // binning rule 1: count only the tiles of the rectangle that the splat can reach.
    // Small rectangles are walked by their own lane; large ones one at a time by the whole
    // wavefront (64 tiles per step), so that one huge splat does not stall 63 idle lanes.
    if (pp.cam.binning == 1u) {
        const TileTest tt = make_tile_test(u, v, cA, cB, cC, opacity_tau(pp, o));
        const u32 area = cnt, w = x1 - x0;
        constexpr u32 kOwn = 16;
        u32 kept = 0;
        if (area > 0 && area <= kOwn) {
            u32 slot = 0;
            for (u32 ty = y0; ty < y1; ++ty)
                for (u32 tx = x0; tx < x1; ++tx, ++slot)
                    if (tile_kept(tt, tx, ty)) { ++kept; kept_mask |= 1u << slot; }
        }
        u64 big = __builtin_amdgcn_ballot_w64(area > kOwn);
        const u32 lane = threadIdx.x & (kWave - 1);
        while (big != 0ull) {
            const int src = (int)__builtin_ctzll(big);
            big &= big - 1ull;
            TileTest bt;
            bt.u = __shfl(tt.u, src, 64); bt.v = __shfl(tt.v, src, 64);
            bt.A = __shfl(tt.A, src, 64); bt.B = __shfl(tt.B, src, 64); bt.C = __shfl(tt.C, src, 64);
            bt.rx = __shfl(tt.rx, src, 64); bt.ry = __shfl(tt.ry, src, 64); bt.tau = __shfl(tt.tau, src, 64);
            const u32 bx0 = __shfl(x0, src, 64), by0 = __shfl(y0, src, 64);
            const u32 bw = __shfl(w, src, 64), barea = __shfl(area, src, 64);
            u32 c = 0;
            bool k0 = false;                                  // this lane's slot of the first 64
            for (u32 t = lane; t < barea; t += kWave) {
                const u32 row = t / bw;
                const bool k = tile_kept(bt, bx0 + (t - row * bw), by0 + row);
                if (t == lane) k0 = k;
                c += k ? 1u : 0u;
            }
#pragma unroll
            for (int o2 = 32; o2 > 0; o2 >>= 1) c += __shfl_xor(c, o2, 64);
            // slots 0..31: the whole mask of a rectangle of up to 32 tiles
            const u32 first_round = (u32)__builtin_amdgcn_ballot_w64(k0);
            if ((int)lane == src) { kept = c; kept_mask = first_round; }
        }
        cnt = kept;
    }

    // view-dependent colour: 0.5 + sum_k Y_k(dir) sh_k, clamped at 0.  The SH records are the bulk of
    // the input bytes and only primitives that survived need theirs.  Where most of a wavefront's 64
    // records are needed, the whole contiguous block of records is streamed in fully coalesced loads
    // through LDS (a lane reading its own 192-byte record directly would touch 64 different cache
    // lines per load instruction); where few are (close-up views cull most primitives), each survivor
    // fetches only its own record and the rest of the block is never read.
    {
        const f32x4 *rec = reinterpret_cast<const f32x4 *>(sh) + (size_t)i * kVec;   // this primitive's record
        const f32x4 *lrec = &s_sh[wv][sh_lane * kSlot];

        float Y[16];
        if (cnt) {
            float dx = mx - pp.cam.cam_pos[0], dy = my - pp.cam.cam_pos[1], dz = mz - pp.cam.cam_pos[2];
            const float inv = 1.0f / sqrtf(dx * dx + dy * dy + dz * dz);
            dx *= inv; dy *= inv; dz *= inv;
            Y[0] = kc.k0;
            if (DEG > 0) { Y[1] = -kc.k1 * dy; Y[2] = kc.k1 * dz; Y[3] = -kc.k1 * dx; }
            const float xx = dx * dx, yy = dy * dy, zz = dz * dz;
            if (DEG > 1) {
                Y[4] = kc.k2 * dx * dy; Y[5] = -kc.k2 * dy * dz;
                Y[6] = kc.k20 * (2.0f * zz - xx - yy);
                Y[7] = -kc.k2 * dx * dz; Y[8] = 0.5f * kc.k2 * (xx - yy);
            }
            if (DEG > 2) {
                Y[9] = -kc.k33 * dy * (3.0f * xx - yy);
                Y[10] = kc.k32 * dx * dy * dz;
                Y[11] = -kc.k31 * dy * (4.0f * zz - xx - yy);
                Y[12] = kc.k30 * dz * (2.0f * zz - 3.0f * xx - 3.0f * yy);
                Y[13] = -kc.k31 * dx * (4.0f * zz - xx - yy);
                Y[14] = kc.k32b * dz * (xx - yy);
                Y[15] = -kc.k33 * dx * (xx - 3.0f * yy);
            }
        }
        // coefficient k of channel ch sits at float [3k + ch] of the record
        float acc[3] = { 0.5f, 0.5f, 0.5f };
#pragma unroll
        for (u32 part = 0; part < kParts; ++part) {
            if (staged) {
                // transpose through LDS, one part of every record at a time: vector idx of the block
                // is vector idx % kVec of record idx / kVec
#pragma unroll
                for (u32 j = 0; j < kVec; ++j) {
                    const u32 idx = j * kWave + sh_lane;
                    const u32 r = idx / kVec, v = idx % kVec;
                    if (r < recs && v / kPart == part) s_sh[wv][r * kSlot + (v - part * kPart)] = buf[j];
                }
                // the loads below read what other lanes of this wavefront stored: LDS accesses of
                // one wavefront complete in program order
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
            if (cnt) {
#pragma unroll
                for (u32 j = 0; j < kPart; ++j) {
                    const u32 jj = part * kPart + j;
                    const f32x4 q = staged ? lrec[j] : __builtin_nontemporal_load(rec + jj);
#pragma unroll
                    for (u32 m = 0; m < 4; ++m) {
                        const u32 e = 4 * jj + m;               // compile-time: coefficient e / 3, channel e % 3
                        if (e / 3 < kCoef) acc[e % 3] += Y[e / 3] * q[m];
                    }
                }
            }
            if (staged && part + 1 < kParts) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
        if (cnt) {
            const float r = fmaxf(acc[0], 0.0f), g = fmaxf(acc[1], 0.0f), bl = fmaxf(acc[2], 0.0f);

            depth[i] = pz;
            rect[i] = make_ushort4((unsigned short)x0, (unsigned short)y0,
                                   (unsigned short)x1, (unsigned short)y1);
            float4 *f = feat + (size_t)i * (LMK_GS_FEAT_STRIDE / 4);
            f[0] = make_float4(u, v, cA, cB);
            f[1] = make_float4(cC, o, r, g);
            f[2] = make_float4(bl, 0.0f, 0.0f, 0.0f);
        }
    }
    if (i < n) {
        tiles_touched[i] = cnt;
        // rectangles of up to 32 tiles: the emit stage expands the kept tiles from this mask
        if (pp.cam.binning == 1u && cnt) tile_masks[i] = kept_mask;
    }
    block_total(cnt, s_part, block_sums);
}

// Exclusive prefix sum (u64) over the workgroup tile counts, in two levels: each workgroup of
// this kernel scans kScanGroup consecutive counts (-> block_offsets, relative to the group) and
// publishes the group's total; a consumer adds the totals of the groups before its own.  D is
// the sum of the group totals, added to the header the preprocess kernel has just cleared.
// (One workgroup scanning everything takes longer than the whole rest of this: its time is
// the latency of one compute unit, not the data.)
__global__ __launch_bounds__(kScanGroup) void scan_block_sums_kernel(
    const u32 *__restrict__ block_sums, u32 nb, u64 *__restrict__ block_offsets,
    u64 *__restrict__ group_totals, ScratchHeader *__restrict__ header)
{
    constexpr u32 kWaves = kScanGroup / kWave;
    __shared__ u64 s_wave[kWaves];
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 b = blockIdx.x * kScanGroup + tid;
    const u32 x = b < nb ? block_sums[b] : 0u;
    u64 incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const u64 t = __shfl_up(incl, o, 64);
        if ((int)lane >= o) incl += t;
    }
    if (lane == kWave - 1) s_wave[wv] = incl;
    __syncthreads();
    u64 before = 0, total = 0;
#pragma unroll
    for (u32 k = 0; k < kWaves; ++k) {
        const u64 w = s_wave[k];
        if (k < wv) before += w;
        total += w;
    }
    if (b < nb) block_offsets[b] = before + incl - x;
    if (tid == 0) {
        group_totals[blockIdx.x] = total;
        if (total) atomicAdd(reinterpret_cast<unsigned long long *>(&header->dup_count), (unsigned long long)total);
    }
}

static hipError_t launch_scan_block_sums(char *scratch, const ScratchLayout &L, hipStream_t stream)
{
    hipLaunchKernelGGL(scan_block_sums_kernel, dim3((L.pre_blocks + kScanGroup - 1) / kScanGroup), dim3(kScanGroup), 0, stream,
                       reinterpret_cast<const u32 *>(scratch + L.block_sums), L.pre_blocks,
                       reinterpret_cast<u64 *>(scratch + L.block_offsets),
                       reinterpret_cast<u64 *>(scratch + L.group_totals),
                       reinterpret_cast<ScratchHeader *>(scratch + L.header));
    return hipGetLastError();
}

hipError_t launch_preprocess(const lmk_gs_gaussians &g, const lmk_gs_voxel_index *index, uint8_t *block_visible,
                             const ProjParams &pp, const lmk_gs_projected &out,
                             char *scratch, const ScratchLayout &L, hipStream_t stream)
{
    static const ShConsts kc = make_sh_consts();
    ScratchHeader *header = reinterpret_cast<ScratchHeader *>(scratch + L.header);
    u32 *tile_count = reinterpret_cast<u32 *>(scratch + L.tile_count);
    u32 *block_sums = reinterpret_cast<u32 *>(scratch + L.block_sums);
    const u32 num_tiles = pp.tiles_x * pp.tiles_y;
    if (L.pre_blocks == 0) {
        hipLaunchKernelGGL(reset_frame_kernel, dim3(16), dim3(256), 0, stream, header, tile_count, num_tiles);
        return hipGetLastError();
    }
    const unsigned char *vflags = nullptr;
    const uint2 *ranges = nullptr;
    u32 num_voxels = 0;
    if (index) {
        num_voxels = index->num_voxels;
        ranges = reinterpret_cast<const uint2 *>(index->block_range);
        if (index->visible) {
            vflags = index->visible;                // this frame's flags, computed by the caller's earlier call
        } else {
            unsigned char *f = reinterpret_cast<unsigned char *>(scratch + L.voxel_flags);
            hipLaunchKernelGGL(voxel_flags_kernel, dim3((num_voxels + 255) / 256), dim3(256), 0, stream,
                               reinterpret_cast<const float4 *>(index->box), num_voxels, pp, f);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            vflags = f;
        }
    }
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(L.pre_blocks), dim3(kPreBlock), 0, stream,
                           g.mean, g.scale, g.rot, g.opacity, g.sh, g.cov3d, g.n, pp, kc,
                           out.depth, out.tiles_touched, reinterpret_cast<ushort4 *>(out.rect),
                           reinterpret_cast<float4 *>(out.feat),
                           reinterpret_cast<u32 *>(scratch + L.tile_masks),
                           vflags, ranges, num_voxels, index ? block_visible : nullptr, header,
                           tile_count, num_tiles, block_sums);
    };
    switch (g.sh_degree) {
        case 0: launch(preprocess_kernel<0>); break;
        case 1: launch(preprocess_kernel<1>); break;
        case 2: launch(preprocess_kernel<2>); break;
        default: launch(preprocess_kernel<3>); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_scan_block_sums(scratch, L, stream);
}

// ---------------------------------------------------------------- hand-over rebuilt from the outputs
// What lmk_gs_preprocess leaves in the scratch for lmk_gs_bin_sort -- the pair count, zeroed
// per-tile counters, the prefix sum over the workgroup tile counts and, under binning rule 1, the
// mask of kept tiles of every rectangle of up to 32 tiles -- recomputed from the per-primitive outputs alone (tiles_touched, rect and the
// feature record), with the arithmetic of preprocess_kernel, so that a caller holding only those
// outputs can run stage 2 on a scratch buffer of its own.
__global__ __launch_bounds__(kPreBlock) void rebuild_handover_kernel(
    const u32 *__restrict__ tiles_touched, const ushort4 *__restrict__ rect, const float4 *__restrict__ feat,
    u32 n, ProjParams pp, u32 *__restrict__ tile_masks, ScratchHeader *__restrict__ header,
    u32 *__restrict__ tile_count, u32 num_tiles, u32 *__restrict__ block_sums)
{
    __shared__ u32 s_part[kPreBlock / kWave];
    const u32 i = blockIdx.x * kPreBlock + threadIdx.x;
    reset_frame_state(header, tile_count, num_tiles, i, gridDim.x * kPreBlock);
    const u32 cnt = i < n ? tiles_touched[i] : 0u;
    if (pp.cam.binning == 1u && cnt) {
        const ushort4 r = rect[i];
        const u32 w = (u32)r.z - (u32)r.x, area = w * ((u32)r.w - (u32)r.y);
        if (area <= 32u) {
            const float4 *f = feat + (size_t)i * (LMK_GS_FEAT_STRIDE / 4);
            const float4 f0 = f[0], f1 = f[1];
            const TileTest tt = make_tile_test(f0.x, f0.y, f0.z, f0.w, f1.x, opacity_tau(pp, f1.y));
            u32 mask = 0, slot = 0;
            for (u32 ty = r.y; ty < r.w; ++ty)
                for (u32 tx = r.x; tx < r.z; ++tx, ++slot)
                    if (tile_kept(tt, tx, ty)) mask |= 1u << slot;
            tile_masks[i] = mask;
        }
    }
    block_total(cnt, s_part, block_sums);
}

hipError_t launch_rebuild_handover(const lmk_gs_projected &proj, u32 n, const ProjParams &pp,
                                   char *scratch, const ScratchLayout &L, hipStream_t stream)
{
    ScratchHeader *header = reinterpret_cast<ScratchHeader *>(scratch + L.header);
    u32 *tile_count = reinterpret_cast<u32 *>(scratch + L.tile_count);
    const u32 num_tiles = pp.tiles_x * pp.tiles_y;
    if (L.pre_blocks == 0) {
        hipLaunchKernelGGL(reset_frame_kernel, dim3(16), dim3(256), 0, stream, header, tile_count, num_tiles);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(rebuild_handover_kernel, dim3(L.pre_blocks), dim3(kPreBlock), 0, stream,
                       proj.tiles_touched, reinterpret_cast<const ushort4 *>(proj.rect),
                       reinterpret_cast<const float4 *>(proj.feat), n, pp,
                       reinterpret_cast<u32 *>(scratch + L.tile_masks), header, tile_count, num_tiles,
                       reinterpret_cast<u32 *>(scratch + L.block_sums));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_scan_block_sums(scratch, L, stream);
}

// {D, status} of the frame from the scratch header to a caller's device array of two 64-bit words
__global__ void copy_status_kernel(const ScratchHeader *__restrict__ header, u64 *__restrict__ out)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = header->dup_count;
        out[1] = (u64)(long long)header->status;
    }
}

hipError_t launch_copy_status(const char *scratch, const ScratchLayout &L, u64 *out, hipStream_t stream)
{
    hipLaunchKernelGGL(copy_status_kernel, dim3(1), dim3(64), 0, stream,
                       reinterpret_cast<const ScratchHeader *>(scratch + L.header), out);
    return hipGetLastError();
}

hipError_t launch_box_flags(const float *box, u32 count, const ProjParams &pp, uint8_t *visible, hipStream_t stream)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(voxel_flags_kernel, dim3((count + 255) / 256), dim3(256), 0, stream,
                       reinterpret_cast<const float4 *>(box), count, pp, visible);
    return hipGetLastError();
}

}  // namespace lmk
