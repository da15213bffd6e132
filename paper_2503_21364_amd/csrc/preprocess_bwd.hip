// Gradient of a scalar loss through stage 1, the per-primitive projection (Sec. 2.2: every
// parameter of the primitives is optimised through the rendering process).  Input: dL/d of the
// feature record {u, v, A, B, C, opacity, r, g, b} of every primitive, as
// lmk_gs_render_backward leaves it.  Output: dL/d{mean, scale, rotation quaternion as stored,
// opacity, SH coefficients}.
//
// One thread per primitive, fp32.  The forward quantities are recomputed (position in camera
// space, rotation matrix, covariance, the two rows T of J W, the 2D covariance) and the steps
// are differentiated in reverse order:
//   conic (A, B, C) = (c, -b, a) / (a c - b^2)
//   a = T0 Sigma T0^T + h, b = T0 Sigma T1^T, c = T1 Sigma T1^T + h
//   T = J W, J from the camera-space position p; where p_x / p_z (p_y / p_z) is outside the guard
//   band it is clamped and J's third column depends on p_z only
//   u = fx p_x / p_z + cx, v likewise;  p = W mean + t
//   Sigma = M M^T, M = R(q / |q|) diag(s)
//   colour = max(0, 0.5 + sum_k Y_k(d) sh_k), d = (mean - camera centre) / |.|
// Culls and clamps are constants of the derivative: a primitive that was not binned
// (tiles_touched == 0) gets zeros, a colour channel clamped at 0 passes nothing on.
//
// Bound by HBM traffic: 36 B of gradient + 56 B of geometry + 192 B of SH in, 44 B + 192 B out
// per binned primitive.
#include <cmath>

#include "lmk_gs_internal.h"

namespace lmk {

namespace {

struct ShK { float k1, k2, k20, k33, k32, k31, k30, k32b, k0; };

ShK make_shk()
{
    const double pi = 3.14159265358979323846;
    ShK k;
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

// real SH basis (order and signs of the forward kernel) and its gradient with respect to the direction
template <u32 DEG>
__device__ __forceinline__ void sh_basis_and_grad(float x, float y, float z, const ShK &k,
                                                  float (&Y)[16], float (&dx)[16], float (&dy)[16], float (&dz)[16])
{
#pragma unroll
    for (u32 i = 0; i < 16; ++i) { Y[i] = 0.f; dx[i] = 0.f; dy[i] = 0.f; dz[i] = 0.f; }
    Y[0] = k.k0;
    if (DEG >= 1) {
        Y[1] = -k.k1 * y;  dy[1] = -k.k1;
        Y[2] = k.k1 * z;   dz[2] = k.k1;
        Y[3] = -k.k1 * x;  dx[3] = -k.k1;
    }
    const float xx = x * x, yy = y * y, zz = z * z;
    if (DEG >= 2) {
        Y[4] = k.k2 * x * y;                  dx[4] = k.k2 * y;          dy[4] = k.k2 * x;
        Y[5] = -k.k2 * y * z;                 dy[5] = -k.k2 * z;         dz[5] = -k.k2 * y;
        Y[6] = k.k20 * (2.f * zz - xx - yy);  dx[6] = -2.f * k.k20 * x;  dy[6] = -2.f * k.k20 * y;  dz[6] = 4.f * k.k20 * z;
        Y[7] = -k.k2 * x * z;                 dx[7] = -k.k2 * z;         dz[7] = -k.k2 * x;
        Y[8] = 0.5f * k.k2 * (xx - yy);       dx[8] = k.k2 * x;          dy[8] = -k.k2 * y;
    }
    if (DEG >= 3) {
        Y[9] = -k.k33 * y * (3.f * xx - yy);
        dx[9] = -k.k33 * 6.f * x * y;         dy[9] = -k.k33 * (3.f * xx - 3.f * yy);
        Y[10] = k.k32 * x * y * z;
        dx[10] = k.k32 * y * z;               dy[10] = k.k32 * x * z;     dz[10] = k.k32 * x * y;
        Y[11] = -k.k31 * y * (4.f * zz - xx - yy);
        dx[11] = k.k31 * 2.f * x * y;         dy[11] = -k.k31 * (4.f * zz - xx - 3.f * yy);   dz[11] = -k.k31 * 8.f * y * z;
        Y[12] = k.k30 * z * (2.f * zz - 3.f * xx - 3.f * yy);
        dx[12] = -k.k30 * 6.f * x * z;        dy[12] = -k.k30 * 6.f * y * z;   dz[12] = k.k30 * (6.f * zz - 3.f * xx - 3.f * yy);
        Y[13] = -k.k31 * x * (4.f * zz - xx - yy);
        dx[13] = -k.k31 * (4.f * zz - 3.f * xx - yy);   dy[13] = k.k31 * 2.f * x * y;   dz[13] = -k.k31 * 8.f * x * z;
        Y[14] = k.k32b * z * (xx - yy);
        dx[14] = k.k32b * 2.f * x * z;        dy[14] = -k.k32b * 2.f * y * z;  dz[14] = k.k32b * (xx - yy);
        Y[15] = -k.k33 * x * (xx - 3.f * yy);
        dx[15] = -k.k33 * (3.f * xx - 3.f * yy);        dy[15] = k.k33 * 6.f * x * y;
    }
}

template <u32 DEG>
__global__ __launch_bounds__(256) void preprocess_backward_kernel(
    const float *__restrict__ mean, const float *__restrict__ scale, const float *__restrict__ rot,
    const float *__restrict__ sh, u32 n, ProjParams pp, ShK shk,
    const u32 *__restrict__ tiles_touched, const float *__restrict__ grad_feat,
    float *__restrict__ g_mean, float *__restrict__ g_scale, float *__restrict__ g_rot,
    float *__restrict__ g_opacity, float *__restrict__ g_sh)
{
    constexpr u32 NC = (DEG + 1) * (DEG + 1);
    constexpr u32 STRIDE = LMK_GS_SH_STRIDE(DEG);
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const size_t N = n;
    float *gsh = g_sh + (size_t)i * STRIDE;
    if (tiles_touched[i] == 0u) {
        g_mean[i] = 0.f; g_mean[N + i] = 0.f; g_mean[2 * N + i] = 0.f;
        g_scale[i] = 0.f; g_scale[N + i] = 0.f; g_scale[2 * N + i] = 0.f;
        g_rot[i] = 0.f; g_rot[N + i] = 0.f; g_rot[2 * N + i] = 0.f; g_rot[3 * N + i] = 0.f;
        g_opacity[i] = 0.f;
        for (u32 k = 0; k < STRIDE / 4; ++k) reinterpret_cast<float4 *>(gsh)[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        return;
    }
    const float *gf = grad_feat + (size_t)i * LMK_GS_FEAT_STRIDE;
    const float gu = gf[0], gv = gf[1], gA = gf[2], gB = gf[3], gC = gf[4];
    const float gcol[3] = { gf[6], gf[7], gf[8] };
    g_opacity[i] = gf[5];

    // forward quantities
    const lmk_gs_camera &cam = pp.cam;
    const float *V = cam.view;
    const float mx = mean[i], my = mean[N + i], mz = mean[2 * N + i];
    const float px = V[0] * mx + V[1] * my + V[2] * mz + V[3];
    const float py = V[4] * mx + V[5] * my + V[6] * mz + V[7];
    const float pz = V[8] * mx + V[9] * my + V[10] * mz + V[11];
    const float q0 = rot[i], q1 = rot[N + i], q2 = rot[2 * N + i], q3 = rot[3 * N + i];
    const float qn = sqrtf(q0 * q0 + q1 * q1 + q2 * q2 + q3 * q3);
    const float w = q0 / qn, x = q1 / qn, y = q2 / qn, z = q3 / qn;
    float R[3][3];
    R[0][0] = 1.f - 2.f * (y * y + z * z); R[0][1] = 2.f * (x * y - w * z); R[0][2] = 2.f * (x * z + w * y);
    R[1][0] = 2.f * (x * y + w * z); R[1][1] = 1.f - 2.f * (x * x + z * z); R[1][2] = 2.f * (y * z - w * x);
    R[2][0] = 2.f * (x * z - w * y); R[2][1] = 2.f * (y * z + w * x); R[2][2] = 1.f - 2.f * (x * x + y * y);
    const float s[3] = { scale[i], scale[N + i], scale[2 * N + i] };
    float M[3][3], Sg[3][3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int c = 0; c < 3; ++c) M[r][c] = R[r][c] * s[c];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int c = 0; c < 3; ++c) Sg[r][c] = M[r][0] * M[c][0] + M[r][1] * M[c][1] + M[r][2] * M[c][2];
    const float iz = 1.f / pz, iz2 = iz * iz;
    const float rx = px * iz, ry = py * iz;
    const float lim_x = pp.lim_x, lim_y = pp.lim_y;
    const bool clx = !(rx > -lim_x) || rx > lim_x, cly = !(ry > -lim_y) || ry > lim_y;
    const float cxr = !(rx > -lim_x) ? -lim_x : (rx > lim_x ? lim_x : rx);
    const float cyr = !(ry > -lim_y) ? -lim_y : (ry > lim_y ? lim_y : ry);
    const float fx = cam.fx, fy = cam.fy;
    const float J00 = fx * iz, J02 = -fx * cxr * iz, J11 = fy * iz, J12 = -fy * cyr * iz;
    float T0[3], T1[3], ST0[3], ST1[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        T0[c] = J00 * V[c] + J02 * V[8 + c];
        T1[c] = J11 * V[4 + c] + J12 * V[8 + c];
    }
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        ST0[c] = Sg[c][0] * T0[0] + Sg[c][1] * T0[1] + Sg[c][2] * T0[2];
        ST1[c] = Sg[c][0] * T1[0] + Sg[c][1] * T1[1] + Sg[c][2] * T1[2];
    }
    const float a = T0[0] * ST0[0] + T0[1] * ST0[1] + T0[2] * ST0[2] + cam.lowpass;
    const float b = T0[0] * ST1[0] + T0[1] * ST1[1] + T0[2] * ST1[2];
    const float c = T1[0] * ST1[0] + T1[1] * ST1[1] + T1[2] * ST1[2] + cam.lowpass;
    const float det = a * c - b * b;
    const float id2 = 1.f / (det * det);

    // conic -> a, b, c
    const float ga = (-gA * c * c + gB * b * c - gC * b * b) * id2;
    const float gb = (2.f * gA * b * c - gB * (a * c + b * b) + 2.f * gC * a * b) * id2;
    const float gc = (-gA * b * b + gB * a * b - gC * a * a) * id2;
    // a, b, c -> Sigma (all nine entries) and the rows of T
    float gS[3][3], gT0[3], gT1[3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int k = 0; k < 3; ++k) gS[r][k] = ga * T0[r] * T0[k] + gb * T0[r] * T1[k] + gc * T1[r] * T1[k];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        gT0[k] = 2.f * ga * ST0[k] + gb * ST1[k];
        gT1[k] = 2.f * gc * ST1[k] + gb * ST0[k];
    }
    // T = J W -> the four non-zero entries of J
    const float gJ00 = gT0[0] * V[0] + gT0[1] * V[1] + gT0[2] * V[2];
    const float gJ02 = gT0[0] * V[8] + gT0[1] * V[9] + gT0[2] * V[10];
    const float gJ11 = gT1[0] * V[4] + gT1[1] * V[5] + gT1[2] * V[6];
    const float gJ12 = gT1[0] * V[8] + gT1[1] * V[9] + gT1[2] * V[10];
    // J and (u, v) -> p
    float gpx = gu * fx * iz, gpy = gv * fy * iz;
    float gpz = -(gJ00 * fx + gJ11 * fy) * iz2 - (gu * fx * px + gv * fy * py) * iz2;
    if (clx) gpz += gJ02 * fx * cxr * iz2;
    else { gpx -= gJ02 * fx * iz2; gpz += gJ02 * 2.f * fx * px * iz2 * iz; }
    if (cly) gpz += gJ12 * fy * cyr * iz2;
    else { gpy -= gJ12 * fy * iz2; gpz += gJ12 * 2.f * fy * py * iz2 * iz; }
    float gm[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) gm[k] = V[k] * gpx + V[4 + k] * gpy + V[8 + k] * gpz;

    // Sigma = M M^T -> M -> s, R
    float gR[3][3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        float gs = 0.f;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const float gM = (gS[r][0] + gS[0][r]) * M[0][k] + (gS[r][1] + gS[1][r]) * M[1][k] + (gS[r][2] + gS[2][r]) * M[2][k];
            gs += gM * R[r][k];
            gR[r][k] = gM * s[k];
        }
        g_scale[(size_t)k * N + i] = gs;
    }
    // R -> unit quaternion -> stored quaternion
    float gq[4];
    gq[0] = 2.f * (-z * gR[0][1] + y * gR[0][2] + z * gR[1][0] - x * gR[1][2] - y * gR[2][0] + x * gR[2][1]);
    gq[1] = 2.f * (y * gR[0][1] + z * gR[0][2] + y * gR[1][0] - 2.f * x * gR[1][1] - w * gR[1][2]
                   + z * gR[2][0] + w * gR[2][1] - 2.f * x * gR[2][2]);
    gq[2] = 2.f * (-2.f * y * gR[0][0] + x * gR[0][1] + w * gR[0][2] + x * gR[1][0] + z * gR[1][2]
                   - w * gR[2][0] + z * gR[2][1] - 2.f * y * gR[2][2]);
    gq[3] = 2.f * (-2.f * z * gR[0][0] - w * gR[0][1] + x * gR[0][2] + w * gR[1][0] - 2.f * z * gR[1][1]
                   + y * gR[1][2] + x * gR[2][0] + y * gR[2][1]);
    const float qd = gq[0] * w + gq[1] * x + gq[2] * y + gq[3] * z;
    g_rot[i] = (gq[0] - w * qd) / qn;
    g_rot[N + i] = (gq[1] - x * qd) / qn;
    g_rot[2 * N + i] = (gq[2] - y * qd) / qn;
    g_rot[3 * N + i] = (gq[3] - z * qd) / qn;

    // colour
    const float vx = mx - cam.cam_pos[0], vy = my - cam.cam_pos[1], vz = mz - cam.cam_pos[2];
    const float len = sqrtf(vx * vx + vy * vy + vz * vz);
    const float dxn = vx / len, dyn = vy / len, dzn = vz / len;
    float Y[16], dYx[16], dYy[16], dYz[16];
    sh_basis_and_grad<DEG>(dxn, dyn, dzn, shk, Y, dYx, dYy, dYz);
    // the SH record and its gradient as whole 16-byte vectors (both are 16-byte aligned records)
    float coef[STRIDE], gout[STRIDE];
    {
        const float4 *c4 = reinterpret_cast<const float4 *>(sh + (size_t)i * STRIDE);
#pragma unroll
        for (u32 k = 0; k < STRIDE / 4; ++k) {
            const float4 t = c4[k];
            coef[4 * k] = t.x; coef[4 * k + 1] = t.y; coef[4 * k + 2] = t.z; coef[4 * k + 3] = t.w;
        }
    }
#pragma unroll
    for (u32 k = 0; k < STRIDE; ++k) gout[k] = 0.f;
    float gdx = 0.f, gdy = 0.f, gdz = 0.f;
#pragma unroll
    for (u32 ch = 0; ch < 3; ++ch) {
        float acc = 0.5f;
#pragma unroll
        for (u32 k = 0; k < NC; ++k) acc += Y[k] * coef[3 * k + ch];
        const float gch = acc > 0.f ? gcol[ch] : 0.f;       // clamped at 0: nothing passes
#pragma unroll
        for (u32 k = 0; k < NC; ++k) {
            const float ck = coef[3 * k + ch];
            gout[3 * k + ch] = Y[k] * gch;
            gdx += gch * ck * dYx[k]; gdy += gch * ck * dYy[k]; gdz += gch * ck * dYz[k];
        }
    }
    {
        float4 *o4 = reinterpret_cast<float4 *>(gsh);
#pragma unroll
        for (u32 k = 0; k < STRIDE / 4; ++k)
            o4[k] = make_float4(gout[4 * k], gout[4 * k + 1], gout[4 * k + 2], gout[4 * k + 3]);
    }
    const float dd = gdx * dxn + gdy * dyn + gdz * dzn;
    gm[0] += (gdx - dxn * dd) / len;
    gm[1] += (gdy - dyn * dd) / len;
    gm[2] += (gdz - dzn * dd) / len;
    g_mean[i] = gm[0]; g_mean[N + i] = gm[1]; g_mean[2 * N + i] = gm[2];
}

}  // namespace

hipError_t launch_preprocess_backward(const lmk_gs_gaussians &g, const ProjParams &pp,
                                      const lmk_gs_projected &proj, const float *grad_feat,
                                      const lmk_gs_gaussian_grads &out, hipStream_t stream)
{
    static const ShK shk = make_shk();
    if (g.n == 0) return hipSuccess;
    const u32 blocks = (g.n + 255u) / 256u;
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, stream,
                           g.mean, g.scale, g.rot, g.sh, g.n, pp, shk, proj.tiles_touched, grad_feat,
                           out.mean, out.scale, out.rot, out.opacity, out.sh);
    };
    switch (g.sh_degree) {
        case 0: launch(preprocess_backward_kernel<0>); break;
        case 1: launch(preprocess_backward_kernel<1>); break;
        case 2: launch(preprocess_backward_kernel<2>); break;
        default: launch(preprocess_backward_kernel<3>); break;
    }
    return hipGetLastError();
}

}  // namespace lmk
