// The block test shared by the compositing kernel and its gradient kernel: can a splat reach
// alpha >= 1/255 anywhere in a square block of pixels?  (The "intersection operations for each
// tile" of Sec. 4.2.1, applied inside the tile.)
#ifndef LMK_GS_BLEND_REACH_H
#define LMK_GS_BLEND_REACH_H
#include "lmk_gs_internal.h"

namespace lmk {

__device__ __forceinline__ float clamp_pm(float v, float h) { return __builtin_amdgcn_fmed3f(v, -h, h); }

// Upper bound, with the rounding margin folded in, of A' dx^2 + B' dx dy + C' dy^2 over the
// square [-half, half]^2 about a centre from which the splat centre lies at (xs, ys).
// t.x = -B'/(2A'), t.y = -B'/(2C').
__device__ __forceinline__ float square_reach(float xs, float ys, float Aq, float Bq, float Cq,
                                              float tx, float ty, float half)
{
    const float kRelMargin = -2e-6f;    // times (A' ex^2 + C' ey^2) <= 0: covers fp32 rounding of the test
    // candidate 1: x clamped into the square, best y on that vertical line
    const float ex1 = clamp_pm(xs, half) - xs;
    const float ey1 = clamp_pm(fmaf(ty, ex1, ys), half) - ys;
    const float m1 = fmaf(Aq * ex1, ex1, Cq * ey1 * ey1);
    const float p1 = fmaf(Bq * ex1, ey1, m1);
    // candidate 2: y clamped, best x on that horizontal line
    const float ey2 = clamp_pm(ys, half) - ys;
    const float ex2 = clamp_pm(fmaf(tx, ey2, xs), half) - xs;
    const float m2 = fmaf(Aq * ex2, ex2, Cq * ey2 * ey2);
    const float p2 = fmaf(Bq * ex2, ey2, m2);
    return fmaxf(fmaf(m1, kRelMargin, p1), fmaf(m2, kRelMargin, p2));
}

// ---- a list entry as the compositing kernels stage it in LDS, and its exponent at a pixel.
// log2(alpha) = lo - 0.5 log2(e) q with q = A dx^2 + 2 B dx dy + C dy^2 (Sec. 2.2 Eq. 10) is not
// evaluated term by term: for a long thin splat the three terms are thousands of times larger than
// their sum, and fp32 rounding of each would move alpha by 1e-3 of its value.  Completing the square,
//   q = A t^2 + (C - B^2 / A) dy^2,   t = dx + (B / A) dy,
// leaves two non-negative terms.  B / A is taken to twice fp32 precision while staging, so that
// C - B^2 / A keeps full relative accuracy however close the conic is to singular; at a pixel, t
// comes out of one fused multiply-add (one rounding, of t itself).
//   geo = { u - X0, v - Y0, A' = -0.5 log2(e) A, -B / A }
//   cop = { -0.5 log2(e) (C - B^2 / A), lo = log2(opacity), r, g }
//   tst = { B' = -log2(e) B, C' = -0.5 log2(e) C, b, -B / C }     (A', B', C', -B/A, -B/C feed square_reach)
struct StagedEntry { float4 geo, cop, tst; };

// a = { u, v, A, B }, b = { C, opacity, r, g } of the feature record; (X0, Y0) = the tile's reference point
__device__ __forceinline__ StagedEntry stage_entry(const float4 a, const float4 b, float blue, float X0, float Y0)
{
    const float kL2E = 1.4426950408889634f;
    const float A = a.z, B = a.w, C = b.x;
    const float r0 = B / A;
    const float r_hi = r0 + fmaf(-r0, A, B) / A;            // B / A to the last bit
    const float r_lo = fmaf(-r_hi, A, B) / A;               // and what fp32 cannot hold of it
    const float c2 = fmaf(-r_lo, B, fmaf(-r_hi, B, C));     // C - B^2 / A
    StagedEntry s;
    s.geo = make_float4(a.x - X0, a.y - Y0, -0.5f * kL2E * A, -r_hi);
    s.cop = make_float4(-0.5f * kL2E * c2, __log2f(b.y), b.z, b.w);
    s.tst = make_float4(-kL2E * B, -0.5f * kL2E * C, blue, -B / C);
    return s;
}

// log2(alpha) of a staged entry at the pixel from which its centre lies at (dx, dy)
__device__ __forceinline__ float log2_alpha(const float4 geo, const float4 cop, float dx, float dy)
{
    const float t = fmaf(-geo.w, dy, dx);
    return fmaf(geo.z * t, t, fmaf(cop.x * dy, dy, cop.y));
}

// log2(alpha_max) >= log2(1/255) - margin passes the block test, i.e. alpha down to 0.99990/255
constexpr float kBlockPass = -7.994353436858858f - 1.5e-4f;

}  // namespace lmk
#endif
