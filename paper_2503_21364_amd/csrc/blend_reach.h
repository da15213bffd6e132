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

// log2(alpha_max) >= log2(1/255) - margin passes the block test, i.e. alpha down to 0.99990/255
constexpr float kBlockPass = -7.994353436858858f - 1.5e-4f;

}  // namespace lmk
#endif
