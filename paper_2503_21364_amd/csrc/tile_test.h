// Binning rule 1 (lmk_gs_camera.binning == 1; the per-tile intersection test of Sec. 4.2.1): can
// the splat reach alpha >= 1/255 on the square spanned by a tile's pixel centres?
// q(d) = d^T conic d is convex: its minimum over the square is at the splat centre if that is
// inside, else on an edge facing it (clamp one coordinate, minimise along that line; two
// candidates cover all cases).  Contributing needs q <= 2 ln(255 o); tau bounds that from above
// from the exponent and the top three mantissa bits of o (table from the host), so no run-time
// logarithm decides an integer.  Every translation unit that includes this header is compiled
// without floating-point contraction and with correctly rounded division: the projection kernel
// counts the kept tiles, the binning kernels enumerate them, and both must take every decision
// alike (and like the CPU definition of the rule, which runs the same fp32 operation sequence).
#ifndef LMK_GS_TILE_TEST_H
#define LMK_GS_TILE_TEST_H
#include "lmk_gs_internal.h"

namespace lmk {

struct TileTest { float u, v, A, B, C, rx, ry, tau; };

__device__ __forceinline__ float opacity_tau(const ProjParams &pp, float o)
{
    const u32 bits = __float_as_uint(o);
    const int E = (int)((bits >> 23) & 0xffu) - 127;
    return pp.tau_tab[(bits >> 20) & 7u] + (float)E * 1.3862944f;
}

__device__ __forceinline__ TileTest make_tile_test(float u, float v, float A, float B, float C, float tau)
{
    TileTest t;
    t.u = u; t.v = v; t.A = A; t.B = B; t.C = C; t.tau = tau;
    t.rx = -B / A; t.ry = -B / C;
    return t;
}

__device__ __forceinline__ float clampf3(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

__device__ __forceinline__ float quad_adj(const TileTest &t, float ex, float ey)
{
    const float m = t.A * ex * ex + t.C * ey * ey;
    const float q = m + 2.0f * t.B * ex * ey;
    return q - 4e-6f * m;
}

__device__ __forceinline__ bool tile_kept(const TileTest &t, u32 tx, u32 ty)
{
    const float h = 0.5f * (float)LMK_GS_TILE - 0.5f;
    const float xs = t.u - ((float)(tx * LMK_GS_TILE) + 0.5f * (float)LMK_GS_TILE);
    const float ys = t.v - ((float)(ty * LMK_GS_TILE) + 0.5f * (float)LMK_GS_TILE);
    const float ex1 = clampf3(xs, -h, h) - xs;
    const float ey1 = clampf3(ys + t.ry * ex1, -h, h) - ys;
    const float ey2 = clampf3(ys, -h, h) - ys;
    const float ex2 = clampf3(xs + t.rx * ey2, -h, h) - xs;
    const float q1 = quad_adj(t, ex1, ey1);
    const float q2 = quad_adj(t, ex2, ey2);
    const float qmin = q1 < q2 ? q1 : q2;
    return qmin <= t.tau;
}

}  // namespace lmk
#endif
