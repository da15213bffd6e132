// Gradient of a scalar loss through the compositing of stage 3 (Sec. 2.2 Eq. 9-10; the text
// after them: the rasteriser is differentiable and every parameter of the primitives is
// optimised through the rendering process).
//
// For a pixel whose walk composited the entries i = 1..m (T_1 = 1, T_{i+1} = T_i (1 - a_i),
// w_i = a_i T_i, C = sum c_i w_i + bg T_{m+1}), with S_i = sum_{j>i} c_j w_j + bg T_{m+1}:
//   dL/dc_i = w_i dL/dC
//   dL/da_i = dL/dC . (T_i c_i - S_i / (1 - a_i)) - dL/dT_end T_end / (1 - a_i)
//   a = o exp(-q/2), q = A dx^2 + 2 B dx dy + C dy^2:  da/do = a / o, da/dq = -a / 2
// The thresholds of the walk are constants of the derivative: skipped entries, the entry that
// stops the walk and everything behind it get nothing; where a was clamped to 0.99 it depends
// on neither o nor q.
//
// One workgroup per 16x16 tile, one thread per pixel, each wavefront an 8x8 block.  Entries are
// staged in LDS in batches of 256.  Per batch every wavefront first tests, one entry per lane,
// which entries can reach alpha >= 1/255 anywhere in its block (the block test of blend_kernel)
// and keeps their slots in a list; its pixels then only walk that list.  Pass 1 repeats the
// forward walk with the arithmetic of blend_kernel (same expression for log2(alpha), same
// comparisons), which gives every pixel its final transmittance and the position of its last
// composited entry.  Pass 2 takes the batches, and each list, back to front: T_i is recovered as
// T_{i+1} / (1 - a_i), S_i is a running sum.  What is summed over the pixels of an entry are not the
// nine gradient components themselves but nine moments from which they follow linearly, with
// m = a dL/da (0 where a was clamped): sum m dx, sum m dy, sum m dx^2, sum m dx dy, sum m dy^2,
// sum m, and sum w dL/dC per channel; the per-entry factors (A, B, C, 1 / opacity) are applied once
// per (tile, entry) when the sums leave the workgroup.  A pixel without a contribution adds zeros,
// so the arithmetic has no branches.  The sums go over the 4 lanes of a quad with DPP adds, over
// the quads and rows of the tile with LDS float atomics, and leave the workgroup as one global
// float atomic per (entry, component): the order of these additions is not fixed, so results
// differ from run to run by fp32 rounding.
//
// Bound by vector-instruction issue (the exponent evaluation of the forward pass, twice, the
// gradient arithmetic and the reductions); HBM traffic is the forward's gather, twice, plus 36
// bytes of atomics per pair.
#include "lmk_gs_internal.h"
#include "blend_reach.h"

namespace lmk {

namespace {

constexpr u32 kBwdThreads = 256, kBwdBatch = 256;
constexpr u32 kBwdWaves = kBwdThreads / kWave;
typedef unsigned char slot_t;               // a slot of the staged batch (kBwdBatch <= 256)
static_assert(kBwdBatch <= 256 && (kBwdBatch & (kBwdBatch - 1)) == 0, "slots are bytes and masked");
static_assert(kBwdBatch <= kBwdThreads, "one thread stages one entry");
constexpr u32 kGradComps = 9;               // u, v, A, B, C, opacity, r, g, b

struct BwdParams {
    u32 width, height, tiles_x, num_tiles;
    float bg0, bg1, bg2;
};

// sum over the 16 lanes of a row, returned in every lane of the row
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// Sums over the 16 lanes of a row, transposed on the way: lane k of every quad ends with the
// row's sums of components k and 4 + k (sA, sB); component 8 ends in every lane (sC).  A step
// pairs two components: the even side of the exchange keeps the first and hands over the second,
// the odd side the other way round, so every step halves the registers in play.
__device__ __forceinline__ void row_sums_transposed(const float (&v)[kGradComps], bool odd, bool upper,
                                                     float &sA, float &sB, float &sC)
{
    float r[4];
#pragma unroll
    for (u32 c = 0; c < 4; ++c) {                                  // lane xor 1: components (2c, 2c + 1)
        const float keep = odd ? v[2 * c + 1] : v[2 * c], send = odd ? v[2 * c] : v[2 * c + 1];
        r[c] = keep + dpp_f<0xB1>(send);                           // quad_perm [1,0,3,2]
    }
    const float r8 = v[8] + dpp_f<0xB1>(v[8]);
    {                                                              // lane xor 2: (r0, r1) and (r2, r3)
        const float keepA = upper ? r[1] : r[0], sendA = upper ? r[0] : r[1];
        const float keepB = upper ? r[3] : r[2], sendB = upper ? r[2] : r[3];
        sA = keepA + dpp_f<0x4E>(sendA);                           // quad_perm [2,3,0,1]
        sB = keepB + dpp_f<0x4E>(sendB);
    }
    sC = r8 + dpp_f<0x4E>(r8);
    // ... and over the four quads of the row (rotations by one and two quads keep a lane's place in its quad)
    sA += dpp_f<0x124>(sA); sB += dpp_f<0x124>(sB); sC += dpp_f<0x124>(sC);      // row_ror:4
    sA += dpp_f<0x128>(sA); sB += dpp_f<0x128>(sB); sC += dpp_f<0x128>(sC);      // row_ror:8
}

// one list entry on its way from the feature records to LDS: fetched a batch ahead, so that the two
// dependent reads (index, then record) are in flight while the previous batch is walked
struct Fetched { float4 a, b; float blue; u32 id; };
__device__ __forceinline__ Fetched fetch_entry(const u32 *__restrict__ vals, const float4 *__restrict__ feat,
                                               u64 pos, bool valid)
{
    Fetched r;
    r.a = r.b = make_float4(0.f, 0.f, 0.f, 0.f); r.blue = 0.0f; r.id = 0u;
    if (valid) {
        r.id = vals[pos];
        const float4 *f = feat + (size_t)r.id * (LMK_GS_FEAT_STRIDE / 4);
        r.a = f[0]; r.b = f[1]; r.blue = f[2].x;
    }
    return r;
}

// the survivors of one batch for one wavefront: slots of the entries that pass the block test
__device__ __forceinline__ u32 block_survivors(const float4 *s_geo, const float4 *s_cop, const float4 *s_tst,
                                               u32 cnt, float bx, float by, u32 lane, slot_t *list)
{
    u32 n8 = 0;
    for (u32 c0 = 0; c0 < cnt; c0 += kWave) {
        const u32 e = c0 + lane;
        const float4 g = s_geo[e < cnt ? e : 0u];
        const float4 t = s_tst[e < cnt ? e : 0u];
        const float4 co = s_cop[e < cnt ? e : 0u];
        const float best = square_reach(g.x - bx, g.y - by, g.z, t.x, t.y, g.w, t.w, 3.5f);
        const bool pass = e < cnt && best + co.y >= kBlockPass;
        const u64 mask = __builtin_amdgcn_ballot_w64(pass);
        const u32 rank = __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
        if (pass) list[n8 + rank] = (slot_t)e;
        n8 += (u32)__builtin_popcountll(mask);
    }
    return n8;
}

// ... and of those, per 4x4 sub-block (the 16 lanes of a row), the ones that can reach it: one
// survivor per lane, tested against the four sub-blocks; list order is kept
__device__ __forceinline__ void subblock_survivors(const float4 *s_geo, const float4 *s_cop, const float4 *s_tst,
                                                   const slot_t *list8, u32 n8, float bx, float by, u32 lane,
                                                   slot_t (*list4)[kBwdBatch], u32 (&n4)[4], const u32 (&limit)[4])
{
    n4[0] = n4[1] = n4[2] = n4[3] = 0u;
    for (u32 k0 = 0; k0 < n8; k0 += kWave) {
        const u32 k = k0 + lane;
        const bool valid = k < n8;
        const u32 e = valid ? (u32)list8[k] : 0u;
        const float4 g = s_geo[e];
        const float4 t = s_tst[e];
        const float4 co = s_cop[e];
        const float xs = g.x - bx, ys = g.y - by;
#pragma unroll
        for (u32 q = 0; q < 4; ++q) {
            const float qx = (q & 1u) ? 2.0f : -2.0f, qy = (q >> 1) ? 2.0f : -2.0f;
            const float best = square_reach(xs - qx, ys - qy, g.z, t.x, t.y, g.w, t.w, 1.5f);
            // limit[q]: slots from there on lie behind the last composited entry of every pixel of the sub-block
            const bool pass = valid && e < limit[q] && best + co.y >= kBlockPass;
            const u64 mask = __builtin_amdgcn_ballot_w64(pass);
            const u32 rank = __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
            if (pass) list4[q][n4[q] + rank] = (slot_t)e;
            n4[q] += (u32)__builtin_popcountll(mask);
        }
    }
}

__global__ __launch_bounds__(kBwdThreads) void blend_backward_kernel(
    const u64 *__restrict__ tile_offsets, const u32 *__restrict__ tile_order, const u32 *__restrict__ vals,
    const float4 *__restrict__ feat, BwdParams bp, const float *__restrict__ grad_rgb,
    const float *__restrict__ grad_T, float *__restrict__ grad_feat)
{
    // the staged form of blend_kernel (stage_entry), so that log2(alpha) is evaluated exactly as there
    __shared__ float4 s_geo[kBwdBatch];          // du, dv, A', -B/A
    __shared__ float4 s_cop[kBwdBatch];          // -0.5 log2(e) (C - B^2/A), lo, r, g
    __shared__ float4 s_tst[kBwdBatch];          // B', C', b, -B/C
    __shared__ u32 s_id[kBwdBatch];              // primitive index
    // double precision: the LDS adds a double in a fraction of the time it takes for a float (measured on
    // this chip: 0.3 against 3 cycles per lane), and the sums of a tile lose nothing on the way
    __shared__ double s_acc[kBwdBatch][kGradComps];
    __shared__ slot_t s_list[kBwdWaves][kBwdBatch];
    __shared__ slot_t s_list4[kBwdWaves][4][kBwdBatch];
    __shared__ u32 s_last[kBwdWaves];

    if (blockIdx.x >= bp.num_tiles) return;
    // the tiles with the longest lists first, when the caller has the hint
    const u32 tile = tile_order ? tile_order[blockIdx.x] : blockIdx.x;
    if (tile >= bp.num_tiles) return;
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 tx = tile % bp.tiles_x, ty = tile / bp.tiles_x;
    const u32 grp = lane >> 4, gl = lane & 15u;                    // 4x4 sub-block of the lane, pixel inside it
    const u32 bi = (grp & 1u) * 4u + (gl & 3u), bj = (grp >> 1) * 4u + (gl >> 2);   // pixel inside the 8x8 block
    const u32 pxi = tx * LMK_GS_TILE + (wv & 1u) * 8u + bi, pyi = ty * LMK_GS_TILE + (wv >> 1) * 8u + bj;
    const bool inside = pxi < bp.width && pyi < bp.height;
    // (X0, Y0) = centre of block 0, the reference point of blend_kernel; this block's centre and this
    // lane's pixel centre relative to it
    const float bx = (float)((wv & 1u) * 8u), by = (float)((wv >> 1) * 8u);
    const float ox = bx + ((float)bi - 3.5f), oy = by + ((float)bj - 3.5f);
    const float X0 = (float)(tx * LMK_GS_TILE) + 4.0f, Y0 = (float)(ty * LMK_GS_TILE) + 4.0f;
    const u64 start = tile_offsets[tile], end = tile_offsets[tile + 1];
    const u64 len64 = end - start;
    const u32 len = len64 < 0xffffff00ull ? (u32)len64 : 0xffffff00u;     // a tile's list is far shorter
    slot_t *my_list = s_list[wv];
    const slot_t *my_list4 = s_list4[wv][grp];

    // ---- pass 1: the forward walk
    float T = 1.0f;
    u32 last = 0;                       // entries of the list up to and including the last composited one
    bool done = !inside;
    Fetched next = fetch_entry(vals, feat, start + tid, tid < kBwdBatch && tid < len);
    for (u32 base = 0; base < len; base += kBwdBatch) {
        if (__syncthreads_and(done)) break;        // also: everyone is past the previous batch
        const u32 cnt = len - base < kBwdBatch ? len - base : kBwdBatch;
        if (tid < cnt) {
            const StagedEntry se = stage_entry(next.a, next.b, 0.0f, X0, Y0);
            s_geo[tid] = se.geo; s_cop[tid] = se.cop; s_tst[tid] = se.tst;
        }
        __syncthreads();
        next = fetch_entry(vals, feat, start + base + kBwdBatch + tid, tid < kBwdBatch && base + kBwdBatch + tid < len);
        if (__builtin_amdgcn_ballot_w64(!done) == 0ull) continue;     // this wavefront is finished
        const u32 n8 = block_survivors(s_geo, s_cop, s_tst, cnt, bx, by, lane, my_list);
        u32 n4[4];
        const u32 no_limit[4] = { kBwdBatch, kBwdBatch, kBwdBatch, kBwdBatch };
        subblock_survivors(s_geo, s_cop, s_tst, my_list, n8, bx, by, lane, s_list4[wv], n4, no_limit);
        const u32 n_mine = grp == 0u ? n4[0] : (grp == 1u ? n4[1] : (grp == 2u ? n4[2] : n4[3]));
        const u32 l01 = n4[0] > n4[1] ? n4[0] : n4[1], l23 = n4[2] > n4[3] ? n4[2] : n4[3];
        const u32 longest = l01 > l23 ? l01 : l23;
        for (u32 k = 0; k < longest; ++k) {
            const bool in_list = k < n_mine;
            const u32 j = (u32)my_list4[in_list ? k : 0u] & (kBwdBatch - 1u);
            const float4 g = s_geo[j];
            const float4 co = s_cop[j];
            const float dx = g.x - ox, dy = g.y - oy;
            const float alpha = fminf(0.99f, __builtin_amdgcn_exp2f(log2_alpha(g, co, dx, dy)));
            const float Tn = fmaf(-T, alpha, T);
            const bool hit = in_list && !done && !(alpha < 1.0f / 255.0f);
            const bool stop = hit && Tn < 1e-4f;
            if (hit && !stop) { T = Tn; last = base + j + 1u; }
            done = done || stop;
            if (__builtin_amdgcn_ballot_w64(!done) == 0ull) break;     // all 64 pixels stopped
        }
    }
    const float T_end = T;

    // the longest walk of each sub-block, of each wavefront and of the tile bound pass 2
    u32 wl = last;
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) {
        const u32 t = (u32)__shfl_xor((int)wl, o, 64);
        wl = t > wl ? t : wl;
    }
    const u32 sub_last[4] = { (u32)__builtin_amdgcn_readlane((int)wl, 0), (u32)__builtin_amdgcn_readlane((int)wl, 16),
                              (u32)__builtin_amdgcn_readlane((int)wl, 32), (u32)__builtin_amdgcn_readlane((int)wl, 48) };
#pragma unroll
    for (int o = 32; o >= 16; o >>= 1) {
        const u32 t = (u32)__shfl_xor((int)wl, o, 64);
        wl = t > wl ? t : wl;
    }
    __syncthreads();                    // pass 1 is over in every wavefront: LDS is free
    if (lane == 0) s_last[wv] = wl;
    __syncthreads();
    u32 max_last = 0;
#pragma unroll
    for (u32 k = 0; k < kBwdWaves; ++k) max_last = s_last[k] > max_last ? s_last[k] : max_last;
    if (max_last == 0) return;

    // ---- pass 2: back to front
    const size_t plane = (size_t)bp.width * bp.height;
    const size_t pix = (size_t)pyi * bp.width + pxi;
    const float gr = inside ? grad_rgb[pix] : 0.0f;
    const float gg = inside ? grad_rgb[plane + pix] : 0.0f;
    const float gb = inside ? grad_rgb[2 * plane + pix] : 0.0f;
    const float gT = (inside && grad_T) ? grad_T[pix] : 0.0f;
    const float gT_end = gT * T_end;
    float Sr = bp.bg0 * T_end, Sg = bp.bg1 * T_end, Sb = bp.bg2 * T_end;
    T = T_end;
    const u32 batches = (max_last + kBwdBatch - 1) / kBwdBatch;
    next = fetch_entry(vals, feat, start + (batches - 1u) * kBwdBatch + tid,
                       tid < kBwdBatch && (batches - 1u) * kBwdBatch + tid < max_last);
    for (u32 b = batches; b-- > 0;) {
        const u32 base = b * kBwdBatch;
        const u32 cnt = max_last - base < kBwdBatch ? max_last - base : kBwdBatch;
        __syncthreads();                // the previous batch has been flushed
        if (tid < cnt) {
            const StagedEntry se = stage_entry(next.a, next.b, next.blue, X0, Y0);
            s_geo[tid] = se.geo; s_cop[tid] = se.cop; s_tst[tid] = se.tst;
            s_id[tid] = next.id;
        }
        // the batch in front of this one (all of its slots lie below max_last)
        next = fetch_entry(vals, feat, start + base - kBwdBatch + tid, b > 0u && tid < kBwdBatch);
        for (u32 k = tid; k < kBwdBatch * kGradComps; k += kBwdThreads) (&s_acc[0][0])[k] = 0.0;
        __syncthreads();
        // a wavefront none of whose pixels walked this far has nothing to add (it still takes part
        // in the barriers and the flush below)
        const u32 n8 = base < wl ? block_survivors(s_geo, s_cop, s_tst, cnt, bx, by, lane, my_list) : 0u;
        u32 n4[4];
        u32 limit[4];
#pragma unroll
        for (u32 q = 0; q < 4; ++q) limit[q] = sub_last[q] > base ? sub_last[q] - base : 0u;
        subblock_survivors(s_geo, s_cop, s_tst, my_list, n8, bx, by, lane, s_list4[wv], n4, limit);
        const u32 n_mine = grp == 0u ? n4[0] : (grp == 1u ? n4[1] : (grp == 2u ? n4[2] : n4[3]));
        const u32 l01 = n4[0] > n4[1] ? n4[0] : n4[1], l23 = n4[2] > n4[3] ? n4[2] : n4[3];
        const u32 longest = l01 > l23 ? l01 : l23;
        for (u32 k = longest; k-- > 0;) {
            const bool in_list = k < n_mine;
            const u32 j = (u32)my_list4[in_list ? k : 0u] & (kBwdBatch - 1u);    // the same for the 16 lanes of a row
            const float4 g = s_geo[j];
            const float4 co = s_cop[j];
            const float dx = g.x - ox, dy = g.y - oy;
            const float raw = __builtin_amdgcn_exp2f(log2_alpha(g, co, dx, dy));
            const float alpha = fminf(0.99f, raw);
            const bool hit = in_list && base + j < last && !(alpha < 1.0f / 255.0f);
            const u64 hits = __builtin_amdgcn_ballot_w64(hit);
            if (hits == 0ull) continue;                                  // nothing from this wavefront
            // a pixel without a contribution goes through the same arithmetic with a = 0: T and S
            // stay as they are and all nine moments are zero
            const float a = hit ? alpha : 0.0f;
            const float blue = s_tst[j].z;
            const float inv = __builtin_amdgcn_rcpf(1.0f - a);     // 1 - a >= 0.01; one ulp is enough here
            // dL/da = (dL/dC . (T c - S) - dL/dT_end T_end) / (1 - a), T = transmittance behind the entry
            const float num = fmaf(gr, fmaf(T, co.z, -Sr), fmaf(gg, fmaf(T, co.w, -Sg), fmaf(gb, fmaf(T, blue, -Sb), -gT_end)));
            T *= inv;                                              // transmittance in front of this entry
            const float w = a * T;
            Sr = fmaf(co.z, w, Sr); Sg = fmaf(co.w, w, Sg); Sb = fmaf(blue, w, Sb);
            const float m = (raw > 0.99f ? 0.0f : a) * (num * inv);     // a dL/da; a clamped alpha depends on nothing
            float v[kGradComps];
            v[0] = m * dx; v[1] = m * dy;
            v[2] = v[0] * dx; v[3] = v[0] * dy; v[4] = v[1] * dy;
            v[5] = m;
            v[6] = w * gr; v[7] = w * gg; v[8] = w * gb;
            // over the row in registers, over the rows of the tile in LDS: the first quad of every row
            // that had a contribution adds, each lane the two components it ended up with
            float sA, sB, sC;
            row_sums_transposed(v, (lane & 1u) != 0u, (lane & 2u) != 0u, sA, sB, sC);
            const bool row_hit = ((hits >> (lane & 48u)) & 0xffffull) != 0ull;
            if (row_hit && (lane & 12u) == 0u) {
                double *rec = s_acc[j];
                atomicAdd(rec + (lane & 3u), (double)sA);
                atomicAdd(rec + 4u + (lane & 3u), (double)sB);
                if ((lane & 3u) == 0u) atomicAdd(rec + 8u, (double)sC);
            }
        }
        __syncthreads();
        // from the moments of an entry to its gradient: q = A dx^2 + 2 B dx dy + C dy^2, da/dq = -a / 2,
        // da/do = a / o; the staged A' = -0.5 log2(e) A, B' = -log2(e) B, C' = -0.5 log2(e) C give
        // d/du = ln 2 (2 A' sum m dx + B' sum m dy), d/dv = ln 2 (B' sum m dx + 2 C' sum m dy).
        // Consecutive lanes take the consecutive components of an entry, so that the atomics of one
        // instruction fall into few cache lines (nine lanes per 36-byte record)
        for (u32 idx = tid; idx < cnt * kGradComps; idx += kBwdThreads) {
            const u32 e = idx / kGradComps, c = idx - e * kGradComps;
            const float kLn2 = 0.6931471805599453f;
            float v = (float)s_acc[e][c];
            if (c < 2u) {
                const float mx = (float)s_acc[e][0], my = (float)s_acc[e][1];
                const float Aq = s_geo[e].z, Bq = s_tst[e].x, Cq = s_tst[e].y;
                v = c == 0u ? kLn2 * fmaf(2.0f * Aq, mx, Bq * my) : kLn2 * fmaf(Bq, mx, 2.0f * Cq * my);
            } else if (c == 2u || c == 4u) {
                v *= -0.5f;
            } else if (c == 3u) {
                v = -v;
            } else if (c == 5u) {
                v *= __builtin_amdgcn_exp2f(-s_cop[e].y);       // 1 / opacity
            }
            if (v != 0.0f) atomicAdd(grad_feat + (size_t)s_id[e] * LMK_GS_FEAT_STRIDE + c, v);
        }
    }
}

__global__ __launch_bounds__(256) void zero_kernel(float4 *__restrict__ p, size_t count4)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count4; i += stride)
        p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

}  // namespace

hipError_t launch_render_backward(const lmk_gs_projected &proj, u32 n, const lmk_gs_binned &binned,
                                  const ProjParams &pp, const float *grad_rgb, const float *grad_T,
                                  float *grad_feat, hipStream_t stream)
{
    // a fill kernel, not a memset node: the call may be captured into a graph
    const size_t count4 = (size_t)n * (LMK_GS_FEAT_STRIDE / 4);
    if (count4 > 0) {
        const size_t blocks = (count4 + 255) / 256;
        hipLaunchKernelGGL(zero_kernel, dim3((u32)(blocks < 8192 ? blocks : 8192)), dim3(256), 0, stream,
                           reinterpret_cast<float4 *>(grad_feat), count4);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    BwdParams bp;
    bp.width = pp.cam.width; bp.height = pp.cam.height;
    bp.tiles_x = pp.tiles_x; bp.num_tiles = pp.tiles_x * pp.tiles_y;
    bp.bg0 = pp.cam.bg[0]; bp.bg1 = pp.cam.bg[1]; bp.bg2 = pp.cam.bg[2];
    if (n == 0 || binned.capacity == 0) return hipSuccess;
    hipLaunchKernelGGL(blend_backward_kernel, dim3(bp.num_tiles), dim3(kBwdThreads), 0, stream,
                       binned.tile_offsets, binned.tile_order, binned.vals,
                       reinterpret_cast<const float4 *>(proj.feat), bp, grad_rgb, grad_T, grad_feat);
    return hipGetLastError();
}

}  // namespace lmk
