// Stage 3: per-tile front-to-back alpha compositing (Sec. 2.2 Eq. 9-10; the
// blend kernel whose share of render time Sec. 4.2.1 reports).
//
// One workgroup (4 wavefronts) per 16x16 tile; each wavefront owns a compact
// 8x8 pixel block, each group of 16 lanes a 4x4 sub-block of it, one pixel per
// lane.  The tile's sorted list is consumed in batches of 256 entries staged in
// LDS (each thread fetches one 48-byte feature record; the next batch's records
// are already in flight while the current batch is composited -- the software
// pipelining of Sec. 4.2.1).
//
// Per batch a wavefront works in three phases:
//  1. lane = entry.  64 entries at a time are tested against the wavefront's
//     pixel block: the maximum of the splat's exponent over the (continuous)
//     block is found in closed form -- the exponent is a concave quadratic, so
//     the maximum sits at the centre if that is inside, else on an edge facing
//     it -- and compared with the entry's threshold -log2(255 opacity), below
//     which alpha < 1/255 everywhere in the block.  This is the exact
//     splat/block intersection ("intersection operations for each tile",
//     Sec. 4.2.1) at 8x8 granularity, costing well under one vector instruction
//     per entry; LDS is read lane-distinct, not broadcast.  Survivors append
//     their LDS offsets, in list order, to a per-wavefront survivor list
//     (ballot + mbcnt ranks).
//  2. lane = survivor.  The same test against each of the four 4x4 sub-blocks,
//     64 survivors at a time, gives every 16-lane group its own survivor
//     list: a splat that reaches the 8x8 block touches on average only
//     about half of its sub-blocks, and the vector units -- the bound of this
//     kernel -- are spent on (pixel, splat) pairs that can contribute.
//  3. lane = pixel.  Each group walks its own list, four entries at a time: one
//     16-byte LDS read yields four record offsets, the four exponentials are
//     independent, the compositing updates follow in order under per-lane
//     select masks.  The loop runs to the longest of the four lists (shorter
//     ones read a null record) and has no data-dependent scalar control flow
//     (the scalar unit, shared by the CU's four SIMDs, was as loaded as the
//     vector units when survivors were walked with scalar bit scans).
// A wavefront whose 64 pixels have all stopped skips the rest (per-wavefront
// progress, Sec. 4.2.1); the tile leaves when all four have.  Bound by FP32
// VALU issue; HBM traffic is the 52 bytes per list entry of the gather.
#include "lmk_gs_internal.h"
#include "blend_reach.h"

namespace lmk {

constexpr u32 kBlendThreads = 256;
constexpr u32 kBatch = 256;
constexpr u32 kXcds = 8;     // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

constexpr u32 kSurv = 4;     // survivors evaluated together (independent exponentials in flight)

struct BlendParams {
    u32 width, height, tiles_x, num_tiles, tiles_per_xcd;
    float bg0, bg1, bg2;
};

struct Rec { float4 a, b, c; };

__device__ __forceinline__ Rec fetch_record(const u32 *__restrict__ vals, const float4 *__restrict__ feat,
                                            u64 pos, bool valid)
{
    Rec r;
    if (valid) {
        const u32 g = vals[pos];
        const float4 *f = feat + (size_t)g * (LMK_GS_FEAT_STRIDE / 4);
        r.a = f[0]; r.b = f[1]; r.c = f[2];
    } else {
        r.a = r.b = r.c = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    return r;
}

constexpr u32 kListLen = kBatch + 8;    // survivors of a batch plus null padding

__global__ __launch_bounds__(kBlendThreads) void blend_kernel(
    const u64 *__restrict__ tile_offsets, const u32 *__restrict__ tile_order,
    const u32 *__restrict__ vals, const float4 *__restrict__ feat, BlendParams bp,
    float *__restrict__ out_rgb, float *__restrict__ out_T)
{
    // The staged form of an entry (stage_entry): (du, dv) = splat centre relative to the centre of
    // block 0, the coefficients of log2(alpha) with the square completed, and what the block tests
    // read.  Slot kBatch is a null record that can never contribute.
    __shared__ float4 s_geo[kBatch + 1];    // du, dv, A', -B/A
    __shared__ float4 s_cop[kBatch + 1];    // -0.5 log2(e) (C - B^2/A), lo, r, g
    __shared__ float4 s_tst[kBatch + 1];    // B', C', b, -B/C
    // survivor lists hold the records' byte offsets inside s_geo / s_cop / s_tst (at most 4096)
    __shared__ __attribute__((aligned(16))) unsigned short s_list8[kBlendThreads / kWave][kListLen];
    __shared__ __attribute__((aligned(16))) unsigned short s_list4[kBlendThreads / kWave][4][kListLen];

    u32 tile;
    if (tile_order) {
        // tiles by descending list length: the longest lists start first, and consecutive
        // workgroup ids (dealt round-robin to the XCDs) spread them over all dies
        if (blockIdx.x >= bp.num_tiles) return;
        tile = tile_order[blockIdx.x];
        if (tile >= bp.num_tiles) return;          // never index past the grid on a corrupt hint
    } else {
        // consecutive workgroup ids land on different XCDs; give each XCD one
        // contiguous band of tiles so neighbouring tiles share that XCD's L2
        tile = (blockIdx.x % kXcds) * bp.tiles_per_xcd + blockIdx.x / kXcds;
        if (blockIdx.x / kXcds >= bp.tiles_per_xcd || tile >= bp.num_tiles) return;
    }

    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 grp = lane >> 4, gl = lane & 15u;                // 4x4 sub-block of the lane, pixel inside it
    const u32 tx = tile % bp.tiles_x, ty = tile / bp.tiles_x;
    const u32 bi = (grp & 1u) * 4u + (gl & 3u), bj = (grp >> 1) * 4u + (gl >> 2);   // pixel inside the 8x8 block
    const u32 pxi = tx * LMK_GS_TILE + (wv & 1u) * 8u + bi, pyi = ty * LMK_GS_TILE + (wv >> 1) * 8u + bj;
    const bool inside = pxi < bp.width && pyi < bp.height;
    // this wavefront's block centre relative to block 0's, and this lane's pixel centre
    const float bx = (float)((wv & 1u) * 8u), by = (float)((wv >> 1) * 8u);
    const float ox = bx + ((float)bi - 3.5f), oy = by + ((float)bj - 3.5f);
    const float X0 = (float)(tx * LMK_GS_TILE) + 4.0f, Y0 = (float)(ty * LMK_GS_TILE) + 4.0f;
    const float kHalf8 = 3.5f;          // pixel centres of a block span [-3.5, 3.5]^2 about its centre
    const float kHalf4 = 1.5f;          // and those of a sub-block [-1.5, 1.5]^2

    const u64 start = tile_offsets[tile], end = tile_offsets[tile + 1];
    float T = 1.0f, cr = 0.0f, cg = 0.0f, cb = 0.0f;
    bool done = !inside;
    const float kPass = kBlockPass;
    constexpr u32 kNullOfs = kBatch * 16u;

    if (tid == 0) {
        s_geo[kBatch] = make_float4(0.f, 0.f, 0.f, 0.f);
        s_cop[kBatch] = make_float4(0.f, -1000.0f, 0.f, 0.f);
        s_tst[kBatch] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    Rec next = fetch_record(vals, feat, start + tid, start + tid < end);

    for (u64 base = start; base < end; base += kBatch) {
        if (__syncthreads_and(done)) break;        // also: everyone is past the previous batch
        const u32 cnt = (u32)((end - base) < (u64)kBatch ? (end - base) : (u64)kBatch);
        {
            // every thread stages one slot; slots past the end of the list can never pass a test
            const bool valid = tid < cnt;
            const StagedEntry se = stage_entry(next.a, next.b, next.c.x, X0, Y0);
            s_geo[tid] = valid ? se.geo : make_float4(0.f, 0.f, 0.f, 0.f);
            s_cop[tid] = valid ? se.cop : make_float4(0.f, -1000.0f, 0.f, 0.f);
            s_tst[tid] = valid ? se.tst : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        __syncthreads();
        {
            const u64 npos = base + kBatch + tid;
            next = fetch_record(vals, feat, npos, npos < end);    // in flight during the loops below
        }
        const u64 alive = __builtin_amdgcn_ballot_w64(!done);
        if (alive == 0ull) continue;                               // this wavefront is finished

        // ---- phase 1: lane = entry; which splats reach this wavefront's block at all?
        u32 n8 = 0;
        for (u32 c0 = 0; c0 < cnt; c0 += kWave) {
            const float4 g = s_geo[c0 + lane];
            const float4 t = s_tst[c0 + lane];
            const float4 co = s_cop[c0 + lane];
            const float xs = g.x - bx, ys = g.y - by;
            const float best = square_reach(xs, ys, g.z, t.x, t.y, g.w, t.w, kHalf8);
            const bool pass = best + co.y >= kPass;
            const u64 mask = __builtin_amdgcn_ballot_w64(pass);
            const u32 rank = __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
            if (pass) s_list8[wv][n8 + rank] = (unsigned short)((c0 + lane) * 16u);
            n8 += (u32)__builtin_popcountll(mask);
        }

        // ---- phase 2: lane = survivor; 64 survivors at a time against the four 4x4 sub-blocks,
        // one list per sub-block; a sub-block whose pixels have all stopped takes nothing more.
        u32 n4[4] = { 0u, 0u, 0u, 0u };
        for (u32 k0 = 0; k0 < n8; k0 += kWave) {
            const u32 k = k0 + lane;
            const u32 ofs = k < n8 ? (u32)s_list8[wv][k] : kNullOfs;   // the null record never passes
            const float4 g = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(s_geo) + ofs);
            const float4 t = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(s_tst) + ofs);
            const float4 co = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(s_cop) + ofs);
            const float xs = g.x - bx, ys = g.y - by;
#pragma unroll
            for (u32 q = 0; q < 4; ++q) {
                const float qx = (q & 1u) ? 2.0f : -2.0f, qy = (q >> 1) ? 2.0f : -2.0f;
                const float best = square_reach(xs - qx, ys - qy, g.z, t.x, t.y, g.w, t.w, kHalf4);
                const bool sub_alive = ((alive >> (16u * q)) & 0xffffull) != 0ull;
                const bool pass = sub_alive && best + co.y >= kPass;
                const u64 mask = __builtin_amdgcn_ballot_w64(pass);
                const u32 rank = __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
                if (pass) s_list4[wv][q][n4[q] + rank] = (unsigned short)ofs;
                n4[q] += (u32)__builtin_popcountll(mask);
            }
        }
        const u32 n_mine = grp == 0u ? n4[0] : (grp == 1u ? n4[1] : (grp == 2u ? n4[2] : n4[3]));
        const u32 l01 = n4[0] > n4[1] ? n4[0] : n4[1], l23 = n4[2] > n4[3] ? n4[2] : n4[3];
        const u32 longest = l01 > l23 ? l01 : l23;
        unsigned short *my_list = s_list4[wv][grp];
        // null records behind every list: a group past its own end keeps reading these
        if (gl < 8u) my_list[n_mine + gl] = (unsigned short)kNullOfs;
        const u32 n4_pad = (n_mine + kSurv - 1u) & ~(kSurv - 1u);

        // ---- phase 3: lane = pixel; composite the group's survivors in list order, kSurv at a time
        for (u32 k = 0; k < longest; k += kSurv) {
            const uint2 ofs4 = *reinterpret_cast<const uint2 *>(my_list + (k < n4_pad ? k : n4_pad));
            const u32 ofs[kSurv] = { ofs4.x & 0xffffu, ofs4.x >> 16, ofs4.y & 0xffffu, ofs4.y >> 16 };
            float alpha[kSurv];
            float4 co[kSurv];
#pragma unroll
            for (u32 q = 0; q < kSurv; ++q) {
                const float4 g = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(s_geo) + ofs[q]);
                co[q] = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(s_cop) + ofs[q]);
                const float dx = g.x - ox, dy = g.y - oy;
                alpha[q] = fminf(0.99f, __builtin_amdgcn_exp2f(log2_alpha(g, co[q], dx, dy)));
            }
#pragma unroll
            for (u32 q = 0; q < kSurv; ++q) {
                const float blue = reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(s_tst) + ofs[q])->z;
                const float Tn = fmaf(-T, alpha[q], T);
                const bool hit = !(alpha[q] < 1.0f / 255.0f) && !done;
                const bool stop = hit && Tn < 1e-4f;
                const bool upd = hit && !stop;
                const float w = upd ? alpha[q] * T : 0.0f;
                cr = fmaf(co[q].z, w, cr); cg = fmaf(co[q].w, w, cg); cb = fmaf(blue, w, cb);
                T = upd ? Tn : T;
                done = done || stop;
            }
            if (__builtin_amdgcn_ballot_w64(!done) == 0ull) break;     // all 64 pixels stopped
        }
    }
    if (inside) {
        const size_t plane = (size_t)bp.width * bp.height;
        const size_t p = (size_t)pyi * bp.width + pxi;
        out_rgb[p] = cr + T * bp.bg0;
        out_rgb[plane + p] = cg + T * bp.bg1;
        out_rgb[2 * plane + p] = cb + T * bp.bg2;
        out_T[p] = T;
    }
}

hipError_t launch_render(const lmk_gs_projected &proj, const lmk_gs_binned &binned, const ProjParams &pp,
                         float *out_rgb, float *out_T, hipStream_t stream)
{
    BlendParams bp;
    bp.width = pp.cam.width; bp.height = pp.cam.height;
    bp.tiles_x = pp.tiles_x; bp.num_tiles = pp.tiles_x * pp.tiles_y;
    bp.tiles_per_xcd = (bp.num_tiles + kXcds - 1) / kXcds;
    bp.bg0 = pp.cam.bg[0]; bp.bg1 = pp.cam.bg[1]; bp.bg2 = pp.cam.bg[2];
    hipLaunchKernelGGL(blend_kernel, dim3(bp.tiles_per_xcd * kXcds), dim3(kBlendThreads), 0, stream,
                       binned.tile_offsets, binned.tile_order, binned.vals,
                       reinterpret_cast<const float4 *>(proj.feat), bp, out_rgb, out_T);
    return hipGetLastError();
}

}  // namespace lmk
