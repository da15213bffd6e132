// Stage 2: duplication of primitives into (tile | depth) keys, sort of the pairs into
// (tile, depth bits, index) order, per-tile range extraction (the "depth sorting ... at the
// granularity of tiles" of Sec. 2.2; duplication with keys is the second kernel named in
// Sec. 4.2.1).
//
// Integer work bound by HBM traffic and, in the per-tile sorts, by LDS bandwidth.  The kernels
// read the pair count D from device memory, so the host never waits for it: grids are sized
// from the caller's capacity and surplus workgroups leave at once.
//
//   emit     one workgroup per 256 primitives, placed by a two-level prefix sum over the
//            workgroup tile counts of the preprocess kernel.  Binning rule 0: a load-balanced
//            expansion, the workgroup's output slots are dealt round-robin to its threads and
//            each slot finds its primitive by binary search in an LDS prefix array, so stores
//            are contiguous whatever the rectangle sizes are.  Rule 1: every thread walks the
//            bit mask of kept tiles the preprocess kernel left for its primitive.  Rectangles of
//            more than 128 tiles (rule 1: more than 32, the width of the mask) are deferred to a
//            list and expanded by emit_deferred_kernel, one wavefront (or, beyond 2048 tiles,
//            one workgroup) each, which under rule 1 repeats the intersection test per tile.
//   partition  stable LSD radix sort over the TILE bits of the keys only (two passes of
//            7 + 6 bits at 1080p).  Per pass: (1) digit counts of every 2048-pair sort tile
//            and the pass's digit totals, (2) one workgroup per digit turns its row of counts
//            into output offsets, (3) scatter: wavefront match-any ranking (ballots over the
//            digit bits) keeps equal digits in order, the tile is sorted by digit in LDS and
//            written out in contiguous runs (128 or fewer bins, so runs are long).
//   ranges   tile_offsets[t] = first position whose tile id is >= t.
//   order    tile ids by descending list length, bucketed by the bit length of the length,
//            which also gives the size classes of the per-tile sort and the chunk list.
//   tile sort  every tile's list is sorted by (depth bits, index) as 64-bit composites with a
//            merge sort in LDS (the order is total, so no stability is needed): one wavefront
//            for lists of up to 512 pairs, 256 threads up to 2048, 512 threads up to 4096.  A
//            list of up to 16384 pairs is cut into 4096-pair chunks, sorted by workgroups of
//            the 512-thread launch and merged in two rounds between the two pair buffers by
//            workgroups of the 256-thread and the one-wavefront launch.  Lists beyond that get
//            a workgroup of 1024 threads each: 16384-pair chunks in LDS, then pairwise merges
//            through LDS-staged windows.  Sorting the 32 depth bits this way costs one read
//            and one write of most pairs instead of four radix passes over all of them.
#include <type_traits>

#include "lmk_gs_internal.h"

namespace lmk {

__device__ __forceinline__ u64 load_D(const ScratchHeader *h, u64 capacity)
{
    const u64 d = h->dup_count;
    return d < capacity ? d : capacity;
}

// ---------------------------------------------------------------- emit
// Primitives whose rectangle has more than kBigArea tiles (binning rule 0; kMaskArea under
// rule 1) are not expanded by their own workgroup: with a spatially ordered scene the close-up
// primitives, tens to hundreds of tiles each, sit in a few workgroups, which would then run many
// times longer than the rest.  Their index and output offset go to a list (one atomic per
// wavefront) that emit_deferred_kernel expands, one wavefront per primitive (one workgroup per
// primitive beyond kGiantArea tiles, from the back of the same list), with the same output positions.
constexpr u32 kBigArea = 128;
constexpr u32 kMaskArea = 32;       // rectangles whose kept tiles the preprocess kernel recorded as a bit mask
constexpr u32 kGiantArea = 2048;

__device__ __forceinline__ void append_deferred(bool want, u32 *counter, bool from_back, u32 i, u64 offset,
                                                u32 *__restrict__ big_idx, u64 *__restrict__ big_off, u32 lane, u32 n)
{
    const u64 m = __builtin_amdgcn_ballot_w64(want);
    if (m == 0ull) return;
    u32 base = 0;
    const int leader = (int)__builtin_ctzll(m);
    if ((int)lane == leader) base = atomicAdd(counter, (u32)__builtin_popcountll(m));
    base = (u32)__builtin_amdgcn_readlane((int)base, leader);
    if (want) {
        const u32 k = base + __builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u));
        if (k < n) {                                  // the list holds one entry per primitive at most
            const u32 slot = from_back ? n - 1 - k : k;
            big_idx[slot] = i;
            big_off[slot] = offset;
        }
    }
}

__device__ __forceinline__ void append_big(u32 area, u32 own_limit, u32 i, u64 offset, ScratchHeader *header,
                                           u32 *__restrict__ big_idx, u64 *__restrict__ big_off, u32 lane, u32 n)
{
    append_deferred(area > own_limit && area <= kGiantArea, &header->big_count, false, i, offset, big_idx, big_off, lane, n);
    append_deferred(area > kGiantArea, &header->giant_count, true, i, offset, big_idx, big_off, lane, n);
}

// Where the pairs of workgroup `b` of the preprocess grid start: its offset inside its group
// of kScanGroup workgroups plus the totals of the groups before.  Called by the whole workgroup
// ahead of a __syncthreads(); `s_part` gets one partial sum per wavefront, summed by block_base_finish.
__device__ __forceinline__ void block_base_start(const u64 *__restrict__ group_totals, u32 b, u64 *s_part,
                                                 u32 tid, u32 lane, u32 wv)
{
    const u32 groups_before = b / kScanGroup;
    u64 part = 0;
    for (u32 g = tid; g < groups_before; g += kPreBlock) part += group_totals[g];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_down(part, o, 64);
    if (lane == 0) s_part[wv] = part;
}
__device__ __forceinline__ u64 block_base_finish(const u64 *__restrict__ block_offsets, u32 b, const u64 *s_part)
{
    u64 base = block_offsets[b];
#pragma unroll
    for (u32 k = 0; k < kPreBlock / kWave; ++k) base += s_part[k];
    return base;
}

// What every workgroup of the emit grid does first.  Returns true when the preprocess kernel
// counted no pair for this workgroup (culled, or a skipped voxel range): then it is done here,
// without reading a primitive.
__device__ __forceinline__ bool emit_prologue(const u32 *__restrict__ block_sums, const u64 *__restrict__ block_offsets,
                                              const u64 *__restrict__ group_totals, u32 n, u64 capacity,
                                              u64 *__restrict__ offsets, ScratchHeader *__restrict__ header,
                                              u64 *__restrict__ digit_totals, u64 *s_gpart, u32 tid, u32 lane, u32 wv)
{
    if (blockIdx.x == 0 && tid == 0 && header->dup_count > capacity) header->status = LMK_GS_ERR_CAPACITY;
    // the partition's digit totals are accumulated with atomics: start from zero
    for (u32 k = blockIdx.x * kPreBlock + tid; k < kMaxPasses * kTotalCopies * kMaxRadix; k += gridDim.x * kPreBlock)
        digit_totals[k] = 0;
    if (block_sums[blockIdx.x] != 0) return false;
    if (offsets) {
        block_base_start(group_totals, blockIdx.x, s_gpart, tid, lane, wv);
        __syncthreads();
        const u64 base = block_base_finish(block_offsets, blockIdx.x, s_gpart);
        const u32 i = blockIdx.x * kPreBlock + tid;
        if (i < n) offsets[i] = base;
        if (i == n - 1) offsets[n] = base;
    }
    return true;
}

__global__ __launch_bounds__(kPreBlock) void emit_kernel(
    const u32 *__restrict__ tiles_touched, const ushort4 *__restrict__ rect,
    const float *__restrict__ depth, const u32 *__restrict__ block_sums, const u64 *__restrict__ block_offsets,
    const u64 *__restrict__ group_totals, u32 n, u32 tiles_x,
    u64 capacity, u64 *__restrict__ keys, u32 *__restrict__ vals, u64 *__restrict__ offsets,
    ScratchHeader *__restrict__ header, u32 *__restrict__ big_idx, u64 *__restrict__ big_off,
    u64 *__restrict__ digit_totals)
{
    __shared__ u64 s_gpart[kPreBlock / kWave];
    __shared__ u32 s_excl[kPreBlock];     // exclusive prefix of the (small) rectangles expanded here
    __shared__ u32 s_off[kPreBlock];      // exclusive prefix of tiles_touched: where a primitive's pairs start
    __shared__ ushort4 s_rect[kPreBlock];
    __shared__ u32 s_depth[kPreBlock];
    __shared__ u32 s_wave[kPreBlock / kWave];
    __shared__ u32 s_wave2[kPreBlock / kWave];

    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 i = blockIdx.x * kPreBlock + tid;
    if (emit_prologue(block_sums, block_offsets, group_totals, n, capacity, offsets, header, digit_totals,
                      s_gpart, tid, lane, wv))
        return;
    block_base_start(group_totals, blockIdx.x, s_gpart, tid, lane, wv);     // summed after the barrier below
    const u32 cnt = i < n ? tiles_touched[i] : 0u;
    const bool big = cnt > kBigArea;
    const u32 small = big ? 0u : cnt;
    if (cnt) {
        s_rect[tid] = rect[i];
        s_depth[tid] = __float_as_uint(depth[i]);
    }
    u32 incl = small, incl2 = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const u32 t = __shfl_up(incl, o, 64), t2 = __shfl_up(incl2, o, 64);
        if ((int)lane >= o) { incl += t; incl2 += t2; }
    }
    if (lane == kWave - 1) { s_wave[wv] = incl; s_wave2[wv] = incl2; }
    __syncthreads();
    u32 wave_base = 0, total = 0, wave_base2 = 0, total2 = 0;
#pragma unroll
    for (u32 k = 0; k < kPreBlock / kWave; ++k) {
        const u32 w = s_wave[k], w2 = s_wave2[k];
        if (k < wv) { wave_base += w; wave_base2 += w2; }
        total += w; total2 += w2;
    }
    s_excl[tid] = wave_base + incl - small;
    const u32 off = wave_base2 + incl2 - cnt;
    s_off[tid] = off;
    const u64 base = block_base_finish(block_offsets, blockIdx.x, s_gpart);
    if (offsets) {
        if (i < n) offsets[i] = base + off;
        if (i == n - 1) offsets[n] = base + total2;
    }
    append_big(cnt, kBigArea, i, base + off, header, big_idx, big_off, lane, n);
    __syncthreads();

    for (u32 j = tid; j < total; j += kPreBlock) {
        // owner = last primitive whose exclusive prefix is <= j (primitives with
        // nothing to expand share a prefix with their successor and are skipped by "last")
        u32 lo = 0, hi = kPreBlock - 1;
        while (lo < hi) {
            const u32 mid = (lo + hi + 1) >> 1;
            if (s_excl[mid] <= j) lo = mid; else hi = mid - 1;
        }
        const ushort4 r = s_rect[lo];
        const u32 local = j - s_excl[lo];
        const u32 w = (u32)r.z - (u32)r.x;
        const u32 row = local / w;
        const u32 tx = (u32)r.x + (local - row * w);
        const u32 ty = (u32)r.y + row;
        const u64 pos = base + s_off[lo] + local;
        if (pos < capacity) {
            keys[pos] = ((u64)(ty * tiles_x + tx) << 32) | (u64)s_depth[lo];
            vals[pos] = blockIdx.x * kPreBlock + lo;
        }
    }
}

// ---------------------------------------------------------------- emit, binning rule 1
// Only the tiles that pass the splat/tile intersection test of lmk_gs_camera.binning == 1 get a
// pair, in (primitive, row-major tile) order: the output position of a kept tile is the
// workgroup's base plus the number of kept tiles before it.  For a rectangle of up to
// kMaskArea tiles (nearly all primitives) the preprocess kernel left the kept tiles as a bit
// mask, which the primitive's own thread walks: no test, no feature record.  Larger rectangles
// go to emit_deferred_kernel, which repeats the test per tile (identical arithmetic to the
// count in the preprocess kernel; this translation unit is compiled without floating-point
// contraction for that reason).  Expanding them here, slot by slot across the workgroup, made
// the workgroups that hold the close-up primitives of a spatially ordered scene the long pole.
__device__ __forceinline__ float emit_clampf(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

__device__ __forceinline__ float emit_quad_adj(float A, float B, float C, float ex, float ey)
{
    const float m = A * ex * ex + C * ey * ey;
    const float q = m + 2.0f * B * ex * ey;
    return q - 4e-6f * m;
}

__global__ __launch_bounds__(kPreBlock) void emit_tight_kernel(
    const u32 *__restrict__ tiles_touched, const ushort4 *__restrict__ rect,
    const float *__restrict__ depth,
    const u32 *__restrict__ block_sums, const u64 *__restrict__ block_offsets,
    const u64 *__restrict__ group_totals, u32 n, u32 tiles_x,
    u64 capacity, u64 *__restrict__ keys, u32 *__restrict__ vals, u64 *__restrict__ offsets,
    ScratchHeader *__restrict__ header, u32 *__restrict__ big_idx, u64 *__restrict__ big_off,
    u64 *__restrict__ digit_totals, const u32 *__restrict__ tile_masks)
{
    __shared__ u64 s_gpart[kPreBlock / kWave];
    __shared__ u32 s_wave[kPreBlock / kWave];

    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 i = blockIdx.x * kPreBlock + tid;
    if (emit_prologue(block_sums, block_offsets, group_totals, n, capacity, offsets, header, digit_totals,
                      s_gpart, tid, lane, wv))
        return;
    block_base_start(group_totals, blockIdx.x, s_gpart, tid, lane, wv);     // summed after the barrier below
    const u32 kept_cnt = i < n ? tiles_touched[i] : 0u;
    u32 area = 0, mask = 0, dbits = 0;
    ushort4 r = make_ushort4(0, 0, 0, 0);
    if (kept_cnt) {
        r = rect[i];
        area = ((u32)r.z - (u32)r.x) * ((u32)r.w - (u32)r.y);
        dbits = __float_as_uint(depth[i]);
        if (area <= kMaskArea) mask = tile_masks[i];
    }
    // prefix sum of the kept counts over the workgroup: where every primitive's pairs start
    u32 incl = kept_cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const u32 t = __shfl_up(incl, o, 64);
        if ((int)lane >= o) incl += t;
    }
    if (lane == kWave - 1) s_wave[wv] = incl;
    __syncthreads();
    u32 wave_base = 0, total = 0;
#pragma unroll
    for (u32 k = 0; k < kPreBlock / kWave; ++k) {
        const u32 w = s_wave[k];
        if (k < wv) wave_base += w;
        total += w;
    }
    const u32 kept_excl = wave_base + incl - kept_cnt;
    const u64 base = block_base_finish(block_offsets, blockIdx.x, s_gpart);
    if (offsets) {
        if (i < n) offsets[i] = base + kept_excl;
        if (i == n - 1) offsets[n] = base + total;
    }
    append_big(area, kMaskArea, i, base + kept_excl, header, big_idx, big_off, lane, n);
    // kept tiles in row-major order = set bits in ascending order
    const u32 w = (u32)r.z - (u32)r.x;
    const u32 inv_w = w ? (65536u + w - 1u) / w : 0u;      // slot / w == (slot * inv_w) >> 16 for slot < 32, w <= 32
    u64 pos = base + kept_excl;
    while (mask) {
        const u32 slot = (u32)__builtin_ctz(mask);
        mask &= mask - 1u;
        const u32 row = (slot * inv_w) >> 16;
        const u32 tx = (u32)r.x + (slot - row * w), ty = (u32)r.y + row;
        if (pos < capacity) {
            keys[pos] = ((u64)(ty * tiles_x + tx) << 32) | (u64)dbits;
            vals[pos] = i;
        }
        ++pos;
    }
}

// One wavefront per deferred primitive (persistent grid striding over the list): its rectangle
// is walked 64 tiles at a time in row-major order; under binning rule 1 (TIGHT) each tile is put
// through the splat/tile intersection test and the kept ones are compacted with ballot ranks,
// so the pairs land exactly where the prefix sums say.
template <bool TIGHT>
__device__ __forceinline__ void emit_big_part(
    u32 block, u32 blocks,
    const ushort4 *__restrict__ rect, const float *__restrict__ depth, const float4 *__restrict__ feat,
    const ProjParams &pp, u32 tiles_x, u64 capacity, u64 *__restrict__ keys, u32 *__restrict__ vals,
    const ScratchHeader *__restrict__ header, const u32 *__restrict__ big_idx, const u64 *__restrict__ big_off,
    u32 list_capacity)
{
    const u32 lane = threadIdx.x & (kWave - 1);
    const u32 wave = (block * kPreBlock + threadIdx.x) / kWave, waves = blocks * (kPreBlock / kWave);
    u32 count = header->big_count;
    if (count > list_capacity) count = list_capacity;       // cannot happen: one entry per primitive at most
    const float h = 0.5f * (float)LMK_GS_TILE - 0.5f;
    for (u32 k = wave; k < count; k += waves) {
        const u32 i = big_idx[k];
        if (i >= list_capacity) continue;                    // an index is a primitive: below n
        const u64 off = big_off[k];
        const ushort4 r = rect[i];
        const u32 dbits = __float_as_uint(depth[i]);
        const u32 w = (u32)r.z - (u32)r.x, area = w * ((u32)r.w - (u32)r.y);
        float u = 0.f, v = 0.f, A = 0.f, B = 0.f, Cc = 0.f, rx = 0.f, ry = 0.f, tau = 0.f;
        if (TIGHT) {
            const float4 *f = feat + (size_t)i * (LMK_GS_FEAT_STRIDE / 4);
            const float4 f0 = f[0], f1 = f[1];
            const u32 bits = __float_as_uint(f1.y);
            const int E = (int)((bits >> 23) & 0xffu) - 127;
            tau = pp.tau_tab[(bits >> 20) & 7u] + (float)E * 1.3862944f;
            u = f0.x; v = f0.y; A = f0.z; B = f0.w; Cc = f1.x;
            rx = -f0.w / f0.z; ry = -f0.w / f1.x;
        }
        u32 running = 0;
        for (u32 t0 = 0; t0 < area; t0 += kWave) {           // area > 0 implies w > 0
            const u32 t = t0 + lane;
            bool keep = t < area;
            const u32 row = t / w;
            const u32 tx = (u32)r.x + (t - row * w), ty = (u32)r.y + row;
            if (TIGHT && keep) {
                const float xs = u - ((float)(tx * LMK_GS_TILE) + 0.5f * (float)LMK_GS_TILE);
                const float ys = v - ((float)(ty * LMK_GS_TILE) + 0.5f * (float)LMK_GS_TILE);
                const float ex1 = emit_clampf(xs, -h, h) - xs;
                const float ey1 = emit_clampf(ys + ry * ex1, -h, h) - ys;
                const float ey2 = emit_clampf(ys, -h, h) - ys;
                const float ex2 = emit_clampf(xs + rx * ey2, -h, h) - xs;
                const float q1 = emit_quad_adj(A, B, Cc, ex1, ey1);
                const float q2 = emit_quad_adj(A, B, Cc, ex2, ey2);
                keep = (q1 < q2 ? q1 : q2) <= tau;
            }
            const u64 mask = __builtin_amdgcn_ballot_w64(keep);
            if (keep) {
                const u64 pos = off + running +
                                __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
                if (pos < capacity) {
                    keys[pos] = ((u64)(ty * tiles_x + tx) << 32) | (u64)dbits;
                    vals[pos] = i;
                }
            }
            running += (u32)__builtin_popcountll(mask);
        }
    }
}

// The same for the few primitives that cover thousands of tiles: one workgroup each, 256 tiles
// per round, kept tiles ranked across the workgroup.
template <bool TIGHT>
__device__ __forceinline__ void emit_giant_part(
    u32 block, u32 blocks,
    const ushort4 *__restrict__ rect, const float *__restrict__ depth, const float4 *__restrict__ feat,
    const ProjParams &pp, u32 tiles_x, u64 capacity, u64 *__restrict__ keys, u32 *__restrict__ vals,
    const ScratchHeader *__restrict__ header, const u32 *__restrict__ big_idx, const u64 *__restrict__ big_off,
    u32 list_capacity)
{
    __shared__ u32 s_wave[kPreBlock / kWave];
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    u32 count = header->giant_count;
    if (count > list_capacity) count = list_capacity;
    const float h = 0.5f * (float)LMK_GS_TILE - 0.5f;
    for (u32 k = block; k < count; k += blocks) {             // block-uniform
        const u32 slot = list_capacity - 1 - k;
        const u32 i = big_idx[slot];
        if (i >= list_capacity) continue;
        const u64 off = big_off[slot];
        const ushort4 r = rect[i];
        const u32 dbits = __float_as_uint(depth[i]);
        const u32 w = (u32)r.z - (u32)r.x, area = w * ((u32)r.w - (u32)r.y);
        float u = 0.f, v = 0.f, A = 0.f, B = 0.f, Cc = 0.f, rx = 0.f, ry = 0.f, tau = 0.f;
        if (TIGHT) {
            const float4 *f = feat + (size_t)i * (LMK_GS_FEAT_STRIDE / 4);
            const float4 f0 = f[0], f1 = f[1];
            const u32 bits = __float_as_uint(f1.y);
            const int E = (int)((bits >> 23) & 0xffu) - 127;
            tau = pp.tau_tab[(bits >> 20) & 7u] + (float)E * 1.3862944f;
            u = f0.x; v = f0.y; A = f0.z; B = f0.w; Cc = f1.x;
            rx = -f0.w / f0.z; ry = -f0.w / f1.x;
        }
        u32 running = 0;
        for (u32 t0 = 0; t0 < area; t0 += kPreBlock) {
            const u32 t = t0 + tid;
            bool keep = t < area;
            const u32 row = t / w;
            const u32 tx = (u32)r.x + (t - row * w), ty = (u32)r.y + row;
            if (TIGHT && keep) {
                const float xs = u - ((float)(tx * LMK_GS_TILE) + 0.5f * (float)LMK_GS_TILE);
                const float ys = v - ((float)(ty * LMK_GS_TILE) + 0.5f * (float)LMK_GS_TILE);
                const float ex1 = emit_clampf(xs, -h, h) - xs;
                const float ey1 = emit_clampf(ys + ry * ex1, -h, h) - ys;
                const float ey2 = emit_clampf(ys, -h, h) - ys;
                const float ex2 = emit_clampf(xs + rx * ey2, -h, h) - xs;
                const float q1 = emit_quad_adj(A, B, Cc, ex1, ey1);
                const float q2 = emit_quad_adj(A, B, Cc, ex2, ey2);
                keep = (q1 < q2 ? q1 : q2) <= tau;
            }
            const u64 mask = __builtin_amdgcn_ballot_w64(keep);
            const u32 rank = __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
            __syncthreads();                               // s_wave free again
            if (lane == 0) s_wave[wv] = (u32)__builtin_popcountll(mask);
            __syncthreads();
            u32 before = 0, round_total = 0;
#pragma unroll
            for (u32 q = 0; q < kPreBlock / kWave; ++q) {
                const u32 c = s_wave[q];
                if (q < wv) before += c;
                round_total += c;
            }
            if (keep) {
                const u64 pos = off + running + before + rank;
                if (pos < capacity) {
                    keys[pos] = ((u64)(ty * tiles_x + tx) << 32) | (u64)dbits;
                    vals[pos] = i;
                }
            }
            running += round_total;
        }
    }
}

// One launch for both: the first kGiantBlocks workgroups take the giants, the rest the big ones.
constexpr u32 kGiantBlocks = 2048;

template <bool TIGHT>
__global__ __launch_bounds__(kPreBlock) void emit_deferred_kernel(
    const ushort4 *__restrict__ rect, const float *__restrict__ depth, const float4 *__restrict__ feat,
    ProjParams pp, u32 tiles_x, u64 capacity, u64 *__restrict__ keys, u32 *__restrict__ vals,
    const ScratchHeader *__restrict__ header, const u32 *__restrict__ big_idx, const u64 *__restrict__ big_off,
    u32 list_capacity)
{
    if (blockIdx.x < kGiantBlocks)
        emit_giant_part<TIGHT>(blockIdx.x, kGiantBlocks, rect, depth, feat, pp, tiles_x, capacity, keys, vals,
                               header, big_idx, big_off, list_capacity);
    else
        emit_big_part<TIGHT>(blockIdx.x - kGiantBlocks, gridDim.x - kGiantBlocks, rect, depth, feat, pp, tiles_x,
                             capacity, keys, vals, header, big_idx, big_off, list_capacity);
}

// ---------------------------------------------------------------- radix sort
// (1) digit counts of every sort tile of this pass -> table[digit][tile]
// Pairs of a spatially ordered scene arrive in runs of one tile: a wavefront whose 64 keys share a
// digit adds once instead of queueing 64 atomics on one LDS word.  Called by whole wavefronts.
__device__ __forceinline__ void wave_hist_add(u32 *hist, u32 d, bool valid, u32 tid)
{
    const u64 live = __builtin_amdgcn_ballot_w64(valid);
    const u32 d0 = (u32)__builtin_amdgcn_readfirstlane((int)d);
    const u64 same = __builtin_amdgcn_ballot_w64(valid && d == d0);
    if (live != 0ull && same == live && (live & 1ull)) {
        if ((tid & (kWave - 1)) == 0) atomicAdd(&hist[d0], (u32)__builtin_popcountll(live));
    } else if (valid) {
        atomicAdd(&hist[d], 1u);
    }
}

// Each pass also adds its digit totals (the row sums of `table`, which the scan needs as the
// base of every digit) to `digit_totals`: kept per workgroup in LDS and flushed with one global
// atomic per non-empty digit when the workgroup is done.  Atomics on one address are served one
// after the other, and a pass over the high tile bits has only a few digits, so the totals are
// kept in kTotalCopies copies (workgroup b adds to copy b % kTotalCopies; the scan adds them up).
template <u32 kSortItems>
__global__ __launch_bounds__(kSortThreads) void radix_hist_kernel(
    const u64 *__restrict__ keys, const ScratchHeader *__restrict__ header, u64 capacity,
    u32 shift, u32 bits, u32 *__restrict__ table, u64 table_stride, u64 *__restrict__ digit_totals)
{
    constexpr u32 kSortTile = kSortThreads * kSortItems;
    __shared__ u32 s_hist[kMaxRadix];
    __shared__ u32 s_tot[kMaxRadix];
    const u64 D = load_D(header, capacity);
    const u64 ntiles = (D + kSortTile - 1) / kSortTile;
    const u32 tid = threadIdx.x;
    const u32 dmask = (1u << bits) - 1u;
    for (u32 d = tid; d < kMaxRadix; d += kSortThreads) s_tot[d] = 0;    // thread d owns s_tot[d]
    // a whole tile needs no bounds checks: the body is instantiated twice
    auto run_tile = [&](u64 tile, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        for (u32 d = tid; d < kMaxRadix; d += kSortThreads) s_hist[d] = 0;
        __syncthreads();
        const u64 t0 = tile * kSortTile;
        u64 k[kSortItems];
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kSortThreads + tid;
            k[j] = (FULL || idx < D) ? keys[idx] : 0ull;
        }
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kSortThreads + tid;
            wave_hist_add(s_hist, (u32)(k[j] >> shift) & dmask, FULL || idx < D, tid);
        }
        __syncthreads();
        for (u32 d = tid; d < kMaxRadix; d += kSortThreads) {
            const u32 c = s_hist[d];
            table[(u64)d * table_stride + tile] = c;
            s_tot[d] += c;
        }
        __syncthreads();
    };
    for (u64 tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if ((tile + 1) * kSortTile <= D) run_tile(tile, std::true_type());
        else run_tile(tile, std::false_type());
    }
    u64 *mine = digit_totals + (size_t)(blockIdx.x % kTotalCopies) * kMaxRadix;
    for (u32 d = tid; d < kMaxRadix; d += kSortThreads) {
        const u32 c = s_tot[d];
        if (c) atomicAdd(reinterpret_cast<unsigned long long *>(&mine[d]), (unsigned long long)c);
    }
}

// (2) one workgroup per digit: exclusive scan of its row of counts, offset by the total of
// all smaller digits -> offsets[digit][tile] (u64)
__global__ __launch_bounds__(kSortThreads) void radix_scan_kernel(
    const ScratchHeader *__restrict__ header, u64 capacity, const u32 *__restrict__ table,
    u64 *__restrict__ offsets, u64 table_stride, const u64 *__restrict__ digit_totals, u32 sort_tile)
{
    __shared__ u64 s_wave[kSortThreads / kWave];
    __shared__ u64 s_carry;
    const u64 D = load_D(header, capacity);
    const u64 ntiles = (D + sort_tile - 1) / sort_tile;
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 digit = blockIdx.x;

    // base = total of the digits below mine
    u64 part = 0;
    for (u32 k = tid; k < kTotalCopies * kMaxRadix; k += kSortThreads)
        if ((k & (kMaxRadix - 1)) < digit) part += digit_totals[k];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_down(part, o, 64);
    if (lane == 0) s_wave[wv] = part;
    __syncthreads();
    if (tid == 0) {
        u64 b = 0;
        for (u32 k = 0; k < kSortThreads / kWave; ++k) b += s_wave[k];
        s_carry = b;
    }
    __syncthreads();

    const u32 *row = table + (u64)digit * table_stride;
    u64 *orow = offsets + (u64)digit * table_stride;
    // rows of 64 consecutive sort tiles per wavefront, so that loads and stores are whole lines;
    // a count is at most 4096, so the sums inside one wavefront's rows fit 32 bits
    constexpr u32 kRows = 8;
    constexpr u32 kWaves = kSortThreads / kWave;
    for (u64 base = 0; base < ntiles; base += (u64)kWaves * kRows * kWave) {
        const u64 first = base + (u64)wv * kRows * kWave + lane;
        u32 x[kRows], inc[kRows], before[kRows];
#pragma unroll
        for (u32 k = 0; k < kRows; ++k) x[k] = first + k * kWave < ntiles ? row[first + k * kWave] : 0u;
        u32 wave_total = 0;
#pragma unroll
        for (u32 k = 0; k < kRows; ++k) {
            u32 v = x[k];
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const u32 t = __shfl_up(v, o, 64);
                if ((int)lane >= o) v += t;
            }
            inc[k] = v;
            before[k] = wave_total;
            wave_total += __shfl(v, kWave - 1, 64);
        }
        __syncthreads();                       // s_wave free again
        if (lane == 0) s_wave[wv] = wave_total;
        __syncthreads();
        u64 run = s_carry;
        for (u32 k = 0; k < wv; ++k) run += s_wave[k];
#pragma unroll
        for (u32 k = 0; k < kRows; ++k)
            if (first + k * kWave < ntiles) orow[first + k * kWave] = run + (before[k] + inc[k] - x[k]);
        __syncthreads();
        if (tid == kSortThreads - 1) s_carry = run + wave_total;
        __syncthreads();
    }
}

// (3) stable scatter of one digit
template <u32 kSortItems>
__global__ __launch_bounds__(kSortThreads) void radix_scatter_kernel(
    const u64 *__restrict__ keys_in, const u32 *__restrict__ vals_in,
    u64 *__restrict__ keys_out, u32 *__restrict__ vals_out,
    const ScratchHeader *__restrict__ header, u64 capacity, u32 shift, u32 bits,
    const u64 *__restrict__ offsets, u64 table_stride)
{
    constexpr u32 kSortTile = kSortThreads * kSortItems;
    constexpr u32 kWaves = kSortThreads / kWave;
    constexpr u32 kPerWave = kSortItems * kWave;       // consecutive pairs per wavefront
    __shared__ u32 s_wave_hist[kWaves][kMaxRadix];     // per-wavefront digit counters, then bases
    __shared__ u32 s_digit_start[kMaxRadix];           // first local position of each digit
    __shared__ u64 s_gofs[kMaxRadix];                  // global offset minus local start
    __shared__ u32 s_scan[kWaves];
    __shared__ u64 s_stage[kSortTile];                 // keys, then (reused) values

    const u64 D = load_D(header, capacity);
    const u64 ntiles = (D + kSortTile - 1) / kSortTile;
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u64 lane_lt = (1ull << lane) - 1ull;
    const u32 radix = 1u << bits, dmask = radix - 1u;

    // a whole tile needs none of the bounds checks: the body is instantiated twice
    auto run_tile = [&](u64 tile, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        for (u32 k = tid; k < kWaves * kMaxRadix; k += kSortThreads) (&s_wave_hist[0][0])[k] = 0;
        __syncthreads();

        const u64 t0 = tile * kSortTile + (u64)wv * kPerWave;
        u64 key[kSortItems];
        u32 val[kSortItems];
        u32 rank[kSortItems];
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kWave + lane;
            const bool valid = FULL || idx < D;
            key[j] = valid ? keys_in[idx] : ~0ull;
            val[j] = valid ? vals_in[idx] : 0u;
        }
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kWave + lane;
            const bool valid = FULL || idx < D;
            const u32 digit = (u32)(key[j] >> shift) & dmask;
            // lanes of this wavefront holding the same digit (match-any by ballots): per digit bit,
            // keep the lanes whose bit equals mine -- with m = 0 / ~0 for my bit 0 / 1 that is
            // peers & ~(ballot ^ m), on the two 32-bit halves
            const u64 live = __builtin_amdgcn_ballot_w64(valid);
            u32 peers_lo = (u32)live, peers_hi = (u32)(live >> 32);
#pragma unroll
            for (u32 b = 0; b < kMaxRadixBits; ++b) {
                if (b < bits) {
                    const u32 m = 0u - ((digit >> b) & 1u);
                    const u64 bal = __builtin_amdgcn_ballot_w64(m != 0u);
                    peers_lo &= ~((u32)bal ^ m);
                    peers_hi &= ~((u32)(bal >> 32) ^ m);
                }
            }
            const u64 peers = ((u64)peers_hi << 32) | (u64)peers_lo;
            const u32 before = __popcll(peers & lane_lt);
            u32 old = 0;
            if (valid && before == 0)                  // lowest peer lane adds for the group
                old = atomicAdd(&s_wave_hist[wv][digit], (u32)__popcll(peers));
            const int leader = valid ? (__ffsll((long long)peers) - 1) : (int)lane;
            old = __shfl(old, leader, 64);
            rank[j] = old + before;                    // position among this wavefront's equal digits
        }
        __syncthreads();

        // thread t owns kDPT consecutive digits: tile totals, per-wavefront bases, local starts
        {
            constexpr u32 kDPT = kMaxRadix / kSortThreads;
            u32 cnt[kDPT];
            u32 mine = 0;
#pragma unroll
            for (u32 h = 0; h < kDPT; ++h) {
                const u32 d = kDPT * tid + h;
                u32 run = 0;
#pragma unroll
                for (u32 k = 0; k < kWaves; ++k) {
                    const u32 c = s_wave_hist[k][d];
                    s_wave_hist[k][d] = run;
                    run += c;
                }
                cnt[h] = run;
                mine += run;
            }
            u32 incl = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const u32 t = __shfl_up(incl, o, 64);
                if ((int)lane >= o) incl += t;
            }
            if (lane == kWave - 1) s_scan[wv] = incl;
            __syncthreads();
            u32 start = incl - mine;
#pragma unroll
            for (u32 k = 0; k < kWaves; ++k) if (k < wv) start += s_scan[k];
#pragma unroll
            for (u32 h = 0; h < kDPT; ++h) {
                const u32 d = kDPT * tid + h;
                s_digit_start[d] = start;
                if (d < radix) s_gofs[d] = offsets[(u64)d * table_stride + tile] - (u64)start;
                start += cnt[h];
            }
        }
        __syncthreads();

        // sort the tile by digit in LDS: keys first, then the values through the same slots
        const u64 tile_base = tile * kSortTile;
        const u32 count = (u32)((D - tile_base) < (u64)kSortTile ? (D - tile_base) : (u64)kSortTile);
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kWave + lane;
            if (FULL || idx < D) {
                const u32 digit = (u32)(key[j] >> shift) & dmask;
                rank[j] = s_digit_start[digit] + s_wave_hist[wv][digit] + rank[j];
                s_stage[rank[j]] = key[j];
            }
        }
        __syncthreads();
        u32 dg[kSortItems];                            // digit of the key that ended up in slot p
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u32 p = j * kSortThreads + tid;
            if (FULL || p < count) {
                const u64 k = s_stage[p];
                dg[j] = (u32)(k >> shift) & dmask;
                keys_out[s_gofs[dg[j]] + p] = k;
            }
        }
        __syncthreads();
        u32 *s_vals = reinterpret_cast<u32 *>(s_stage);
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kWave + lane;
            if (FULL || idx < D) s_vals[rank[j]] = val[j];
        }
        __syncthreads();
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u32 p = j * kSortThreads + tid;
            if (FULL || p < count) vals_out[s_gofs[dg[j]] + p] = s_vals[p];
        }
        __syncthreads();
    };
    for (u64 tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if ((tile + 1) * kSortTile <= D) run_tile(tile, std::true_type());
        else run_tile(tile, std::false_type());
    }
}

// ---------------------------------------------------------------- ranges
__global__ __launch_bounds__(256) void tile_ranges_kernel(
    const u64 *__restrict__ keys, ScratchHeader *__restrict__ header, u64 capacity,
    u32 num_tiles, u64 *__restrict__ tile_offsets, u64 *__restrict__ offsets_if_empty)
{
    // the emit stage's list of deferred primitives has been consumed: empty it for the next call
    if (blockIdx.x == 0 && threadIdx.x == 0) { header->big_count = 0; header->giant_count = 0; }
    // with no primitives the emit kernel never runs: the one-entry prefix sum is written here
    if (offsets_if_empty && blockIdx.x == 0 && threadIdx.x == 0) offsets_if_empty[0] = 0;
    const u64 D = load_D(header, capacity);
    const u64 stride = (u64)gridDim.x * blockDim.x;
    const u64 first = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (D == 0) {
        for (u64 t = first; t <= num_tiles; t += stride) tile_offsets[t] = 0;
        return;
    }
    for (u64 i = first; i < D; i += stride) {
        u64 t = keys[i] >> 32;
        if (t > num_tiles) t = num_tiles;
        u64 tp;     // tiles in (tp, t] start at i
        if (i == 0) {
            for (u64 k = 0; k <= t; ++k) tile_offsets[k] = 0;
        } else {
            tp = keys[i - 1] >> 32;
            if (tp > num_tiles) tp = num_tiles;
            for (u64 k = tp + 1; k <= t; ++k) tile_offsets[k] = i;
        }
        if (i == D - 1)
            for (u64 k = t + 1; k <= num_tiles; ++k) tile_offsets[k] = D;
    }
}

// ---------------------------------------------------------------- order + size classes
// Tile ids by descending list length, bucketed by the bit length of (length - 1), so that
// the size classes of the per-tile sort are whole buckets.  From the front of `order`:
//   classes[0]  lists longer than kHuge pairs          one workgroup each, merges between the pair buffers
//   classes[3]  kMid + 1 .. kHuge ("long")             cut into chunks of kMid pairs, see below
//   classes[1]  kLow + 1 .. kMid                       one workgroup of 512
//   classes[2]  kSmallCap + 1 .. kLow                  one workgroup of 256
//   the rest                                           one wavefront each
// Within a bucket the order is whatever the atomics give -- it only decides which workgroup
// starts first, never a result.  A long list is sorted as 2 .. 4 chunks by workgroups of the
// 512-thread kernel and merged in two rounds by workgroups of the next two kernels, so that it
// costs no kernel of its own: chunk_list = (tile, chunk) of every such chunk, classes[4] = how many.
// One workgroup.
constexpr u32 kSmallThreads = 64, kSmallItems = 8, kSmallCap = kSmallThreads * kSmallItems;   // 512
constexpr u32 kLowThreads = 256, kLowItems = 8;                                               // 2048
constexpr u32 kMidThreads = 512, kMidItems = 8, kMid = kMidThreads * kMidItems;               // 4096
constexpr u32 kHugeThreads = 1024, kHugeItems = 16, kHuge = kHugeThreads * kHugeItems;        // 16384
static_assert(kMid == kChunk, "the launch bounds on the host use kChunk");

__device__ __forceinline__ u32 length_bucket(u64 len)
{
    return len > 1 ? 64u - (u32)__builtin_clzll(len - 1) : 0u;   // len in (2^(b-1), 2^b]
}
constexpr u32 kSmallBucket = 9, kLowBucket = 11, kMidBucket = 12, kHugeBucket = 14;   // 2^9 = kSmallCap, 2^11 = kLow, 2^12 = kMid, 2^14 = kHuge

// Most tiles fall into a handful of buckets, and LDS atomics on one word are served one after
// the other: every bucket has kOrderCopies counters, picked by the low lane bits, so that the 64
// atomics of a wavefront spread over that many words.  An exclusive scan over
// [bucket][copy] turns the counts into the first slot of every (bucket, copy).
constexpr u32 kOrderCopies = 16, kOrderCounters = 65 * kOrderCopies, kOrderBatch = 8, kOrderStage = 32768;

__global__ __launch_bounds__(1024) void tile_order_kernel(
    const u64 *__restrict__ tile_offsets, u32 num_tiles, u32 *__restrict__ order,
    u32 *__restrict__ order_copy, u32 *__restrict__ classes, uint2 *__restrict__ chunk_list, u64 chunk_capacity)
{
    __shared__ u32 s_cnt[kOrderCounters];
    __shared__ u32 s_long[2];                  // first long tile in `order`, number of long tiles
    __shared__ u32 s_wave[1024 / kWave];
    // slots are scattered and one compute unit does all the address work: the order is put
    // together in LDS and written out in whole lines (images of up to kOrderStage tiles)
    __shared__ u32 s_order[kOrderStage];
    const bool staged = num_tiles <= kOrderStage;
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 copy = tid & (kOrderCopies - 1);
    for (u32 k = tid; k < kOrderCounters; k += 1024) s_cnt[k] = 0;
    __syncthreads();
    // kOrderBatch tiles per thread and round: all their loads are in flight together
    for (u32 base = 0; base < num_tiles; base += kOrderBatch * 1024) {
        u32 b[kOrderBatch];
#pragma unroll
        for (u32 j = 0; j < kOrderBatch; ++j) {
            const u32 t = base + j * 1024 + tid;
            b[j] = t < num_tiles ? length_bucket(tile_offsets[t + 1] - tile_offsets[t]) : 0xffu;
        }
#pragma unroll
        for (u32 j = 0; j < kOrderBatch; ++j)
            if (b[j] != 0xffu) atomicAdd(&s_cnt[(64 - b[j]) * kOrderCopies + copy], 1u);     // long lists first
    }
    __syncthreads();
    // exclusive scan of the counters, two per thread (kOrderCounters <= 2048)
    const u32 k0 = 2 * tid, k1 = 2 * tid + 1;
    const u32 c0 = k0 < kOrderCounters ? s_cnt[k0] : 0u, c1 = k1 < kOrderCounters ? s_cnt[k1] : 0u;
    u32 incl = c0 + c1;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const u32 v = __shfl_up(incl, o, 64);
        if ((int)lane >= o) incl += v;
    }
    if (lane == kWave - 1) s_wave[wv] = incl;
    __syncthreads();
    u32 before = 0;
    for (u32 k = 0; k < wv; ++k) before += s_wave[k];
    const u32 excl = before + incl - (c0 + c1);
    if (k0 < kOrderCounters) s_cnt[k0] = excl;
    if (k1 < kOrderCounters) s_cnt[k1] = excl + c0;
    __syncthreads();
    if (tid == 0) {
        // tiles in buckets above a class limit = first slot of the first bucket at or below it
        const u32 huge = s_cnt[(64 - kHugeBucket) * kOrderCopies];
        const u32 lng = s_cnt[(64 - kMidBucket) * kOrderCopies];
        const u32 mid = s_cnt[(64 - kLowBucket) * kOrderCopies];
        const u32 low = s_cnt[(64 - kSmallBucket) * kOrderCopies];
        classes[0] = huge; classes[3] = lng - huge; classes[1] = mid - lng; classes[2] = low - mid;
        s_long[0] = huge; s_long[1] = lng - huge;
    }
    __syncthreads();
    for (u32 base = 0; base < num_tiles; base += kOrderBatch * 1024) {
        u32 b[kOrderBatch];
#pragma unroll
        for (u32 j = 0; j < kOrderBatch; ++j) {
            const u32 t = base + j * 1024 + tid;
            b[j] = t < num_tiles ? length_bucket(tile_offsets[t + 1] - tile_offsets[t]) : 0xffu;
        }
#pragma unroll
        for (u32 j = 0; j < kOrderBatch; ++j) {
            if (b[j] == 0xffu) continue;
            const u32 t = base + j * 1024 + tid;
            const u32 slot = atomicAdd(&s_cnt[(64 - b[j]) * kOrderCopies + copy], 1u);
            if (staged) {
                s_order[slot] = t;
            } else {
                order[slot] = t;
                if (order_copy) order_copy[slot] = t;
            }
        }
    }
    if (staged) {
        __syncthreads();
        for (u32 k = tid; k < num_tiles; k += 1024) {
            const u32 t = s_order[k];
            order[k] = t;
            if (order_copy) order_copy[k] = t;
        }
    } else {
        __threadfence_block();                 // this workgroup reads its own writes of `order` below
        __syncthreads();
    }
    // the chunks of the long lists: an exclusive scan of their chunk counts places the entries
    const u32 long_first = s_long[0], long_count = s_long[1];
    u32 carry = 0;
    for (u32 base = 0; base < long_count; base += 1024) {
        const u32 k = base + tid;
        u32 tile = 0, nch = 0;
        if (k < long_count) {
            tile = staged ? s_order[long_first + k] : order[long_first + k];
            nch = (u32)((tile_offsets[tile + 1] - tile_offsets[tile] + kMid - 1) / kMid);
        }
        u32 incl = nch;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const u32 v = __shfl_up(incl, o, 64);
            if ((int)lane >= o) incl += v;
        }
        __syncthreads();                       // s_wave free again
        if (lane == kWave - 1) s_wave[wv] = incl;
        __syncthreads();
        u32 before = carry, total = carry;
        for (u32 w = 0; w < 1024 / kWave; ++w) {
            const u32 c = s_wave[w];
            if (w < wv) before += c;
            total += c;
        }
        const u32 at = before + incl - nch;
        for (u32 c = 0; c < nch; ++c)
            if ((u64)at + c < chunk_capacity) chunk_list[at + c] = make_uint2(tile, c);
        carry = total;
    }
    if (tid == 0) classes[4] = (u64)carry < chunk_capacity ? carry : (u32)chunk_capacity;
}

// ---------------------------------------------------------------- per-tile sort
// Sorts up to THREADS * ITEMS pairs of one tile by (depth bits, index) with a merge sort:
// each thread sorts ITEMS composites in registers (a fixed network, no memory traffic), the
// runs of 2, 4 and 8 neighbouring lanes are merged in registers too (bitonic merges with DPP
// lane exchanges), and from there the sorted runs are merged pairwise through LDS, run length
// doubling: a thread finds where its ITEMS outputs start in the two runs (merge-path binary
// search) and merges them sequentially.  Runs are stored with one padding slot per 16 elements
// so that the strided accesses of neighbouring threads spread over the LDS banks.  Instances:
// 64 threads x 2 / 4 / 8 (one wavefront per short list, which is most tiles), 256 x 8,
// 512 x 8, and 1024 x 16 (most of a compute unit's LDS) for the chunks of the longest lists.
__device__ __forceinline__ u32 ts_slot(u32 p) { return p + (p >> 4); }

__device__ __forceinline__ void ts_cswap(u64 &a, u64 &b)
{
    const u64 lo = a < b ? a : b, hi = a < b ? b : a;
    a = lo; b = hi;
}

// ITEMS outputs, starting at output `diag`, of the merge of the sorted runs s[a0, a1) and s[a1, b1)
template <u32 ITEMS>
__device__ __forceinline__ void merge_from_lds(const u64 *s, u32 a0, u32 a1, u32 b1, u32 diag, u64 (&e)[ITEMS])
{
    const u32 lenA = a1 - a0, lenB = b1 - a1;
    u32 l0 = diag > lenB ? diag - lenB : 0, h0 = diag < lenA ? diag : lenA;
    while (l0 < h0) {
        const u32 mid = (l0 + h0) >> 1;
        if (s[ts_slot(a0 + mid)] < s[ts_slot(a1 + diag - 1 - mid)]) l0 = mid + 1; else h0 = mid;
    }
    u32 i = a0 + l0, j = a1 + (diag - l0);
    u64 ka = i < a1 ? s[ts_slot(i)] : ~0ull;
    u64 kb = j < b1 ? s[ts_slot(j)] : ~0ull;
    // Straight-line steps, selects only: an exhausted run shows the maximum value, which also is
    // what the padding holds, so "A first unless B is smaller" needs no bounds in the comparison
    // (a tie is between padding values, where the side does not matter).  The one LDS read per
    // step is not branched around: when the run has just been used up it reads slot 0 and the
    // value is dropped.
#pragma unroll
    for (u32 k = 0; k < ITEMS; ++k) {
        const bool takeA = ka <= kb;
        e[k] = takeA ? ka : kb;
        const u32 next = (takeA ? i : j) + 1u;
        const u32 lim = takeA ? a1 : b1;
        const bool more = next < lim;
        const u32 at = more ? next : 0u;
        const u64 v = s[ts_slot(at)];
        const u64 nv = more ? v : ~0ull;
        i = takeA ? next : i;
        j = takeA ? j : next;
        ka = takeA ? nv : ka;
        kb = takeA ? kb : nv;
    }
}

// The first three merge rounds need no LDS: the runs of 2, 4 and 8 neighbouring lanes are merged
// with a bitonic merge network whose lane exchanges are DPP moves (mirror within 2 / 4 / 8
// lanes for the first, "flip" stage, lane xor 1 / 2 for the half-cleaners that follow).
template <int CTRL>
__device__ __forceinline__ u64 ts_dpp(u64 v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(u32)v, CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(u32)(v >> 32), CTRL, 0xf, 0xf, true);
    return ((u64)(u32)hi << 32) | (u64)(u32)lo;
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E;            // quad_perm [1,0,3,2], [2,3,0,1]
constexpr int kDppMirror4 = 0x1B, kDppMirror8 = 0x141;     // quad_perm [3,2,1,0], row_half_mirror

// one stage across lanes: element k meets element k (FLIP: ITEMS - 1 - k) of the partner lane;
// the lower lane of the pair keeps the smaller value
template <int CTRL, bool FLIP, u32 ITEMS>
__device__ __forceinline__ void ts_lane_stage(u64 (&e)[ITEMS], bool upper)
{
    u64 p[ITEMS];
#pragma unroll
    for (u32 k = 0; k < ITEMS; ++k) p[k] = ts_dpp<CTRL>(e[FLIP ? ITEMS - 1 - k : k]);
#pragma unroll
    for (u32 k = 0; k < ITEMS; ++k) {
        const bool mine = (e[k] < p[k]) != upper;           // lower keeps the smaller, upper the larger
        e[k] = mine ? e[k] : p[k];
    }
}

// a bitonic sequence of ITEMS values in registers -> ascending
template <u32 ITEMS>
__device__ __forceinline__ void ts_clean(u64 (&e)[ITEMS])
{
#pragma unroll
    for (u32 j = ITEMS >> 1; j > 0; j >>= 1) {
#pragma unroll
        for (u32 i = 0; i < ITEMS; ++i)
            if ((i & j) == 0) ts_cswap(e[i], e[i | j]);
    }
}

template <u32 THREADS, u32 ITEMS>
__device__ __forceinline__ void sort_pairs_in_lds(u64 *keys, u32 *vals, u64 beg, u32 n, u32 tile, u64 *s,
                                                  u64 *keys_out = nullptr, u32 *vals_out = nullptr)
{
    if (!keys_out) { keys_out = keys; vals_out = vals; }    // in place unless the caller wants the result elsewhere
    constexpr u32 CAP = THREADS * ITEMS;
    constexpr u32 kLaneRun = 8 * ITEMS;                     // sorted run length after the lane merges
    const u32 tid = threadIdx.x;
    const u32 m = (n + ITEMS - 1) / ITEMS * ITEMS;          // elements in play: n rounded up to whole runs
    const u32 o0 = tid * ITEMS;
    const bool active = o0 < m;
    // each thread's ITEMS consecutive pairs as composites; beyond n the maximum value, which sorts to the end
    u64 e[ITEMS];
#pragma unroll
    for (u32 k = 0; k < ITEMS; ++k)
        e[k] = o0 + k < n ? ((keys[beg + o0 + k] << 32) | (u64)vals[beg + o0 + k]) : ~0ull;
    // sort the run in registers (bitonic network)
#pragma unroll
    for (u32 k = 2; k <= ITEMS; k <<= 1) {
#pragma unroll
        for (u32 j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (u32 i = 0; i < ITEMS; ++i) {
                const u32 l = i ^ j;
                if (l > i) {
                    if ((i & k) == 0) ts_cswap(e[i], e[l]); else ts_cswap(e[l], e[i]);
                }
            }
        }
    }
    // runs of 2, 4, 8 lanes (every lane takes part; lanes beyond m hold the maximum value)
    ts_lane_stage<kDppXor1, true, ITEMS>(e, (tid & 1u) != 0u);
    ts_clean<ITEMS>(e);
    ts_lane_stage<kDppMirror4, true, ITEMS>(e, (tid & 2u) != 0u);
    ts_lane_stage<kDppXor1, false, ITEMS>(e, (tid & 1u) != 0u);
    ts_clean<ITEMS>(e);
    ts_lane_stage<kDppMirror8, true, ITEMS>(e, (tid & 4u) != 0u);
    ts_lane_stage<kDppXor2, false, ITEMS>(e, (tid & 2u) != 0u);
    ts_lane_stage<kDppXor1, false, ITEMS>(e, (tid & 1u) != 0u);
    ts_clean<ITEMS>(e);
    if (active) {
#pragma unroll
        for (u32 k = 0; k < ITEMS; ++k) s[ts_slot(o0 + k)] = e[k];
    }
    __syncthreads();

    for (u32 run = kLaneRun; run < m && run < CAP; run <<= 1) {
        if (active) {
            // outputs [o0, o0 + ITEMS) of the pair of runs holding them: A = [a0, a1), B = [a1, b1)
            const u32 a0 = (o0 / (2 * run)) * (2 * run);
            const u32 a1 = a0 + run < m ? a0 + run : m;
            const u32 b1 = a0 + 2 * run < m ? a0 + 2 * run : m;
            merge_from_lds<ITEMS>(s, a0, a1, b1, o0 - a0, e);
        }
        __syncthreads();
        if (active) {
#pragma unroll
            for (u32 k = 0; k < ITEMS; ++k) s[ts_slot(o0 + k)] = e[k];
        }
        __syncthreads();
    }
    const u64 hi_bits = (u64)tile << 32;
    for (u32 p = tid; p < n; p += THREADS) {
        const u64 c = s[ts_slot(p)];
        keys_out[beg + p] = hi_bits | (c >> 32);
        vals_out[beg + p] = (u32)c;
    }
    __syncthreads();                                        // s may be refilled by the caller
}

// ---------------------------------------------------------------- merges between the pair buffers
__device__ __forceinline__ bool pair_less(u64 ka, u32 va, u64 kb, u32 vb)
{
    return ka < kb || (ka == kb && va < vb);
}

// Merge-path split by one wavefront: the number of elements of A = [a0, a1) among the first
// `diag` outputs of the merge of A and B = [a1, b1) (sorted runs in global memory).  Every
// round the 64 lanes probe 64 evenly spaced candidates, which narrows the range 64-fold.
__device__ __forceinline__ u64 wave_merge_split(const u64 *__restrict__ sk, const u32 *__restrict__ sv,
                                                u64 a0, u64 a1, u64 b1, u64 diag, u32 lane)
{
    const u64 lenA = a1 - a0, lenB = b1 - a1;
    u64 lo = diag > lenB ? diag - lenB : 0, hi = diag < lenA ? diag : lenA;
    while (lo < hi) {                                       // wave-uniform
        const u64 step = (hi - lo + 63) / 64;
        const u64 m = lo + (u64)(lane + 1) * step - 1;
        bool p = false;
        if (m < hi) {
            const u64 jb = a1 + (diag - 1 - m);
            p = pair_less(sk[a0 + m], sv[a0 + m], sk[jb], sv[jb]);
        }
        const u64 c = (u64)__builtin_popcountll(__builtin_amdgcn_ballot_w64(p));   // leading run of "true"
        const u64 nlo = lo + c * step;
        const u64 nhi = lo + (c + 1) * step - 1;
        hi = nhi < hi ? nhi : hi;
        lo = nlo;
    }
    return lo;
}

// One output segment of THREADS * ITEMS pairs of a merge round over the sorted runs of length
// `run` of one tile's list (L pairs at sk/sv, result to dk/dv): two wavefronts find where the
// segment starts and ends in its pair of runs, the two input windows are staged in LDS as
// composites, merged there and written out coalesced.  A run without a partner is copied.
// Called by the whole workgroup; `s` holds THREADS * ITEMS composites (padded), s_split two words.
template <u32 THREADS, u32 ITEMS>
__device__ __forceinline__ void merge_segment(const u64 *__restrict__ sk, const u32 *__restrict__ sv,
                                              u64 *__restrict__ dk, u32 *__restrict__ dv,
                                              u64 L, u64 run, u64 seg, u32 tile, u64 *s, u64 *s_split)
{
    constexpr u32 CAP = THREADS * ITEMS;
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u64 o = seg * CAP;
    if (o >= L) return;                                     // the same for the whole workgroup
    const u64 a0 = (o / (2 * run)) * (2 * run);
    const u64 a1 = a0 + run < L ? a0 + run : L;
    const u64 b1 = a0 + 2 * run < L ? a0 + 2 * run : L;
    const u64 oe = o + CAP < b1 ? o + CAP : b1;
    if (wv == 0) {
        const u64 i0 = wave_merge_split(sk, sv, a0, a1, b1, o - a0, lane);
        if (lane == 0) s_split[0] = i0;
    }
    if (wv == (THREADS > kWave ? 1u : 0u)) {
        const u64 i1 = wave_merge_split(sk, sv, a0, a1, b1, oe - a0, lane);
        if (lane == 0) s_split[1] = i1;
    }
    __syncthreads();
    const u64 i0 = s_split[0], i1 = s_split[1];
    const u64 j0 = (o - a0) - i0;                           // elements of B before the segment
    const u32 la = (u32)(i1 - i0), total = (u32)(oe - o);
    for (u32 p = tid; p < total; p += THREADS) {
        const u64 src = p < la ? a0 + i0 + p : a1 + j0 + (p - la);
        s[ts_slot(p)] = (sk[src] << 32) | (u64)sv[src];
    }
    __syncthreads();
    const u32 o0 = tid * ITEMS;
    u64 e[ITEMS];
    if (o0 < total) merge_from_lds<ITEMS>(s, 0u, la, total, o0, e);
    __syncthreads();
    if (o0 < total) {
#pragma unroll
        for (u32 k = 0; k < ITEMS; ++k)
            if (o0 + k < total) s[ts_slot(o0 + k)] = e[k];
    }
    __syncthreads();
    const u64 hi_bits = (u64)tile << 32;
    for (u32 p = tid; p < total; p += THREADS) {
        const u64 c = s[ts_slot(p)];
        dk[o + p] = hi_bits | (c >> 32);
        dv[o + p] = (u32)c;
    }
    __syncthreads();                                        // s and s_split may be reused by the caller
}

// Lists of kLow + 1 .. kMid pairs, one workgroup each, and before them the chunks of the long
// lists (kMid + 1 .. kHuge pairs), which are sorted in place like a list of their own.
// Both count for more than kLow pairs each, which bounds the grid.
__global__ __launch_bounds__(kMidThreads) void tile_sort_mid_kernel(
    u64 *__restrict__ keys, u32 *__restrict__ vals, const u64 *__restrict__ tile_offsets,
    const u32 *__restrict__ order, const u32 *__restrict__ classes, const uint2 *__restrict__ chunk_list,
    u32 num_tiles)
{
    __shared__ u64 s[kMid + kMid / 16];
    const u32 chunks = classes[4];
    if (blockIdx.x < chunks) {
        const uint2 c = chunk_list[blockIdx.x];
        if (c.x >= num_tiles) return;
        const u64 beg = tile_offsets[c.x];
        const u64 len = tile_offsets[c.x + 1] - beg;
        const u64 c0 = (u64)c.y * kMid;
        if (c0 >= len) return;                              // cannot happen with a consistent table
        const u32 n = (u32)(len - c0 < (u64)kMid ? len - c0 : (u64)kMid);
        if (n >= 2) sort_pairs_in_lds<kMidThreads, kMidItems>(keys, vals, beg + c0, n, c.x, s);
        return;
    }
    const u32 k = blockIdx.x - chunks;
    const u32 first = classes[0] + classes[3];
    if (k >= classes[1] || first + k >= num_tiles) return;
    const u32 tile = order[first + k];
    if (tile >= num_tiles) return;
    const u64 beg = tile_offsets[tile];
    const u64 len = tile_offsets[tile + 1] - beg;
    if (len < 2 || len > (u64)kMid) return;                 // cannot happen with a consistent table
    sort_pairs_in_lds<kMidThreads, kMidItems>(keys, vals, beg, (u32)len, tile, s);
}

// Lists of kSmallCap + 1 .. kLow pairs, one workgroup each, and before them the first merge round
// of the long lists (runs of kMid pairs, pair buffers -> alternate buffers), kLow outputs per
// workgroup: a fixed number of workgroups walks the segments.
constexpr u32 kMergeBlocks1 = 1024, kMergeBlocks2 = 2048;
__global__ __launch_bounds__(kLowThreads) void tile_sort_low_kernel(
    u64 *__restrict__ keys, u32 *__restrict__ vals, u64 *__restrict__ keys_alt, u32 *__restrict__ vals_alt,
    const u64 *__restrict__ tile_offsets, const u32 *__restrict__ order, const u32 *__restrict__ classes,
    const uint2 *__restrict__ chunk_list, u32 num_tiles, u32 merge_blocks)
{
    constexpr u32 CAP = kLowThreads * kLowItems;
    constexpr u32 kPerChunk = kMid / CAP;                   // output segments per chunk
    __shared__ u64 s[CAP + CAP / 16];
    __shared__ u64 s_split[2];
    if (blockIdx.x < merge_blocks) {
        const u64 segments = (u64)classes[4] * kPerChunk;
        for (u64 g = blockIdx.x; g < segments; g += merge_blocks) {
            const uint2 c = chunk_list[g / kPerChunk];
            if (c.x >= num_tiles) continue;
            const u64 beg = tile_offsets[c.x];
            const u64 len = tile_offsets[c.x + 1] - beg;
            merge_segment<kLowThreads, kLowItems>(keys + beg, vals + beg, keys_alt + beg, vals_alt + beg, len,
                                                  (u64)kMid, (u64)c.y * kPerChunk + g % kPerChunk, c.x, s, s_split);
        }
        return;
    }
    const u32 k = blockIdx.x - merge_blocks;
    const u32 first = classes[0] + classes[3] + classes[1];
    if (k >= classes[2] || first + k >= num_tiles) return;
    const u32 tile = order[first + k];
    if (tile >= num_tiles) return;
    const u64 beg = tile_offsets[tile];
    const u64 len = tile_offsets[tile + 1] - beg;
    if (len < 2 || len > (u64)CAP) return;                  // cannot happen with a consistent table
    sort_pairs_in_lds<kLowThreads, kLowItems>(keys, vals, beg, (u32)len, tile, s);
}

// Short lists (2 .. 512 pairs): one wavefront each, walking `order` from its short end.  Before
// them the second and last merge round of the long lists (runs of 2 * kMid pairs, alternate
// buffers -> pair buffers; a list of one such run is copied), kSmallCap outputs per segment.
__global__ __launch_bounds__(kSmallThreads) void tile_sort_small_kernel(
    u64 *__restrict__ keys, u32 *__restrict__ vals, const u64 *__restrict__ keys_alt, const u32 *__restrict__ vals_alt,
    const u64 *__restrict__ tile_offsets, const u32 *__restrict__ order, const u32 *__restrict__ classes,
    const uint2 *__restrict__ chunk_list, u32 num_tiles, u32 merge_blocks)
{
    constexpr u32 kPerChunk = kMid / kSmallCap;
    __shared__ u64 s[kSmallCap + kSmallCap / 16];
    __shared__ u64 s_split[2];
    if (blockIdx.x < merge_blocks) {
        const u64 segments = (u64)classes[4] * kPerChunk;
        for (u64 g = blockIdx.x; g < segments; g += merge_blocks) {
            const uint2 c = chunk_list[g / kPerChunk];
            if (c.x >= num_tiles) continue;
            const u64 beg = tile_offsets[c.x];
            const u64 len = tile_offsets[c.x + 1] - beg;
            merge_segment<kSmallThreads, kSmallItems>(keys_alt + beg, vals_alt + beg, keys + beg, vals + beg, len,
                                                      2 * (u64)kMid, (u64)c.y * kPerChunk + g % kPerChunk, c.x, s, s_split);
        }
        return;
    }
    const u32 k = blockIdx.x - merge_blocks;
    if (k >= num_tiles) return;
    const u32 tile = order[num_tiles - 1 - k];
    if (tile >= num_tiles) return;
    const u64 beg = tile_offsets[tile];
    const u64 len = tile_offsets[tile + 1] - beg;
    if (len < 2 || len > (u64)kSmallCap) return;
    // fewer elements per lane for shorter lists: all 64 lanes work in every merge round
    if (len <= 2u * kSmallThreads) sort_pairs_in_lds<kSmallThreads, 2u>(keys, vals, beg, (u32)len, tile, s);
    else if (len <= 4u * kSmallThreads) sort_pairs_in_lds<kSmallThreads, 4u>(keys, vals, beg, (u32)len, tile, s);
    else sort_pairs_in_lds<kSmallThreads, kSmallItems>(keys, vals, beg, (u32)len, tile, s);
}

// ---------------------------------------------------------------- lists beyond kHuge pairs
// One workgroup of 1024 threads per tile whose list is longer than kHuge pairs (the front of
// `order`): chunks of kHuge pairs are sorted in LDS, then merged pairwise (run length
// doubling) between the two pair buffers, kHuge outputs at a time: sixteen wavefronts find the
// splits of sixteen output segments, then each segment's two input windows are staged in
// LDS, merged there and written out coalesced.  The result ends in keys/vals.
__global__ __launch_bounds__(kHugeThreads) void tile_sort_huge_kernel(
    u64 *__restrict__ keys, u32 *__restrict__ vals, u64 *__restrict__ keys_alt, u32 *__restrict__ vals_alt,
    const u64 *__restrict__ tile_offsets, const u32 *__restrict__ order, const u32 *__restrict__ classes,
    u32 num_tiles)
{
    __shared__ u64 s[kHuge + kHuge / 16];
    __shared__ u64 s_split[kHugeThreads / kWave][2];
    if (blockIdx.x >= classes[0] || blockIdx.x >= num_tiles) return;
    const u32 tile = order[blockIdx.x];
    if (tile >= num_tiles) return;
    const u64 beg = tile_offsets[tile];
    const u64 L = tile_offsets[tile + 1] - beg;
    if (L <= (u64)kHuge) return;                            // cannot happen with a consistent table
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    constexpr u32 kWaves = kHugeThreads / kWave;

    // an odd number of merge rounds: the chunk sorts write to the alternate buffers, so that the
    // last round ends in keys/vals either way
    u32 rounds = 0;
    for (u64 run = kHuge; run < L; run <<= 1) ++rounds;
    const bool start_alt = (rounds & 1u) != 0u;
    u64 *k0 = start_alt ? keys_alt : keys, *k1 = start_alt ? keys : keys_alt;
    u32 *v0 = start_alt ? vals_alt : vals, *v1 = start_alt ? vals : vals_alt;
    for (u64 c0 = 0; c0 < L; c0 += kHuge) {
        const u32 n = (u32)(L - c0 < (u64)kHuge ? L - c0 : (u64)kHuge);
        if (n >= 2) sort_pairs_in_lds<kHugeThreads, kHugeItems>(keys, vals, beg + c0, n, tile, s, k0, v0);
        else if (start_alt && tid == 0) { k0[beg + c0] = keys[beg + c0]; v0[beg + c0] = vals[beg + c0]; }
    }
    // the chunk sorts of this workgroup wrote the runs the merges read
    __threadfence_block();
    __syncthreads();

    u64 *sk = k0 + beg, *dk = k1 + beg;
    u32 *sv = v0 + beg, *dv = v1 + beg;
    const u64 hi_bits = (u64)tile << 32;
    const u64 nseg = (L + kHuge - 1) / kHuge;
    for (u64 run = kHuge; run < L; run <<= 1) {
        for (u64 seg0 = 0; seg0 < nseg; seg0 += kWaves) {
            {   // wavefront wv: the splits at both ends of output segment seg0 + wv
                const u64 seg = seg0 + wv;
                if (seg < nseg) {
                    const u64 o = seg * kHuge;
                    const u64 a0 = (o / (2 * run)) * (2 * run);
                    const u64 a1 = a0 + run < L ? a0 + run : L;
                    const u64 b1 = a0 + 2 * run < L ? a0 + 2 * run : L;
                    const u64 oe = o + kHuge < b1 ? o + kHuge : b1;
                    const u64 i0 = wave_merge_split(sk, sv, a0, a1, b1, o - a0, lane);
                    const u64 i1 = wave_merge_split(sk, sv, a0, a1, b1, oe - a0, lane);
                    if (lane == 0) { s_split[wv][0] = i0; s_split[wv][1] = i1; }
                }
            }
            __syncthreads();
            for (u32 w = 0; w < kWaves && seg0 + w < nseg; ++w) {
                const u64 o = (seg0 + w) * kHuge;
                const u64 a0 = (o / (2 * run)) * (2 * run);
                const u64 a1 = a0 + run < L ? a0 + run : L;
                const u64 b1 = a0 + 2 * run < L ? a0 + 2 * run : L;
                const u64 oe = o + kHuge < b1 ? o + kHuge : b1;
                const u64 i0 = s_split[w][0], i1 = s_split[w][1];
                const u64 j0 = (o - a0) - i0;                // elements of B before the segment
                const u32 la = (u32)(i1 - i0), total = (u32)(oe - o);
                // stage A[i0, i1) then B[j0, j0 + total - la) as composites
                for (u32 p = tid; p < total; p += kHugeThreads) {
                    const u64 src = p < la ? a0 + i0 + p : a1 + j0 + (p - la);
                    s[ts_slot(p)] = (sk[src] << 32) | (u64)sv[src];
                }
                __syncthreads();
                const u32 o0 = tid * kHugeItems;
                u64 e[kHugeItems];
                if (o0 < total) merge_from_lds<kHugeItems>(s, 0u, la, total, o0, e);
                __syncthreads();
                if (o0 < total) {
#pragma unroll
                    for (u32 k = 0; k < kHugeItems; ++k)
                        if (o0 + k < total) s[ts_slot(o0 + k)] = e[k];
                }
                __syncthreads();
                for (u32 p = tid; p < total; p += kHugeThreads) {
                    const u64 c = s[ts_slot(p)];
                    dk[o + p] = hi_bits | (c >> 32);
                    dv[o + p] = (u32)c;
                }
                __syncthreads();
            }
        }
        // this workgroup's writes of the round are read by all its threads in the next one
        __threadfence_block();
        __syncthreads();
        u64 *tk = sk; sk = dk; dk = tk;
        u32 *tv = sv; sv = dv; dv = tv;
    }
}

// ---------------------------------------------------------------- launcher
static inline u32 grid_for(u64 work_items, u32 cap)
{
    if (work_items < 1) work_items = 1;
    return (u32)(work_items < (u64)cap ? work_items : (u64)cap);
}

hipError_t launch_bin_sort(const lmk_gs_projected &proj, u32 n, const ProjParams &pp, const lmk_gs_binned &out,
                           char *scratch, const ScratchLayout &L, hipStream_t stream)
{
    ScratchHeader *header = reinterpret_cast<ScratchHeader *>(scratch + L.header);
    const u32 *block_sums = reinterpret_cast<const u32 *>(scratch + L.block_sums);
    u64 *block_offsets = reinterpret_cast<u64 *>(scratch + L.block_offsets);
    const u64 *group_totals = reinterpret_cast<const u64 *>(scratch + L.group_totals);
    u64 *digit_totals = reinterpret_cast<u64 *>(scratch + L.digit_totals);
    u32 *table = reinterpret_cast<u32 *>(scratch + L.table);
    u64 *offsets = reinterpret_cast<u64 *>(scratch + L.offsets);
    u32 *order = reinterpret_cast<u32 *>(scratch + L.order);
    u32 *classes = reinterpret_cast<u32 *>(scratch + L.classes);
    u32 *big_idx = reinterpret_cast<u32 *>(scratch + L.big_idx);
    u64 *big_off = reinterpret_cast<u64 *>(scratch + L.big_off);
    const u32 num_tiles = pp.tiles_x * pp.tiles_y;
    const SortPlan plan = sort_plan(num_tiles);

    // ping-pong so that the last pass lands in keys/vals
    u64 *kin = (plan.passes & 1u) ? out.keys_alt : out.keys;
    u32 *vin = (plan.passes & 1u) ? out.vals_alt : out.vals;
    u64 *kout = (plan.passes & 1u) ? out.keys : out.keys_alt;
    u32 *vout = (plan.passes & 1u) ? out.vals : out.vals_alt;

    if (L.pre_blocks > 0) {
        // the deferred primitives are expanded by a fixed grid of wavefronts striding over the list
        const u32 big_grid = kGiantBlocks + (L.pre_blocks < 2048u ? L.pre_blocks : 2048u);
        if (pp.cam.binning == 1u) {
            hipLaunchKernelGGL(emit_tight_kernel, dim3(L.pre_blocks), dim3(kPreBlock), 0, stream,
                               proj.tiles_touched, reinterpret_cast<const ushort4 *>(proj.rect), proj.depth,
                               block_sums, block_offsets, group_totals, n, pp.tiles_x, out.capacity, kin, vin, proj.offsets, header,
                               big_idx, big_off, digit_totals, reinterpret_cast<const u32 *>(scratch + L.tile_masks));
            hipLaunchKernelGGL(emit_deferred_kernel<true>, dim3(big_grid), dim3(kPreBlock), 0, stream,
                               reinterpret_cast<const ushort4 *>(proj.rect), proj.depth,
                               reinterpret_cast<const float4 *>(proj.feat), pp, pp.tiles_x, out.capacity,
                               kin, vin, header, big_idx, big_off, n);
        } else {
            hipLaunchKernelGGL(emit_kernel, dim3(L.pre_blocks), dim3(kPreBlock), 0, stream,
                               proj.tiles_touched, reinterpret_cast<const ushort4 *>(proj.rect), proj.depth,
                               block_sums, block_offsets, group_totals, n, pp.tiles_x, out.capacity, kin, vin, proj.offsets, header,
                               big_idx, big_off, digit_totals);
            hipLaunchKernelGGL(emit_deferred_kernel<false>, dim3(big_grid), dim3(kPreBlock), 0, stream,
                               reinterpret_cast<const ushort4 *>(proj.rect), proj.depth,
                               reinterpret_cast<const float4 *>(proj.feat), pp, pp.tiles_x, out.capacity,
                               kin, vin, header, big_idx, big_off, n);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }

    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // enough resident workgroups to fill 256 CUs several times over; each loops over sort tiles
    const u32 grid = grid_for(L.sort_tiles, 256u * 16u);
    const bool many = sort_items(out.capacity) == kSortItemsMany;
    for (u32 p = 0; p < plan.passes; ++p) {
        u64 *totals = digit_totals + (size_t)p * kTotalCopies * kMaxRadix;
        if (many)
            hipLaunchKernelGGL(radix_hist_kernel<kSortItemsMany>, dim3(grid), dim3(kSortThreads), 0, stream,
                               kin, header, out.capacity, plan.shift[p], plan.bits[p], table, L.sort_tiles, totals);
        else
            hipLaunchKernelGGL(radix_hist_kernel<kSortItemsFew>, dim3(grid), dim3(kSortThreads), 0, stream,
                               kin, header, out.capacity, plan.shift[p], plan.bits[p], table, L.sort_tiles, totals);
        hipLaunchKernelGGL(radix_scan_kernel, dim3(1u << plan.bits[p]), dim3(kSortThreads), 0, stream,
                           header, out.capacity, table, offsets, L.sort_tiles, totals, sort_tile_pairs(out.capacity));
        if (many)
            hipLaunchKernelGGL(radix_scatter_kernel<kSortItemsMany>, dim3(grid), dim3(kSortThreads), 0, stream,
                               kin, vin, kout, vout, header, out.capacity, plan.shift[p], plan.bits[p],
                               offsets, L.sort_tiles);
        else
            hipLaunchKernelGGL(radix_scatter_kernel<kSortItemsFew>, dim3(grid), dim3(kSortThreads), 0, stream,
                               kin, vin, kout, vout, header, out.capacity, plan.shift[p], plan.bits[p],
                               offsets, L.sort_tiles);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        u64 *tk = kin; kin = kout; kout = tk;
        u32 *tv = vin; vin = vout; vout = tv;
    }
    // after the last swap `kin` is the partitioned buffer == out.keys
    const u32 rgrid = grid_for((out.capacity + 255) / 256, 256u * 16u);
    hipLaunchKernelGGL(tile_ranges_kernel, dim3(rgrid), dim3(256), 0, stream,
                       out.keys, header, out.capacity, num_tiles, out.tile_offsets,
                       n == 0 ? proj.offsets : nullptr);
    uint2 *chunk_list = reinterpret_cast<uint2 *>(scratch + L.chunk_list);
    hipLaunchKernelGGL(tile_order_kernel, dim3(1), dim3(1024), 0, stream,
                       out.tile_offsets, num_tiles, order, out.tile_order, classes, chunk_list,
                       out.capacity / 2048 + 2);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    // The lists beyond kHuge pairs first (few workgroups that run long), then by falling length.
    // The grids are upper bounds from the capacity, surplus workgroups leave at once: a list of
    // the class above kHuge / kLow / kSmallCap pairs, and likewise every chunk of a long list,
    // counts for more than that many pairs.
    auto at_most = [](u64 a, u64 b) { return (u32)(a < b ? a : b); };
    const u32 max_huge = at_most(out.capacity / (kHuge + 1) + 1, num_tiles);
    const u32 max_mid = at_most(out.capacity / (kLowThreads * kLowItems + 1) + 1, 4ull * num_tiles);
    const u32 max_low = at_most(out.capacity / (kSmallCap + 1) + 1, num_tiles);
    const u32 merge1 = at_most(2ull * max_mid, kMergeBlocks1), merge2 = at_most(8ull * max_mid, kMergeBlocks2);
    hipLaunchKernelGGL(tile_sort_huge_kernel, dim3(max_huge), dim3(kHugeThreads), 0, stream,
                       out.keys, out.vals, out.keys_alt, out.vals_alt, out.tile_offsets, order, classes, num_tiles);
    hipLaunchKernelGGL(tile_sort_mid_kernel, dim3(max_mid), dim3(kMidThreads), 0, stream,
                       out.keys, out.vals, out.tile_offsets, order, classes, chunk_list, num_tiles);
    hipLaunchKernelGGL(tile_sort_low_kernel, dim3(merge1 + max_low), dim3(kLowThreads), 0, stream,
                       out.keys, out.vals, out.keys_alt, out.vals_alt, out.tile_offsets, order, classes,
                       chunk_list, num_tiles, merge1);
    hipLaunchKernelGGL(tile_sort_small_kernel, dim3(merge2 + num_tiles), dim3(kSmallThreads), 0, stream,
                       out.keys, out.vals, out.keys_alt, out.vals_alt, out.tile_offsets, order, classes,
                       chunk_list, num_tiles, merge2);
    return hipGetLastError();
}

}  // namespace lmk
