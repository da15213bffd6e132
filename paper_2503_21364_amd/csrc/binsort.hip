// Stage 2: duplication of primitives into (tile | depth) keys, sort of the pairs into
// (tile, depth bits, index) order, per-tile ranges (the "depth sorting ... at the granularity of
// tiles" of Sec. 2.2; duplication with keys is the second kernel named in Sec. 4.2.1).
//
// The sorted order is total -- (tile, depth bits, primitive index) has no ties -- so it does not
// matter in which order a tile's pairs arrive in the tile's slice of the buffers: the per-tile
// sort fixes it.  The pairs are therefore written straight into their tile's slice, never
// partitioned by a sort over the tile bits: count per tile, scan, then write on a second walk.
//
//   count    one workgroup per kBinBlock (2048) consecutive primitives.  A rectangle of up to 32 tiles (nearly
//            all of them) is walked by its own lane -- binning rule 0: every tile; rule 1: the kept
//            tiles, from the bit mask the projection kernel left -- and counted per tile in LDS.  A
//            scene in spatial order puts a workgroup's pairs into few tiles, and the workgroup then
//            adds to the global per-tile counts with ONE returning atomic per tile it touched, not
//            per pair: the value returned is where its run starts inside that tile's slice.  The
//            (tile, start) list goes to memory for the emit kernel, at a place that follows from
//            the prefix sum over the workgroup pair counts which the projection stage left (a list
//            has at most one entry per pair).  Larger rectangles go to a list of their own.
//   count (large rectangles)  one wavefront per listed primitive (one workgroup beyond 2048 tiles)
//            walks its rectangle 64 tiles per step in row-major order (rule 1: with the
//            intersection test), one atomic per pair.  Lanes hold consecutive tiles, so the
//            atomics of one instruction fall into one or two cache lines and the memory side takes
//            them together (ten times the rate of scattered ones).  The close-up primitives of a
//            frame sit in a few workgroups; the list spreads them over the whole chip.
//   scan     one workgroup: the capacity check, exclusive prefix sum of the per-tile counts = the
//            per-tile ranges, a running position per tile for the listed primitives, the tiles by
//            descending list length with the size classes and the chunk list of the per-tile
//            sort; it leaves the counters zero.
//   emit     the same walks again.  A workgroup sets its LDS counters to range start + run start
//            for the tiles of its list and hands out positions from them.  A listed primitive
//            advances the tile's running position pair by pair, again with lane-consecutive
//            atomics, eight steps in flight.  What is written is the composite the list is
//            ordered by, depth bits << 32 | index.
//   tile sort  every tile's slice is sorted by that composite with a merge sort in LDS and
//            rewritten in its final form (key = tile << 32 | depth bits, value = index): one
//            wavefront for lists of up to 512 pairs, 256 threads up to 2048, 512 threads up to
//            4096.  A list of up to 16384 pairs is cut into 4096-pair chunks, sorted by
//            workgroups of the 512-thread launch and merged in two rounds between the two pair
//            buffers by workgroups of the 256-thread and the one-wavefront launch.  Lists beyond
//            that get a workgroup of 1024 threads each: 16384-pair chunks in LDS, then pairwise
//            merges through LDS-staged windows.
//
// Integer work, bound by HBM traffic, global atomic throughput and, in the per-tile sorts, by
// LDS bandwidth and vector issue.  Atomics on one address are served one after the other (about
// 12 ns each), so nothing here funnels every workgroup through one counter.  The kernels read the
// pair count from device memory, so the host never waits for it: grids are sized from the
// caller's capacity and surplus workgroups leave at once.  If D exceeds the capacity nothing is
// emitted: every range is empty, the status word says so and D tells the caller how much room a
// retry needs.
#include <type_traits>

#include "lmk_gs_internal.h"
#include "tile_test.h"

namespace lmk {

constexpr u32 kMaskArea = 32;       // rectangles whose kept tiles the projection kernel recorded as a bit mask

// ---------------------------------------------------------------- walking a primitive's tiles
// t / w and t % w for t < 2^22 (a tile grid has at most 2^22 tiles), 1 <= w <= 4096; inv_w = 1 / w
__device__ __forceinline__ void div_tiles(u32 t, u32 w, float inv_w, u32 &row, u32 &col)
{
    u32 q = (u32)((float)t * inv_w);            // within one of the quotient
    int r = (int)(t - q * w);
    if (r < 0) { q -= 1u; r += (int)w; }
    else if (r >= (int)w) { q += 1u; r -= (int)w; }
    row = q; col = (u32)r;
}

// A rectangle of up to kMaskArea tiles, walked by its own lane: f(tile id) for every tile that
// gets a pair, in row-major order.  Under binning rule 1 (TIGHT) those are the set bits of `mask`.
template <bool TIGHT, class F>
__device__ __forceinline__ void walk_small(ushort4 r, u32 area, u32 mask, u32 tiles_x, F &&f)
{
    const u32 w = (u32)r.z - (u32)r.x;
    const u32 inv_w = w ? (65536u + w - 1u) / w : 0u;       // slot / w == (slot * inv_w) >> 16 for slot < 32, w <= 32
    if (TIGHT) {
        while (mask) {
            const u32 slot = (u32)__builtin_ctz(mask);
            mask &= mask - 1u;
            const u32 row = (slot * inv_w) >> 16;
            f(((u32)r.y + row) * tiles_x + (u32)r.x + (slot - row * w));
        }
    } else {
        for (u32 slot = 0; slot < area; ++slot) {
            const u32 row = (slot * inv_w) >> 16;
            f(((u32)r.y + row) * tiles_x + (u32)r.x + (slot - row * w));
        }
    }
}

// One listed primitive, walked by a whole wavefront, 64 tiles of its rectangle per step in
// row-major order.  For every tile that gets a pair (under binning rule 1, TIGHT, every tile goes
// through the intersection test), first value = issue(tile, rank), then commit(tile, rank, value)
// -- kLargeBatch steps at a time, all their `issue` calls ahead of the first `commit`: `issue`
// starts a memory operation (a returning atomic) whose latency would otherwise be paid once per
// step, one after the other.  rank = the pair's number among those this wavefront found.
constexpr u32 kLargeBatch = 8;

// A rectangle shared by several wavefronts: wavefront `part` of `parts` takes batches part, part + parts, ...
template <bool TIGHT, class Issue, class Commit>
__device__ __forceinline__ void walk_large(ushort4 r, const float4 *__restrict__ feat_i, const ProjParams &pp,
                                           u32 lane, u32 part, u32 parts, Issue &&issue, Commit &&commit)
{
    const u32 w = (u32)r.z - (u32)r.x, area = w * ((u32)r.w - (u32)r.y);
    TileTest tt = make_tile_test(0.f, 0.f, 1.f, 0.f, 1.f, 0.f);
    if (TIGHT) {
        const float4 f0 = feat_i[0], f1 = feat_i[1];
        tt = make_tile_test(f0.x, f0.y, f0.z, f0.w, f1.x, opacity_tau(pp, f1.y));
    }
    const float inv_w = 1.0f / (float)w;
    u32 running = 0;
    for (u32 t0 = part * kWave * kLargeBatch; t0 < area; t0 += parts * kWave * kLargeBatch) {   // area > 0 implies w > 0; wave-uniform
        bool keep[kLargeBatch];
        u32 tile[kLargeBatch], rank[kLargeBatch];
        u64 value[kLargeBatch];
#pragma unroll
        for (u32 b = 0; b < kLargeBatch; ++b) {
            keep[b] = false; tile[b] = 0; rank[b] = 0;
            if (t0 + b * kWave < area) {                        // wave-uniform
                const u32 t = t0 + b * kWave + lane;
                bool k = t < area;
                u32 row = 0, col = 0;
                if (k) div_tiles(t, w, inv_w, row, col);
                const u32 tx = (u32)r.x + col, ty = (u32)r.y + row;
                if (TIGHT && k) k = tile_kept(tt, tx, ty);
                const u64 m = __builtin_amdgcn_ballot_w64(k);
                keep[b] = k;
                tile[b] = ty * pp.tiles_x + tx;
                rank[b] = running + __builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u));
                running += (u32)__builtin_popcountll(m);
            }
        }
#pragma unroll
        for (u32 b = 0; b < kLargeBatch; ++b) value[b] = keep[b] ? issue(tile[b], rank[b]) : 0ull;
#pragma unroll
        for (u32 b = 0; b < kLargeBatch; ++b)
            if (keep[b]) commit(tile[b], rank[b], value[b]);
    }
}

// ---------------------------------------------------------------- count
// LDS_TILES > 0: the image has at most LDS_TILES tiles, rectangles of up to kMaskArea tiles are
// counted in LDS, larger ones listed.  LDS_TILES == 0 (images of more tiles): every primitive is
// listed.
// A workgroup takes kBinBlock consecutive primitives, kBinBlock / THREADS per thread (primitive
// tid + j THREADS in round j).  What bounds these kernels is the chain of memory round trips of a
// workgroup, so the compute unit should be full of wavefronts: with 32 KB of counters four
// workgroups fit, and four workgroups of 512 threads are all the wavefronts it can hold.
constexpr u32 kRunBits = 11;             // a workgroup's pairs in one tile, minus one, fit these many bits
static_assert(kBinBlock <= (1u << kRunBits), "(count - 1) of a run is packed into kRunBits bits");
template <u32 LDS_TILES> struct BinShape {
    static constexpr u32 kThreads = LDS_TILES == kLdsTilesSmall ? kBinBlock / 4u : 1024u;
    static constexpr u32 kPer = kBinBlock / kThreads;
    static constexpr u32 kWaves = kThreads / kWave;
    static constexpr u32 kRounds = LDS_TILES / kThreads;    // counters per thread
};
constexpr u32 kGiantArea = 2048;    // listed rectangles beyond this many tiles get a workgroup, not a wavefront

// Where the list of counting workgroup b starts: the pairs of all primitives before its own, from
// the two-level prefix sum the projection stage left (block_offsets inside a group of kScanGroup
// preprocess workgroups, plus the totals of the groups before).  Called by the whole workgroup
// ahead of a barrier; one partial sum per wavefront goes to s_part, list_first_finish adds them.
template <u32 THREADS>
__device__ __forceinline__ void list_first_start(const u64 *__restrict__ group_totals, u32 b, u64 *s_part,
                                                 u32 tid, u32 lane, u32 wv)
{
    const u32 groups_before = (b * (kBinBlock / kPreBlock)) / kScanGroup;
    u64 part = 0;
    for (u32 g = tid; g < groups_before; g += THREADS) part += group_totals[g];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_down(part, o, 64);
    if (lane == 0) s_part[wv] = part;
}
template <u32 WAVES>
__device__ __forceinline__ u64 list_first_finish(const u64 *__restrict__ block_offsets, u32 b, const u64 *s_part)
{
    u64 first = block_offsets[b * (kBinBlock / kPreBlock)];
#pragma unroll
    for (u32 k = 0; k < WAVES; ++k) first += s_part[k];
    return first;
}

template <u32 LDS_TILES, bool TIGHT>
__global__ __launch_bounds__(BinShape<LDS_TILES>::kThreads) void count_kernel(
    const u32 *__restrict__ tiles_touched, const ushort4 *__restrict__ rect, const u32 *__restrict__ tile_masks,
    u32 n, u32 tiles_x, u32 num_tiles, u32 *__restrict__ tile_count,
    ScratchHeader *__restrict__ header, u32 *__restrict__ big_idx,
    const u32 *__restrict__ block_sums, u32 pre_blocks,
    const u64 *__restrict__ block_offsets, const u64 *__restrict__ group_totals,
    u32 *__restrict__ bin_count, uint2 *__restrict__ list, u64 list_capacity)
{
    constexpr bool LDS = LDS_TILES > 0;
    constexpr u32 kThreads = BinShape<LDS_TILES>::kThreads, kPer = BinShape<LDS_TILES>::kPer;
    constexpr u32 kWaves = BinShape<LDS_TILES>::kWaves;
    constexpr u32 kRounds = LDS ? BinShape<LDS_TILES>::kRounds : 1;
    constexpr u32 kSmallMax = LDS ? kMaskArea : 0u;
    __shared__ u32 s_hist[LDS ? LDS_TILES : 1];
    __shared__ u32 s_next;
    __shared__ u32 s_wave[kWaves][2];
    __shared__ u32 s_base[2];
    __shared__ u64 s_part[kWaves];
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    {   // the projection stage counted the pairs of every 256 primitives: a workgroup none of whose
        // primitives was binned (culled, or a skipped voxel range) leaves without reading one
        u32 pairs = 0;
#pragma unroll
        for (u32 q = 0; q < kBinBlock / kPreBlock; ++q) {
            const u32 pb = blockIdx.x * (kBinBlock / kPreBlock) + q;
            pairs |= pb < pre_blocks ? block_sums[pb] : 0u;
        }
        if (pairs == 0u) {                                  // the same for the whole workgroup
            if (LDS && tid == 0) bin_count[blockIdx.x] = 0;
            return;
        }
    }
    // everything this thread will need is requested at once: one round trip to memory
    u32 cnt[kPer], mask[kPer];
    ushort4 r[kPer];
    bool any = false;
#pragma unroll
    for (u32 j = 0; j < kPer; ++j) {
        const u32 i = blockIdx.x * kBinBlock + j * kThreads + tid;
        cnt[j] = i < n ? tiles_touched[i] : 0u;
        r[j] = i < n ? rect[i] : make_ushort4(0, 0, 0, 0);
        mask[j] = (TIGHT && LDS && i < n) ? tile_masks[i] : 0u;
    }
    if (LDS) {
        list_first_start<kThreads>(group_totals, blockIdx.x, s_part, tid, lane, wv);
        for (u32 t = tid; t < num_tiles; t += kThreads) s_hist[t] = 0;
        if (tid == 0) s_next = 0;
    }
#pragma unroll
    for (u32 j = 0; j < kPer; ++j) any = any || cnt[j] != 0u;
    if (!__syncthreads_or(any)) {                           // nothing of this workgroup was binned
        if (LDS && tid == 0) bin_count[blockIdx.x] = 0;
        return;
    }
    u32 large_bits = 0, giant_bits = 0;                     // bit j: primitive j of this thread goes to the list
#pragma unroll
    for (u32 j = 0; j < kPer; ++j) {
        const u32 area = cnt[j] ? ((u32)r[j].z - (u32)r[j].x) * ((u32)r[j].w - (u32)r[j].y) : 0u;
        if (LDS && area > 0u && area <= kSmallMax) {
            walk_small<TIGHT>(r[j], area, mask[j], tiles_x, [&](u32 tile) {
                if (tile < num_tiles) atomicAdd(&s_hist[tile], 1u);     // a rectangle never leaves the grid; a corrupt one must not either
            });
        }
        if (area > kGiantArea) giant_bits |= 1u << j;
        else if (area > kSmallMax) large_bits |= 1u << j;
    }
    // the lists of the other primitives (wavefront-sized rectangles from the front of big_idx,
    // workgroup-sized ones from the back): one global atomic each per workgroup that has any
    const u32 my_large = (u32)__builtin_popcount(large_bits), my_giant = (u32)__builtin_popcount(giant_bits);
    if (__syncthreads_or((my_large | my_giant) != 0u)) {    // also: every LDS count above is done
        u32 incl = my_large, incl2 = my_giant;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const u32 v = __shfl_up(incl, o, 64), v2 = __shfl_up(incl2, o, 64);
            if ((int)lane >= o) { incl += v; incl2 += v2; }
        }
        if (lane == kWave - 1) { s_wave[wv][0] = incl; s_wave[wv][1] = incl2; }
        __syncthreads();
        u32 before = 0, total = 0, before2 = 0, total2 = 0;
#pragma unroll
        for (u32 k = 0; k < kWaves; ++k) {
            const u32 w = s_wave[k][0], w2 = s_wave[k][1];
            if (k < wv) { before += w; before2 += w2; }
            total += w; total2 += w2;
        }
        if (tid == 0) {
            s_base[0] = total ? atomicAdd(&header->big_count, total) : 0u;
            s_base[1] = total2 ? atomicAdd(&header->giant_count, total2) : 0u;
        }
        __syncthreads();
        u32 slot = s_base[0] + before + incl - my_large;
        u32 slot2 = s_base[1] + before2 + incl2 - my_giant;
#pragma unroll
        for (u32 j = 0; j < kPer; ++j) {
            const u32 i = blockIdx.x * kBinBlock + j * kThreads + tid;
            // the two lists hold one entry per primitive at most, n in all, and never meet
            if (large_bits & (1u << j)) { if (slot < n) big_idx[slot] = i; ++slot; }
            if (giant_bits & (1u << j)) { if (slot2 < n) big_idx[n - 1u - slot2] = i; ++slot2; }
        }
    }
    if (!LDS) return;
    // The tiles this workgroup touched, compacted to the front of s_hist as tile << kRunBits | (count - 1)
    // (a workgroup holds kBinBlock primitives and a primitive has one pair per tile at most): every
    // thread first reads its counters, then, all reads done, the entries are written.
    u32 c[kRounds];
#pragma unroll
    for (u32 k = 0; k < kRounds; ++k) {
        const u32 t = k * kThreads + tid;
        c[k] = t < num_tiles ? s_hist[t] : 0u;
    }
    __syncthreads();
#pragma unroll
    for (u32 k = 0; k < kRounds; ++k) {
        const u64 nz = __builtin_amdgcn_ballot_w64(c[k] != 0u);
        if (nz == 0ull) continue;                           // wave-uniform
        u32 at = 0;
        const int leader = (int)__builtin_ctzll(nz);
        if ((int)lane == leader) at = atomicAdd(&s_next, (u32)__builtin_popcountll(nz));
        at = __shfl(at, leader, 64);
        if (c[k] != 0u)
            s_hist[at + __builtin_amdgcn_mbcnt_hi((u32)(nz >> 32), __builtin_amdgcn_mbcnt_lo((u32)nz, 0u))] =
                ((k * kThreads + tid) << kRunBits) | ((c[k] - 1u) & ((1u << kRunBits) - 1u));
    }
    __syncthreads();
    const u32 touched = s_next;
    const u64 first = list_first_finish<kWaves>(block_offsets, blockIdx.x, s_part);
    if (tid == 0) bin_count[blockIdx.x] = touched;
    // one reservation per touched tile: the run of this workgroup starts where the tile's counter
    // stood; up to kFlush entries per thread with their atomics in flight together
    constexpr u32 kFlush = 4;
    for (u32 k0 = 0; k0 < touched; k0 += kFlush * kThreads) {
        u32 ent[kFlush], start[kFlush];
#pragma unroll
        for (u32 q = 0; q < kFlush; ++q) {
            const u32 k = k0 + q * kThreads + tid;
            ent[q] = k < touched ? s_hist[k] : 0u;
            start[q] = k < touched ? atomicAdd(&tile_count[ent[q] >> kRunBits], (ent[q] & ((1u << kRunBits) - 1u)) + 1u) : 0u;
        }
#pragma unroll
        for (u32 q = 0; q < kFlush; ++q) {
            const u32 k = k0 + q * kThreads + tid;
            if (k < touched && first + k < list_capacity) list[first + k] = make_uint2(ent[q] >> kRunBits, start[q]);
        }
    }
}

// Fixed grids stride over the deferred lists: the first kGiantBlocks workgroups take the
// workgroup-sized rectangles (their wavefronts share a rectangle batch by batch), the wavefronts of
// the others the wavefront-sized ones.
constexpr u32 kLargeThreads = 256, kLargeBlocks = 2048, kGiantBlocks = 1024;

// f(rectangle index, primitive index, part, parts) for every listed primitive this wavefront
// has a share of: workgroup `block` of `blocks`, THREADS threads each; the first `giant_blocks` of
// them take the list of workgroup-sized rectangles.
template <u32 THREADS, class F>
__device__ __forceinline__ void for_each_listed(const ScratchHeader *__restrict__ header, const u32 *__restrict__ big_idx,
                                                u32 n, u32 block, u32 blocks, u32 giant_blocks, u32 tid, F &&f)
{
    constexpr u32 kWaves = THREADS / kWave;
    if (block < giant_blocks) {
        u32 count = header->giant_count;
        if (count > n) count = n;                           // cannot happen: one entry per primitive at most
        for (u32 k = block; k < count; k += giant_blocks) { // uniform
            const u32 i = big_idx[n - 1u - k];
            if (i < n) f(i, tid / kWave, kWaves);
        }
    } else {
        const u32 wave = ((block - giant_blocks) * THREADS + tid) / kWave, waves = (blocks - giant_blocks) * kWaves;
        u32 count = header->big_count;
        if (count > n) count = n;
        for (u32 k = wave; k < count; k += waves) {         // wave-uniform
            const u32 i = big_idx[k];
            if (i < n) f(i, 0u, 1u);
        }
    }
}

template <bool TIGHT>
__global__ __launch_bounds__(kLargeThreads) void count_large_kernel(
    const ushort4 *__restrict__ rect, const float4 *__restrict__ feat, ProjParams pp, u32 n, u32 num_tiles,
    u32 *__restrict__ large_count, const ScratchHeader *__restrict__ header, const u32 *__restrict__ big_idx,
    u32 giant_blocks)
{
    const u32 lane = threadIdx.x & (kWave - 1);
    for_each_listed<kLargeThreads>(header, big_idx, n, blockIdx.x, gridDim.x, giant_blocks, threadIdx.x,
        [&](u32 i, u32 part, u32 parts) {
            walk_large<TIGHT>(rect[i], feat + (size_t)i * (LMK_GS_FEAT_STRIDE / 4), pp, lane, part, parts,
                [&](u32 tile, u32) -> u64 { if (tile < num_tiles) atomicAdd(&large_count[tile], 1u); return 0ull; },
                [&](u32, u32, u64) {});
        });
}

// ---------------------------------------------------------------- scan + order + size classes
// Two workgroups, each of which is a chain of memory round trips and barriers rather than data, so
// they run side by side.  Both: (1) D = sum of the per-tile counts; more than the buffers hold:
// status, and every list is treated as empty from here on.  Workgroup 0: (2) tile_offsets =
// exclusive prefix sum of the counts.  Workgroup 1: (3) tile ids by descending list length, bucketed by the bit length of (length - 1), so that
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
// The counters stay as they are until both workgroups are done with them; the first kernel of the
// per-tile sort leaves them zero for the next call.
// With SMALL (up to 8192 tiles) every thread reads its eight counters once and everything else works
// from registers and LDS.
constexpr u32 kSmallThreads = 64, kSmallItems = 8, kSmallCap = kSmallThreads * kSmallItems;   // 512
constexpr u32 kLowThreads = 256, kLowItems = 8;                                               // 2048
constexpr u32 kMidThreads = 512, kMidItems = 8, kMid = kMidThreads * kMidItems;               // 4096
constexpr u32 kHugeThreads = 1024, kHugeItems = 16, kHuge = kHugeThreads * kHugeItems;        // 16384
static_assert(kMid == kChunk, "the launch bounds on the host use kChunk");

__device__ __forceinline__ u32 length_bucket(u32 len)
{
    return len > 1u ? 32u - (u32)__builtin_clz(len - 1u) : 0u;   // len in (2^(b-1), 2^b]
}
constexpr u32 kSmallBucket = 9, kLowBucket = 11, kMidBucket = 12, kHugeBucket = 14;   // 2^9 = kSmallCap, 2^11 = kLow, 2^12 = kMid, 2^14 = kHuge

// Most tiles fall into a handful of buckets, and LDS atomics on one word are served one after
// the other: every bucket has kOrderCopies counters, picked by the low lane bits, so that the 64
// atomics of a wavefront spread over that many words.  An exclusive scan over
// [bucket][copy] turns the counts into the first slot of every (bucket, copy).
constexpr u32 kScanThreads = 1024, kScanItems = 8;
constexpr u32 kOrderCopies = 16, kOrderBuckets = 33, kOrderCounters = kOrderBuckets * kOrderCopies;
constexpr u32 kOrderStage = 32768;
static_assert(kOrderCounters <= 2 * kScanThreads, "the counters are scanned two per thread");
static_assert(kLdsTilesSmall == kScanThreads * kScanItems, "SMALL: one round of kScanItems tiles per thread");

template <bool SMALL>
__global__ __launch_bounds__(kScanThreads) void tile_scan_kernel(
    const u32 *__restrict__ tile_count, const u32 *__restrict__ large_count, u32 num_tiles, u64 capacity, ScratchHeader *__restrict__ header,
    u64 *__restrict__ tile_offsets, u32 *__restrict__ tile_cursor, u64 *__restrict__ prim_offsets_if_empty,
    u32 *__restrict__ order, u32 *__restrict__ order_copy, u32 *__restrict__ classes,
    uint2 *__restrict__ chunk_list, u64 chunk_capacity)
{
    constexpr u32 kWaves = kScanThreads / kWave;
    // the running positions of the emit kernel are 32 bits wide: absolute where every position
    // fits (they start at the tile's range start), else relative to the range start
    const bool wide = capacity > 0xffffffffull;
    __shared__ u64 s_sum[kWaves];
    __shared__ u32 s_cnt[kOrderCounters];
    __shared__ u32 s_long[2];                  // first long tile in `order`, number of long tiles
    __shared__ u32 s_wave[kWaves];
    // slots are scattered and one compute unit does all the address work: the order is put
    // together in LDS and written out in whole lines (images of up to kOrderStage tiles)
    __shared__ u32 s_order[SMALL ? kLdsTilesSmall : kOrderStage];
    __shared__ u32 s_len[SMALL ? kLdsTilesSmall : 1];      // SMALL: the list lengths, for the chunk list
    const bool staged = SMALL || num_tiles <= kOrderStage;
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;

    // ---- (1) D
    // a tile's list = the runs of the counting workgroups (tile_count) followed by the pairs of
    // the listed primitives (large_count)
    u32 mine8[kScanItems], runs8[kScanItems];  // SMALL: list length and length of the runs of tiles tid * kScanItems + j
    u64 part = 0;
    if (SMALL) {
#pragma unroll
        for (u32 j = 0; j < kScanItems; ++j) {
            const u32 t = tid * kScanItems + j;
            runs8[j] = t < num_tiles ? tile_count[t] : 0u;
            mine8[j] = runs8[j] + (t < num_tiles ? large_count[t] : 0u);
            part += mine8[j];
        }
    } else {
        for (u32 t = tid; t < num_tiles; t += kScanThreads) part += (u64)tile_count[t] + large_count[t];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_down(part, o, 64);
    if (lane == 0) s_sum[wv] = part;
    __syncthreads();
    u64 D = 0;
#pragma unroll
    for (u32 k = 0; k < kWaves; ++k) D += s_sum[k];
    const bool overflow = D > capacity;
    // two workgroups share the work: 0 writes D, the status and the ranges, 1 the order, the size
    // classes and the chunk list; both need the list lengths and D
    const bool ranges_part = blockIdx.x == 0;
    if (tid == 0 && ranges_part) {
        header->dup_count = D;
        header->status = overflow ? LMK_GS_ERR_CAPACITY : LMK_GS_OK;      // of this call; the frame's earlier calls do not count
        // with no primitives nothing else writes the one-entry prefix sum over the primitives
        if (prim_offsets_if_empty) prim_offsets_if_empty[0] = 0;
    }
    if (SMALL) {
#pragma unroll
        for (u32 j = 0; j < kScanItems; ++j) {
            if (overflow) { mine8[j] = 0u; runs8[j] = 0u; }
            s_len[tid * kScanItems + j] = mine8[j];
        }
    }
    __syncthreads();                           // s_sum is reused below

    // ---- (2) per-tile ranges: kScanItems consecutive tiles per thread, entry num_tiles = the end
    u64 carry = 0;
    for (u32 base = 0; ranges_part && base <= num_tiles; base += kScanThreads * kScanItems) {
        const u32 t0 = base + tid * kScanItems;
        u32 c[kScanItems], runs[kScanItems];
        u64 mine = 0;
#pragma unroll
        for (u32 j = 0; j < kScanItems; ++j) {
            if (SMALL) {
                c[j] = base == 0u ? mine8[j] : 0u;
                runs[j] = base == 0u ? runs8[j] : 0u;
            } else {
                const bool in = !overflow && t0 + j < num_tiles;
                runs[j] = in ? tile_count[t0 + j] : 0u;
                c[j] = runs[j] + (in ? large_count[t0 + j] : 0u);
            }
            mine += c[j];
        }
        u64 incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const u64 v = __shfl_up(incl, o, 64);
            if ((int)lane >= o) incl += v;
        }
        if (lane == kWave - 1) s_sum[wv] = incl;
        __syncthreads();
        u64 before = carry, total = carry;
#pragma unroll
        for (u32 k = 0; k < kWaves; ++k) {
            const u64 v = s_sum[k];
            if (k < wv) before += v;
            total += v;
        }
        u64 run = before + incl - mine;
#pragma unroll
        for (u32 j = 0; j < kScanItems; ++j) {
            if (t0 + j <= num_tiles) {
                tile_offsets[t0 + j] = run;
                tile_cursor[t0 + j] = (wide ? 0u : (u32)run) + runs[j];   // the listed primitives' pairs follow the runs
            }
            run += c[j];
        }
        carry = total;
        __syncthreads();                       // s_sum free again
    }

    if (ranges_part) return;

    // ---- (3) order and size classes.  Tile of (thread, round j): SMALL tid * kScanItems + j, else
    // base + j * kScanThreads + tid.
    const u32 copy = tid & (kOrderCopies - 1);
    for (u32 k = tid; k < kOrderCounters; k += kScanThreads) s_cnt[k] = 0;
    __syncthreads();
    const u32 sweep = SMALL ? 1u : kScanThreads * kScanItems;
    for (u32 base = 0; base < (SMALL ? 1u : num_tiles); base += sweep) {
#pragma unroll
        for (u32 j = 0; j < kScanItems; ++j) {
            const u32 t = SMALL ? tid * kScanItems + j : base + j * kScanThreads + tid;
            if (t < num_tiles) {
                const u32 b = length_bucket(SMALL ? mine8[j] : (overflow ? 0u : tile_count[t] + large_count[t]));
                atomicAdd(&s_cnt[(32 - b) * kOrderCopies + copy], 1u);      // long lists first
            }
        }
    }
    __syncthreads();
    // exclusive scan of the counters, two per thread
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
        const u32 huge = s_cnt[(32 - kHugeBucket) * kOrderCopies];
        const u32 lng = s_cnt[(32 - kMidBucket) * kOrderCopies];
        const u32 mid = s_cnt[(32 - kLowBucket) * kOrderCopies];
        const u32 low = s_cnt[(32 - kSmallBucket) * kOrderCopies];
        classes[0] = huge; classes[3] = lng - huge; classes[1] = mid - lng; classes[2] = low - mid;
        s_long[0] = huge; s_long[1] = lng - huge;
    }
    __syncthreads();
    for (u32 base = 0; base < (SMALL ? 1u : num_tiles); base += sweep) {
#pragma unroll
        for (u32 j = 0; j < kScanItems; ++j) {
            const u32 t = SMALL ? tid * kScanItems + j : base + j * kScanThreads + tid;
            if (t >= num_tiles) continue;
            const u32 b = length_bucket(SMALL ? mine8[j] : (overflow ? 0u : tile_count[t] + large_count[t]));
            const u32 slot = atomicAdd(&s_cnt[(32 - b) * kOrderCopies + copy], 1u);
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
        for (u32 k = tid; k < num_tiles; k += kScanThreads) {
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
    u32 chunk_carry = 0;
    for (u32 base = 0; base < long_count; base += kScanThreads) {
        const u32 k = base + tid;
        u32 tile = 0, nch = 0;
        if (k < long_count) {
            tile = staged ? s_order[long_first + k] : order[long_first + k];
            if (tile < num_tiles) nch = ((SMALL ? s_len[tile] : tile_count[tile] + large_count[tile]) + kMid - 1) / kMid;
        }
        u32 inc = nch;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const u32 v = __shfl_up(inc, o, 64);
            if ((int)lane >= o) inc += v;
        }
        __syncthreads();                       // s_wave free again
        if (lane == kWave - 1) s_wave[wv] = inc;
        __syncthreads();
        u32 bef = chunk_carry, total = chunk_carry;
        for (u32 w = 0; w < kWaves; ++w) {
            const u32 c = s_wave[w];
            if (w < wv) bef += c;
            total += c;
        }
        const u32 at = bef + inc - nch;
        for (u32 c = 0; c < nch; ++c)
            if ((u64)at + c < chunk_capacity) chunk_list[at + c] = make_uint2(tile, c);
        chunk_carry = total;
    }
    if (tid == 0) classes[4] = (u64)chunk_carry < chunk_capacity ? chunk_carry : (u32)chunk_capacity;
    // the counters are left as they are: the other workgroup may still be reading them; the first
    // kernel of the per-tile sort zeroes them
}

// ---------------------------------------------------------------- emit
// Workgroups [0, bin_blocks) repeat the walk of the small rectangles of their kBinBlock primitives; the
// LDS counters now start at the tile's range start + the workgroup's run start and hand out
// positions.  The workgroups behind them walk the listed primitives and advance the tiles'
// running positions pair by pair.
// WIDE: positions need 64 bits (capacity of 2^32 pairs or more): LDS counters and running
// positions are then relative to the tile's range start, which is read from memory for every pair.
template <u32 LDS_TILES, bool TIGHT, bool WIDE>
__global__ __launch_bounds__(BinShape<LDS_TILES>::kThreads) void emit_kernel(
    const u32 *__restrict__ tiles_touched, const ushort4 *__restrict__ rect, const float *__restrict__ depth,
    const float4 *__restrict__ feat, const u32 *__restrict__ tile_masks, u32 n, ProjParams pp, u32 num_tiles,
    const u64 *__restrict__ tile_offsets, u32 *__restrict__ tile_cursor, const ScratchHeader *__restrict__ header,
    const u32 *__restrict__ big_idx, const u64 *__restrict__ block_offsets, const u64 *__restrict__ group_totals,
    const u32 *__restrict__ bin_count, const uint2 *__restrict__ list, u64 list_capacity,
    u32 bin_blocks, u32 giant_blocks, u64 capacity, u64 *__restrict__ keys)
{
    constexpr bool LDS = LDS_TILES > 0;
    constexpr u32 kThreads = BinShape<LDS_TILES>::kThreads, kPer = BinShape<LDS_TILES>::kPer;
    constexpr u32 kWaves = BinShape<LDS_TILES>::kWaves;
    __shared__ u32 s_cur[LDS ? LDS_TILES : 1];
    __shared__ u64 s_part[kWaves];
    if (header->status != LMK_GS_OK) return;                // more pairs than the buffers hold: nothing is emitted
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    if (blockIdx.x >= bin_blocks) {
        for_each_listed<kThreads>(header, big_idx, n, blockIdx.x - bin_blocks, gridDim.x - bin_blocks, giant_blocks, tid,
            [&](u32 i, u32 part, u32 parts) {
                const u64 comp = ((u64)__float_as_uint(depth[i]) << 32) | (u64)i;
                walk_large<TIGHT>(rect[i], feat + (size_t)i * (LMK_GS_FEAT_STRIDE / 4), pp, lane, part, parts,
                    [&](u32 tile, u32) -> u64 {
                        if (tile >= num_tiles) return ~0ull;
                        const u32 at = atomicAdd(&tile_cursor[tile], 1u);
                        return WIDE ? tile_offsets[tile] + at : (u64)at;
                    },
                    [&](u32, u32, u64 pos) { if (pos < capacity) keys[pos] = comp; });
            });
        return;
    }
    if (!LDS) return;                                       // every primitive is on a list
    const u32 entries = bin_count[blockIdx.x];
    if (entries == 0u) return;                              // the same for the whole workgroup
    list_first_start<kThreads>(group_totals, blockIdx.x, s_part, tid, lane, wv);
    // this thread's primitives: requested now, used after the counters are set up
    u32 cnt[kPer], mask[kPer], dbits[kPer];
    ushort4 r[kPer];
#pragma unroll
    for (u32 j = 0; j < kPer; ++j) {
        const u32 i = blockIdx.x * kBinBlock + j * kThreads + tid;
        cnt[j] = i < n ? tiles_touched[i] : 0u;
        r[j] = i < n ? rect[i] : make_ushort4(0, 0, 0, 0);
        mask[j] = (TIGHT && i < n) ? tile_masks[i] : 0u;
        dbits[j] = i < n ? __float_as_uint(depth[i]) : 0u;
    }
    __syncthreads();
    const u64 first = list_first_finish<kWaves>(block_offsets, blockIdx.x, s_part);
    for (u32 k = tid; k < entries; k += kThreads) {
        if (first + k >= list_capacity) break;
        const uint2 e = list[first + k];
        if (e.x < num_tiles) s_cur[e.x] = WIDE ? e.y : (u32)tile_offsets[e.x] + e.y;
    }
    __syncthreads();
#pragma unroll
    for (u32 j = 0; j < kPer; ++j) {
        const u32 area = cnt[j] ? ((u32)r[j].z - (u32)r[j].x) * ((u32)r[j].w - (u32)r[j].y) : 0u;
        if (area == 0u || area > kMaskArea) continue;
        const u64 comp = ((u64)dbits[j] << 32) | (u64)(blockIdx.x * kBinBlock + j * kThreads + tid);
        walk_small<TIGHT>(r[j], area, mask[j], pp.tiles_x, [&](u32 tile) {
            if (tile >= num_tiles) return;
            const u32 at = atomicAdd(&s_cur[tile], 1u);
            const u64 pos = WIDE ? tile_offsets[tile] + at : (u64)at;
            if (pos < capacity) keys[pos] = comp;
        });
    }
}

// ---------------------------------------------------------------- prefix sum over the primitives
// lmk_gs_projected.offsets (optional output): exclusive prefix sum of tiles_touched -- the scan
// inside every group of 256 primitives on top of the two-level prefix sum over the groups that the
// projection stage left.  Nothing else in this stage depends on it.
__global__ __launch_bounds__(kPreBlock) void prim_offsets_kernel(
    const u32 *__restrict__ tiles_touched, u32 n, const u64 *__restrict__ block_offsets,
    const u64 *__restrict__ group_totals, u64 *__restrict__ offsets)
{
    __shared__ u64 s_gpart[kPreBlock / kWave];
    __shared__ u32 s_wave[kPreBlock / kWave];
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 i = blockIdx.x * kPreBlock + tid;
    // totals of the groups before this workgroup's own
    const u32 groups_before = blockIdx.x / kScanGroup;
    u64 part = 0;
    for (u32 g = tid; g < groups_before; g += kPreBlock) part += group_totals[g];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_down(part, o, 64);
    if (lane == 0) s_gpart[wv] = part;
    const u32 cnt = i < n ? tiles_touched[i] : 0u;
    u32 incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const u32 t = __shfl_up(incl, o, 64);
        if ((int)lane >= o) incl += t;
    }
    if (lane == kWave - 1) s_wave[wv] = incl;
    __syncthreads();
    u64 base = block_offsets[blockIdx.x];
    u32 wave_base = 0, total = 0;
#pragma unroll
    for (u32 k = 0; k < kPreBlock / kWave; ++k) {
        base += s_gpart[k];
        const u32 w = s_wave[k];
        if (k < wv) wave_base += w;
        total += w;
    }
    if (i < n) offsets[i] = base + wave_base + incl - cnt;
    if (i == n - 1) offsets[n] = base + total;
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

// On entry keys[beg .. beg + n) holds what the emit kernel wrote: depth bits << 32 | primitive index,
// the composite the list is ordered by.  On return keys/vals (or keys_out/vals_out) hold the
// sorted pairs in their final form, key = tile << 32 | depth bits, value = primitive index.
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
    // each thread's ITEMS consecutive composites; beyond n the maximum value, which sorts to the end
    u64 e[ITEMS];
#pragma unroll
    for (u32 k = 0; k < ITEMS; ++k)
        e[k] = o0 + k < n ? keys[beg + o0 + k] : ~0ull;
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
        sort_pairs_in_lds<kMidThreads, kMidItems>(keys, vals, beg + c0, n, c.x, s);     // n >= 1
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

// Short lists (1 .. 512 pairs): one wavefront each, walking `order` from its short end.  Before
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
    if (len < 1 || len > (u64)kSmallCap) return;
    if (len == 1) {                                         // nothing to sort: only the pair's form changes
        if (threadIdx.x == 0) {
            const u64 c = keys[beg];
            keys[beg] = ((u64)tile << 32) | (c >> 32); vals[beg] = (u32)c;
        }
        return;
    }
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
    u32 num_tiles, ScratchHeader *__restrict__ header, u32 *__restrict__ tile_count)
{
    __shared__ u64 s[kHuge + kHuge / 16];
    __shared__ u64 s_split[kHugeThreads / kWave][2];
    // the scan has read the per-tile counters (both halves) and the emit kernel has consumed the
    // deferred list: leave them empty for the next call
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) { header->big_count = 0; header->giant_count = 0; }
        for (u32 t = threadIdx.x; t < 2u * (num_tiles + 1u); t += kHugeThreads) tile_count[t] = 0;
    }
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
        else if (tid == 0) {                                 // a chunk of one pair: only its form changes
            const u64 c = keys[beg + c0];
            k0[beg + c0] = ((u64)tile << 32) | (c >> 32); v0[beg + c0] = (u32)c;
        }
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
hipError_t launch_bin_sort(const lmk_gs_projected &proj, u32 n, const ProjParams &pp, const lmk_gs_binned &out,
                           char *scratch, const ScratchLayout &L, hipStream_t stream)
{
    ScratchHeader *header = reinterpret_cast<ScratchHeader *>(scratch + L.header);
    const u32 num_tiles = pp.tiles_x * pp.tiles_y;
    u32 *tile_count = reinterpret_cast<u32 *>(scratch + L.tile_count);
    u32 *large_count = tile_count + (num_tiles + 1);
    const u64 *block_offsets = reinterpret_cast<const u64 *>(scratch + L.block_offsets);
    const u64 *group_totals = reinterpret_cast<const u64 *>(scratch + L.group_totals);
    const u32 *tile_masks = reinterpret_cast<const u32 *>(scratch + L.tile_masks);
    u32 *bin_count = reinterpret_cast<u32 *>(scratch + L.bin_count);
    u32 *tile_cursor = reinterpret_cast<u32 *>(scratch + L.tile_cursor);
    u32 *big_idx = reinterpret_cast<u32 *>(scratch + L.big_idx);
    u32 *order = reinterpret_cast<u32 *>(scratch + L.order);
    u32 *classes = reinterpret_cast<u32 *>(scratch + L.classes);
    uint2 *chunk_list = reinterpret_cast<uint2 *>(scratch + L.chunk_list);
    const ushort4 *rect = reinterpret_cast<const ushort4 *>(proj.rect);
    const float4 *feat = reinterpret_cast<const float4 *>(proj.feat);
    // the (tile, start) lists of the counting workgroups live in the alternate key buffer, which
    // nothing else uses before the merge rounds of the per-tile sort; a list has at most one entry
    // per pair of its workgroup and starts at the number of pairs before the workgroup
    uint2 *list = reinterpret_cast<uint2 *>(out.keys_alt);
    const bool tight = pp.cam.binning == 1u;
    const bool wide = out.capacity > 0xffffffffull;
    const u32 lds_tiles = num_tiles <= kLdsTilesSmall ? kLdsTilesSmall : (num_tiles <= kLdsTilesLarge ? kLdsTilesLarge : 0u);
    const u32 bin_threads = lds_tiles == kLdsTilesSmall ? BinShape<kLdsTilesSmall>::kThreads : BinShape<kLdsTilesLarge>::kThreads;
    // the listed primitives are walked by fixed grids striding over the two lists: as workgroups of
    // kLargeThreads threads in the counting pass, as workgroups of the emit kernel behind its own
    const u32 large_blocks = 4u * L.bin_blocks < kLargeBlocks ? 4u * L.bin_blocks : kLargeBlocks;
    const u32 giant_blocks = L.bin_blocks < kGiantBlocks ? L.bin_blocks : kGiantBlocks;
    const u32 large_blocks_emit = (large_blocks * kLargeThreads + bin_threads - 1) / bin_threads;
    hipError_t e;

    if (L.bin_blocks > 0) {
        auto count = [&](auto kernel) {
            hipLaunchKernelGGL(kernel, dim3(L.bin_blocks), dim3(bin_threads), 0, stream,
                               proj.tiles_touched, rect, tile_masks, n, pp.tiles_x, num_tiles, tile_count, header, big_idx,
                               reinterpret_cast<const u32 *>(scratch + L.block_sums), L.pre_blocks,
                               block_offsets, group_totals, bin_count, list, out.capacity);
        };
        if (lds_tiles == kLdsTilesSmall) { if (tight) count(count_kernel<kLdsTilesSmall, true>); else count(count_kernel<kLdsTilesSmall, false>); }
        else if (lds_tiles == kLdsTilesLarge) { if (tight) count(count_kernel<kLdsTilesLarge, true>); else count(count_kernel<kLdsTilesLarge, false>); }
        else { if (tight) count(count_kernel<0u, true>); else count(count_kernel<0u, false>); }
        if (tight)
            hipLaunchKernelGGL(count_large_kernel<true>, dim3(giant_blocks + large_blocks), dim3(kLargeThreads), 0, stream,
                               rect, feat, pp, n, num_tiles, large_count, header, big_idx, giant_blocks);
        else
            hipLaunchKernelGGL(count_large_kernel<false>, dim3(giant_blocks + large_blocks), dim3(kLargeThreads), 0, stream,
                               rect, feat, pp, n, num_tiles, large_count, header, big_idx, giant_blocks);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (num_tiles <= kLdsTilesSmall)
        hipLaunchKernelGGL(tile_scan_kernel<true>, dim3(2), dim3(kScanThreads), 0, stream,
                           tile_count, large_count, num_tiles, out.capacity, header, out.tile_offsets, tile_cursor,
                           n == 0 ? proj.offsets : nullptr, order, out.tile_order, classes, chunk_list,
                           out.capacity / 2048 + 2);
    else
        hipLaunchKernelGGL(tile_scan_kernel<false>, dim3(2), dim3(kScanThreads), 0, stream,
                           tile_count, large_count, num_tiles, out.capacity, header, out.tile_offsets, tile_cursor,
                           n == 0 ? proj.offsets : nullptr, order, out.tile_order, classes, chunk_list,
                           out.capacity / 2048 + 2);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (L.bin_blocks > 0) {
        auto emit = [&](auto kernel) {
            hipLaunchKernelGGL(kernel, dim3(L.bin_blocks + giant_blocks + large_blocks_emit), dim3(bin_threads), 0, stream,
                               proj.tiles_touched, rect, proj.depth, feat, tile_masks, n, pp, num_tiles,
                               out.tile_offsets, tile_cursor, header, big_idx, block_offsets, group_totals,
                               bin_count, list, out.capacity, L.bin_blocks, giant_blocks, out.capacity, out.keys);
        };
        auto emit_for = [&](auto lds_tag) {
            constexpr u32 LT = decltype(lds_tag)::value;
            if (tight) { if (wide) emit(emit_kernel<LT, true, true>); else emit(emit_kernel<LT, true, false>); }
            else { if (wide) emit(emit_kernel<LT, false, true>); else emit(emit_kernel<LT, false, false>); }
        };
        if (lds_tiles == kLdsTilesSmall) emit_for(std::integral_constant<u32, kLdsTilesSmall>());
        else if (lds_tiles == kLdsTilesLarge) emit_for(std::integral_constant<u32, kLdsTilesLarge>());
        else emit_for(std::integral_constant<u32, 0u>());
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (proj.offsets) {
            hipLaunchKernelGGL(prim_offsets_kernel, dim3(L.pre_blocks), dim3(kPreBlock), 0, stream,
                               proj.tiles_touched, n, block_offsets, group_totals, proj.offsets);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
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
                       out.keys, out.vals, out.keys_alt, out.vals_alt, out.tile_offsets, order, classes, num_tiles, header,
                       tile_count);
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
