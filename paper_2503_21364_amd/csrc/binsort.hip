// Stage 2: duplication of primitives into (tile | depth) keys, stable LSD radix
// sort of the pairs, per-tile range extraction (the "depth sorting ... at the
// granularity of tiles" of Sec. 2.2; duplication with keys is the second
// kernel named in Sec. 4.2.1).
//
// All of it is integer work bound by HBM traffic.  The kernels read the pair
// count D from device memory, so the host never waits for it: grids are sized
// from the caller's capacity and surplus workgroups leave at once.
//
//   emit     one workgroup per 256 primitives; a load-balanced expansion: the
//            workgroup's output slots are dealt round-robin to its threads and
//            each slot finds its primitive by binary search in an LDS prefix
//            array, so stores are contiguous whatever the rectangle sizes are.
//   sort     stable LSD radix sort, digits of up to 9 bits (5 passes at 1080p).
//            One up-front kernel reads the keys once and builds the global digit
//            histogram of every pass (so every pass knows where each digit's
//            output starts).  Per pass: (1) digit counts of every 4096-pair sort
//            tile, (2) one workgroup per digit turns its row of counts into
//            output offsets, (3) scatter: wavefront match-any ranking (ballots
//            over the digit bits) keeps equal digits in order, the tile is
//            sorted by digit in LDS and written out in contiguous runs.
//            (A single-kernel pass with a chained scan over tiles was measured
//            slower here: with 512 counters per tile the look-back chain costs
//            more than the two extra small kernels.)
//   ranges   tile_offsets[t] = first sorted position whose tile id is >= t.
#include "lmk_gs_internal.h"

namespace lmk {

__device__ __forceinline__ u64 load_D(const ScratchHeader *h, u64 capacity)
{
    const u64 d = h->dup_count;
    return d < capacity ? d : capacity;
}

// ---------------------------------------------------------------- emit
__global__ __launch_bounds__(kPreBlock) void emit_kernel(
    const u32 *__restrict__ tiles_touched, const ushort4 *__restrict__ rect,
    const float *__restrict__ depth, const u64 *__restrict__ block_offsets, u32 n, u32 tiles_x,
    u64 capacity, u64 *__restrict__ keys, u32 *__restrict__ vals, u64 *__restrict__ offsets,
    ScratchHeader *__restrict__ header)
{
    __shared__ u32 s_excl[kPreBlock];     // exclusive prefix of tiles_touched inside the workgroup
    __shared__ ushort4 s_rect[kPreBlock];
    __shared__ u32 s_depth[kPreBlock];
    __shared__ u32 s_wave[kPreBlock / kWave];

    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 i = blockIdx.x * kPreBlock + tid;
    const u32 cnt = i < n ? tiles_touched[i] : 0u;
    if (cnt) {
        s_rect[tid] = rect[i];
        s_depth[tid] = __float_as_uint(depth[i]);
    }
    u32 incl = cnt;
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
    const u32 excl = wave_base + incl - cnt;
    s_excl[tid] = excl;
    const u64 base = block_offsets[blockIdx.x];
    if (offsets) {
        if (i < n) offsets[i] = base + excl;
        if (i == n - 1) offsets[n] = base + total;
    }
    if (blockIdx.x == 0 && tid == 0 && header->dup_count > capacity) header->status = LMK_GS_ERR_CAPACITY;
    __syncthreads();

    for (u32 j = tid; j < total; j += kPreBlock) {
        // owner = last primitive whose exclusive prefix is <= j (primitives with
        // zero tiles share a prefix with their successor and are skipped by "last")
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
        const u64 pos = base + j;
        if (pos < capacity) {
            keys[pos] = ((u64)(ty * tiles_x + tx) << 32) | (u64)s_depth[lo];
            vals[pos] = blockIdx.x * kPreBlock + lo;
        }
    }
}

// ---------------------------------------------------------------- emit, binning rule 1
// Same expansion over the slots of every support rectangle, but each slot is first put
// through the splat/tile intersection test of lmk_gs_camera.binning == 1 (identical
// arithmetic to the count in the preprocess kernel; this translation unit is compiled
// without floating-point contraction for that reason) and the kept slots are compacted:
// the output position of a kept slot is the workgroup's base plus the number of kept
// slots before it, so pairs still come out in (primitive, row-major tile) order.
struct EmitTest { float u, v, A, B, C, rx, ry, tau; };

__device__ __forceinline__ float emit_clampf(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

__device__ __forceinline__ float emit_quad_adj(float A, float B, float C, float ex, float ey)
{
    const float m = A * ex * ex + C * ey * ey;
    const float q = m + 2.0f * B * ex * ey;
    return q - 4e-6f * m;
}

__global__ __launch_bounds__(kPreBlock) void emit_tight_kernel(
    const u32 *__restrict__ tiles_touched, const ushort4 *__restrict__ rect,
    const float *__restrict__ depth, const float4 *__restrict__ feat, ProjParams pp,
    const u64 *__restrict__ block_offsets, u32 n, u32 tiles_x,
    u64 capacity, u64 *__restrict__ keys, u32 *__restrict__ vals, u64 *__restrict__ offsets,
    ScratchHeader *__restrict__ header)
{
    __shared__ u32 s_excl[kPreBlock];     // exclusive prefix of rectangle areas inside the workgroup
    __shared__ ushort4 s_rect[kPreBlock];
    __shared__ u32 s_depth[kPreBlock];
    __shared__ float4 s_t0[kPreBlock];    // u, v, A, B
    __shared__ float4 s_t1[kPreBlock];    // C, rx, ry, tau
    __shared__ u32 s_wave[kPreBlock / kWave];
    __shared__ u32 s_wave2[kPreBlock / kWave];

    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 i = blockIdx.x * kPreBlock + tid;
    const u32 kept_cnt = i < n ? tiles_touched[i] : 0u;
    u32 area = 0;
    if (kept_cnt) {
        const ushort4 r = rect[i];
        s_rect[tid] = r;
        area = ((u32)r.z - (u32)r.x) * ((u32)r.w - (u32)r.y);
        s_depth[tid] = __float_as_uint(depth[i]);
        const float4 *f = feat + (size_t)i * (LMK_GS_FEAT_STRIDE / 4);
        const float4 f0 = f[0], f1 = f[1];
        const u32 bits = __float_as_uint(f1.y);
        const int E = (int)((bits >> 23) & 0xffu) - 127;
        const float tau = pp.tau_tab[(bits >> 20) & 7u] + (float)E * 1.3862944f;
        s_t0[tid] = f0;
        s_t1[tid] = make_float4(f1.x, -f0.w / f0.z, -f0.w / f1.x, tau);
    }
    // prefix sums over the workgroup: rectangle areas (slot ownership) and kept counts (offsets[])
    u32 incl = area, incl2 = kept_cnt;
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
    s_excl[tid] = wave_base + incl - area;
    const u64 base = block_offsets[blockIdx.x];
    if (offsets) {
        if (i < n) offsets[i] = base + (wave_base2 + incl2 - kept_cnt);
        if (i == n - 1) offsets[n] = base + total2;
    }
    if (blockIdx.x == 0 && tid == 0 && header->dup_count > capacity) header->status = LMK_GS_ERR_CAPACITY;
    __syncthreads();

    const float h = 0.5f * (float)LMK_GS_TILE - 0.5f;
    u32 running = 0;                                       // kept slots of earlier rounds (uniform)
    for (u32 j0 = 0; j0 < total; j0 += kPreBlock) {
        const u32 j = j0 + tid;
        bool keep = false;
        u32 lo = 0, tile = 0;
        if (j < total) {
            u32 hi = kPreBlock - 1;
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
            tile = ty * tiles_x + tx;
            const float4 t0 = s_t0[lo], t1 = s_t1[lo];
            const float xs = t0.x - ((float)(tx * LMK_GS_TILE) + 0.5f * (float)LMK_GS_TILE);
            const float ys = t0.y - ((float)(ty * LMK_GS_TILE) + 0.5f * (float)LMK_GS_TILE);
            const float ex1 = emit_clampf(xs, -h, h) - xs;
            const float ey1 = emit_clampf(ys + t1.z * ex1, -h, h) - ys;
            const float ey2 = emit_clampf(ys, -h, h) - ys;
            const float ex2 = emit_clampf(xs + t1.y * ey2, -h, h) - xs;
            const float q1 = emit_quad_adj(t0.z, t0.w, t1.x, ex1, ey1);
            const float q2 = emit_quad_adj(t0.z, t0.w, t1.x, ex2, ey2);
            const float qmin = q1 < q2 ? q1 : q2;
            keep = qmin <= t1.w;
        }
        const u64 mask = __builtin_amdgcn_ballot_w64(keep);
        const u32 rank = __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
        __syncthreads();                                   // s_wave free again
        if (lane == 0) s_wave[wv] = (u32)__builtin_popcountll(mask);
        __syncthreads();
        u32 before = 0, round_total = 0;
#pragma unroll
        for (u32 k = 0; k < kPreBlock / kWave; ++k) {
            const u32 c = s_wave[k];
            if (k < wv) before += c;
            round_total += c;
        }
        if (keep) {
            const u64 pos = base + running + before + rank;
            if (pos < capacity) {
                keys[pos] = ((u64)tile << 32) | (u64)s_depth[lo];
                vals[pos] = blockIdx.x * kPreBlock + lo;
            }
        }
        running += round_total;
    }
}

// ---------------------------------------------------------------- radix sort
// (0a) one read of the keys: digit histograms of every pass, one partial per workgroup
constexpr u32 kPrehistUnroll = 8;

__global__ __launch_bounds__(kSortThreads) void sort_prehist_kernel(
    const u64 *__restrict__ keys, const ScratchHeader *__restrict__ header, u64 capacity,
    SortPlan plan, u32 *__restrict__ partials, u64 *__restrict__ digit_totals)
{
    __shared__ u32 s_hist[kMaxPasses][kMaxRadix];
    const u64 D = load_D(header, capacity);
    const u32 tid = threadIdx.x;
    for (u32 k = tid; k < kMaxPasses * kMaxRadix; k += kSortThreads) (&s_hist[0][0])[k] = 0;
    if (blockIdx.x == 0)
        for (u32 k = tid; k < kMaxPasses * kMaxRadix; k += kSortThreads) digit_totals[k] = 0;
    __syncthreads();
    const u64 chunk = (u64)kSortThreads * kPrehistUnroll;
    for (u64 base = (u64)blockIdx.x * chunk; base < D; base += (u64)gridDim.x * chunk) {
        u64 k[kPrehistUnroll];
#pragma unroll
        for (u32 j = 0; j < kPrehistUnroll; ++j) {
            const u64 i = base + (u64)j * kSortThreads + tid;
            k[j] = i < D ? keys[i] : 0ull;
        }
#pragma unroll
        for (u32 j = 0; j < kPrehistUnroll; ++j) {
            const u64 i = base + (u64)j * kSortThreads + tid;
            if (i < D) {
#pragma unroll
                for (u32 p = 0; p < kMaxPasses; ++p)
                    if (p < plan.passes)
                        atomicAdd(&s_hist[p][(u32)(k[j] >> plan.shift[p]) & ((1u << plan.bits[p]) - 1u)], 1u);
            }
        }
    }
    __syncthreads();
    u32 *out = partials + (size_t)blockIdx.x * kMaxPasses * kMaxRadix;
    for (u32 k = tid; k < plan.passes * kMaxRadix; k += kSortThreads) out[k] = (&s_hist[0][0])[k];
}

// (0b) sums the partial histograms: workgroup (pass, slice) adds its slice of partials and
// contributes one atomic per digit.
constexpr u32 kReduceSlices = 32;

__global__ __launch_bounds__(kMaxRadix) void sort_reduce_kernel(
    const u32 *__restrict__ partials, u32 nblocks, u64 *__restrict__ digit_totals)
{
    const u32 d = threadIdx.x, pass = blockIdx.x / kReduceSlices, slice = blockIdx.x % kReduceSlices;
    const u32 per = (nblocks + kReduceSlices - 1) / kReduceSlices;
    const u32 b0 = slice * per, b1 = (b0 + per) < nblocks ? (b0 + per) : nblocks;
    u64 total = 0;
#pragma unroll 16
    for (u32 b = b0; b < b1; ++b)
        total += partials[((size_t)b * kMaxPasses + pass) * kMaxRadix + d];
    if (total) atomicAdd(reinterpret_cast<unsigned long long *>(&digit_totals[(size_t)pass * kMaxRadix + d]),
                         (unsigned long long)total);
}

// (1) digit counts of every sort tile of this pass -> table[digit][tile]
__global__ __launch_bounds__(kSortThreads) void radix_hist_kernel(
    const u64 *__restrict__ keys, const ScratchHeader *__restrict__ header, u64 capacity,
    u32 shift, u32 bits, u32 *__restrict__ table, u64 table_stride)
{
    __shared__ u32 s_hist[kMaxRadix];
    const u64 D = load_D(header, capacity);
    const u64 ntiles = (D + kSortTile - 1) / kSortTile;
    const u32 tid = threadIdx.x;
    const u32 dmask = (1u << bits) - 1u;
    for (u64 tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        for (u32 d = tid; d < kMaxRadix; d += kSortThreads) s_hist[d] = 0;
        __syncthreads();
        const u64 t0 = tile * kSortTile;
        u64 k[kSortItems];
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kSortThreads + tid;
            k[j] = idx < D ? keys[idx] : 0ull;
        }
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kSortThreads + tid;
            if (idx < D) atomicAdd(&s_hist[(u32)(k[j] >> shift) & dmask], 1u);
        }
        __syncthreads();
        for (u32 d = tid; d < kMaxRadix; d += kSortThreads) table[(u64)d * table_stride + tile] = s_hist[d];
        __syncthreads();
    }
}

// (2) one workgroup per digit: exclusive scan of its row of counts, offset by the total of
// all smaller digits -> offsets[digit][tile] (u64)
__global__ __launch_bounds__(kSortThreads) void radix_scan_kernel(
    const ScratchHeader *__restrict__ header, u64 capacity, const u32 *__restrict__ table,
    u64 *__restrict__ offsets, u64 table_stride, const u64 *__restrict__ digit_totals)
{
    __shared__ u64 s_wave[kSortThreads / kWave];
    __shared__ u64 s_carry;
    const u64 D = load_D(header, capacity);
    const u64 ntiles = (D + kSortTile - 1) / kSortTile;
    const u32 tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const u32 digit = blockIdx.x;

    // base = total of the digits below mine
    u64 part = 0;
    for (u32 d = tid; d < digit; d += kSortThreads) part += digit_totals[d];
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
    constexpr u32 kItems = 8;                  // consecutive sort tiles per thread, loaded together
    for (u64 base = 0; base < ntiles; base += (u64)kSortThreads * kItems) {
        const u64 first = base + (u64)tid * kItems;
        u32 v[kItems];
        u64 mine = 0;
#pragma unroll
        for (u32 k = 0; k < kItems; ++k) v[k] = first + k < ntiles ? row[first + k] : 0u;
#pragma unroll
        for (u32 k = 0; k < kItems; ++k) mine += v[k];
        u64 incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const u64 t = __shfl_up(incl, o, 64);
            if ((int)lane >= o) incl += t;
        }
        __syncthreads();                       // s_wave free again
        if (lane == kWave - 1) s_wave[wv] = incl;
        __syncthreads();
        u64 run = s_carry + incl - mine;
        for (u32 k = 0; k < wv; ++k) run += s_wave[k];
#pragma unroll
        for (u32 k = 0; k < kItems; ++k) {
            if (first + k < ntiles) orow[first + k] = run;
            run += v[k];
        }
        __syncthreads();
        if (tid == kSortThreads - 1) s_carry = run;
        __syncthreads();
    }
}

// (3) stable scatter of one digit
__global__ __launch_bounds__(kSortThreads) void radix_scatter_kernel(
    const u64 *__restrict__ keys_in, const u32 *__restrict__ vals_in,
    u64 *__restrict__ keys_out, u32 *__restrict__ vals_out,
    const ScratchHeader *__restrict__ header, u64 capacity, u32 shift, u32 bits,
    const u64 *__restrict__ offsets, u64 table_stride)
{
    constexpr u32 kWaves = kSortThreads / kWave;
    constexpr u32 kPerWave = kSortItems * kWave;       // 1024 consecutive pairs per wavefront
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

    for (u64 tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        for (u32 k = tid; k < kWaves * kMaxRadix; k += kSortThreads) (&s_wave_hist[0][0])[k] = 0;
        __syncthreads();

        const u64 t0 = tile * kSortTile + (u64)wv * kPerWave;
        u64 key[kSortItems];
        u32 val[kSortItems];
        u32 rank[kSortItems];
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kWave + lane;
            const bool valid = idx < D;
            key[j] = valid ? keys_in[idx] : ~0ull;
            val[j] = valid ? vals_in[idx] : 0u;
        }
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u64 idx = t0 + (u64)j * kWave + lane;
            const bool valid = idx < D;
            const u32 digit = (u32)(key[j] >> shift) & dmask;
            // lanes of this wavefront holding the same digit (match-any by ballots)
            u64 peers = __builtin_amdgcn_ballot_w64(valid);
#pragma unroll
            for (u32 b = 0; b < kMaxRadixBits; ++b) {
                if (b < bits) {
                    const bool bit = (digit >> b) & 1u;
                    const u64 bal = __builtin_amdgcn_ballot_w64(bit);
                    peers &= bit ? bal : ~bal;
                }
            }
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
            if (idx < D) {
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
            if (p < count) {
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
            if (idx < D) s_vals[rank[j]] = val[j];
        }
        __syncthreads();
#pragma unroll
        for (u32 j = 0; j < kSortItems; ++j) {
            const u32 p = j * kSortThreads + tid;
            if (p < count) vals_out[s_gofs[dg[j]] + p] = s_vals[p];
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------- ranges
__global__ __launch_bounds__(256) void tile_ranges_kernel(
    const u64 *__restrict__ keys, const ScratchHeader *__restrict__ header, u64 capacity,
    u32 num_tiles, u64 *__restrict__ tile_offsets, u64 *__restrict__ offsets_if_empty)
{
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

// ---------------------------------------------------------------- schedule hint
// Tile ids by descending list length, bucketed by the position of the length's top bit
// (one workgroup; within a bucket the order is whatever the atomics give -- it only
// decides which workgroup of the blend kernel starts first, never a result).
__global__ __launch_bounds__(1024) void tile_order_kernel(
    const u64 *__restrict__ tile_offsets, u32 num_tiles, u32 *__restrict__ order)
{
    __shared__ u32 s_cnt[65];
    const u32 tid = threadIdx.x;
    if (tid < 65) s_cnt[tid] = 0;
    __syncthreads();
    for (u32 t = tid; t < num_tiles; t += 1024) {
        const u64 len = tile_offsets[t + 1] - tile_offsets[t];
        const u32 b = len ? 64u - (u32)__builtin_clzll(len) : 0u;     // 0..64
        atomicAdd(&s_cnt[64 - b], 1u);                                 // long lists first
    }
    __syncthreads();
    if (tid == 0) {
        u32 run = 0;
        for (u32 k = 0; k < 65; ++k) { const u32 c = s_cnt[k]; s_cnt[k] = run; run += c; }
    }
    __syncthreads();
    for (u32 t = tid; t < num_tiles; t += 1024) {
        const u64 len = tile_offsets[t + 1] - tile_offsets[t];
        const u32 b = len ? 64u - (u32)__builtin_clzll(len) : 0u;
        order[atomicAdd(&s_cnt[64 - b], 1u)] = t;
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
    u64 *block_offsets = reinterpret_cast<u64 *>(scratch + L.block_offsets);
    u64 *digit_totals = reinterpret_cast<u64 *>(scratch + L.digit_totals);
    u32 *partials = reinterpret_cast<u32 *>(scratch + L.partials);
    u32 *table = reinterpret_cast<u32 *>(scratch + L.table);
    u64 *offsets = reinterpret_cast<u64 *>(scratch + L.offsets);
    const u32 num_tiles = pp.tiles_x * pp.tiles_y;
    const SortPlan plan = sort_plan(num_tiles);

    // ping-pong so that the last pass lands in keys/vals
    u64 *kin = (plan.passes & 1u) ? out.keys_alt : out.keys;
    u32 *vin = (plan.passes & 1u) ? out.vals_alt : out.vals;
    u64 *kout = (plan.passes & 1u) ? out.keys : out.keys_alt;
    u32 *vout = (plan.passes & 1u) ? out.vals : out.vals_alt;

    if (L.pre_blocks > 0) {
        if (pp.cam.binning == 1u)
            hipLaunchKernelGGL(emit_tight_kernel, dim3(L.pre_blocks), dim3(kPreBlock), 0, stream,
                               proj.tiles_touched, reinterpret_cast<const ushort4 *>(proj.rect), proj.depth,
                               reinterpret_cast<const float4 *>(proj.feat), pp,
                               block_offsets, n, pp.tiles_x, out.capacity, kin, vin, proj.offsets, header);
        else
            hipLaunchKernelGGL(emit_kernel, dim3(L.pre_blocks), dim3(kPreBlock), 0, stream,
                               proj.tiles_touched, reinterpret_cast<const ushort4 *>(proj.rect), proj.depth,
                               block_offsets, n, pp.tiles_x, out.capacity, kin, vin, proj.offsets, header);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }

    const u32 hist_blocks = (u32)(L.sort_tiles < kHistBlocks ? L.sort_tiles : kHistBlocks);
    hipLaunchKernelGGL(sort_prehist_kernel, dim3(hist_blocks), dim3(kSortThreads), 0, stream,
                       kin, header, out.capacity, plan, partials, digit_totals);
    hipLaunchKernelGGL(sort_reduce_kernel, dim3(plan.passes * kReduceSlices), dim3(kMaxRadix), 0, stream,
                       partials, hist_blocks, digit_totals);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // enough resident workgroups to fill 256 CUs several times over; each loops over sort tiles
    const u32 grid = grid_for(L.sort_tiles, 256u * 16u);
    for (u32 p = 0; p < plan.passes; ++p) {
        const u64 *totals = digit_totals + (size_t)p * kMaxRadix;
        hipLaunchKernelGGL(radix_hist_kernel, dim3(grid), dim3(kSortThreads), 0, stream,
                           kin, header, out.capacity, plan.shift[p], plan.bits[p], table, L.sort_tiles);
        hipLaunchKernelGGL(radix_scan_kernel, dim3(1u << plan.bits[p]), dim3(kSortThreads), 0, stream,
                           header, out.capacity, table, offsets, L.sort_tiles, totals);
        hipLaunchKernelGGL(radix_scatter_kernel, dim3(grid), dim3(kSortThreads), 0, stream,
                           kin, vin, kout, vout, header, out.capacity, plan.shift[p], plan.bits[p],
                           offsets, L.sort_tiles);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        u64 *tk = kin; kin = kout; kout = tk;
        u32 *tv = vin; vin = vout; vout = tv;
    }
    // after the last swap `kin` is the sorted buffer == out.keys
    const u32 rgrid = grid_for((out.capacity + 255) / 256, 256u * 16u);
    hipLaunchKernelGGL(tile_ranges_kernel, dim3(rgrid), dim3(256), 0, stream,
                       out.keys, header, out.capacity, num_tiles, out.tile_offsets,
                       n == 0 ? proj.offsets : nullptr);
    if (out.tile_order)
        hipLaunchKernelGGL(tile_order_kernel, dim3(1), dim3(1024), 0, stream,
                           out.tile_offsets, num_tiles, out.tile_order);
    return hipGetLastError();
}

}  // namespace lmk
