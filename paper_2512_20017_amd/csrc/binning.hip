// Tile binning: per-splat tile count + raster record, device prefix sums, key/value duplication in index order, stable
// sort by tile, tile ranges, depth order inside each tile's list. These are the steps between pts_splatting and the
// per-pixel blend that realise "sorts these view-dependent splats by their distance to the camera plane" (paper
// Sec. 2.1) per 16x16 tile.  All HBM- or latency-bound integer work.
//
// The tile lists are ordered by the 64-bit key (tile << 32 | depth bits), ties by splat index. That order is made in
// two halves: the (tile, point) pairs are emitted in point-index order and sorted stably by tile id (two radix passes
// over the P pairs), which leaves every tile's list in index order; one workgroup per tile then sorts its list stably
// by the 32 depth bits (k_tile_depth_sort, radix_sort.hip: in LDS for lists up to 2048 entries). The same permutation
// as a six-pass radix sort of P 64-bit keys, in a third of the launches of the earlier scheme (depth digits sorted on
// the points before duplication: twelve launches for 0.5 M keys, every one of them at the latency floor).
#include "pbdr_internal.h"
#include "binning_common.h"

namespace pbdr {

// Tiles touched by every point (0 for culled points) and, per block of 256 consecutive points, the number of points
// that touch at least one tile - those are the points binning lists ("visible" below) - and the number of their pairs.
// A state made by the preprocessing calls has radius == 0 for every point without a tile; a caller-made state with
// radius > 0 and an empty tile rectangle is treated as culled here, so every listed point owns at least one pair.
// Four consecutive points per thread (one 16-byte load of the radii, one 16-byte store of the counts: with one point
// per thread the launch did not keep enough bytes in flight, 2 TB/s at eight million points: 32 -> 21 us there), so a
// wavefront covers exactly one block of 256 points and its two sums need no LDS and no barrier.
__global__ __launch_bounds__(256) void k_count_visible(BinInput in, CamDev cam, uint32_t* __restrict__ tiles_touched,
                                                       uint32_t* __restrict__ blk_vis, uint32_t* __restrict__ blk_pairs,
                                                       uint32_t* __restrict__ status, uint32_t* __restrict__ ranges, uint32_t nranges)
{
    const uint32_t gid = blockIdx.x * 256u + threadIdx.x;
    const int lane = threadIdx.x & 63;
    // first launch of a binning call: the status words and the tile ranges start at zero (every later kernel of the call
    // comes after this one on the stream)
    if (gid < (uint32_t)kStCleared) status[gid] = 0u;
    for (uint32_t k = gid; k < nranges; k += gridDim.x * 256u) ranges[k] = 0u;
    const size_t i0 = (size_t)gid * 4u;
    const size_t n = (size_t)in.n;
    int r[4] = {0, 0, 0, 0};
    if (i0 + 4u <= n && (reinterpret_cast<uintptr_t>(in.radius) & 15u) == 0u) {
        const int4 v = *reinterpret_cast<const int4*>(in.radius + i0);
        r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) if (i0 + k < n) r[k] = in.radius[i0 + k];
    }
    uint32_t t[4];
    uint32_t vis = 0u, pairs = 0u;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        t[k] = 0u;
        if (r[k] > 0) {      // (r[k] is 0 past the end)
            int x0, y0, x1, y1;
            tile_rect(cam, in.mean2d[i0 + k], in.mean2d[n + i0 + k], r[k], x0, y0, x1, y1);
            t[k] = (uint32_t)(max(x1 - x0, 0) * max(y1 - y0, 0));       // <= 2^24: the grid has at most 4096 x 4096 tiles
        }
        vis += t[k] > 0u ? 1u : 0u;
        pairs = sat_add(pairs, t[k]);
    }
    if (i0 + 4u <= n) {
        *reinterpret_cast<uint4*>(tiles_touched + i0) = make_uint4(t[0], t[1], t[2], t[3]);      // (the array starts on a 256-byte boundary)
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) if (i0 + k < n) tiles_touched[i0 + k] = t[k];
    }
    const uint32_t inc = wave_inclusive_scan_sat(pairs);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) vis += (uint32_t)__shfl_xor((int)vis, d, 64);
    const size_t blk = (size_t)blockIdx.x * 4u + (threadIdx.x >> 6);      // the wavefront's 256 points
    if (lane == 63 && blk * 256u < n) {
        blk_vis[blk] = vis;
        blk_pairs[blk] = inc;
    }
}

// Exclusive prefix sums of the per-block counts of listed points and of pairs (the latter saturating), the totals into the
// status words and the pair total behind the last rank's offset. Also the order in which the packing kernel takes the
// blocks: those with kHeavyBlockPairs pairs or more first (in index order), the others after them (from the back, in
// reverse index order: one pass, no second scan).
// Workgroup g takes the 1024 kPer blocks from g * 1024 kPer on. What came before them it adds up by itself from the
// counts (a few coalesced loads per thread), so no workgroup waits for another, and eight million points are eight
// workgroups that each do one chunk instead of one that does eight in a row.
constexpr uint32_t kHeavyBlockPairs = 1536;      // about twice the benchmark view's mean
// kPer consecutive blocks per thread, 1024 kPer per workgroup: one up to two million points (four workgroups at a
// million: 5.4 us against 6.9 for one), four beyond (eight million points: 10.7 us against 13.8 for 31 workgroups
// of 1024 blocks, whose sums over what precedes them then take longer than their own chunk)
template <uint32_t kPer>
__global__ __launch_bounds__(1024) void k_scan_blocks(const uint32_t* __restrict__ blk_vis, const uint32_t* __restrict__ blk_pairs, uint32_t nb,
                                                      uint32_t* __restrict__ blk_vis_at, uint32_t* __restrict__ blk_pairs_at,
                                                      uint32_t* __restrict__ status, uint32_t* __restrict__ offsets, uint32_t n,
                                                      uint32_t* __restrict__ blk_order)
{
    constexpr uint32_t kScanChunk = 1024u * kPer;
    __shared__ uint32_t sV[16], sP[16], sH[16];
    __shared__ uint32_t cV[16], cP[16], cH[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t start = blockIdx.x * kScanChunk;
    // totals of the chunks before this one
    uint32_t carry_v = 0, carry_p = 0, carry_h = 0;
    if (start > 0u) {
        for (uint32_t i = threadIdx.x; i < start; i += kScanChunk) {      // (start is a multiple of kScanChunk: no tail)
            uint32_t vv[kPer], pv[kPer];
#pragma unroll
            for (uint32_t k = 0; k < kPer; ++k) { vv[k] = blk_vis[i + k * 1024u]; pv[k] = blk_pairs[i + k * 1024u]; }
#pragma unroll
            for (uint32_t k = 0; k < kPer; ++k) {
                carry_v += vv[k]; carry_p = sat_add(carry_p, pv[k]); carry_h += pv[k] >= kHeavyBlockPairs ? 1u : 0u;
            }
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            carry_v += __shfl_xor(carry_v, d, 64); carry_p = sat_add(carry_p, __shfl_xor(carry_p, d, 64)); carry_h += __shfl_xor(carry_h, d, 64);
        }
        if (lane == 0) { cV[wave] = carry_v; cP[wave] = carry_p; cH[wave] = carry_h; }
        __syncthreads();
        carry_v = 0; carry_p = 0; carry_h = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) { carry_v += cV[w]; carry_p = sat_add(carry_p, cP[w]); carry_h += cH[w]; }
    }
    const uint32_t idx0 = start + threadIdx.x * kPer;
    uint32_t v[kPer], p[kPer], h[kPer];
    uint32_t tv = 0, tp = 0, th = 0;         // this thread's totals
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) {
        v[k] = idx0 + k < nb ? blk_vis[idx0 + k] : 0u;
        p[k] = idx0 + k < nb ? blk_pairs[idx0 + k] : 0u;
        h[k] = p[k] >= kHeavyBlockPairs ? 1u : 0u;
        tv += v[k]; tp = sat_add(tp, p[k]); th += h[k];
    }
    uint32_t iv = tv, ip = tp, ih = th;      // inclusive over the wavefront's threads
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t uv = __shfl_up(iv, d, 64), up = __shfl_up(ip, d, 64), uh = __shfl_up(ih, d, 64);
        if (lane >= d) { iv += uv; ip = sat_add(ip, up); ih += uh; }
    }
    if (lane == 63) { sV[wave] = iv; sP[wave] = ip; sH[wave] = ih; }
    __syncthreads();
    uint32_t bv = carry_v, bp = carry_p, bh = carry_h, cv = carry_v, cp = carry_p;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const uint32_t wv = sV[w], wp = sP[w], wh = sH[w];
        if (w < wave) { bv += wv; bp = sat_add(bp, wp); bh += wh; }
        cv += wv; cp = sat_add(cp, wp);
    }
    // exclusive over the threads before this one = the lane below's inclusive sum
    const uint32_t ep = __shfl_up(ip, 1, 64);
    uint32_t ev = bv + iv - tv, eh = bh + ih - th;
    uint32_t epairs = sat_add(bp, lane == 0 ? 0u : ep);
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) {
        const uint32_t idx = idx0 + k;
        if (idx < nb) {
            blk_vis_at[idx] = ev;
            blk_pairs_at[idx] = epairs;
            eh += h[k];                      // heavy blocks among 0 .. idx
            if (h[k]) blk_order[eh - 1u] = idx;
            else blk_order[nb - 1u - (idx - eh)] = idx;
        }
        ev += v[k];
        epairs = sat_add(epairs, p[k]);
    }
    if (threadIdx.x == 0 && start + kScanChunk >= nb) {      // the last chunk: cv, cp are the totals
        const uint32_t m = min(cv, n);
        status[kStNumVis] = m;
        status[kStNumDup] = cp;
        offsets[m] = cp;
    }
}

// 3D Gaussians: the 48-byte raster record of a listed point (see binning_common.h for the rest of the block's work).
__global__ __launch_bounds__(256) void k_pack_dup(SplatsDev sp, CamDev cam, BinArrays A, Packed* __restrict__ packed)
{
    const size_t N = (size_t)sp.n;
    pack_dup_block(BinInput{sp.n, sp.mean2d, sp.radius}, cam, A, sp.depth, [&](int i) {
        float4* dst = reinterpret_cast<float4*>(packed + i);
        dst[0] = make_float4(sp.mean2d[i], sp.mean2d[N + i], sp.conic[i], sp.conic[N + i]);
        dst[1] = make_float4(sp.conic[2 * N + i], sp.opacity[i], sp.color[i], sp.color[N + i]);
        dst[2] = make_float4(sp.color[2 * N + i], __int_as_float(sp.radius[i]), sp.depth[i], 0.f);
    });
}

__global__ __launch_bounds__(256) void k_bin_begin(uint32_t* __restrict__ status, uint32_t* __restrict__ ranges, size_t nranges,
                                                   uint32_t* __restrict__ tile_order)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < (size_t)kStCleared) status[i] = 0u;
    if (i < nranges) ranges[i] = 0u;
    if (2 * i < nranges) tile_order[i] = (uint32_t)i;      // no lists: any order will do
}

// Four consecutive sorted pairs per thread: mark where each tile's run starts and ends.
__global__ __launch_bounds__(256) void k_tile_ranges(const uint32_t* __restrict__ tkeys, const uint32_t* __restrict__ status,
                                                     uint32_t cap, uint32_t ntiles, uint32_t* __restrict__ ranges)
{
    const uint32_t P = min(status[kStNumDup], cap);
    const uint32_t i0 = (blockIdx.x * 256u + threadIdx.x) * 4u;
    if (i0 >= P) return;
    uint32_t t[6];      // the pair before, the four of this thread, the pair after
    if (i0 + 4u <= P) {
        const uint4 v = *reinterpret_cast<const uint4*>(tkeys + i0);
        t[1] = v.x; t[2] = v.y; t[3] = v.z; t[4] = v.w;
    } else {
#pragma unroll
        for (uint32_t k = 0; k < 4u; ++k) t[1 + k] = i0 + k < P ? tkeys[i0 + k] : 0xffffffffu;
    }
    t[0] = i0 > 0u ? tkeys[i0 - 1u] : 0xffffffffu;
    t[5] = i0 + 4u < P ? tkeys[i0 + 4u] : 0xffffffffu;
#pragma unroll
    for (uint32_t k = 0; k < 4u; ++k) {
        const uint32_t i = i0 + k, tile = t[1 + k];
        if (i >= P || tile >= ntiles) continue;     // tile >= ntiles cannot happen for keys written by the packing kernels; keeps the writes in bounds regardless
        if (i == 0u || t[k] != tile) ranges[2 * tile] = i;
        if (i + 1u == P || t[2 + k] != tile) ranges[2 * tile + 1] = i + 1u;
    }
}

// The order in which the compositing kernels take the tiles: longest lists first. Workgroups start in index order and a
// tile's cost grows with its list, so in image order a launch ends on whatever long tiles happen to come late, with
// most of the chip idle. Tiles are put in classes of list length, two per octave (class 0 = longest); within a class
// they keep the image order, so neighbours in the order are still neighbours in the image and share splat records in L2.
// That is a stable counting sort on the class, done by one workgroup: wavefront w owns a contiguous run of tiles and
// takes it 64 at a time. A lane finds the lanes of its class from six ballots, one per bit of the class, with no loop
// over the classes present: the kernel runs on one compute unit, so its instruction count is its duration.
constexpr int kOrderClasses = 40;           // < 63; class 63 stands for "no tile"
constexpr uint32_t kOrderRounds = 1;        // rounds of 64 tiles per wavefront: 1,024 tiles per workgroup (measured: 8 rounds 12.0 us, 2 rounds 6.3, 1 round 5.5 for 8,160 tiles)
// lists of kWaveListMax - 1 = 1023 entries or more are sorted by a whole workgroup; length + 1 < 1024 = 2^10 means a
// class code of at most 2 * 9 + 1
static_assert(kWaveListMax == 1024, "kFirstSmallClass is the class that starts at this length");
constexpr uint32_t kFirstSmallClass = (uint32_t)(kOrderClasses - 1) - 19u;

__device__ __forceinline__ uint32_t order_class(uint32_t len)
{
    const uint32_t x = len + 1u;
    const int e = 31 - __clz((int)x);
    const uint32_t half = e > 0 ? (x >> (e - 1)) & 1u : 0u;
    return (uint32_t)(kOrderClasses - 1) - min(2u * (uint32_t)e + half, (uint32_t)(kOrderClasses - 1));
}

// classes of the tiles tb + 64 k + lane, k = 0 .. kOrderRounds - 1, of the run that ends at t1
__device__ __forceinline__ void order_classes(const uint2* __restrict__ range2, uint32_t tb, uint32_t t1, uint32_t lane,
                                              uint32_t (&cls)[kOrderRounds])
{
    uint2 r[kOrderRounds];
#pragma unroll
    for (uint32_t k = 0; k < kOrderRounds; ++k) {
        const uint32_t t = tb + k * 64u + lane;
        r[k] = t < t1 ? range2[t] : make_uint2(0u, 0u);
    }
#pragma unroll
    for (uint32_t k = 0; k < kOrderRounds; ++k) cls[k] = tb + k * 64u + lane < t1 ? order_class(r[k].y - r[k].x) : 63u;
}

// the lanes of the wavefront whose class equals this lane's
__device__ __forceinline__ uint64_t lanes_of_my_class(uint32_t cls)
{
    uint64_t same = ~0ull;
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        const bool bit = ((cls >> b) & 1u) != 0u;
        const uint64_t set = __ballot(bit);
        same &= bit ? set : ~set;
    }
    return same;
}

// Workgroup g orders the kOrderChunk tiles from g * kOrderChunk on (1,024 of them: the ballot-ranked counting and placing of its own tiles is what takes a workgroup's time). Where
// they go also depends on the other workgroups' tiles: how many of each class lie in earlier chunks, and in later ones.
// Every workgroup counts those for itself from the ranges, so none waits for another.
constexpr uint32_t kOrderChunk = 16u * kOrderRounds * 64u;
template <bool kMulti>                      // more than one chunk
__global__ __launch_bounds__(1024) void k_tile_order(const uint32_t* __restrict__ ranges, uint32_t ntiles, uint32_t* __restrict__ tile_order,
                                                     uint32_t* __restrict__ status)
{
    // per class: (earlier chunks,) the 16 wavefronts of this one(, later chunks)
    constexpr uint32_t kOrderSlots = kMulti ? 18u : 16u, kFirst = kMulti ? 1u : 0u;
    constexpr int kPer = (kOrderClasses * kOrderSlots + 63) / 64;
    __shared__ uint32_t count[64 * kOrderSlots];      // [class][slot]: tiles, then where the next tile of (class, slot) goes (class 63: unused, in bounds)
    const uint32_t lane = threadIdx.x & 63u, w = threadIdx.x >> 6;
    const uint32_t c0 = blockIdx.x * kOrderChunk, c1 = min(ntiles, c0 + kOrderChunk);
    const uint32_t t0 = min(c1, c0 + w * (kOrderRounds * 64u)), t1 = min(c1, t0 + kOrderRounds * 64u);
    const uint64_t below = (1ull << lane) - 1ull;
    const uint2* range2 = reinterpret_cast<const uint2*>(ranges);

    __shared__ uint32_t other[kMulti ? 2 * kOrderClasses * 16 : 1];      // [earlier, later chunks][class][lane % 16]
    for (uint32_t i = threadIdx.x; i < 64u * kOrderSlots; i += 1024u) count[i] = 0u;
    if (kMulti)
        for (uint32_t i = threadIdx.x; i < 2u * kOrderClasses * 16u; i += 1024u) other[i] = 0u;
    __syncthreads();
    uint32_t cls[kOrderRounds];
    order_classes(range2, t0, t1, lane, cls);
#pragma unroll
    for (uint32_t k = 0; k < kOrderRounds; ++k) {
        const uint64_t same = lanes_of_my_class(cls[k]);
        if ((same & below) == 0ull && cls[k] != 63u) count[cls[k] * kOrderSlots + kFirst + w] += (uint32_t)__popcll(same);      // first lane of its class
    }
    if (kMulti) {      // the tiles of the other chunks, by class
        // (one of 16 counters per side and class, by lane: a wavefront's tiles are mostly of one class, and additions to
        // one LDS address take their turns)
        for (uint32_t ib = threadIdx.x; ib < ntiles; ib += 4u * 1024u) {
            uint2 r[4];
#pragma unroll
            for (uint32_t k = 0; k < 4u; ++k) {
                const uint32_t i = ib + k * 1024u;
                r[k] = i < ntiles ? range2[i] : make_uint2(0u, 0u);
            }
#pragma unroll
            for (uint32_t k = 0; k < 4u; ++k) {
                const uint32_t i = ib + k * 1024u;
                if (i < ntiles && (i < c0 || i >= c1))
                    atomicAdd(&other[((i < c0 ? 0u : (uint32_t)kOrderClasses) + order_class(r[k].y - r[k].x)) * 16u + (lane & 15u)], 1u);
            }
        }
        __syncthreads();
        if (threadIdx.x < 2u * kOrderClasses) {
            uint32_t sum = 0;
#pragma unroll
            for (uint32_t k = 0; k < 16u; ++k) sum += other[threadIdx.x * 16u + k];
            const uint32_t c = threadIdx.x < (uint32_t)kOrderClasses ? threadIdx.x : threadIdx.x - (uint32_t)kOrderClasses;
            count[c * kOrderSlots + (threadIdx.x < (uint32_t)kOrderClasses ? 0u : kOrderSlots - 1u)] = sum;
        }
    }
    __syncthreads();
    if (w == 0) {      // exclusive prefix sums over (class, slot), classes 0 .. kOrderClasses - 1: kPer consecutive entries per lane
        uint32_t v[kPer], sum = 0;
#pragma unroll
        for (int k = 0; k < kPer; ++k) { v[k] = count[lane * kPer + k]; sum += v[k]; }
        uint32_t incl = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t up = __shfl_up(incl, d);
            if (lane >= (uint32_t)d) incl += up;
        }
        uint32_t at = incl - sum;
#pragma unroll
        for (int k = 0; k < kPer; ++k) { count[lane * kPer + k] = at; at += v[k]; }
    }
    __syncthreads();
    // how many tiles hold kWaveListMax - 1 entries or more: they come first in the order, and the depth sort gives each a whole
    // workgroup (the classes are cut at powers of two of length + 1, so this is where a class starts)
    if (threadIdx.x == 0 && blockIdx.x == 0) status[kStNumBig] = count[kFirstSmallClass * kOrderSlots];
#pragma unroll
    for (uint32_t k = 0; k < kOrderRounds; ++k) {
        const uint64_t same = lanes_of_my_class(cls[k]);
        const uint32_t slot = cls[k] * kOrderSlots + kFirst + w;
        const uint32_t at = count[slot];      // every lane of the class reads it before its first lane moves it on
        if (cls[k] != 63u) {
            tile_order[at + (uint32_t)__popcll(same & below)] = t0 + k * 64u + lane;
            if ((same & below) == 0ull) count[slot] = at + (uint32_t)__popcll(same);
        }
    }
}

// Inspection only: the 64-bit keys (tile << 32 | depth bits) of the sorted pairs, rebuilt from the tile ranges, the
// sorted point indices and the per-point depth bits. One workgroup per tile.
__global__ __launch_bounds__(256) void k_make_keys64(const uint32_t* __restrict__ ranges, const uint32_t* __restrict__ tvals,
                                                     const uint32_t* __restrict__ depth_bits, uint32_t cap, uint64_t* __restrict__ keys64)
{
    const uint32_t tile = blockIdx.x;
    const uint32_t s = ranges[2 * tile], e = min(ranges[2 * tile + 1], cap);
    for (uint32_t i = s + threadIdx.x; i < e; i += 256u) keys64[i] = ((uint64_t)tile << 32) | depth_bits[tvals[i]];
}

hipError_t launch_make_keys64(const Layout& L, char* ws, hipStream_t s)
{
    const uint32_t* tv = reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L));
    hipLaunchKernelGGL(k_make_keys64, dim3((unsigned)L.tiles), dim3(256), 0, s, reinterpret_cast<const uint32_t*>(ws + L.off_ranges), tv,
                       reinterpret_cast<const uint32_t*>(ws + L.off_depth_bits), L.cap, reinterpret_cast<uint64_t*>(ws + L.off_keys64));
    return hipGetLastError();
}

hipError_t launch_bin_begin(const Layout& L, char* ws, hipStream_t s)
{
    uint32_t* status = reinterpret_cast<uint32_t*>(ws + L.off_status);
    uint32_t* ranges = reinterpret_cast<uint32_t*>(ws + L.off_ranges);
    // status words and tile ranges start at zero (one launch)
    ProfScope prof(kKFill, s);
    hipLaunchKernelGGL(k_bin_begin, dim3((unsigned)((2 * (size_t)L.tiles + 255) / 256)), dim3(256), 0, s, status, ranges,
                       2 * (size_t)L.tiles, reinterpret_cast<uint32_t*>(ws + L.off_tile_order));
    return hipGetLastError();
}

BinArrays bin_arrays(const Layout& L, char* ws)
{
    BinArrays A;
    A.touched = reinterpret_cast<const uint32_t*>(ws + L.off_touched);
    A.blk_vis = reinterpret_cast<const uint32_t*>(ws + L.off_blk_vis_at);
    A.blk_pairs = reinterpret_cast<const uint32_t*>(ws + L.off_blk_pairs_at);
    A.blk_order = reinterpret_cast<const uint32_t*>(ws + L.off_blk_order);
    A.blk_count = reinterpret_cast<const uint32_t*>(ws + L.off_blk_vis);
    A.order = reinterpret_cast<uint32_t*>(ws + L.off_order);
    A.offsets = reinterpret_cast<uint32_t*>(ws + L.off_offsets);
    A.slot_base = reinterpret_cast<uint32_t*>(ws + L.off_slot_base);
    A.depth_bits = reinterpret_cast<uint32_t*>(ws + L.off_depth_bits);
    A.tkeys = reinterpret_cast<uint32_t*>(ws + L.off_tkey0);
    A.tvals = reinterpret_cast<uint32_t*>(ws + L.off_tval0);
    A.chunk_rank = reinterpret_cast<uint32_t*>(ws + L.off_chunk_rank);
    A.cap = L.cap;
    A.status = reinterpret_cast<uint32_t*>(ws + L.off_status);
    return A;
}

// Tiles per point, listed points and pairs per block of 256 points and their prefix sums; leaves the listed count and the
// pair total in the status words. Also the call's first launch: clears the status words and the tile ranges.
hipError_t launch_count_visible(const BinInput& in, const CamDev& cam, const Layout& L, char* ws, hipStream_t s)
{
    const int n = in.n;
    if (n == 0) return hipSuccess;
    uint32_t* blk_vis = reinterpret_cast<uint32_t*>(ws + L.off_blk_vis);
    uint32_t* blk_pairs = reinterpret_cast<uint32_t*>(ws + L.off_blk_pairs);
    uint32_t* status = reinterpret_cast<uint32_t*>(ws + L.off_status);
    const unsigned nb = (unsigned)((n + 255) / 256);
    ProfScope prof(kKCountPack, s);
    hipLaunchKernelGGL(k_count_visible, dim3((nb + 3u) / 4u), dim3(256), 0, s, in, cam, reinterpret_cast<uint32_t*>(ws + L.off_touched), blk_vis,
                       blk_pairs, status, reinterpret_cast<uint32_t*>(ws + L.off_ranges), (uint32_t)(2 * (size_t)L.tiles));
    uint32_t* const vis_at = reinterpret_cast<uint32_t*>(ws + L.off_blk_vis_at);
    uint32_t* const pairs_at = reinterpret_cast<uint32_t*>(ws + L.off_blk_pairs_at);
    uint32_t* const offsets = reinterpret_cast<uint32_t*>(ws + L.off_offsets);
    uint32_t* const blk_order = reinterpret_cast<uint32_t*>(ws + L.off_blk_order);
    if (nb <= 8192u)
        hipLaunchKernelGGL(k_scan_blocks<1>, dim3((nb + 1023u) / 1024u), dim3(1024), 0, s, blk_vis, blk_pairs, nb, vis_at, pairs_at, status,
                           offsets, (uint32_t)n, blk_order);
    else
        hipLaunchKernelGGL(k_scan_blocks<4>, dim3((nb + 4095u) / 4096u), dim3(1024), 0, s, blk_vis, blk_pairs, nb, vis_at, pairs_at, status,
                           offsets, (uint32_t)n, blk_order);
    return hipGetLastError();
}

// Everything after the pairs are in place (in point order): stable sort by tile, tile ranges, the order in which the
// compositing kernels take the tiles, depth order inside every tile's list.
hipError_t launch_bin_finish(const BinInput& sp, const CamDev& cam, const Layout& L, char* ws, hipStream_t s)
{
    if (sp.n == 0) return hipSuccess;
    uint32_t* status = reinterpret_cast<uint32_t*>(ws + L.off_status);
    uint32_t* ranges = reinterpret_cast<uint32_t*>(ws + L.off_ranges);
    uint32_t* tk[2] = {reinterpret_cast<uint32_t*>(ws + L.off_tkey0), reinterpret_cast<uint32_t*>(ws + L.off_tkey1)};
    uint32_t* tv[2] = {reinterpret_cast<uint32_t*>(ws + L.off_tval0), reinterpret_cast<uint32_t*>(ws + L.off_tval1)};
    uint32_t* totals = reinterpret_cast<uint32_t*>(ws + L.off_totals);
    uint32_t* tile_hist = reinterpret_cast<uint32_t*>(ws + L.off_tile_hist);
    // tile digits: stable sort of the P pairs by tile id
    hipError_t e = launch_radix_sort32(tk, tv, status + kStNumDup, L.cap, L.tile_bits, totals, tile_hist, s);
    if (e != hipSuccess) return e;
    const int fin = L.tile_passes & 1;
    const uint32_t ntiles = (uint32_t)(cam.TX * cam.TY);      // the call's tile grid (a patch covers fewer tiles than the image the workspace is sized for)
    uint32_t* tile_order = reinterpret_cast<uint32_t*>(ws + L.off_tile_order);
    {
        ProfScope prof(kKTileRanges, s);
        hipLaunchKernelGGL(k_tile_ranges, dim3((L.cap + 1023u) / 1024u), dim3(256), 0, s, tk[fin], status, L.cap, (uint32_t)L.tiles, ranges);
        if (ntiles <= kOrderChunk) hipLaunchKernelGGL(k_tile_order<false>, dim3(1), dim3(1024), 0, s, ranges, ntiles, tile_order, status);
        else hipLaunchKernelGGL(k_tile_order<true>, dim3((ntiles + kOrderChunk - 1u) / kOrderChunk), dim3(1024), 0, s, ranges, ntiles, tile_order, status);
    }
    // depth digits: every tile's list, now in point order, into depth order (the tile ids in tk[fin] are spent: that
    // array and the other pair of buffers are the scratch of lists too long for LDS)
    return launch_tile_depth_sort(ranges, tile_order, ntiles, status, reinterpret_cast<const uint32_t*>(ws + L.off_depth_bits), L.cap,
                                  tk[fin], tv[fin], tk[fin ^ 1], tv[fin ^ 1], s);
}

hipError_t launch_bin_sort(const SplatsDev& sp, const CamDev& cam, const Layout& L, char* ws, hipStream_t s)
{
    if (sp.n == 0) return launch_bin_begin(L, ws, s);      // nothing to count: only the cleared status words and ranges
    hipError_t e = launch_count_visible(BinInput{sp.n, sp.mean2d, sp.radius}, cam, L, ws, s);
    if (e != hipSuccess) return e;
    {
        ProfScope prof(kKDuplicate, s);
        hipLaunchKernelGGL(k_pack_dup, dim3((unsigned)((sp.n + 255) / 256)), dim3(256), 0, s, sp, cam, bin_arrays(L, ws),
                           reinterpret_cast<Packed*>(ws + L.off_packed));
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return launch_bin_finish(BinInput{sp.n, sp.mean2d, sp.radius}, cam, L, ws, s);
}

}  // namespace pbdr
