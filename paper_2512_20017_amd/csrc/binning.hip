// Tile binning: per-splat tile count + raster record, depth order of the splats, device prefix sum, key/value
// duplication in depth order, stable sort by tile, tile ranges. These are the steps between pts_splatting and the
// per-pixel blend that realise "sorts these view-dependent splats by their distance to the camera plane" (paper
// Sec. 2.1) per 16x16 tile.  All HBM-bound, integer work.
//
// The tile lists are ordered by the 64-bit key (tile << 32 | depth bits), ties by splat index. The sort is a
// least-significant-digit radix sort of that key whose four depth digits are sorted on the n splats, before
// duplication (every duplicate of a splat carries the same depth bits), and whose tile digits are sorted on the P
// pairs afterwards: the same permutation for a fraction of the traffic.
#include "pbdr_internal.h"
#include "pair_reduce.h"

namespace pbdr {

// Tiles touched by every point (0 for culled points) and, per block of 256 consecutive points, the number of points
// that touch at least one tile: those are the points binning lists ("visible" below). A state made by the
// preprocessing calls has radius == 0 for every point without a tile; a caller-made state with radius > 0 and an
// empty tile rectangle is treated as culled here, so every listed point owns at least one pair.
__global__ __launch_bounds__(256) void k_count_visible(BinInput in, CamDev cam, uint32_t* __restrict__ tiles_touched,
                                                       uint32_t* __restrict__ vis_block, uint32_t* __restrict__ status,
                                                       uint32_t* __restrict__ ranges, uint32_t nranges)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    // first launch of a binning call: the status words and the tile ranges start at zero (every later kernel of the call
    // comes after this one on the stream)
    if (i < kStCleared) status[i] = 0u;
    for (uint32_t k = (uint32_t)i; k < nranges; k += gridDim.x * 256u) ranges[k] = 0u;
    uint32_t t = 0;
    if (i < in.n) {
        const int r = in.radius[i];
        if (r > 0) {
            int x0, y0, x1, y1;
            tile_rect(cam, in.mean2d[i], in.mean2d[(size_t)in.n + i], r, x0, y0, x1, y1);
            t = (uint32_t)(max(x1 - x0, 0) * max(y1 - y0, 0));
        }
        tiles_touched[i] = t;
    }
    const int c = __syncthreads_count(t > 0);
    if (threadIdx.x == 0) vis_block[blockIdx.x] = (uint32_t)c;
}

// One thread per point. A visible point gets: the number of tiles its square touches, the 48-byte raster record,
// and a slot in the compact list of visible points, kept in ascending point order (the block's first slot comes from
// the scanned block counts, the slot within the block from ballots), where its (depth bits, index) pair for the depth
// sort goes. Culled points cost one 4-byte read and nothing downstream.
__global__ __launch_bounds__(256) void k_count_pack(SplatsDev sp, CamDev cam, const uint32_t* __restrict__ vis_block,
                                                    const uint32_t* __restrict__ tiles_touched, Packed* __restrict__ packed,
                                                    uint32_t* __restrict__ dkey, uint32_t* __restrict__ dval,
                                                    uint32_t* __restrict__ depth_bits)
{
    __shared__ uint32_t sWave[4];
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t N = (size_t)sp.n;
    const bool vis = (i < sp.n) && tiles_touched[i] > 0;
    const unsigned long long m = __ballot(vis);
    if (lane == 0) sWave[wave] = (uint32_t)__popcll(m);
    __syncthreads();
    if (!vis) return;
    uint32_t slot = vis_block[blockIdx.x] + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
#pragma unroll
    for (int w = 0; w < 3; ++w) if (w < wave) slot += sWave[w];
    const int r = sp.radius[i];
    const float mx = sp.mean2d[i], my = sp.mean2d[N + i];
    float4* dst = reinterpret_cast<float4*>(packed + i);
    dst[0] = make_float4(mx, my, sp.conic[i], sp.conic[N + i]);
    dst[1] = make_float4(sp.conic[2 * N + i], sp.opacity[i], sp.color[i], sp.color[N + i]);
    const float depth = sp.depth[i];
    const uint32_t key = __float_as_uint(depth);
    dst[2] = make_float4(sp.color[2 * N + i], __int_as_float(r), depth, 0.f);
    dkey[slot] = key;
    dval[slot] = (uint32_t)i;
    depth_bits[i] = key;
}

// tile counts in depth order (rank r < m holds the visible point order[r]); ranks m..n get 0, and slot n is the
// sentinel that makes the scan leave the pair total at offsets[n]
__global__ __launch_bounds__(256) void k_rank_counts(int n, const uint32_t* __restrict__ status, const uint32_t* __restrict__ order,
                                                     const uint32_t* __restrict__ tiles_touched, uint32_t* __restrict__ counts)
{
    // four consecutive ranks per thread (offsets, counts and order start on 16-byte boundaries)
    const uint32_t r0 = (blockIdx.x * 256u + threadIdx.x) * 4u;
    if (r0 > (uint32_t)n) return;
    const uint32_t m = min(status[kStNumVis], (uint32_t)n);
    uint32_t c[4] = {0u, 0u, 0u, 0u};
    if (r0 + 4u <= m) {
        const uint4 o = *reinterpret_cast<const uint4*>(order + r0);
        c[0] = tiles_touched[o.x]; c[1] = tiles_touched[o.y]; c[2] = tiles_touched[o.z]; c[3] = tiles_touched[o.w];
    } else {
#pragma unroll
        for (uint32_t k = 0; k < 4u; ++k) if (r0 + k < m) c[k] = tiles_touched[order[r0 + k]];
    }
    if (r0 + 4u <= (uint32_t)n + 1u) {
        *reinterpret_cast<uint4*>(counts + r0) = make_uint4(c[0], c[1], c[2], c[3]);
    } else {
#pragma unroll
        for (uint32_t k = 0; k < 4u; ++k) if (r0 + k <= (uint32_t)n) counts[r0 + k] = c[k];
    }
}

// ---------------------------------------------------------------------------------------------
// Exclusive prefix sum over uint32: reduce per 4096-element block, scan the block sums in one
// workgroup, rescan each block with its offset. No inter-workgroup waiting.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

// exclusive scan of one value per thread across a 256-thread block; returns the block total through `total`
__device__ __forceinline__ uint32_t block_exclusive_scan_256(uint32_t v, uint32_t* lds_wave /*[4]*/, uint32_t& total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t inc = wave_inclusive_scan(v);
    if (lane == 63) lds_wave[wave] = inc;
    __syncthreads();
    uint32_t base = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t t = lds_wave[w];
        if (w < wave) base += t;
    }
    total = lds_wave[0] + lds_wave[1] + lds_wave[2] + lds_wave[3];
    __syncthreads();
    return base + inc - v;
}

constexpr int kScanPerThread = kScanItems / 256;  // 16

__global__ __launch_bounds__(256) void k_scan_reduce(const uint32_t* __restrict__ in, uint32_t n, uint32_t* __restrict__ partials)
{
    __shared__ uint32_t lds[4];
    const uint32_t base = blockIdx.x * (uint32_t)kScanItems + threadIdx.x * kScanPerThread;
    uint32_t s = 0;
    if (base + kScanPerThread <= n) {
        const uint4* p = reinterpret_cast<const uint4*>(in + base);
#pragma unroll
        for (int k = 0; k < kScanPerThread / 4; ++k) { const uint4 v = p[k]; s += v.x + v.y + v.z + v.w; }
    } else {
        for (int k = 0; k < kScanPerThread; ++k) if (base + k < n) s += in[base + k];
    }
    uint32_t total;
    (void)block_exclusive_scan_256(s, lds, total);
    if (threadIdx.x == 0) partials[blockIdx.x] = total;
}

// one workgroup of 1024 threads scans the `nb` block sums in place (exclusive); writes the grand total
__global__ __launch_bounds__(1024) void k_scan_partials(uint32_t* __restrict__ partials, uint32_t nb, uint32_t* __restrict__ total_out)
{
    __shared__ uint32_t lds[16];
    __shared__ uint32_t carry_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (uint32_t start = 0; start < nb; start += 1024) {
        const uint32_t idx = start + threadIdx.x;
        const uint32_t v = idx < nb ? partials[idx] : 0u;
        const uint32_t inc = wave_inclusive_scan(v);
        if (lane == 63) lds[wave] = inc;
        __syncthreads();
        uint32_t base = carry_s, chunk = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) { const uint32_t t = lds[w]; if (w < wave) base += t; chunk += t; }
        if (idx < nb) partials[idx] = base + inc - v;
        __syncthreads();
        if (threadIdx.x == 0) carry_s += chunk;
        __syncthreads();
    }
    if (threadIdx.x == 0) { partials[nb] = carry_s; if (total_out) *total_out = carry_s; }
}

// `in` and `out` may be the same array: every thread reads its 16 elements before it writes them
__global__ __launch_bounds__(256) void k_scan_apply(const uint32_t* in, uint32_t* out, uint32_t n,
                                                    const uint32_t* __restrict__ partials)
{
    __shared__ uint32_t lds[4];
    const uint32_t base = blockIdx.x * (uint32_t)kScanItems + threadIdx.x * kScanPerThread;
    uint32_t v[kScanPerThread];
    const bool full = base + kScanPerThread <= n;
    if (full) {
        const uint4* p = reinterpret_cast<const uint4*>(in + base);
#pragma unroll
        for (int k = 0; k < kScanPerThread / 4; ++k) { const uint4 t = p[k]; v[4 * k] = t.x; v[4 * k + 1] = t.y; v[4 * k + 2] = t.z; v[4 * k + 3] = t.w; }
    } else {
#pragma unroll
        for (int k = 0; k < kScanPerThread; ++k) v[k] = (base + k < n) ? in[base + k] : 0u;
    }
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) s += v[k];
    uint32_t total;
    uint32_t run = block_exclusive_scan_256(s, lds, total) + partials[blockIdx.x];
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) { const uint32_t t = v[k]; v[k] = run; run += t; }
    if (full) {
        uint4* q = reinterpret_cast<uint4*>(out + base);
#pragma unroll
        for (int k = 0; k < kScanPerThread / 4; ++k) q[k] = make_uint4(v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]);
    } else {
#pragma unroll
        for (int k = 0; k < kScanPerThread; ++k) if (base + k < n) out[base + k] = v[k];
    }
}

hipError_t launch_exclusive_scan(const uint32_t* in, uint32_t* out, uint32_t n, uint32_t* partials, uint32_t* total_out,
                                 hipStream_t s)
{
    const uint32_t nb = (n + kScanItems - 1) / kScanItems;
    ProfScope prof(kKScan, s);
    if (nb > 0) hipLaunchKernelGGL(k_scan_reduce, dim3(nb), dim3(256), 0, s, in, n, partials);
    hipLaunchKernelGGL(k_scan_partials, dim3(1), dim3(1024), 0, s, partials, nb, total_out);
    if (nb > 0) hipLaunchKernelGGL(k_scan_apply, dim3(nb), dim3(256), 0, s, in, out, n, partials);
    return hipGetLastError();
}

// Duplication, in depth order: rank r handles point order[r]. Every (tile, splat) pair of a wavefront's 64
// consecutive ranks is written by whichever lane comes next, so the work is balanced whatever the mix of small and
// large splats. The pairs of those 64 ranks occupy one contiguous range of the output (offsets are a prefix sum);
// lane l writes slots B + l, B + l + 64, ... and finds the owning rank of a slot by binary search over the 64 range
// ends kept in LDS. Pair order within a point: row-major over its tile rectangle. Also records, per point, where
// its pairs start (slot_base), which the backward pass uses to address its per-pair sums.
__global__ __launch_bounds__(256) void k_duplicate(BinInput sp, CamDev cam, const uint32_t* __restrict__ order,
                                                   const uint32_t* __restrict__ offsets, uint32_t* __restrict__ tkeys,
                                                   uint32_t* __restrict__ tvals, uint32_t* __restrict__ slot_base,
                                                   uint32_t* __restrict__ chunk_rank, uint32_t cap, uint32_t* __restrict__ status)
{
    __shared__ uint32_t sEnd[4][64];
    const int r = blockIdx.x * 256 + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int x0 = 0, y0 = 0, x1 = 0, y1 = 0;
    uint32_t at = 0, id = 0;
    const uint32_t m = min(status[kStNumVis], (uint32_t)sp.n);     // ranks below m hold visible points
    if ((uint32_t)r < m) {
        at = offsets[r];
        id = order[r];
        const int rad = sp.radius[id];
        if (rad > 0) tile_rect(cam, sp.mean2d[id], sp.mean2d[(size_t)sp.n + id], rad, x0, y0, x1, y1);
        slot_base[id] = at;
    } else {
        at = offsets[sp.n];                    // the pair total (sentinel slot of the prefix sum)
    }
    const int w = x1 - x0;
    const uint32_t cnt = (uint32_t)(w * (y1 - y0));
    if ((uint32_t)r < m) {   // which rank owns every 256th pair (for the pair-balanced gather of the backward pass)
        const uint32_t end = min(at + cnt, cap);
        for (uint32_t c = (at + kChunkPairs - 1) / kChunkPairs; (uint64_t)c * kChunkPairs < end; ++c) chunk_rank[c] = (uint32_t)r;
    }
    sEnd[wave][lane] = at + cnt;
    const uint32_t first = (uint32_t)__builtin_amdgcn_readlane((int)at, 0);
    const uint32_t last = (uint32_t)__builtin_amdgcn_readlane((int)(at + cnt), 63);
    __builtin_amdgcn_wave_barrier();
    bool dropped = false;
    // Uniform trip count: every lane takes part in the cross-lane reads of each step (a lane that has left the loop
    // could not be read by the others), only lanes with a slot in range store.
    for (uint32_t base = first; base < last; base += 64) {
        const uint32_t u = base + lane;
        const bool mine = u < last;
        // owner = first lane whose range end exceeds u (clamped for lanes without a slot)
        int lo = 0;
#pragma unroll
        for (int step = 32; step >= 1; step >>= 1)
            if (sEnd[wave][lo + step - 1] <= u) lo += step;
        const int ox0 = __shfl(x0, lo, 64), oy0 = __shfl(y0, lo, 64), ow = __shfl(w, lo, 64);
        const uint32_t oid = (uint32_t)__shfl((int)id, lo, 64), oat = (uint32_t)__shfl((int)at, lo, 64);
        if (mine && ow > 0) {
            const int t = (int)(u - oat);
            const int ty = oy0 + t / ow, tx = ox0 + t - (t / ow) * ow;
            if (u < cap) {
                tkeys[u] = (uint32_t)(ty * cam.TX + tx);
                tvals[u] = oid;
            } else {
                dropped = true;
            }
        }
    }
    if (dropped) status[kStOverflow] = 1u;
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
        if (i >= P || tile >= ntiles) continue;     // tile >= ntiles cannot happen for keys written by k_duplicate; keeps the writes in bounds regardless
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
constexpr uint32_t kOrderRounds = 8;        // rounds of 64 tiles whose ranges are loaded together (one trip to memory, not eight)

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

__global__ __launch_bounds__(1024) void k_tile_order(const uint32_t* __restrict__ ranges, uint32_t ntiles, uint32_t* __restrict__ tile_order)
{
    __shared__ uint32_t count[64 * 16];      // [class][wavefront]: tiles, then where the wavefront's next tile of the class goes
    const uint32_t lane = threadIdx.x & 63u, w = threadIdx.x >> 6;
    const uint32_t per_wave = ((ntiles + 1023u) / 1024u) * 64u;
    const uint32_t t0 = w * per_wave, t1 = min(ntiles, t0 + per_wave);
    const uint64_t below = (1ull << lane) - 1ull;
    const uint2* range2 = reinterpret_cast<const uint2*>(ranges);

    count[threadIdx.x] = 0u;
    __syncthreads();
    uint32_t cls[kOrderRounds];
    for (uint32_t tb = t0; tb < t1; tb += kOrderRounds * 64u) {
        order_classes(range2, tb, t1, lane, cls);
#pragma unroll
        for (uint32_t k = 0; k < kOrderRounds; ++k) {
            const uint64_t same = lanes_of_my_class(cls[k]);
            if ((same & below) == 0ull && cls[k] != 63u) count[cls[k] * 16u + w] += (uint32_t)__popcll(same);      // first lane of its class
        }
    }
    __syncthreads();
    if (w == 0) {      // exclusive prefix sums over (class, wavefront), classes 0 .. kOrderClasses - 1: 10 consecutive entries per lane
        constexpr int kPer = kOrderClasses * 16 / 64;
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
    for (uint32_t tb = t0; tb < t1; tb += kOrderRounds * 64u) {
        if (per_wave > kOrderRounds * 64u) order_classes(range2, tb, t1, lane, cls);      // else still there from the counting pass
#pragma unroll
        for (uint32_t k = 0; k < kOrderRounds; ++k) {
            const uint64_t same = lanes_of_my_class(cls[k]);
            const uint32_t slot = cls[k] * 16u + w;
            const uint32_t at = count[slot];      // every lane of the class reads it before its first lane moves it on
            if (cls[k] != 63u) {
                tile_order[at + (uint32_t)__popcll(same & below)] = tb + k * 64u + lane;
                if ((same & below) == 0ull) count[slot] = at + (uint32_t)__popcll(same);
            }
        }
    }
}

// Inspection only: the 64-bit keys (tile << 32 | depth bits) of the sorted pairs, rebuilt from the sorted tile ids
// and the per-point depth bits.
__global__ __launch_bounds__(256) void k_make_keys64(const uint32_t* __restrict__ tkeys, const uint32_t* __restrict__ tvals,
                                                     const uint32_t* __restrict__ depth_bits, const uint32_t* __restrict__ status,
                                                     uint32_t cap, uint64_t* __restrict__ keys64)
{
    const uint32_t P = min(status[kStNumDup], cap);
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= P) return;
    keys64[i] = ((uint64_t)tkeys[i] << 32) | depth_bits[tvals[i]];
}

hipError_t launch_make_keys64(const Layout& L, char* ws, hipStream_t s)
{
    const uint32_t* status = reinterpret_cast<const uint32_t*>(ws + L.off_status);
    const uint32_t* tk = reinterpret_cast<const uint32_t*>(ws + sorted_tkeys_off(L));
    const uint32_t* tv = reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L));
    hipLaunchKernelGGL(k_make_keys64, dim3((L.cap + 255u) / 256u), dim3(256), 0, s, tk, tv,
                       reinterpret_cast<const uint32_t*>(ws + L.off_depth_bits), status, L.cap,
                       reinterpret_cast<uint64_t*>(ws + L.off_keys64));
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

// visible points per block of 256, scanned in place; leaves the visible count in the status words. Also the call's
// first launch: clears the status words and the tile ranges.
hipError_t launch_count_visible(const BinInput& in, const CamDev& cam, const Layout& L, char* ws, hipStream_t s)
{
    const int n = in.n;
    if (n == 0) return hipSuccess;
    uint32_t* vis_block = reinterpret_cast<uint32_t*>(ws + L.off_vis_block);
    uint32_t* status = reinterpret_cast<uint32_t*>(ws + L.off_status);
    const unsigned nb = (unsigned)((n + 255) / 256);
    ProfScope prof(kKCountPack, s);
    hipLaunchKernelGGL(k_count_visible, dim3(nb), dim3(256), 0, s, in, cam, reinterpret_cast<uint32_t*>(ws + L.off_touched), vis_block,
                       status, reinterpret_cast<uint32_t*>(ws + L.off_ranges), (uint32_t)(2 * (size_t)L.tiles));
    hipLaunchKernelGGL(k_scan_partials, dim3(1), dim3(1024), 0, s, vis_block, nb, status + kStNumVis);
    return hipGetLastError();
}

hipError_t launch_count_pack(const SplatsDev& sp, const CamDev& cam, const Layout& L, char* ws, hipStream_t s)
{
    if (sp.n == 0) return hipSuccess;
    hipError_t e = launch_count_visible(BinInput{sp.n, sp.mean2d, sp.radius}, cam, L, ws, s);
    if (e != hipSuccess) return e;
    ProfScope prof(kKCountPack, s);
    hipLaunchKernelGGL(k_count_pack, dim3((unsigned)((sp.n + 255) / 256)), dim3(256), 0, s, sp, cam,
                       reinterpret_cast<const uint32_t*>(ws + L.off_vis_block), reinterpret_cast<const uint32_t*>(ws + L.off_touched), reinterpret_cast<Packed*>(ws + L.off_packed),
                       reinterpret_cast<uint32_t*>(ws + L.off_dkey0), reinterpret_cast<uint32_t*>(ws + L.off_dval0),
                       reinterpret_cast<uint32_t*>(ws + L.off_depth_bits));
    return hipGetLastError();
}

// Everything after the per-point counts and (depth bits, index) pairs are in place: depth order, prefix sum,
// duplication, tile sort, tile ranges.
hipError_t launch_bin_finish(const BinInput& sp, const CamDev& cam, const Layout& L, char* ws, hipStream_t s)
{
    if (sp.n == 0) return hipSuccess;
    uint32_t* status = reinterpret_cast<uint32_t*>(ws + L.off_status);
    uint32_t* touched = reinterpret_cast<uint32_t*>(ws + L.off_touched);
    uint32_t* offsets = reinterpret_cast<uint32_t*>(ws + L.off_offsets);
    uint32_t* slot_base = reinterpret_cast<uint32_t*>(ws + L.off_slot_base);
    uint32_t* part = reinterpret_cast<uint32_t*>(ws + L.off_scan_part);
    uint32_t* ranges = reinterpret_cast<uint32_t*>(ws + L.off_ranges);
    uint32_t* dk[2] = {reinterpret_cast<uint32_t*>(ws + L.off_dkey0), reinterpret_cast<uint32_t*>(ws + L.off_dkey1)};
    uint32_t* dv[2] = {reinterpret_cast<uint32_t*>(ws + L.off_dval0), reinterpret_cast<uint32_t*>(ws + L.off_dval1)};
    uint32_t* tk[2] = {reinterpret_cast<uint32_t*>(ws + L.off_tkey0), reinterpret_cast<uint32_t*>(ws + L.off_tkey1)};
    uint32_t* tv[2] = {reinterpret_cast<uint32_t*>(ws + L.off_tval0), reinterpret_cast<uint32_t*>(ws + L.off_tval1)};
    uint32_t* totals = reinterpret_cast<uint32_t*>(ws + L.off_totals);
    uint32_t* tile_hist = reinterpret_cast<uint32_t*>(ws + L.off_tile_hist);
    const unsigned nblk = (unsigned)((sp.n + 255) / 256);
    // depth digits: sort the visible splats by their 32 depth bits (four passes, result back in the "0" buffers)
    hipError_t e = launch_radix_sort32(dk, dv, status + kStNumVis, (uint32_t)sp.n, 32, totals, tile_hist, s);
    if (e != hipSuccess) return e;
    const uint32_t* order = dv[radix_pass_count(32) & 1];
    {
        ProfScope prof(kKCountPack, s);
        hipLaunchKernelGGL(k_rank_counts, dim3((unsigned)(sp.n / 1024 + 1)), dim3(256), 0, s, sp.n, status, order, touched, offsets);
    }
    e = launch_exclusive_scan(offsets, offsets, (uint32_t)sp.n + 1u, part, status + kStNumDup, s);
    if (e != hipSuccess) return e;
    {
        ProfScope prof(kKDuplicate, s);
        hipLaunchKernelGGL(k_duplicate, dim3(nblk), dim3(256), 0, s, sp, cam, order, offsets, tk[0], tv[0], slot_base,
                           reinterpret_cast<uint32_t*>(ws + L.off_chunk_rank), L.cap, status);
    }
    // tile digits: stable sort of the P pairs by tile id
    e = launch_radix_sort32(tk, tv, status + kStNumDup, L.cap, L.tile_bits, totals + kRadixMaxBins, tile_hist, s);
    if (e != hipSuccess) return e;
    {
        ProfScope prof(kKTileRanges, s);
        const uint32_t* sorted = reinterpret_cast<const uint32_t*>(ws + sorted_tkeys_off(L));
        hipLaunchKernelGGL(k_tile_ranges, dim3((L.cap + 1023u) / 1024u), dim3(256), 0, s, sorted, status, L.cap, (uint32_t)L.tiles, ranges);
        // the call's tile grid (a patch covers fewer tiles than the image the workspace is sized for)
        hipLaunchKernelGGL(k_tile_order, dim3(1), dim3(1024), 0, s, ranges, (uint32_t)(cam.TX * cam.TY),
                           reinterpret_cast<uint32_t*>(ws + L.off_tile_order));
    }
    return hipGetLastError();
}

hipError_t launch_bin_sort(const SplatsDev& sp, const CamDev& cam, const Layout& L, char* ws, hipStream_t s)
{
    if (sp.n == 0) return launch_bin_begin(L, ws, s);      // nothing to count: only the cleared status words and ranges
    hipError_t e = launch_count_pack(sp, cam, L, ws, s);
    if (e != hipSuccess) return e;
    return launch_bin_finish(BinInput{sp.n, sp.mean2d, sp.radius}, cam, L, ws, s);
}

}  // namespace pbdr
