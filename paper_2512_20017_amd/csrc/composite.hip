// Per-tile compositing, forward and backward (image_render and image_render.backward: paper Sec. 2.1 "computes the
// color of each pixel front to back, blending the overlapping splats until full opacity is reached"; Alg. 1
// lines 12 and 18).
//
// One workgroup (4 wavefronts of 64) per 16x16 tile; each wavefront owns one 8x8 pixel quadrant. The tile's
// depth-sorted list is staged through LDS 256 splats at a time (one 48-byte record per thread). While staging, each
// thread works out which of the four quadrants its splat can reach at all with alpha >= 1/255 (exact minimum of
// the quadratic form over the quadrant rectangle, taken conservatively), and the wavefronts ballot these into one
// 256-bit mask per quadrant. A wavefront then walks only the set bits of its own mask with scalar bit scans, so a
// splat that cannot touch the quadrant costs it nothing. The cull never changes a result: every visited
// (pixel, splat) pair still takes the full per-pixel tests.
//
// The per-pair arithmetic is branch-free and in the log2 domain: alpha = min(0.99, 2^(log2 o - q(d))) with
// q = log2(e) * sigma folded into the staged conic. Plain VALU work: no dense contraction, so no MFMA.
#include "composite_common.h"
#include "pair_reduce.h"

#include <type_traits>

namespace pbdr {

// value of q(dx,dy) = A dx^2 + B dx dy + C dy^2
__device__ __forceinline__ float qform(float A, float B, float C, float dx, float dy)
{
    return (A * dx + B * dy) * dx + C * dy * dy;
}

// Minimum of the positive-definite form q over the rectangle [lx,hx] x [ly,hy] (offsets from the splat centre).
// With (xs, ys) the point of the rectangle nearest the centre coordinate by coordinate, the minimum lies on the
// segment x = xs or on the segment y = ys of the rectangle: q is convex with its minimum 0 at the centre, so from the
// minimiser a step towards the centre must leave the rectangle, which makes x = xs or y = ys there (and if the centre
// is inside, both segments pass through it). Two one-dimensional minimisations instead of one per edge.
__device__ __forceinline__ float qform_min_rect(float A, float B, float C, float lx, float hx, float ly, float hy)
{
    const float xs = fminf(hx, fmaxf(lx, 0.f)), ys = fminf(hy, fmaxf(ly, 0.f));
    const float i2C = 0.5f / C, i2A = 0.5f / A;
    const float yv = fminf(hy, fmaxf(ly, -B * xs * i2C));
    const float xh = fminf(hx, fmaxf(lx, -B * ys * i2A));
    return fminf(qform(A, B, C, xs, yv), qform(A, B, C, xh, ys));
}

constexpr int kAccStride = 9;    // floats between the LDS accumulators of consecutive splats of a batch (odd)

// A staged splat of the forward kernel: 48 bytes, so that one LDS address register serves the three reads of a visit.
struct StageRec {
    float4 a;                              // mx, my, A = log2e/2 * qa, B = log2e * qb
    float4 b;                              // C = log2e/2 * qc, L = log2(opacity), red, green
    float c, pad[3];                       // blue
};

// LDS image of one staged batch of kB splats of the backward kernel (kB a multiple of 64, at most the workgroup size):
// the three parts of a record in arrays of their own, 36 bytes a splat - that kernel's occupancy is set by its LDS
// (the forward kernel measured 7 % slower with this layout).
template <int kB>
struct Stage {
    float4 va[kB];
    float4 vb[kB];
    float vc[kB];
    unsigned long long mask[4][kB / 64];   // [quadrant][staging wavefront]: which of its 64 splats reach the quadrant
    uint32_t definite[kB / 64];            // [staging wavefront]: all of its splats have a positive-definite conic, with margin
    __device__ __forceinline__ void put(int j, const float4& a, const float4& b, float c) { va[j] = a; vb[j] = b; vc[j] = c; }
    __device__ __forceinline__ float4 a(int j) const { return va[j]; }
    __device__ __forceinline__ float4 b(int j) const { return vb[j]; }
    __device__ __forceinline__ float c(int j) const { return vc[j]; }
};

// Can the splat reach the quadrant whose first pixel centre lies at (lx, ly) from the splat centre, with alpha >= 1/255,
// i.e. q(d) <= tau = L + log2(255) somewhere on it? Exact minimum of the form over the rectangle, kept when in doubt:
// rounding can only keep more. pd: the conic is positive definite (else every quadrant is kept).
__device__ __forceinline__ bool quadrant_reach(float A, float B, float C, float tau, bool pd, float lx, float ly)
{
    if (tau < -0.05f) return false;
    if (!pd) return true;
    const float hx = lx + 7.f, hy = ly + 7.f;
    const float mn = qform_min_rect(A, B, C, lx, hx, ly, hy);
    const float mxd = fmaxf(fabsf(lx), fabsf(hx)), myd = fmaxf(fabsf(ly), fabsf(hy));
    const float big = A * mxd * mxd + C * myd * myd + fabsf(B) * mxd * myd;
    return !(mn > tau + 0.05f + 4e-6f * big);
}

// "positive definite with a margin that rounding cannot bridge": the quadratic form is then never negative and the
// per-pixel sign test can be left out (see the walk loops)
__device__ __forceinline__ bool safely_definite(float A, float B, float C)
{
    return (A > 0.f) && (C > 0.f) && (4.f * A * C > 1.00001f * (B * B));
}

// Backward pass: stage list entries [first, first+count) of the tile, count <= kB, one per thread. Returns this thread's
// splat index, raw conic/opacity and (mean2d, extent). All 256 threads must call it.
// reach_bits: four bytes per list position, one per quadrant, written by the forward pass's wavefront of that quadrant
// for the positions it staged (bit 0: the splat can reach the quadrant). The backward pass walks a prefix of what each
// forward wavefront walked, so every byte it acts on was written by this view's forward pass; the bytes of positions a
// quadrant never came to are stale or zero, and the walk of that quadrant never gets there (its pixels' last indices
// end earlier).
template <int kB>
__device__ __forceinline__ void stage_batch_bwd(Stage<kB>& S, const uint32_t* __restrict__ vals,
                                                const Packed* __restrict__ packed, const uint32_t* __restrict__ reach_words,
                                                uint32_t first, int count, uint32_t id_ahead, uint32_t& id, float4& raw, float4& geo)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool have = (int)threadIdx.x < count;
    uint32_t bits = 0;
    bool definite = true;
    id = 0; raw = make_float4(0.f, 0.f, 0.f, 0.f); geo = raw;
    if (have) {
        id = id_ahead;                 // vals[first + threadIdx.x], asked for a batch ahead
        bits = reach_words[first + threadIdx.x];
        const float4* rec = reinterpret_cast<const float4*>(packed + id);
        const float4 r0 = rec[0], r1 = rec[1], r2 = rec[2];
        const float mx = r0.x, my = r0.y, qa = r0.z, qb = r0.w, qc = r1.x, o = r1.y;
        raw = make_float4(qa, qb, qc, o);
        geo = make_float4(mx, my, r2.y, 0.f);   // r2.y carries the extent (integer bits)
        const float A = 0.5f * kLog2e * qa, B = kLog2e * qb, C = 0.5f * kLog2e * qc;
        const float L = __log2f(o);
        S.put(threadIdx.x, make_float4(mx, my, A, B), make_float4(C, L, r1.z, r1.w), r2.x);
        definite = safely_definite(A, B, C);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const unsigned long long m = __ballot(((bits >> (8 * q)) & 1u) != 0u);
        if (lane == 0 && wave < kB / 64) S.mask[q][wave] = m;
    }
    const unsigned long long dm = __ballot(definite);
    if (lane == 0 && wave < kB / 64) S.definite[wave] = (dm == ~0ull) ? 1u : 0u;
}

// Forward. The four wavefronts of a tile do not wait for each other: each stages the list for itself, 64 splats at a
// time (one per lane, into its own 3 KB of LDS), tests them against its own quadrant only, and stops when its 64 pixels
// have ended. (When the four staged 256 splats together, every batch ended with the quadrants waiting at a barrier for
// the one with the most splats to visit; the records are read four times now, from L2.)
constexpr int kFwdBatch = 64;

__global__ __launch_bounds__(256) void k_composite_fwd(CamDev cam, const uint32_t* __restrict__ ranges, const uint32_t* __restrict__ tile_order,
                                                       const uint32_t* __restrict__ vals, const Packed* __restrict__ packed,
                                                       uint8_t* __restrict__ reach_bits, float bg0, float bg1, float bg2,
                                                       float* __restrict__ image, float* __restrict__ final_T,
                                                       uint32_t* __restrict__ last_idx)
{
    __shared__ StageRec sRec[4][kFwdBatch];
    const TileCtx c = tile_ctx(cam, ranges, tile_order);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    StageRec* const rec_w = sRec[wave];
    const float fx = (float)c.px + 0.5f, fy = (float)c.py + 0.5f;
    // centre of the quadrant's first pixel
    const float qx0 = (float)(c.tx0 + (wave & 1) * 8) + 0.5f, qy0 = (float)(c.ty0 + (wave >> 1) * 8) + 0.5f;
    float T = 1.f, C0 = 0.f, C1 = 0.f, C2 = 0.f;
    uint32_t last = 0;
    bool live = c.inside;
    for (uint32_t base = c.start; base < c.end; base += kFwdBatch) {
        if (__ballot(live) == 0ull) break;           // every pixel of the quadrant has ended
        const int cnt = (int)min((uint32_t)kFwdBatch, c.end - base);
        bool reach = false, definite = true;
        if (lane < cnt) {
            const uint32_t id = vals[base + lane];
            const float4* rec = reinterpret_cast<const float4*>(packed + id);
            const float4 r0 = rec[0], r1 = rec[1], r2 = rec[2];
            const float mx = r0.x, my = r0.y;
            const float A = 0.5f * kLog2e * r0.z, B = kLog2e * r0.w, C = 0.5f * kLog2e * r1.x;
            const float L = __log2f(r1.y);
            rec_w[lane].a = make_float4(mx, my, A, B);
            rec_w[lane].b = make_float4(C, L, r1.z, r1.w);
            rec_w[lane].c = r2.x;
            const bool pd = (A > 0.f) && (C > 0.f) && (4.f * A * C > B * B);
            definite = safely_definite(A, B, C);
            reach = quadrant_reach(A, B, C, L + kLog2_255, pd, qx0 - mx, qy0 - my);      // alpha >= 1/255 <=> q(d) <= L + log2(255)
            reach_bits[(size_t)4 * (base + lane) + wave] = reach ? 1 : 0;
        }
        unsigned long long m = __ballot(reach);
        const bool all_definite = __ballot(!definite) == 0ull;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t pos0 = base - c.start + 1u;
        // kSign: keep the "quadratic form < 0 -> skip" test per pixel; not needed when every splat of the batch has a
        // positive-definite conic (every state that pbdr_preprocess writes)
        auto walk = [&](auto sign_test) {
            constexpr bool kSign = decltype(sign_test)::value;
            // alpha of one visit: everything that does not depend on the pixel's running state
            auto eval = [&](int j, float& alpha, bool& ok, float& r, float& g, float& bl) {
                const float4 a = rec_w[j].a;
                const float4 b = rec_w[j].b;
                bl = rec_w[j].c; r = b.z; g = b.w;
                const float dx = fx - a.x, dy = fy - a.y;
                const float q = (a.z * dx + a.w * dy) * dx + b.x * dy * dy;
                alpha = fminf(kAlphaMax, __builtin_amdgcn_exp2f(b.y - q));
                ok = (!kSign || q >= 0.f) && (alpha >= kAlphaMin);
            };
            auto blend_one = [&](int j, float alpha, bool ok, float r, float g, float bl) {
                const bool valid = live && ok;
                const float aT = alpha * T;
                const float Tn = T - aT;            // T (1 - alpha), with the product the weight needs anyway
                const bool stop = valid && (Tn < kTStop);
                const bool blend = valid && !stop;
                live = live && !stop;
                const float w = blend ? aT : 0.f;
                C0 += r * w; C1 += g * w; C2 += bl * w;
                T = blend ? Tn : T;
                last = blend ? pos0 + (uint32_t)j : last;
            };
            // two visits per trip while there are two: their alphas do not depend on each other, which gives the
            // vector ALU two independent chains to interleave; the blends stay in list order (four per trip measured slower)
            while (m & (m - 1ull)) {
                const int j0 = __builtin_ctzll(m);
                m &= m - 1ull;
                const int j1 = __builtin_ctzll(m);
                m &= m - 1ull;
                float al0, r0, g0, b0, al1, r1, g1, b1;
                bool ok0, ok1;
                eval(j0, al0, ok0, r0, g0, b0);
                eval(j1, al1, ok1, r1, g1, b1);
                blend_one(j0, al0, ok0, r0, g0, b0);
                blend_one(j1, al1, ok1, r1, g1, b1);
            }
            if (m) {
                const int j0 = __builtin_ctzll(m);
                float al0, r0, g0, b0;
                bool ok0;
                eval(j0, al0, ok0, r0, g0, b0);
                blend_one(j0, al0, ok0, r0, g0, b0);
            }
        };
        if (all_definite) walk(std::false_type{});
        else walk(std::true_type{});
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();             // the next batch overwrites the staged records
    }
    if (c.inside) {
        const size_t HW = (size_t)cam.W * cam.H;
        image[c.pix] = C0 + T * bg0;
        image[HW + c.pix] = C1 + T * bg1;
        image[2 * HW + c.pix] = C2 + T * bg2;
        final_T[c.pix] = T;
        last_idx[c.pix] = last;
    }
}

// Backward. Per pixel, back to front from its last blended splat: T_k = T_{k+1} / (1 - alpha_k),
//   dL/dalpha_k = T_k (c_k . g) - S_k / (1 - alpha_k),  S_k = sum_{i>k} w_i (c_i . g) + T_final (bg . g).
// With ds = dL/dsigma = -alpha dL/dalpha (zero where alpha was clamped), every splat gradient is a sum over pixels of
//   w g_c (3 colours)  and the six moments  ds (1, dx, dy, dx^2, dx dy, dy^2):
//   d conic = (S3/2, S4, S5/2), d mean2d = -(qa S1 + qb S2, qc S2 + qb S1), d opacity = -S0 / o.
//
// The sums over pixels are taken four visits at a time. A visit only stores its ds and w as two rows of 64 floats in
// LDS (a transpose: the values of one visit sit across the lanes, the sums want the pixels of one visit inside a lane).
// After four visits a quarter of the wavefront (16 lanes, one DPP row) takes each visit: a lane reads ds and w of four
// neighbouring pixels, forms their nine weighted sums with weights it holds for the whole tile (the pixels' dL/dcolour
// and their coordinates X, Y inside the tile: with dx = X0 + X, dy = Y0 + Y for a per-(tile, splat) offset (X0, Y0),
// the six moments follow from the moments of ds against 1, X, Y, X^2, XY, Y^2, whatever the splat), and one butterfly
// over the row finishes four visits at once: about 13 vector instructions per visit instead of 39 when every visit
// reduced its own nine products over the 64 lanes.
// (Measured and dropped: one wavefront per tile that takes the four quadrants in turn, with no barriers and plain
// read-modify-writes: 371 us against 239, the few tiles with thousands of splats then run four times longer on one
// wavefront and the launch waits for them. Reading the next splat's staged record while the current one is worked on:
// no change. The same contraction as sixteen v_mfma_f32_16x16x4_f32 per eight visits: an fp32 matrix
// instruction holds the SIMD for its 32 cycles - plain vector instructions of other wavefronts do not overlap with it -
// and only 9 of its 32 output columns are of use, so it came out slower than the butterfly it replaced.)
//
// No atomics, global or LDS: a wavefront stores the row results in its quadrant's accumulator of the staged splat, and
// the thread that staged splat j adds the four quadrants' nine sums, turns them into gradients and writes them
// to partial[u] (12 floats per pair), where u is the pair's position in the unsorted duplicate list (slot_base[id] +
// rank of this tile in the splat's rectangle). A splat's pairs are contiguous there, so a per-splat kernel adds them
// up afterwards (k_gather_splat_grads).
constexpr int kVisitSlots = 4;    // visits staged per reduction: one per row of 16 lanes
constexpr int kBwdBatch = 64;    // splats staged at a time by the backward kernel: what the per-quadrant accumulators leave room for

// 7 workgroups per compute unit: 72 registers
__global__ __launch_bounds__(256, 7) void k_composite_bwd(CamDev cam, const uint32_t* __restrict__ ranges, const uint32_t* __restrict__ tile_order,
                                                       const uint32_t* __restrict__ vals, const Packed* __restrict__ packed,
                                                       uint8_t* __restrict__ reach_bits, const uint32_t* __restrict__ slot_base,
                                                       float bg0, float bg1, float bg2, const float* __restrict__ final_T,
                                                       const uint32_t* __restrict__ last_idx,
                                                       const float* __restrict__ dL_dimage, uint32_t cap,
                                                       const uint32_t* __restrict__ status, float4* __restrict__ partial)
{
    __shared__ Stage<kBwdBatch> S;
    // [quadrant][splat of the batch][value], 9 floats apart (odd: the per-thread reads at the end of a batch are
    // conflict-free): three colour sums, then the moments of ds against 1, X, Y, X^2, XY, Y^2. A wavefront visits a splat
    // at most once per batch, so it writes its quadrant's sums with plain stores; the thread that staged the splat adds
    // the four up. (One accumulator per splat shared by the quadrants takes LDS float atomics, which cost the LDS about
    // 2.5 cycles per active lane: a quarter of this kernel's time when it was built that way.)
    __shared__ float sAcc[4][kAccStride * kBwdBatch];
    __shared__ __align__(16) float sV[4][2 * kVisitSlots * 64];   // per wavefront: rows 2s (ds) and 2s + 1 (w) of visit slot s
    __shared__ uint32_t sMax[4];
    const TileCtx c = tile_ctx(cam, ranges, tile_order);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float fx = (float)c.px + 0.5f, fy = (float)c.py + 0.5f;
    const size_t HW = (size_t)cam.W * cam.H;
    // this call, counted from one (uniform values, kept on the scalar side: the kernel has no vector register to spare)
    const uint32_t epoch_lo = __builtin_amdgcn_readfirstlane(status[kStEpoch]) + 1u;
    const uint32_t epoch_hi = __builtin_amdgcn_readfirstlane(status[kStEpoch + 1]) + (epoch_lo == 0u ? 1u : 0u);
    float T = 1.f, g0 = 0.f, g1 = 0.f, g2c = 0.f;
    uint32_t last = 0;
    if (c.inside) {
        T = final_T[c.pix];
        last = min(last_idx[c.pix], c.end - c.start);   // never walk past the tile's list, whatever the caller passed
        g0 = dL_dimage[c.pix]; g1 = dL_dimage[HW + c.pix]; g2c = dL_dimage[2 * HW + c.pix];
    }
    float Sfx = T * (bg0 * g0 + bg1 * g1 + bg2 * g2c);
    uint32_t wmax = last;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) wmax = max(wmax, (uint32_t)__shfl_xor((int)wmax, d, 64));
    if (lane == 0) sMax[wave] = wmax;
    __syncthreads();
    const uint32_t tile_last = __builtin_amdgcn_readfirstlane(max(max(sMax[0], sMax[1]), max(sMax[2], sMax[3])));
    if (tile_last == 0) return;
    const int tile_x = c.tix, tile_y = c.tiy;
    float* const sVw = sV[wave];
    float* const sAccW = sAcc[wave];
    // In a reduction lane l takes visit slot l / 16 and the four pixels held by the wavefront's lanes 4 pg .. 4 pg + 3,
    // pg = l % 16: half a pixel row of the quadrant. Their dL/dcolour come from those lanes, through LDS.
    const int pg = lane & 15;
    float4 G0, G1, G2;
    {
        sVw[lane] = g0; sVw[64 + lane] = g1; sVw[128 + lane] = g2c;
        __builtin_amdgcn_wave_barrier();
        G0 = *reinterpret_cast<const float4*>(sVw + 4 * pg);
        G1 = *reinterpret_cast<const float4*>(sVw + 64 + 4 * pg);
        G2 = *reinterpret_cast<const float4*>(sVw + 128 + 4 * pg);
        __builtin_amdgcn_wave_barrier();
    }
    // tile coordinates of the first of the four pixels; the others are X + 1, X + 2, X + 3 on the same row
    const float PX = (float)((wave & 1) * 8 + 4 * (pg & 1)), PY = (float)((wave >> 1) * 8 + (pg >> 1));
    const float* const rd_row = sVw + 128 * (lane >> 4) + 4 * pg;
    float* const wr_row = sVw + lane;
    const bool bit1 = (lane & 2) != 0;
    const bool ninth_lane = pg == 15;
    const bool add_lane = ninth_lane || (lane & 1) == 0;
    const int acc_slot = ninth_lane ? 8 : (lane >> 1) & 7;
    int slot_acc = 0;      // lane s: where visit slot s adds its sums (kAccStride * its splat's position in the batch)
    int nslot = 0;         // visits staged since the last reduction (uniform)
    // Reduces the staged rows and adds the sums of the first `count` visit slots to their splats' accumulators.
    auto reduce_slots = [&](int count) {
        __builtin_amdgcn_wave_barrier();
        const float4 d = *reinterpret_cast<const float4*>(rd_row);
        const float4 w = *reinterpret_cast<const float4*>(rd_row + 64);
        __builtin_amdgcn_wave_barrier();
        const float m0 = (d.x + d.y) + (d.z + d.w);
        const float s1 = d.y + 2.f * d.z + 3.f * d.w;             // sum of ds i and of ds i^2 over the pixels X + i
        const float s2 = d.y + 4.f * d.z + 9.f * d.w;
        const float mx = PX * m0 + s1;
        const float mxx = PX * (mx + s1) + s2;                    // sum of ds (PX + i)^2 = PX (PX m0 + 2 s1) + s2
        const float my = PY * m0;
        const float v8[8] = {w.x * G0.x + w.y * G0.y + w.z * G0.z + w.w * G0.w,
                             w.x * G1.x + w.y * G1.y + w.z * G1.z + w.w * G1.w,
                             w.x * G2.x + w.y * G2.y + w.z * G2.z + w.w * G2.w,
                             m0, mx, my, mxx, PY * mx};
        const float part = row_sum8(v8, bit1);
        const float ninth = row_sum16(PY * my);
        const int base = __shfl(slot_acc, lane >> 4, 64);
        if (add_lane && (lane >> 4) < count) sAccW[base + acc_slot] = ninth_lane ? ninth : part;
    };
    const int nbatch = (int)((tile_last + kBwdBatch - 1) / kBwdBatch);
    // the splat index of a thread's entry is asked for one batch ahead: one trip to memory per batch (the record) instead
    // of two in a row
    uint32_t id_ahead = 0;
    {
        const uint32_t p = (uint32_t)(nbatch - 1) * kBwdBatch + threadIdx.x;
        if (threadIdx.x < kBwdBatch && p < tile_last) id_ahead = vals[c.start + p];
    }
    for (int bi = nbatch - 1; bi >= 0; --bi) {
        const uint32_t boff = (uint32_t)bi * kBwdBatch;            // 0-based list position of the batch's first splat
        const int cnt = (int)min((uint32_t)kBwdBatch, tile_last - boff);
        uint32_t id; float4 raw, geo;
        stage_batch_bwd(S, vals, packed, reinterpret_cast<const uint32_t*>(reach_bits), c.start + boff, cnt, id_ahead, id, raw, geo);
        if (bi > 0 && threadIdx.x < kBwdBatch) id_ahead = vals[c.start + boff - kBwdBatch + threadIdx.x];
        // asked for now, used when the batch's records are written: the walk hides the trip
        const uint32_t pair_base = (int)threadIdx.x < cnt ? slot_base[id] : 0u;
#pragma unroll
        for (int k = 0; k < 4 * kAccStride * kBwdBatch / 256; ++k) (&sAcc[0][0])[k * 256 + threadIdx.x] = 0.f;
        __syncthreads();
        if (wmax > boff) {            // else nothing of this batch was blended by this wavefront (uniform per wave)
            // kSign: as in the forward kernel, the per-pixel sign test of the quadratic form is only kept for batches that
            // hold a splat whose conic is not safely positive definite
            auto walk = [&](auto sign_test) {
                constexpr bool kSign = decltype(sign_test)::value;
                for (int k = kBwdBatch / 64 - 1; k >= 0; --k) {
                    unsigned long long m = uniform_u64(S.mask[wave][k]);
                    while (m) {
                        const int bit = 63 - __builtin_clzll(m);
                        m &= ~(1ull << bit);
                        const int j = k * 64 + bit;
                        const uint32_t pos = boff + (uint32_t)j + 1u;           // 1-based list position
                        const float4 a = S.a(j);
                        const float4 b = S.b(j);
                        const float cb = S.c(j);
                        const float dx = fx - a.x, dy = fy - a.y;
                        const float q = (a.z * dx + a.w * dy) * dx + b.x * dy * dy;
                        const float e = __builtin_amdgcn_exp2f(b.y - q);
                        const float alpha = fminf(kAlphaMax, e);
                        const bool hit = (pos <= last) && (!kSign || q >= 0.f) && (alpha >= kAlphaMin);
                        if (__ballot(hit) == 0ull) continue;                   // uniform per wave
                        const float ioma = __builtin_amdgcn_rcpf(1.f - alpha);
                        const float Tk = T * ioma;                              // transmittance in front of this splat
                        const float w = hit ? alpha * Tk : 0.f;
                        const float cg = b.z * g0 + b.w * g1 + cb * g2c;
                        const float dL_dalpha = Tk * cg - Sfx * ioma;
                        const float ds = (hit && e < kAlphaMax) ? -alpha * dL_dalpha : 0.f;
                        T = hit ? Tk : T;
                        Sfx += w * cg;
                        float* const rows = wr_row + 128 * nslot;
                        rows[0] = ds;
                        rows[64] = w;
                        slot_acc = lane == nslot ? kAccStride * j : slot_acc;
                        if (++nslot == kVisitSlots) { reduce_slots(kVisitSlots); nslot = 0; }
                    }
                }
            };
            bool all_definite = true;
#pragma unroll
            for (int k = 0; k < kBwdBatch / 64; ++k) all_definite = all_definite && S.definite[k] != 0u;
            if (all_definite) walk(std::false_type{});
            else walk(std::true_type{});
            if (nslot) { reduce_slots(nslot); nslot = 0; }
        }
        __syncthreads();
        if ((int)threadIdx.x < cnt) {
            // where this (tile, splat) pair sits in the unsorted duplicate list
            int x0, y0, x1, y1;
            tile_rect(cam, geo.x, geo.y, __float_as_int(geo.z), x0, y0, x1, y1);
            const uint32_t u = pair_base + (uint32_t)((tile_y - y0) * (x1 - x0) + (tile_x - x0));
            if (u < cap && tile_x >= x0 && tile_x < x1 && tile_y >= y0 && tile_y < y1) {
                float acc[kAccStride];
#pragma unroll
                for (int k = 0; k < kAccStride; ++k) {
                    const int e = kAccStride * (int)threadIdx.x + k;
                    acc[k] = (sAcc[0][e] + sAcc[1][e]) + (sAcc[2][e] + sAcc[3][e]);
                }
                // from the tile's frame to offsets from the splat centre: dx = X0 + X, dy = Y0 + Y
                int ox = c.tx0, oy = c.ty0;
                asm volatile("" : "+s"(ox), "+s"(oy));      // converted here, per batch: hoisted out of the loop the two floats cost vector registers the walk has not got
                const float X0 = (float)ox + 0.5f - geo.x, Y0 = (float)oy + 0.5f - geo.y;
                const float m0 = acc[3], mx = acc[4], my = acc[5];
                const float s0 = m0, s1 = X0 * m0 + mx, s2 = Y0 * m0 + my;
                const float s3 = X0 * (X0 * m0 + 2.f * mx) + acc[6];
                const float s4 = X0 * (Y0 * m0 + my) + Y0 * mx + acc[7];
                const float s5 = Y0 * (Y0 * m0 + 2.f * my) + acc[8];
                float4* dst = partial + (size_t)3 * u;
                dst[0] = make_float4(-(raw.x * s1 + raw.y * s2), -(raw.z * s2 + raw.y * s1),          // d mean2d
                                     0.5f * s3, s4);                                                  // d conic a, b
                dst[1] = make_float4(0.5f * s5, raw.w > 0.f ? -s0 / raw.w : 0.f,                       // d conic c, d opacity
                                     acc[0], acc[1]);                                                 // d red, d green
                // d blue, then the stamp that tells the gather this record belongs to this backward call
                dst[2] = make_float4(acc[2], 0.f, __uint_as_float(epoch_lo), __uint_as_float(epoch_hi));
            }
        }
        __syncthreads();   // sAcc and the stage are rewritten by the next batch
    }
}

// Adds up, per point, the per-tile partial sums of its pairs (contiguous in the unsorted duplicate list, 48 bytes
// each) into dL/d(splat state) of the visible points; culled points are not written. Balanced by pairs: see
// pair_reduce.h.
// The sums are first stored as one 48-byte record per point, by point index (nine 4-byte stores per point into nine
// planes touch nine cache lines where this touches one),
// then a streaming kernel over all points copies the records of listed points into the planes of the splat-state
// gradient.
struct StoreSplatGrad {
    float4* rec;
    const uint32_t* order;
    __device__ __forceinline__ void operator()(uint32_t rank, const float (&v)[9]) const
    {
        float4* dst = rec + (size_t)3 * order[rank];
        dst[0] = make_float4(v[0], v[1], v[2], v[3]);
        dst[1] = make_float4(v[4], v[5], v[6], v[7]);
        dst[2] = make_float4(v[8], 0.f, 0.f, 0.f);
    }
};

__global__ __launch_bounds__(256) void k_gather_splat_grads(int n, const uint32_t* __restrict__ status,
                                                            const uint32_t* __restrict__ order,
                                                            const uint32_t* __restrict__ offsets,
                                                            const uint32_t* __restrict__ chunk_rank,
                                                            const float4* __restrict__ partial, uint32_t cap,
                                                            float* __restrict__ carry, float4* __restrict__ rec)
{
    __shared__ uint32_t sEnd[4][64];
    const uint32_t w = blockIdx.x * 4u + (threadIdx.x >> 6);
    gather_wave<3, 9, true>(w, n, status, offsets, chunk_rank, partial, cap, carry, sEnd[threadIdx.x >> 6], StoreSplatGrad{rec, order});
}

// also closes the backward call's epoch: the next call stamps its records with a new number
__global__ __launch_bounds__(256) void k_gather_fixup(int n, uint32_t* __restrict__ status, const uint32_t* __restrict__ order,
                                                      uint32_t cap, const float* __restrict__ carry, float4* __restrict__ rec)
{
    gather_fixup<9>(blockIdx.x * 256u + threadIdx.x, status, cap, carry, StoreSplatGrad{rec, order});
    if (blockIdx.x == 0 && threadIdx.x == 0) {      // 64-bit count of backward calls on this workspace
        const uint32_t lo = status[kStEpoch] + 1u;
        status[kStEpoch] = lo;
        if (lo == 0u) status[kStEpoch + 1] = status[kStEpoch + 1] + 1u;
    }
}

// records -> planes, for the points binning listed (tiles_touched > 0)
__global__ __launch_bounds__(256) void k_grad_records_to_planes(int n, const uint32_t* __restrict__ tiles_touched,
                                                                const float4* __restrict__ rec, SplatGradDev g2)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n || tiles_touched[i] == 0) return;
    const size_t N = (size_t)n;
    const float4 a = rec[(size_t)3 * i], b = rec[(size_t)3 * i + 1], c = rec[(size_t)3 * i + 2];
    g2.mean2d[i] = a.x; g2.mean2d[N + i] = a.y;
    g2.conic[i] = a.z; g2.conic[N + i] = a.w; g2.conic[2 * N + i] = b.x;
    g2.opacity[i] = b.y;
    g2.color[i] = b.z; g2.color[N + i] = b.w; g2.color[2 * N + i] = c.x;
}

// Measurement aid: the forward walk with counters instead of colours. counters[0] += list entries examined per pixel
// (up to and including the one that ends the pixel), counters[1] += pairs blended.
__global__ __launch_bounds__(256) void k_render_stats(CamDev cam, const uint32_t* __restrict__ ranges, const uint32_t* __restrict__ tile_order,
                                                      const uint32_t* __restrict__ vals, const Packed* __restrict__ packed,
                                                      unsigned long long* __restrict__ counters)
{
    __shared__ float4 sA[kBatch];
    __shared__ float4 sB[kBatch];
    __shared__ unsigned long long sCnt[2];
    const TileCtx c = tile_ctx(cam, ranges, tile_order);
    const float fx = (float)c.px + 0.5f, fy = (float)c.py + 0.5f;
    float T = 1.f;
    uint32_t examined = 0, blended = 0;
    bool done = !c.inside;
    if (threadIdx.x < 2) sCnt[threadIdx.x] = 0ull;
    for (uint32_t base = c.start; base < c.end; base += kBatch) {
        if (__syncthreads_count(!done) == 0) break;
        const uint32_t idx = base + threadIdx.x;
        if (idx < c.end) {
            const float4* rec = reinterpret_cast<const float4*>(packed + vals[idx]);
            sA[threadIdx.x] = rec[0]; sB[threadIdx.x] = rec[1];
        }
        __syncthreads();
        const int cnt = (int)min((uint32_t)kBatch, c.end - base);
        if (!done) {
            for (int j = 0; j < cnt; ++j) {
                const float4 a = sA[j];
                const float4 b = sB[j];
                const float dx = fx - a.x, dy = fy - a.y;
                const float sigma = 0.5f * (a.z * dx * dx + b.x * dy * dy) + a.w * dx * dy;
                ++examined;
                if (sigma < 0.f) continue;
                const float alpha = fminf(kAlphaMax, b.y * __expf(-sigma));
                if (alpha < kAlphaMin) continue;
                const float Tn = T - alpha * T;     // as the forward kernel forms it
                if (Tn < kTStop) { done = true; break; }
                T = Tn;
                ++blended;
            }
        }
    }
    __syncthreads();
    atomicAdd(&sCnt[0], (unsigned long long)examined);
    atomicAdd(&sCnt[1], (unsigned long long)blended);
    __syncthreads();
    if (threadIdx.x < 2 && sCnt[threadIdx.x]) atomicAdd(&counters[threadIdx.x], sCnt[threadIdx.x]);
}

__global__ __launch_bounds__(256) void k_fill_f32(float* __restrict__ p, float v, size_t count)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = v;
}

hipError_t launch_composite_fwd(const CamDev& cam, const Layout& L, char* ws, const float bg[3], float* image,
                                float* final_T, uint32_t* last_idx, hipStream_t s)
{
    const uint32_t* ranges = reinterpret_cast<const uint32_t*>(ws + L.off_ranges);
    const uint32_t* tile_order = reinterpret_cast<const uint32_t*>(ws + L.off_tile_order);
    const uint32_t* vals = reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L));
    const Packed* packed = reinterpret_cast<const Packed*>(ws + L.off_packed);
    ProfScope prof(kKCompositeFwd, s);
    hipLaunchKernelGGL(k_composite_fwd, dim3((unsigned)(cam.TX * cam.TY)), dim3(256), 0, s, cam, ranges, tile_order, vals, packed,
                       reinterpret_cast<uint8_t*>(ws + L.off_reach), bg[0], bg[1], bg[2], image, final_T, last_idx);
    return hipGetLastError();
}

CarryFold carry_fold(const Layout& L, char* ws)
{
    return CarryFold{reinterpret_cast<const float*>(ws + L.off_carry), reinterpret_cast<const uint32_t*>(ws + L.off_slot_base),
                     reinterpret_cast<uint32_t*>(ws + L.off_status), L.cap};
}

hipError_t launch_composite_bwd(const CamDev& cam, const Layout& L, char* ws, int n, const float bg[3], const float* final_T, const uint32_t* last_idx, const float* dL_dimage,
                                const SplatGradDev& g2, hipStream_t s)
{
    const uint32_t* ranges = reinterpret_cast<const uint32_t*>(ws + L.off_ranges);
    const uint32_t* tile_order = reinterpret_cast<const uint32_t*>(ws + L.off_tile_order);
    const uint32_t* vals = reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L));
    const Packed* packed = reinterpret_cast<const Packed*>(ws + L.off_packed);
    const uint32_t* offsets = reinterpret_cast<const uint32_t*>(ws + L.off_offsets);
    const uint32_t* slot_base = reinterpret_cast<const uint32_t*>(ws + L.off_slot_base);
    const uint32_t* order = reinterpret_cast<const uint32_t*>(ws + L.off_order);
    uint32_t* status = reinterpret_cast<uint32_t*>(ws + L.off_status);
    float4* partial = reinterpret_cast<float4*>(ws + L.off_partial);
    {
        ProfScope prof(kKCompositeBwd, s);
        hipLaunchKernelGGL(k_composite_bwd, dim3((unsigned)(cam.TX * cam.TY)), dim3(256), 0, s, cam, ranges, tile_order, vals, packed,
                           reinterpret_cast<uint8_t*>(ws + L.off_reach), slot_base, bg[0], bg[1], bg[2], final_T, last_idx, dL_dimage,
                           L.cap, status, partial);
    }
    if (n > 0) {
        ProfScope prof(kKGather, s);
        const uint32_t* chunk_rank = reinterpret_cast<const uint32_t*>(ws + L.off_chunk_rank);
        float* carry = reinterpret_cast<float*>(ws + L.off_carry);
        const unsigned nwave = (unsigned)((L.cap + kChunkPairs - 1) / kChunkPairs);
        float4* rec = reinterpret_cast<float4*>(ws + L.off_grad_rec);
        hipLaunchKernelGGL(k_gather_splat_grads, dim3((nwave + 3) / 4), dim3(256), 0, s, n, status, order, offsets, chunk_rank,
                           partial, L.cap, carry, rec);
        if (g2.mean2d != nullptr) {
            hipLaunchKernelGGL(k_gather_fixup, dim3((nwave + 255) / 256), dim3(256), 0, s, n, status, order, L.cap, carry, rec);
            hipLaunchKernelGGL(k_grad_records_to_planes, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, n,
                               reinterpret_cast<const uint32_t*>(ws + L.off_touched), rec, g2);
        }
        // else the caller goes on from the records with launch_preprocess_bwd_records, whose kernel puts the records cut
        // by wavefront boundaries together itself and closes the epoch (carry_fold below): one launch fewer
    }
    return hipGetLastError();
}

hipError_t launch_render_stats(const CamDev& cam, const Layout& L, char* ws, uint64_t* counters, hipStream_t s)
{
    const uint32_t* ranges = reinterpret_cast<const uint32_t*>(ws + L.off_ranges);
    const uint32_t* tile_order = reinterpret_cast<const uint32_t*>(ws + L.off_tile_order);
    const uint32_t* vals = reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L));
    const Packed* packed = reinterpret_cast<const Packed*>(ws + L.off_packed);
    ProfScope prof(kKStats, s);
    hipLaunchKernelGGL(k_fill_f32, dim3(1), dim3(256), 0, s, reinterpret_cast<float*>(counters), 0.f, (size_t)4);
    hipLaunchKernelGGL(k_render_stats, dim3((unsigned)(cam.TX * cam.TY)), dim3(256), 0, s, cam, ranges, tile_order, vals, packed,
                       reinterpret_cast<unsigned long long*>(counters));
    return hipGetLastError();
}

}  // namespace pbdr
