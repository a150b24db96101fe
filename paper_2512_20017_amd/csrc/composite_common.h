// Device helpers shared by the compositing kernels of the 3D-Gaussian and the 2D-surfel variants.
#pragma once
#include "pbdr_internal.h"

namespace pbdr {

constexpr int kBatch = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLog2_255 = 7.994353436858858f;

struct TileCtx {
    int px, py;       // this lane's pixel (image coordinates)
    int tx0, ty0;     // tile origin in pixels (image coordinates)
    int tix, tiy;     // tile coordinates within the call's tile grid
    bool inside;      // the pixel belongs to the rendered patch
    uint32_t pix;     // its index in the output buffers
    uint32_t start, end;
};

// Workgroup b takes tile tile_order[b]: the hardware starts workgroups in index order, and the order array lists the
// tiles with the longest lists first (k_tile_order), so the launch does not end on a few long tiles with the chip idle.
__device__ __forceinline__ TileCtx tile_ctx(const CamDev& cam, const uint32_t* __restrict__ ranges,
                                            const uint32_t* __restrict__ tile_order)
{
    TileCtx c;
    const int tile = (int)tile_order[blockIdx.x];
    const int ty = tile / cam.TX, tx = tile - ty * cam.TX;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    c.tix = tx; c.tiy = ty;
    c.tx0 = (cam.otx + tx) * kTile; c.ty0 = (cam.oty + ty) * kTile;
    c.px = c.tx0 + (wave & 1) * 8 + (lane & 7);
    c.py = c.ty0 + (wave >> 1) * 8 + (lane >> 3);
    c.inside = c.px >= cam.rx0 && c.px < cam.rx1 && c.py >= cam.ry0 && c.py < cam.ry1;
    c.pix = (uint32_t)(c.py - cam.ry0) * (uint32_t)cam.W + (uint32_t)(c.px - cam.rx0);
    c.start = ranges[2 * tile];
    c.end = ranges[2 * tile + 1];
    return c;
}

__device__ __forceinline__ unsigned long long uniform_u64(unsigned long long v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}

template <int kCtrl>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xf, 0xf, false));
}

// Sums eight values over each row of 16 lanes at once by recursive halving: at each of three exchange steps a lane
// keeps half of its values and adds its partner's copy of that half, then one more pairing finishes.
//   step 1: partner lane ^ 8 (row_ror:8);           lanes with bit 3 clear keep values 0..3, the others 4..7
//   step 2: partner lane ^ 7 (row_half_mirror);     lanes with bit 2 clear keep the first two of those, the others the rest
//   step 3: partner lane ^ 3 (quad_perm [3,2,1,0]); lanes with bit 1 clear keep the first of those two
//   last  : partner lane ^ 1 (quad_perm [1,0,3,2]); plain add
// Each partner differs from the lane in exactly the bit that decides the step and in none of the bits that decided
// earlier steps, so both hold the same values. Bits 3 and 2 are the quad a lane sits in, which is what a DPP bank
// mask selects: steps 1 and 2 are two masked adds per output and no select (written as assembly because the compiler
// has no form for a masked DPP write; the s_nop's cover the VALU-write -> DPP-read wait states inside and on both
// sides of the block). 16 VALU instructions instead of 8 x 4. Every lane of the wavefront must be active.
// On return the lane holds the row sum of value number (lane >> 1) & 7; lanes 2k and 2k+1 hold the same number.
__device__ __forceinline__ float row_sum8(const float v[8], bool bit1)
{
    float a[4], c[2];
    asm volatile(
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %6, %6 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %1, %7, %7 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %2, %8, %8 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %3, %9, %9 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %0, %10, %10 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %1, %11, %11 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %2, %12, %12 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %3, %13, %13 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %4, %0, %0 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %5, %1, %1 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %4, %2, %2 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %5, %3, %3 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
        "s_nop 1"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3]), "=&v"(c[0]), "=&v"(c[1])
        : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]));
    const float keep = bit1 ? c[1] : c[0], send = bit1 ? c[0] : c[1];
    float d = keep + dpp_move<0x1B>(send);         // quad_perm:[3,2,1,0]
    d += dpp_move<0xB1>(d);                        // quad_perm:[1,0,3,2]
    return d;
}

// Adds the four rows of 16 lanes of a wavefront lane by lane; every row ends up with the total.
// v_permlane16_swap (gfx950) exchanges the odd rows of its first operand with the even rows of its second, in both
// registers: from two copies of v = [r0 r1 r2 r3] it leaves [r0 r0 r2 r2] and [r1 r1 r3 r3], whose sum holds r0 + r1 in
// rows 0, 1 and r2 + r3 in rows 2, 3. v_permlane32_swap does the same with the halves of the wavefront. Written as
// assembly because both registers are results (the compiler's builtin hands back only one of them correctly); the
// s_nop covers the wait states between a VALU write of an operand and the swap.
__device__ __forceinline__ float sum_rows(float v)
{
    float a = v, b = v;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    const float s = a + b;
    a = s; b = s;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return a + b;
}

// sum over each row of 16 lanes, left in every lane of the row: partners lane ^ 1, ^ 2, ^ 7 (within eight), ^ 15
__device__ __forceinline__ float row_sum16(float v)
{
    asm volatile("" : "+v"(v));   // keeps a product that feeds v from being fused into the first add (which would cost the DPP form)
    v += dpp_move<0xB1>(v);    // quad_perm:[1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm:[2,3,0,1]
    v += dpp_move<0x141>(v);   // row_half_mirror
    v += dpp_move<0x140>(v);   // row_mirror
    return v;
}

}  // namespace pbdr
