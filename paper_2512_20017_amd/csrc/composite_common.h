// Device helpers shared by the compositing kernels of the 3D-Gaussian and the 2D-surfel variants.
#pragma once
#include "pbdr_internal.h"

namespace pbdr {

constexpr int kBatch = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLog2_255 = 7.994353436858858f;

struct TileCtx {
    int px, py;       // this lane's pixel
    int tx0, ty0;     // tile origin in pixels
    bool inside;
    uint32_t pix;
    uint32_t start, end;
};

__device__ __forceinline__ TileCtx tile_ctx(const CamDev& cam, const uint32_t* __restrict__ ranges)
{
    TileCtx c;
    const int tile = blockIdx.x;
    const int ty = tile / cam.TX, tx = tile - ty * cam.TX;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    c.tx0 = tx * kTile; c.ty0 = ty * kTile;
    c.px = c.tx0 + (wave & 1) * 8 + (lane & 7);
    c.py = c.ty0 + (wave >> 1) * 8 + (lane >> 3);
    c.inside = c.px < cam.W && c.py < cam.H;
    c.pix = (uint32_t)c.py * (uint32_t)cam.W + (uint32_t)c.px;
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

// Sum over the 64 lanes of a wavefront with DPP row shifts and row broadcasts (no LDS traffic); the total ends
// up in lane 63 and is returned in every lane through a readlane.
__device__ __forceinline__ float wave_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111, 0xf, 0xf, true));  // row_shr:1
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x112, 0xf, 0xf, true));  // row_shr:2
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x114, 0xf, 0xf, true));  // row_shr:4
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x118, 0xf, 0xf, true));  // row_shr:8
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xa, 0xf, false)); // row_bcast:15
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xc, 0xf, false)); // row_bcast:31
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

template <int kCtrl>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xf, 0xf, false));
}

// Sums eight values over each row of 16 lanes at once by recursive halving: at each of three exchange steps a lane
// keeps half of its values and hands the other half to its partner (lane ^ 1, lane ^ 3, lane ^ 7: DPP quad
// permutes and the half-row mirror), then one full-row mirror add finishes. 22 VALU instructions instead of 8 x 4.
// On return the lane holds the row sum of value number 4*r1 + 2*r2 + r3, where, with b_i the bits of its lane
// number, r1 = b0^b1, r2 = b1^b2, r3 = b2^b3 (each pairing flips exactly one of the rules it must, and none of the
// earlier ones).
__device__ __forceinline__ float row_sum8(const float v[8], bool r1, bool r2, bool r3)
{
    float a[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float keep = r1 ? v[i + 4] : v[i], send = r1 ? v[i] : v[i + 4];
        a[i] = keep + dpp_move<0xB1>(send);        // quad_perm:[1,0,3,2]
    }
    float c[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const float keep = r2 ? a[i + 2] : a[i], send = r2 ? a[i] : a[i + 2];
        c[i] = keep + dpp_move<0x1B>(send);        // quad_perm:[3,2,1,0]
    }
    const float keep = r3 ? c[1] : c[0], send = r3 ? c[0] : c[1];
    float d = keep + dpp_move<0x141>(send);        // row_half_mirror
    d += dpp_move<0x140>(d);                       // row_mirror
    return d;
}

// Adds the four rows of 16 lanes of a wavefront lane by lane; the total is valid in lanes 48..63 only.
// v_permlane16_swap / v_permlane32_swap (gfx950) exchange odd rows (the upper half) of their first operand with even
// rows (the lower half) of the second: with both operands equal, rows 1 and 3 receive rows 0 and 2, then the upper
// half receives the lower half. Only the first result of each builtin is used.
__device__ __forceinline__ float rows_sum_to_row3(float v)
{
    const unsigned u = __builtin_bit_cast(unsigned, v);
    const float s = v + __builtin_bit_cast(float, __builtin_amdgcn_permlane16_swap(u, u, false, false)[0]);
    const unsigned us = __builtin_bit_cast(unsigned, s);
    return s + __builtin_bit_cast(float, __builtin_amdgcn_permlane32_swap(us, us, false, false)[0]);
}

// inclusive row scan by shifts: lane 15 of each row ends up with the row sum
__device__ __forceinline__ float row_sum_to_lane15(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x112, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x114, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x118, 0xf, 0xf, true));
    return v;
}

}  // namespace pbdr
