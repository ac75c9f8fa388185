// Cross-lane helpers of the serial tree builders: DPP moves, lane reads, wave-wide maximum, sum
// and scan in fp64, and the segment pick with the totals spread over lanes.
#pragma once
#include "vocab_common.h"

namespace dyspec {

// Cross-lane moves of the vector ALU (DPP) for the serial builder's reductions and scan; a
// shuffle would go through the LDS crossbar and wait for it at every step.
constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i of a group of 8 <-> lane 7-i
constexpr int kDppMirror = 0x140;       // lane i of a row of 16 <-> lane 15-i
constexpr int kDppBcast15 = 0x142;      // lane 15 of a row to the next row
constexpr int kDppBcast31 = 0x143;      // lane 31 to rows 2 and 3
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp_or_zero(int x)   // the picked lane's x; 0 where there is none or the row is masked off
{
    return __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ double dpp_or_zero(double x)
{
    return __hiloint2double(dpp_or_zero<CTRL, ROW_MASK>(__double2hiint(x)), dpp_or_zero<CTRL, ROW_MASK>(__double2loint(x)));
}
// Largest value of the wave (values >= -1, no NaN), the same in every lane.
__device__ __forceinline__ double wave_max_dpp(double x)
{
    x = fmax(x, dpp_or_zero<kDppXor1>(x));
    x = fmax(x, dpp_or_zero<kDppXor2>(x));
    x = fmax(x, dpp_or_zero<kDppHalfMirror>(x));
    x = fmax(x, dpp_or_zero<kDppMirror>(x));
    double r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        r[k] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), 16 * k), __builtin_amdgcn_readlane(__double2loint(x), 16 * k));
    return fmax(fmax(r[0], r[1]), fmax(r[2], r[3]));
}
// Sum over the wave, the same in every lane.
__device__ __forceinline__ double wave_sum_dpp(double x)
{
    x += dpp_or_zero<kDppXor1>(x);
    x += dpp_or_zero<kDppXor2>(x);
    x += dpp_or_zero<kDppHalfMirror>(x);
    x += dpp_or_zero<kDppMirror>(x);
    double r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        r[k] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), 16 * k), __builtin_amdgcn_readlane(__double2loint(x), 16 * k));
    return (r[0] + r[1]) + (r[2] + r[3]);
}
// Inclusive scan over the wave in lane order.
__device__ __forceinline__ double wave_scan_dpp(double x)
{
    x += dpp_or_zero<0x111>(x);                  // row_shr:1, 2, 4, 8: scan inside each row of 16
    x += dpp_or_zero<0x112>(x);
    x += dpp_or_zero<0x114>(x);
    x += dpp_or_zero<0x118>(x);
    x += dpp_or_zero<kDppBcast15, 0xa>(x);       // rows 1 and 3 add the total of the row before
    x += dpp_or_zero<kDppBcast31, 0xc>(x);       // rows 2 and 3 add the total of the first two rows
    return x;
}

__device__ __forceinline__ double readlane_f64(double x, int l)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), l), __builtin_amdgcn_readlane(__double2loint(x), l));
}
__device__ __forceinline__ float readlane_f32(float x, int l)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}
// Among the lanes of `lanes` (a ballot, not empty) the one with the smallest idx; idx of that lane.
__device__ __forceinline__ int first_of_equals(unsigned long long lanes, int idx, int* lane_out)
{
    int l = __builtin_ctzll(lanes);
    int best = __builtin_amdgcn_readlane(idx, l);
    for (unsigned long long rest = lanes & (lanes - 1); rest; rest &= rest - 1) {    // ties only
        const int l2 = __builtin_ctzll(rest);
        const int i2 = __builtin_amdgcn_readlane(idx, l2);
        if (i2 < best) { best = i2; l = l2; }
    }
    *lane_out = l;
    return best;
}
// The segment pick of pick_segment() with total j in lanes j, j + 16, ... (t: this lane's
// total): an inclusive scan over each row of 16 lanes, a ballot for the first segment with
// weight whose running sum is past u * W, the last segment with weight if rounding leaves none.
__device__ __forceinline__ SegPick pick_segment_lanes(double t, double u)
{
    double c = t;
    c += dpp_or_zero<0x111>(c);
    c += dpp_or_zero<0x112>(c);
    c += dpp_or_zero<0x114>(c);
    c += dpp_or_zero<0x118>(c);
    SegPick pk;
    pk.W = readlane_f64(c, 15);
    pk.target = u * pk.W;
    const uint32_t hit = (uint32_t)__ballot(t > 0.0 && c > pk.target) & 0xffffu;
    const uint32_t live = (uint32_t)__ballot(t > 0.0) & 0xffffu;
    pk.js = hit ? __builtin_ctz(hit) : live ? 31 - __builtin_clz(live) : 0;
    pk.cum_js = readlane_f64(c - t, pk.js);
    return pk;
}


}  // namespace dyspec
