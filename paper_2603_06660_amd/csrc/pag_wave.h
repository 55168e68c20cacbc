// Wave-wide sums of per-lane fp64 partials and extremes of 32-bit values on gfx950 (64 lanes): DPP within rows of
// 16 lanes, lane-swap instructions or scalar registers across rows.  No LDS traffic.
#pragma once

#include "pag_internal.h"

namespace pagk {

template <int CTRL>
__device__ __forceinline__ double dpp_move(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// sum over each row of 16 lanes, result in every lane of the row: DPP quad_perm [1,0,3,2],
// quad_perm [2,3,0,1], row_half_mirror, row_mirror (no LDS traffic)
__device__ __forceinline__ double row16_sum(double x) {
    x += dpp_move<0xB1>(x);
    x += dpp_move<0x4E>(x);
    x += dpp_move<0x141>(x);
    x += dpp_move<0x140>(x);
    return x;
}

// x' + y' after exchanging the upper half of x with the lower half of y (HALF32), or the odd
// 16-lane rows of x with the even rows of y: lanes of the lower half (even rows) end up with
// x[l] + x[partner], the others with y[partner] + y[l].  gfx950's lane-swap instructions do this
// without LDS traffic.
template <bool HALF32>
__device__ __forceinline__ double swap_add(double x, double y) {
    const u32 xl = (u32)__double2loint(x), xh = (u32)__double2hiint(x);
    const u32 yl = (u32)__double2loint(y), yh = (u32)__double2hiint(y);
    if constexpr (HALF32) {
        const auto lo = __builtin_amdgcn_permlane32_swap(xl, yl, false, false);
        const auto hi = __builtin_amdgcn_permlane32_swap(xh, yh, false, false);
        return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
    } else {
        const auto lo = __builtin_amdgcn_permlane16_swap(xl, yl, false, false);
        const auto hi = __builtin_amdgcn_permlane16_swap(xh, yh, false, false);
        return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
    }
}

// Sums of G per-lane partials over the wave at once: the cross-row steps fold the G values
// onto the four rows, the in-row steps are DPP.  Afterwards every lane of row r holds the
// total of value r (G = 4), r / 2 (G = 2) or 0 (G = 1).
template <int G>
__device__ __forceinline__ double fold_sum(const double* acc) {
    double k;
    if constexpr (G == 4) {
        const double k0 = swap_add<true>(acc[0], acc[2]);   // lower half: value 0, upper half: value 2
        const double k1 = swap_add<true>(acc[1], acc[3]);   //             value 1,             value 3
        k = swap_add<false>(k0, k1);
    } else if constexpr (G == 2) {
        k = swap_add<true>(acc[0], acc[1]);
        k = swap_add<false>(k, k);
    } else {
        k = swap_add<true>(acc[0], acc[0]);
        k = swap_add<false>(k, k);
    }
    return row16_sum(k);
}

// the total that fold_sum left for value g (of G), broadcast to every lane
template <int G>
__device__ __forceinline__ double fold_total(double tot, int g) {
    const int src = g * (64 / G);
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(tot), src),
                            __builtin_amdgcn_readlane(__double2loint(tot), src));
}

// Wave-wide minimum / maximum of one 32-bit value per lane: four DPP steps leave every row of 16 lanes with its
// extreme, the four rows are then combined through scalar registers.  The result is uniform.
template <bool MAX>
__device__ __forceinline__ u32 pick32(u32 a, u32 b) {
    if constexpr (MAX) return a > b ? a : b;
    else return a < b ? a : b;
}

template <int CTRL>
__device__ __forceinline__ u32 dpp_move_u32(u32 x) {
    return (u32)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, false);
}

template <bool MAX>
__device__ __forceinline__ u32 wave_extreme_u32(u32 x) {
    x = pick32<MAX>(x, dpp_move_u32<0xB1>(x));     // quad_perm [1,0,3,2]
    x = pick32<MAX>(x, dpp_move_u32<0x4E>(x));     // quad_perm [2,3,0,1]
    x = pick32<MAX>(x, dpp_move_u32<0x141>(x));    // row_half_mirror
    x = pick32<MAX>(x, dpp_move_u32<0x140>(x));    // row_mirror
    const u32 r0 = (u32)__builtin_amdgcn_readlane((int)x, 0), r1 = (u32)__builtin_amdgcn_readlane((int)x, 16);
    const u32 r2 = (u32)__builtin_amdgcn_readlane((int)x, 32), r3 = (u32)__builtin_amdgcn_readlane((int)x, 48);
    return pick32<MAX>(pick32<MAX>(r0, r1), pick32<MAX>(r2, r3));
}

// The same over lanes 0 .. 15 only: the extreme of row 0 (the other rows take no part), uniform.
template <bool MAX>
__device__ __forceinline__ u32 row0_extreme_u32(u32 x) {
    x = pick32<MAX>(x, dpp_move_u32<0xB1>(x));
    x = pick32<MAX>(x, dpp_move_u32<0x4E>(x));
    x = pick32<MAX>(x, dpp_move_u32<0x141>(x));
    x = pick32<MAX>(x, dpp_move_u32<0x140>(x));
    return (u32)__builtin_amdgcn_readlane((int)x, 0);
}

}  // namespace pagk
