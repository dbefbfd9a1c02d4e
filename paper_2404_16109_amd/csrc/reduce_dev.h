// Wavefront and workgroup sums of field elements.
#pragma once
#include "fr_dev.h"

namespace zkmi {

// One step of a wavefront reduction through the data-parallel primitives: every
// limb of v is fetched from the lane the control word names (zero where there is
// none) and added as a field element.  These moves run at VALU rate, unlike the
// lane permutations that go through the LDS crossbar.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ Fr dpp_add_step(const Fr& v) {
    Fr o;
#pragma unroll
    for (int k = 0; k < 8; ++k)
        o.l[k] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v.l[k], CTRL, ROW_MASK, 0xf, true);
    return fr_add(v, o);
}

// Sum over the first WIDTH lanes (16, 32 or 64) of a wavefront, returned in every
// lane.  Shifts by 1, 2, 4, 8 within each row of 16 lanes leave a row's sum in its
// last lane; the two broadcasts carry the sums of rows 0 and 2 into rows 1 and 3
// and then that of the lower half into the upper.
template <int WIDTH>
__device__ __forceinline__ Fr lanes_sum(Fr v) {
    static_assert(WIDTH == 16 || WIDTH == 32 || WIDTH == 64, "whole rows only");
    v = dpp_add_step<0x111, 0xf>(v);  // row_shr:1
    v = dpp_add_step<0x112, 0xf>(v);  // row_shr:2
    v = dpp_add_step<0x114, 0xf>(v);  // row_shr:4
    v = dpp_add_step<0x118, 0xf>(v);  // row_shr:8
    if constexpr (WIDTH >= 32) v = dpp_add_step<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    if constexpr (WIDTH >= 64) v = dpp_add_step<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
    Fr out;
#pragma unroll
    for (int k = 0; k < 8; ++k) out.l[k] = (uint32_t)__builtin_amdgcn_readlane((int)v.l[k], WIDTH - 1);
    return out;
}

// Sum over the 64 lanes of a wavefront, in every lane.
__device__ __forceinline__ Fr wave_sum(const Fr& v) { return lanes_sum<64>(v); }

// Sum of NV values per thread over a workgroup of kWaves wavefronts (at most 64).  `lds` needs kWaves*NV*8 words.  Thread 0 returns the totals
// in v[].  The wavefronts' sums are added up by the lanes of the first
// wavefront, not one after the other.
template <int NV, int kWaves>
__device__ __forceinline__ void block_sum(Fr (&v)[NV], uint32_t* lds) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        v[q] = wave_sum(v[q]);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < 8; ++k) lds[(wave * NV + q) * 8 + k] = v[q].l[k];
        }
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            Fr o = fr_zero();
            if (lane < kWaves) {
#pragma unroll
                for (int k = 0; k < 8; ++k) o.l[k] = lds[(lane * NV + q) * 8 + k];
            }
            v[q] = lanes_sum<(kWaves <= 16 ? 16 : kWaves <= 32 ? 32 : 64)>(o);
        }
    }
    __syncthreads();
}

}  // namespace zkmi
