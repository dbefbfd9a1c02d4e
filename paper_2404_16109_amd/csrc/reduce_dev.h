// Wavefront and workgroup sums of field elements.
#pragma once
#include "fr_dev.h"

namespace zkmi {

// Sum over the 64 lanes of a wavefront; lane 0 holds the result.
__device__ __forceinline__ Fr wave_sum(Fr v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        Fr o;
#pragma unroll
        for (int k = 0; k < 8; ++k) o.l[k] = __shfl_down(v.l[k], off, 64);
        v = fr_add(v, o);
    }
    return v;
}

// Sum over the first WIDTH lanes (a power of two) of a wavefront; lane 0 holds the result.
template <int WIDTH>
__device__ __forceinline__ Fr lanes_sum(Fr v) {
#pragma unroll
    for (int off = WIDTH / 2; off >= 1; off >>= 1) {
        Fr o;
#pragma unroll
        for (int k = 0; k < 8; ++k) o.l[k] = __shfl_down(v.l[k], off, 64);
        v = fr_add(v, o);
    }
    return v;
}

// Sum of NV values per thread over a workgroup of kWaves wavefronts (a power of
// two, at most 64).  `lds` needs kWaves*NV*8 words.  Thread 0 returns the totals
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
            v[q] = lanes_sum<kWaves>(o);
        }
    }
    __syncthreads();
}

}  // namespace zkmi
