// Data side of the large folding rounds of the tlookup sumcheck (Section 4, the
// second form of the identity; Section 3.3 for the protocol), on 29-bit limbs.
//
// Same sums as round_data_block<true> (tlookup_kernels.h): with w the weight of a pair and (A0, A1),
// (S0, S1) its entries after binding the previous variable,
//   q0 = w A0 (S0+beta), q1 = w A1 (S1+beta), qinf = w (A1-A0)(S1-S0), sA0 = A0, sA1 = A1.
// These rounds are bound by instruction issue, so they run on fr29_dev.h's
// arithmetic (one multiply-add per limb product, no carry folds, lazy sums).
//
// Arrays between such rounds hold 29-bit limbs (PairArray29), normalized but not
// reduced: every fold adds up to 2 r to the bound on the values (they start
// below r), which is why at most kMaxLazyRounds rounds run back to back before
// one of them writes fully reduced 32-bit words again.
#pragma once
#include "fr29_dev.h"
#include "small_dev.h"
#include "tlookup_kernels.h"

namespace zkmi {

static const int kMaxLazyRounds = 8;  // values stay below 17 r: a thread's sum of 16 of them fits nine limbs

// An array of 29-bit-limb elements in HBM: limbs 0..3 of element i as one uint4
// at q0[i], limbs 4..7 at q1[i], limb 8 at l8[i] (a wavefront reads 1 KiB, 1 KiB
// and 256 B, each contiguous).  As a source it can instead be an ordinary vector
// of eight 32-bit word planes (words, ws).
struct PairArray29 {
    const uint32_t* words;
    size_t ws;
    const uint4* q0;
    const uint4* q1;
    const uint32_t* l8;
    uint4* dq0;  // destination: 29-bit limbs ...
    uint4* dq1;
    uint32_t* dl8;
    uint32_t* dwords;  // ... or fully reduced 32-bit word planes
    size_t dws;
};

struct DataRound29Args {
    PairArray29 A, S;
    size_t half;
    size_t block_span;
    F29 r_prev;  // the challenge times 2^261
    F29 beta;    // times 2^256, like the vectors
    EqSplit eq;  // eq.lo_off: the low table scaled by 2^10 (so times 2^266), eq.hi_off: unscaled
    uint32_t* partials;
    size_t pstride;
    // SMALL_S: S is given as small integers (small_dev.h) and folded from them
    const int32_t* sx;
    const int32_t* sy;      // may be null
    const SmallFold4* sf;   // device memory: the constants of the fold by r_prev
};

template <bool WORDS32>
__device__ __forceinline__ F29 f29_load(const PairArray29& a, size_t i) {
    if constexpr (WORDS32) {
        uint32_t w[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) w[k] = a.words[k * a.ws + i];
        return f29_unpack(w);
    } else {
        const uint4 u = a.q0[i], v = a.q1[i];
        return F29{{u.x, u.y, u.z, u.w, v.x, v.y, v.z, v.w, a.l8[i]}};
    }
}

// x: normalized, below 2^261.
template <bool WORDS32>
__device__ __forceinline__ void f29_store(const PairArray29& a, size_t i, const F29& x) {
    if constexpr (WORDS32) {
        uint32_t w[8];
        f29_canonical(w, x);
#pragma unroll
        for (int k = 0; k < 8; ++k) a.dwords[k * a.dws + i] = w[k];
    } else {
        a.dq0[i] = make_uint4(x.l[0], x.l[1], x.l[2], x.l[3]);
        a.dq1[i] = make_uint4(x.l[4], x.l[5], x.l[6], x.l[7]);
        a.dl8[i] = x.l[8];
    }
}

// Binds the previous variable for the pair of index p: x0 = y0 + r (y2 - y0),
// x1 = y1 + r (y3 - y1) with y_t at p + t*half, written back and returned
// normalized.
template <bool IN32, bool OUT32>
__device__ __forceinline__ void fold_pair29(const PairArray29& a, size_t p, size_t half, const F29& r, F29& x0, F29& x1) {
    {
        F29 y0 = f29_load<IN32>(a, p), y2 = f29_load<IN32>(a, p + 2 * half);
        x0 = f29_normalize(f29_add(f29_mul(f29_sub(y2, y0), r), y0));
    }
    f29_store<OUT32>(a, p, x0);
    {
        F29 y1 = f29_load<IN32>(a, p + half), y3 = f29_load<IN32>(a, p + 3 * half);
        x1 = f29_normalize(f29_add(f29_mul(f29_sub(y3, y1), r), y1));
    }
    f29_store<OUT32>(a, p + half, x1);
}

// The pair of S for the first folding round when S comes as small integers:
// folded entries straight from the four integers each, reduced, then as 29-bit limbs.
template <bool OUT32>
__device__ __forceinline__ void fold_pair29_small(const DataRound29Args& g, size_t p, F29& x0, F29& x1) {
    const size_t half = g.half;
    auto entry = [&](size_t i0, size_t i1) {
        uint32_t w[8];
        small_fold_combined(w, g.sx[i0], g.sy ? g.sy[i0] : 0, g.sx[i1], g.sy ? g.sy[i1] : 0, *g.sf);
        return f29_unpack(w);
    };
    x0 = entry(p, p + 2 * half);
    f29_store<OUT32>(g.S, p, x0);
    x1 = entry(p + half, p + 3 * half);
    f29_store<OUT32>(g.S, p + half, x1);
}


template <bool IN32, bool OUT32, bool SMALL_S = false>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(3, 3))) k_round_data29(DataRound29Args g) {
    static_assert(!SMALL_S || IN32, "integers are what the first folding round reads");
    __shared__ uint32_t lds[4 * 6 * 8];
    F29Wide wide0 = f29_wide_zero(), wide1 = f29_wide_zero(), wide2 = f29_wide_zero();
    F29 sA0 = f29_zero(), sA1 = f29_zero();
    const size_t start = blockIdx.x * g.block_span;
    const size_t lo_mask = ((size_t)1 << g.eq.lbits) - 1;
    int since = 0;
    for (size_t p = start + threadIdx.x; p < start + g.block_span; p += kBlock) {
        F29 a0, a1, s0, s1;
        fold_pair29<IN32, OUT32>(g.A, p, g.half, g.r_prev, a0, a1);
        if constexpr (SMALL_S) fold_pair29_small<OUT32>(g, p, s0, s1);
        else fold_pair29<IN32, OUT32>(g.S, p, g.half, g.r_prev, s0, s1);
        F29 w;
        {
            uint32_t ww[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) ww[k] = g.eq.pool[k * g.eq.stride + g.eq.lo_off + (p & lo_mask)];
            w = f29_unpack(ww);
        }
        sA0 = f29_add(sA0, a0);
        sA1 = f29_add(sA1, a1);
        const F29 wa0 = f29_mul(a0, w), wa1 = f29_mul(a1, w);  // below 2 r
        f29_wide_mac(wide0, wa0, f29_add(s0, g.beta));
        f29_wide_mac(wide1, wa1, f29_add(s1, g.beta));
        f29_wide_mac(wide2, f29_normalize(f29_sub(s1, s0)), f29_sub_small(wa1, wa0));
        if (++since == 4) {  // lazy limbs have room for eight additions
            since = 0;
            f29_wide_normalize(wide0);
            f29_wide_normalize(wide1);
            f29_wide_normalize(wide2);
            sA0 = f29_normalize(sA0);
            sA1 = f29_normalize(sA1);
        }
    }
    Fr tot[5];
    f29_wide_normalize(wide0);
    f29_wide_normalize(wide1);
    f29_wide_normalize(wide2);
    f29_canonical_big(tot[0].l, f29_wide_reduce(wide0));
    f29_canonical_big(tot[1].l, f29_wide_reduce(wide1));
    f29_canonical_big(tot[2].l, f29_wide_reduce(wide2));
    f29_canonical_big(tot[3].l, f29_normalize(sA0));
    f29_canonical_big(tot[4].l, f29_normalize(sA1));
    block_sum<5, 4>(tot, lds);
    if (threadIdx.x == 0) {
        if (g.eq.has_hi) {
            Fr hf = fr_load(g.eq.pool, g.eq.stride, g.eq.hi_off + (start >> g.eq.lbits));
            tot[0] = fr_mul(tot[0], hf);
            tot[1] = fr_mul(tot[1], hf);
            tot[2] = fr_mul(tot[2], hf);
        }
#pragma unroll
        for (int q = 0; q < 5; ++q) fr_store(g.partials, g.pstride, (size_t)blockIdx.x * 5 + q, tot[q]);
    }
}

}  // namespace zkmi
