// Data side of the large rounds of the tlookup sumcheck (Section 4, the second form
// of the identity; Section 3.3 for the protocol), on 29-bit limbs: the first pass,
// which serves the first two rounds (k_round_data01, schedule in round01_dev.h), and
// the large folding rounds (k_round_data29, schedule in round29_dev.h).
//
// These kernels move data at close to the rate of a plain copy only if their
// arithmetic keeps up, so they run on fr29_dev.h's multiplier (one multiply-add per
// limb product, no carry folds, lazy sums) and compute only what cannot be had
// otherwise.  A folding round forms per pair the two folds of A and of S, the two
// weighted entries of A, and the sums q0 = sum w A0 (S0+beta), qinf = sum w (A1-A0)(S1-S0)
// and sA0 = sum A0; the round's other two sums, q1 and sA1, follow on the host from
// the running claim and from the previous round's sums of A.  The first of these
// rounds after k_round_data01 binds two variables at once (FOLD2).
//
// Arrays between such rounds hold 29-bit limbs, normalized but not reduced: every
// fold adds up to 2 r to the bound on the values (they start below r), which is
// why at most kMaxLazyRounds folds happen before a round writes fully reduced
// 32-bit words again.
#pragma once
#include "round01_dev.h"
#include "round29_dev.h"
#include "small_dev.h"
#include "tlookup_kernels.h"

namespace zkmi {

// `count` elements of nine 29-bit limbs in three planes: limbs 0..3 of element i
// as one uint4 at base[i], limbs 4..7 at base[count + i], limb 8 as a word at
// ((uint32_t*)(base + 2 count))[i] (a wavefront reads 1 KiB, 1 KiB and 256 B, each
// contiguous).  36 * count bytes.
struct Planes29 {
    uint4* base;
    size_t count;
};

__device__ __forceinline__ F29 planes29_load(const Planes29& a, size_t i) {
    const uint4 u = a.base[i], v = a.base[a.count + i];
    const uint32_t top = reinterpret_cast<const uint32_t*>(a.base + 2 * a.count)[i];
    return F29{{u.x, u.y, u.z, u.w, v.x, v.y, v.z, v.w, top}};
}

__device__ __forceinline__ void planes29_store(const Planes29& a, size_t i, const F29& x) {
    a.base[i] = make_uint4(x.l[0], x.l[1], x.l[2], x.l[3]);
    a.base[a.count + i] = make_uint4(x.l[4], x.l[5], x.l[6], x.l[7]);
    reinterpret_cast<uint32_t*>(a.base + 2 * a.count)[i] = x.l[8];
}

// One of the two arrays a round folds.  It arrives as eight planes of 32-bit
// words (fully reduced: the first of a run of such rounds) or in `planes`, and
// leaves in `planes` (in place) or as fully reduced words (the last of a run).
struct Array29 {
    const uint32_t* words_in;
    size_t ws_in;
    Planes29 planes;
    uint32_t* words_out;
    size_t ws_out;
};

struct DataRound29Args {
    Array29 A, S;
    size_t half;
    size_t block_span;
    // Which entry of a pair the sums are taken over: pair p consists of the entries p + off0 (whose folds feed q0 and
    // sA0) and p + off1; (off0, off1) = (0, half) sums the X = 0 side of the round, (half, 0) the X = 1 side.
    size_t off0, off1;
    F29 r_prev;  // the challenge times 2^261
    F29 r_first; // FOLD2: the challenge before it (the first round's), and the product of the two, times 2^261
    F29 r_both;
    F29 beta;    // times 2^256, like the vectors
    Planes29 weights;  // the pool of low weight tables, entries times 2^266 (a weighted entry then has the vectors' form)
    uint32_t lo_off;   // this round's table in it
    int lbits;
    int has_hi;        // the workgroup's pairs share one more factor, from the pool of 32-bit tables:
    const uint32_t* hi_pool;
    size_t hi_stride;
    uint32_t hi_off;
    uint32_t* partials;  // five values per workgroup: q0, (unused), qinf, sA0, (unused)
    size_t pstride;
    // INTS: S is given as small integers (small_dev.h) and folded from them
    const int32_t* sx;
    const int32_t* sy;      // may be null
    const SmallFold4* sf;   // device memory: the constants of the fold by r_prev
};

template <bool WORDS32>
__device__ __forceinline__ F29 array29_load(const Array29& a, size_t i) {
    if constexpr (WORDS32) {
        uint32_t w[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) w[k] = a.words_in[k * a.ws_in + i];
        return f29_unpack(w);
    } else {
        return planes29_load(a.planes, i);
    }
}

// x: normalized, below 2^261.
template <bool WORDS32>
__device__ __forceinline__ void array29_store(const Array29& a, size_t i, const F29& x) {
    if constexpr (WORDS32) {
        uint32_t w[8];
        f29_canonical(w, x);
#pragma unroll
        for (int k = 0; k < 8; ++k) a.words_out[k * a.ws_out + i] = w[k];
    } else {
        planes29_store(a.planes, i, x);
    }
}

// Binds the previous variable for the two entries p0 and p1 of a pair: x = y + r (y' - y)
// with y at the entry's index and y' at that plus 2*half, written back (to the
// entry's index) and returned.  FOLD2 binds the two previous variables at once
// (the first pass has served two rounds and folded nothing): the entry at i comes
// from the four at i + c Q, c = 2 x_0 + x_1, Q = 2*half (round29_fold2).
template <bool IN32, bool OUT32, bool FOLD2>
__device__ __forceinline__ void fold_pair29(const Array29& a, size_t p0, size_t p1, size_t half, const F29& r,
                                            const Round29Fold2& r2, F29& x0, F29& x1) {
    if constexpr (FOLD2) {
        const size_t Q = 2 * half;
        x0 = round29_fold2(array29_load<IN32>(a, p0), array29_load<IN32>(a, p0 + Q), array29_load<IN32>(a, p0 + 2 * Q),
                           array29_load<IN32>(a, p0 + 3 * Q), r2);
        array29_store<OUT32>(a, p0, x0);
        x1 = round29_fold2(array29_load<IN32>(a, p1), array29_load<IN32>(a, p1 + Q), array29_load<IN32>(a, p1 + 2 * Q),
                           array29_load<IN32>(a, p1 + 3 * Q), r2);
        array29_store<OUT32>(a, p1, x1);
    } else {
        x0 = round29_fold(array29_load<IN32>(a, p0), array29_load<IN32>(a, p0 + 2 * half), r);
        array29_store<OUT32>(a, p0, x0);
        x1 = round29_fold(array29_load<IN32>(a, p1), array29_load<IN32>(a, p1 + 2 * half), r);
        array29_store<OUT32>(a, p1, x1);
    }
}

// The pair of S for the first folding round when S comes as small integers:
// folded entries straight from the four integers each, reduced, then as 29-bit limbs.
template <bool OUT32>
__device__ __forceinline__ void fold_pair29_ints(const DataRound29Args& g, size_t p0, size_t p1, F29& x0, F29& x1) {
    const size_t half = g.half;
    auto entry = [&](size_t i0, size_t i1) {
        uint32_t w[8];
        small_fold_combined(w, g.sx[i0], g.sy ? g.sy[i0] : 0, g.sx[i1], g.sy ? g.sy[i1] : 0, *g.sf);
        return f29_unpack(w);
    };
    x0 = entry(p0, p0 + 2 * half);
    array29_store<OUT32>(g.S, p0, x0);
    x1 = entry(p1, p1 + 2 * half);
    array29_store<OUT32>(g.S, p1, x1);
}

// Sums of lazy values over a wavefront: limbs are added lane to lane (data-parallel
// moves, as in reduce_dev.h) and carried every second step, before they can
// outgrow their words.  v: normalized, below 8 r; the result, in every lane, is
// normalized and below 64 times that (below 2^264, which is about 565 r).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ F29 dpp_add29(const F29& v) {
    F29 o;
#pragma unroll
    for (int k = 0; k < 9; ++k)
        o.l[k] = v.l[k] + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v.l[k], CTRL, ROW_MASK, 0xf, true);
    return o;
}

__device__ __forceinline__ F29 wave_sum29(F29 v) {
    v = dpp_add29<0x111, 0xf>(v);  // row_shr:1
    v = dpp_add29<0x112, 0xf>(v);  // row_shr:2
    v = f29_normalize(v);
    v = dpp_add29<0x114, 0xf>(v);  // row_shr:4
    v = dpp_add29<0x118, 0xf>(v);  // row_shr:8
    v = f29_normalize(v);
    v = dpp_add29<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    v = dpp_add29<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
    v = f29_normalize(v);
    F29 out;
#pragma unroll
    for (int k = 0; k < 9; ++k) out.l[k] = (uint32_t)__builtin_amdgcn_readlane((int)v.l[k], 63);
    return out;
}

template <bool IN32, bool OUT32, bool INTS = false, bool FOLD2 = false>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4, 4))) k_round_data29(DataRound29Args g) {
    static_assert(!INTS || IN32, "integers are what the first folding round reads");
    static_assert(!FOLD2 || (IN32 && !INTS), "two variables at once are bound from the arrays as they came");
    __shared__ uint32_t lds[4 * 3 * 9];
    Round29Sums sums;
    round29_begin(sums);
    const size_t start = blockIdx.x * g.block_span;
    const size_t lo_mask = ((size_t)1 << g.lbits) - 1;
    const Round29Fold2 r2{g.r_first, g.r_prev, g.r_both};
    for (size_t p = start + threadIdx.x; p < start + g.block_span; p += blockDim.x) {  // at most kRound29MaxPairs times
        F29 a0, a1, s0, s1;
        fold_pair29<IN32, OUT32, FOLD2>(g.A, p + g.off0, p + g.off1, g.half, g.r_prev, r2, a0, a1);
        if constexpr (INTS) fold_pair29_ints<OUT32>(g, p + g.off0, p + g.off1, s0, s1);
        else fold_pair29<IN32, OUT32, FOLD2>(g.S, p + g.off0, p + g.off1, g.half, g.r_prev, r2, s0, s1);
        const F29 w = planes29_load(g.weights, g.lo_off + (p & lo_mask));
        round29_pair(sums, a0, a1, s0, s1, w, g.beta);
    }
    F29 tot[3];
    round29_end(sums, tot);
    // over the wavefront, then over the workgroup's wavefronts (two to four) through LDS
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        tot[q] = f29_shrink(wave_sum29(tot[q]));  // below 77 r, 166 r, 403 r, then below 2.1 r, 3.4 r, 6.7 r
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < 9; ++k) lds[(wave * 3 + q) * 9 + k] = tot[q].l[k];
        }
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        const int q = threadIdx.x;
        F29 v = f29_zero();
        for (int w = 0; w < nwaves; ++w) {
#pragma unroll
            for (int k = 0; k < 9; ++k) v.l[k] += lds[(w * 3 + q) * 9 + k];
        }
        Fr out;
        f29_canonical(out.l, f29_normalize(v));  // below 27 r < 2^261
        if (q < 2 && g.has_hi) out = fr_mul(out, fr_load(g.hi_pool, g.hi_stride, g.hi_off + (start >> g.lbits)));
        // q0, qinf, sA0 at the places the five sums of a round have in a workgroup's partial values
        const int slot = q == 0 ? 0 : q == 1 ? 2 : 3;
        fr_store(g.partials, g.pstride, (size_t)blockIdx.x * 5 + slot, out);
    } else if (threadIdx.x < 5) {
        fr_store(g.partials, g.pstride, (size_t)blockIdx.x * 5 + (threadIdx.x == 3 ? 1 : 4), fr_zero());
    }
}

// ---- the first pass, serving the first two rounds (round01_dev.h) -------------------
//
// Workgroup b covers the quads p in [b * block_span, (b + 1) * block_span) of the
// first quarter of the arrays (entries at p + c * quarter, c = 0..3), at most
// kRound01MaxQuads per thread.  Weights are the SECOND round's (its pairs are
// indexed by p), low table in 29-bit planes, the high factor applied once per
// workgroup.  Out, per workgroup: c20, c21, qd, T, qe (partD, five per workgroup)
// and the four sums of A followed by two zeros (partT, six per workgroup).
struct DataRound01Args {
    const uint32_t* A;
    size_t as;
    const uint32_t* S;
    size_t ss;
    size_t quarter;
    size_t block_span;
    Planes29 weights;
    uint32_t lo_off;
    int lbits;
    int has_hi;
    const uint32_t* hi_pool;
    size_t hi_stride;
    uint32_t hi_off;
    uint32_t* partD;
    size_t pstrideD;
    uint32_t* partT;
    size_t pstrideT;
};

__device__ __forceinline__ F29 words29_load(const uint32_t* base, size_t stride, size_t i) {
    uint32_t w[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = base[k * stride + i];
    return f29_unpack(w);
}

__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2, 2))) k_round_data01(DataRound01Args g) {
    __shared__ uint32_t lds[4 * 9 * 9];
    Round01Sums sums;
    round01_begin(sums);
    const size_t start = blockIdx.x * g.block_span;
    const size_t lo_mask = ((size_t)1 << g.lbits) - 1;
    for (size_t p = start + threadIdx.x; p < start + g.block_span; p += kBlock) {
        // A's entries first and done with before S's are loaded: with both in flight the registers do not suffice
        Round01Weighted x;
        {
            F29 a[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) a[c] = words29_load(g.A, g.as, p + c * g.quarter);
            const F29 w = planes29_load(g.weights, g.lo_off + (p & lo_mask));
            round01_quad_a(sums, a, w, x);
        }
        __builtin_amdgcn_sched_barrier(0);
        {
            F29 s[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) s[c] = words29_load(g.S, g.ss, p + c * g.quarter);
            round01_quad_s(sums, s, x);
        }
    }
    F29 tot[9];
    round01_end(sums, tot);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int q = 0; q < 9; ++q) {
        tot[q] = f29_shrink(wave_sum29(tot[q]));  // below 128 r, then below 2.9 r
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < 9; ++k) lds[(wave * 9 + q) * 9 + k] = tot[q].l[k];
        }
    }
    __syncthreads();
    if (threadIdx.x < 9) {
        const int q = threadIdx.x;
        F29 v = f29_zero();
        for (int w = 0; w < 4; ++w) {
#pragma unroll
            for (int k = 0; k < 9; ++k) v.l[k] += lds[(w * 9 + q) * 9 + k];
        }
        Fr out;
        f29_canonical(out.l, f29_normalize(v));  // below 12 r < 2^261
        if (q < 5) {
            if (g.has_hi) out = fr_mul(out, fr_load(g.hi_pool, g.hi_stride, g.hi_off + (start >> g.lbits)));
            fr_store(g.partD, g.pstrideD, (size_t)blockIdx.x * 5 + q, out);
        } else {
            fr_store(g.partT, g.pstrideT, (size_t)blockIdx.x * 6 + (q - 5), out);
        }
    } else if (threadIdx.x < 11) {
        fr_store(g.partT, g.pstrideT, (size_t)blockIdx.x * 6 + (threadIdx.x - 5), fr_zero());
    }
}

}  // namespace zkmi
