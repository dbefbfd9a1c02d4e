// What one thread of the large folding rounds of the tlookup sumcheck computes
// (Section 4, second form of the identity; Section 3.3 for the protocol), as plain
// functions on 29-bit limbs: the kernel (tlookup_round29.h) adds the loads, the
// stores and the sums across lanes.  No device-only construct: the same schedule
// runs on the host, where it is checked against big integers at its bounds.
//
// Per pair, with (y0, y1, y2, y3) the four entries of an array that the previous
// challenge r folds into the pair (x0, x1) = (y0 + r (y2 - y0), y1 + r (y3 - y1)),
// w the pair's weight, (a0, a1) the pair of A and (s0, s1) that of S:
//   q0   += (w a0) (s0 + beta)
//   qinf += (w a1 - w a0) (s1 - s0)
//   sA0  += a0
// The other two sums of the round are not computed: the values at X = 1 follow
// from identities the prover's own earlier messages fix (sA0 + sA1 is the
// previous round's sum of A at its challenge; g(0) + g(1) is the running claim),
// which the host applies.
//
// Bounds.  Entries are normalized and below 17 r (they start below r, every fold
// adds less than 2 r, and after kMaxLazyRounds rounds they are written out fully
// reduced).  w, beta and the challenge are normalized and below r.
#pragma once
#include "fr29_dev.h"

namespace zkmi {

static constexpr int kMaxLazyRounds = 8;       // values stay below 17 r
static constexpr int kRound29MaxPairs = 22;    // pairs per thread: the sum of 22 entries (374 r) stays below 2^264 (565 r)

struct Round29Sums {
    F29Wide q0, qinf;  // sums of products as unreduced 18-limb integers, limbs lazy between normalizations
    F29 sA0;
    int pairs;
};

ZK_HD void round29_begin(Round29Sums& t) {
    t.q0 = f29_wide_zero();
    t.qinf = f29_wide_zero();
    t.sA0 = f29_zero();
    t.pairs = 0;
}

// y0 + r (y2 - y0), normalized, below y0 + 1.8 r.  r: the challenge times 2^261.
ZK_HD F29 round29_fold(const F29& y0, const F29& y2, const F29& r) { return f29_mul_add(f29_sub(y2, y0), r, y0); }

// Two variables bound at once, for entries that nothing has folded yet (fully
// reduced): with y_c the four entries of a quad, c = 2 x_0 + x_1,
//   y_00 + r0 (y_10 - y_00) + r1 (y_01 - y_00) + r0 r1 (y_11 - y_01 - y_10 + y_00),
// which is what binding x_0 with r0 and then x_1 with r1 gives; the three products
// share one reduction.  r0, r1, r01 = r0 r1: times 2^261, normalized, below r.
// Normalized, below y_00 + 124 r r / 2^261 + r < y_00 + 2.8 r, so below 3.8 r: within
// what two single folds may reach (5 r).
struct Round29Fold2 {
    F29 r0, r1, r01;
};

ZK_HD F29 round29_fold2(const F29& y00, const F29& y01, const F29& y10, const F29& y11, const Round29Fold2& r) {
    const F29 dx = f29_normalize(f29_sub(y10, y00));                                           // below 41 r
    const F29 dy = f29_normalize(f29_sub(y01, y00));
    const F29 dxy = f29_normalize(f29_sub(f29_add(y11, y00), f29_normalize(f29_add(y01, y10))));  // below 42 r
    return f29_mul3_add(dx, r.r0, dy, r.r1, dxy, r.r01, y00);
}

// w: the weight in the form that makes w a0 come out in the vectors' form.
ZK_HD void round29_pair(Round29Sums& t, const F29& a0, const F29& a1, const F29& s0, const F29& s1, const F29& w,
                        const F29& beta) {
    t.sA0 = f29_add(t.sA0, a0);
    const F29 wa0 = f29_mul(a0, w), wa1 = f29_mul(a1, w);  // normalized, below 2 r
    f29_wide_mac(t.q0, wa0, f29_add(s0, beta));                                      // limbs below 2^29 and 2^30
    f29_wide_mac(t.qinf, f29_normalize(f29_sub(s1, s0)), f29_sub_small(wa1, wa0));  // below 2^29 and 2^29 + 2^30
    ++t.pairs;
    if ((t.pairs & 3) == 0) {  // lazy limbs have room for eight additions
        f29_wide_normalize(t.q0);
        f29_wide_normalize(t.qinf);
        t.sA0 = f29_normalize(t.sA0);
    }
}

// The thread's three sums, each normalized and below 6.3 r (so that the sum over a
// wavefront, at most 403 r, stays below 2^264, about 565 r): out[0] = q0, out[1] = qinf, out[2] = sA0, the
// first two divided by 2^261 like any product.
ZK_HD void round29_end(Round29Sums& t, F29 (&out)[3]) {
    f29_wide_normalize(t.q0);
    f29_wide_normalize(t.qinf);
    const F29 q0 = f29_wide_reduce(t.q0), qinf = f29_wide_reduce(t.qinf);
    // with r / 2^261 about 1 / 70.7 and at most kRound29MaxPairs pairs:
    out[0] = f29_shrink(q0);    // below 22 * 2 r * 18 r / 2^261 + r < 13 r, then below 1.2 r
    out[1] = f29_shrink(qinf);  // below 22 * 57 r * 6 r / 2^261 + r < 108 r (top limb below 2^30), then below 2.6 r
    out[2] = f29_shrink(f29_normalize(t.sA0));     // below 22 * 17 r = 374 r < 2^264, then below 6.3 r
}

}  // namespace zkmi
