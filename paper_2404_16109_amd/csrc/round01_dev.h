// What one thread of the FIRST pass of the tlookup sumcheck computes when that pass
// serves the first two rounds at once (Section 4, second form of the identity;
// Section 3.3 for the protocol), as plain functions on 29-bit limbs; the kernel
// (tlookup_round29.h) adds loads and the sums across lanes.  No device-only
// construct: the same schedule runs on the host, where it is checked against big
// integers at its bounds.
//
// Why one pass is enough for two rounds.  The first round binds x_0, the second
// x_1.  A "quad" is the four entries of an array whose indices differ in those two
// bits only: y_c at p + c Q, c = 2 x_0 + x_1, Q a quarter of the array's length.
// After the first challenge r the second round's pair is
//   (y'_0, y'_1) = (y_00 + r (y_10 - y_00), y_01 + r (y_11 - y_01)),
// so each of its sums is a polynomial of degree two in r whose coefficients are
// sums over the quads that do not depend on r.  With w the second round's weight
// of the quad, B(x, y) = sum w x y, and because A_i (S_i + beta) = 1 holds exactly
// for every entry before any folding (so B(A_c, S_c + beta) = sum w = 1):
//   q(0)  = 1 - r (1 - r) B(A_10 - A_00, S_10 - S_00)          [c20]
//   q(1)  = 1 - r (1 - r) B(A_11 - A_01, S_11 - S_01)          [c21]
//   q_inf = qd + r (T - qd - qe) + r^2 qe, with
//           qd = B(A_01 - A_00, S_01 - S_00),  T = B(A_11 - A_10, S_11 - S_10),
//           qe = B(A_11 - A_01 - A_10 + A_00, S_11 - S_01 - S_10 + S_00)
//   sA(x_1) = sum A_0x + r (sum A_1x - sum A_0x)
// and the first round's own leading coefficient is (1 - u_1) c20 + u_1 c21.  The
// pass therefore accumulates five sums of products and the four sums of A, the host
// forms both rounds' messages, and the next pass over the data binds two
// variables at once.
//
// Bounds.  Entries are fully reduced (below r, normalized); w is normalized and
// below r, in the form that makes w x come out in the form of x.
#pragma once
#include "fr29_dev.h"

namespace zkmi {

static constexpr int kRound01MaxQuads = 16;  // quads per thread (its lazy sums are normalized after every seven)

struct Round01Sums {
    F29Wide c20, c21, qd, T, qe;  // unreduced 18-limb integers, limbs lazy (at most seven additions between normalizations)
    F29 sa[4];                    // sums of A_00, A_01, A_10, A_11: lazy limbs, likewise
    int quads;
};

ZK_HD void round01_begin(Round01Sums& t) {
    t.c20 = f29_wide_zero();
    t.c21 = f29_wide_zero();
    t.qd = f29_wide_zero();
    t.T = f29_wide_zero();
    t.qe = f29_wide_zero();
    for (int c = 0; c < 4; ++c) t.sa[c] = f29_zero();
    t.quads = 0;
}

// On the device, keeps the compiler from starting the next product's operands
// before this product is done (all five at once do not fit the registers).
ZK_HD void round01_one_at_a_time() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_sched_barrier(0);
#endif
}

// A quad is taken in two steps, so that a kernel can load A's entries, be done with
// them, and only then load S's: the weighted differences of A's entries are what
// passes from one step to the other.
struct Round01Weighted {
    F29 wx0, wx1;  // w (A_10 - A_00), w (A_11 - A_01): normalized, below 1.6 r
    F29 wd0, wd1;  // w (A_01 - A_00), w (A_11 - A_10): normalized, below 1.6 r and 7.2 r
    F29 we;        // w (A_11 - A_01 - A_10 + A_00): below 5.6 r, limbs below 1.5 * 2^30
};

// a[c]: the quad's entries of A, c = 2 x_0 + x_1.  At most kRound01MaxQuads quads per thread.
ZK_HD void round01_quad_a(Round01Sums& t, const F29 (&a)[4], const F29& w, Round01Weighted& x) {
#pragma unroll
    for (int c = 0; c < 4; ++c) t.sa[c] = f29_add(t.sa[c], a[c]);
    // three products, the others are sums of those.  A difference is below 41 r with limbs below 1.5 * 2^30; its
    // product with w is normalized and below 41 r r / 2^261 + r < 1.6 r (r / 2^261 is about 1 / 70.7).
    x.wx0 = f29_mul(f29_sub(a[2], a[0]), w);
    round01_one_at_a_time();
    x.wx1 = f29_mul(f29_sub(a[3], a[1]), w);
    round01_one_at_a_time();
    x.wd0 = f29_mul(f29_sub(a[1], a[0]), w);
    round01_one_at_a_time();
    x.we = f29_sub_small(x.wx1, x.wx0);
    x.wd1 = f29_normalize(f29_add(x.wd0, x.we));
}

// s[c]: the quad's entries of S.
ZK_HD void round01_quad_s(Round01Sums& t, const F29 (&s)[4], const Round01Weighted& x) {
    // one factor of a product must be normalized, the other may have limbs up to 1.5 * 2^30: the weighted differences
    // of A are normalized (all but the mixed one), so the plain differences of S (below 41 r) can stay as they are
    f29_wide_mac(t.c20, x.wx0, f29_sub(s[2], s[0]));
    round01_one_at_a_time();
    f29_wide_mac(t.c21, x.wx1, f29_sub(s[3], s[1]));
    round01_one_at_a_time();
    f29_wide_mac(t.qd, x.wd0, f29_sub(s[1], s[0]));
    round01_one_at_a_time();
    f29_wide_mac(t.T, x.wd1, f29_sub(s[3], s[2]));
    round01_one_at_a_time();
    // the mixed difference of S (below 42 r) is normalized, the mixed weighted difference of A is not
    f29_wide_mac(t.qe, f29_normalize(f29_sub(f29_add(s[3], s[0]), f29_normalize(f29_add(s[1], s[2])))), x.we);
    ++t.quads;
    if (t.quads % 7 == 0) {  // a normalized limb (below 2^29) has room for seven additions of as much
        f29_wide_normalize(t.c20);
        f29_wide_normalize(t.c21);
        f29_wide_normalize(t.qd);
        f29_wide_normalize(t.T);
        f29_wide_normalize(t.qe);
#pragma unroll
        for (int c = 0; c < 4; ++c) t.sa[c] = f29_normalize(t.sa[c]);
    }
}

// The thread's nine sums, each normalized and below 2 r (so that a sum over a
// wavefront stays below 2^264, about 565 r): out[0..4] = c20, c21, qd, T, qe (divided by
// 2^261 like any product), out[5..8] = the four sums of A.
// at most 16 * 42 r * 7.2 r / 2^261 + r < 70 r once reduced, below 2 r after the shrink
ZK_HD F29 round01_finish(F29Wide& w) {
    f29_wide_normalize(w);
    return f29_shrink(f29_wide_reduce(w));
}

ZK_HD void round01_end(Round01Sums& t, F29 (&out)[9]) {
    out[0] = round01_finish(t.c20);
    out[1] = round01_finish(t.c21);
    out[2] = round01_finish(t.qd);
    out[3] = round01_finish(t.T);
    out[4] = round01_finish(t.qe);
    out[5] = f29_shrink(f29_normalize(t.sa[0]));  // below 16 r before, 1.3 r after
    out[6] = f29_shrink(f29_normalize(t.sa[1]));
    out[7] = f29_shrink(f29_normalize(t.sa[2]));
    out[8] = f29_shrink(f29_normalize(t.sa[3]));
}

}  // namespace zkmi
