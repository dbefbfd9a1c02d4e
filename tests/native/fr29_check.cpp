// Host build of the 29-bit-limb field arithmetic (csrc/fr29_dev.h) with a C
// interface, so that tests can compare it with Python's big integers.  Compiled
// with g++ by tests/test_fr29_host.py; nothing here runs on a GPU.
#include "../../paper_2404_16109_amd/csrc/round01_dev.h"
#include "../../paper_2404_16109_amd/csrc/round29_dev.h"

using namespace zkmi;

extern "C" {
void c_unpack(const uint32_t* w, uint32_t* out) { F29 a = f29_unpack(w); for (int i = 0; i < 9; ++i) out[i] = a.l[i]; }
void c_pack(const uint32_t* l, uint32_t* w) { F29 a; for (int i = 0; i < 9; ++i) a.l[i] = l[i]; f29_pack(w, a); }
void c_normalize(const uint32_t* l, uint32_t* out) { F29 a; for (int i = 0; i < 9; ++i) a.l[i] = l[i]; a = f29_normalize(a); for (int i = 0; i < 9; ++i) out[i] = a.l[i]; }
void c_sub(const uint32_t* x, const uint32_t* y, uint32_t* out) {
    F29 a, b; for (int i = 0; i < 9; ++i) { a.l[i] = x[i]; b.l[i] = y[i]; }
    F29 o = f29_sub(a, b); for (int i = 0; i < 9; ++i) out[i] = o.l[i];
}
void c_sub_small(const uint32_t* x, const uint32_t* y, uint32_t* out) {
    F29 a, b; for (int i = 0; i < 9; ++i) { a.l[i] = x[i]; b.l[i] = y[i]; }
    F29 o = f29_sub_small(a, b); for (int i = 0; i < 9; ++i) out[i] = o.l[i];
}
void c_mul(const uint32_t* x, const uint32_t* y, uint32_t* out) {
    F29 a, b; for (int i = 0; i < 9; ++i) { a.l[i] = x[i]; b.l[i] = y[i]; }
    F29 o = f29_mul(a, b); for (int i = 0; i < 9; ++i) out[i] = o.l[i];
}
void c_wide_mac(uint32_t* w, const uint32_t* x, const uint32_t* y) {
    F29Wide W; F29 a, b;
    for (int i = 0; i < 18; ++i) W.l[i] = w[i];
    for (int i = 0; i < 9; ++i) { a.l[i] = x[i]; b.l[i] = y[i]; }
    f29_wide_mac(W, a, b);
    for (int i = 0; i < 18; ++i) w[i] = W.l[i];
}
void c_wide_normalize(uint32_t* w) { F29Wide W; for (int i = 0; i < 18; ++i) W.l[i] = w[i]; f29_wide_normalize(W); for (int i = 0; i < 18; ++i) w[i] = W.l[i]; }
void c_wide_reduce(const uint32_t* w, uint32_t* out) { F29Wide W; for (int i = 0; i < 18; ++i) W.l[i] = w[i]; F29 o = f29_wide_reduce(W); for (int i = 0; i < 9; ++i) out[i] = o.l[i]; }
static F29 f29_of(const uint32_t* l) { F29 a; for (int i = 0; i < 9; ++i) a.l[i] = l[i]; return a; }
static void f29_out(uint32_t* out, const F29& a) { for (int i = 0; i < 9; ++i) out[i] = a.l[i]; }

void c_mul_add(const uint32_t* x, const uint32_t* y, const uint32_t* z, uint32_t* out) {
    f29_out(out, f29_mul_add(f29_of(x), f29_of(y), f29_of(z)));
}
void c_shrink(const uint32_t* x, uint32_t* out) { f29_out(out, f29_shrink(f29_of(x))); }
// One thread of a large folding round, as the kernel runs it: `pairs` pairs, each given by the eight entries that
// fold into it (A: y0 y1 y2 y3, then S: y0 y1 y2 y3; nine limbs each) and its weight; r: the challenge (times 2^261),
// beta.  folded: per pair the four folded entries a0 a1 s0 s1; out: the thread's three sums (q0, qinf, sA0).
// peak (may be null): the largest value a limb of the two unreduced sums held before a normalization.
void c_round29_thread(int pairs, const uint32_t* entries, const uint32_t* weights, const uint32_t* r, const uint32_t* beta,
                      uint32_t* folded, uint32_t* out, uint64_t* peak) {
    Round29Sums t;
    round29_begin(t);
    const F29 rr = f29_of(r), bb = f29_of(beta);
    uint64_t top = 0;
    for (int j = 0; j < pairs; ++j) {
        const uint32_t* e = entries + 72 * j;
        const F29 a0 = round29_fold(f29_of(e), f29_of(e + 18), rr), a1 = round29_fold(f29_of(e + 9), f29_of(e + 27), rr);
        const F29 s0 = round29_fold(f29_of(e + 36), f29_of(e + 54), rr), s1 = round29_fold(f29_of(e + 45), f29_of(e + 63), rr);
        f29_out(folded + 36 * j, a0); f29_out(folded + 36 * j + 9, a1);
        f29_out(folded + 36 * j + 18, s0); f29_out(folded + 36 * j + 27, s1);
        if (peak && (j & 3) == 3) {
            // what the lazy limbs hold just before this pair's normalization: run the pair on a copy without it
            Round29Sums probe = t;
            probe.pairs = 0;  // a count after the pair that is no multiple of four: no normalization
            round29_pair(probe, a0, a1, s0, s1, f29_of(weights + 9 * j), bb);
            for (int c = 0; c < 18; ++c) { if (probe.q0.l[c] > top) top = probe.q0.l[c]; if (probe.qinf.l[c] > top) top = probe.qinf.l[c]; }
        }
        round29_pair(t, a0, a1, s0, s1, f29_of(weights + 9 * j), bb);
    }
    F29 o[3];
    round29_end(t, o);
    for (int q = 0; q < 3; ++q) f29_out(out + 9 * q, o[q]);
    if (peak) *peak = top;
}
// One thread of the first pass when it serves two rounds, as the kernel runs it: `quads` quads, each given by its four
// entries of A then its four of S (c = 2 x_0 + x_1; nine limbs each) and its weight.  out: the thread's nine sums
// (c20, c21, qd, T, qe, then the four sums of A).  peak (may be null): the largest value a limb of the unreduced sums
// held before a normalization.
void c_round01_thread(int quads, const uint32_t* entries, const uint32_t* weights, uint32_t* out, uint64_t* peak) {
    Round01Sums t;
    round01_begin(t);
    uint64_t top = 0;
    auto look = [&](const Round01Sums& u) {
        const F29Wide* wide[5] = {&u.c20, &u.c21, &u.qd, &u.T, &u.qe};
        for (int q = 0; q < 5; ++q) for (int c = 0; c < 18; ++c) if (wide[q]->l[c] > top) top = wide[q]->l[c];
        for (int q = 0; q < 4; ++q) for (int c = 0; c < 9; ++c) if (u.sa[q].l[c] > top) top = u.sa[q].l[c];
    };
    for (int j = 0; j < quads; ++j) {
        const uint32_t* e = entries + 72 * j;
        F29 a[4], s[4];
        for (int c = 0; c < 4; ++c) { a[c] = f29_of(e + 9 * c); s[c] = f29_of(e + 36 + 9 * c); }
        if (peak && j % 7 == 6) {
            // what the lazy limbs hold just before this quad's normalization: run the quad on a copy without it
            Round01Sums probe = t;
            probe.quads = 0;
            Round01Weighted y;
            round01_quad_a(probe, a, f29_of(weights + 9 * j), y);
            round01_quad_s(probe, s, y);
            look(probe);
        }
        Round01Weighted x;
        round01_quad_a(t, a, f29_of(weights + 9 * j), x);
        round01_quad_s(t, s, x);
    }
    if (peak) {
        look(t);
        *peak = top;
    }
    F29 o[9];
    round01_end(t, o);
    for (int q = 0; q < 9; ++q) f29_out(out + 9 * q, o[q]);
}
// An entry bound by two challenges at once, as the kernel does after that pass: y: the four entries y_00 y_01 y_10
// y_11; r_first, r and their product, each times 2^261.
void c_fold2(const uint32_t* y, const uint32_t* r_first, const uint32_t* r, const uint32_t* r_both, uint32_t* out) {
    const Round29Fold2 r2{f29_of(r_first), f29_of(r), f29_of(r_both)};
    f29_out(out, round29_fold2(f29_of(y), f29_of(y + 9), f29_of(y + 18), f29_of(y + 27), r2));
}
void c_mul3_add(const uint32_t* v, uint32_t* out) {
    f29_out(out, f29_mul3_add(f29_of(v), f29_of(v + 9), f29_of(v + 18), f29_of(v + 27), f29_of(v + 36), f29_of(v + 45), f29_of(v + 54)));
}
void c_canonical(const uint32_t* l, uint32_t* w) { F29 a; for (int i = 0; i < 9; ++i) a.l[i] = l[i]; f29_canonical(w, a); }
void c_canonical_big(const uint32_t* l, uint32_t* w) { F29 a; for (int i = 0; i < 9; ++i) a.l[i] = l[i]; f29_canonical_big(w, a); }
}
