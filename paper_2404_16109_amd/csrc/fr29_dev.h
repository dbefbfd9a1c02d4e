// Fr arithmetic on nine 29-bit limbs, for the kernels that are bound by
// instruction issue.
//
// With 32-bit limbs every limb product needs a second instruction to catch the
// carry out of the 64-bit accumulator.  With 29-bit limbs a column of a product
// (nine limb products, nine reduction products) stays below 2^64, so a product
// is one v_mad_u64_u32 per limb product and a shift per column, written as plain
// C++.  Nine limbs hold 261 bits, six more than r has, and that slack is spent
// on laziness: sums and differences are not reduced, only kept below 2^261-ish
// bounds that are stated with each function.
//
// Montgomery factor.  f29_mul(a, b) = a b / 2^261 mod r.  Vectors stay in the
// library's usual form x * 2^256 mod r ("R256 form"); a factor that is uniform
// or comes from a table built for the purpose is supplied as y * 2^261 mod r
// ("R261 form"), so that the product is again in R256 form.
//
// The header has no device-only construct: it also compiles for the host, where
// the prover prepares uniform operands and where the arithmetic is tested
// against big integers.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define ZK_HD __host__ __device__ __forceinline__
#else
#define ZK_HD inline
#endif

namespace zkmi {

struct F29 {
    uint32_t l[9];  // value = sum l[i] 2^(29 i); "normalized": l[0..7] < 2^29
};

struct F29Wide {
    uint32_t l[18];
};

static constexpr uint32_t kM29 = (1u << 29) - 1;

// acc + x for a 64-bit accumulator and a 32-bit x.  On the device the sum is
// written as a multiply-add by a one the compiler cannot see through: a single
// v_mad_u64_u32, where the plain sum costs a move (to widen x) and a 64-bit add.
ZK_HD uint64_t f29_acc_add(uint64_t acc, uint32_t x) {
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t one = 1;
    asm("" : "+s"(one));
    return acc + (uint64_t)x * one;
#else
    return acc + x;
#endif
}

// r in 29-bit limbs.  r = 1 mod 2^29, so the Montgomery digit of a column is
// its negated low limb and the r_0 term adds exactly that digit.
#define ZK_R29_LIMBS \
    { 0x00000001u, 0x1ffffff8u, 0x1f96ffbfu, 0x1b4805ffu, 0x1d80553bu, 0x0c0404d0u, 0x1520cce7u, 0x0a6533afu, 0x0073eda7u }

// 2^261 mod r, normalized: multiplying by it leaves the value unchanged (mod r).
#define ZK_ONE261_LIMBS \
    { 0x1fffffbau, 0x0000022fu, 0x1cb61180u, 0x0a4e5c00u, 0x0ee8b1a2u, 0x16e6aedfu, 0x1907f8bbu, 0x0853ddf7u, 0x004d043fu }

// 40 r with every limb but the top one raised by 2^29 (borrowed from the limb
// above): a - b + this is a - b mod r and has no negative limb as long as b is
// normalized and b < 2^232 * (top limb of 40 r) ~ 39.99 r.
#define ZK_SUBPAD_LIMBS \
    { 0x20000028u, 0x3ffffebfu, 0x2f97f5feu, 0x2340effeu, 0x3c0d5159u, 0x20a0c0a3u, 0x2d200426u, 0x3fd01371u, 0x121d2223u }

// 4 r padded the same way, for subtrahends below 3.99 r (products are below 2 r):
// the difference then stays below a + 4 r.
#define ZK_SUBPAD4_LIMBS \
    { 0x20000004u, 0x3fffffdfu, 0x3e5bfefeu, 0x2d2017feu, 0x360154eeu, 0x30101342u, 0x3483339cu, 0x2994cebdu, 0x01cfb69cu }

// ---- layout changes --------------------------------------------------------------

// Eight 32-bit words (any value below 2^256) -> normalized limbs.
ZK_HD F29 f29_unpack(const uint32_t w[8]) {
    F29 a;
#pragma unroll
    for (int i = 0; i < 9; ++i) {
        const int bit = 29 * i, j = bit >> 5, s = bit & 31;
        uint32_t v = w[j] >> s;
        if (s > 3 && j + 1 < 8) v |= w[j + 1] << (32 - s);
        a.l[i] = v & kM29;
    }
    return a;
}

// Normalized limbs of a value below 2^256 -> eight 32-bit words.
ZK_HD void f29_pack(uint32_t w[8], const F29& a) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int bit = 32 * j, i = bit / 29, s = bit - 29 * i;  // word j starts at bit s of limb i
        uint32_t v = a.l[i] >> s;
        v |= a.l[i + 1] << (29 - s);  // 29 - s >= 8 for every j, and limb i + 2 never reaches into word j
        w[j] = v;
    }
}

// Carries pushed upward: l[0..7] < 2^29 afterwards, l[8] takes what is left.
ZK_HD F29 f29_normalize(const F29& a) {
    F29 o;
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t v = a.l[i] + c;
        o.l[i] = v & kM29;
        c = v >> 29;
    }
    o.l[8] = a.l[8] + c;
    return o;
}

// ---- lazy sums and differences ------------------------------------------------

ZK_HD F29 f29_zero() {
    F29 o;
#pragma unroll
    for (int i = 0; i < 9; ++i) o.l[i] = 0;
    return o;
}

// Limb-wise sum; the caller keeps limbs below 2^32.
ZK_HD F29 f29_add(const F29& a, const F29& b) {
    F29 o;
#pragma unroll
    for (int i = 0; i < 9; ++i) o.l[i] = a.l[i] + b.l[i];
    return o;
}

// a - b + 40 r, limb-wise.  b must be normalized and below 39.99 r; the limbs of
// the result are below (limbs of a) + 2^30 and its value below a + 40 r.
ZK_HD F29 f29_sub(const F29& a, const F29& b) {
    constexpr uint32_t pad[9] = ZK_SUBPAD_LIMBS;
    F29 o;
#pragma unroll
    for (int i = 0; i < 9; ++i) o.l[i] = a.l[i] - b.l[i] + pad[i];
    return o;
}

// a - b + 4 r, limb-wise, for a normalized b below 3.99 r.
ZK_HD F29 f29_sub_small(const F29& a, const F29& b) {
    constexpr uint32_t pad[9] = ZK_SUBPAD4_LIMBS;
    F29 o;
#pragma unroll
    for (int i = 0; i < 9; ++i) o.l[i] = a.l[i] - b.l[i] + pad[i];
    return o;
}

// ---- products ---------------------------------------------------------------------
//
// Column sums are kept in 64 bits: with limbs of a below La and limbs of b below
// Lb a column holds at most 9 La Lb + 9 * 2^58 + 2^36, which must stay below 2^64:
// e.g. La = 1.5 * 2^30 with Lb = 2^29, or La = Lb = 2^30.

template <int C>
ZK_HD void f29_column_low(uint64_t& acc, const uint32_t* a, const uint32_t* b, uint32_t* m) {
    constexpr uint32_t r[9] = ZK_R29_LIMBS;
#pragma unroll
    for (int j = 0; j <= C; ++j) acc += (uint64_t)a[j] * b[C - j];
#pragma unroll
    for (int i = 0; i < C; ++i) acc += (uint64_t)m[i] * r[C - i];
    m[C] = (0u - (uint32_t)acc) & kM29;
    acc = f29_acc_add(acc, m[C]);  // the r_0 term: clears the low 29 bits
    acc >>= 29;
}

template <int C>
ZK_HD void f29_column_high(uint64_t& acc, const uint32_t* a, const uint32_t* b, const uint32_t* m, uint32_t* t) {
    constexpr uint32_t r[9] = ZK_R29_LIMBS;
#pragma unroll
    for (int j = C - 8; j <= 8; ++j) acc += (uint64_t)a[j] * b[C - j];
#pragma unroll
    for (int i = C - 8; i <= 8; ++i) acc += (uint64_t)m[i] * r[C - i];
    t[C - 9] = (uint32_t)acc & kM29;
    acc >>= 29;
}

// a b / 2^261 mod r, normalized, value below a b / 2^261 + r (so below 2^256
// whenever a b < 2^516).
ZK_HD F29 f29_mul(const F29& a, const F29& b) {
    uint32_t m[9];
    F29 t;
    uint64_t acc = 0;
    f29_column_low<0>(acc, a.l, b.l, m);
    f29_column_low<1>(acc, a.l, b.l, m);
    f29_column_low<2>(acc, a.l, b.l, m);
    f29_column_low<3>(acc, a.l, b.l, m);
    f29_column_low<4>(acc, a.l, b.l, m);
    f29_column_low<5>(acc, a.l, b.l, m);
    f29_column_low<6>(acc, a.l, b.l, m);
    f29_column_low<7>(acc, a.l, b.l, m);
    f29_column_low<8>(acc, a.l, b.l, m);
    f29_column_high<9>(acc, a.l, b.l, m, t.l);
    f29_column_high<10>(acc, a.l, b.l, m, t.l);
    f29_column_high<11>(acc, a.l, b.l, m, t.l);
    f29_column_high<12>(acc, a.l, b.l, m, t.l);
    f29_column_high<13>(acc, a.l, b.l, m, t.l);
    f29_column_high<14>(acc, a.l, b.l, m, t.l);
    f29_column_high<15>(acc, a.l, b.l, m, t.l);
    f29_column_high<16>(acc, a.l, b.l, m, t.l);
    t.l[8] = (uint32_t)acc;
    return t;
}

// The same with the addend's limb taken into each result column before it is cut:
// a b / 2^261 + c mod r, normalized, value below a b / 2^261 + r + c.  c must be
// normalized.  (One pass of carries serves the product and the sum.)
template <int C>
ZK_HD void f29_column_high_add(uint64_t& acc, const uint32_t* a, const uint32_t* b, const uint32_t* m, const uint32_t* c,
                               uint32_t* t) {
    constexpr uint32_t r[9] = ZK_R29_LIMBS;
#pragma unroll
    for (int j = C - 8; j <= 8; ++j) acc += (uint64_t)a[j] * b[C - j];
#pragma unroll
    for (int i = C - 8; i <= 8; ++i) acc += (uint64_t)m[i] * r[C - i];
    acc = f29_acc_add(acc, c[C - 9]);
    t[C - 9] = (uint32_t)acc & kM29;
    acc >>= 29;
}

ZK_HD F29 f29_mul_add(const F29& a, const F29& b, const F29& c) {
    uint32_t m[9];
    F29 t;
    uint64_t acc = 0;
    f29_column_low<0>(acc, a.l, b.l, m);
    f29_column_low<1>(acc, a.l, b.l, m);
    f29_column_low<2>(acc, a.l, b.l, m);
    f29_column_low<3>(acc, a.l, b.l, m);
    f29_column_low<4>(acc, a.l, b.l, m);
    f29_column_low<5>(acc, a.l, b.l, m);
    f29_column_low<6>(acc, a.l, b.l, m);
    f29_column_low<7>(acc, a.l, b.l, m);
    f29_column_low<8>(acc, a.l, b.l, m);
    f29_column_high_add<9>(acc, a.l, b.l, m, c.l, t.l);
    f29_column_high_add<10>(acc, a.l, b.l, m, c.l, t.l);
    f29_column_high_add<11>(acc, a.l, b.l, m, c.l, t.l);
    f29_column_high_add<12>(acc, a.l, b.l, m, c.l, t.l);
    f29_column_high_add<13>(acc, a.l, b.l, m, c.l, t.l);
    f29_column_high_add<14>(acc, a.l, b.l, m, c.l, t.l);
    f29_column_high_add<15>(acc, a.l, b.l, m, c.l, t.l);
    f29_column_high_add<16>(acc, a.l, b.l, m, c.l, t.l);
    t.l[8] = (uint32_t)acc + c.l[8];
    return t;
}

// Three products under one reduction: (a0 b0 + a1 b1 + a2 b2) / 2^261 + c mod r,
// normalized, value below (a0 b0 + a1 b1 + a2 b2) / 2^261 + r + c.  All seven operands
// normalized (limbs below 2^29): a column then holds at most 27 + 9 products of
// 2^58 each, below 2^64.  Costs 243 + 81 multiply-adds where three separate
// products cost 486.
template <int C>
ZK_HD void f29_column3_low(uint64_t& acc, const uint32_t* a0, const uint32_t* b0, const uint32_t* a1, const uint32_t* b1,
                           const uint32_t* a2, const uint32_t* b2, uint32_t* m) {
    constexpr uint32_t r[9] = ZK_R29_LIMBS;
#pragma unroll
    for (int j = 0; j <= C; ++j) acc += (uint64_t)a0[j] * b0[C - j];
#pragma unroll
    for (int j = 0; j <= C; ++j) acc += (uint64_t)a1[j] * b1[C - j];
#pragma unroll
    for (int j = 0; j <= C; ++j) acc += (uint64_t)a2[j] * b2[C - j];
#pragma unroll
    for (int i = 0; i < C; ++i) acc += (uint64_t)m[i] * r[C - i];
    m[C] = (0u - (uint32_t)acc) & kM29;
    acc = f29_acc_add(acc, m[C]);
    acc >>= 29;
}

template <int C>
ZK_HD void f29_column3_high_add(uint64_t& acc, const uint32_t* a0, const uint32_t* b0, const uint32_t* a1, const uint32_t* b1,
                                const uint32_t* a2, const uint32_t* b2, const uint32_t* m, const uint32_t* c, uint32_t* t) {
    constexpr uint32_t r[9] = ZK_R29_LIMBS;
#pragma unroll
    for (int j = C - 8; j <= 8; ++j) acc += (uint64_t)a0[j] * b0[C - j];
#pragma unroll
    for (int j = C - 8; j <= 8; ++j) acc += (uint64_t)a1[j] * b1[C - j];
#pragma unroll
    for (int j = C - 8; j <= 8; ++j) acc += (uint64_t)a2[j] * b2[C - j];
#pragma unroll
    for (int i = C - 8; i <= 8; ++i) acc += (uint64_t)m[i] * r[C - i];
    acc = f29_acc_add(acc, c[C - 9]);
    t[C - 9] = (uint32_t)acc & kM29;
    acc >>= 29;
}

ZK_HD F29 f29_mul3_add(const F29& a0, const F29& b0, const F29& a1, const F29& b1, const F29& a2, const F29& b2, const F29& c) {
    uint32_t m[9];
    F29 t;
    uint64_t acc = 0;
    f29_column3_low<0>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m);
    f29_column3_low<1>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m);
    f29_column3_low<2>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m);
    f29_column3_low<3>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m);
    f29_column3_low<4>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m);
    f29_column3_low<5>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m);
    f29_column3_low<6>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m);
    f29_column3_low<7>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m);
    f29_column3_low<8>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m);
    f29_column3_high_add<9>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m, c.l, t.l);
    f29_column3_high_add<10>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m, c.l, t.l);
    f29_column3_high_add<11>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m, c.l, t.l);
    f29_column3_high_add<12>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m, c.l, t.l);
    f29_column3_high_add<13>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m, c.l, t.l);
    f29_column3_high_add<14>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m, c.l, t.l);
    f29_column3_high_add<15>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m, c.l, t.l);
    f29_column3_high_add<16>(acc, a0.l, b0.l, a1.l, b1.l, a2.l, b2.l, m, c.l, t.l);
    t.l[8] = (uint32_t)acc + c.l[8];
    return t;
}

// ---- sums of products, unreduced --------------------------------------------------

ZK_HD F29Wide f29_wide_zero() {
    F29Wide w;
#pragma unroll
    for (int i = 0; i < 18; ++i) w.l[i] = 0;
    return w;
}

// w += a b as integers.  The product's columns are cut into 29-bit limbs and
// added to w's limbs without carrying: eight such additions fit between two
// calls of f29_wide_normalize.
ZK_HD void f29_wide_mac(F29Wide& w, const F29& a, const F29& b) {
    uint64_t acc = 0;
#pragma unroll
    for (int c = 0; c < 17; ++c) {
        const int lo = c < 9 ? 0 : c - 8, hi = c < 9 ? c : 8;
#pragma unroll
        for (int j = lo; j <= hi; ++j) acc += (uint64_t)a.l[j] * b.l[c - j];
        w.l[c] += (uint32_t)acc & kM29;
        acc >>= 29;
    }
    w.l[17] += (uint32_t)acc;
}

ZK_HD void f29_wide_normalize(F29Wide& w) {
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < 17; ++i) {
        uint32_t v = w.l[i] + c;
        w.l[i] = v & kM29;
        c = v >> 29;
    }
    w.l[17] += c;
}

// w / 2^261 mod r for a normalized w; limbs 0..7 normalized, value below
// w / 2^261 + r (the top limb takes whatever that needs).
ZK_HD F29 f29_wide_reduce(const F29Wide& w) {
    constexpr uint32_t r[9] = ZK_R29_LIMBS;
    uint32_t m[9];
    F29 t;
    uint64_t acc = 0;
#pragma unroll
    for (int c = 0; c < 9; ++c) {
        acc = f29_acc_add(acc, w.l[c]);
#pragma unroll
        for (int i = 0; i < c; ++i) acc += (uint64_t)m[i] * r[c - i];
        m[c] = (0u - (uint32_t)acc) & kM29;
        acc = f29_acc_add(acc, m[c]);
        acc >>= 29;
    }
#pragma unroll
    for (int c = 9; c < 17; ++c) {
        acc = f29_acc_add(acc, w.l[c]);
#pragma unroll
        for (int i = c - 8; i <= 8; ++i) acc += (uint64_t)m[i] * r[c - i];
        t.l[c - 9] = (uint32_t)acc & kM29;
        acc >>= 29;
    }
    t.l[8] = (uint32_t)(acc + w.l[17]);
    return t;
}

// x times one (2^261 mod r as the second factor): the same value mod r, normalized
// and below x / 2^261 + r, i.e. a lazy value of up to 2^264 brought below 9 r.
ZK_HD F29 f29_shrink(const F29& x) {
    constexpr F29 unit = {ZK_ONE261_LIMBS};
    return f29_mul(x, unit);
}

// ---- back to the canonical representative ---------------------------------------------

// x (limbs 0..7 normalized, value below 2^256 and below 2 r) -> x mod r in eight words.
ZK_HD void f29_pack_reduced(uint32_t w[8], const F29& x) {
    constexpr uint32_t r32[8] = {0x00000001u, 0xffffffffu, 0xfffe5bfeu, 0x53bda402u,
                                 0x09a1d805u, 0x3339d808u, 0x299d7d48u, 0x73eda753u};
    uint32_t t[8], d[8];
    f29_pack(t, x);
    uint64_t borrow = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint64_t v = (uint64_t)t[k] - r32[k] - borrow;
        d[k] = (uint32_t)v;
        borrow = (v >> 32) & 1u;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = borrow ? t[k] : d[k];
}

// The fully reduced value of x in eight words.  x: limbs 0..7 normalized, value
// below 2^261 (one multiplication by the unit brings it below 2 r).
ZK_HD void f29_canonical(uint32_t w[8], const F29& x) {
    constexpr F29 unit = {ZK_ONE261_LIMBS};
    f29_pack_reduced(w, f29_mul(x, unit));
}

// The same for a sum of many lazy values: x below 2^264 (two multiplications by
// the unit: below 9 r, then below 1.2 r).
ZK_HD void f29_canonical_big(uint32_t w[8], const F29& x) {
    constexpr F29 unit = {ZK_ONE261_LIMBS};
    f29_pack_reduced(w, f29_mul(f29_mul(x, unit), unit));
}

}  // namespace zkmi
