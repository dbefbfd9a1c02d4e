// Host-side Fr arithmetic for the library's glue code: Fiat-Shamir challenges,
// assembling round polynomials from the sums the kernels return, and the
// verifiers' O(log D) checks.  Montgomery form in four 64-bit limbs, the same
// representation (x * 2^256 mod r) the device uses, so values move between host
// and device kernels as raw limbs.
#pragma once
#include <stdint.h>
#include <string.h>

#include "../../include/zkmi.h"

namespace zkmi {
namespace host {

typedef unsigned __int128 u128;

struct F {
    uint64_t w[4];  // Montgomery form, < r
};

static const uint64_t kMod[4] = {0xffffffff00000001ULL, 0x53bda402fffe5bfeULL, 0x3339d80809a1d805ULL,
                                 0x73eda753299d7d48ULL};
static const uint64_t kOne[4] = {0x00000001fffffffeULL, 0x5884b7fa00034802ULL, 0x998c4fefecbc4ff5ULL,
                                 0x1824b159acc5056fULL};  // 2^256 mod r
static const uint64_t kRR[4] = {0xc999e990f3f29c6dULL, 0x2b6cedcb87925c23ULL, 0x05d314967254398fULL,
                                0x0748d9d99f59ff11ULL};   // 2^512 mod r
static const uint64_t kNegInv64 = 0xfffffffeffffffffULL;  // -r^-1 mod 2^64

inline bool geq_mod(const uint64_t a[4]) {
    for (int i = 3; i >= 0; --i) {
        if (a[i] > kMod[i]) return true;
        if (a[i] < kMod[i]) return false;
    }
    return true;
}

inline void sub_mod_inplace(uint64_t a[4]) {
    uint64_t borrow = 0;
    for (int i = 0; i < 4; ++i) {
        u128 d = (u128)a[i] - kMod[i] - borrow;
        a[i] = (uint64_t)d;
        borrow = (uint64_t)(d >> 64) & 1;
    }
}

inline F zero() { return F{{0, 0, 0, 0}}; }
inline F one() { return F{{kOne[0], kOne[1], kOne[2], kOne[3]}}; }
inline bool is_zero(const F& a) { return (a.w[0] | a.w[1] | a.w[2] | a.w[3]) == 0; }
inline bool equal(const F& a, const F& b) { return memcmp(a.w, b.w, sizeof a.w) == 0; }

inline F add(const F& a, const F& b) {
    F s;
    uint64_t carry = 0;
    for (int i = 0; i < 4; ++i) {
        u128 t = (u128)a.w[i] + b.w[i] + carry;
        s.w[i] = (uint64_t)t;
        carry = (uint64_t)(t >> 64);
    }
    if (geq_mod(s.w)) sub_mod_inplace(s.w);
    return s;
}

inline F sub(const F& a, const F& b) {
    F d;
    uint64_t borrow = 0;
    for (int i = 0; i < 4; ++i) {
        u128 t = (u128)a.w[i] - b.w[i] - borrow;
        d.w[i] = (uint64_t)t;
        borrow = (uint64_t)(t >> 64) & 1;
    }
    if (borrow) {
        uint64_t carry = 0;
        for (int i = 0; i < 4; ++i) {
            u128 t = (u128)d.w[i] + kMod[i] + carry;
            d.w[i] = (uint64_t)t;
            carry = (uint64_t)(t >> 64);
        }
    }
    return d;
}

inline F neg(const F& a) { return sub(zero(), a); }

// Montgomery product for raw 256-bit inputs with a*b < 2^256 * r.
inline F mul_raw(const uint64_t a[4], const uint64_t b[4]) {
    uint64_t t[6] = {0, 0, 0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) {
        uint64_t carry = 0;
        for (int j = 0; j < 4; ++j) {
            u128 p = (u128)a[j] * b[i] + t[j] + carry;
            t[j] = (uint64_t)p;
            carry = (uint64_t)(p >> 64);
        }
        u128 s = (u128)t[4] + carry;
        t[4] = (uint64_t)s;
        t[5] = (uint64_t)(s >> 64);
        uint64_t m = t[0] * kNegInv64;
        u128 p = (u128)m * kMod[0] + t[0];
        carry = (uint64_t)(p >> 64);
        for (int j = 1; j < 4; ++j) {
            p = (u128)m * kMod[j] + t[j] + carry;
            t[j - 1] = (uint64_t)p;
            carry = (uint64_t)(p >> 64);
        }
        s = (u128)t[4] + carry;
        t[3] = (uint64_t)s;
        t[4] = t[5] + (uint64_t)(s >> 64);
    }
    F o = {{t[0], t[1], t[2], t[3]}};
    if (t[4] || geq_mod(o.w)) sub_mod_inplace(o.w);
    return o;
}

inline F mul(const F& a, const F& b) { return mul_raw(a.w, b.w); }
inline F sqr(const F& a) { return mul_raw(a.w, a.w); }

inline F from_u64(uint64_t x) {
    uint64_t c[4] = {x, 0, 0, 0};
    return mul_raw(c, kRR);
}

inline F pow(const F& a, const uint64_t e[4]) {
    F acc = one();
    for (int bit = 255; bit >= 0; --bit) {
        acc = sqr(acc);
        if ((e[bit / 64] >> (bit % 64)) & 1) acc = mul(acc, a);
    }
    return acc;
}

inline F inv(const F& a) {  // a != 0
    uint64_t e[4] = {kMod[0] - 2, kMod[1], kMod[2], kMod[3]};
    return pow(a, e);
}

// canonical fr_t <-> Montgomery F
inline F from_canonical(const fr_t& c) {
    uint64_t w[4];
    for (int i = 0; i < 4; ++i) w[i] = (uint64_t)c.l[2 * i] | ((uint64_t)c.l[2 * i + 1] << 32);
    return mul_raw(w, kRR);
}

inline fr_t to_canonical(const F& a) {
    uint64_t unit[4] = {1, 0, 0, 0};
    F c = mul_raw(a.w, unit);
    fr_t o;
    for (int i = 0; i < 4; ++i) {
        o.l[2 * i] = (uint32_t)c.w[i];
        o.l[2 * i + 1] = (uint32_t)(c.w[i] >> 32);
    }
    return o;
}

inline bool canonical_in_range(const fr_t& c) {
    uint64_t w[4];
    for (int i = 0; i < 4; ++i) w[i] = (uint64_t)c.l[2 * i] | ((uint64_t)c.l[2 * i + 1] << 32);
    return !geq_mod(w);
}

inline void to_bytes(uint8_t out[32], const F& a) {
    fr_t c = to_canonical(a);
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j) out[4 * i + j] = (uint8_t)(c.l[i] >> (8 * j));
}

// 32 little-endian bytes -> F; false if the integer is not < r.
inline bool from_bytes(F* out, const uint8_t in[32]) {
    fr_t c;
    for (int i = 0; i < 8; ++i)
        c.l[i] = (uint32_t)in[4 * i] | ((uint32_t)in[4 * i + 1] << 8) | ((uint32_t)in[4 * i + 2] << 16) |
                 ((uint32_t)in[4 * i + 3] << 24);
    if (!canonical_in_range(c)) return false;
    *out = from_canonical(c);
    return true;
}

// 64 bytes as a 512-bit big-endian integer, reduced mod r: with the integer
// split as hi * 2^256 + lo, its Montgomery form is lo*R + (hi*R)*R.
inline F from_be512(const uint8_t in[64]) {
    uint64_t hi[4], lo[4];
    for (int i = 0; i < 4; ++i) {
        uint64_t h = 0, l = 0;
        for (int j = 0; j < 8; ++j) {
            h = (h << 8) | in[(3 - i) * 8 + j];
            l = (l << 8) | in[32 + (3 - i) * 8 + j];
        }
        hi[i] = h;
        lo[i] = l;
    }
    F lo_m = mul_raw(lo, kRR);
    F hi_m = mul_raw(hi, kRR);
    F rr = {{kRR[0], kRR[1], kRR[2], kRR[3]}};
    return add(lo_m, mul(hi_m, rr));
}

// Montgomery limbs as the device reads them (eight 32-bit words).
inline void to_device_limbs(uint32_t out[8], const F& a) {
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = (uint32_t)a.w[i];
        out[2 * i + 1] = (uint32_t)(a.w[i] >> 32);
    }
}

inline F from_device_limbs(const uint32_t in[8]) {
    F a;
    for (int i = 0; i < 4; ++i) a.w[i] = (uint64_t)in[2 * i] | ((uint64_t)in[2 * i + 1] << 32);
    return a;
}

// e~(u, v) = prod_t (u_t v_t + (1-u_t)(1-v_t))
inline F eq_point(const F* u, const F* v, int n) {
    F acc = one();
    for (int t = 0; t < n; ++t) {
        F uv = mul(u[t], v[t]);
        // uv + (1-u)(1-v) = 1 - u - v + 2uv
        F term = add(sub(sub(one(), u[t]), v[t]), add(uv, uv));
        acc = mul(acc, term);
    }
    return acc;
}

// Value at x of the polynomial of degree <= npts-1 through (j, y_j), j = 0..npts-1
// (npts = 3 or 4), by Newton forward differences:
// p(x) = d0 + d1 x + d2 x(x-1)/2 + d3 x(x-1)(x-2)/6.
inline F interpolate_at(const F* y, int npts, const F& x) {
    static const F inv2 = inv(from_u64(2));
    static const F inv6 = inv(from_u64(6));
    F d[4];
    for (int j = 0; j < npts; ++j) d[j] = y[j];
    for (int level = 1; level < npts; ++level)
        for (int j = npts - 1; j >= level; --j) d[j] = sub(d[j], d[j - 1]);
    F acc = d[0];
    if (npts > 1) acc = add(acc, mul(d[1], x));
    F xx1 = mul(x, sub(x, one()));
    if (npts > 2) acc = add(acc, mul(d[2], mul(xx1, inv2)));
    if (npts > 3) acc = add(acc, mul(d[3], mul(mul(xx1, sub(x, from_u64(2))), inv6)));
    return acc;
}

}  // namespace host
}  // namespace zkmi
