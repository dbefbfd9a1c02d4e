// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// Plain big-integer arithmetic in the BLS12-381 scalar field Fr (the field the
// paper's implementation works in, Section 7.2 / Section 8).  Values are kept
// as canonical integers in [0, r): four 64-bit words, least significant first.
// There is no Montgomery form here on purpose: the device library works in
// Montgomery form, so every conversion it does is checked by this code too.
//
//   r = z^4 - z^2 + 1 with the BLS12-381 parameter z = -0xd201000000010000
//
// Multiplication is the schoolbook 4x4-word product followed by Barrett
// reduction as in the Handbook of Applied Cryptography, Algorithm 14.42, with
// b = 2^64 and k = 4; mu = floor(b^(2k) / r) is computed at start-up by
// bit-serial long division, not typed in.  Inversion is Fermat: a^(r-2).
//
// This file shares nothing with the HIP library and must never be included
// from it.
#pragma once
#include <cstdint>
#include <cstring>

namespace oracle {

typedef unsigned __int128 u128;

struct Fr {
    uint64_t w[4];
};

static const uint64_t MODULUS[4] = {0xffffffff00000001ULL, 0x53bda402fffe5bfeULL,
                                    0x3339d80809a1d805ULL, 0x73eda753299d7d48ULL};

// ---- little-endian multi-word helpers -------------------------------------

inline int cmp_words(const uint64_t* a, const uint64_t* b, int n) {
    for (int i = n - 1; i >= 0; --i) {
        if (a[i] < b[i]) return -1;
        if (a[i] > b[i]) return 1;
    }
    return 0;
}

inline uint64_t add_words(uint64_t* out, const uint64_t* a, const uint64_t* b, int n) {
    uint64_t carry = 0;
    for (int i = 0; i < n; ++i) {
        u128 s = (u128)a[i] + b[i] + carry;
        out[i] = (uint64_t)s;
        carry = (uint64_t)(s >> 64);
    }
    return carry;
}

inline uint64_t sub_words(uint64_t* out, const uint64_t* a, const uint64_t* b, int n) {
    uint64_t borrow = 0;
    for (int i = 0; i < n; ++i) {
        u128 d = (u128)a[i] - b[i] - borrow;
        out[i] = (uint64_t)d;
        borrow = (uint64_t)(d >> 64) & 1;
    }
    return borrow;
}

// out[0 .. na+nb) = a * b
inline void mul_words(uint64_t* out, const uint64_t* a, int na, const uint64_t* b, int nb) {
    for (int i = 0; i < na + nb; ++i) out[i] = 0;
    for (int i = 0; i < na; ++i) {
        uint64_t carry = 0;
        for (int j = 0; j < nb; ++j) {
            u128 t = (u128)a[i] * b[j] + out[i + j] + carry;
            out[i + j] = (uint64_t)t;
            carry = (uint64_t)(t >> 64);
        }
        out[i + nb] = carry;
    }
}

// ---- Barrett constant ------------------------------------------------------

struct BarrettMu {
    uint64_t mu[5];  // floor(2^512 / r), 258 bits
    BarrettMu() {
        // Long division of 2^512 by r, one bit at a time.
        uint64_t rem[5] = {0, 0, 0, 0, 0};
        for (int i = 0; i < 5; ++i) mu[i] = 0;
        uint64_t m5[5] = {MODULUS[0], MODULUS[1], MODULUS[2], MODULUS[3], 0};
        for (int bit = 512; bit >= 0; --bit) {
            // rem = 2*rem + (bit == 512)
            for (int i = 4; i > 0; --i) rem[i] = (rem[i] << 1) | (rem[i - 1] >> 63);
            rem[0] = (rem[0] << 1) | (bit == 512 ? 1u : 0u);
            if (cmp_words(rem, m5, 5) >= 0) {
                sub_words(rem, rem, m5, 5);
                mu[bit / 64] |= (uint64_t)1 << (bit % 64);  // bit < 320 whenever this fires
            }
        }
    }
};

inline const BarrettMu& barrett_mu() {
    static const BarrettMu k;
    return k;
}

// ---- field operations ------------------------------------------------------

inline Fr fr_zero() { return Fr{{0, 0, 0, 0}}; }
inline Fr fr_one() { return Fr{{1, 0, 0, 0}}; }

inline bool fr_is_zero(const Fr& a) { return (a.w[0] | a.w[1] | a.w[2] | a.w[3]) == 0; }
inline bool fr_eq(const Fr& a, const Fr& b) { return cmp_words(a.w, b.w, 4) == 0; }
inline bool fr_is_canonical(const Fr& a) { return cmp_words(a.w, MODULUS, 4) < 0; }

// x is any 512-bit integer; result is x mod r.
inline Fr reduce512(const uint64_t x[8]) {
    const uint64_t* mu = barrett_mu().mu;
    uint64_t q2[10];
    mul_words(q2, x + 3, 5, mu, 5);          // q1 = floor(x / b^3); q2 = q1 * mu
    const uint64_t* q3 = q2 + 5;             // q3 = floor(q2 / b^5)
    uint64_t t[9];
    mul_words(t, q3, 5, MODULUS, 4);         // q3 * r, low 5 words are r2
    uint64_t rr[5];
    sub_words(rr, x, t, 5);                  // r1 - r2 mod b^5 (a borrow is the "+ b^(k+1)" step)
    uint64_t m5[5] = {MODULUS[0], MODULUS[1], MODULUS[2], MODULUS[3], 0};
    while (cmp_words(rr, m5, 5) >= 0) sub_words(rr, rr, m5, 5);
    return Fr{{rr[0], rr[1], rr[2], rr[3]}};
}

inline Fr fr_add(const Fr& a, const Fr& b) {
    Fr s;
    add_words(s.w, a.w, b.w, 4);  // a, b < 2^255, no carry out
    if (cmp_words(s.w, MODULUS, 4) >= 0) sub_words(s.w, s.w, MODULUS, 4);
    return s;
}

inline Fr fr_sub(const Fr& a, const Fr& b) {
    Fr d;
    if (cmp_words(a.w, b.w, 4) >= 0) {
        sub_words(d.w, a.w, b.w, 4);
    } else {
        Fr t;
        sub_words(t.w, MODULUS, b.w, 4);
        add_words(d.w, a.w, t.w, 4);
    }
    return d;
}

inline Fr fr_neg(const Fr& a) { return fr_sub(fr_zero(), a); }

inline Fr fr_mul(const Fr& a, const Fr& b) {
    uint64_t p[8];
    mul_words(p, a.w, 4, b.w, 4);
    return reduce512(p);
}

// a^e for a 256-bit exponent, square-and-multiply from the top bit.
inline Fr fr_pow(const Fr& a, const uint64_t e[4]) {
    Fr acc = fr_one();
    for (int bit = 255; bit >= 0; --bit) {
        acc = fr_mul(acc, acc);
        if ((e[bit / 64] >> (bit % 64)) & 1) acc = fr_mul(acc, a);
    }
    return acc;
}

// a^(r-2); the caller makes sure a != 0.
inline Fr fr_inv(const Fr& a) {
    uint64_t e[4] = {MODULUS[0] - 2, MODULUS[1], MODULUS[2], MODULUS[3]};
    return fr_pow(a, e);
}

inline Fr fr_from_u64(uint64_t x) { return Fr{{x, 0, 0, 0}}; }

// Signed embedding (Section 3.3, "discretized into a finite field"): x >= 0 is
// x itself, x < 0 is r - |x|.
inline Fr fr_from_i64(int64_t x) {
    if (x >= 0) return fr_from_u64((uint64_t)x);
    uint64_t mag = (uint64_t)0 - (uint64_t)x;
    return fr_neg(fr_from_u64(mag));
}

// 32 bytes, little-endian, of the canonical integer.
inline void fr_to_bytes(uint8_t out[32], const Fr& a) {
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 8; ++j) out[8 * i + j] = (uint8_t)(a.w[i] >> (8 * j));
}

inline Fr fr_from_bytes(const uint8_t in[32]) {
    Fr a = fr_zero();
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 8; ++j) a.w[i] |= (uint64_t)in[8 * i + j] << (8 * j);
    return a;
}

// 64 bytes read as one big-endian 512-bit integer, reduced mod r.
inline Fr fr_from_be512(const uint8_t in[64]) {
    uint64_t x[8];
    for (int i = 0; i < 8; ++i) {
        uint64_t v = 0;
        for (int j = 0; j < 8; ++j) v = (v << 8) | in[(7 - i) * 8 + j];
        x[i] = v;
    }
    return reduce512(x);
}

inline Fr fr_two_inv_pow(unsigned h) {  // 2^(-h)
    Fr half = fr_inv(fr_from_u64(2));
    Fr acc = fr_one();
    for (unsigned i = 0; i < h; ++i) acc = fr_mul(acc, half);
    return acc;
}

}  // namespace oracle
