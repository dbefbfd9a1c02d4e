// Arithmetic on small integers against field elements, for tensors that are
// still the integers they were quantised to (before the first fold of a
// sumcheck): a product of a 256-bit field element with a 32- or 64-bit integer
// is 8 or 16 multiply-adds and needs no reduction until the end of a sum, or
// only a short one (two or three word steps of Montgomery's reduction instead
// of eight) when a single element has to come out reduced.
//
// Plain C++: the header also compiles for the host, where it is tested against
// big integers.
#pragma once
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define ZK_SHD __host__ __device__ __forceinline__
#else
#define ZK_SHD inline
#endif

namespace zkmi {

// r in 32-bit words.  r = 1 mod 2^32, so the digit of a reduction step is the
// negated low word.
#define ZK_SMALL_R_WORDS \
    { 0x00000001u, 0xffffffffu, 0xfffe5bfeu, 0x53bda402u, 0x09a1d805u, 0x3339d808u, 0x299d7d48u, 0x73eda753u }

// t (NL words, little endian) += c (8 words) * m * 2^(32 OFF), carries propagated
// to the top.  The caller keeps the total below 2^(32 NL).
template <int NL, int OFF = 0>
ZK_SHD void small_mac32(uint32_t (&t)[NL], const uint32_t (&c)[8], uint32_t m) {
    static_assert(NL >= OFF + 9, "room for the product");
    uint64_t carry = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        carry += (uint64_t)c[j] * m + t[OFF + j];  // (2^32-1)^2 + 2 (2^32-1) < 2^64
        t[OFF + j] = (uint32_t)carry;
        carry >>= 32;
    }
#pragma unroll
    for (int j = OFF + 8; j < NL; ++j) {
        carry += t[j];
        t[j] = (uint32_t)carry;
        carry >>= 32;
    }
}

template <int NL>
ZK_SHD void small_mac64(uint32_t (&t)[NL], const uint32_t (&c)[8], uint64_t m) {
    small_mac32<NL, 0>(t, c, (uint32_t)m);
    small_mac32<NL, 1>(t, c, (uint32_t)(m >> 32));
}

// STEPS word steps of Montgomery's reduction on t (8 + STEPS + 1 words, the top
// one zero or small): returns t / 2^(32 STEPS) mod r, fully reduced, in eight
// words.  Needs t < r 2^(32 STEPS), so that the quotient plus r stays below 2 r.
template <int STEPS>
ZK_SHD void small_reduce(uint32_t (&out)[8], uint32_t (&t)[8 + STEPS + 1]) {
    constexpr uint32_t r[8] = ZK_SMALL_R_WORDS;
    constexpr int NL = 8 + STEPS + 1;
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
        const uint32_t m = 0u - t[s];
        uint64_t carry = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            carry += (uint64_t)m * r[j] + t[s + j];
            t[s + j] = (uint32_t)carry;
            carry >>= 32;
        }
#pragma unroll
        for (int j = s + 8; j < NL; ++j) {
            carry += t[j];
            t[j] = (uint32_t)carry;
            carry >>= 32;
        }
    }
    // t[STEPS .. STEPS+8) < 2 r < 2^256 (the top word is zero by now): one conditional subtraction
    uint32_t d[8];
    uint64_t borrow = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint64_t v = (uint64_t)t[STEPS + k] - r[k] - borrow;
        d[k] = (uint32_t)v;
        borrow = (v >> 32) & 1u;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) out[k] = borrow ? t[STEPS + k] : d[k];
}

// The four constants a small integer is folded with: for x' = a + rho (b - a),
// scaled by s, all in Montgomery form and times 2^64 (the factor
// small_reduce<2> takes away again):
//   plus_a = s, minus_a = -s, plus_d = rho s, minus_d = -rho s.
struct SmallFoldConsts {
    uint32_t plus_a[8], minus_a[8], plus_d[8], minus_d[8];
};

// a + rho (b - a), times s, for 64-bit signed a and b with |a|, |b| < 2^62.
ZK_SHD void small_fold64(uint32_t (&out)[8], int64_t a, int64_t b, const SmallFoldConsts& k) {
    uint32_t t[11];
#pragma unroll
    for (int j = 0; j < 11; ++j) t[j] = 0;
    const int64_t d = b - a;  // |d| < 2^63
    const uint64_t ma = a < 0 ? 0ull - (uint64_t)a : (uint64_t)a, md = d < 0 ? 0ull - (uint64_t)d : (uint64_t)d;
    uint32_t ca[8], cd[8];  // selected per lane, so that the products are not written twice under a branch
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        ca[j] = a < 0 ? k.minus_a[j] : k.plus_a[j];
        cd[j] = d < 0 ? k.minus_d[j] : k.plus_d[j];
    }
    small_mac64(t, ca, ma);
    small_mac64(t, cd, md);
    small_reduce<2>(out, t);  // t < (2^62 + 2^63) r < r 2^64
}

// The same for unsigned 32-bit a and b.
ZK_SHD void small_fold32(uint32_t (&out)[8], uint32_t a, uint32_t b, const SmallFoldConsts& k) {
    uint32_t t[11];
#pragma unroll
    for (int j = 0; j < 11; ++j) t[j] = 0;
    uint32_t cd[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) cd[j] = b < a ? k.minus_d[j] : k.plus_d[j];
    small_mac32(t, k.plus_a, a);
    small_mac32(t, cd, b < a ? a - b : b - a);
    small_reduce<2>(out, t);  // t < 2^33 r < r 2^64
}

// A tensor given as small integers: S_i = x_i + rho y_i for signed 32-bit x, y
// (a pair of columns combined by a field element, Section 4's reduction of a
// function table to a set; y == nullptr: S_i = x_i).  The constants are in
// Montgomery form and times 2^64, as in SmallFoldConsts.
struct SmallSource {
    const int32_t* x;  // nullptr: there is no such source
    const int32_t* y;
    uint32_t plus_one[8], minus_one[8], plus_rho[8], minus_rho[8];
};

ZK_SHD uint32_t small_abs32(int32_t v) { return v < 0 ? 0u - (uint32_t)v : (uint32_t)v; }

// x + rho y as a reduced field element in Montgomery form.
ZK_SHD void small_combine32(uint32_t (&out)[8], int32_t x, int32_t y, const SmallSource& k) {
    uint32_t t[11];
#pragma unroll
    for (int j = 0; j < 11; ++j) t[j] = 0;
    uint32_t cx[8], cy[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        cx[j] = x < 0 ? k.minus_one[j] : k.plus_one[j];
        cy[j] = y < 0 ? k.minus_rho[j] : k.plus_rho[j];
    }
    small_mac32(t, cx, small_abs32(x));
    small_mac32(t, cy, small_abs32(y));
    small_reduce<2>(out, t);  // t < 2^32 r < r 2^64
}

ZK_SHD void small_source_load(uint32_t (&out)[8], const SmallSource& k, size_t i) {
    small_combine32(out, k.x[i], k.y ? k.y[i] : 0, k);
}

// The fold of two such entries by a challenge: (x0 + rho y0) + c ((x1 + rho y1) - (x0 + rho y0))
//   = x0 + c (x1 - x0) + rho y0 + rho c (y1 - y0),
// four small integers against eight constants (plus and minus of 1, c, rho, rho c;
// Montgomery form, times 2^64).
struct SmallFold4 {
    uint32_t plus_one[8], minus_one[8], plus_c[8], minus_c[8], plus_rho[8], minus_rho[8], plus_rho_c[8], minus_rho_c[8];
};

ZK_SHD void small_fold_combined(uint32_t (&out)[8], int32_t x0, int32_t y0, int32_t x1, int32_t y1, const SmallFold4& k) {
    uint32_t t[11];
#pragma unroll
    for (int j = 0; j < 11; ++j) t[j] = 0;
    const int64_t dx = (int64_t)x1 - x0, dy = (int64_t)y1 - y0;  // 33 bits with sign
    const uint64_t mdx = dx < 0 ? 0ull - (uint64_t)dx : (uint64_t)dx, mdy = dy < 0 ? 0ull - (uint64_t)dy : (uint64_t)dy;
    uint32_t c0[8], c1[8], c2[8], c3[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        c0[j] = x0 < 0 ? k.minus_one[j] : k.plus_one[j];
        c1[j] = dx < 0 ? k.minus_c[j] : k.plus_c[j];
        c2[j] = y0 < 0 ? k.minus_rho[j] : k.plus_rho[j];
        c3[j] = dy < 0 ? k.minus_rho_c[j] : k.plus_rho_c[j];
    }
    small_mac32(t, c0, small_abs32(x0));
    small_mac64(t, c1, mdx);
    small_mac32(t, c2, small_abs32(y0));
    small_mac64(t, c3, mdy);
    small_reduce<2>(out, t);  // t < (2^31 + 2^32 + 2^31 + 2^32) r < r 2^64
}

}  // namespace zkmi
