// Device-side arithmetic in the BLS12-381 scalar field Fr for gfx950.
//
// An element lives in eight 32-bit VGPRs in Montgomery form (x * 2^256 mod r),
// always fully reduced, so equality of values is equality of limbs.  In HBM a
// vector is limb-major: limb k of element i at limbs[k*stride + i], which makes
// every limb load of a wavefront one contiguous 256-byte segment.
//
// On gfx950 v_mad_u64_u32 issues at the same rate as a 32-bit add, so the cost
// of a multiplication is its instruction count, not its multiplier count.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zkmi {

struct Fr {
    uint32_t l[8];
};

// r, least significant limb first.  r = 1 mod 2^32, hence -r^-1 mod 2^32 = 2^32 - 1
// and the Montgomery quotient digit is simply the negated low limb.
#define ZK_R0 0x00000001u
#define ZK_R1 0xffffffffu
#define ZK_R2 0xfffe5bfeu
#define ZK_R3 0x53bda402u
#define ZK_R4 0x09a1d805u
#define ZK_R5 0x3339d808u
#define ZK_R6 0x299d7d48u
#define ZK_R7 0x73eda753u

// 2^256 mod r: the Montgomery form of 1.
#define ZK_ONE0 0xfffffffeu
#define ZK_ONE1 0x00000001u
#define ZK_ONE2 0x00034802u
#define ZK_ONE3 0x5884b7fau
#define ZK_ONE4 0xecbc4ff5u
#define ZK_ONE5 0x998c4fefu
#define ZK_ONE6 0xacc5056fu
#define ZK_ONE7 0x1824b159u

// 2^512 mod r: multiplying by it converts a canonical integer to Montgomery form.
#define ZK_RR0 0xf3f29c6du
#define ZK_RR1 0xc999e990u
#define ZK_RR2 0x87925c23u
#define ZK_RR3 0x2b6cedcbu
#define ZK_RR4 0x7254398fu
#define ZK_RR5 0x05d31496u
#define ZK_RR6 0x9f59ff11u
#define ZK_RR7 0x0748d9d9u

__device__ __forceinline__ Fr fr_zero() { return Fr{{0, 0, 0, 0, 0, 0, 0, 0}}; }
__device__ __forceinline__ Fr fr_one() {
    return Fr{{ZK_ONE0, ZK_ONE1, ZK_ONE2, ZK_ONE3, ZK_ONE4, ZK_ONE5, ZK_ONE6, ZK_ONE7}};
}
__device__ __forceinline__ Fr fr_rr() {
    return Fr{{ZK_RR0, ZK_RR1, ZK_RR2, ZK_RR3, ZK_RR4, ZK_RR5, ZK_RR6, ZK_RR7}};
}

__device__ __forceinline__ bool fr_is_zero(const Fr& a) {
    return (a.l[0] | a.l[1] | a.l[2] | a.l[3] | a.l[4] | a.l[5] | a.l[6] | a.l[7]) == 0;
}

__device__ __forceinline__ bool fr_equal(const Fr& a, const Fr& b) {
    uint32_t d = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) d |= a.l[k] ^ b.l[k];
    return d == 0;
}

// t (8 limbs, < 2r) -> t mod r
__device__ __forceinline__ Fr fr_reduce_once(const uint32_t t[8]) {
    const uint32_t r[8] = {ZK_R0, ZK_R1, ZK_R2, ZK_R3, ZK_R4, ZK_R5, ZK_R6, ZK_R7};
    uint32_t d[8];
    uint32_t borrow = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint32_t bo;
        d[k] = __builtin_subc(t[k], r[k], borrow, &bo);
        borrow = bo;
    }
    Fr o;
#pragma unroll
    for (int k = 0; k < 8; ++k) o.l[k] = borrow ? t[k] : d[k];
    return o;
}

__device__ __forceinline__ Fr fr_add(const Fr& a, const Fr& b) {
    uint32_t s[8];
    uint32_t carry = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint32_t co;
        s[k] = __builtin_addc(a.l[k], b.l[k], carry, &co);
        carry = co;
    }
    // a, b < r < 2^255: no carry out of the top limb
    return fr_reduce_once(s);
}

__device__ __forceinline__ Fr fr_sub(const Fr& a, const Fr& b) {
    const uint32_t r[8] = {ZK_R0, ZK_R1, ZK_R2, ZK_R3, ZK_R4, ZK_R5, ZK_R6, ZK_R7};
    uint32_t d[8];
    uint32_t borrow = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint32_t bo;
        d[k] = __builtin_subc(a.l[k], b.l[k], borrow, &bo);
        borrow = bo;
    }
    // add r back if the difference went negative
    uint32_t mask = 0u - borrow;
    uint32_t carry = 0;
    Fr o;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint32_t co;
        o.l[k] = __builtin_addc(d[k], r[k] & mask, carry, &co);
        carry = co;
    }
    return o;
}

__device__ __forceinline__ Fr fr_neg(const Fr& a) { return fr_sub(fr_zero(), a); }

__device__ __forceinline__ Fr fr_double(const Fr& a) { return fr_add(a, a); }

// Montgomery product a * b / 2^256 mod r (coarsely integrated operand scanning,
// one row of a*b_i then one reduction step per i).
__device__ __forceinline__ Fr fr_mul(const Fr& a, const Fr& b) {
    const uint32_t r[8] = {ZK_R0, ZK_R1, ZK_R2, ZK_R3, ZK_R4, ZK_R5, ZK_R6, ZK_R7};
    uint32_t t[10];
#pragma unroll
    for (int k = 0; k < 10; ++k) t[k] = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint64_t c = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint64_t p = (uint64_t)a.l[j] * b.l[i] + t[j] + c;
            t[j] = (uint32_t)p;
            c = p >> 32;
        }
        uint64_t s = (uint64_t)t[8] + c;
        t[8] = (uint32_t)s;
        t[9] = (uint32_t)(s >> 32);
        // quotient digit m = t0 * (-r^-1) = -t0; t0 + m*r0 = 2^32 * [t0 != 0]
        uint32_t m = 0u - t[0];
        c = (t[0] != 0) ? 1u : 0u;
#pragma unroll
        for (int j = 1; j < 8; ++j) {
            uint64_t p = (uint64_t)m * r[j] + t[j] + c;
            t[j - 1] = (uint32_t)p;
            c = p >> 32;
        }
        s = (uint64_t)t[8] + c;
        t[7] = (uint32_t)s;
        t[8] = t[9] + (uint32_t)(s >> 32);
    }
    return fr_reduce_once(t);
}

__device__ __forceinline__ Fr fr_sqr(const Fr& a) { return fr_mul(a, a); }

// canonical integer (8 limbs, < 2^256) -> Montgomery form
__device__ __forceinline__ Fr fr_to_mont(const Fr& canonical) { return fr_mul(canonical, fr_rr()); }

// Montgomery form -> canonical integer in [0, r)
__device__ __forceinline__ Fr fr_from_mont(const Fr& a) {
    Fr one = Fr{{1, 0, 0, 0, 0, 0, 0, 0}};
    return fr_mul(a, one);
}

// Small unsigned integer -> Montgomery form.
__device__ __forceinline__ Fr fr_from_u32(uint32_t x) {
    Fr c = Fr{{x, 0, 0, 0, 0, 0, 0, 0}};
    return fr_to_mont(c);
}

// ---- limb-major vectors in HBM ----------------------------------------------

struct VecView {
    uint32_t* p;
    size_t stride;
};

__device__ __forceinline__ Fr fr_load(const uint32_t* __restrict__ p, size_t stride, size_t i) {
    Fr a;
#pragma unroll
    for (int k = 0; k < 8; ++k) a.l[k] = p[k * stride + i];
    return a;
}

__device__ __forceinline__ void fr_store(uint32_t* __restrict__ p, size_t stride, size_t i, const Fr& a) {
#pragma unroll
    for (int k = 0; k < 8; ++k) p[k * stride + i] = a.l[k];
}

// a0 + r * (a1 - a0): one variable of a multilinear extension bound to r.
__device__ __forceinline__ Fr fr_fold(const Fr& a0, const Fr& a1, const Fr& r) {
    return fr_add(a0, fr_mul(r, fr_sub(a1, a0)));
}

}  // namespace zkmi
