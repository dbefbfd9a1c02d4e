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

// acc (64 bits) and ex (overflow count) form a 96-bit column accumulator.
// fr_macN adds N limb products to it: each v_mad_u64_u32 leaves the carry out of
// bit 63 in VCC and the v_addc_co_u32 behind it folds that carry into ex, two
// full-rate instructions per limb product.  A whole column goes into one asm
// statement so that the compiler's hazard padding between statements is paid
// once per column, not once per product.  The K variants take wave-uniform
// second factors (limbs of r) from scalar registers.  With FIRST the statement
// opens a column: ex is written, not updated (its first carry fold adds to zero),
// so that it needs no clearing and can be allocated straight into the register
// it has to end up in.
#define ZK_MAC(x, y) "v_mad_u64_u32 %0, vcc, %" #x ", %" #y ", %0\n\tv_addc_co_u32 %1, vcc, 0, %1, vcc\n\t"
#define ZK_MAC0(x, y) "v_mad_u64_u32 %0, vcc, %" #x ", %" #y ", %0\n\tv_addc_co_u32 %1, vcc, 0, 0, vcc\n\t"
template <bool FIRST = false>
__device__ __forceinline__ void fr_mac1(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) : "+v"(acc), "=&v"(ex) : "v"(x0), "v"(y0) : "vcc");
    else asm(ZK_MAC(2, 3) : "+v"(acc), "+v"(ex) : "v"(x0), "v"(y0) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mack1(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) : "+v"(acc), "=&v"(ex) : "v"(x0), "s"(y0) : "vcc");
    else asm(ZK_MAC(2, 3) : "+v"(acc), "+v"(ex) : "v"(x0), "s"(y0) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mac2(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) : "+v"(acc), "=&v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) : "+v"(acc), "+v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mack2(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) : "+v"(acc), "=&v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) : "+v"(acc), "+v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mac3(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) : "+v"(acc), "=&v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) : "+v"(acc), "+v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mack3(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) : "+v"(acc), "=&v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) : "+v"(acc), "+v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mac4(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) : "+v"(acc), "=&v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) : "+v"(acc), "+v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mack4(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) : "+v"(acc), "=&v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) : "+v"(acc), "+v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mac5(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3, uint32_t x4, uint32_t y4) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) : "+v"(acc), "=&v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3), "v"(x4), "v"(y4) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) : "+v"(acc), "+v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3), "v"(x4), "v"(y4) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mack5(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3, uint32_t x4, uint32_t y4) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) : "+v"(acc), "=&v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3), "v"(x4), "s"(y4) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) : "+v"(acc), "+v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3), "v"(x4), "s"(y4) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mac6(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3, uint32_t x4, uint32_t y4, uint32_t x5, uint32_t y5) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) : "+v"(acc), "=&v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3), "v"(x4), "v"(y4), "v"(x5), "v"(y5) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) : "+v"(acc), "+v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3), "v"(x4), "v"(y4), "v"(x5), "v"(y5) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mack6(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3, uint32_t x4, uint32_t y4, uint32_t x5, uint32_t y5) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) : "+v"(acc), "=&v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3), "v"(x4), "s"(y4), "v"(x5), "s"(y5) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) : "+v"(acc), "+v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3), "v"(x4), "s"(y4), "v"(x5), "s"(y5) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mac7(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3, uint32_t x4, uint32_t y4, uint32_t x5, uint32_t y5, uint32_t x6, uint32_t y6) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) ZK_MAC(14, 15) : "+v"(acc), "=&v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3), "v"(x4), "v"(y4), "v"(x5), "v"(y5), "v"(x6), "v"(y6) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) ZK_MAC(14, 15) : "+v"(acc), "+v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3), "v"(x4), "v"(y4), "v"(x5), "v"(y5), "v"(x6), "v"(y6) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mack7(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3, uint32_t x4, uint32_t y4, uint32_t x5, uint32_t y5, uint32_t x6, uint32_t y6) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) ZK_MAC(14, 15) : "+v"(acc), "=&v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3), "v"(x4), "s"(y4), "v"(x5), "s"(y5), "v"(x6), "s"(y6) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) ZK_MAC(14, 15) : "+v"(acc), "+v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3), "v"(x4), "s"(y4), "v"(x5), "s"(y5), "v"(x6), "s"(y6) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mac8(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3, uint32_t x4, uint32_t y4, uint32_t x5, uint32_t y5, uint32_t x6, uint32_t y6, uint32_t x7, uint32_t y7) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) ZK_MAC(14, 15) ZK_MAC(16, 17) : "+v"(acc), "=&v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3), "v"(x4), "v"(y4), "v"(x5), "v"(y5), "v"(x6), "v"(y6), "v"(x7), "v"(y7) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) ZK_MAC(14, 15) ZK_MAC(16, 17) : "+v"(acc), "+v"(ex) : "v"(x0), "v"(y0), "v"(x1), "v"(y1), "v"(x2), "v"(y2), "v"(x3), "v"(y3), "v"(x4), "v"(y4), "v"(x5), "v"(y5), "v"(x6), "v"(y6), "v"(x7), "v"(y7) : "vcc");
}
template <bool FIRST = false>
__device__ __forceinline__ void fr_mack8(uint64_t& acc, uint32_t& ex, uint32_t x0, uint32_t y0, uint32_t x1, uint32_t y1, uint32_t x2, uint32_t y2, uint32_t x3, uint32_t y3, uint32_t x4, uint32_t y4, uint32_t x5, uint32_t y5, uint32_t x6, uint32_t y6, uint32_t x7, uint32_t y7) {
    if constexpr (FIRST) asm(ZK_MAC0(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) ZK_MAC(14, 15) ZK_MAC(16, 17) : "+v"(acc), "=&v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3), "v"(x4), "s"(y4), "v"(x5), "s"(y5), "v"(x6), "s"(y6), "v"(x7), "s"(y7) : "vcc");
    else asm(ZK_MAC(2, 3) ZK_MAC(4, 5) ZK_MAC(6, 7) ZK_MAC(8, 9) ZK_MAC(10, 11) ZK_MAC(12, 13) ZK_MAC(14, 15) ZK_MAC(16, 17) : "+v"(acc), "+v"(ex) : "v"(x0), "s"(y0), "v"(x1), "s"(y1), "v"(x2), "s"(y2), "v"(x3), "s"(y3), "v"(x4), "s"(y4), "v"(x5), "s"(y5), "v"(x6), "s"(y6), "v"(x7), "s"(y7) : "vcc");
}

// Adds a_lo..a_hi times the matching b limbs of column c (indices j, c-j).
template <int C, int LO, int N, bool FIRST = false>
__device__ __forceinline__ void fr_col_products(uint64_t& acc, uint32_t& ex, const uint32_t* a, const uint32_t* b) {
    if constexpr (N == 1) fr_mac1<FIRST>(acc, ex, a[LO], b[C - LO]);
    if constexpr (N == 2) fr_mac2<FIRST>(acc, ex, a[LO], b[C - LO], a[LO + 1], b[C - LO - 1]);
    if constexpr (N == 3) fr_mac3<FIRST>(acc, ex, a[LO], b[C - LO], a[LO + 1], b[C - LO - 1], a[LO + 2], b[C - LO - 2]);
    if constexpr (N == 4) fr_mac4<FIRST>(acc, ex, a[LO], b[C - LO], a[LO + 1], b[C - LO - 1], a[LO + 2], b[C - LO - 2], a[LO + 3], b[C - LO - 3]);
    if constexpr (N == 5) fr_mac5<FIRST>(acc, ex, a[LO], b[C - LO], a[LO + 1], b[C - LO - 1], a[LO + 2], b[C - LO - 2], a[LO + 3], b[C - LO - 3], a[LO + 4], b[C - LO - 4]);
    if constexpr (N == 6) fr_mac6<FIRST>(acc, ex, a[LO], b[C - LO], a[LO + 1], b[C - LO - 1], a[LO + 2], b[C - LO - 2], a[LO + 3], b[C - LO - 3], a[LO + 4], b[C - LO - 4], a[LO + 5], b[C - LO - 5]);
    if constexpr (N == 7) fr_mac7<FIRST>(acc, ex, a[LO], b[C - LO], a[LO + 1], b[C - LO - 1], a[LO + 2], b[C - LO - 2], a[LO + 3], b[C - LO - 3], a[LO + 4], b[C - LO - 4], a[LO + 5], b[C - LO - 5], a[LO + 6], b[C - LO - 6]);
    if constexpr (N == 8) fr_mac8<FIRST>(acc, ex, a[LO], b[C - LO], a[LO + 1], b[C - LO - 1], a[LO + 2], b[C - LO - 2], a[LO + 3], b[C - LO - 3], a[LO + 4], b[C - LO - 4], a[LO + 5], b[C - LO - 5], a[LO + 6], b[C - LO - 6], a[LO + 7], b[C - LO - 7]);
}

// Adds m_lo..m_hi times the matching limbs of r of column c (indices i, c-i).
template <int C, int LO, int N, bool FIRST = false>
__device__ __forceinline__ void fr_col_reductions(uint64_t& acc, uint32_t& ex, const uint32_t* m) {
    constexpr uint32_t r[8] = {ZK_R0, ZK_R1, ZK_R2, ZK_R3, ZK_R4, ZK_R5, ZK_R6, ZK_R7};
    if constexpr (N == 1) fr_mack1<FIRST>(acc, ex, m[LO], r[C - LO]);
    if constexpr (N == 2) fr_mack2<FIRST>(acc, ex, m[LO], r[C - LO], m[LO + 1], r[C - LO - 1]);
    if constexpr (N == 3) fr_mack3<FIRST>(acc, ex, m[LO], r[C - LO], m[LO + 1], r[C - LO - 1], m[LO + 2], r[C - LO - 2]);
    if constexpr (N == 4) fr_mack4<FIRST>(acc, ex, m[LO], r[C - LO], m[LO + 1], r[C - LO - 1], m[LO + 2], r[C - LO - 2], m[LO + 3], r[C - LO - 3]);
    if constexpr (N == 5) fr_mack5<FIRST>(acc, ex, m[LO], r[C - LO], m[LO + 1], r[C - LO - 1], m[LO + 2], r[C - LO - 2], m[LO + 3], r[C - LO - 3], m[LO + 4], r[C - LO - 4]);
    if constexpr (N == 6) fr_mack6<FIRST>(acc, ex, m[LO], r[C - LO], m[LO + 1], r[C - LO - 1], m[LO + 2], r[C - LO - 2], m[LO + 3], r[C - LO - 3], m[LO + 4], r[C - LO - 4], m[LO + 5], r[C - LO - 5]);
    if constexpr (N == 7) fr_mack7<FIRST>(acc, ex, m[LO], r[C - LO], m[LO + 1], r[C - LO - 1], m[LO + 2], r[C - LO - 2], m[LO + 3], r[C - LO - 3], m[LO + 4], r[C - LO - 4], m[LO + 5], r[C - LO - 5], m[LO + 6], r[C - LO - 6]);
    if constexpr (N == 8) fr_mack8<FIRST>(acc, ex, m[LO], r[C - LO], m[LO + 1], r[C - LO - 1], m[LO + 2], r[C - LO - 2], m[LO + 3], r[C - LO - 3], m[LO + 4], r[C - LO - 4], m[LO + 5], r[C - LO - 5], m[LO + 6], r[C - LO - 6], m[LO + 7], r[C - LO - 7]);
}

// Same as fr_col_products with the b limbs wave-uniform (scalar registers).
template <int C, int LO, int N, bool FIRST = false>
__device__ __forceinline__ void fr_col_products_k(uint64_t& acc, uint32_t& ex, const uint32_t* a, const uint32_t* k) {
    if constexpr (N == 1) fr_mack1<FIRST>(acc, ex, a[LO], k[C - LO]);
    if constexpr (N == 2) fr_mack2<FIRST>(acc, ex, a[LO], k[C - LO], a[LO + 1], k[C - LO - 1]);
    if constexpr (N == 3) fr_mack3<FIRST>(acc, ex, a[LO], k[C - LO], a[LO + 1], k[C - LO - 1], a[LO + 2], k[C - LO - 2]);
    if constexpr (N == 4) fr_mack4<FIRST>(acc, ex, a[LO], k[C - LO], a[LO + 1], k[C - LO - 1], a[LO + 2], k[C - LO - 2], a[LO + 3], k[C - LO - 3]);
    if constexpr (N == 5) fr_mack5<FIRST>(acc, ex, a[LO], k[C - LO], a[LO + 1], k[C - LO - 1], a[LO + 2], k[C - LO - 2], a[LO + 3], k[C - LO - 3], a[LO + 4], k[C - LO - 4]);
    if constexpr (N == 6) fr_mack6<FIRST>(acc, ex, a[LO], k[C - LO], a[LO + 1], k[C - LO - 1], a[LO + 2], k[C - LO - 2], a[LO + 3], k[C - LO - 3], a[LO + 4], k[C - LO - 4], a[LO + 5], k[C - LO - 5]);
    if constexpr (N == 7) fr_mack7<FIRST>(acc, ex, a[LO], k[C - LO], a[LO + 1], k[C - LO - 1], a[LO + 2], k[C - LO - 2], a[LO + 3], k[C - LO - 3], a[LO + 4], k[C - LO - 4], a[LO + 5], k[C - LO - 5], a[LO + 6], k[C - LO - 6]);
    if constexpr (N == 8) fr_mack8<FIRST>(acc, ex, a[LO], k[C - LO], a[LO + 1], k[C - LO - 1], a[LO + 2], k[C - LO - 2], a[LO + 3], k[C - LO - 3], a[LO + 4], k[C - LO - 4], a[LO + 5], k[C - LO - 5], a[LO + 6], k[C - LO - 6], a[LO + 7], k[C - LO - 7]);
}

// ---- from one column to the next ------------------------------------------------
//
// After a column, the accumulator's upper word and the overflow count become the
// next column's accumulator.  The upper word of a 64-bit register pair can only
// become a lower word by being written again, so these steps make that write do
// some work: it takes in what the next column starts from (the carry of a word
// that has just been cleared, a limb of a wide accumulator).

// next = (acc >> 32) + (ex << 32)
__device__ __forceinline__ uint64_t fr_col_next(uint64_t acc, uint32_t ex) {
    return (acc >> 32) | ((uint64_t)ex << 32);
}

// The same plus a 32-bit addend for the next column.
__device__ __forceinline__ uint64_t fr_col_next_plus(uint64_t acc, uint32_t ex, uint32_t addend) {
    uint32_t hi = (uint32_t)(acc >> 32), nlo, nhi;
    asm("v_add_co_u32 %0, vcc, %2, %3\n\tv_addc_co_u32 %1, vcc, 0, %4, vcc"
        : "=&v"(nlo), "=v"(nhi)
        : "v"(hi), "v"(addend), "v"(ex)
        : "vcc");
    return nlo | ((uint64_t)nhi << 32);
}

// After the Montgomery digit m = -lo of a column has been chosen: adding
// m * r_0 = m clears the column's low word and carries one unless that word was
// zero already, so next = hi + (lo != 0) + (ex << 32) and the product m * r_0 is
// never formed.
__device__ __forceinline__ uint64_t fr_col_next_cleared(uint64_t acc, uint32_t ex) {
    uint32_t lo = (uint32_t)acc, hi = (uint32_t)(acc >> 32), nlo, nhi;
    asm("v_cmp_ne_u32 vcc, 0, %2\n\tv_addc_co_u32 %0, vcc, 0, %3, vcc\n\tv_addc_co_u32 %1, vcc, 0, %4, vcc"
        : "=&v"(nlo), "=v"(nhi)
        : "v"(lo), "v"(hi), "v"(ex)
        : "vcc");
    return nlo | ((uint64_t)nhi << 32);
}

// Both: next = hi + (lo != 0) + addend + (ex << 32).
__device__ __forceinline__ uint64_t fr_col_next_cleared_plus(uint64_t acc, uint32_t ex, uint32_t addend) {
    uint32_t lo = (uint32_t)acc, hi = (uint32_t)(acc >> 32), nlo, nhi;
    asm("v_cmp_ne_u32 vcc, 0, %2\n\tv_addc_co_u32 %0, vcc, %3, %5, vcc\n\tv_addc_co_u32 %1, vcc, 0, %4, vcc"
        : "=&v"(nlo), "=v"(nhi)
        : "v"(lo), "v"(hi), "v"(ex), "v"(addend)
        : "vcc");
    return nlo | ((uint64_t)nhi << 32);
}

template <bool UNIFORM_B, int C>
__device__ __forceinline__ uint64_t fr_mul_low_column(uint64_t acc, const uint32_t* a, const uint32_t* b, uint32_t* m) {
    uint32_t ex;
    if constexpr (UNIFORM_B) fr_col_products_k<C, 0, C + 1, true>(acc, ex, a, b);
    else fr_col_products<C, 0, C + 1, true>(acc, ex, a, b);
    fr_col_reductions<C, 0, C>(acc, ex, m);
    m[C] = 0u - (uint32_t)acc;
    return fr_col_next_cleared(acc, ex);
}

template <bool UNIFORM_B, int C>
__device__ __forceinline__ uint64_t fr_mul_high_column(uint64_t acc, const uint32_t* a, const uint32_t* b,
                                                       const uint32_t* m, uint32_t* t) {
    uint32_t ex;
    if constexpr (UNIFORM_B) fr_col_products_k<C, C - 7, 15 - C, true>(acc, ex, a, b);
    else fr_col_products<C, C - 7, 15 - C, true>(acc, ex, a, b);
    fr_col_reductions<C, C - 7, 15 - C>(acc, ex, m);
    t[C - 8] = (uint32_t)acc;
    return fr_col_next(acc, ex);
}

// Montgomery product a * b / 2^256 mod r, column by column (product scanning with
// the reduction interleaved): column c collects a_j b_(c-j) and m_i r_(c-i); for
// c < 8 the digit m_c = -column (r = 1 mod 2^32) is the one whose r_0 term clears
// the column's low word.  120 multiply-adds, each with one carry fold.
template <bool UNIFORM_B>
__device__ __forceinline__ Fr fr_mul_impl(const Fr& a, const Fr& b) {
    uint32_t m[8];
    uint32_t t[8];
    uint64_t acc = (uint64_t)a.l[0] * b.l[0];  // column 0 has a single product
    m[0] = 0u - (uint32_t)acc;
    acc = fr_col_next_cleared(acc, 0u);
    acc = fr_mul_low_column<UNIFORM_B, 1>(acc, a.l, b.l, m);
    acc = fr_mul_low_column<UNIFORM_B, 2>(acc, a.l, b.l, m);
    acc = fr_mul_low_column<UNIFORM_B, 3>(acc, a.l, b.l, m);
    acc = fr_mul_low_column<UNIFORM_B, 4>(acc, a.l, b.l, m);
    acc = fr_mul_low_column<UNIFORM_B, 5>(acc, a.l, b.l, m);
    acc = fr_mul_low_column<UNIFORM_B, 6>(acc, a.l, b.l, m);
    acc = fr_mul_low_column<UNIFORM_B, 7>(acc, a.l, b.l, m);
    acc = fr_mul_high_column<UNIFORM_B, 8>(acc, a.l, b.l, m, t);
    acc = fr_mul_high_column<UNIFORM_B, 9>(acc, a.l, b.l, m, t);
    acc = fr_mul_high_column<UNIFORM_B, 10>(acc, a.l, b.l, m, t);
    acc = fr_mul_high_column<UNIFORM_B, 11>(acc, a.l, b.l, m, t);
    acc = fr_mul_high_column<UNIFORM_B, 12>(acc, a.l, b.l, m, t);
    acc = fr_mul_high_column<UNIFORM_B, 13>(acc, a.l, b.l, m, t);
    acc = fr_mul_high_column<UNIFORM_B, 14>(acc, a.l, b.l, m, t);
    // column 15 holds only what was carried up; the result is < 2r < 2^256
    t[7] = (uint32_t)acc;
    return fr_reduce_once(t);
}

__device__ __forceinline__ Fr fr_mul(const Fr& a, const Fr& b) { return fr_mul_impl<false>(a, b); }

// a * k for a wave-uniform k (a kernel argument or a constant): its limbs stay in
// scalar registers and cost no vector registers.
__device__ __forceinline__ Fr fr_mul_uniform(const Fr& a, const Fr& k) { return fr_mul_impl<true>(a, k); }

// ---- sums of products without intermediate reductions ---------------------------
//
// A sum of Montgomery products sum_i a_i b_i / 2^256 needs only one reduction:
// the 512-bit integer products are added up first.  FrWide holds such a sum as
// sixteen limbs with the invariant (upper half) < r, i.e. value < r * 2^256, which
// is what a single Montgomery reduction can take; after each addition the upper
// half is brought back below r by one conditional subtraction (the product adds
// less than 0.46 r to it).
struct FrWide {
    uint32_t l[16];
};

__device__ __forceinline__ FrWide fr_wide_zero() {
    FrWide w;
#pragma unroll
    for (int k = 0; k < 16; ++k) w.l[k] = 0;
    return w;
}

// Column C of w += a * b.  The accumulator comes in holding the carry of the
// column below plus w's own limb C, and leaves holding the same for column C + 1.
template <int C>
__device__ __forceinline__ uint64_t fr_wide_column(uint64_t acc, FrWide& w, const uint32_t* a, const uint32_t* b) {
    uint32_t ex;
    if constexpr (C < 8) fr_col_products<C, 0, C + 1, true>(acc, ex, a, b);
    else fr_col_products<C, C - 7, 15 - C, true>(acc, ex, a, b);
    w.l[C] = (uint32_t)acc;
    return fr_col_next_plus(acc, ex, w.l[C + 1]);
}

// w += a * b (as integers), keeping the invariant.
__device__ __forceinline__ void fr_wide_mac(FrWide& w, const Fr& a, const Fr& b) {
    uint64_t acc = w.l[0];
    acc = fr_wide_column<0>(acc, w, a.l, b.l);
    acc = fr_wide_column<1>(acc, w, a.l, b.l);
    acc = fr_wide_column<2>(acc, w, a.l, b.l);
    acc = fr_wide_column<3>(acc, w, a.l, b.l);
    acc = fr_wide_column<4>(acc, w, a.l, b.l);
    acc = fr_wide_column<5>(acc, w, a.l, b.l);
    acc = fr_wide_column<6>(acc, w, a.l, b.l);
    acc = fr_wide_column<7>(acc, w, a.l, b.l);
    acc = fr_wide_column<8>(acc, w, a.l, b.l);
    acc = fr_wide_column<9>(acc, w, a.l, b.l);
    acc = fr_wide_column<10>(acc, w, a.l, b.l);
    acc = fr_wide_column<11>(acc, w, a.l, b.l);
    acc = fr_wide_column<12>(acc, w, a.l, b.l);
    acc = fr_wide_column<13>(acc, w, a.l, b.l);
    acc = fr_wide_column<14>(acc, w, a.l, b.l);
    w.l[15] = (uint32_t)acc;  // upper half stays below 1.46 r < 2^256: nothing above this word
    Fr hi = fr_reduce_once(&w.l[8]);
#pragma unroll
    for (int k = 0; k < 8; ++k) w.l[8 + k] = hi.l[k];
}

// w / 2^256 mod r, fully reduced: the reduction half of a Montgomery product.
// Column c < 8: w_c + sum_{i<c} m_i r_(c-i), then m_c clears it; columns 8..14
// give the result.  As in fr_wide_mac the accumulator enters a column already
// holding w's limb of that column.
__device__ __forceinline__ Fr fr_wide_reduce(const FrWide& w) {
    uint32_t m[8];
    uint32_t t[8];
    uint64_t acc = w.l[0];
    m[0] = 0u - (uint32_t)acc;
    acc = fr_col_next_cleared_plus(acc, 0u, w.l[1]);
#define ZK_WIDE_LOW(C)                                         \
    {                                                          \
        uint32_t ex;                                           \
        fr_col_reductions<C, 0, C, true>(acc, ex, m);          \
        m[C] = 0u - (uint32_t)acc;                             \
        acc = fr_col_next_cleared_plus(acc, ex, w.l[C + 1]);   \
    }
    ZK_WIDE_LOW(1) ZK_WIDE_LOW(2) ZK_WIDE_LOW(3) ZK_WIDE_LOW(4) ZK_WIDE_LOW(5) ZK_WIDE_LOW(6) ZK_WIDE_LOW(7)
#undef ZK_WIDE_LOW
#define ZK_WIDE_HIGH(C)                                        \
    {                                                          \
        uint32_t ex;                                           \
        fr_col_reductions<C, C - 7, 15 - C, true>(acc, ex, m); \
        t[C - 8] = (uint32_t)acc;                              \
        acc = fr_col_next_plus(acc, ex, w.l[C + 1]);           \
    }
    ZK_WIDE_HIGH(8) ZK_WIDE_HIGH(9) ZK_WIDE_HIGH(10) ZK_WIDE_HIGH(11) ZK_WIDE_HIGH(12) ZK_WIDE_HIGH(13) ZK_WIDE_HIGH(14)
#undef ZK_WIDE_HIGH
    t[7] = (uint32_t)acc;  // result < 2r < 2^256
    return fr_reduce_once(t);
}

__device__ __forceinline__ Fr fr_sqr(const Fr& a) { return fr_mul(a, a); }

// canonical integer (8 limbs, < 2^256) -> Montgomery form
__device__ __forceinline__ Fr fr_to_mont(const Fr& canonical) { return fr_mul_uniform(canonical, fr_rr()); }

// Montgomery form -> canonical integer in [0, r): a / 2^256 mod r is the
// reduction half of a product alone, applied to a as the low half of a wide value.
__device__ __forceinline__ Fr fr_from_mont(const Fr& a) {
    FrWide w;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        w.l[k] = a.l[k];
        w.l[8 + k] = 0;
    }
    return fr_wide_reduce(w);
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

// The element's address is kept per lane in vector registers and stepped from
// one limb plane to the next; holding eight scalar plane pointers per array
// instead would exhaust the scalar register file in kernels that touch several
// arrays.
__device__ __forceinline__ Fr fr_load(const uint32_t* __restrict__ p, size_t stride, size_t i) {
    const uint32_t* q = p + i;
    asm("" : "+v"(q));
    Fr a;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        a.l[k] = *q;
        q += stride;
    }
    return a;
}

__device__ __forceinline__ void fr_store(uint32_t* __restrict__ p, size_t stride, size_t i, const Fr& a) {
    uint32_t* q = p + i;
    asm("" : "+v"(q));
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        *q = a.l[k];
        q += stride;
    }
}

// a0 + r * (a1 - a0): one variable of a multilinear extension bound to r, the
// same r for the whole wavefront.
__device__ __forceinline__ Fr fr_fold(const Fr& a0, const Fr& a1, const Fr& r) {
    return fr_add(a0, fr_mul_uniform(fr_sub(a1, a0), r));
}

}  // namespace zkmi
