// SHA-256 (FIPS 180-4) for device code, one message per lane: the compression
// function on a 16-word block held in registers.  Used for the digests that
// stand in for commitments (of m, A and B) in the tlookup transcript; the
// host-side hash of the transcript itself is in transcript.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zkmi {

__device__ __forceinline__ uint32_t sha_rotr(uint32_t x, int n) { return __builtin_amdgcn_alignbit(x, x, (uint32_t)n); }

// Three-input bitwise functions in one instruction (gfx950's v_bitop3_b32; the
// constant is the truth table with inputs weighted 0xf0, 0xcc, 0xaa).
__device__ __forceinline__ uint32_t sha_xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}
__device__ __forceinline__ uint32_t sha_ch(uint32_t e, uint32_t f, uint32_t g) {  // (e & f) ^ (~e & g)
    return __builtin_amdgcn_bitop3_b32(e, f, g, 0xca);
}
__device__ __forceinline__ uint32_t sha_maj(uint32_t a, uint32_t b, uint32_t c) {  // (a & b) ^ (a & c) ^ (b & c)
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0xe8);
}

static __constant__ const uint32_t kShaK[64] = {
    0x428a2f98u, 0x71374491u, 0xb5c0fbcfu, 0xe9b5dba5u, 0x3956c25bu, 0x59f111f1u, 0x923f82a4u, 0xab1c5ed5u,
    0xd807aa98u, 0x12835b01u, 0x243185beu, 0x550c7dc3u, 0x72be5d74u, 0x80deb1feu, 0x9bdc06a7u, 0xc19bf174u,
    0xe49b69c1u, 0xefbe4786u, 0x0fc19dc6u, 0x240ca1ccu, 0x2de92c6fu, 0x4a7484aau, 0x5cb0a9dcu, 0x76f988dau,
    0x983e5152u, 0xa831c66du, 0xb00327c8u, 0xbf597fc7u, 0xc6e00bf3u, 0xd5a79147u, 0x06ca6351u, 0x14292967u,
    0x27b70a85u, 0x2e1b2138u, 0x4d2c6dfcu, 0x53380d13u, 0x650a7354u, 0x766a0abbu, 0x81c2c92eu, 0x92722c85u,
    0xa2bfe8a1u, 0xa81a664bu, 0xc24b8b70u, 0xc76c51a3u, 0xd192e819u, 0xd6990624u, 0xf40e3585u, 0x106aa070u,
    0x19a4c116u, 0x1e376c08u, 0x2748774cu, 0x34b0bcb5u, 0x391c0cb3u, 0x4ed8aa4au, 0x5b9cca4fu, 0x682e6ff3u,
    0x748f82eeu, 0x78a5636fu, 0x84c87814u, 0x8cc70208u, 0x90befffau, 0xa4506cebu, 0xbef9a3f7u, 0xc67178f2u};

__device__ __forceinline__ void sha256_init(uint32_t (&h)[8]) {
    h[0] = 0x6a09e667u; h[1] = 0xbb67ae85u; h[2] = 0x3c6ef372u; h[3] = 0xa54ff53au;
    h[4] = 0x510e527fu; h[5] = 0x9b05688cu; h[6] = 0x1f83d9abu; h[7] = 0x5be0cd19u;
}

// h <- compress(h, w).  w holds the block as sixteen big-endian words and is used
// as the rolling message schedule (its contents are gone afterwards).
__device__ __forceinline__ void sha256_compress(uint32_t (&h)[8], uint32_t (&w)[16]) {
    uint32_t s[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = h[i];
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        if (i >= 16) {
            const uint32_t x = w[(i + 1) & 15], y = w[(i + 14) & 15];
            w[i & 15] += sha_xor3(sha_rotr(x, 7), sha_rotr(x, 18), x >> 3) + w[(i + 9) & 15] +
                         sha_xor3(sha_rotr(y, 17), sha_rotr(y, 19), y >> 10);
        }
        const uint32_t t1 = s[7] + sha_xor3(sha_rotr(s[4], 6), sha_rotr(s[4], 11), sha_rotr(s[4], 25)) +
                            sha_ch(s[4], s[5], s[6]) + kShaK[i] + w[i & 15];
        const uint32_t t2 = sha_xor3(sha_rotr(s[0], 2), sha_rotr(s[0], 13), sha_rotr(s[0], 22)) + sha_maj(s[0], s[1], s[2]);
        s[7] = s[6]; s[6] = s[5]; s[5] = s[4]; s[4] = s[3] + t1;
        s[3] = s[2]; s[2] = s[1]; s[1] = s[0]; s[0] = t1 + t2;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] += s[i];
}

// The closing block of a message of `bytes` bytes that ended on a block boundary.
__device__ __forceinline__ void sha256_finish_aligned(uint32_t (&h)[8], uint64_t bytes) {
    uint32_t w[16];
    w[0] = 0x80000000u;
#pragma unroll
    for (int i = 1; i < 14; ++i) w[i] = 0;
    w[14] = (uint32_t)((bytes * 8) >> 32);
    w[15] = (uint32_t)(bytes * 8);
    sha256_compress(h, w);
}

}  // namespace zkmi
