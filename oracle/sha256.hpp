// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// SHA-256 written from FIPS 180-4 (sections 4.1.2, 4.2.2, 5.1.1, 5.3.3, 6.2),
// one-shot interface over a byte string.  The round constants are derived at
// start-up from their definition (first 32 bits of the fractional parts of the
// cube roots of the first 64 primes; square roots of the first 8 primes for
// the initial hash value) with exact integer root extraction, not typed in.
#pragma once
#include <cstdint>
#include <cstring>
#include <string>
#include <vector>

namespace oracle {

struct Sha256Tables {
    uint32_t K[64];
    uint32_t H0[8];

    // floor( frac( p^(1/root) ) * 2^32 ) by binary search on integers:
    // the largest y with y^root <= p * 2^(32*root).
    static uint32_t frac_root(unsigned p, int root) {
        typedef unsigned __int128 u128;
        // y < 2^32 * p^(1/root) <= 2^32 * 18 for p <= 311, so y fits in 37 bits
        // and y^3 in 111 bits.
        u128 target = (u128)p << (32 * root);
        uint64_t lo = 0, hi = (uint64_t)1 << 37;
        while (hi - lo > 1) {
            uint64_t mid = lo + (hi - lo) / 2;
            u128 v = (u128)mid * mid;
            if (root == 3) v *= mid;
            if (v <= target) lo = mid; else hi = mid;
        }
        return (uint32_t)lo;  // low 32 bits = the fractional part
    }

    Sha256Tables() {
        unsigned primes[64];
        int n = 0;
        for (unsigned c = 2; n < 64; ++c) {
            bool is_prime = true;
            for (unsigned d = 2; d * d <= c; ++d)
                if (c % d == 0) { is_prime = false; break; }
            if (is_prime) primes[n++] = c;
        }
        for (int i = 0; i < 64; ++i) K[i] = frac_root(primes[i], 3);
        for (int i = 0; i < 8; ++i) H0[i] = frac_root(primes[i], 2);
    }
};

inline const Sha256Tables& sha256_tables() {
    static const Sha256Tables t;
    return t;
}

inline uint32_t rotr32(uint32_t x, int n) { return (x >> n) | (x << (32 - n)); }

inline void sha256_compress(uint32_t h[8], const uint8_t block[64]) {
    const uint32_t* K = sha256_tables().K;
    uint32_t w[64];
    for (int t = 0; t < 16; ++t)
        w[t] = ((uint32_t)block[4 * t] << 24) | ((uint32_t)block[4 * t + 1] << 16) |
               ((uint32_t)block[4 * t + 2] << 8) | (uint32_t)block[4 * t + 3];
    for (int t = 16; t < 64; ++t) {
        uint32_t s0 = rotr32(w[t - 15], 7) ^ rotr32(w[t - 15], 18) ^ (w[t - 15] >> 3);
        uint32_t s1 = rotr32(w[t - 2], 17) ^ rotr32(w[t - 2], 19) ^ (w[t - 2] >> 10);
        w[t] = s1 + w[t - 7] + s0 + w[t - 16];
    }
    uint32_t a = h[0], b = h[1], c = h[2], d = h[3], e = h[4], f = h[5], g = h[6], hh = h[7];
    for (int t = 0; t < 64; ++t) {
        uint32_t S1 = rotr32(e, 6) ^ rotr32(e, 11) ^ rotr32(e, 25);
        uint32_t ch = (e & f) ^ (~e & g);
        uint32_t t1 = hh + S1 + ch + K[t] + w[t];
        uint32_t S0 = rotr32(a, 2) ^ rotr32(a, 13) ^ rotr32(a, 22);
        uint32_t maj = (a & b) ^ (a & c) ^ (b & c);
        uint32_t t2 = S0 + maj;
        hh = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
    }
    h[0] += a; h[1] += b; h[2] += c; h[3] += d; h[4] += e; h[5] += f; h[6] += g; h[7] += hh;
}

inline void sha256(uint8_t out[32], const uint8_t* data, size_t len) {
    uint32_t h[8];
    memcpy(h, sha256_tables().H0, sizeof h);
    size_t full = len / 64;
    for (size_t i = 0; i < full; ++i) sha256_compress(h, data + 64 * i);
    uint8_t tail[128];
    size_t rem = len - 64 * full;
    memset(tail, 0, sizeof tail);
    if (rem) memcpy(tail, data + 64 * full, rem);
    tail[rem] = 0x80;
    size_t tail_len = (rem + 1 + 8 <= 64) ? 64 : 128;
    uint64_t bits = (uint64_t)len * 8;
    for (int i = 0; i < 8; ++i) tail[tail_len - 1 - i] = (uint8_t)(bits >> (8 * i));
    sha256_compress(h, tail);
    if (tail_len == 128) sha256_compress(h, tail + 64);
    for (int i = 0; i < 8; ++i) {
        out[4 * i] = (uint8_t)(h[i] >> 24);
        out[4 * i + 1] = (uint8_t)(h[i] >> 16);
        out[4 * i + 2] = (uint8_t)(h[i] >> 8);
        out[4 * i + 3] = (uint8_t)h[i];
    }
}

// Byte-string builder for hash inputs.
struct Bytes {
    std::vector<uint8_t> v;
    Bytes& raw(const void* p, size_t n) {
        const uint8_t* b = (const uint8_t*)p;
        v.insert(v.end(), b, b + n);
        return *this;
    }
    Bytes& str(const char* s) { return raw(s, strlen(s)); }
    Bytes& le64(uint64_t x) {
        for (int i = 0; i < 8; ++i) v.push_back((uint8_t)(x >> (8 * i)));
        return *this;
    }
    Bytes& byte(uint8_t b) { v.push_back(b); return *this; }
    void digest(uint8_t out[32]) const { sha256(out, v.data(), v.size()); }
};

}  // namespace oracle
