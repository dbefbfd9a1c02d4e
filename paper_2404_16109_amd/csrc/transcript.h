// SHA-256 (FIPS 180-4) and the Fiat-Shamir transcript of the library, host side.
//
//   absorb(tag, data): state <- SHA256(state || tag || LE64(len) || data)
//   challenge(tag)   : c = (SHA256(state||tag||0) || SHA256(state||tag||1)) as a
//                      512-bit big-endian integer mod r;
//                      state <- SHA256(state || tag || 2)
#pragma once
#include <stdint.h>
#include <string.h>

#include <string>

#if defined(__x86_64__)
#include <immintrin.h>
#endif

#include "host_fr.h"

namespace zkmi {
namespace host {

class Sha256 {
public:
    Sha256() { reset(); }

    void reset() {
        static const uint32_t init[8] = {0x6a09e667u, 0xbb67ae85u, 0x3c6ef372u, 0xa54ff53au,
                                         0x510e527fu, 0x9b05688cu, 0x1f83d9abu, 0x5be0cd19u};
        memcpy(h_, init, sizeof h_);
        fill_ = 0;
        total_ = 0;
    }

    void update(const void* data, size_t len) {
        const uint8_t* p = (const uint8_t*)data;
        total_ += len;
        while (len) {
            size_t take = 64 - fill_;
            if (take > len) take = len;
            memcpy(buf_ + fill_, p, take);
            fill_ += take;
            p += take;
            len -= take;
            if (fill_ == 64) {
                block(buf_);
                fill_ = 0;
            }
        }
    }

    void finish(uint8_t out[32]) {
        const uint64_t bits = total_ * 8;
        buf_[fill_++] = 0x80;
        if (fill_ > 56) {
            memset(buf_ + fill_, 0, 64 - fill_);
            block(buf_);
            fill_ = 0;
        }
        memset(buf_ + fill_, 0, 56 - fill_);
        for (int i = 0; i < 8; ++i) buf_[56 + i] = (uint8_t)(bits >> (56 - 8 * i));
        block(buf_);
        fill_ = 0;
        for (int i = 0; i < 8; ++i) {
            out[4 * i] = (uint8_t)(h_[i] >> 24);
            out[4 * i + 1] = (uint8_t)(h_[i] >> 16);
            out[4 * i + 2] = (uint8_t)(h_[i] >> 8);
            out[4 * i + 3] = (uint8_t)h_[i];
        }
    }

    // Tests can switch the instruction-set path off to compare the two.
    static bool& use_sha_instructions() {
#if defined(__x86_64__)
        static bool on = __builtin_cpu_supports("sha") && __builtin_cpu_supports("sse4.1") && __builtin_cpu_supports("ssse3");
#else
        static bool on = false;
#endif
        return on;
    }

private:
    static uint32_t ror(uint32_t x, int n) { return (x >> n) | (x << (32 - n)); }

    static const uint32_t* round_constants() {
        static const uint32_t k[64] = {
            0x428a2f98u, 0x71374491u, 0xb5c0fbcfu, 0xe9b5dba5u, 0x3956c25bu, 0x59f111f1u, 0x923f82a4u, 0xab1c5ed5u,
            0xd807aa98u, 0x12835b01u, 0x243185beu, 0x550c7dc3u, 0x72be5d74u, 0x80deb1feu, 0x9bdc06a7u, 0xc19bf174u,
            0xe49b69c1u, 0xefbe4786u, 0x0fc19dc6u, 0x240ca1ccu, 0x2de92c6fu, 0x4a7484aau, 0x5cb0a9dcu, 0x76f988dau,
            0x983e5152u, 0xa831c66du, 0xb00327c8u, 0xbf597fc7u, 0xc6e00bf3u, 0xd5a79147u, 0x06ca6351u, 0x14292967u,
            0x27b70a85u, 0x2e1b2138u, 0x4d2c6dfcu, 0x53380d13u, 0x650a7354u, 0x766a0abbu, 0x81c2c92eu, 0x92722c85u,
            0xa2bfe8a1u, 0xa81a664bu, 0xc24b8b70u, 0xc76c51a3u, 0xd192e819u, 0xd6990624u, 0xf40e3585u, 0x106aa070u,
            0x19a4c116u, 0x1e376c08u, 0x2748774cu, 0x34b0bcb5u, 0x391c0cb3u, 0x4ed8aa4au, 0x5b9cca4fu, 0x682e6ff3u,
            0x748f82eeu, 0x78a5636fu, 0x84c87814u, 0x8cc70208u, 0x90befffau, 0xa4506cebu, 0xbef9a3f7u, 0xc67178f2u};
        return k;
    }

#if defined(__x86_64__)
    // One block with the x86 SHA extensions.  sha256rnds2 does two rounds on the
    // state split as (A,B,E,F) and (C,D,G,H), taking W+K of those rounds from the
    // low half of its third operand; sha256msg1/msg2 produce four schedule words
    // from the sixteen before them.
    __attribute__((target("sha,sse4.1,ssse3"))) void block_shani(const uint8_t* b) {
        const __m128i* kk = (const __m128i*)round_constants();
        const __m128i bswap = _mm_set_epi64x(0x0c0d0e0f08090a0bULL, 0x0405060700010203ULL);
        __m128i abcd = _mm_loadu_si128((const __m128i*)&h_[0]);  // lanes: a b c d (a lowest)
        __m128i efgh = _mm_loadu_si128((const __m128i*)&h_[4]);
        // -> (F,E,B,A) and (H,G,D,C), highest lane first, as the instruction expects
        __m128i t = _mm_shuffle_epi32(abcd, 0xB1);        // b a d c
        __m128i u = _mm_shuffle_epi32(efgh, 0x1B);        // h g f e
        __m128i abef = _mm_alignr_epi8(t, u, 8);          // f e b a   (lane0 = f)
        __m128i cdgh = _mm_blend_epi16(u, t, 0xF0);       // h g d c   (lane0 = h)
        const __m128i abef0 = abef, cdgh0 = cdgh;
        __m128i w[4];
        for (int i = 0; i < 4; ++i) w[i] = _mm_shuffle_epi8(_mm_loadu_si128((const __m128i*)(b + 16 * i)), bswap);
        for (int g = 0; g < 16; ++g) {  // four rounds per step
            __m128i cur;
            if (g < 4) {
                cur = w[g];
            } else {
                // W[4g..4g+3] from the four vectors before it
                __m128i x = _mm_sha256msg1_epu32(w[g & 3], w[(g + 1) & 3]);
                x = _mm_add_epi32(x, _mm_alignr_epi8(w[(g + 3) & 3], w[(g + 2) & 3], 4));
                cur = _mm_sha256msg2_epu32(x, w[(g + 3) & 3]);
                w[g & 3] = cur;
            }
            __m128i wk = _mm_add_epi32(cur, _mm_loadu_si128(kk + g));
            cdgh = _mm_sha256rnds2_epu32(cdgh, abef, wk);
            abef = _mm_sha256rnds2_epu32(abef, cdgh, _mm_shuffle_epi32(wk, 0x0E));
        }
        abef = _mm_add_epi32(abef, abef0);
        cdgh = _mm_add_epi32(cdgh, cdgh0);
        // back to a b c d / e f g h
        t = _mm_shuffle_epi32(abef, 0x1B);                // a b e f  (lane0 = a)
        u = _mm_shuffle_epi32(cdgh, 0xB1);                // g h c d  (lane0 = g)
        _mm_storeu_si128((__m128i*)&h_[0], _mm_blend_epi16(t, u, 0xF0));       // a b c d
        _mm_storeu_si128((__m128i*)&h_[4], _mm_alignr_epi8(u, t, 8));          // e f g h
    }
#endif

    void block(const uint8_t* b) {
#if defined(__x86_64__)
        if (use_sha_instructions()) {
            block_shani(b);
            return;
        }
#endif
        const uint32_t* k = round_constants();
        uint32_t w[16];
        for (int i = 0; i < 16; ++i)
            w[i] = ((uint32_t)b[4 * i] << 24) | ((uint32_t)b[4 * i + 1] << 16) | ((uint32_t)b[4 * i + 2] << 8) |
                   (uint32_t)b[4 * i + 3];
        uint32_t v[8];
        memcpy(v, h_, sizeof v);
        for (int i = 0; i < 64; ++i) {
            if (i >= 16) {
                uint32_t x = w[(i + 1) & 15], y = w[(i + 14) & 15];
                w[i & 15] += (ror(x, 7) ^ ror(x, 18) ^ (x >> 3)) + w[(i + 9) & 15] +
                             (ror(y, 17) ^ ror(y, 19) ^ (y >> 10));
            }
            uint32_t e = v[4], a = v[0];
            uint32_t t1 = v[7] + (ror(e, 6) ^ ror(e, 11) ^ ror(e, 25)) + ((e & v[5]) ^ (~e & v[6])) + k[i] + w[i & 15];
            uint32_t t2 = (ror(a, 2) ^ ror(a, 13) ^ ror(a, 22)) + ((a & v[1]) ^ (a & v[2]) ^ (v[1] & v[2]));
            v[7] = v[6]; v[6] = v[5]; v[5] = v[4]; v[4] = v[3] + t1;
            v[3] = v[2]; v[2] = v[1]; v[1] = v[0]; v[0] = t1 + t2;
        }
        for (int i = 0; i < 8; ++i) h_[i] += v[i];
    }

    uint32_t h_[8];
    uint8_t buf_[64];
    size_t fill_;
    uint64_t total_;
};

inline void put_le64(uint8_t out[8], uint64_t x) {
    for (int i = 0; i < 8; ++i) out[i] = (uint8_t)(x >> (8 * i));
}

inline uint64_t get_le64(const uint8_t in[8]) {
    uint64_t x = 0;
    for (int i = 0; i < 8; ++i) x |= (uint64_t)in[i] << (8 * i);
    return x;
}

class Transcript {
public:
    // state = SHA256(label || seed || LE64(dims[0]) || ...)
    // (more public parameters may follow the dimensions as raw bytes)
    Transcript(const char* label, const uint8_t seed[32], const uint64_t* dims, int ndims, const uint8_t* extra = nullptr,
               size_t extra_len = 0) {
        Sha256 h;
        h.update(label, strlen(label));
        h.update(seed, 32);
        for (int i = 0; i < ndims; ++i) {
            uint8_t le[8];
            put_le64(le, dims[i]);
            h.update(le, 8);
        }
        if (extra_len) h.update(extra, extra_len);
        h.finish(state_);
    }

    void absorb(const char* tag, const void* data, size_t len) {
        Sha256 h;
        uint8_t le[8];
        put_le64(le, len);
        h.update(state_, 32);
        h.update(tag, strlen(tag));
        h.update(le, 8);
        h.update(data, len);
        h.finish(state_);
    }

    void absorb_elements(const char* tag, const F* xs, int count) {
        uint8_t buf[32 * 8];
        for (int i = 0; i < count; ++i) to_bytes(buf + 32 * i, xs[i]);
        absorb(tag, buf, 32 * (size_t)count);
    }

    F challenge(const char* tag) {
        uint8_t wide[64], next[32];
        for (uint8_t which = 0; which < 3; ++which) {
            Sha256 h;
            h.update(state_, 32);
            h.update(tag, strlen(tag));
            h.update(&which, 1);
            h.finish(which == 0 ? wide : which == 1 ? wide + 32 : next);
        }
        memcpy(state_, next, 32);
        return from_be512(wide);
    }

private:
    uint8_t state_[32];
};

}  // namespace host
}  // namespace zkmi
