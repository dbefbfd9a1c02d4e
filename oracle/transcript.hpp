// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// Fiat-Shamir transcript.  The paper's protocols are interactive: the verifier
// sends beta (Protocol 1, tlookup-Prove, first step), alpha and u (Section 4,
// before the tlookup sumcheck equation) and one challenge per sumcheck round
// (Section 3.3).  Here every verifier message is replaced by a hash of all
// prover messages so far.  Rules (this build's own; the paper has none):
//
//   state            : 32 bytes
//   absorb(tag,data) : state <- SHA256(state || tag || LE64(len(data)) || data)
//   challenge(tag)   : h0 = SHA256(state || tag || 0x00)
//                      h1 = SHA256(state || tag || 0x01)
//                      c  = (h0 || h1 read as a 512-bit big-endian integer) mod r
//                      state <- SHA256(state || tag || 0x02)
#pragma once
#include "fr.hpp"
#include "sha256.hpp"

namespace oracle {

struct Transcript {
    uint8_t state[32];

    explicit Transcript(const Bytes& init) { init.digest(state); }

    void absorb(const char* tag, const uint8_t* data, size_t len) {
        Bytes b;
        b.raw(state, 32).str(tag).le64(len).raw(data, len);
        b.digest(state);
    }

    void absorb_fr(const char* tag, const Fr* xs, size_t count) {
        std::vector<uint8_t> buf(32 * count);
        for (size_t i = 0; i < count; ++i) fr_to_bytes(&buf[32 * i], xs[i]);
        absorb(tag, buf.data(), buf.size());
    }

    Fr challenge(const char* tag) {
        uint8_t wide[64], next[32];
        Bytes b0, b1, b2;
        b0.raw(state, 32).str(tag).byte(0x00);
        b1.raw(state, 32).str(tag).byte(0x01);
        b2.raw(state, 32).str(tag).byte(0x02);
        b0.digest(wide);
        b1.digest(wide + 32);
        b2.digest(next);
        memcpy(state, next, 32);
        return fr_from_be512(wide);
    }
};

}  // namespace oracle
