// Host build of the 29-bit-limb field arithmetic (csrc/fr29_dev.h) with a C
// interface, so that tests can compare it with Python's big integers.  Compiled
// with g++ by tests/test_fr29_host.py; nothing here runs on a GPU.
#include "../../paper_2404_16109_amd/csrc/fr29_dev.h"

using namespace zkmi;

extern "C" {
void c_unpack(const uint32_t* w, uint32_t* out) { F29 a = f29_unpack(w); for (int i = 0; i < 9; ++i) out[i] = a.l[i]; }
void c_pack(const uint32_t* l, uint32_t* w) { F29 a; for (int i = 0; i < 9; ++i) a.l[i] = l[i]; f29_pack(w, a); }
void c_normalize(const uint32_t* l, uint32_t* out) { F29 a; for (int i = 0; i < 9; ++i) a.l[i] = l[i]; a = f29_normalize(a); for (int i = 0; i < 9; ++i) out[i] = a.l[i]; }
void c_sub(const uint32_t* x, const uint32_t* y, uint32_t* out) {
    F29 a, b; for (int i = 0; i < 9; ++i) { a.l[i] = x[i]; b.l[i] = y[i]; }
    F29 o = f29_sub(a, b); for (int i = 0; i < 9; ++i) out[i] = o.l[i];
}
void c_sub_small(const uint32_t* x, const uint32_t* y, uint32_t* out) {
    F29 a, b; for (int i = 0; i < 9; ++i) { a.l[i] = x[i]; b.l[i] = y[i]; }
    F29 o = f29_sub_small(a, b); for (int i = 0; i < 9; ++i) out[i] = o.l[i];
}
void c_mul(const uint32_t* x, const uint32_t* y, uint32_t* out) {
    F29 a, b; for (int i = 0; i < 9; ++i) { a.l[i] = x[i]; b.l[i] = y[i]; }
    F29 o = f29_mul(a, b); for (int i = 0; i < 9; ++i) out[i] = o.l[i];
}
void c_wide_mac(uint32_t* w, const uint32_t* x, const uint32_t* y) {
    F29Wide W; F29 a, b;
    for (int i = 0; i < 18; ++i) W.l[i] = w[i];
    for (int i = 0; i < 9; ++i) { a.l[i] = x[i]; b.l[i] = y[i]; }
    f29_wide_mac(W, a, b);
    for (int i = 0; i < 18; ++i) w[i] = W.l[i];
}
void c_wide_normalize(uint32_t* w) { F29Wide W; for (int i = 0; i < 18; ++i) W.l[i] = w[i]; f29_wide_normalize(W); for (int i = 0; i < 18; ++i) w[i] = W.l[i]; }
void c_wide_reduce(const uint32_t* w, uint32_t* out) { F29Wide W; for (int i = 0; i < 18; ++i) W.l[i] = w[i]; F29 o = f29_wide_reduce(W); for (int i = 0; i < 9; ++i) out[i] = o.l[i]; }
void c_canonical(const uint32_t* l, uint32_t* w) { F29 a; for (int i = 0; i < 9; ++i) a.l[i] = l[i]; f29_canonical(w, a); }
void c_canonical_big(const uint32_t* l, uint32_t* w) { F29 a; for (int i = 0; i < 9; ++i) a.l[i] = l[i]; f29_canonical_big(w, a); }
}
