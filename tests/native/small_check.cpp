// Host build of the small-integer arithmetic of the device library
// (csrc/small_dev.h) with a C interface, so that tests can compare it with
// Python's big integers.  Compiled with g++ by tests/test_small_host.py; nothing
// here runs on a GPU.
#include "../../paper_2404_16109_amd/csrc/small_dev.h"

using namespace zkmi;

extern "C" {
void c_mac32(uint32_t* t11, const uint32_t* c, uint32_t m) {
    uint32_t t[11], k[8];
    for (int i = 0; i < 11; ++i) t[i] = t11[i];
    for (int i = 0; i < 8; ++i) k[i] = c[i];
    small_mac32(t, k, m);
    for (int i = 0; i < 11; ++i) t11[i] = t[i];
}
void c_mac64(uint32_t* t11, const uint32_t* c, uint64_t m) {
    uint32_t t[11], k[8];
    for (int i = 0; i < 11; ++i) t[i] = t11[i];
    for (int i = 0; i < 8; ++i) k[i] = c[i];
    small_mac64(t, k, m);
    for (int i = 0; i < 11; ++i) t11[i] = t[i];
}
void c_reduce2(const uint32_t* t11, uint32_t* out) {
    uint32_t t[11], o[8];
    for (int i = 0; i < 11; ++i) t[i] = t11[i];
    small_reduce<2>(o, t);
    for (int i = 0; i < 8; ++i) out[i] = o[i];
}
void c_reduce3(const uint32_t* t12, uint32_t* out) {
    uint32_t t[12], o[8];
    for (int i = 0; i < 12; ++i) t[i] = t12[i];
    small_reduce<3>(o, t);
    for (int i = 0; i < 8; ++i) out[i] = o[i];
}
static SmallFoldConsts consts_of(const uint32_t* k32) {
    SmallFoldConsts k;
    for (int i = 0; i < 8; ++i) {
        k.plus_a[i] = k32[i];
        k.minus_a[i] = k32[8 + i];
        k.plus_d[i] = k32[16 + i];
        k.minus_d[i] = k32[24 + i];
    }
    return k;
}
void c_fold64(int64_t a, int64_t b, const uint32_t* k32, uint32_t* out) {
    uint32_t o[8];
    small_fold64(o, a, b, consts_of(k32));
    for (int i = 0; i < 8; ++i) out[i] = o[i];
}
void c_combine32(int32_t x, int32_t y, const uint32_t* k32, uint32_t* out) {
    SmallSource k;
    k.x = nullptr; k.y = nullptr;
    for (int i = 0; i < 8; ++i) {
        k.plus_one[i] = k32[i]; k.minus_one[i] = k32[8 + i]; k.plus_rho[i] = k32[16 + i]; k.minus_rho[i] = k32[24 + i];
    }
    uint32_t o[8];
    small_combine32(o, x, y, k);
    for (int i = 0; i < 8; ++i) out[i] = o[i];
}
void c_fold_combined(int32_t x0, int32_t y0, int32_t x1, int32_t y1, const uint32_t* k64, uint32_t* out) {
    SmallFold4 k;
    uint32_t* dst[8] = {k.plus_one, k.minus_one, k.plus_c, k.minus_c, k.plus_rho, k.minus_rho, k.plus_rho_c, k.minus_rho_c};
    for (int q = 0; q < 8; ++q)
        for (int i = 0; i < 8; ++i) dst[q][i] = k64[8 * q + i];
    uint32_t o[8];
    small_fold_combined(o, x0, y0, x1, y1, k);
    for (int i = 0; i < 8; ++i) out[i] = o[i];
}
void c_fold32(uint32_t a, uint32_t b, const uint32_t* k32, uint32_t* out) {
    uint32_t o[8];
    small_fold32(o, a, b, consts_of(k32));
    for (int i = 0; i < 8; ++i) out[i] = o[i];
}
}
