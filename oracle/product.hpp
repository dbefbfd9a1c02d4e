// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// Product sumcheck and the matrix-multiplication proof of Section 6.1.1:
//
//   C~(u, v) = sum_{k in {0,1}^ceil(log2 n)} A~(u, k) B~(k, v)
//
// for C = A B with A of shape D0 x D1 and B of shape D1 x D2; every dimension is
// zero-padded to a power of two (Section 3.3), u and v come from the
// transcript.  The prover forms a_k = A~(u, k) and b_k = B~(k, v) and runs the
// generic sumcheck (Section 3.3) on sum_k a_k b_k.  A round polynomial has
// degree <= 2 and is sent as its values at X = 0, 1, 2; variables are bound in
// written order (top index bit first).
//
// Proof bytes, product sumcheck:
//   "ZKSP" | u32 version=1 | LE64 d | claim | d x [g(0) g(1) g(2)] | a~(r) b~(r)
// matmul:
//   "ZKMM" | u32 version=1 | LE64 D0 | LE64 D1 | LE64 D2 | claim
//          | d x [g(0) g(1) g(2)] | A~(u,r) B~(r,v)
#pragma once
#include "tlookup.hpp"

namespace oracle {

inline int ceil_log2(uint64_t v) {
    int n = 0;
    while (((uint64_t)1 << n) < v) ++n;
    return n;
}

inline size_t product_proof_bytes(int d) { return 16 + 32 + (size_t)d * 96 + 64; }
inline size_t matmul_proof_bytes(int d) { return 32 + 32 + (size_t)d * 96 + 64; }

// Rounds of sum_x a(x) b(x) = claim on an existing transcript (the claim is
// already absorbed).  Writes d x 3 round values and the two final values to
// `out`; returns the challenges in r_out.
inline void product_rounds(Transcript& tr, std::vector<Fr> a, std::vector<Fr> b, uint8_t* out, Fr* r_out,
                           int threads) {
    int d = log2_exact(a.size());
    int workers = std::max(1, threads);
    for (int k = 0; k < d; ++k) {
        size_t half = a.size() / 2;
        std::vector<std::array<Fr, 3>> partial(workers);
        for (auto& p : partial) p = {fr_zero(), fr_zero(), fr_zero()};
        parallel_ranges(half, workers, [&](size_t lo, size_t hi, int w) {
            std::array<Fr, 3> acc = {fr_zero(), fr_zero(), fr_zero()};
            for (size_t p = lo; p < hi; ++p) {
                Fr x = a[p], dx = fr_sub(a[p + half], a[p]);
                Fr y = b[p], dy = fr_sub(b[p + half], b[p]);
                for (int X = 0; X < 3; ++X) {
                    acc[X] = fr_add(acc[X], fr_mul(x, y));
                    x = fr_add(x, dx);
                    y = fr_add(y, dy);
                }
            }
            partial[w] = acc;
        });
        Fr g[3] = {fr_zero(), fr_zero(), fr_zero()};
        for (auto& p : partial)
            for (int X = 0; X < 3; ++X) g[X] = fr_add(g[X], p[X]);
        for (int X = 0; X < 3; ++X) fr_to_bytes(out + 32 * X, g[X]);
        out += 96;
        tr.absorb_fr("g", g, 3);
        Fr r = tr.challenge("r");
        if (r_out) r_out[k] = r;
        fold_top(a, r, threads);
        fold_top(b, r, threads);
    }
    Fr fin[2] = {a[0], b[0]};
    fr_to_bytes(out, fin[0]);
    fr_to_bytes(out + 32, fin[1]);
    tr.absorb_fr("final", fin, 2);
}

// Checks d rounds against `claim`; leaves the challenges in r and the final
// claim value in *last.  Returns false on a failed consistency check.
inline bool product_rounds_check(Transcript& tr, const Fr* el, int d, Fr claim, Fr* r, Fr* last) {
    for (int k = 0; k < d; ++k) {
        const Fr* g = el + 3 * k;
        if (!fr_eq(fr_add(g[0], g[1]), claim)) return false;
        tr.absorb_fr("g", g, 3);
        r[k] = tr.challenge("r");
        claim = lagrange_eval(g, 3, r[k]);
    }
    *last = claim;
    return true;
}

inline int sumcheck_prove_product(const uint8_t seed[32], const Fr* a, const Fr* b, uint64_t n, const Fr* claim,
                                  uint8_t* proof, uint64_t cap, uint64_t* len, Fr* r_out, int threads) {
    int d = log2_exact(n);
    if (!seed || !a || !b || !claim || d < 0) return E_BADARG;
    size_t need = product_proof_bytes(d);
    if (len) *len = need;
    if (!proof || cap < need) return E_BUFSZ;
    Bytes init;
    init.str("zkmi/sumcheck-product/v1").raw(seed, 32).le64((uint64_t)d);
    Transcript tr(init);
    tr.absorb_fr("claim", claim, 1);
    memcpy(proof, "ZKSP", 4);
    proof[4] = 1; proof[5] = proof[6] = proof[7] = 0;
    for (int i = 0; i < 8; ++i) proof[8 + i] = (uint8_t)((uint64_t)d >> (8 * i));
    fr_to_bytes(proof + 16, *claim);
    product_rounds(tr, std::vector<Fr>(a, a + n), std::vector<Fr>(b, b + n), proof + 48, r_out, threads);
    return OK;
}

// Accepts iff the rounds are consistent and the last claim equals a~(r) b~(r)
// as stated in the proof; if a and b are given, those two values are recomputed.
inline int sumcheck_verify_product(const uint8_t seed[32], const uint8_t* proof, uint64_t len, uint64_t n,
                                   const Fr* a, const Fr* b, Fr* r_out, int threads) {
    int d = log2_exact(n);
    if (!seed || !proof || d < 0) return E_BADARG;
    if (len != product_proof_bytes(d) || memcmp(proof, "ZKSP\x01\0\0\0", 8) != 0) return E_REJECT;
    uint64_t dp = 0;
    for (int i = 0; i < 8; ++i) dp |= (uint64_t)proof[8 + i] << (8 * i);
    if (dp != (uint64_t)d) return E_REJECT;
    size_t nfr = 1 + 3 * (size_t)d + 2;
    std::vector<Fr> el(nfr);
    for (size_t i = 0; i < nfr; ++i) {
        el[i] = fr_from_bytes(proof + 16 + 32 * i);
        if (!fr_is_canonical(el[i])) return E_REJECT;
    }
    Bytes init;
    init.str("zkmi/sumcheck-product/v1").raw(seed, 32).le64((uint64_t)d);
    Transcript tr(init);
    tr.absorb_fr("claim", &el[0], 1);
    std::vector<Fr> r(d);
    Fr last;
    if (!product_rounds_check(tr, &el[1], d, el[0], r.data(), &last)) return E_REJECT;
    const Fr* fin = &el[1 + 3 * d];
    if (!fr_eq(fr_mul(fin[0], fin[1]), last)) return E_REJECT;
    if (a && !fr_eq(mle_eval(a, d, r.data(), threads), fin[0])) return E_REJECT;
    if (b && !fr_eq(mle_eval(b, d, r.data(), threads), fin[1])) return E_REJECT;
    if (r_out) for (int k = 0; k < d; ++k) r_out[k] = r[k];
    return OK;
}

inline Transcript matmul_transcript(const uint8_t seed[32], uint64_t D0, uint64_t D1, uint64_t D2) {
    Bytes init;
    init.str("zkmi/matmul/v1").raw(seed, 32).le64(D0).le64(D1).le64(D2);
    return Transcript(init);
}

// X: D0 x D1 row-major, W: D1 x D2 row-major, small signed integers embedded
// in the field by the caller's choice of representation (here: int64 values).
inline int matmul_sumcheck_prove(const uint8_t seed[32], const int64_t* X, uint64_t D0, uint64_t D1,
                                 const int64_t* W, uint64_t D2, uint8_t* proof, uint64_t cap, uint64_t* len,
                                 Fr* u_out, Fr* v_out, Fr* r_out, int threads) {
    if (!seed || !X || !W || D0 == 0 || D1 == 0 || D2 == 0) return E_BADARG;
    int n0 = ceil_log2(D0), n1 = ceil_log2(D1), n2 = ceil_log2(D2);
    size_t need = matmul_proof_bytes(n1);
    if (len) *len = need;
    if (!proof || cap < need) return E_BUFSZ;
    Transcript tr = matmul_transcript(seed, D0, D1, D2);
    std::vector<Fr> u(n0), v(n2);
    for (int t = 0; t < n0; ++t) u[t] = tr.challenge("u");
    for (int t = 0; t < n2; ++t) v[t] = tr.challenge("v");
    if (u_out) for (int t = 0; t < n0; ++t) u_out[t] = u[t];
    if (v_out) for (int t = 0; t < n2; ++t) v_out[t] = v[t];

    // a_k = sum_i e~(u, i) X[i, k];  b_k = sum_j W[k, j] e~(v, j); padded rows
    // and columns are zero and contribute nothing.
    std::vector<Fr> eu = eq_table(u.data(), n0, threads), ev = eq_table(v.data(), n2, threads);
    size_t P1 = (size_t)1 << n1;
    std::vector<Fr> a(P1, fr_zero()), b(P1, fr_zero());
    parallel_ranges(D1, threads, [&](size_t lo, size_t hi, int) {
        for (size_t k = lo; k < hi; ++k) {
            Fr sa = fr_zero(), sb = fr_zero();
            for (uint64_t i = 0; i < D0; ++i) sa = fr_add(sa, fr_mul(eu[i], fr_from_i64(X[i * D1 + k])));
            for (uint64_t j = 0; j < D2; ++j) sb = fr_add(sb, fr_mul(fr_from_i64(W[k * D2 + j]), ev[j]));
            a[k] = sa;
            b[k] = sb;
        }
    });
    Fr claim = fr_zero();
    for (size_t k = 0; k < P1; ++k) claim = fr_add(claim, fr_mul(a[k], b[k]));
    tr.absorb_fr("claim", &claim, 1);

    memcpy(proof, "ZKMM", 4);
    proof[4] = 1; proof[5] = proof[6] = proof[7] = 0;
    for (int i = 0; i < 8; ++i) {
        proof[8 + i] = (uint8_t)(D0 >> (8 * i));
        proof[16 + i] = (uint8_t)(D1 >> (8 * i));
        proof[24 + i] = (uint8_t)(D2 >> (8 * i));
    }
    fr_to_bytes(proof + 32, claim);
    product_rounds(tr, a, b, proof + 64, r_out, threads);
    return OK;
}

// Verifier for the matmul proof.  If Y (D0 x D2, the claimed product, int64 as
// field embeddings given by the caller in canonical form) is supplied, the
// claim is checked against Y~(u, v); if X and W are supplied, the two final
// values are recomputed from them.
inline int matmul_sumcheck_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, uint64_t D0,
                                  uint64_t D1, uint64_t D2, const Fr* Y, const int64_t* X, const int64_t* W,
                                  int threads) {
    if (!seed || !proof || D0 == 0 || D1 == 0 || D2 == 0) return E_BADARG;
    int n0 = ceil_log2(D0), n1 = ceil_log2(D1), n2 = ceil_log2(D2);
    if (len != matmul_proof_bytes(n1) || memcmp(proof, "ZKMM\x01\0\0\0", 8) != 0) return E_REJECT;
    uint64_t dims[3] = {0, 0, 0};
    for (int q = 0; q < 3; ++q)
        for (int i = 0; i < 8; ++i) dims[q] |= (uint64_t)proof[8 + 8 * q + i] << (8 * i);
    if (dims[0] != D0 || dims[1] != D1 || dims[2] != D2) return E_REJECT;
    size_t nfr = 1 + 3 * (size_t)n1 + 2;
    std::vector<Fr> el(nfr);
    for (size_t i = 0; i < nfr; ++i) {
        el[i] = fr_from_bytes(proof + 32 + 32 * i);
        if (!fr_is_canonical(el[i])) return E_REJECT;
    }
    Transcript tr = matmul_transcript(seed, D0, D1, D2);
    std::vector<Fr> u(n0), v(n2), r(n1);
    for (int t = 0; t < n0; ++t) u[t] = tr.challenge("u");
    for (int t = 0; t < n2; ++t) v[t] = tr.challenge("v");
    tr.absorb_fr("claim", &el[0], 1);
    Fr last;
    if (!product_rounds_check(tr, &el[1], n1, el[0], r.data(), &last)) return E_REJECT;
    const Fr* fin = &el[1 + 3 * n1];
    if (!fr_eq(fr_mul(fin[0], fin[1]), last)) return E_REJECT;

    std::vector<Fr> eu = eq_table(u.data(), n0, threads), ev = eq_table(v.data(), n2, threads);
    if (Y) {
        Fr y = fr_zero();
        for (uint64_t i = 0; i < D0; ++i)
            for (uint64_t j = 0; j < D2; ++j) y = fr_add(y, fr_mul(fr_mul(eu[i], ev[j]), Y[i * D2 + j]));
        if (!fr_eq(y, el[0])) return E_REJECT;
    }
    if (X || W) {
        std::vector<Fr> er = eq_table(r.data(), n1, threads);
        if (X) {
            Fr x = fr_zero();
            for (uint64_t i = 0; i < D0; ++i)
                for (uint64_t k = 0; k < D1; ++k)
                    x = fr_add(x, fr_mul(fr_mul(eu[i], er[k]), fr_from_i64(X[i * D1 + k])));
            if (!fr_eq(x, fin[0])) return E_REJECT;
        }
        if (W) {
            Fr w = fr_zero();
            for (uint64_t k = 0; k < D1; ++k)
                for (uint64_t j = 0; j < D2; ++j)
                    w = fr_add(w, fr_mul(fr_mul(er[k], ev[j]), fr_from_i64(W[k * D2 + j])));
            if (!fr_eq(w, fin[1])) return E_REJECT;
        }
    }
    return OK;
}

}  // namespace oracle
