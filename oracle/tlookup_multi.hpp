// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// Several tlookup instances of ANY shapes proved by ONE sumcheck, so that all
// their claims end at one point.  The paper proves each lookup on its own and
// says nothing of this; it is this build's reading of layers that look one tensor
// up in two tables of different lengths in a row (LayerNorm, Section 6.1.3).
//
// Instance k has D_k = 2^n_k entries against N_k = 2^l_k rows.  The sumcheck runs
// over n = max_k n_k variables; instance k lives on the LAST n_k of them
// (skip_k = n - n_k) and its summand does not depend on the first skip_k:
//   f(x) = sum_k lambda^k 2^-skip_k f_k(x_[skip_k:]),
// f_k the tlookup summand (Section 4, second form of the identity) built with
// u_[skip_k:].  Summed over the cube that is sum_k lambda^k (alpha + alpha^2), as
// for instances of one shape.  A round that binds one of the first skip_k
// variables sees instance k as a constant; from round skip_k on its arrays are
// folded as in a proof of its own, with the shared challenges.  The final claims
// of instance k are at v_[skip_k:] (table side: v_[skip_k + h_k:]).
//
// Transcript: SHA256("zkmi/tlookup-multi/v1" || seed || LE64 K || K x (LE64 D_k, LE64 N_k));
// then as for one shape: absorb("m", digest(m_k)) for all k; beta; absorb("A", .),
// absorb("B", .) for all k; alpha; u_0..u_{n-1}; lambda; per round absorb("g", 4
// values), r = challenge("r"); absorb("final", K x 5 claims).
//
// Proof bytes: "ZKTM" | u32 version=1 | LE64 K | K x (LE64 D_k, LE64 N_k) | K x digest(m_k)
//              | K x [digest(A_k) digest(B_k)] | n x [g(0) g(1) g(2) g(3)]
//              | K x [A~ S~ B~ m~ T~].
#pragma once
#include "tlookup_batch.hpp"

namespace oracle {

inline size_t tlookup_multi_proof_bytes(int n_max, uint64_t K) { return 16 + 16 * K + 96 * K + (size_t)n_max * 128 + 160 * K; }

inline Transcript tlookup_multi_transcript(const uint8_t seed[32], const uint64_t* D, const uint64_t* N, uint64_t K) {
    Bytes init;
    init.str("zkmi/tlookup-multi/v1").raw(seed, 32).le64(K);
    for (uint64_t k = 0; k < K; ++k) init.le64(D[k]).le64(N[k]);
    return Transcript(init);
}

struct MultiShape {
    int n = 0, l = 0, h = 0, skip = 0;
};

// n_max, and per instance its shape; false if some shape is not allowed.
inline bool tlookup_multi_shapes(const uint64_t* D, const uint64_t* N, uint64_t K, std::vector<MultiShape>& sh, int& n_max) {
    if (!D || !N || K == 0 || K > 8) return false;
    sh.assign(K, MultiShape());
    n_max = 0;
    for (uint64_t k = 0; k < K; ++k) {
        sh[k].n = log2_exact(D[k]);
        sh[k].l = log2_exact(N[k]);
        if (sh[k].n < 0 || sh[k].l < 0 || N[k] > D[k] || D[k] > ((uint64_t)1 << 31)) return false;
        sh[k].h = sh[k].n - sh[k].l;
        n_max = std::max(n_max, sh[k].n);
    }
    for (uint64_t k = 0; k < K; ++k) sh[k].skip = n_max - sh[k].n;
    return true;
}

// S_in[k]: D[k] elements, T_in[k]: N[k] elements.  aux_out (may be null): beta,
// alpha, lambda, then per instance sum_A, sum_mB.  v_out: n_max challenges.
inline int tlookup_multi_prove(const uint8_t seed[32], const Fr* const* S_in, const Fr* const* T_in, uint64_t K,
                               const uint64_t* D, const uint64_t* N, uint8_t* proof, uint64_t cap, uint64_t* len,
                               Fr* aux_out, Fr* v_out, uint64_t* bad_instance, uint64_t* bad_index, int threads) {
    std::vector<MultiShape> sh;
    int n = 0;
    if (!seed || !S_in || !T_in || !tlookup_multi_shapes(D, N, K, sh, n)) return E_BADARG;
    size_t need = tlookup_multi_proof_bytes(n, K);
    if (len) *len = need;
    if (!proof || cap < need) return E_BUFSZ;

    std::vector<BatchInstance> inst(K);
    Transcript tr = tlookup_multi_transcript(seed, D, N, K);
    uint8_t* out = proof;
    memcpy(out, "ZKTM", 4);
    out[4] = 1; out[5] = out[6] = out[7] = 0;
    for (int i = 0; i < 8; ++i) out[8 + i] = (uint8_t)(K >> (8 * i));
    out += 16;
    for (uint64_t k = 0; k < K; ++k) {
        for (int i = 0; i < 8; ++i) {
            out[i] = (uint8_t)(D[k] >> (8 * i));
            out[8 + i] = (uint8_t)(N[k] >> (8 * i));
        }
        out += 16;
    }
    for (uint64_t k = 0; k < K; ++k) {
        int rc = multiplicities(S_in[k], D[k], T_in[k], N[k], inst[k].counts, bad_index, threads);
        if (rc != OK) {
            if (bad_instance) *bad_instance = k;
            return rc;
        }
        uint8_t md[32];
        m_digest(md, inst[k].counts);
        tr.absorb("m", md, 32);
        memcpy(out, md, 32);
        out += 32;
    }

    Fr beta = tr.challenge("beta");
    for (uint64_t k = 0; k < K; ++k) {
        BatchInstance& I = inst[k];
        I.S.assign(S_in[k], S_in[k] + D[k]);
        I.T.assign(T_in[k], T_in[k] + N[k]);
        I.A.resize(D[k]);
        I.B.resize(N[k]);
        I.M.resize(N[k]);
        for (uint64_t j = 0; j < N[k]; ++j) {
            Fr den = fr_add(beta, I.T[j]);
            if (fr_is_zero(den)) return E_ZERO_DENOM;
            I.B[j] = fr_inv(den);
            I.M[j] = fr_from_u64(I.counts[j]);
        }
        std::vector<int> zero_seen(std::max(1, threads), 0);
        parallel_ranges(D[k], threads, [&](size_t lo, size_t hi, int w) {
            for (size_t i = lo; i < hi; ++i) {
                Fr den = fr_add(beta, I.S[i]);
                if (fr_is_zero(den)) { zero_seen[w] = 1; return; }
                I.A[i] = fr_inv(den);
            }
        });
        for (int z : zero_seen) if (z) return E_ZERO_DENOM;
    }
    for (uint64_t k = 0; k < K; ++k) {
        uint8_t dA[32], dB[32];
        vec_digest(dA, inst[k].A.data(), D[k], threads);
        vec_digest(dB, inst[k].B.data(), N[k], threads);
        tr.absorb("A", dA, 32);
        tr.absorb("B", dB, 32);
        memcpy(out, dA, 32);
        memcpy(out + 32, dB, 32);
        out += 64;
    }

    Fr alpha = tr.challenge("alpha");
    Fr alpha2 = fr_mul(alpha, alpha);
    std::vector<Fr> u(n);
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");
    Fr lambda = tr.challenge("lambda");
    // weight of instance k: lambda^k 2^-skip_k
    std::vector<Fr> weight(K);
    {
        Fr lam = fr_one();
        for (uint64_t k = 0; k < K; ++k) {
            weight[k] = fr_mul(lam, fr_two_inv_pow((unsigned)sh[k].skip));
            lam = fr_mul(lam, lambda);
        }
    }
    if (aux_out) {
        aux_out[0] = beta;
        aux_out[1] = alpha;
        aux_out[2] = lambda;
        for (uint64_t k = 0; k < K; ++k) {
            Fr sA = fr_zero(), sMB = fr_zero();
            for (uint64_t i = 0; i < D[k]; ++i) sA = fr_add(sA, inst[k].A[i]);
            for (uint64_t j = 0; j < N[k]; ++j) sMB = fr_add(sMB, fr_mul(inst[k].M[j], inst[k].B[j]));
            aux_out[3 + 2 * k] = sA;
            aux_out[4 + 2 * k] = sMB;
        }
    }

    // per instance: e~(u_[skip:], .) over its data indices, e~(u_[skip+h:], .) over its rows
    std::vector<std::vector<Fr>> E(K), Et(K);
    std::vector<Fr> scale(K);
    for (uint64_t k = 0; k < K; ++k) {
        E[k] = eq_table(u.data() + sh[k].skip, sh[k].n, threads);
        Et[k] = eq_table(u.data() + sh[k].skip + sh[k].h, sh[k].l, threads);
        scale[k] = fr_two_inv_pow((unsigned)sh[k].h);
    }

    for (int round = 0; round < n; ++round) {
        const size_t half = (size_t)1 << (n - round - 1);  // pairs of the whole cube in this round
        Fr g[4] = {fr_zero(), fr_zero(), fr_zero(), fr_zero()};
        for (uint64_t k = 0; k < K; ++k) {
            const BatchInstance& I = inst[k];
            const bool mine = round >= sh[k].skip;                  // the variable is one of instance k's
            const bool table_bound = round >= sh[k].skip + sh[k].h;  // ... and one of its table's
            const size_t size = I.A.size();                          // current length of the data arrays
            const size_t rows = I.B.size();                          // current length of the table arrays
            Fr acc[4] = {fr_zero(), fr_zero(), fr_zero(), fr_zero()};
            for (size_t p = 0; p < half; ++p) {
                // the pair (p, p + half) of the cube, seen by instance k: both entries are entry p mod size of its
                // arrays while the variable is not its own, entries q and q + size/2 afterwards
                const size_t q = mine ? p : p % size;
                const size_t step = mine ? size / 2 : 0;
                const size_t j = table_bound ? q : q % rows;
                const size_t jstep = table_bound ? rows / 2 : 0;
                Fr a = I.A[q], da = fr_sub(I.A[q + step], a);
                Fr s = I.S[q], ds = fr_sub(I.S[q + step], s);
                Fr e = E[k][q], de = fr_sub(E[k][q + step], e);
                Fr b = I.B[j], db = fr_sub(I.B[j + jstep], b);
                Fr t = I.T[j], dt = fr_sub(I.T[j + jstep], t);
                Fr mm = I.M[j], dm = fr_sub(I.M[j + jstep], mm);
                Fr et = Et[k][j], det = fr_sub(Et[k][j + jstep], et);
                for (int X = 0; X < 4; ++X) {
                    acc[X] = fr_add(acc[X], tlookup_summand(a, s, e, b, t, et, mm, alpha, alpha2, beta, scale[k]));
                    a = fr_add(a, da); s = fr_add(s, ds); e = fr_add(e, de);
                    b = fr_add(b, db); t = fr_add(t, dt); et = fr_add(et, det); mm = fr_add(mm, dm);
                }
            }
            for (int X = 0; X < 4; ++X) g[X] = fr_add(g[X], fr_mul(weight[k], acc[X]));
        }
        for (int X = 0; X < 4; ++X) fr_to_bytes(out + 32 * X, g[X]);
        out += 128;
        tr.absorb_fr("g", g, 4);
        Fr r = tr.challenge("r");
        if (v_out) v_out[round] = r;
        for (uint64_t k = 0; k < K; ++k) {
            if (round < sh[k].skip) continue;
            fold_top(E[k], r, threads);
            fold_top(inst[k].A, r, threads);
            fold_top(inst[k].S, r, threads);
            if (round >= sh[k].skip + sh[k].h) {
                fold_top(Et[k], r, threads);
                fold_top(inst[k].B, r, threads);
                fold_top(inst[k].T, r, threads);
                fold_top(inst[k].M, r, threads);
            }
        }
    }
    std::vector<Fr> claims;
    for (uint64_t k = 0; k < K; ++k) {
        const BatchInstance& I = inst[k];
        Fr c[5] = {I.A[0], I.S[0], I.B[0], I.M[0], I.T[0]};
        for (int i = 0; i < 5; ++i) {
            fr_to_bytes(out, c[i]);
            out += 32;
            claims.push_back(c[i]);
        }
    }
    tr.absorb_fr("final", claims.data(), claims.size());
    return OK;
}

// Verifier: rounds, final identity, T~_k from the public tables; S_k and m_k
// (counts) are checked against their claims when given.
inline int tlookup_multi_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, const Fr* const* T,
                                uint64_t K, const uint64_t* D, const uint64_t* N, const Fr* const* S,
                                const uint64_t* const* m_counts, Fr* v_out, int threads) {
    std::vector<MultiShape> sh;
    int n = 0;
    if (!seed || !proof || !T || !tlookup_multi_shapes(D, N, K, sh, n)) return E_BADARG;
    if (len != tlookup_multi_proof_bytes(n, K)) return E_REJECT;
    if (memcmp(proof, "ZKTM\x01\0\0\0", 8) != 0) return E_REJECT;
    auto le64 = [&](const uint8_t* p) {
        uint64_t v = 0;
        for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i);
        return v;
    };
    if (le64(proof + 8) != K) return E_REJECT;
    for (uint64_t k = 0; k < K; ++k)
        if (le64(proof + 16 + 16 * k) != D[k] || le64(proof + 24 + 16 * k) != N[k]) return E_REJECT;
    const uint8_t* digests = proof + 16 + 16 * K;
    const uint8_t* ab = digests + 32 * K;
    const uint8_t* body = ab + 64 * K;
    size_t nfr = (size_t)4 * n + 5 * K;
    std::vector<Fr> el(nfr);
    for (size_t i = 0; i < nfr; ++i) {
        el[i] = fr_from_bytes(body + 32 * i);
        if (!fr_is_canonical(el[i])) return E_REJECT;
    }
    Transcript tr = tlookup_multi_transcript(seed, D, N, K);
    for (uint64_t k = 0; k < K; ++k) tr.absorb("m", digests + 32 * k, 32);
    Fr beta = tr.challenge("beta");
    for (uint64_t k = 0; k < K; ++k) {
        tr.absorb("A", ab + 64 * k, 32);
        tr.absorb("B", ab + 64 * k + 32, 32);
    }
    Fr alpha = tr.challenge("alpha");
    Fr alpha2 = fr_mul(alpha, alpha);
    std::vector<Fr> u(n), v(n);
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");
    Fr lambda = tr.challenge("lambda");
    Fr lam_sum = fr_zero(), lam_pow = fr_one();
    std::vector<Fr> lam(K);
    for (uint64_t k = 0; k < K; ++k) {
        lam[k] = lam_pow;
        lam_sum = fr_add(lam_sum, lam_pow);
        lam_pow = fr_mul(lam_pow, lambda);
    }
    Fr claim = fr_mul(lam_sum, fr_add(alpha, alpha2));
    for (int k = 0; k < n; ++k) {
        const Fr* g = &el[4 * k];
        if (!fr_eq(fr_add(g[0], g[1]), claim)) return E_REJECT;
        tr.absorb_fr("g", g, 4);
        v[k] = tr.challenge("r");
        claim = lagrange_eval(g, 4, v[k]);
    }
    const Fr* fin = &el[4 * n];
    tr.absorb_fr("final", fin, 5 * K);
    Fr total = fr_zero();
    for (uint64_t k = 0; k < K; ++k) {
        const Fr* c = fin + 5 * k;
        const int skip = sh[k].skip, h = sh[k].h;
        Fr e_full = eq_at_point(u.data() + skip, v.data() + skip, sh[k].n);
        Fr e_tab = eq_at_point(u.data() + skip + h, v.data() + skip + h, sh[k].l);
        Fr fk = tlookup_summand(c[0], c[1], e_full, c[2], c[4], e_tab, c[3], alpha, alpha2, beta, fr_two_inv_pow((unsigned)h));
        total = fr_add(total, fr_mul(fr_mul(lam[k], fr_two_inv_pow((unsigned)skip)), fk));
    }
    if (!fr_eq(total, claim)) return E_REJECT;
    for (uint64_t k = 0; k < K; ++k) {
        const Fr* c = fin + 5 * k;
        const int skip = sh[k].skip, h = sh[k].h;
        if (!fr_eq(mle_eval(T[k], sh[k].l, v.data() + skip + h, threads), c[4])) return E_REJECT;
        if (S && S[k] && !fr_eq(mle_eval(S[k], sh[k].n, v.data() + skip, threads), c[1])) return E_REJECT;
        if (m_counts && m_counts[k]) {
            std::vector<Fr> M(N[k]);
            std::vector<uint64_t> mc(m_counts[k], m_counts[k] + N[k]);
            for (uint64_t j = 0; j < N[k]; ++j) M[j] = fr_from_u64(mc[j]);
            if (!fr_eq(mle_eval(M.data(), sh[k].l, v.data() + skip + h, threads), c[3])) return E_REJECT;
            uint8_t md[32];
            m_digest(md, mc);
            if (memcmp(md, digests + 32 * k, 32) != 0) return E_REJECT;
        }
    }
    if (v_out) for (int t = 0; t < n; ++t) v_out[t] = v[t];
    return OK;
}

}  // namespace oracle
