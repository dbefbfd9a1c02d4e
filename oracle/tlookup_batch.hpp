// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// Several tlookup instances of one shape proved by ONE sumcheck.  The paper
// proves every lookup of an attention layer separately (Protocol 2) and does not
// describe batching them; this is this build's reading of a workload that asks
// for "two tlookup instances plus the batched sumcheck over them": K instances
// (S_k, T_k) with common D and N share beta, alpha and u, and the sumcheck runs on
//   f = sum_k lambda^k f_k,   claim_0 = (sum_k lambda^k) (alpha + alpha^2),
// with f_k the tlookup summand of instance k (Section 4, second form of the
// identity) and lambda one more challenge.  All rounds share their challenges.
//
// Transcript: SHA256("zkmi/tlookup-batch/v2" || seed || LE64 D || LE64 N || LE64 K);
// absorb("m", digest(m_k)) for k = 0..K-1; beta = challenge("beta");
// absorb("A", digest(A_k)), absorb("B", digest(B_k)) for k = 0..K-1 (Protocol 1's
// order: the inverse vectors are sent after beta and before the sumcheck);
// alpha = challenge("alpha"); u_t = challenge("u"), t = 0..n-1;
// lambda = challenge("lambda"); per round absorb("g", 4 values), r = challenge("r");
// absorb("final", K x 5 claims).
//
// Proof bytes: "ZKTB" | u32 version=2 | LE64 D | LE64 N | LE64 K | K x digest(m_k)
//              | K x [digest(A_k) digest(B_k)]
//              | n x [g(0) g(1) g(2) g(3)] | K x [A~(v) S~(v) B~(v') m~(v') T~(v')].
#pragma once
#include "tlookup.hpp"

namespace oracle {

inline size_t tlookup_batch_proof_bytes(int n, uint64_t K) { return 32 + 96 * K + (size_t)n * 128 + 160 * K; }

inline Transcript tlookup_batch_transcript(const uint8_t seed[32], uint64_t D, uint64_t N, uint64_t K) {
    Bytes init;
    init.str("zkmi/tlookup-batch/v2").raw(seed, 32).le64(D).le64(N).le64(K);
    return Transcript(init);
}

struct BatchInstance {
    std::vector<Fr> A, S, B, T, M;
    std::vector<uint64_t> counts;
};

// S_in[k]: D elements, T_in[k]: N elements.  aux_out (may be null): beta, alpha,
// lambda, then per instance sum_A, sum_mB.
inline int tlookup_batch_prove(const uint8_t seed[32], const Fr* const* S_in, const Fr* const* T_in, uint64_t K,
                               uint64_t D, uint64_t N, uint8_t* proof, uint64_t cap, uint64_t* len, Fr* aux_out,
                               Fr* v_out, uint64_t* bad_instance, uint64_t* bad_index, int threads) {
    int n = log2_exact(D), l = log2_exact(N);
    if (!seed || !S_in || !T_in || K == 0 || K > 8 || n < 0 || l < 0 || N > D || D > ((uint64_t)1 << 31)) return E_BADARG;
    int h = n - l;
    size_t need = tlookup_batch_proof_bytes(n, K);
    if (len) *len = need;
    if (!proof || cap < need) return E_BUFSZ;

    std::vector<BatchInstance> inst(K);
    Transcript tr = tlookup_batch_transcript(seed, D, N, K);
    uint8_t* out = proof;
    memcpy(out, "ZKTB", 4);
    out[4] = 2; out[5] = out[6] = out[7] = 0;
    for (int i = 0; i < 8; ++i) {
        out[8 + i] = (uint8_t)(D >> (8 * i));
        out[16 + i] = (uint8_t)(N >> (8 * i));
        out[24 + i] = (uint8_t)(K >> (8 * i));
    }
    out += 32;
    for (uint64_t k = 0; k < K; ++k) {
        int rc = multiplicities(S_in[k], D, T_in[k], N, inst[k].counts, bad_index, threads);
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
        I.S.assign(S_in[k], S_in[k] + D);
        I.T.assign(T_in[k], T_in[k] + N);
        I.A.resize(D);
        I.B.resize(N);
        I.M.resize(N);
        for (uint64_t j = 0; j < N; ++j) {
            Fr den = fr_add(beta, I.T[j]);
            if (fr_is_zero(den)) return E_ZERO_DENOM;
            I.B[j] = fr_inv(den);
            I.M[j] = fr_from_u64(I.counts[j]);
        }
        std::vector<int> zero_seen(std::max(1, threads), 0);
        parallel_ranges(D, threads, [&](size_t lo, size_t hi, int w) {
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
        vec_digest(dA, inst[k].A.data(), D, threads);
        vec_digest(dB, inst[k].B.data(), N, threads);
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
    std::vector<Fr> lam(K);  // lambda^k
    lam[0] = fr_one();
    for (uint64_t k = 1; k < K; ++k) lam[k] = fr_mul(lam[k - 1], lambda);
    if (aux_out) {
        aux_out[0] = beta;
        aux_out[1] = alpha;
        aux_out[2] = lambda;
        for (uint64_t k = 0; k < K; ++k) {
            Fr sA = fr_zero(), sMB = fr_zero();
            for (uint64_t i = 0; i < D; ++i) sA = fr_add(sA, inst[k].A[i]);
            for (uint64_t j = 0; j < N; ++j) sMB = fr_add(sMB, fr_mul(inst[k].M[j], inst[k].B[j]));
            aux_out[3 + 2 * k] = sA;
            aux_out[4 + 2 * k] = sMB;
        }
    }

    std::vector<Fr> E = eq_table(u.data(), n, threads);
    std::vector<Fr> Et = eq_table(u.data() + h, l, threads);
    Fr scale = fr_two_inv_pow((unsigned)h);

    int workers = std::max(1, threads);
    for (int round = 0; round < n; ++round) {
        size_t half = E.size() / 2;
        bool table_bound = (round >= h);
        std::vector<std::array<Fr, 4>> partial(workers);
        for (auto& p : partial) p = {fr_zero(), fr_zero(), fr_zero(), fr_zero()};
        parallel_ranges(half, workers, [&](size_t lo, size_t hi, int w) {
            std::array<Fr, 4> acc = {fr_zero(), fr_zero(), fr_zero(), fr_zero()};
            for (size_t p = lo; p < hi; ++p) {
                Fr e0 = E[p], de = fr_sub(E[p + half], E[p]);
                size_t j = p % N;
                Fr et0 = table_bound ? Et[p] : Et[j];
                Fr det = table_bound ? fr_sub(Et[p + half], Et[p]) : fr_zero();
                for (uint64_t k = 0; k < K; ++k) {
                    const BatchInstance& I = inst[k];
                    Fr a = I.A[p], da = fr_sub(I.A[p + half], I.A[p]);
                    Fr s = I.S[p], ds = fr_sub(I.S[p + half], I.S[p]);
                    Fr e = e0, et = et0;
                    Fr b, db, t, dt, mm, dm;
                    if (table_bound) {
                        b = I.B[p]; db = fr_sub(I.B[p + half], I.B[p]);
                        t = I.T[p]; dt = fr_sub(I.T[p + half], I.T[p]);
                        mm = I.M[p]; dm = fr_sub(I.M[p + half], I.M[p]);
                    } else {
                        b = I.B[j]; t = I.T[j]; mm = I.M[j];
                        db = dt = dm = fr_zero();
                    }
                    for (int X = 0; X < 4; ++X) {
                        Fr fk = tlookup_summand(a, s, e, b, t, et, mm, alpha, alpha2, beta, scale);
                        acc[X] = fr_add(acc[X], fr_mul(lam[k], fk));
                        a = fr_add(a, da); s = fr_add(s, ds); e = fr_add(e, de);
                        b = fr_add(b, db); t = fr_add(t, dt); et = fr_add(et, det); mm = fr_add(mm, dm);
                    }
                }
            }
            partial[w] = acc;
        });
        Fr g[4] = {fr_zero(), fr_zero(), fr_zero(), fr_zero()};
        for (auto& p : partial)
            for (int X = 0; X < 4; ++X) g[X] = fr_add(g[X], p[X]);
        for (int X = 0; X < 4; ++X) fr_to_bytes(out + 32 * X, g[X]);
        out += 128;
        tr.absorb_fr("g", g, 4);
        Fr r = tr.challenge("r");
        if (v_out) v_out[round] = r;
        fold_top(E, r, threads);
        if (table_bound) fold_top(Et, r, threads);
        for (uint64_t k = 0; k < K; ++k) {
            fold_top(inst[k].A, r, threads);
            fold_top(inst[k].S, r, threads);
            if (table_bound) {
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

// Verifier: rounds, final identity, T~_k(v') from the public tables; S_k and
// m_k (counts) are checked against their claims when given.
inline int tlookup_batch_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, const Fr* const* T,
                                uint64_t K, uint64_t D, uint64_t N, const Fr* const* S, const uint64_t* const* m_counts,
                                Fr* v_out, int threads) {
    int n = log2_exact(D), l = log2_exact(N);
    if (!seed || !proof || !T || K == 0 || K > 8 || n < 0 || l < 0 || N > D) return E_BADARG;
    int h = n - l;
    if (len != tlookup_batch_proof_bytes(n, K)) return E_REJECT;
    if (memcmp(proof, "ZKTB\x02\0\0\0", 8) != 0) return E_REJECT;
    uint64_t Dp = 0, Np = 0, Kp = 0;
    for (int i = 0; i < 8; ++i) {
        Dp |= (uint64_t)proof[8 + i] << (8 * i);
        Np |= (uint64_t)proof[16 + i] << (8 * i);
        Kp |= (uint64_t)proof[24 + i] << (8 * i);
    }
    if (Dp != D || Np != N || Kp != K) return E_REJECT;
    const uint8_t* body = proof + 32 + 96 * K;
    size_t nfr = (size_t)4 * n + 5 * K;
    std::vector<Fr> el(nfr);
    for (size_t i = 0; i < nfr; ++i) {
        el[i] = fr_from_bytes(body + 32 * i);
        if (!fr_is_canonical(el[i])) return E_REJECT;
    }
    Transcript tr = tlookup_batch_transcript(seed, D, N, K);
    for (uint64_t k = 0; k < K; ++k) tr.absorb("m", proof + 32 + 32 * k, 32);
    Fr beta = tr.challenge("beta");
    for (uint64_t k = 0; k < K; ++k) {
        tr.absorb("A", proof + 32 + 32 * K + 64 * k, 32);
        tr.absorb("B", proof + 32 + 32 * K + 64 * k + 32, 32);
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
    Fr e_full = eq_at_point(u.data(), v.data(), n);
    Fr e_tab = eq_at_point(u.data() + h, v.data() + h, l);
    Fr scale = fr_two_inv_pow((unsigned)h);
    Fr total = fr_zero();
    for (uint64_t k = 0; k < K; ++k) {
        const Fr* c = fin + 5 * k;
        Fr fk = tlookup_summand(c[0], c[1], e_full, c[2], c[4], e_tab, c[3], alpha, alpha2, beta, scale);
        total = fr_add(total, fr_mul(lam[k], fk));
    }
    if (!fr_eq(total, claim)) return E_REJECT;
    for (uint64_t k = 0; k < K; ++k) {
        const Fr* c = fin + 5 * k;
        if (!fr_eq(mle_eval(T[k], l, v.data() + h, threads), c[4])) return E_REJECT;
        if (S && S[k] && !fr_eq(mle_eval(S[k], n, v.data(), threads), c[1])) return E_REJECT;
        if (m_counts && m_counts[k]) {
            std::vector<Fr> M(N);
            std::vector<uint64_t> mc(m_counts[k], m_counts[k] + N);
            for (uint64_t j = 0; j < N; ++j) M[j] = fr_from_u64(mc[j]);
            if (!fr_eq(mle_eval(M.data(), l, v.data() + h, threads), c[3])) return E_REJECT;
            uint8_t md[32];
            m_digest(md, mc);
            if (memcmp(md, proof + 32 + 32 * k, 32) != 0) return E_REJECT;
        }
    }
    if (v_out) for (int t = 0; t < n; ++t) v_out[t] = v[t];
    return OK;
}

}  // namespace oracle
