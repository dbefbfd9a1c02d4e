// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// tlookup (Section 4, Protocol 1) made non-interactive with the transcript of
// transcript.hpp, every quantity computed from its definition:
//
//   m_j = |{ i : S_i = T_j }|                      (multiplicities, Section 4)
//   A_i = 1/(beta + S_i),  B_j = 1/(beta + T_j)    (inverse vectors, Section 4)
//   sumcheck of the tlookup identity (Section 4, second form):
//     alpha + alpha^2 = sum_x f(x),  x = i (+) j,  h = log2(D/N),
//     f(x) = A(x) (alpha e~(u,x) (S(x)+beta) + 1)
//            + 2^-h B(j) (alpha^2 e~(u_[h:], j) (T(j)+beta) - m(j))
//   with the generic sumcheck rounds of Section 3.3.
//
// Readings where the paper is silent (all this build's own):
//   * duplicate table entries: an S_i is credited to the LOWEST j with
//     T_j = S_i (any split verifies; one rule is needed for equal bytes);
//   * S_i not in T is an error that reports the smallest such i;
//   * variables are bound in written order, w_0 (top index bit) first, so the
//     first h rounds see the table side only as a constant;
//   * a round polynomial (degree <= 3) is sent as its values at X = 0,1,2,3;
//   * the commitments of Protocol 1 are outside this build: the seed stands in
//     for the commitments of T and S, a digest of m for the commitment of m,
//     digests of A and B for theirs.  Message order is Protocol 1's: m is sent
//     before beta is drawn, A and B after beta and before the sumcheck, so that
//     alpha, u and every round challenge depend on them;
//   * digest of m: counts as 32-bit little-endian words, cut into leaves of
//     128 counts, leaf digests concatenated and hashed once more;
//   * digest of a vector of field elements (vec_digest below): a hash tree over
//     the elements' canonical bytes.
//
// Proof bytes: "ZKTL" | u32 version=2 | LE64 D | LE64 N | digest(m) (32)
//              | digest(A) (32) | digest(B) (32)
//              | n x [g(0) g(1) g(2) g(3)] | A~(v) S~(v) B~(v') m~(v') T~(v')
// with every field element as 32 little-endian bytes of its canonical integer,
// n = log2 D and v' = v_[h:].
#pragma once
#include <array>
#include <map>

#include "poly.hpp"
#include "transcript.hpp"

namespace oracle {

enum {
    OK = 0,
    E_BADARG = -1,
    E_NOT_IN_TABLE = -2,
    E_ZERO_DENOM = -3,
    E_REJECT = -4,
    E_BUFSZ = -5,
};

static const size_t M_LEAF = 128;

static const size_t VEC_LEAF = 128;     // elements per leaf of vec_digest
static const size_t TLOOKUP_HEADER = 120;  // magic, version, D, N and the three digests

inline size_t tlookup_proof_bytes(int n) { return TLOOKUP_HEADER + (size_t)n * 128 + 160; }

// m_j by counting.  Returns OK or E_NOT_IN_TABLE (then *bad_index is the
// smallest i with S_i outside T).
inline int multiplicities(const Fr* S, uint64_t D, const Fr* T, uint64_t N, std::vector<uint64_t>& m,
                          uint64_t* bad_index, int threads) {
    std::map<std::array<uint64_t, 4>, uint64_t> first_row;
    for (uint64_t j = 0; j < N; ++j) {
        std::array<uint64_t, 4> key = {T[j].w[0], T[j].w[1], T[j].w[2], T[j].w[3]};
        first_row.insert({key, j});  // keeps the lowest j of equal entries
    }
    int workers = std::max(1, threads);
    std::vector<std::vector<uint64_t>> local(workers);
    std::vector<uint64_t> bad(workers, UINT64_MAX);
    parallel_ranges(D, workers, [&](size_t lo, size_t hi, int w) {
        local[w].assign(N, 0);
        for (size_t i = lo; i < hi; ++i) {
            std::array<uint64_t, 4> key = {S[i].w[0], S[i].w[1], S[i].w[2], S[i].w[3]};
            auto it = first_row.find(key);
            if (it == first_row.end()) {
                if (bad[w] == UINT64_MAX) bad[w] = i;
            } else {
                local[w][it->second] += 1;
            }
        }
    });
    m.assign(N, 0);
    uint64_t worst = UINT64_MAX;
    for (int w = 0; w < workers; ++w) {
        worst = std::min(worst, bad[w]);
        if (local[w].size() == N)
            for (uint64_t j = 0; j < N; ++j) m[j] += local[w][j];
    }
    if (worst != UINT64_MAX) {
        if (bad_index) *bad_index = worst;
        return E_NOT_IN_TABLE;
    }
    return OK;
}

inline void m_digest(uint8_t out[32], const std::vector<uint64_t>& m) {
    Bytes leaves;
    for (size_t base = 0; base < m.size(); base += M_LEAF) {
        Bytes leaf;
        size_t end = std::min(m.size(), base + M_LEAF);
        for (size_t j = base; j < end; ++j) {
            uint32_t c = (uint32_t)m[j];
            uint8_t le[4] = {(uint8_t)c, (uint8_t)(c >> 8), (uint8_t)(c >> 16), (uint8_t)(c >> 24)};
            leaf.raw(le, 4);
        }
        uint8_t d[32];
        leaf.digest(d);
        leaves.raw(d, 32);
    }
    leaves.digest(out);
}

// Digest of a vector of n field elements (n a power of two), the stand-in for
// its commitment.  With L = max(1, n / 128) leaves, leaf i is the SHA-256 of the
// canonical bytes of elements i, i + L, i + 2L, ... in that order (128 of them,
// or all n when n < 128).  The leaf digests are then hashed upward: consecutive
// digests in groups of four (the two that are left, if only two are) give the
// next row, until one digest remains.
inline void vec_digest(uint8_t out[32], const Fr* v, size_t n, int threads = 1) {
    const size_t L = n / VEC_LEAF ? n / VEC_LEAF : 1;
    std::vector<uint8_t> row(32 * L);
    parallel_ranges(L, std::max(1, threads), [&](size_t lo, size_t hi, int) {
        for (size_t i = lo; i < hi; ++i) {
            Bytes leaf;
            for (size_t x = i; x < n; x += L) {
                uint8_t b[32];
                fr_to_bytes(b, v[x]);
                leaf.raw(b, 32);
            }
            leaf.digest(&row[32 * i]);
        }
    });
    size_t count = L;
    while (count > 1) {
        const size_t group = count >= 4 ? 4 : 2;
        std::vector<uint8_t> next(32 * (count / group));
        for (size_t i = 0; i < count / group; ++i) sha256(&next[32 * i], &row[32 * group * i], 32 * group);
        row.swap(next);
        count /= group;
    }
    memcpy(out, row.data(), 32);
}

inline Transcript tlookup_transcript(const uint8_t seed[32], uint64_t D, uint64_t N) {
    Bytes init;
    init.str("zkmi/tlookup/v2").raw(seed, 32).le64(D).le64(N);
    return Transcript(init);
}

struct TlookupAux {
    Fr beta, alpha;
    Fr sum_A;   // sum_i A_i
    Fr sum_mB;  // sum_j m_j B_j   (the two sides of the log-derivative identity)
};

// f at one point of a round: the summand of the tlookup identity with every
// array already evaluated at that point.
inline Fr tlookup_summand(const Fr& A, const Fr& S, const Fr& E, const Fr& B, const Fr& T, const Fr& Et,
                          const Fr& m, const Fr& alpha, const Fr& alpha2, const Fr& beta, const Fr& scale) {
    Fr left = fr_mul(A, fr_add(fr_mul(alpha, fr_mul(E, fr_add(S, beta))), fr_one()));
    Fr right = fr_mul(scale, fr_mul(B, fr_sub(fr_mul(alpha2, fr_mul(Et, fr_add(T, beta))), m)));
    return fr_add(left, right);
}

// Prover.  S: D canonical elements, T: N canonical elements.  forced_beta, if
// not null, replaces the transcript's beta (testing the zero-denominator
// path); the transcript state still advances as usual.
inline int tlookup_prove(const uint8_t seed[32], const Fr* S_in, uint64_t D, const Fr* T_in, uint64_t N,
                         uint8_t* proof, uint64_t cap, uint64_t* len, TlookupAux* aux, Fr* u_out, Fr* v_out,
                         uint64_t* bad_index, const Fr* forced_beta, int threads) {
    int n = log2_exact(D), l = log2_exact(N);
    if (!seed || !S_in || !T_in || n < 0 || l < 0 || N > D || D > ((uint64_t)1 << 31)) return E_BADARG;
    int h = n - l;
    size_t need = tlookup_proof_bytes(n);
    if (len) *len = need;
    if (!proof || cap < need) return E_BUFSZ;

    // Prep: multiplicities.
    std::vector<uint64_t> counts;
    int rc = multiplicities(S_in, D, T_in, N, counts, bad_index, threads);
    if (rc != OK) return rc;

    Transcript tr = tlookup_transcript(seed, D, N);
    uint8_t md[32];
    m_digest(md, counts);
    tr.absorb("m", md, 32);

    // Prove: beta, then the inverse vectors.
    Fr beta = tr.challenge("beta");
    if (forced_beta) beta = *forced_beta;
    std::vector<Fr> A(D), S(S_in, S_in + D), B(N), T(T_in, T_in + N), M(N);
    bool zero = false;
    for (uint64_t j = 0; j < N; ++j) {
        Fr den = fr_add(beta, T[j]);
        if (fr_is_zero(den)) { zero = true; break; }
        B[j] = fr_inv(den);
        M[j] = fr_from_u64(counts[j]);
    }
    if (zero) return E_ZERO_DENOM;
    std::vector<int> zero_seen(std::max(1, threads), 0);
    parallel_ranges(D, threads, [&](size_t lo, size_t hi, int w) {
        for (size_t i = lo; i < hi; ++i) {
            Fr den = fr_add(beta, S[i]);
            if (fr_is_zero(den)) { zero_seen[w] = 1; return; }
            A[i] = fr_inv(den);
        }
    });
    for (int z : zero_seen) if (z) return E_ZERO_DENOM;

    Fr sum_A = fr_zero(), sum_mB = fr_zero();
    for (uint64_t i = 0; i < D; ++i) sum_A = fr_add(sum_A, A[i]);
    for (uint64_t j = 0; j < N; ++j) sum_mB = fr_add(sum_mB, fr_mul(M[j], B[j]));

    // The prover sends A and B (their digests here) before the sumcheck starts.
    uint8_t dA[32], dB[32];
    vec_digest(dA, A.data(), D, threads);
    vec_digest(dB, B.data(), N, threads);
    tr.absorb("A", dA, 32);
    tr.absorb("B", dB, 32);

    Fr alpha = tr.challenge("alpha");
    Fr alpha2 = fr_mul(alpha, alpha);
    std::vector<Fr> u(n);
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");
    if (aux) *aux = TlookupAux{beta, alpha, sum_A, sum_mB};
    if (u_out) for (int t = 0; t < n; ++t) u_out[t] = u[t];

    std::vector<Fr> E = eq_table(u.data(), n, threads);
    std::vector<Fr> Et = eq_table(u.data() + h, l, threads);
    Fr scale = fr_two_inv_pow((unsigned)h);  // N / D

    // Header.
    uint8_t* out = proof;
    memcpy(out, "ZKTL", 4);
    out[4] = 2; out[5] = out[6] = out[7] = 0;
    for (int i = 0; i < 8; ++i) out[8 + i] = (uint8_t)(D >> (8 * i));
    for (int i = 0; i < 8; ++i) out[16 + i] = (uint8_t)(N >> (8 * i));
    memcpy(out + 24, md, 32);
    memcpy(out + 56, dA, 32);
    memcpy(out + 88, dB, 32);
    out += TLOOKUP_HEADER;

    // Rounds.
    int workers = std::max(1, threads);
    for (int k = 0; k < n; ++k) {
        size_t half = A.size() / 2;
        bool table_bound = (k >= h);  // the variable being bound is one of the table's
        std::vector<std::array<Fr, 4>> partial(workers);
        for (auto& p : partial) p = {fr_zero(), fr_zero(), fr_zero(), fr_zero()};
        parallel_ranges(half, workers, [&](size_t lo, size_t hi, int w) {
            std::array<Fr, 4> acc = {fr_zero(), fr_zero(), fr_zero(), fr_zero()};
            for (size_t p = lo; p < hi; ++p) {
                // Every array as a line in X through its two entries.
                Fr a = A[p], da = fr_sub(A[p + half], A[p]);
                Fr s = S[p], ds = fr_sub(S[p + half], S[p]);
                Fr e = E[p], de = fr_sub(E[p + half], E[p]);
                Fr b, db, t, dt, et, det, mm, dm;
                if (table_bound) {
                    b = B[p]; db = fr_sub(B[p + half], B[p]);
                    t = T[p]; dt = fr_sub(T[p + half], T[p]);
                    et = Et[p]; det = fr_sub(Et[p + half], Et[p]);
                    mm = M[p]; dm = fr_sub(M[p + half], M[p]);
                } else {
                    size_t j = p % N;  // the table does not depend on this variable
                    b = B[j]; t = T[j]; et = Et[j]; mm = M[j];
                    db = dt = det = dm = fr_zero();
                }
                for (int X = 0; X < 4; ++X) {
                    acc[X] = fr_add(acc[X], tlookup_summand(a, s, e, b, t, et, mm, alpha, alpha2, beta, scale));
                    a = fr_add(a, da); s = fr_add(s, ds); e = fr_add(e, de);
                    b = fr_add(b, db); t = fr_add(t, dt); et = fr_add(et, det); mm = fr_add(mm, dm);
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
        if (v_out) v_out[k] = r;
        fold_top(A, r, threads);
        fold_top(S, r, threads);
        fold_top(E, r, threads);
        if (table_bound) {
            fold_top(B, r, threads);
            fold_top(T, r, threads);
            fold_top(Et, r, threads);
            fold_top(M, r, threads);
        }
    }

    // Final claims.  With N = 1 the table arrays were never folded and have
    // one entry already.
    Fr claims[5] = {A[0], S[0], B[0], M[0], T[0]};
    for (int i = 0; i < 5; ++i) fr_to_bytes(out + 32 * i, claims[i]);
    tr.absorb_fr("final", claims, 5);
    return OK;
}

// What the verifier keeps after checking the rounds: the point and the claims
// that the paper discharges with proofs of evaluation on commitments.
struct TlookupClaims {
    Fr A_v, S_v, B_vp, m_vp, T_vp;
};

// Verifier.  T is public and its claim is recomputed.  If S, A, B (field
// elements) and m_counts are given, the other four claims are recomputed from
// them too, standing in for the openings of the commitments; otherwise they
// are returned for the caller to discharge.  `stage`, if not null, receives
// which check failed (0 = none, 1 = header, 2 = round k consistency, 3 = final
// identity, 4 = a claim disagrees with its tensor).
inline int tlookup_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, const Fr* T, uint64_t D,
                          uint64_t N, const Fr* S, const uint64_t* m_counts, const Fr* A, const Fr* B,
                          TlookupClaims* claims_out, Fr* v_out, int* stage, int threads) {
    if (stage) *stage = 0;
    int n = log2_exact(D), l = log2_exact(N);
    if (!seed || !proof || !T || n < 0 || l < 0 || N > D) return E_BADARG;
    int h = n - l;
    auto fail = [&](int s) { if (stage) *stage = s; return (int)E_REJECT; };
    if (len != tlookup_proof_bytes(n)) return fail(1);
    if (memcmp(proof, "ZKTL", 4) != 0 || proof[4] != 2 || proof[5] || proof[6] || proof[7]) return fail(1);
    uint64_t Dp = 0, Np = 0;
    for (int i = 0; i < 8; ++i) { Dp |= (uint64_t)proof[8 + i] << (8 * i); Np |= (uint64_t)proof[16 + i] << (8 * i); }
    if (Dp != D || Np != N) return fail(1);

    // Every field element in the proof must be canonical.
    size_t nfr = (size_t)4 * n + 5;
    std::vector<Fr> el(nfr);
    for (size_t i = 0; i < nfr; ++i) {
        el[i] = fr_from_bytes(proof + TLOOKUP_HEADER + 32 * i);
        if (!fr_is_canonical(el[i])) return fail(1);
    }

    Transcript tr = tlookup_transcript(seed, D, N);
    tr.absorb("m", proof + 24, 32);
    Fr beta = tr.challenge("beta");
    tr.absorb("A", proof + 56, 32);
    tr.absorb("B", proof + 88, 32);
    Fr alpha = tr.challenge("alpha");
    Fr alpha2 = fr_mul(alpha, alpha);
    std::vector<Fr> u(n), v(n);
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");

    Fr claim = fr_add(alpha, alpha2);
    for (int k = 0; k < n; ++k) {
        const Fr* g = &el[4 * k];
        if (!fr_eq(fr_add(g[0], g[1]), claim)) return fail(2);
        tr.absorb_fr("g", g, 4);
        v[k] = tr.challenge("r");
        claim = lagrange_eval(g, 4, v[k]);
    }
    const Fr* fin = &el[4 * n];
    tr.absorb_fr("final", fin, 5);
    TlookupClaims c = {fin[0], fin[1], fin[2], fin[3], fin[4]};

    Fr e_full = eq_at_point(u.data(), v.data(), n);
    Fr e_tab = eq_at_point(u.data() + h, v.data() + h, l);
    Fr expect = tlookup_summand(c.A_v, c.S_v, e_full, c.B_vp, c.T_vp, e_tab, c.m_vp, alpha, alpha2, beta,
                                fr_two_inv_pow((unsigned)h));
    if (!fr_eq(expect, claim)) return fail(3);

    if (!fr_eq(mle_eval(T, l, v.data() + h, threads), c.T_vp)) return fail(4);
    if (S && !fr_eq(mle_eval(S, n, v.data(), threads), c.S_v)) return fail(4);
    // A and B, when given, must also be the vectors whose digests the proof carries
    uint8_t dv[32];
    if (A) {
        if (!fr_eq(mle_eval(A, n, v.data(), threads), c.A_v)) return fail(4);
        vec_digest(dv, A, D, threads);
        if (memcmp(dv, proof + 56, 32) != 0) return fail(4);
    }
    if (B) {
        if (!fr_eq(mle_eval(B, l, v.data() + h, threads), c.B_vp)) return fail(4);
        vec_digest(dv, B, N, threads);
        if (memcmp(dv, proof + 88, 32) != 0) return fail(4);
    }
    if (m_counts) {
        std::vector<Fr> M(N);
        for (uint64_t j = 0; j < N; ++j) M[j] = fr_from_u64(m_counts[j]);
        if (!fr_eq(mle_eval(M.data(), l, v.data() + h, threads), c.m_vp)) return fail(4);
        // the digest in the proof must be the digest of these counts
        std::vector<uint64_t> mc(m_counts, m_counts + N);
        uint8_t md[32];
        m_digest(md, mc);
        if (memcmp(md, proof + 24, 32) != 0) return fail(4);
    }
    if (claims_out) *claims_out = c;
    if (v_out) for (int t = 0; t < n; ++t) v_out[t] = v[t];
    return OK;
}

}  // namespace oracle
