// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// C entry points of the oracle for the tests, the smoke check and the bench's
// CPU-baseline leg.  Field elements cross this boundary as 32 little-endian
// bytes of the canonical integer; on a little-endian host that is exactly the
// in-memory form of oracle::Fr, which the static assertion below pins.
#include <cstdio>

#include "product.hpp"
#include "tlookup_batch.hpp"
#include "tlookup_multi.hpp"
#include "zkattn_link.hpp"

#if !defined(__BYTE_ORDER__) || __BYTE_ORDER__ != __ORDER_LITTLE_ENDIAN__
#error "the oracle's C boundary assumes a little-endian host"
#endif

using namespace oracle;
static_assert(sizeof(Fr) == 32, "Fr must be 32 bytes");

static const Fr* as_fr(const uint8_t* p) { return reinterpret_cast<const Fr*>(p); }
static Fr* as_fr(uint8_t* p) { return reinterpret_cast<Fr*>(p); }

extern "C" {

void oracle_fr_modulus(uint8_t out[32]) {
    Fr m = {{MODULUS[0], MODULUS[1], MODULUS[2], MODULUS[3]}};
    fr_to_bytes(out, m);
}

void oracle_fr_barrett_mu(uint8_t out[40]) {
    const uint64_t* mu = barrett_mu().mu;
    for (int i = 0; i < 5; ++i)
        for (int j = 0; j < 8; ++j) out[8 * i + j] = (uint8_t)(mu[i] >> (8 * j));
}

// 1 if every one of the n elements is < r.
int oracle_fr_all_canonical(const uint8_t* a, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i)
        if (!fr_is_canonical(as_fr(a)[i])) return 0;
    return 1;
}

void oracle_fr_add(uint8_t* out, const uint8_t* a, const uint8_t* b, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) as_fr(out)[i] = fr_add(as_fr(a)[i], as_fr(b)[i]);
}
void oracle_fr_sub(uint8_t* out, const uint8_t* a, const uint8_t* b, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) as_fr(out)[i] = fr_sub(as_fr(a)[i], as_fr(b)[i]);
}
void oracle_fr_mul(uint8_t* out, const uint8_t* a, const uint8_t* b, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) as_fr(out)[i] = fr_mul(as_fr(a)[i], as_fr(b)[i]);
}
// out = x + s * y, elementwise (y may be null: out = x + s)
void oracle_fr_axpy(uint8_t* out, const uint8_t* x, const uint8_t s[32], const uint8_t* y, uint64_t n,
                    int threads) {
    Fr sc = fr_from_bytes(s);
    parallel_ranges(n, threads, [&](size_t lo, size_t hi, int) {
        for (size_t i = lo; i < hi; ++i)
            as_fr(out)[i] = y ? fr_add(as_fr(x)[i], fr_mul(sc, as_fr(y)[i])) : fr_add(as_fr(x)[i], sc);
    });
}
void oracle_fr_mul_scalar(uint8_t* out, const uint8_t* x, const uint8_t s[32], uint64_t n) {
    Fr sc = fr_from_bytes(s);
    for (uint64_t i = 0; i < n; ++i) as_fr(out)[i] = fr_mul(as_fr(x)[i], sc);
}
int oracle_fr_inv(uint8_t* out, const uint8_t* a, uint64_t n, int threads) {
    std::vector<int> zero(std::max(1, threads), 0);
    parallel_ranges(n, threads, [&](size_t lo, size_t hi, int w) {
        for (size_t i = lo; i < hi; ++i) {
            if (fr_is_zero(as_fr(a)[i])) { zero[w] = 1; continue; }
            as_fr(out)[i] = fr_inv(as_fr(a)[i]);
        }
    });
    for (int z : zero) if (z) return E_ZERO_DENOM;
    return OK;
}
void oracle_fr_pow(uint8_t out[32], const uint8_t a[32], const uint8_t e[32]) {
    Fr ee = fr_from_bytes(e);
    *as_fr(out) = fr_pow(fr_from_bytes(a), ee.w);
}
void oracle_fr_sum(uint8_t out[32], const uint8_t* a, uint64_t n) {
    Fr acc = fr_zero();
    for (uint64_t i = 0; i < n; ++i) acc = fr_add(acc, as_fr(a)[i]);
    *as_fr(out) = acc;
}
void oracle_fr_from_i64(uint8_t* out, const int64_t* in, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) as_fr(out)[i] = fr_from_i64(in[i]);
}
void oracle_fr_from_be512(uint8_t out[32], const uint8_t in[64]) { *as_fr(out) = fr_from_be512(in); }

void oracle_sha256(uint8_t out[32], const uint8_t* data, uint64_t len) { sha256(out, data, len); }

void oracle_transcript_init(uint8_t state[32], const uint8_t* data, uint64_t len) { sha256(state, data, len); }
void oracle_transcript_absorb(uint8_t state[32], const char* tag, const uint8_t* data, uint64_t len) {
    Bytes none;
    Transcript tr(none);
    memcpy(tr.state, state, 32);
    tr.absorb(tag, data, len);
    memcpy(state, tr.state, 32);
}
void oracle_transcript_challenge(uint8_t state[32], const char* tag, uint8_t out[32]) {
    Bytes none;
    Transcript tr(none);
    memcpy(tr.state, state, 32);
    *as_fr(out) = tr.challenge(tag);
    memcpy(state, tr.state, 32);
}

// The combiner of a pair table (Section 4, last paragraph: X + rho Y against
// T_X + rho T_Y with rho chosen by the verifier).  It is drawn before S and T
// exist, from a transcript of its own.
void oracle_pair_combiner(const uint8_t seed[32], uint8_t out[32]) {
    Bytes init;
    init.str("zkmi/rho/v1").raw(seed, 32);
    Transcript tr(init);
    *as_fr(out) = tr.challenge("rho");
}

void oracle_eq_table(uint8_t* out, const uint8_t* u, int nvars, int threads) {
    std::vector<Fr> e = eq_table(as_fr(u), nvars, threads);
    memcpy(out, e.data(), e.size() * sizeof(Fr));
}
void oracle_eq_at_point(uint8_t out[32], const uint8_t* u, const uint8_t* v, int nvars) {
    *as_fr(out) = eq_at_point(as_fr(u), as_fr(v), nvars);
}
void oracle_mle_eval(uint8_t out[32], const uint8_t* s, int nvars, const uint8_t* point, int threads) {
    *as_fr(out) = mle_eval(as_fr(s), nvars, as_fr(point), threads);
}
void oracle_lagrange_eval(uint8_t out[32], const uint8_t* y, int npts, const uint8_t at[32]) {
    *as_fr(out) = lagrange_eval(as_fr(y), npts, fr_from_bytes(at));
}

int oracle_multiplicities(uint64_t* m_out, const uint8_t* S, uint64_t D, const uint8_t* T, uint64_t N,
                          uint64_t* bad_index, int threads) {
    std::vector<uint64_t> m;
    int rc = multiplicities(as_fr(S), D, as_fr(T), N, m, bad_index, threads);
    if (rc == OK) memcpy(m_out, m.data(), N * sizeof(uint64_t));
    return rc;
}
void oracle_m_digest(uint8_t out[32], const uint64_t* m, uint64_t N) {
    std::vector<uint64_t> mv(m, m + N);
    m_digest(out, mv);
}

void oracle_vec_digest(uint8_t out[32], const uint8_t* v, uint64_t n, int threads) { vec_digest(out, as_fr(v), n, threads); }

uint64_t oracle_tlookup_proof_bytes(uint64_t D) { return tlookup_proof_bytes(log2_exact(D)); }

// aux: beta | alpha | sum_A | sum_mB (4 x 32 bytes); u_out, v_out: log2(D) elements each.
int oracle_tlookup_prove(const uint8_t seed[32], const uint8_t* S, uint64_t D, const uint8_t* T, uint64_t N,
                         uint8_t* proof, uint64_t cap, uint64_t* len, uint8_t* aux, uint8_t* u_out,
                         uint8_t* v_out, uint64_t* bad_index, const uint8_t* forced_beta, int threads) {
    TlookupAux ax;
    Fr fb;
    if (forced_beta) fb = fr_from_bytes(forced_beta);
    int rc = tlookup_prove(seed, as_fr(S), D, as_fr(T), N, proof, cap, len, &ax, u_out ? as_fr(u_out) : nullptr,
                           v_out ? as_fr(v_out) : nullptr, bad_index, forced_beta ? &fb : nullptr, threads);
    if (rc == OK && aux) memcpy(aux, &ax, sizeof ax);
    return rc;
}

// claims_out: A~(v) S~(v) B~(v') m~(v') T~(v') (5 x 32 bytes).
int oracle_tlookup_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, const uint8_t* T,
                          uint64_t D, uint64_t N, const uint8_t* S, const uint64_t* m_counts, const uint8_t* A,
                          const uint8_t* B, uint8_t* claims_out, uint8_t* v_out, int* stage, int threads) {
    TlookupClaims c;
    int rc = tlookup_verify(seed, proof, len, as_fr(T), D, N, S ? as_fr(S) : nullptr, m_counts,
                            A ? as_fr(A) : nullptr, B ? as_fr(B) : nullptr, &c, v_out ? as_fr(v_out) : nullptr,
                            stage, threads);
    if (rc == OK && claims_out) memcpy(claims_out, &c, sizeof c);
    return rc;
}

uint64_t oracle_tlookup_batch_proof_bytes(uint64_t D, uint64_t K) {
    return tlookup_batch_proof_bytes(log2_exact(D), K);
}

// S, T: arrays of K pointers.  aux: beta | alpha | lambda | K x (sum_A, sum_mB).
int oracle_tlookup_batch_prove(const uint8_t seed[32], const uint8_t* const* S, const uint8_t* const* T, uint64_t K,
                               uint64_t D, uint64_t N, uint8_t* proof, uint64_t cap, uint64_t* len, uint8_t* aux,
                               uint8_t* v_out, uint64_t* bad_instance, uint64_t* bad_index, int threads) {
    return tlookup_batch_prove(seed, reinterpret_cast<const Fr* const*>(S), reinterpret_cast<const Fr* const*>(T), K, D,
                               N, proof, cap, len, aux ? as_fr(aux) : nullptr, v_out ? as_fr(v_out) : nullptr,
                               bad_instance, bad_index, threads);
}

int oracle_tlookup_batch_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, const uint8_t* const* T,
                                uint64_t K, uint64_t D, uint64_t N, const uint8_t* const* S,
                                const uint64_t* const* m_counts, uint8_t* v_out, int threads) {
    return tlookup_batch_verify(seed, proof, len, reinterpret_cast<const Fr* const*>(T), K, D, N,
                                reinterpret_cast<const Fr* const*>(S), m_counts, v_out ? as_fr(v_out) : nullptr,
                                threads);
}

uint64_t oracle_tlookup_multi_proof_bytes(uint64_t n_max, uint64_t K) { return tlookup_multi_proof_bytes((int)n_max, K); }

// S, T: arrays of K pointers; D, N: K lengths.  aux: beta | alpha | lambda | K x (sum_A, sum_mB).
int oracle_tlookup_multi_prove(const uint8_t seed[32], const uint8_t* const* S, const uint8_t* const* T, uint64_t K,
                               const uint64_t* D, const uint64_t* N, uint8_t* proof, uint64_t cap, uint64_t* len,
                               uint8_t* aux, uint8_t* v_out, uint64_t* bad_instance, uint64_t* bad_index, int threads) {
    return tlookup_multi_prove(seed, reinterpret_cast<const Fr* const*>(S), reinterpret_cast<const Fr* const*>(T), K, D,
                               N, proof, cap, len, aux ? as_fr(aux) : nullptr, v_out ? as_fr(v_out) : nullptr,
                               bad_instance, bad_index, threads);
}

int oracle_tlookup_multi_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, const uint8_t* const* T,
                                uint64_t K, const uint64_t* D, const uint64_t* N, const uint8_t* const* S,
                                const uint64_t* const* m_counts, uint8_t* v_out, int threads) {
    return tlookup_multi_verify(seed, proof, len, reinterpret_cast<const Fr* const*>(T), K, D, N,
                                reinterpret_cast<const Fr* const*>(S), m_counts, v_out ? as_fr(v_out) : nullptr,
                                threads);
}

uint64_t oracle_product_proof_bytes(uint64_t n) { return product_proof_bytes(log2_exact(n)); }
uint64_t oracle_matmul_proof_bytes(uint64_t D1) { return matmul_proof_bytes(ceil_log2(D1)); }

int oracle_sumcheck_prove_product(const uint8_t seed[32], const uint8_t* a, const uint8_t* b, uint64_t n,
                                  const uint8_t claim[32], uint8_t* proof, uint64_t cap, uint64_t* len,
                                  uint8_t* r_out, int threads) {
    Fr c = fr_from_bytes(claim);
    return sumcheck_prove_product(seed, as_fr(a), as_fr(b), n, &c, proof, cap, len,
                                  r_out ? as_fr(r_out) : nullptr, threads);
}
int oracle_sumcheck_verify_product(const uint8_t seed[32], const uint8_t* proof, uint64_t len, uint64_t n,
                                   const uint8_t* a, const uint8_t* b, uint8_t* r_out, int threads) {
    return sumcheck_verify_product(seed, proof, len, n, a ? as_fr(a) : nullptr, b ? as_fr(b) : nullptr,
                                   r_out ? as_fr(r_out) : nullptr, threads);
}
int oracle_matmul_sumcheck_prove(const uint8_t seed[32], const int64_t* X, uint64_t D0, uint64_t D1,
                                 const int64_t* W, uint64_t D2, uint8_t* proof, uint64_t cap, uint64_t* len,
                                 uint8_t* u_out, uint8_t* v_out, uint8_t* r_out, int threads) {
    return matmul_sumcheck_prove(seed, X, D0, D1, W, D2, proof, cap, len, u_out ? as_fr(u_out) : nullptr,
                                 v_out ? as_fr(v_out) : nullptr, r_out ? as_fr(r_out) : nullptr, threads);
}
int oracle_matmul_sumcheck_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, uint64_t D0,
                                  uint64_t D1, uint64_t D2, const uint8_t* Y, const int64_t* X, const int64_t* W,
                                  int threads) {
    return matmul_sumcheck_verify(seed, proof, len, D0, D1, D2, Y ? as_fr(Y) : nullptr, X, W, threads);
}

uint64_t oracle_link_proof_bytes(uint64_t rows, uint64_t cols, uint64_t K) {
    return link_proof_bytes(log2_exact(rows) + log2_exact(cols), (int)K);
}
// X, Yk: arrays of K pointers; bases: K elements.
int oracle_zkattn_link_prove(const uint8_t seed[32], const uint8_t* Zp, const uint8_t* const* X, const uint8_t* Y,
                             const uint8_t* const* Yk, const uint8_t* yhat, const uint8_t* bases, uint64_t rows,
                             uint64_t cols, uint64_t K, uint8_t* proof, uint64_t cap, uint64_t* len, uint8_t* point_out,
                             int threads) {
    return zkattn_link_prove(seed, as_fr(Zp), reinterpret_cast<const Fr* const*>(X), as_fr(Y),
                             reinterpret_cast<const Fr* const*>(Yk), as_fr(yhat), as_fr(bases), rows, cols, (int)K, proof,
                             cap, len, point_out ? as_fr(point_out) : nullptr, threads);
}
// Any of Zp, X (or its entries), Y, Yk (or its entries), yhat may be null.
int oracle_zkattn_link_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, uint64_t rows, uint64_t cols,
                              uint64_t K, const uint8_t* bases, const uint8_t* Zp, const uint8_t* const* X,
                              const uint8_t* Y, const uint8_t* const* Yk, const uint8_t* yhat, uint8_t* point_out,
                              int threads) {
    return zkattn_link_verify(seed, proof, len, rows, cols, (int)K, as_fr(bases), Zp ? as_fr(Zp) : nullptr,
                              reinterpret_cast<const Fr* const*>(X), Y ? as_fr(Y) : nullptr,
                              reinterpret_cast<const Fr* const*>(Yk), yhat ? as_fr(yhat) : nullptr,
                              point_out ? as_fr(point_out) : nullptr, threads);
}

}  // extern "C"
