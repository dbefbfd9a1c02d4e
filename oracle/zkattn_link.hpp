// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// The sumcheck that closes zkAttn-Prove (Protocol 2, last step; Section 5.1 for
// the relations).  For an attention-score matrix of `rows` x `cols` entries
// (both powers of two, flattened row-major, D = rows * cols) and K segments the
// prover holds
//     Z'            the shifted scores (Z minus the row-wise constant),
//     X^(k), Y^(k)  the k-th digit of -Z' and its table output, k < K,
//     Y             the product of the Y^(k),
//     yhat          the row sums of Y,
// and shows, for public bases B^(k) (B^(0) = 1 in the paper's decomposition),
//     Z'_x + sum_k B^(k) X^(k)_x = 0        (the decomposition is valid),
//     Y_x = prod_k Y^(k)_x                  (the factors multiply to the output),
//     yhat_i = sum_j Y_(i,j)                (the row sums).
// The paper names these relations and says "run the sumcheck"; the batching is
// the standard one (Section 3.3: a random point and a random linear
// combination): with u in F^(log2 D) and alpha from the transcript,
//
//   alpha^2 yhat~(u_rows) = sum_x [ e~(u,x) ( Z'(x) + sum_k B^(k) X^(k)(x) )
//                                  + alpha e~(u,x) ( Y(x) - prod_k Y^(k)(x) )
//                                  + alpha^2 e~(u_rows, x_rows) Y(x) ],
//
// where u_rows are the first log2(rows) coordinates of u and x_rows the row
// bits of x.  Each summand is a polynomial of degree <= K + 1 in every variable,
// so a round polynomial is sent as its values at X = 0 .. K+1.  The segments
// without a table output (the paper's L least significant ones) are the case
// Y^(k) = 1 and are not treated separately here.
//
// Transcript: SHA256("zkmi/zkattn-link/v1" || seed || LE64 rows || LE64 cols ||
// LE64 K || B^(0..K-1)); u_t = challenge("u"); absorb("yhat", yhat~(u_rows));
// alpha = challenge("alpha"); per round absorb("g", K+2 values), r =
// challenge("r"); absorb("final", the 2K+2 claims).
//
// Proof bytes:
//   "ZKAL" | u32 version=1 | LE64 rows | LE64 cols | LE64 K | yhat~(u_rows)
//          | n x (K+2) round values | Z'~(v) X^(0..K-1)~(v) Y~(v) Y^(0..K-1)~(v)
#pragma once
#include "tlookup.hpp"

namespace oracle {

static const int LINK_MAX_SEGMENTS = 4;

inline size_t link_proof_bytes(int n, int K) { return 32 + 32 + (size_t)n * (K + 2) * 32 + (size_t)(2 * K + 2) * 32; }

inline Transcript link_transcript(const uint8_t seed[32], uint64_t rows, uint64_t cols, int K, const Fr* bases) {
    Bytes init;
    init.str("zkmi/zkattn-link/v1").raw(seed, 32).le64(rows).le64(cols).le64((uint64_t)K);
    for (int k = 0; k < K; ++k) {
        uint8_t b[32];
        fr_to_bytes(b, bases[k]);
        init.raw(b, 32);
    }
    return Transcript(init);
}

// The summand at one point, given the values of all its parts there.
inline Fr link_summand(const Fr& e, const Fr& erow, const Fr& z, const Fr* x, const Fr& y, const Fr* yk, const Fr* bases,
                       int K, const Fr& alpha) {
    Fr lin = z;
    Fr prod = fr_one();
    for (int k = 0; k < K; ++k) {
        lin = fr_add(lin, fr_mul(bases[k], x[k]));
        prod = fr_mul(prod, yk[k]);
    }
    Fr inner = fr_add(lin, fr_mul(alpha, fr_sub(y, prod)));
    Fr alpha2 = fr_mul(alpha, alpha);
    return fr_add(fr_mul(e, inner), fr_mul(alpha2, fr_mul(erow, y)));
}

// Returns OK, E_BADARG, E_BUFSZ, or E_REJECT when the tensors do not satisfy the
// relations (seen in the first round: the sum is not the claimed one).
inline int zkattn_link_prove(const uint8_t seed[32], const Fr* Zp, const Fr* const* X, const Fr* Y, const Fr* const* Yk,
                             const Fr* yhat, const Fr* bases, uint64_t rows, uint64_t cols, int K, uint8_t* proof,
                             uint64_t cap, uint64_t* len, Fr* point_out, int threads) {
    int nr = log2_exact(rows), nc = log2_exact(cols);
    if (!seed || !Zp || !X || !Y || !Yk || !yhat || !bases || nr < 0 || nc < 0 || K < 1 || K > LINK_MAX_SEGMENTS)
        return E_BADARG;
    const int n = nr + nc;
    const size_t D = (size_t)1 << n;
    size_t need = link_proof_bytes(n, K);
    if (len) *len = need;
    if (!proof || cap < need) return E_BUFSZ;
    const int npts = K + 2;
    int workers = std::max(1, threads);

    Transcript tr = link_transcript(seed, rows, cols, K, bases);
    std::vector<Fr> u(n);
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");
    Fr cy = mle_eval(yhat, nr, u.data(), threads);
    tr.absorb_fr("yhat", &cy, 1);
    Fr alpha = tr.challenge("alpha");
    Fr claim = fr_mul(fr_mul(alpha, alpha), cy);

    // every part of the summand as a table over the cube
    std::vector<Fr> E = eq_table(u.data(), n, threads);
    std::vector<Fr> erow_small = eq_table(u.data(), nr, threads);
    std::vector<Fr> Erow(D);
    for (size_t x = 0; x < D; ++x) Erow[x] = erow_small[x >> nc];
    std::vector<Fr> z(Zp, Zp + D), y(Y, Y + D);
    std::vector<std::vector<Fr>> xs(K), ys(K);
    for (int k = 0; k < K; ++k) {
        xs[k].assign(X[k], X[k] + D);
        ys[k].assign(Yk[k], Yk[k] + D);
    }

    memcpy(proof, "ZKAL", 4);
    proof[4] = 1; proof[5] = proof[6] = proof[7] = 0;
    for (int i = 0; i < 8; ++i) {
        proof[8 + i] = (uint8_t)(rows >> (8 * i));
        proof[16 + i] = (uint8_t)(cols >> (8 * i));
        proof[24 + i] = (uint8_t)((uint64_t)K >> (8 * i));
    }
    fr_to_bytes(proof + 32, cy);
    uint8_t* out = proof + 64;

    for (int round = 0; round < n; ++round) {
        size_t half = E.size() / 2;
        std::vector<std::vector<Fr>> partial(workers, std::vector<Fr>(npts, fr_zero()));
        parallel_ranges(half, workers, [&](size_t lo, size_t hi, int w) {
            std::vector<Fr> acc(npts, fr_zero());
            for (size_t p = lo; p < hi; ++p) {
                // every part is linear in the variable being bound: value at X = a0 + X (a1 - a0)
                Fr e = E[p], de = fr_sub(E[p + half], E[p]);
                Fr er = Erow[p], der = fr_sub(Erow[p + half], Erow[p]);
                Fr zz = z[p], dz = fr_sub(z[p + half], z[p]);
                Fr yy = y[p], dy = fr_sub(y[p + half], y[p]);
                Fr xv[LINK_MAX_SEGMENTS], dx[LINK_MAX_SEGMENTS], yv[LINK_MAX_SEGMENTS], dyk[LINK_MAX_SEGMENTS];
                for (int k = 0; k < K; ++k) {
                    xv[k] = xs[k][p];
                    dx[k] = fr_sub(xs[k][p + half], xs[k][p]);
                    yv[k] = ys[k][p];
                    dyk[k] = fr_sub(ys[k][p + half], ys[k][p]);
                }
                for (int Xp = 0; Xp < npts; ++Xp) {
                    acc[Xp] = fr_add(acc[Xp], link_summand(e, er, zz, xv, yy, yv, bases, K, alpha));
                    e = fr_add(e, de);
                    er = fr_add(er, der);
                    zz = fr_add(zz, dz);
                    yy = fr_add(yy, dy);
                    for (int k = 0; k < K; ++k) {
                        xv[k] = fr_add(xv[k], dx[k]);
                        yv[k] = fr_add(yv[k], dyk[k]);
                    }
                }
            }
            partial[w] = acc;
        });
        std::vector<Fr> g(npts, fr_zero());
        for (auto& pw : partial)
            for (int Xp = 0; Xp < npts; ++Xp) g[Xp] = fr_add(g[Xp], pw[Xp]);
        if (round == 0 && !fr_eq(fr_add(g[0], g[1]), claim)) return E_REJECT;
        for (int Xp = 0; Xp < npts; ++Xp) fr_to_bytes(out + 32 * Xp, g[Xp]);
        out += 32 * npts;
        tr.absorb_fr("g", g.data(), npts);
        Fr r = tr.challenge("r");
        if (point_out) point_out[round] = r;
        fold_top(E, r, threads);
        fold_top(Erow, r, threads);
        fold_top(z, r, threads);
        fold_top(y, r, threads);
        for (int k = 0; k < K; ++k) {
            fold_top(xs[k], r, threads);
            fold_top(ys[k], r, threads);
        }
    }
    std::vector<Fr> fin;
    fin.push_back(z[0]);
    for (int k = 0; k < K; ++k) fin.push_back(xs[k][0]);
    fin.push_back(y[0]);
    for (int k = 0; k < K; ++k) fin.push_back(ys[k][0]);
    if (n == 0) {
        // a single entry: no round has checked the claim
        Fr xv[LINK_MAX_SEGMENTS], yv[LINK_MAX_SEGMENTS];
        for (int k = 0; k < K; ++k) {
            xv[k] = xs[k][0];
            yv[k] = ys[k][0];
        }
        if (!fr_eq(link_summand(E[0], Erow[0], z[0], xv, y[0], yv, bases, K, alpha), claim)) return E_REJECT;
    }
    for (size_t i = 0; i < fin.size(); ++i) fr_to_bytes(out + 32 * i, fin[i]);
    tr.absorb_fr("final", fin.data(), fin.size());
    return OK;
}

// Replays the transcript, checks g(0) + g(1) against the running claim in every
// round and the last claim against the summand at the final point built from the
// 2K+2 stated values.  Tensors that are given (any may be null) have their
// stated value recomputed from the definition of the multilinear extension;
// yhat, if given, is checked against the stated yhat~(u_rows).
inline int zkattn_link_verify(const uint8_t seed[32], const uint8_t* proof, uint64_t len, uint64_t rows, uint64_t cols,
                              int K, const Fr* bases, const Fr* Zp, const Fr* const* X, const Fr* Y,
                              const Fr* const* Yk, const Fr* yhat, Fr* point_out, int threads) {
    int nr = log2_exact(rows), nc = log2_exact(cols);
    if (!seed || !proof || !bases || nr < 0 || nc < 0 || K < 1 || K > LINK_MAX_SEGMENTS) return E_BADARG;
    const int n = nr + nc, npts = K + 2;
    if (len != link_proof_bytes(n, K) || memcmp(proof, "ZKAL\x01\0\0\0", 8) != 0) return E_REJECT;
    uint64_t dims[3] = {0, 0, 0};
    for (int q = 0; q < 3; ++q)
        for (int i = 0; i < 8; ++i) dims[q] |= (uint64_t)proof[8 + 8 * q + i] << (8 * i);
    if (dims[0] != rows || dims[1] != cols || dims[2] != (uint64_t)K) return E_REJECT;
    size_t nfr = 1 + (size_t)n * npts + 2 * K + 2;
    std::vector<Fr> el(nfr);
    for (size_t i = 0; i < nfr; ++i) {
        el[i] = fr_from_bytes(proof + 32 + 32 * i);
        if (!fr_is_canonical(el[i])) return E_REJECT;
    }
    Transcript tr = link_transcript(seed, rows, cols, K, bases);
    std::vector<Fr> u(n), v(n);
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");
    const Fr cy = el[0];
    tr.absorb_fr("yhat", &cy, 1);
    Fr alpha = tr.challenge("alpha");
    Fr claim = fr_mul(fr_mul(alpha, alpha), cy);
    for (int round = 0; round < n; ++round) {
        const Fr* g = &el[1 + (size_t)round * npts];
        if (!fr_eq(fr_add(g[0], g[1]), claim)) return E_REJECT;
        tr.absorb_fr("g", g, npts);
        v[round] = tr.challenge("r");
        claim = lagrange_eval(g, npts, v[round]);
    }
    const Fr* fin = &el[1 + (size_t)n * npts];
    const Fr& fz = fin[0];
    const Fr* fx = fin + 1;
    const Fr& fy = fin[1 + K];
    const Fr* fyk = fin + 2 + K;
    Fr e = eq_at_point(u.data(), v.data(), n), erow = eq_at_point(u.data(), v.data(), nr);
    if (!fr_eq(link_summand(e, erow, fz, fx, fy, fyk, bases, K, alpha), claim)) return E_REJECT;
    if (yhat && !fr_eq(mle_eval(yhat, nr, u.data(), threads), cy)) return E_REJECT;
    if (Zp && !fr_eq(mle_eval(Zp, n, v.data(), threads), fz)) return E_REJECT;
    if (Y && !fr_eq(mle_eval(Y, n, v.data(), threads), fy)) return E_REJECT;
    for (int k = 0; k < K; ++k) {
        if (X && X[k] && !fr_eq(mle_eval(X[k], n, v.data(), threads), fx[k])) return E_REJECT;
        if (Yk && Yk[k] && !fr_eq(mle_eval(Yk[k], n, v.data(), threads), fyk[k])) return E_REJECT;
    }
    if (point_out) for (int t = 0; t < n; ++t) point_out[t] = v[t];
    return OK;
}

}  // namespace oracle
