// Product sumcheck (Section 3.3 of the paper) and the matrix-multiplication
// proof built on it (Section 6.1.1):
//   Y~(u,v) = sum_k X~(u,k) W~(k,v),  a_k = X~(u,k) = sum_i e~(u,i) X[i,k],
//                                      b_k = W~(k,v) = sum_j W[k,j] e~(v,j).
#include "internal.h"
#include "tlookup_kernels.h"
#include "transcript.h"

namespace zkmi {

struct ProductRoundArgs {
    PairArray a, b;
    size_t half;
    size_t block_span;
    Fr r_prev;
    uint32_t* partials;  // 3 values per workgroup
    size_t pstride;
};

// g(0) = sum a0 b0, g(1) = sum a1 b1 and the leading coefficient sum (a1-a0)(b1-b0).
template <bool FOLD>
__global__ void __launch_bounds__(kBlock) k_round_product(ProductRoundArgs g) {
    __shared__ uint32_t lds[4 * 3 * 8];
    Fr tot[3] = {fr_zero(), fr_zero(), fr_zero()};
    const size_t start = blockIdx.x * g.block_span;
    for (size_t p = start + threadIdx.x; p < start + g.block_span; p += kBlock) {
        Fr a0, a1, b0, b1;
        load_pair<FOLD>(g.a, p, g.half, g.r_prev, a0, a1);
        load_pair<FOLD>(g.b, p, g.half, g.r_prev, b0, b1);
        tot[0] = fr_add(tot[0], fr_mul(a0, b0));
        tot[1] = fr_add(tot[1], fr_mul(a1, b1));
        tot[2] = fr_add(tot[2], fr_mul(fr_sub(a1, a0), fr_sub(b1, b0)));
    }
    block_sum<3, 4>(tot, lds);
    if (threadIdx.x == 0) {
#pragma unroll
        for (int q = 0; q < 3; ++q) fr_store(g.partials, g.pstride, (size_t)blockIdx.x * 3 + q, tot[q]);
    }
}

static size_t product_scratch_bytes() {
    Carver cv(nullptr, 0);
    cv.limbs((size_t)kMaxPartialBlocks * 3);
    cv.take(256);  // ticket of the final sums
    return cv.used();
}

// d rounds over a and b (2^d elements, stride given, folded in place).  The
// claim is absorbed here: either the caller's, or (claim == nullptr) the one
// the first round's sums imply, g(0) + g(1); it is written to claim_bytes.
// `out` receives d x 3 round values and the two final values.
static int product_rounds_run(host::Transcript& tr, uint32_t* a, size_t as, uint32_t* b, size_t bs, int d,
                              const host::F* claim, uint8_t* claim_bytes, uint8_t* out, Carver& cv, Mailbox* mb,
                              hipStream_t stream) {
    using namespace host;
    uint32_t* partials = cv.limbs((size_t)kMaxPartialBlocks * 3);
    uint32_t* ticket = (uint32_t*)cv.take(256);
    if (!partials || !ticket) return ZK_E_BUFSZ;
    launch_fill_u32(ticket, 1, 0u, stream);
    const size_t pstride = (size_t)kMaxPartialBlocks * 3;
    F r_prev = zero();
    bool claim_done = false;
    if (claim) {
        to_bytes(claim_bytes, *claim);
        tr.absorb("claim", claim_bytes, 32);
        claim_done = true;
    }
    for (int k = 0; k < d; ++k) {
        const size_t half = (size_t)1 << (d - k - 1);
        size_t span = half / kMaxPartialBlocks;
        if (span < (size_t)kBlock * 4) span = (size_t)kBlock * 4;
        if (span > half) span = half;
        const unsigned blocks = (unsigned)(half / span);
        ProductRoundArgs g;
        g.a = PairArray{a, as, a, as};
        g.b = PairArray{b, bs, b, bs};
        g.half = half;
        g.block_span = span;
        g.r_prev = to_dev(r_prev);
        g.partials = partials;
        g.pstride = pstride;
        if (k > 0) hipLaunchKernelGGL(k_round_product<true>, dim3(blocks), dim3(kBlock), 0, stream, g);
        else hipLaunchKernelGGL(k_round_product<false>, dim3(blocks), dim3(kBlock), 0, stream, g);
        const uint32_t seq = mb->next_seq();
        launch_final_sum(partials, pstride, blocks, 3, mb->words, mb->words, seq, ticket, stream);
        ZK_HIP_TRY(hipGetLastError());
        ZK_TRY(mailbox_wait(mb, seq, stream));
        F g0 = from_dev(mb->words), g1 = from_dev(mb->words + 8), lead = from_dev(mb->words + 16);
        if (!claim_done) {
            to_bytes(claim_bytes, add(g0, g1));
            tr.absorb("claim", claim_bytes, 32);
            claim_done = true;
        }
        F g2 = add(sub(add(g1, g1), g0), add(lead, lead));
        to_bytes(out, g0);
        to_bytes(out + 32, g1);
        to_bytes(out + 64, g2);
        tr.absorb("g", out, 96);
        out += 96;
        r_prev = tr.challenge("r");
    }
    FinalArgs f;
    memset(&f, 0, sizeof f);
    f.count = 2;
    f.r = to_dev(r_prev);
    f.p[0] = a; f.stride[0] = as; f.fold[0] = d >= 1;
    f.p[1] = b; f.stride[1] = bs; f.fold[1] = d >= 1;
    const uint32_t seq = mb->next_seq();
    hipLaunchKernelGGL(k_final_values, dim3(1), dim3(64), 0, stream, f, mb->words, mb->words, seq);
    ZK_HIP_TRY(hipGetLastError());
    ZK_TRY(mailbox_wait(mb, seq, stream));
    ZK_HIP_TRY(hipStreamSynchronize(stream));  // everything of this call has left the device
    F fa = from_dev(mb->words), fb = from_dev(mb->words + 8);
    if (!claim_done) {  // d == 0: the sum is the single product
        to_bytes(claim_bytes, mul(fa, fb));
        tr.absorb("claim", claim_bytes, 32);
    }
    to_bytes(out, fa);
    to_bytes(out + 32, fb);
    tr.absorb("final", out, 64);
    return ZK_OK;
}

// Host replay of d product rounds.  el: d*3 round values then 2 final values.
static bool product_rounds_check(host::Transcript& tr, const uint8_t* body, int d, host::F claim, host::F* point,
                                 host::F fin[2]) {
    using namespace host;
    for (int k = 0; k < d; ++k) {
        F g[3];
        for (int X = 0; X < 3; ++X)
            if (!from_bytes(&g[X], body + 96 * k + 32 * X)) return false;
        if (!equal(add(g[0], g[1]), claim)) return false;
        tr.absorb("g", body + 96 * k, 96);
        point[k] = tr.challenge("r");
        claim = interpolate_at(g, 3, point[k]);
    }
    if (!from_bytes(&fin[0], body + 96 * d) || !from_bytes(&fin[1], body + 96 * d + 32)) return false;
    tr.absorb("final", body + 96 * d, 64);
    return equal(mul(fin[0], fin[1]), claim);
}

// ---- partial evaluations of a matrix -------------------------------------------------------

// part[c][k] = sum over rows i of chunk c of e[i] * X[i][k]; thread per column.
__global__ void __launch_bounds__(kBlock) k_colsum_partial(const uint32_t* __restrict__ X, size_t xs, size_t D0,
                                                           size_t D1, const uint32_t* __restrict__ e, size_t es,
                                                           size_t rows_per_chunk, uint32_t* __restrict__ part,
                                                           size_t ps, size_t P1) {
    size_t k = blockIdx.x * (size_t)kBlock + threadIdx.x;
    if (k >= D1) return;
    size_t i0 = blockIdx.y * rows_per_chunk, i1 = i0 + rows_per_chunk;
    if (i1 > D0) i1 = D0;
    Fr acc = fr_zero();
    for (size_t i = i0; i < i1; ++i) acc = fr_add(acc, fr_mul(fr_load(e, es, i), fr_load(X, xs, i * D1 + k)));
    fr_store(part, ps, blockIdx.y * P1 + k, acc);
}

// a[k] = sum_c part[c][k] for k < D1, zero for D1 <= k < P1.
__global__ void __launch_bounds__(kBlock) k_colsum_reduce(uint32_t* __restrict__ a, size_t as,
                                                          const uint32_t* __restrict__ part, size_t ps, size_t chunks,
                                                          size_t D1, size_t P1) {
    size_t k = blockIdx.x * (size_t)kBlock + threadIdx.x;
    if (k >= P1) return;
    Fr acc = fr_zero();
    if (k < D1)
        for (size_t c = 0; c < chunks; ++c) acc = fr_add(acc, fr_load(part, ps, c * P1 + k));
    fr_store(a, as, k, acc);
}

// b[k] = sum_j W[k][j] e[j]; one workgroup per row; rows D1 <= k < P1 are zero.
__global__ void __launch_bounds__(kBlock) k_rowdot(uint32_t* __restrict__ b, size_t bs, const uint32_t* __restrict__ W,
                                                   size_t ws, size_t D1, size_t D2, const uint32_t* __restrict__ e,
                                                   size_t es) {
    __shared__ uint32_t lds[4 * 8];
    size_t k = blockIdx.x;
    Fr acc[1] = {fr_zero()};
    if (k < D1)
        for (size_t j = threadIdx.x; j < D2; j += kBlock)
            acc[0] = fr_add(acc[0], fr_mul(fr_load(W, ws, k * D2 + j), fr_load(e, es, j)));
    block_sum<1, 4>(acc, lds);
    if (threadIdx.x == 0) fr_store(b, bs, k, acc[0]);
}

__global__ void __launch_bounds__(kBlock) k_dot_partial(const uint32_t* __restrict__ x, size_t xs,
                                                        const uint32_t* __restrict__ y, size_t ys, size_t n,
                                                        uint32_t* __restrict__ partials, size_t pstride) {
    __shared__ uint32_t lds[4 * 8];
    Fr acc[1] = {fr_zero()};
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
        acc[0] = fr_add(acc[0], fr_mul(fr_load(x, xs, i), fr_load(y, ys, i)));
    block_sum<1, 4>(acc, lds);
    if (threadIdx.x == 0) fr_store(partials, pstride, blockIdx.x, acc[0]);
}

static const size_t kColChunks = 64;

struct MatmulWs {
    uint32_t *eu, *ev, *a, *b, *part, *dot;
    size_t P0, P1, P2;
};

static void carve_matmul(MatmulWs& w, Carver& cv, size_t D0, size_t D1, size_t D2) {
    w.P0 = (size_t)1 << log2_ceil(D0);
    w.P1 = (size_t)1 << log2_ceil(D1);
    w.P2 = (size_t)1 << log2_ceil(D2);
    w.eu = cv.limbs(w.P0);
    w.ev = cv.limbs(w.P2);
    w.a = cv.limbs(w.P1);
    w.b = cv.limbs(w.P1);
    size_t widest = w.P1 > w.P2 ? w.P1 : w.P2;
    w.part = cv.limbs(kColChunks * widest);
    w.dot = cv.limbs(kMaxPartialBlocks);
}

// a_k = sum_i e0[i] M[i][k] over an R x C row-major matrix, into `a` (PC entries, zero padded).
static void colsum_run(uint32_t* a, size_t PC, const uint32_t* M, size_t ms, size_t R, size_t C, const uint32_t* e0,
                       size_t e0s, uint32_t* part, hipStream_t stream) {
    size_t rows_per_chunk = div_up(R, kColChunks);
    size_t chunks = div_up(R, rows_per_chunk);
    hipLaunchKernelGGL(k_colsum_partial, dim3((unsigned)div_up(C, kBlock), (unsigned)chunks), dim3(kBlock), 0, stream, M,
                       ms, R, C, e0, e0s, rows_per_chunk, part, kColChunks * PC, PC);
    hipLaunchKernelGGL(k_colsum_reduce, dim3((unsigned)div_up(PC, kBlock)), dim3(kBlock), 0, stream, a, PC, part,
                       kColChunks * PC, chunks, C, PC);
}

static void rowdot_run(uint32_t* b, size_t PR, const uint32_t* M, size_t ms, size_t R, size_t C, const uint32_t* e1,
                       size_t e1s, hipStream_t stream) {
    hipLaunchKernelGGL(k_rowdot, dim3((unsigned)PR), dim3(kBlock), 0, stream, b, PR, M, ms, R, C, e1, e1s);
}

static int dot_run(const uint32_t* x, size_t xs, const uint32_t* y, size_t ys, size_t n, uint32_t* partials,
                   uint32_t* out_words, hipStream_t stream) {
    unsigned blocks = grid_for(n, kBlock * 4, kMaxPartialBlocks);
    hipLaunchKernelGGL(k_dot_partial, dim3(blocks), dim3(kBlock), 0, stream, x, xs, y, ys, n, partials,
                       (size_t)kMaxPartialBlocks);
    launch_final_sum(partials, kMaxPartialBlocks, blocks, 1, out_words, out_words, 0, nullptr, stream);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

}  // namespace zkmi

using namespace zkmi;

extern "C" {

size_t sumcheck_product_proof_bytes(size_t n) { return 16 + 32 + (size_t)log2_floor(n ? n : 1) * 96 + 64; }
size_t sumcheck_product_workspace_bytes(size_t) { return product_scratch_bytes(); }

int sumcheck_prove_product(const uint8_t seed[32], fr_vec a, fr_vec b, const fr_t* claim, uint8_t* proof, size_t cap,
                           size_t* len, void* ws, size_t ws_bytes, void* stream) {
    const size_t n = a.n;
    if (!seed || !claim || !is_pow2(n) || b.n != n || !vec_ok(a, n) || !vec_ok(b, n)) return ZK_E_BADARG;
    if (n > ((size_t)1 << 31) || !host::canonical_in_range(*claim)) return ZK_E_BADARG;
    const int d = log2_floor(n);
    const size_t need = sumcheck_product_proof_bytes(n);
    if (len) *len = need;
    if (!proof || cap < need) return ZK_E_BUFSZ;
    if (!ws || ws_bytes < product_scratch_bytes()) return ZK_E_BUFSZ;
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(ws, ws_bytes);
    uint64_t dims[1] = {(uint64_t)d};
    host::Transcript tr("zkmi/sumcheck-product/v1", seed, dims, 1);
    memcpy(proof, "ZKSP\x01\0\0\0", 8);
    host::put_le64(proof + 8, (uint64_t)d);
    host::F c = host::from_canonical(*claim);
    return product_rounds_run(tr, a.limbs, a.stride, b.limbs, b.stride, d, &c, proof + 16, proof + 48, cv, mb,
                              as_stream(stream));
}

int sumcheck_verify_product(const uint8_t seed[32], const uint8_t* proof, size_t len, size_t n, fr_t final_claims[2],
                            fr_t* point) {
    if (!seed || !proof || !is_pow2(n) || n > ((size_t)1 << 31)) return ZK_E_BADARG;
    const int d = log2_floor(n);
    if (len != sumcheck_product_proof_bytes(n)) return ZK_E_REJECT;
    if (memcmp(proof, "ZKSP\x01\0\0\0", 8) != 0 || host::get_le64(proof + 8) != (uint64_t)d) return ZK_E_REJECT;
    host::F claim;
    if (!host::from_bytes(&claim, proof + 16)) return ZK_E_REJECT;
    uint64_t dims[1] = {(uint64_t)d};
    host::Transcript tr("zkmi/sumcheck-product/v1", seed, dims, 1);
    tr.absorb("claim", proof + 16, 32);
    host::F pt[32], fin[2];
    if (!product_rounds_check(tr, proof + 48, d, claim, pt, fin)) return ZK_E_REJECT;
    if (final_claims) {
        final_claims[0] = host::to_canonical(fin[0]);
        final_claims[1] = host::to_canonical(fin[1]);
    }
    if (point)
        for (int k = 0; k < d; ++k) point[k] = host::to_canonical(pt[k]);
    return ZK_OK;
}

size_t matmul_proof_bytes(size_t D1) { return 32 + 32 + (size_t)log2_ceil(D1 ? D1 : 1) * 96 + 64; }

size_t matmul_workspace_bytes(size_t D0, size_t D1, size_t D2) {
    if (!D0 || !D1 || !D2) return 0;
    Carver cv(nullptr, 0);
    MatmulWs w;
    carve_matmul(w, cv, D0, D1, D2);
    cv.limbs((size_t)kMaxPartialBlocks * 3);  // round partial sums (prover)
    cv.take(256);                             // ticket of the final sums
    cv.limbs(w.P2);                           // column sums of Y (verifier)
    cv.limbs(w.P1);                           // e~(r, .) (verifier)
    return cv.used();
}

static bool matmul_dims_ok(size_t D0, size_t D1, size_t D2) {
    const size_t lim = (size_t)1 << 31;
    return D0 && D1 && D2 && D0 <= lim && D1 <= lim && D2 <= lim && D0 * D1 / D1 == D0 && D1 * D2 / D2 == D1;
}

int matmul_sumcheck_prove(const uint8_t seed[32], fr_vec X, size_t D0, size_t D1, fr_vec W, size_t D2, uint8_t* proof,
                          size_t cap, size_t* len, void* ws, size_t ws_bytes, void* stream_v) {
    if (!seed || !matmul_dims_ok(D0, D1, D2) || !vec_ok(X, D0 * D1) || !vec_ok(W, D1 * D2)) return ZK_E_BADARG;
    const int n0 = log2_ceil(D0), n1 = log2_ceil(D1), n2 = log2_ceil(D2);
    const size_t need = matmul_proof_bytes(D1);
    if (len) *len = need;
    if (!proof || cap < need) return ZK_E_BUFSZ;
    if (!ws || ws_bytes < matmul_workspace_bytes(D0, D1, D2)) return ZK_E_BUFSZ;
    hipStream_t stream = as_stream(stream_v);
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(ws, ws_bytes);
    MatmulWs w;
    carve_matmul(w, cv, D0, D1, D2);
    uint64_t dims[3] = {D0, D1, D2};
    host::Transcript tr("zkmi/matmul/v1", seed, dims, 3);
    host::F u[32], v[32];
    for (int t = 0; t < n0; ++t) u[t] = tr.challenge("u");
    for (int t = 0; t < n2; ++t) v[t] = tr.challenge("v");
    ZK_TRY(eq_table_run(w.eu, w.P0, u, n0, stream));
    ZK_TRY(eq_table_run(w.ev, w.P2, v, n2, stream));
    colsum_run(w.a, w.P1, X.limbs, X.stride, D0, D1, w.eu, w.P0, w.part, stream);
    rowdot_run(w.b, w.P1, W.limbs, W.stride, D1, D2, w.ev, w.P2, stream);
    ZK_HIP_TRY(hipGetLastError());
    memcpy(proof, "ZKMM\x01\0\0\0", 8);
    host::put_le64(proof + 8, D0);
    host::put_le64(proof + 16, D1);
    host::put_le64(proof + 24, D2);
    return product_rounds_run(tr, w.a, w.P1, w.b, w.P1, n1, nullptr, proof + 32, proof + 64, cv, mb, stream);
}

size_t matmul_verify_workspace_bytes(size_t D0, size_t D1, size_t D2) { return matmul_workspace_bytes(D0, D1, D2); }

int matmul_sumcheck_verify(const uint8_t seed[32], const uint8_t* proof, size_t len, size_t D0, size_t D1, size_t D2,
                           fr_vec Y, fr_vec X, fr_vec W, void* ws, size_t ws_bytes, void* stream_v) {
    using namespace host;
    if (!seed || !proof || !matmul_dims_ok(D0, D1, D2)) return ZK_E_BADARG;
    const int n0 = log2_ceil(D0), n1 = log2_ceil(D1), n2 = log2_ceil(D2);
    if (len != matmul_proof_bytes(D1) || memcmp(proof, "ZKMM\x01\0\0\0", 8) != 0) return ZK_E_REJECT;
    if (get_le64(proof + 8) != D0 || get_le64(proof + 16) != D1 || get_le64(proof + 24) != D2) return ZK_E_REJECT;
    F claim;
    if (!from_bytes(&claim, proof + 32)) return ZK_E_REJECT;
    uint64_t dims[3] = {D0, D1, D2};
    Transcript tr("zkmi/matmul/v1", seed, dims, 3);
    F u[32], v[32], r[32], fin[2];
    for (int t = 0; t < n0; ++t) u[t] = tr.challenge("u");
    for (int t = 0; t < n2; ++t) v[t] = tr.challenge("v");
    tr.absorb("claim", proof + 32, 32);
    if (!product_rounds_check(tr, proof + 64, n1, claim, r, fin)) return ZK_E_REJECT;
    const bool want_Y = Y.limbs != nullptr, want_X = X.limbs != nullptr, want_W = W.limbs != nullptr;
    if (!want_Y && !want_X && !want_W) return ZK_OK;
    if ((want_Y && !vec_ok(Y, D0 * D2)) || (want_X && !vec_ok(X, D0 * D1)) || (want_W && !vec_ok(W, D1 * D2)))
        return ZK_E_BADARG;
    if (!ws || ws_bytes < matmul_workspace_bytes(D0, D1, D2)) return ZK_E_BUFSZ;
    hipStream_t stream = as_stream(stream_v);
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(ws, ws_bytes);
    MatmulWs w;
    carve_matmul(w, cv, D0, D1, D2);
    ZK_TRY(eq_table_run(w.eu, w.P0, u, n0, stream));
    ZK_TRY(eq_table_run(w.ev, w.P2, v, n2, stream));
    // Y~(u,v) = sum_j (sum_i e~(u,i) Y[i][j]) e~(v,j)
    if (want_Y) {
        uint32_t* ycols = cv.limbs(w.P2);
        if (!ycols) return ZK_E_BUFSZ;
        colsum_run(ycols, w.P2, Y.limbs, Y.stride, D0, D2, w.eu, w.P0, w.part, stream);
        ZK_TRY(dot_run(ycols, w.P2, w.ev, w.P2, D2, w.dot, mb->words, stream));
        ZK_HIP_TRY(hipStreamSynchronize(stream));
        if (!equal(from_dev(mb->words), claim)) return ZK_E_REJECT;
    }
    if (want_X || want_W) {
        uint32_t* er = cv.limbs(w.P1);
        if (!er) return ZK_E_BUFSZ;
        ZK_TRY(eq_table_run(er, w.P1, r, n1, stream));
        if (want_X) {
            colsum_run(w.a, w.P1, X.limbs, X.stride, D0, D1, w.eu, w.P0, w.part, stream);
            ZK_TRY(dot_run(w.a, w.P1, er, w.P1, D1, w.dot, mb->words, stream));
            ZK_HIP_TRY(hipStreamSynchronize(stream));
            if (!equal(from_dev(mb->words), fin[0])) return ZK_E_REJECT;
        }
        if (want_W) {
            rowdot_run(w.b, w.P1, W.limbs, W.stride, D1, D2, w.ev, w.P2, stream);
            ZK_TRY(dot_run(w.b, w.P1, er, w.P1, D1, w.dot, mb->words, stream));
            ZK_HIP_TRY(hipStreamSynchronize(stream));
            if (!equal(from_dev(mb->words), fin[1])) return ZK_E_REJECT;
        }
    }
    return ZK_OK;
}

}  // extern "C"
