// The sumcheck that closes zkAttn-Prove (Protocol 2 of the paper, last step):
// one proof that, for a rows x cols score matrix and K digit segments,
//     Z'_x + sum_k B^(k) X^(k)_x = 0,   Y_x = prod_k Y^(k)_x,   yhat_i = sum_j Y_(i,j)
// (the relations of Section 5.1 plus the row sums of Protocol 2's compute step).
// The paper names the relations and leaves the batching open; with u in F^n,
// n = log2(rows cols), and alpha from the transcript the identity proved is
//
//   alpha^2 yhat~(u_rows) = sum_x [ e~(u,x) ( Z'(x) + sum_k B^(k) X^(k)(x) + alpha Y(x) )
//                                  - alpha e~(u,x) prod_k Y^(k)(x)
//                                  + alpha^2 e~(u_rows, x_rows) Y(x) ]
//
// by the generic sumcheck of Section 3.3, degree K+1 per variable, row variables
// (the top index bits) first.
//
// How a round is computed.  With x = (X, rest) after binding t variables,
// e~(u,x) = c_t e~(u_t,X) e_rest(rest), c_t = prod_{s<t} e~(u_s,r_s), and e_rest
// is never folded: while a row variable is being bound it is the product of a
// table over the remaining row variables (one factor per workgroup, a workgroup
// never straddles rows) and the table over all column variables; afterwards it
// is one table over the remaining column variables.  The factor over the row
// variables is at the same time the weight e~(u_rows, .) of the row-sum term.
// Per round the device returns
//     L(0), L(1)        of  L(X) = sum_rest e_rest (Z' + sum_k B^(k) X^(k) + alpha Y)(X,rest)  (linear),
//     Q(0..K)           of  Q(X) = sum_rest e_rest prod_k Y^(k)(X,rest)                        (degree K),
//     sY(0), sY(1)      of  sY(X) = sum_rest [row weight] alpha Y(X,rest)                      (linear),
// and the host forms g(X) = c_t e~(u_t,X) (L(X) - alpha Q(X)) + alpha w(X) sY(X),
// w(X) = c_t e~(u_t,X) in the row rounds and the constant c_(log2 rows) after them.
//
// The linear relation leaves the rounds after the first.  Z' + sum_k B^(k) X^(k)
// is multilinear and zero on the whole cube, hence the zero polynomial: once the
// first round has found its weighted sum to be zero, every folded entry of it is
// zero too, L(X) is alpha times the weighted sum of Y alone, and Z' and the X^(k)
// are neither folded nor read again.  Their values at the final point, which the
// proof ends with, are multilinear evaluations of the tensors as they came
// (k_link_mle: one pass, against two small tables of e~(v, .)), and
// Z'~(v) = - sum_k B^(k) X^(k)~(v).
//
// Y is multiplied by alpha on the way: in the first round on the fly, in the
// second when the folded array is first written; from then on the array holds
// the scaled values (the final claim is scaled back on the host).
#include "internal.h"
#include "small_dev.h"
#include "tlookup_kernels.h"
#include "transcript.h"

namespace zkmi {

static const int kLinkMaxK = 3;

template <int K>
struct LinkRoundArgs {
    PairArray Z, Y;
    PairArray X[K], Yk[K];
    Fr base[K];  // B^(k)
    int scale_x[K];  // 0: B^(k) = 1 (or already applied)
    Fr alpha;
    size_t half;
    size_t block_span;
    Fr r_prev;
    EqSplit eq;
    int row_round;  // the workgroup's high factor also weighs the sums of Y
    uint32_t* partials;  // K + 5 values per workgroup: L0 L1 Q0..QK sY0 sY1
    size_t pstride;
    // The tensors as the integers they are (zkattn_link_prove_small), read by the
    // first two rounds instead of the PairArray sources.
    const int64_t* Zs;
    const uint64_t* Ys;
    const uint32_t* Xs[K];
    const uint32_t* Yks[K];
    // second round: what the integers are folded with by the first challenge, in device
    // memory (as launch arguments they would crowd the scalar registers):
    // [0] scaled by 1 (the Y^(k)), [1] by alpha (Y)
    const SmallFoldConsts* fold;
    uint64_t base_small[K];
    uint32_t yk_bound;   // segment outputs stay below it, so that products of K extrapolated factors fit 63 bits
    Fr raw_scale;        // 2^96: what turns a short-reduced raw sum into its Montgomery form
    uint32_t* bad;       // device word: 1 = a relation fails somewhere, 2 = an entry is out of range
};

// x0 = fold of (in[p], in[p + 2 half]), x1 = fold of (in[p + half], in[p + 3 half]), as field
// elements (scaled, see SmallFoldConsts), written to dst and returned.
__device__ __forceinline__ void small_pair64(const int64_t* __restrict__ in, size_t p, size_t half, const SmallFoldConsts& k,
                                             const PairArray& dst, Fr& x0, Fr& x1) {
    small_fold64(x0.l, in[p], in[p + 2 * half], k);
    small_fold64(x1.l, in[p + half], in[p + 3 * half], k);
    fr_store(dst.dst, dst.ds, p, x0);
    fr_store(dst.dst, dst.ds, p + half, x1);
}
__device__ __forceinline__ void small_pair32(const uint32_t* __restrict__ in, size_t p, size_t half, const SmallFoldConsts& k,
                                             const PairArray& dst, Fr& x0, Fr& x1) {
    small_fold32(x0.l, in[p], in[p + 2 * half], k);
    small_fold32(x1.l, in[p + half], in[p + 3 * half], k);
    fr_store(dst.dst, dst.ds, p, x0);
    fr_store(dst.dst, dst.ds, p + half, x1);
}

// FOLD: bind the previous variable first and write the folded entries back.
// SCALE: the sources hold unscaled X^(k) and Y (the first two rounds).
// SMALL (with FOLD and SCALE, the second round): the sources are the integer tensors.
// LIN: Z' and the X^(k) take part (the first round only, which never folds).
template <int K, bool FOLD, bool SCALE, bool SMALL = false, bool LIN = false>
static __global__ void __launch_bounds__(kBlock) k_link_round(LinkRoundArgs<K> g) {
    static_assert(!SMALL || (FOLD && SCALE), "integer sources are read by the first two rounds only");
    static_assert(!LIN || (!FOLD && !SMALL), "the linear relation is only summed in the first round");
    constexpr int NV = K + 5;
    __shared__ uint32_t lds[4 * NV * 8];
    Fr tot[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) tot[q] = fr_zero();
    const size_t start = blockIdx.x * g.block_span;
    const size_t lo_mask = ((size_t)1 << g.eq.lbits) - 1;
    for (size_t p = start + threadIdx.x; p < start + g.block_span; p += kBlock) {
        const Fr w = fr_load(g.eq.pool, g.eq.stride, g.eq.lo_off + (p & lo_mask));
        Fr lin0 = fr_zero(), lin1 = fr_zero();
        if constexpr (LIN) load_pair<false>(g.Z, p, g.half, g.r_prev, lin0, lin1);
        {
            Fr y0, y1;
            if constexpr (SMALL) small_pair64((const int64_t*)g.Ys, p, g.half, g.fold[1], g.Y, y0, y1);
            else load_pair<FOLD, !SCALE>(g.Y, p, g.half, g.r_prev, y0, y1);
            if constexpr (SCALE && !SMALL) {
                y0 = fr_mul(y0, g.alpha);
                y1 = fr_mul(y1, g.alpha);
                if constexpr (FOLD) {
                    fr_store(g.Y.dst, g.Y.ds, p, y0);
                    fr_store(g.Y.dst, g.Y.ds, p + g.half, y1);
                }
            }
            tot[K + 3] = fr_add(tot[K + 3], y0);
            tot[K + 4] = fr_add(tot[K + 4], y1);
            lin0 = fr_add(lin0, y0);
            lin1 = fr_add(lin1, y1);
        }
        if constexpr (LIN) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                Fr x0, x1;
                load_pair<false>(g.X[k], p, g.half, g.r_prev, x0, x1);
                if (g.scale_x[k]) {
                    x0 = fr_mul(x0, g.base[k]);
                    x1 = fr_mul(x1, g.base[k]);
                }
                lin0 = fr_add(lin0, x0);
                lin1 = fr_add(lin1, x1);
            }
        }
        tot[0] = fr_add(tot[0], fr_mul(w, lin0));
        tot[1] = fr_add(tot[1], fr_mul(w, lin1));
        // the product of the segment outputs at X = 0..K, the weight folded into the first factor
        Fr f[K], d[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            Fr a0, a1;
            if constexpr (SMALL) small_pair32(g.Yks[k], p, g.half, g.fold[0], g.Yk[k], a0, a1);
            else load_pair<FOLD>(g.Yk[k], p, g.half, g.r_prev, a0, a1);
            if (k == 0) {
                a0 = fr_mul(a0, w);
                a1 = fr_mul(a1, w);
            }
            f[k] = a0;
            d[k] = fr_sub(a1, a0);
        }
#pragma unroll
        for (int X = 0; X <= K; ++X) {
            Fr prod = f[0];
#pragma unroll
            for (int k = 1; k < K; ++k) prod = fr_mul(prod, f[k]);
            tot[2 + X] = fr_add(tot[2 + X], prod);
            if (X < K) {
#pragma unroll
                for (int k = 0; k < K; ++k) f[k] = fr_add(f[k], d[k]);
            }
        }
    }
    block_sum<NV, 4>(tot, lds);
    if (threadIdx.x == 0) {
        if (g.eq.has_hi) {
            const Fr hf = fr_load(g.eq.pool, g.eq.stride, g.eq.hi_off + (start >> g.eq.lbits));
#pragma unroll
            for (int q = 0; q < K + 3; ++q) tot[q] = fr_mul(tot[q], hf);
            if (g.row_round) {
                tot[K + 3] = fr_mul(tot[K + 3], hf);
                tot[K + 4] = fr_mul(tot[K + 4], hf);
            }
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) fr_store(g.partials, g.pstride, (size_t)blockIdx.x * NV + q, tot[q]);
    }
}

struct LinkFoldConsts {
    SmallFoldConsts c[2];
};
static __global__ void k_store_fold_consts(LinkFoldConsts v, SmallFoldConsts* dst, int count) {
    const int which = threadIdx.x >> 5, word = threadIdx.x & 31;
    if (which < count) ((uint32_t*)&dst[which])[word] = ((const uint32_t*)&v.c[which])[word];
}

// t += w m.  Values are mostly below 2^32: lanes whose high word is zero skip its
// eight products (the branch is taken by no lane of most wavefronts).
template <int NL>
__device__ __forceinline__ void link_mac(uint32_t (&t)[NL], const Fr& w, uint64_t m) {
    small_mac32<NL, 0>(t, w.l, (uint32_t)m);
    if (m >> 32) small_mac32<NL, 1>(t, w.l, (uint32_t)(m >> 32));
}

// The first round on the integer tensors.  Every entry is checked against the
// relations exactly (Z' + sum_k B^(k) X^(k) = 0 and Y = prod_k Y^(k) as integers),
// so what is left of the round's sums is
//   L(X) = alpha sum w Y(X),  Q(X) = sum w Y(X)  at X = 0, 1,
//   Q(X) = sum w prod_k (Y^(k)_0 + X (Y^(k)_1 - Y^(k)_0))  at X = 2..K,   sY(X) = alpha sum Y(X),
// all of them sums of a weight times a small integer: sixteen multiply-adds per
// term, accumulated unreduced and reduced once per thread.
template <int K>
static __global__ void __launch_bounds__(kBlock) k_link_round0_small(LinkRoundArgs<K> g) {
    constexpr int NV = K + 5, NS = K + 3;  // sums taken here: S0 S1 P2..PK sy0 sy1
    __shared__ uint32_t lds[4 * NS * 8];
    uint32_t s0[12], s1[12], pos[K > 1 ? K - 1 : 1][12], neg[K > 1 ? K - 1 : 1][12];
#pragma unroll
    for (int j = 0; j < 12; ++j) {
        s0[j] = s1[j] = 0;
#pragma unroll
        for (int q = 0; q < K - 1; ++q) pos[q][j] = neg[q][j] = 0;
    }
    unsigned __int128 sy0 = 0, sy1 = 0;
    uint32_t bad = 0;
    const size_t start = blockIdx.x * g.block_span;
    const size_t lo_mask = ((size_t)1 << g.eq.lbits) - 1;
    const int64_t zlim = (int64_t)1 << 62;
    for (size_t p = start + threadIdx.x; p < start + g.block_span; p += kBlock) {
        const Fr w = fr_load(g.eq.pool, g.eq.stride, g.eq.lo_off + (p & lo_mask));
        uint64_t y[2];
        int64_t yk[K][2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const size_t i = p + e * g.half;
            const int64_t z = g.Zs[i];
            y[e] = g.Ys[i];
            if (z <= -zlim || z >= zlim || y[e] >= (uint64_t)zlim) bad |= 2;
            __int128 lin = z;
            uint64_t prod = 1;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                lin += (__int128)g.base_small[k] * g.Xs[k][i];
                const uint32_t v = g.Yks[k][i];
                if (v >= g.yk_bound) bad |= 2;
                yk[k][e] = v;
                prod *= v;  // below 2^63 when every factor is in range (else the entry is reported anyway)
            }
            if (lin != 0 || prod != y[e]) bad |= 1;
        }
        link_mac(s0, w, y[0]);
        link_mac(s1, w, y[1]);
        sy0 += y[0];
        sy1 += y[1];
#pragma unroll
        for (int X = 2; X <= K; ++X) {
            int64_t pr = 1;
#pragma unroll
            for (int k = 0; k < K; ++k) pr *= yk[k][0] + X * (yk[k][1] - yk[k][0]);
            if (pr < 0) link_mac(neg[X - 2], w, 0ull - (uint64_t)pr);
            else link_mac(pos[X - 2], w, (uint64_t)pr);
        }
    }
    if (bad) atomicOr(g.bad, bad);
    // raw sums (below 16 * 2^63 * 2^256 < r 2^96) to field elements
    Fr tot[NS];
    auto to_field = [&](uint32_t (&t)[12]) {
        Fr x;
        small_reduce<3>(x.l, t);
        return fr_mul(x, g.raw_scale);
    };
    tot[0] = to_field(s0);
    tot[1] = to_field(s1);
#pragma unroll
    for (int q = 0; q < K - 1; ++q) tot[2 + q] = fr_sub(to_field(pos[q]), to_field(neg[q]));
    {
        Fr c0 = fr_zero(), c1 = fr_zero();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            c0.l[j] = (uint32_t)(sy0 >> (32 * j));
            c1.l[j] = (uint32_t)(sy1 >> (32 * j));
        }
        tot[K + 1] = fr_to_mont(c0);
        tot[K + 2] = fr_to_mont(c1);
    }
    block_sum<NS, 4>(tot, lds);
    if (threadIdx.x == 0) {
        Fr out[NV];
        Fr S0 = tot[0], S1 = tot[1], y0 = fr_mul(tot[K + 1], g.alpha), y1 = fr_mul(tot[K + 2], g.alpha);
        if (g.eq.has_hi) {
            const Fr hf = fr_load(g.eq.pool, g.eq.stride, g.eq.hi_off + (start >> g.eq.lbits));
            S0 = fr_mul(S0, hf);
            S1 = fr_mul(S1, hf);
#pragma unroll
            for (int q = 0; q < K - 1; ++q) tot[2 + q] = fr_mul(tot[2 + q], hf);
            if (g.row_round) {
                y0 = fr_mul(y0, hf);
                y1 = fr_mul(y1, hf);
            }
        }
        out[0] = fr_mul(S0, g.alpha);
        out[1] = fr_mul(S1, g.alpha);
        out[2] = S0;
        out[3] = S1;
#pragma unroll
        for (int q = 0; q < K - 1; ++q) out[4 + q] = tot[2 + q];
        out[K + 3] = y0;
        out[K + 4] = y1;
#pragma unroll
        for (int q = 0; q < NV; ++q) fr_store(g.partials, g.pstride, (size_t)blockIdx.x * NV + q, out[q]);
    }
}

// X^(k)~(v) for the K digit tensors at once: sum_i e~(v, i) X^(k)_i with
// e~(v, i) = hi[i >> lbits] lo[i & (2^lbits - 1)].  A workgroup takes 2^lbits
// consecutive entries (one value of the high index), workgroup (b, k) writes its
// part of tensor k to partials[b K + k].  SMALL: the tensors are 32-bit integers.
template <bool SMALL>
struct LinkMleArgs {
    const uint32_t* src[kLinkMaxK];  // SMALL: the integers themselves; else eight word planes
    size_t stride[kLinkMaxK];
    int K;
    EqSplit eq;        // lo and hi tables of the point
    Fr raw_scale;      // 2^64 (see SmallFoldConsts): short-reduced raw sums to Montgomery form
    uint32_t* partials;
    size_t pstride;
};

template <bool SMALL>
static __global__ void __launch_bounds__(kBlock) k_link_mle(LinkMleArgs<SMALL> g) {
    __shared__ uint32_t lds[4 * 8];
    const int k = blockIdx.y;
    const size_t span = (size_t)1 << g.eq.lbits;
    const size_t start = blockIdx.x * span;
    Fr tot[1];
    if constexpr (SMALL) {
        uint32_t t[11];
#pragma unroll
        for (int j = 0; j < 11; ++j) t[j] = 0;
        // at most 2^12 / 256 = 16 terms below 2^288 each
        for (size_t c = threadIdx.x; c < span; c += kBlock) {
            const Fr w = fr_load(g.eq.pool, g.eq.stride, g.eq.lo_off + c);
            small_mac32(t, w.l, g.src[k][start + c]);
        }
        Fr x;
        small_reduce<2>(x.l, t);
        tot[0] = fr_mul(x, g.raw_scale);
    } else {
        WideInRegs wide;
        wide.clear();
        for (size_t c = threadIdx.x; c < span; c += kBlock)
            wide.mac(0, fr_load(g.eq.pool, g.eq.stride, g.eq.lo_off + c), fr_load(g.src[k], g.stride[k], start + c));
        tot[0] = wide.finish(0);
    }
    block_sum<1, 4>(tot, lds);
    if (threadIdx.x == 0) {
        if (g.eq.has_hi) tot[0] = fr_mul(tot[0], fr_load(g.eq.pool, g.eq.stride, g.eq.hi_off + blockIdx.x));
        fr_store(g.partials, g.pstride, (size_t)blockIdx.x * g.K + k, tot[0]);
    }
}

// ---- weight tables -------------------------------------------------------------------------
//
// Round t < nr (row variables):  hi over variables t+1 .. nr-1, lo over nr .. n-1.
// Round t >= nr (column variables): lo over variables t+1 .. n-1.
struct LinkTables {
    uint32_t* pool = nullptr;
    size_t stride = 0;
    uint32_t row_off[32];  // hi table of row round t
    uint32_t cols_off = 0; // the table over all column variables
    uint32_t col_off[32];  // lo table of column round t (index t - nr)
    int nr = 0, nc = 0;

    static size_t entries(int nr, int nc) {
        size_t total = 0;
        for (int t = 0; t < nr; ++t) total += (size_t)1 << (nr - t - 1);
        total += (size_t)1 << nc;
        for (int t = 0; t < nc; ++t) total += (size_t)1 << (nc - t - 1);
        return total;
    }

    EqSplit round(int t) const {
        EqSplit e;
        e.pool = pool;
        e.stride = stride;
        if (t < nr) {
            e.lbits = nc;
            e.lo_off = cols_off;
            e.has_hi = 1;
            e.hi_off = row_off[t];
        } else {
            e.lbits = nr + nc - t - 1;
            e.lo_off = col_off[t - nr];
            e.has_hi = 0;
            e.hi_off = 0;
        }
        return e;
    }
};

static int link_tables_build(LinkTables& lt, const host::F* u, int nr, int nc, Carver& cv, hipStream_t stream) {
    lt.nr = nr;
    lt.nc = nc;
    lt.stride = LinkTables::entries(nr, nc);
    lt.pool = cv.limbs(lt.stride);
    if (!lt.pool) return ZK_E_BUFSZ;
    EqPoolArgs args;
    memset(&args, 0, sizeof args);
    const int n = nr + nc;
    for (int t = 0; t < n; ++t) args.u[t] = to_dev(u[t]);
    int q = 0;
    uint32_t off = 0;
    auto table = [&](int var0, int nvars) {
        args.offset[q] = off;
        args.var0[q] = (uint8_t)var0;
        args.nvars[q] = (uint8_t)nvars;
        uint32_t at = off;
        off += 1u << nvars;
        ++q;
        return at;
    };
    for (int t = 0; t < nr; ++t) lt.row_off[t] = table(t + 1, nr - t - 1);
    lt.cols_off = table(nr, nc);
    for (int t = nr; t < n; ++t) lt.col_off[t - nr] = table(t + 1, n - t - 1);
    args.ntables = q;
    args.total = off;
    if (q > 64) return ZK_E_BADARG;
    args.scale = to_dev(host::one());
    hipLaunchKernelGGL(k_eq_pool, dim3(grid_for(off)), dim3(kBlock), 0, stream, lt.pool, lt.stride, args);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

// ---- prover -----------------------------------------------------------------------------------

static size_t link_proof_len(int n, int K) { return 64 + (size_t)n * (K + 2) * 32 + (size_t)(2 * K + 2) * 32; }

static const int kLinkMleLoBits = 12;  // low table of the final point's weights: up to this many variables

struct LinkWs {
    uint32_t* Y;
    uint32_t* Yk[kLinkMaxK];
    uint32_t* mle_tables;    // 2^lb + 2^(n - lb) entries, lb = min(n, kLinkMleLoBits)
    uint32_t* mle_partials;  // K 2^(n - lb) entries
    size_t mle_entries;
    uint32_t* partials;
    uint32_t* ticket;
    SmallFoldConsts* fold;  // 2 + K sets of constants of the integer path
    size_t part_blocks;
};

// Pairs per workgroup in round t: a workgroup's pairs share the high factor of
// their weights, i.e. lie in one row while row variables are being bound.
static size_t link_span(int t, int nr, int nc) {
    const int n = nr + nc;
    const size_t half = (size_t)1 << (n - t - 1);
    const int lbits = t < nr ? nc : n - t - 1;
    size_t span = half / 1024;
    if (span < (size_t)kBlock) span = (size_t)kBlock;
    if (span > ((size_t)1 << lbits)) span = (size_t)1 << lbits;
    if (span > half) span = half;
    return span;
}

static size_t link_blocks_max(int nr, int nc) {
    size_t most = 1;
    for (int t = 0; t < nr + nc; ++t) {
        size_t b = ((size_t)1 << (nr + nc - t - 1)) / link_span(t, nr, nc);
        if (b > most) most = b;
    }
    return most;
}

static void carve_link(LinkWs& w, Carver& cv, size_t D, size_t cols, int K) {
    const size_t h = D / 2 ? D / 2 : 1;
    w.Y = cv.limbs(h);
    for (int k = 0; k < K; ++k) w.Yk[k] = cv.limbs(h);
    {
        const int n = log2_floor(D), lb = n < kLinkMleLoBits ? n : kLinkMleLoBits;
        w.mle_entries = ((size_t)1 << lb) + ((size_t)1 << (n - lb));
        w.mle_tables = cv.limbs(w.mle_entries);
        w.mle_partials = cv.limbs((size_t)K << (n - lb));
    }
    w.part_blocks = link_blocks_max(log2_floor(D / cols), log2_floor(cols));
    w.partials = cv.limbs(w.part_blocks * (K + 5));
    w.ticket = (uint32_t*)cv.take(256);
    w.fold = (SmallFoldConsts*)cv.take(sizeof(SmallFoldConsts) * 2);
}

static size_t link_ws_bytes(size_t rows, size_t cols, int K) {
    Carver cv(nullptr, 0);
    LinkWs w;
    carve_link(w, cv, rows * cols, cols, K);
    cv.limbs(LinkTables::entries(log2_floor(rows), log2_floor(cols)));
    cv.take(mle_scratch_bytes(log2_floor(rows)));
    return cv.used();
}

// Value at X = npts of the polynomial of degree < npts through y[0..npts) at 0..npts-1.
static host::F extrapolate_next(const host::F* y, int npts) {
    using namespace host;
    F d[8];
    for (int j = 0; j < npts; ++j) d[j] = y[j];
    // the npts-th forward difference vanishes: y[npts] = sum of the last entries of the difference table
    F next = zero();
    for (int level = 0; level < npts; ++level) {
        next = add(next, d[npts - 1 - level]);
        for (int j = 0; j + 1 < npts - level; ++j) d[j] = sub(d[j + 1], d[j]);
    }
    return next;
}

// The tensors as device arrays of integers (zkattn_link_prove_small).
struct LinkSmallIn {
    const int64_t* Zp;
    const uint32_t* const* X;
    const uint64_t* Y;
    const uint32_t* const* Yk;
    const uint64_t* bases;
};

static SmallFoldConsts small_fold_consts(const host::F& scale, const host::F& rho) {
    using namespace host;
    const F two32 = from_u64((uint64_t)1 << 32);
    const F a = mul(scale, mul(two32, two32)), d = mul(a, rho);
    SmallFoldConsts k;
    to_device_limbs(k.plus_a, a);
    to_device_limbs(k.minus_a, neg(a));
    to_device_limbs(k.plus_d, d);
    to_device_limbs(k.minus_d, neg(d));
    return k;
}

// small != null: the tensors come as integers (Zp, X, Y, Yk and bases are then unused).
template <int K>
static int link_prove_k(const uint8_t seed[32], fr_vec Zp, const fr_vec* X, fr_vec Y, const fr_vec* Yk, fr_vec yhat,
                        const fr_t* bases, size_t rows, size_t cols, uint8_t* proof, void* ws, size_t ws_bytes,
                        hipStream_t stream, const LinkSmallIn* small = nullptr) {
    using namespace host;
    const int nr = log2_floor(rows), nc = log2_floor(cols), n = nr + nc;
    const size_t D = rows * cols;
    constexpr int NV = K + 5, NPTS = K + 2;
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(ws, ws_bytes);
    LinkWs w;
    carve_link(w, cv, D, cols, K);
    if (cv.overflow()) return ZK_E_BUFSZ;
    launch_fill_u32(w.ticket, 1, 0u, stream);

    F base[K];
    uint64_t dims[3] = {rows, cols, (uint64_t)K};
    uint8_t extra[32 * K];
    for (int k = 0; k < K; ++k) {
        if (small) {
            base[k] = from_u64(small->bases[k]);
        } else {
            if (!canonical_in_range(bases[k])) return ZK_E_BADARG;
            base[k] = from_canonical(bases[k]);
        }
        if (is_zero(base[k])) return ZK_E_BADARG;
        to_bytes(extra + 32 * k, base[k]);
    }
    uint32_t* bad_word = w.ticket + 16;  // within the ticket's 256 bytes
    if (small) launch_fill_u32(bad_word, 1, 0u, stream);
    Transcript tr("zkmi/zkattn-link/v1", seed, dims, 3, extra, sizeof extra);
    F u[32];
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");

    // yhat~(u_rows)
    F cy;
    {
        Carver mcv = cv;
        const uint32_t seq = mb->next_seq();
        ZK_TRY(mle_eval_run(yhat.limbs, yhat.stride, nr, u, mcv, mb, seq, stream));
        ZK_TRY(mailbox_wait(mb, seq, stream));
        cy = from_dev(mb->words);
    }
    uint8_t* out = proof;
    memcpy(out, "ZKAL", 4);
    out[4] = 1; out[5] = out[6] = out[7] = 0;
    put_le64(out + 8, rows);
    put_le64(out + 16, cols);
    put_le64(out + 24, (uint64_t)K);
    to_bytes(out + 32, cy);
    tr.absorb("yhat", out + 32, 32);
    out += 64;
    const F alpha = tr.challenge("alpha");
    if (is_zero(alpha)) return ZK_E_ZERO_DENOM;  // the scaled Y could not be scaled back (probability 1/|F|)
    F claim = mul(sqr(alpha), cy);

    LinkTables lt;
    ZK_TRY(link_tables_build(lt, u, nr, nc, cv, stream));

    F c = one();      // prod_{s<t} e~(u_s, r_s)
    F c_rows = one(); // its value once the row variables are bound
    F r_prev = zero();
    F point[32];      // the challenges: where the final claims are
    for (int t = 0; t < n; ++t) {
        const size_t half = (size_t)1 << (n - t - 1);
        const EqSplit eq = lt.round(t);
        const size_t span = link_span(t, nr, nc);
        const unsigned blocks = (unsigned)(half / span);
        if (blocks > w.part_blocks) return ZK_E_BUFSZ;
        LinkRoundArgs<K> g;
        memset(&g, 0, sizeof g);
        // sources: the caller's tensors in the first two rounds, the workspace afterwards;
        // Z' and the X^(k) are only read by the first round
        const bool from_input = t <= 1 && !small;  // (the integer tensors have sources of their own)
        if (t == 0 && !small) g.Z = PairArray{Zp.limbs, Zp.stride, nullptr, 0};
        g.Y = PairArray{from_input ? Y.limbs : w.Y, from_input ? Y.stride : D / 2, w.Y, D / 2};
        for (int k = 0; k < K; ++k) {
            if (t == 0 && !small) g.X[k] = PairArray{X[k].limbs, X[k].stride, nullptr, 0};
            g.Yk[k] = PairArray{from_input ? Yk[k].limbs : w.Yk[k], from_input ? Yk[k].stride : D / 2, w.Yk[k], D / 2};
            g.base[k] = to_dev(base[k]);
            g.scale_x[k] = equal(base[k], one()) ? 0 : 1;
        }
        g.alpha = to_dev(alpha);
        g.half = half;
        g.block_span = span;
        g.r_prev = to_dev(r_prev);
        g.eq = eq;
        g.row_round = t < nr ? 1 : 0;
        g.partials = w.partials;
        g.pstride = w.part_blocks * NV;
        if (small && t <= 1) {
            g.Zs = small->Zp;
            g.Ys = small->Y;
            for (int k = 0; k < K; ++k) {
                g.Xs[k] = small->X[k];
                g.Yks[k] = small->Yk[k];
                g.base_small[k] = small->bases[k];
            }
            g.fold = w.fold;
            if (t == 1) {
                LinkFoldConsts fc;
                fc.c[0] = small_fold_consts(one(), r_prev);
                fc.c[1] = small_fold_consts(alpha, r_prev);
                hipLaunchKernelGGL(k_store_fold_consts, dim3(1), dim3(64), 0, stream, fc, w.fold, 2);
            }
            g.yk_bound = K == 1 ? 0xffffffffu : K == 2 ? 1u << 30 : 1u << 18;
            const F two32 = from_u64((uint64_t)1 << 32);
            g.raw_scale = to_dev(mul(two32, mul(two32, two32)));
            g.bad = bad_word;
        }
        if (small && t == 0) hipLaunchKernelGGL(k_link_round0_small<K>, dim3(blocks), dim3(kBlock), 0, stream, g);
        else if (small && t == 1) hipLaunchKernelGGL((k_link_round<K, true, true, true>), dim3(blocks), dim3(kBlock), 0, stream, g);
        else if (t == 0) hipLaunchKernelGGL((k_link_round<K, false, true, false, true>), dim3(blocks), dim3(kBlock), 0, stream, g);
        else if (t == 1) hipLaunchKernelGGL((k_link_round<K, true, true>), dim3(blocks), dim3(kBlock), 0, stream, g);
        else hipLaunchKernelGGL((k_link_round<K, true, false>), dim3(blocks), dim3(kBlock), 0, stream, g);
        const uint32_t seq = mb->next_seq();
        launch_final_sum(w.partials, g.pstride, blocks, NV, mb->words, mb->words, seq, w.ticket, stream);
        ZK_HIP_TRY(hipGetLastError());
        ZK_TRY(mailbox_wait(mb, seq, stream));
        if (small && t == 0) {
            // what the first round found entry by entry
            uint32_t bad = 0;
            ZK_HIP_TRY(hipMemcpyAsync(&bad, bad_word, 4, hipMemcpyDeviceToHost, stream));
            ZK_HIP_TRY(hipStreamSynchronize(stream));
            if (bad & 2) return ZK_E_BADARG;  // an entry outside the ranges the integer path is written for
            if (bad & 1) return ZK_E_REJECT;  // the tensors do not satisfy the relations
        }

        F L0 = from_dev(mb->words), L1 = from_dev(mb->words + 8);
        F Q[NPTS];
        for (int pt = 0; pt <= K; ++pt) Q[pt] = from_dev(mb->words + 8 * (2 + pt));
        Q[K + 1] = extrapolate_next(Q, K + 1);
        F s0 = from_dev(mb->words + 8 * (K + 3)), s1 = from_dev(mb->words + 8 * (K + 4));
        F gX[NPTS];
        F e = sub(one(), u[t]), de = sub(u[t], e);  // e~(u_t, X) = (1-u_t) + X (2 u_t - 1)
        F L = L0, dL = sub(L1, L0), s = s0, ds = sub(s1, s0);
        for (int pt = 0; pt < NPTS; ++pt) {
            F ce = mul(c, e);
            F wy = t < nr ? ce : c_rows;
            gX[pt] = add(mul(ce, sub(L, mul(alpha, Q[pt]))), mul(alpha, mul(wy, s)));
            e = add(e, de);
            L = add(L, dL);
            s = add(s, ds);
        }
        if (t == 0 && !equal(add(gX[0], gX[1]), claim)) {
            ZK_HIP_TRY(hipStreamSynchronize(stream));
            return ZK_E_REJECT;  // the tensors do not satisfy the relations
        }
        for (int pt = 0; pt < NPTS; ++pt) to_bytes(out + 32 * pt, gX[pt]);
        tr.absorb("g", out, 32 * NPTS);
        out += 32 * NPTS;
        const F r = tr.challenge("r");
        c = mul(c, add(mul(sub(one(), u[t]), sub(one(), r)), mul(u[t], r)));
        if (t == nr - 1) c_rows = c;
        r_prev = r;
        point[t] = r;
    }

    // -- final claims: Z' X^(0..K-1) Y Y^(0..K-1) at the point of the challenges -----------------
    {
        F fin[2 * kLinkMaxK + 2];
        const bool folded = n >= 2;  // the workspace holds Y and the Y^(k) (Y scaled) once a second round has run
        if (!folded) {
            // at most one round: everything from the tensors as they came
            FinalArgs f;
            memset(&f, 0, sizeof f);
            f.count = 2 * K + 2;
            f.r = to_dev(r_prev);
            auto src = [&](int slot, fr_vec in) {
                f.p[slot] = in.limbs;
                f.stride[slot] = in.stride;
                f.fold[slot] = n >= 1;
            };
            src(0, Zp);
            for (int k = 0; k < K; ++k) src(1 + k, X[k]);
            src(1 + K, Y);
            for (int k = 0; k < K; ++k) src(2 + K + k, Yk[k]);
            const uint32_t seq = mb->next_seq();
            hipLaunchKernelGGL(k_final_values, dim3(1), dim3(64), 0, stream, f, mb->words, mb->words, seq);
            ZK_HIP_TRY(hipGetLastError());
            ZK_TRY(mailbox_wait(mb, seq, stream));
            ZK_HIP_TRY(hipStreamSynchronize(stream));
            for (int q = 0; q < 2 * K + 2; ++q) fin[q] = from_dev(mb->words + 8 * q);
        } else {
            // Y and the Y^(k) from the folded arrays; the X^(k) by evaluating the tensors at the point;
            // Z' from them (the linear relation holds as an identity of multilinear polynomials)
            FinalArgs f;
            memset(&f, 0, sizeof f);
            f.count = K + 1;
            f.r = to_dev(r_prev);
            f.p[0] = w.Y; f.stride[0] = D / 2; f.fold[0] = 1;
            for (int k = 0; k < K; ++k) { f.p[1 + k] = w.Yk[k]; f.stride[1 + k] = D / 2; f.fold[1 + k] = 1; }
            uint32_t seq = mb->next_seq();
            hipLaunchKernelGGL(k_final_values, dim3(1), dim3(64), 0, stream, f, mb->words, mb->words, seq);
            ZK_HIP_TRY(hipGetLastError());
            ZK_TRY(mailbox_wait(mb, seq, stream));
            fin[1 + K] = mul(from_dev(mb->words), inv(alpha));  // scaled back
            for (int k = 0; k < K; ++k) fin[2 + K + k] = from_dev(mb->words + 8 * (1 + k));

            const int lb = n < kLinkMleLoBits ? n : kLinkMleLoBits;
            EqPoolArgs ea;
            memset(&ea, 0, sizeof ea);
            for (int t = 0; t < n; ++t) ea.u[t] = to_dev(point[t]);
            ea.offset[0] = 0; ea.var0[0] = (uint8_t)(n - lb); ea.nvars[0] = (uint8_t)lb;        // low variables
            ea.offset[1] = 1u << lb; ea.var0[1] = 0; ea.nvars[1] = (uint8_t)(n - lb);           // high variables
            ea.ntables = 2;
            ea.total = (uint32_t)w.mle_entries;
            ea.scale = to_dev(one());
            hipLaunchKernelGGL(k_eq_pool, dim3(grid_for(ea.total)), dim3(kBlock), 0, stream, w.mle_tables, w.mle_entries, ea);
            const EqSplit eq{w.mle_tables, w.mle_entries, 0, 1u << lb, lb, 1};
            const unsigned blocks = 1u << (n - lb);
            if (small) {
                LinkMleArgs<true> a;
                memset(&a, 0, sizeof a);
                for (int k = 0; k < K; ++k) a.src[k] = small->X[k];
                a.K = K;
                a.eq = eq;
                const F two32 = from_u64((uint64_t)1 << 32);
                a.raw_scale = to_dev(mul(two32, two32));
                a.partials = w.mle_partials;
                a.pstride = (size_t)K * blocks;
                hipLaunchKernelGGL(k_link_mle<true>, dim3(blocks, K), dim3(kBlock), 0, stream, a);
            } else {
                LinkMleArgs<false> a;
                memset(&a, 0, sizeof a);
                for (int k = 0; k < K; ++k) { a.src[k] = X[k].limbs; a.stride[k] = X[k].stride; }
                a.K = K;
                a.eq = eq;
                a.partials = w.mle_partials;
                a.pstride = (size_t)K * blocks;
                hipLaunchKernelGGL(k_link_mle<false>, dim3(blocks, K), dim3(kBlock), 0, stream, a);
            }
            seq = mb->next_seq();
            launch_final_sum(w.mle_partials, (size_t)K * blocks, blocks, K, mb->words, mb->words, seq, w.ticket, stream);
            ZK_HIP_TRY(hipGetLastError());
            ZK_TRY(mailbox_wait(mb, seq, stream));
            ZK_HIP_TRY(hipStreamSynchronize(stream));  // everything of this call has left the device
            fin[0] = zero();
            for (int k = 0; k < K; ++k) {
                fin[1 + k] = from_dev(mb->words + 8 * k);
                fin[0] = sub(fin[0], mul(base[k], fin[1 + k]));
            }
        }
        if (n == 0) {
            // a single entry: no round has compared the sum with the claim
            F lin = fin[0], prod = one();
            for (int k = 0; k < K; ++k) {
                lin = add(lin, mul(base[k], fin[1 + k]));
                prod = mul(prod, fin[2 + K + k]);
            }
            F val = add(add(lin, mul(alpha, sub(fin[1 + K], prod))), mul(sqr(alpha), fin[1 + K]));
            if (!equal(val, claim)) return ZK_E_REJECT;
        }
        for (int q = 0; q < 2 * K + 2; ++q) to_bytes(out + 32 * q, fin[q]);
        tr.absorb("final", out, 32 * (2 * K + 2));
    }
    return ZK_OK;
}

// Value at x of the polynomial of degree < npts through y[j] at X = j (Newton's
// forward differences: p(x) = sum_j (Delta^j y)(0) binom(x, j)).
static host::F newton_at(const host::F* y, int npts, const host::F& x) {
    using namespace host;
    static const F inv_small[8] = {zero(), one(), inv(from_u64(2)), inv(from_u64(3)), inv(from_u64(4)),
                                   inv(from_u64(5)), inv(from_u64(6)), inv(from_u64(7))};
    F d[8];
    for (int j = 0; j < npts; ++j) d[j] = y[j];
    for (int level = 1; level < npts; ++level)
        for (int j = npts - 1; j >= level; --j) d[j] = sub(d[j], d[j - 1]);
    F acc = d[0], binom = one();
    for (int j = 1; j < npts; ++j) {
        binom = mul(mul(binom, sub(x, from_u64((uint64_t)(j - 1)))), inv_small[j]);
        acc = add(acc, mul(d[j], binom));
    }
    return acc;
}

static int link_verify(const uint8_t seed[32], const uint8_t* proof, size_t len, size_t rows, size_t cols, int K,
                       const fr_t* bases, const zkattn_link_witness* wit, zkattn_link_claims* claims, void* ws,
                       size_t ws_bytes, hipStream_t stream) {
    using namespace host;
    const int nr = log2_floor(rows), nc = log2_floor(cols), n = nr + nc, npts = K + 2;
    const size_t D = rows * cols;
    if (len != link_proof_len(n, K) || memcmp(proof, "ZKAL\x01\0\0\0", 8) != 0) return ZK_E_REJECT;
    if (get_le64(proof + 8) != rows || get_le64(proof + 16) != cols || get_le64(proof + 24) != (uint64_t)K)
        return ZK_E_REJECT;
    F base[kLinkMaxK];
    uint8_t extra[32 * kLinkMaxK];
    for (int k = 0; k < K; ++k) {
        if (!canonical_in_range(bases[k])) return ZK_E_BADARG;
        base[k] = from_canonical(bases[k]);
        to_bytes(extra + 32 * k, base[k]);
    }
    uint64_t dims[3] = {rows, cols, (uint64_t)K};
    Transcript tr("zkmi/zkattn-link/v1", seed, dims, 3, extra, 32 * (size_t)K);
    F u[32], v[32];
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");
    F cy;
    if (!from_bytes(&cy, proof + 32)) return ZK_E_REJECT;
    tr.absorb("yhat", proof + 32, 32);
    const F alpha = tr.challenge("alpha");
    F claim = mul(sqr(alpha), cy);
    const uint8_t* body = proof + 64;
    for (int t = 0; t < n; ++t) {
        F g[8];
        for (int X = 0; X < npts; ++X)
            if (!from_bytes(&g[X], body + 32 * X)) return ZK_E_REJECT;
        if (!equal(add(g[0], g[1]), claim)) return ZK_E_REJECT;
        tr.absorb("g", body, 32 * (size_t)npts);
        body += 32 * npts;
        v[t] = tr.challenge("r");
        claim = newton_at(g, npts, v[t]);
    }
    F fin[2 * kLinkMaxK + 2];
    for (int q = 0; q < 2 * K + 2; ++q)
        if (!from_bytes(&fin[q], body + 32 * q)) return ZK_E_REJECT;
    // the summand at the final point
    F e = one(), erow = one();
    for (int t = 0; t < n; ++t) {
        e = mul(e, add(mul(u[t], v[t]), mul(sub(one(), u[t]), sub(one(), v[t]))));
        if (t == nr - 1) erow = e;
    }
    if (nr == 0) erow = one();
    F lin = fin[0], prod = one();
    for (int k = 0; k < K; ++k) {
        lin = add(lin, mul(base[k], fin[1 + k]));
        prod = mul(prod, fin[2 + K + k]);
    }
    const F& fy = fin[1 + K];
    F val = add(mul(e, add(lin, mul(alpha, sub(fy, prod)))), mul(sqr(alpha), mul(erow, fy)));
    if (!equal(val, claim)) return ZK_E_REJECT;

    if (claims) {
        memset(claims, 0, sizeof *claims);
        claims->nvars = n;
        claims->K = K;
        claims->yhat_u = to_canonical(cy);
        claims->Zp_v = to_canonical(fin[0]);
        claims->Y_v = to_canonical(fy);
        for (int k = 0; k < K; ++k) {
            claims->X_v[k] = to_canonical(fin[1 + k]);
            claims->Yk_v[k] = to_canonical(fin[2 + K + k]);
        }
        for (int t = 0; t < n; ++t) {
            claims->u[t] = to_canonical(u[t]);
            claims->v[t] = to_canonical(v[t]);
        }
    }
    if (!wit) return ZK_OK;

    // tensors standing in for the openings: recompute the stated values from them
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    if (!ws || ws_bytes < mle_scratch_bytes(n)) return ZK_E_BUFSZ;
    Carver cv(ws, ws_bytes);
    auto check = [&](fr_vec a, size_t count, int nv, const F* pt, const F& want) -> int {
        if (!a.limbs) return ZK_OK;
        if (!vec_ok(a, count)) return ZK_E_BADARG;
        Carver scratch = cv;
        uint32_t seq = mb->next_seq();
        ZK_TRY(mle_eval_run(a.limbs, a.stride, nv, pt, scratch, mb, seq, stream));
        ZK_TRY(mailbox_wait(mb, seq, stream));
        ZK_HIP_TRY(hipStreamSynchronize(stream));
        return equal(from_dev(mb->words), want) ? ZK_OK : ZK_E_REJECT;
    };
    ZK_TRY(check(wit->yhat, rows, nr, u, cy));
    ZK_TRY(check(wit->Zp, D, n, v, fin[0]));
    ZK_TRY(check(wit->Y, D, n, v, fy));
    for (int k = 0; k < K; ++k) {
        ZK_TRY(check(wit->X[k], D, n, v, fin[1 + k]));
        ZK_TRY(check(wit->Yk[k], D, n, v, fin[2 + K + k]));
    }
    return ZK_OK;
}

}  // namespace zkmi

using namespace zkmi;

extern "C" {

size_t zkattn_link_proof_bytes(size_t rows, size_t cols, size_t K) {
    if (!is_pow2(rows) || !is_pow2(cols) || K < 1 || K > (size_t)kLinkMaxK) return 0;
    return link_proof_len(log2_floor(rows) + log2_floor(cols), (int)K);
}

size_t zkattn_link_workspace_bytes(size_t rows, size_t cols, size_t K) {
    if (!is_pow2(rows) || !is_pow2(cols) || K < 1 || K > (size_t)kLinkMaxK) return 0;
    return link_ws_bytes(rows, cols, (int)K);
}

int zkattn_link_prove(const uint8_t seed[32], fr_vec Zp, const fr_vec* X, fr_vec Y, const fr_vec* Yk, fr_vec yhat,
                      const fr_t* bases, size_t rows, size_t cols, size_t K, uint8_t* proof, size_t cap, size_t* len,
                      void* ws, size_t ws_bytes, void* stream) {
    if (!seed || !X || !Yk || !bases || !is_pow2(rows) || !is_pow2(cols) || K < 1 || K > (size_t)kLinkMaxK)
        return ZK_E_BADARG;
    if (rows > ((size_t)1 << 31) / cols) return ZK_E_BADARG;
    const size_t D = rows * cols;
    if (!vec_ok(Zp, D) || !vec_ok(Y, D) || !vec_ok(yhat, rows)) return ZK_E_BADARG;
    for (size_t k = 0; k < K; ++k)
        if (!vec_ok(X[k], D) || !vec_ok(Yk[k], D)) return ZK_E_BADARG;
    const size_t need = link_proof_len(log2_floor(rows) + log2_floor(cols), (int)K);
    if (len) *len = need;
    if (!proof || cap < need) return ZK_E_BUFSZ;
    if (!ws || ws_bytes < link_ws_bytes(rows, cols, (int)K)) return ZK_E_BUFSZ;
    hipStream_t s = as_stream(stream);
    switch (K) {
        case 1: return link_prove_k<1>(seed, Zp, X, Y, Yk, yhat, bases, rows, cols, proof, ws, ws_bytes, s);
        case 2: return link_prove_k<2>(seed, Zp, X, Y, Yk, yhat, bases, rows, cols, proof, ws, ws_bytes, s);
        default: return link_prove_k<3>(seed, Zp, X, Y, Yk, yhat, bases, rows, cols, proof, ws, ws_bytes, s);
    }
}

int zkattn_link_prove_small(const uint8_t seed[32], const int64_t* Zp, const uint32_t* const* X, const uint64_t* Y,
                            const uint32_t* const* Yk, fr_vec yhat, const uint64_t* bases, size_t rows, size_t cols, size_t K,
                            uint8_t* proof, size_t cap, size_t* len, void* ws, size_t ws_bytes, void* stream) {
    if (!seed || !Zp || !X || !Y || !Yk || !bases || !is_pow2(rows) || !is_pow2(cols) || K < 1 || K > (size_t)kLinkMaxK)
        return ZK_E_BADARG;
    if (rows > ((size_t)1 << 31) / cols || rows * cols < 4) return ZK_E_BADARG;  // two rounds read the integers
    if (!vec_ok(yhat, rows)) return ZK_E_BADARG;
    for (size_t k = 0; k < K; ++k)
        if (!X[k] || !Yk[k] || bases[k] == 0 || bases[k] >= ((uint64_t)1 << 32)) return ZK_E_BADARG;
    const size_t need = link_proof_len(log2_floor(rows) + log2_floor(cols), (int)K);
    if (len) *len = need;
    if (!proof || cap < need) return ZK_E_BUFSZ;
    if (!ws || ws_bytes < link_ws_bytes(rows, cols, (int)K)) return ZK_E_BUFSZ;
    hipStream_t s = as_stream(stream);
    const LinkSmallIn in{Zp, X, Y, Yk, bases};
    const fr_vec none = {nullptr, 0, 0};
    switch (K) {
        case 1: return link_prove_k<1>(seed, none, nullptr, none, nullptr, yhat, nullptr, rows, cols, proof, ws, ws_bytes, s, &in);
        case 2: return link_prove_k<2>(seed, none, nullptr, none, nullptr, yhat, nullptr, rows, cols, proof, ws, ws_bytes, s, &in);
        default: return link_prove_k<3>(seed, none, nullptr, none, nullptr, yhat, nullptr, rows, cols, proof, ws, ws_bytes, s, &in);
    }
}

size_t zkattn_link_verify_workspace_bytes(size_t rows, size_t cols) {
    if (!is_pow2(rows) || !is_pow2(cols)) return 0;
    return mle_scratch_bytes(log2_floor(rows) + log2_floor(cols)) + 256;
}

int zkattn_link_verify(const uint8_t seed[32], const uint8_t* proof, size_t len, size_t rows, size_t cols, size_t K,
                       const fr_t* bases, const zkattn_link_witness* witness, zkattn_link_claims* claims, void* ws,
                       size_t ws_bytes, void* stream) {
    if (!seed || !proof || !bases || !is_pow2(rows) || !is_pow2(cols) || K < 1 || K > (size_t)kLinkMaxK)
        return ZK_E_BADARG;
    if (rows > ((size_t)1 << 31) / cols) return ZK_E_BADARG;
    return link_verify(seed, proof, len, rows, cols, (int)K, bases, witness, claims, ws, ws_bytes, as_stream(stream));
}

}  // extern "C"
