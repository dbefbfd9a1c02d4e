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

// ---- the last rounds in one resident kernel ----------------------------------------------------
//
// A round over a few hundred pairs is a few microseconds of arithmetic; launched on
// its own it costs a kernel launch, a second one for the totals and two trips
// through the runtime's queue, about 40 us.  Once the arrays have shrunk to
// kTailPairs pairs one workgroup stays resident for all remaining rounds: it
// writes a round's three sums to the host's mailbox, waits (bounded) for the
// challenge on the command channel, folds and goes on; at the end it writes the
// two final values.  Every thread takes every barrier, and a wait that fails
// ends the kernel for all of them.
//
// The very last rounds are the host's: a round of 64 pairs is a few hundred
// multiplications, which the host does in a fraction of the thirty microseconds a
// trip to it and back costs.  So the kernel stops before the first round of at
// most kHostPairs pairs (if it has run a round by then), binds the last challenge,
// writes both arrays (at most 2 kHostPairs elements each) behind the mailbox's
// result words and ends; the host computes the remaining rounds' sums, folds and
// the two final values itself -- the same sums over the same values, exact
// arithmetic, so the same bytes.
static const int kTailThreads = 1024;
static const size_t kTailPairs = 1024;
static const size_t kHostPairs = 64;
static_assert(2 * 2 * kHostPairs * 8 <= kMailboxWords - kMailboxShip, "both arrays fit behind the result words");

struct ProductTailArgs {
    uint32_t* a;
    size_t as;
    uint32_t* b;
    size_t bs;
    size_t half0;       // pairs in the first of these rounds
    int nrounds;        // rounds run here (>= 1)
    int fold_first;     // the first of them binds the previous variable to r_prev
    Fr r_prev;
    uint32_t* words;    // mailbox: sums at words[0..24), final values at words[0..16)
    const uint32_t* cmd;
    uint32_t out_seq[33];  // [i]: the sums of round i are there; [nrounds]: the final values are
    uint32_t cmd_seq[32];  // [i]: the challenge of round i
    uint32_t spin_limit;
    // not zero: after the last round both arrays go to the host instead of the final values, ship_count elements
    // of a, then of b, each with that round's variable bound, eight words per element from words[kMailboxShip] on
    uint32_t ship_count;
};

static __global__ void __launch_bounds__(kTailThreads) k_product_tail(ProductTailArgs g) {
    __shared__ uint32_t lds[16 * 3 * 8];
    __shared__ uint32_t sh_r[8];
    __shared__ int sh_ok;
    Fr r = g.r_prev;
    bool fold = g.fold_first != 0;
    size_t half = g.half0;
    bool ok = true;
    for (int i = 0; i < g.nrounds; ++i, half >>= 1) {
        Fr tot[3] = {fr_zero(), fr_zero(), fr_zero()};
        const size_t p = threadIdx.x;
        if (p < half) {
            const PairArray A{g.a, g.as, g.a, g.as}, B{g.b, g.bs, g.b, g.bs};
            Fr a0, a1, b0, b1;
            if (fold) {
                load_pair<true>(A, p, half, r, a0, a1);
                load_pair<true>(B, p, half, r, b0, b1);
            } else {
                load_pair<false>(A, p, half, r, a0, a1);
                load_pair<false>(B, p, half, r, b0, b1);
            }
            tot[0] = fr_mul(a0, b0);
            tot[1] = fr_mul(a1, b1);
            tot[2] = fr_mul(fr_sub(a1, a0), fr_sub(b1, b0));
        }
        block_sum<3, 16>(tot, lds);
        if (threadIdx.x == 0) {
#pragma unroll
            for (int q = 0; q < 3; ++q)
#pragma unroll
                for (int k = 0; k < 8; ++k) g.words[8 * q + k] = tot[q].l[k];
            mailbox_written();
            mailbox_publish(g.words, g.out_seq[i]);
            uint32_t limbs[8];
            const bool got = mailbox_receive_challenge(g.cmd, g.cmd_seq[i], g.spin_limit, limbs);
            if (got) {
#pragma unroll
                for (int k = 0; k < 8; ++k) sh_r[k] = limbs[k];
            }
            sh_ok = got ? 1 : 0;
        }
        __syncthreads();  // the folded entries written in this round are visible to the workgroup from here on
        ok = sh_ok != 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) r.l[k] = __builtin_amdgcn_readfirstlane(sh_r[k]);
        __syncthreads();  // sh_ok and sh_r are free to be written again
        if (!ok) break;   // the same for every thread
        fold = true;
    }
    if (ok && g.ship_count) {
        for (uint32_t t = threadIdx.x; t < 2 * g.ship_count; t += kTailThreads) {
            const bool first = t < g.ship_count;
            const uint32_t* arr = first ? g.a : g.b;
            const size_t stride = first ? g.as : g.bs;
            const uint32_t j = first ? t : t - g.ship_count;
            Fr v = fr_fold(fr_load(arr, stride, j), fr_load(arr, stride, j + g.ship_count), r);
#pragma unroll
            for (int k = 0; k < 8; ++k) g.words[kMailboxShip + 8 * (size_t)t + k] = v.l[k];
            mailbox_written();
        }
    } else if (ok && threadIdx.x < 2) {
        const uint32_t* arr = threadIdx.x == 0 ? g.a : g.b;
        const size_t stride = threadIdx.x == 0 ? g.as : g.bs;
        Fr v = fr_fold(fr_load(arr, stride, 0), fr_load(arr, stride, 1), r);
#pragma unroll
        for (int k = 0; k < 8; ++k) g.words[8 * threadIdx.x + k] = v.l[k];
        mailbox_written();
    }
    __syncthreads();
    if (ok && threadIdx.x == 0) mailbox_publish(g.words, g.out_seq[g.nrounds]);
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
    // rounds with at most kTailPairs pairs run in one resident kernel (see k_product_tail)
    int tail_first = d;
    for (int k = 0; k < d; ++k)
        if (((size_t)1 << (d - k - 1)) <= kTailPairs) {
            tail_first = k;
            break;
        }
    auto emit_round = [&](const F& g0, const F& g1, const F& lead) {
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
    };
    for (int k = 0; k < tail_first; ++k) {
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
        emit_round(from_dev(mb->words), from_dev(mb->words + 8), from_dev(mb->words + 16));
    }
    if (tail_first < d) {
        ProductTailArgs g;
        memset(&g, 0, sizeof g);
        g.a = a; g.as = as; g.b = b; g.bs = bs;
        g.half0 = (size_t)1 << (d - tail_first - 1);
        // the kernel's rounds end before the first one (after its own first) of at most kHostPairs pairs
        int k_host = tail_first + 1;
        while (k_host < d && ((size_t)1 << (d - k_host - 1)) > kHostPairs) ++k_host;
        g.nrounds = k_host - tail_first;
        g.ship_count = k_host < d ? (uint32_t)1 << (d - k_host) : 0;
        g.fold_first = tail_first > 0;
        g.r_prev = to_dev(r_prev);
        g.words = mb->words;
        g.cmd = mb->cmd;
        for (int i = 0; i <= g.nrounds; ++i) g.out_seq[i] = mb->next_seq();
        for (int i = 0; i < g.nrounds; ++i) g.cmd_seq[i] = mb->next_cmd_seq();
        g.spin_limit = device_spin_limit();
        mailbox_channel_reset(mb);
        TailGuard guard{mb, stream};
        hipLaunchKernelGGL(k_product_tail, dim3(1), dim3(kTailThreads), 0, stream, g);
        ZK_HIP_TRY(hipGetLastError());
        guard.armed = true;
        for (int i = 0; i < g.nrounds; ++i) {
            ZK_TRY(mailbox_wait(mb, g.out_seq[i], stream));
            emit_round(from_dev(mb->words), from_dev(mb->words + 8), from_dev(mb->words + 16));
            mailbox_send_challenge(mb, g.cmd_seq[i], to_dev(r_prev).l);
        }
        ZK_TRY(mailbox_wait(mb, g.out_seq[g.nrounds], stream));
        guard.armed = false;
        ZK_HIP_TRY(hipStreamSynchronize(stream));  // everything of this call has left the device
        F fa = from_dev(mb->words), fb = from_dev(mb->words + 8);
        if (g.ship_count) {
            // the host's rounds, on the arrays the kernel has handed over
            F ha[2 * kHostPairs], hb[2 * kHostPairs];
            const uint32_t* at = mb->words + kMailboxShip;
            for (uint32_t j = 0; j < g.ship_count; ++j, at += 8) ha[j] = from_dev(at);
            for (uint32_t j = 0; j < g.ship_count; ++j, at += 8) hb[j] = from_dev(at);
            for (size_t half = g.ship_count / 2; half >= 1; half >>= 1) {
                F g0 = zero(), g1 = zero(), lead = zero();
                for (size_t p = 0; p < half; ++p) {
                    g0 = add(g0, mul(ha[p], hb[p]));
                    g1 = add(g1, mul(ha[p + half], hb[p + half]));
                    lead = add(lead, mul(sub(ha[p + half], ha[p]), sub(hb[p + half], hb[p])));
                }
                emit_round(g0, g1, lead);
                for (size_t p = 0; p < half; ++p) {
                    ha[p] = add(ha[p], mul(r_prev, sub(ha[p + half], ha[p])));
                    hb[p] = add(hb[p], mul(r_prev, sub(hb[p + half], hb[p])));
                }
            }
            fa = ha[0];
            fb = hb[0];
        }
        to_bytes(out, fa);
        to_bytes(out + 32, fb);
        tr.absorb("final", out, 64);
        return ZK_OK;
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

// ---- the same for matrices of small integers -----------------------------------------------
//
// Quantised activations and weights are 16-bit integers.  With x' = x + 2^15 (so
// 0 <= x' < 2^16) a sum  sum_i e_i x_i  of field elements times matrix entries is
// sum_i e_i x'_i - 2^15 sum_i e_i.  A product e_i x'_i is eight 32x32-bit products
// of at most 48 bits, added limb by limb into 64-bit accumulators with no carries
// and no reduction (2^16 terms fit); the sums leave the kernels as plain 288-bit
// integers ("raw", nine 32-bit limbs, limb-major) and one small kernel reduces
// them mod r and subtracts the constant.  Per matrix entry that is eight
// multiply-adds and two bytes of traffic instead of a field multiplication and 32.
static const int kRawLimbs = 9;
static const size_t kSmallTermsMax = 1 << 15;  // terms per accumulator: 2^48 * 2^15 = 2^63

__device__ __forceinline__ void small_mac(uint64_t (&acc)[8], const Fr& e, int16_t x) {
    const uint32_t xp = (uint32_t)((int)x + 32768);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += (uint64_t)e.l[j] * xp;
}

// sum_j acc[j] 2^(32 j) as nine 32-bit limbs (acc[j] < 2^63).
__device__ __forceinline__ void small_normalize(uint32_t (&out)[kRawLimbs], const uint64_t (&acc)[8]) {
    uint64_t carry = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint64_t s = (acc[j] & 0xffffffffu) + (carry & 0xffffffffu);
        out[j] = (uint32_t)s;
        carry = (acc[j] >> 32) + (carry >> 32) + (s >> 32);
    }
    out[8] = (uint32_t)carry;  // the sum is below 2^288
}

// raw part[c][limb][k] = sum over rows i of chunk c of e[i] * (X[i][k] + 2^15); thread per column.
__global__ void __launch_bounds__(kBlock) k_colsum_partial_i16(const int16_t* __restrict__ X, size_t D0, size_t D1,
                                                               const uint32_t* __restrict__ e, size_t es,
                                                               size_t rows_per_chunk, uint32_t* __restrict__ part,
                                                               size_t P1) {
    size_t k = blockIdx.x * (size_t)kBlock + threadIdx.x;
    if (k >= D1) return;
    size_t i0 = blockIdx.y * rows_per_chunk, i1 = i0 + rows_per_chunk;
    if (i1 > D0) i1 = D0;
    uint64_t acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0;
    size_t i = i0;
    for (; i + 4 <= i1; i += 4) {  // four rows at a time: their loads are in flight together
        int16_t x[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) x[q] = X[(i + q) * D1 + k];
#pragma unroll
        for (int q = 0; q < 4; ++q) small_mac(acc, fr_load(e, es, i + q), x[q]);
    }
    for (; i < i1; ++i) small_mac(acc, fr_load(e, es, i), X[i * D1 + k]);
    uint32_t raw[kRawLimbs];
    small_normalize(raw, acc);
#pragma unroll
    for (int j = 0; j < kRawLimbs; ++j) part[((size_t)blockIdx.y * kRawLimbs + j) * P1 + k] = raw[j];
}

// raw rows[limb][k] = sum_j (W[k][j] + 2^15) e[j]; one wavefront per four rows, lanes over j.
static const int kRowsPerWave = 4;
__global__ void __launch_bounds__(64) k_rowdot_i16(uint32_t* __restrict__ raw_out, size_t P1, const int16_t* __restrict__ W,
                                                   size_t D1, size_t D2, const uint32_t* __restrict__ e, size_t es) {
    const size_t k0 = (size_t)blockIdx.x * kRowsPerWave;
    if (k0 >= D1) return;
    uint64_t acc[kRowsPerWave][8];
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[r][j] = 0;
    const int rows = D1 - k0 < (size_t)kRowsPerWave ? (int)(D1 - k0) : kRowsPerWave;
    size_t j = 0;
    if ((D2 & 3) == 0 && (es & 3) == 0 && (reinterpret_cast<uintptr_t>(W) & 7) == 0 && (reinterpret_cast<uintptr_t>(e) & 15) == 0) {
        // four consecutive columns per lane: eight 16-byte loads bring four elements of e
        // (limb-major: limb k of columns j..j+3 is one uint4) and one 8-byte load per row four entries of W
        for (j = 4 * (size_t)threadIdx.x; j + 3 < D2; j += 4 * 64) {
            uint4 el[8];
            uint2 xw[kRowsPerWave];
#pragma unroll
            for (int k = 0; k < 8; ++k) el[k] = *reinterpret_cast<const uint4*>(e + k * es + j);
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r)
                xw[r] = r < rows ? *reinterpret_cast<const uint2*>(W + (k0 + r) * D2 + j) : make_uint2(0x80008000u, 0x80008000u);
            Fr ej[4];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                ej[0].l[k] = el[k].x;
                ej[1].l[k] = el[k].y;
                ej[2].l[k] = el[k].z;
                ej[3].l[k] = el[k].w;
            }
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) {
                small_mac(acc[r], ej[0], (int16_t)(xw[r].x & 0xffffu));
                small_mac(acc[r], ej[1], (int16_t)(xw[r].x >> 16));
                small_mac(acc[r], ej[2], (int16_t)(xw[r].y & 0xffffu));
                small_mac(acc[r], ej[3], (int16_t)(xw[r].y >> 16));
            }
        }
        j = D2;  // D2 is a multiple of four: the loop above has covered every column
    }
    for (j += threadIdx.x; j < D2; j += 64) {
        const Fr ej = fr_load(e, es, j);
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r)
            if (r < rows) small_mac(acc[r], ej, W[(k0 + r) * D2 + j]);
    }
    // the wavefront's sum of a limb is below 2^48 * D2 <= 2^63 (the caller keeps D2 <= 2^15)
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
#pragma unroll
        for (int limb = 0; limb < 8; ++limb) {
            uint64_t v = acc[r][limb];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
            acc[r][limb] = v;
        }
    }
    if (threadIdx.x == 0) {
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            if (k0 + r >= D1) break;
            uint32_t raw[kRawLimbs];
            small_normalize(raw, acc[r]);
#pragma unroll
            for (int limb = 0; limb < kRawLimbs; ++limb) raw_out[(size_t)limb * P1 + k0 + r] = raw[limb];
        }
    }
}

// dst[k] = (sum over `chunks` raw values of entry k) mod r - 2^15 * (*esum), zero for k >= count.
__global__ void __launch_bounds__(kBlock) k_small_finish(uint32_t* __restrict__ dst, size_t ds, const uint32_t* __restrict__ raw,
                                                         size_t P, size_t chunks, size_t count, const uint32_t* __restrict__ esum) {
    size_t k = blockIdx.x * (size_t)kBlock + threadIdx.x;
    if (k >= P) return;
    if (k >= count) {
        fr_store(dst, ds, k, fr_zero());
        return;
    }
    uint64_t limb[kRawLimbs];
#pragma unroll
    for (int j = 0; j < kRawLimbs; ++j) limb[j] = 0;
    size_t c = 0;
    for (; c + 8 <= chunks; c += 8) {  // eight chunks per trip: 72 loads in flight
        uint32_t v[8][kRawLimbs];
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int j = 0; j < kRawLimbs; ++j) v[q][j] = raw[((c + q) * kRawLimbs + j) * P + k];
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int j = 0; j < kRawLimbs; ++j) limb[j] += v[q][j];
    }
    for (; c < chunks; ++c)
#pragma unroll
        for (int j = 0; j < kRawLimbs; ++j) limb[j] += raw[(c * kRawLimbs + j) * P + k];
    // carry: the total is below 2^288 * chunks, chunks <= 2^16
    Fr lo, hi = fr_zero();
    uint64_t carry = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint64_t s = limb[j] + carry;
        lo.l[j] = (uint32_t)s;
        carry = s >> 32;
    }
    uint64_t top = limb[8] + carry;
    hi.l[0] = (uint32_t)top;
    hi.l[1] = (uint32_t)(top >> 32);
    // lo (any value below 2^256) mod r = lo * 2^512 / 2^256 / 2^256; hi * 2^256 mod r = hi * 2^512 / 2^256
    Fr one_raw = fr_zero();
    one_raw.l[0] = 1;
    Fr sum = fr_add(fr_mul(fr_mul(lo, fr_rr()), one_raw), fr_mul(hi, fr_rr()));
    Fr shift = fr_zero();
    shift.l[0] = 32768;
    shift = fr_mul(shift, fr_rr());  // 2^15 in Montgomery form
    fr_store(dst, ds, k, fr_sub(sum, fr_mul(shift, fr_load(esum, 1, 0))));
}

// out (eight words, Montgomery limbs of one element) = sum_{i < n} e[i]; one workgroup.
__global__ void __launch_bounds__(1024) k_sum_one(uint32_t* __restrict__ out, const uint32_t* __restrict__ e, size_t es, size_t n) {
    __shared__ uint32_t lds[16 * 8];
    Fr acc[1] = {fr_zero()};
    for (size_t i = threadIdx.x; i < n; i += 1024) acc[0] = fr_add(acc[0], fr_load(e, es, i));
    block_sum<1, 16>(acc, lds);
    if (threadIdx.x == 0) fr_store(out, 1, 0, acc[0]);
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
    // chunk sums as field elements (8 words each) or raw (9 words each, plus one element)
    w.part = cv.limbs(2 * kColChunks * widest + 8);
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

static void colsum_i16_run(uint32_t* a, size_t PC, const int16_t* M, size_t R, size_t C, const uint32_t* e0, size_t e0s,
                           uint32_t* scratch, hipStream_t stream) {
    size_t rows_per_chunk = div_up(R, kColChunks);
    size_t chunks = div_up(R, rows_per_chunk);
    uint32_t* raw = scratch;
    uint32_t* esum = scratch + kColChunks * kRawLimbs * PC;
    hipLaunchKernelGGL(k_sum_one, dim3(1), dim3(1024), 0, stream, esum, e0, e0s, R);
    hipLaunchKernelGGL(k_colsum_partial_i16, dim3((unsigned)div_up(C, kBlock), (unsigned)chunks), dim3(kBlock), 0, stream, M,
                       R, C, e0, e0s, rows_per_chunk, raw, PC);
    hipLaunchKernelGGL(k_small_finish, dim3((unsigned)div_up(PC, kBlock)), dim3(kBlock), 0, stream, a, PC, raw, PC, chunks,
                       C, esum);
}

static void rowdot_i16_run(uint32_t* b, size_t PR, const int16_t* M, size_t R, size_t C, const uint32_t* e1, size_t e1s,
                           uint32_t* scratch, hipStream_t stream) {
    uint32_t* raw = scratch;
    uint32_t* esum = scratch + kColChunks * kRawLimbs * PR;
    hipLaunchKernelGGL(k_sum_one, dim3(1), dim3(1024), 0, stream, esum, e1, e1s, C);
    hipLaunchKernelGGL(k_rowdot_i16, dim3((unsigned)div_up(R, kRowsPerWave)), dim3(64), 0, stream, raw, PR, M, R, C, e1, e1s);
    hipLaunchKernelGGL(k_small_finish, dim3((unsigned)div_up(PR, kBlock)), dim3(kBlock), 0, stream, b, PR, raw, PR,
                       (size_t)1, R, esum);
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

// X, W as field vectors, or (X16, W16 non-null) as row-major 16-bit integers.
static int matmul_prove_any(const uint8_t seed[32], fr_vec X, const int16_t* X16, size_t D0, size_t D1, fr_vec W,
                            const int16_t* W16, size_t D2, uint8_t* proof, size_t cap, size_t* len, void* ws,
                            size_t ws_bytes, void* stream_v) {
    const bool small = X16 != nullptr;
    if (!seed || !matmul_dims_ok(D0, D1, D2)) return ZK_E_BADARG;
    if (small ? !W16 : (!vec_ok(X, D0 * D1) || !vec_ok(W, D1 * D2))) return ZK_E_BADARG;
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
    if (small) {
        // entries per accumulator: rows of X per chunk, columns of W per lane
        if (D0 > kColChunks * kSmallTermsMax || D2 > kSmallTermsMax) return ZK_E_BADARG;
        colsum_i16_run(w.a, w.P1, X16, D0, D1, w.eu, w.P0, w.part, stream);
        rowdot_i16_run(w.b, w.P1, W16, D1, D2, w.ev, w.P2, w.part, stream);
    } else {
        colsum_run(w.a, w.P1, X.limbs, X.stride, D0, D1, w.eu, w.P0, w.part, stream);
        rowdot_run(w.b, w.P1, W.limbs, W.stride, D1, D2, w.ev, w.P2, stream);
    }
    ZK_HIP_TRY(hipGetLastError());
    memcpy(proof, "ZKMM\x01\0\0\0", 8);
    host::put_le64(proof + 8, D0);
    host::put_le64(proof + 16, D1);
    host::put_le64(proof + 24, D2);
    return product_rounds_run(tr, w.a, w.P1, w.b, w.P1, n1, nullptr, proof + 32, proof + 64, cv, mb, stream);
}

int zkmi_selftest_resident_wait(void* ws, size_t ws_bytes, void* stream_v) {
    // The last rounds run in a kernel that waits for the host between rounds.  Here
    // the host never answers: with a bound of a few polls the kernel must give up by
    // itself, having published its first round's sums and nothing after them.
    if (!ws || ws_bytes < 4 * 32 * 4 + 512) return ZK_E_BUFSZ;
    hipStream_t stream = as_stream(stream_v);
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(ws, ws_bytes);
    uint32_t* a = cv.limbs(4);
    uint32_t* b = cv.limbs(4);
    launch_fill_u32(a, 32, 1u, stream);
    launch_fill_u32(b, 32, 1u, stream);
    ProductTailArgs g;
    memset(&g, 0, sizeof g);
    g.a = a; g.as = 4; g.b = b; g.bs = 4;
    g.half0 = 2;
    g.nrounds = 2;
    g.fold_first = 0;
    g.r_prev = to_dev(host::zero());
    g.words = mb->words;
    g.cmd = mb->cmd;
    for (int i = 0; i <= g.nrounds; ++i) g.out_seq[i] = mb->next_seq();
    for (int i = 0; i < g.nrounds; ++i) g.cmd_seq[i] = mb->next_cmd_seq();
    g.spin_limit = 8;
    mailbox_channel_reset(mb);
    hipLaunchKernelGGL(k_product_tail, dim3(1), dim3(kTailThreads), 0, stream, g);
    ZK_HIP_TRY(hipGetLastError());
    ZK_TRY(mailbox_wait(mb, g.out_seq[0], stream));          // the first round's sums arrive
    ZK_HIP_TRY(hipStreamSynchronize(stream));                 // and the kernel ends without an answer
    const uint32_t flag = mb->words[kMailboxFlag];
    if (flag != g.out_seq[0]) return ZK_E_HIP;                // nothing was published after them
    // A call that ends early leaves an abort in the channel.  The next kernel must
    // not see it: this one is answered and has to run to its end.
    mailbox_send_abort(mb);
    for (int i = 0; i <= g.nrounds; ++i) g.out_seq[i] = mb->next_seq();
    for (int i = 0; i < g.nrounds; ++i) g.cmd_seq[i] = mb->next_cmd_seq();
    g.spin_limit = device_spin_limit();
    mailbox_channel_reset(mb);
    TailGuard guard{mb, stream};
    hipLaunchKernelGGL(k_product_tail, dim3(1), dim3(kTailThreads), 0, stream, g);
    ZK_HIP_TRY(hipGetLastError());
    guard.armed = true;
    for (int i = 0; i < g.nrounds; ++i) {
        ZK_TRY(mailbox_wait(mb, g.out_seq[i], stream));
        mailbox_send_challenge(mb, g.cmd_seq[i], to_dev(host::one()).l);
    }
    ZK_TRY(mailbox_wait(mb, g.out_seq[g.nrounds], stream));
    guard.armed = false;
    ZK_HIP_TRY(hipStreamSynchronize(stream));
    return ZK_OK;
}

int matmul_sumcheck_prove(const uint8_t seed[32], fr_vec X, size_t D0, size_t D1, fr_vec W, size_t D2, uint8_t* proof,
                          size_t cap, size_t* len, void* ws, size_t ws_bytes, void* stream) {
    return matmul_prove_any(seed, X, nullptr, D0, D1, W, nullptr, D2, proof, cap, len, ws, ws_bytes, stream);
}

int matmul_sumcheck_prove_i16(const uint8_t seed[32], const int16_t* X, size_t D0, size_t D1, const int16_t* W, size_t D2,
                              uint8_t* proof, size_t cap, size_t* len, void* ws, size_t ws_bytes, void* stream) {
    if (!X || !W) return ZK_E_BADARG;
    fr_vec none = {nullptr, 0, 0};
    return matmul_prove_any(seed, none, X, D0, D1, none, W, D2, proof, cap, len, ws, ws_bytes, stream);
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
