// tlookup prover and verifier (Section 4 of the paper, Protocol 1), host
// orchestration.  All arithmetic on tensors runs in the kernels of
// tlookup_kernels.h, batch_inverse.hip and poly.hip; the host only drives the
// Fiat-Shamir transcript and turns the handful of sums a round returns into
// the round polynomial.
//
// How a round is computed.  With x = (X, rest) after binding k variables,
//   e~(u, x) = c_k * e~(u_k, X) * e_rest(rest),   c_k = prod_{t<k} e~(u_t, r_t),
// so the data side of g_k is  alpha c_k e~(u_k, X) q(X) + sA(X)  with
//   q(X) = sum_rest e_rest A(X,rest) (S(X,rest)+beta)   (degree 2 in X),
//   sA(X) = sum_rest A(X,rest)                          (degree 1),
// and e_rest never has to be folded: it is looked up in two small tables (low
// and high remaining variables).  The table side is the constant
// 2^-(k+1) * c_B while the variable being bound is not one of the table's, and
// 2^-h (alpha^2 c'_k e~(u_k,X) qT(X) - bm(X)) afterwards.
//
// Which kernel computes a round's sums is decided by plan_round.  From a vector
// of field elements the first pass over A and S yields the sums of the first TWO
// rounds (round01_dev.h) and the third round's kernel binds both variables at
// once; in the large folding rounds the kernel sums one side of the round (X = 0
// or X = 1) and the other side follows here from the running claim.
#include "internal.h"
#include "tlookup_kernels.h"
#include "tlookup_round29.h"
#include "transcript.h"

namespace zkmi {

static const int kLoBits = 12;  // low eq table covers up to this many variables

// Pool of eq tables for a point u of n variables.
//   suffix[s], s = 0..min(kLoBits, n-1): e~ over the last s variables;
//   suffix29[s]: the same times 2^10, for the rounds on 29-bit limbs, whose
//                multiplication divides by 2^261 instead of 2^256 (twice on the way
//                into a sum of products);
//   high[k], for rounds k with n-k-1 > kLoBits: e~ over variables k+1 .. n-kLoBits-1.
struct EqPool {
    uint32_t* pool = nullptr;
    size_t stride = 0;
    uint32_t suffix_off[kLoBits + 1];
    uint32_t suffix29_off[kLoBits + 1];  // within pool29
    uint32_t high_off[32];
    uint4* pool29 = nullptr;  // the scaled suffix tables as 29-bit limbs, three planes of count29 elements
    size_t count29 = 0;
    int n = 0;

    static size_t entries29(int n) {
        size_t total = 0;
        int smax = n - 1 < kLoBits ? n - 1 : kLoBits;
        for (int s = 0; s <= smax; ++s) total += (size_t)1 << s;
        return total ? total : 1;
    }

    static size_t entries(int n) {
        size_t total = 0;
        int smax = n - 1 < kLoBits ? n - 1 : kLoBits;
        for (int s = 0; s <= smax; ++s) total += (size_t)2 << s;
        for (int k = 0; k < n; ++k) {
            int rest = n - k - 1;
            if (rest > kLoBits) total += (size_t)1 << (rest - kLoBits);
        }
        return total ? total : 1;
    }

    // Weights of round k (remaining variables k+1 .. n-1).
    EqSplit round(int k) const {
        int rest = n - k - 1;
        EqSplit e;
        e.pool = pool;
        e.stride = stride;
        e.lbits = rest < kLoBits ? rest : kLoBits;
        e.lo_off = suffix_off[e.lbits];
        e.has_hi = rest > kLoBits;
        e.hi_off = e.has_hi ? high_off[k] : 0;
        return e;
    }
};

static int eq_pool_build(EqPool& ep, const host::F* u, int n, Carver& cv, hipStream_t stream) {
    ep.n = n;
    ep.stride = EqPool::entries(n);
    ep.pool = cv.limbs(ep.stride);
    ep.count29 = EqPool::entries29(n);
    ep.pool29 = (uint4*)cv.take(ep.count29 * 36);
    if (!ep.pool || !ep.pool29) return ZK_E_BUFSZ;
    EqPoolArgs args;
    memset(&args, 0, sizeof args);
    for (int t = 0; t < n; ++t) args.u[t] = to_dev(u[t]);
    int q = 0;
    uint32_t off = 0;
    int smax = n - 1 < kLoBits ? n - 1 : kLoBits;
    for (int s = 0; s <= smax; ++s) {
        ep.suffix_off[s] = off;
        args.offset[q] = off;
        args.var0[q] = (uint8_t)(n - s);
        args.nvars[q] = (uint8_t)s;
        off += 1u << s;
        ++q;
    }
    if (n == 0) ep.suffix_off[0] = 0;
    args.scale = to_dev(host::from_u64(1024));
    args.pool29 = ep.pool29;
    args.count29 = ep.count29;
    args.first29 = off;
    for (int s = 0; s <= smax; ++s) {
        ep.suffix29_off[s] = off - args.first29;
        args.offset[q] = off;
        args.var0[q] = (uint8_t)(n - s);
        args.nvars[q] = (uint8_t)s;
        args.scaled[q] = 1;
        off += 1u << s;
        ++q;
    }
    for (int k = 0; k < n; ++k) {
        int rest = n - k - 1;
        if (rest <= kLoBits) continue;
        ep.high_off[k] = off;
        args.offset[q] = off;
        args.var0[q] = (uint8_t)(k + 1);
        args.nvars[q] = (uint8_t)(rest - kLoBits);
        off += 1u << (rest - kLoBits);
        ++q;
    }
    args.ntables = q;
    args.total = off;
    if (q > 64) return ZK_E_BADARG;
    if (off) {
        hipLaunchKernelGGL(k_eq_pool, dim3(grid_for(off)), dim3(kBlock), 0, stream, ep.pool, ep.stride, args);
        ZK_HIP_TRY(hipGetLastError());
    }
    return ZK_OK;
}

// Quadratic through value(0), value(1) and leading coefficient, at X = 0..3.
static void quad_values(host::F out[4], const host::F& v0, const host::F& v1, const host::F& lead) {
    using namespace host;
    out[0] = v0;
    out[1] = v1;
    F lead2 = add(lead, lead);
    out[2] = add(sub(add(v1, v1), v0), lead2);                                 // 2 v1 - v0 + 2 lead
    out[3] = add(sub(add(add(v1, v1), v1), add(v0, v0)), add(add(lead2, lead2), lead2));  // 3 v1 - 2 v0 + 6 lead
}

// Line through value(0), value(1) at X = 0..3.
static void line_values(host::F out[4], const host::F& v0, const host::F& v1) {
    using namespace host;
    F d = sub(v1, v0);
    out[0] = v0;
    out[1] = v1;
    out[2] = add(v1, d);
    out[3] = add(out[2], d);
}

// ---- workspace layout -------------------------------------------------------------

struct ProveWs {
    uint32_t* A;        // D
    uint32_t* Sf;       // D/2
    uint4* A29;         // folded A and S while they are held in 29-bit limbs: D/2 elements of 36 bytes each
    uint4* S29;
    uint32_t* B;        // N
    uint32_t* Bf;       // N/2: B is folded back and forth between B and Bf
    uint32_t* Tf;       // N/2
    uint32_t* M;        // N
    uint32_t* m;        // N counts
    uint32_t* slots;    // hash of T
    uint32_t cap_mask;
    uint32_t* canon;    // N
    uint4* rows;        // N rows of T, eight words each
    uint32_t* hist;     // per-workgroup histograms (tables of up to 2^16 rows), else null
    uint32_t hist_parts;
    uint32_t* flags;    // [0] duplicate flag, [1] ticket of the final sums, [2..3] smallest bad index (64-bit)
    SmallFold4* fold4;  // constants of the first fold when S comes as small integers (tlookup_prove_small)
    uint32_t* leaves;   // nleaves * 8 words
    uint32_t nleaves;
    uint32_t* dig_leaves;  // leaf digests of the hash trees over A and B
    uint32_t* dig_rows;    // the shorter rows of A's tree above kTreeChunk leaves
    uint32_t* dig_rows_b;  // the same for B
    size_t part_blocks; // capacity of the two partial-sum buffers, in workgroups
    uint32_t* partD;    // part_blocks * 5
    uint32_t* partT;    // part_blocks * 6
};

// Most workgroups a round kernel can be launched with: spans never shrink below
// 2^kLoBits pairs while high weight tables are in use.
static size_t round_blocks_max(size_t D) {
    size_t by_span = (D / 2) >> kLoBits;
    return by_span > kMaxPartialBlocks ? by_span : kMaxPartialBlocks;
}

static const size_t kLdsHistMaxRows = (size_t)1 << 16;  // packed 16-bit counters: 128 KiB of LDS
static const uint32_t kHistParts = 256;                // one workgroup per compute unit

// ---- digest of a vector (stand-in for its commitment) ----------------------------------
// Scratch: the leaf digests and, for rows longer than kTreeChunk, the rows above
// them (each at most 1/kTreeChunk of the one below: twice the first is room for all).
static size_t vec_digest_leaves(size_t n) { return n / kVecLeaf ? n / kVecLeaf : 1; }
static size_t vec_digest_row_digests(size_t n) {
    const size_t first = vec_digest_leaves(n) / kTreeChunk;
    return first ? 2 * first : 1;
}

// Enqueues the hash trees over one or two vectors (n elements each, powers of two;
// v2 may be null); a digest's eight state words go to its out_words (device
// memory or the mailbox `words`, in which case seq != 0 publishes completion of
// the whole call; `ticket`: one zeroed word of device memory, left zero).
// leaves: room for vec_digest_leaves(n1) + vec_digest_leaves(n2) digests;
// rows1, rows2: vec_digest_row_digests(n) digests each.
struct VecDigestJob {
    const uint32_t* v;
    size_t stride, n;
    uint32_t* rows;
    uint32_t* out_words;
};

static void vec_digest_launch(const VecDigestJob& one, const VecDigestJob* two, uint32_t* leaves, uint32_t* words,
                              uint32_t seq, uint32_t* ticket, hipStream_t stream) {
    const VecDigestJob* jobs[2] = {&one, two};
    const int njobs = two ? 2 : 1;
    // the shorter vector's leaves first: its few long chains start at once
    const int order[2] = {njobs == 2 && two->n < one.n ? 1 : 0, njobs == 2 && two->n < one.n ? 0 : 1};
    VecLeavesJob lv[2];
    const uint32_t* in[2];
    size_t cnt[2];
    uint32_t* rows[2];
    size_t total = 0;
    for (int q = 0; q < 2; ++q) {
        lv[q] = VecLeavesJob{nullptr, 0, 0, 0, nullptr};
        if (q >= njobs) continue;
        const VecDigestJob& j = *jobs[order[q]];
        lv[q] = VecLeavesJob{j.v, j.stride, j.n, vec_digest_leaves(j.n), leaves + total * 8};
        in[q] = lv[q].out;
        cnt[q] = lv[q].L;
        rows[q] = j.rows;
        total += lv[q].L;
    }
    hipLaunchKernelGGL(k_vec_leaves, dim3(grid_for(total)), dim3(kBlock), 0, stream, lv[0], lv[1]);
    // up the trees, both rows in one launch, a factor of up to kTreeChunk per launch
    bool done[2] = {false, njobs < 2};
    while (!done[0] || !done[1]) {
        DigestTreeJob tj[2];
        bool finishing = true;
        for (int q = 0; q < 2; ++q) {
            tj[q] = DigestTreeJob{nullptr, nullptr, 0, 0};
            if (done[q]) continue;
            const size_t chunk = cnt[q] > kTreeChunk ? kTreeChunk : cnt[q];
            const size_t blocks = cnt[q] / chunk;
            uint32_t* out = blocks == 1 ? jobs[order[q]]->out_words : rows[q];
            tj[q] = DigestTreeJob{in[q], out, (uint32_t)chunk, (uint32_t)blocks};
            in[q] = out;
            cnt[q] = blocks;
            if (blocks == 1) done[q] = true;
            else {
                rows[q] += blocks * 8;
                finishing = false;
            }
        }
        hipLaunchKernelGGL(k_digest_tree, dim3(tj[0].blocks + tj[1].blocks), dim3(kBlock), 0, stream, tj[0], tj[1], words,
                           finishing ? seq : 0u, ticket);
    }
}

// Hash-state words -> the digest's bytes.
static void digest_bytes(uint8_t out[32], const uint32_t* state_words) {
    for (int k = 0; k < 8; ++k) {
        const uint32_t v = state_words[k];
        out[4 * k] = (uint8_t)(v >> 24);
        out[4 * k + 1] = (uint8_t)(v >> 16);
        out[4 * k + 2] = (uint8_t)(v >> 8);
        out[4 * k + 3] = (uint8_t)v;
    }
}

static uint32_t hash_capacity(size_t N) {
    size_t cap = 64;
    while (cap < 2 * N) cap <<= 1;
    return (uint32_t)cap;
}

static int carve_prove(ProveWs& w, Carver& cv, size_t D, size_t N) {
    w.A = cv.limbs(D);
    w.Sf = cv.limbs(D / 2 ? D / 2 : 1);
    w.A29 = (uint4*)cv.take((D / 2 ? D / 2 : 1) * 36);
    w.S29 = (uint4*)cv.take((D / 2 ? D / 2 : 1) * 36);
    w.B = cv.limbs(N);
    w.Bf = cv.limbs(N / 2 ? N / 2 : 1);
    w.Tf = cv.limbs(N / 2 ? N / 2 : 1);
    w.M = cv.limbs(N);
    w.m = (uint32_t*)cv.take(N * 4);
    uint32_t cap = hash_capacity(N);
    w.cap_mask = cap - 1;
    w.slots = (uint32_t*)cv.take((size_t)cap * 4);
    w.canon = (uint32_t*)cv.take(N * 4);
    w.rows = (uint4*)cv.take(N * 32);
    w.hist_parts = N <= kLdsHistMaxRows ? kHistParts : 0;
    w.hist = w.hist_parts ? (uint32_t*)cv.take((size_t)w.hist_parts * N * 4) : nullptr;
    w.flags = (uint32_t*)cv.take(64);
    w.fold4 = (SmallFold4*)cv.take(sizeof(SmallFold4));
    w.nleaves = (uint32_t)div_up(N, kLeafCounts);
    w.leaves = (uint32_t*)cv.take((size_t)w.nleaves * 32);
    w.dig_leaves = (uint32_t*)cv.take((vec_digest_leaves(D) + vec_digest_leaves(N)) * 32);
    w.dig_rows = (uint32_t*)cv.take(vec_digest_row_digests(D) * 32);
    w.dig_rows_b = (uint32_t*)cv.take(vec_digest_row_digests(N) * 32);
    w.part_blocks = round_blocks_max(D);
    w.partD = cv.limbs(w.part_blocks * 5);
    w.partT = cv.limbs(w.part_blocks * 6);
    return ZK_OK;
}

// K instances: their buffers, one pool of weight tables per distinct length of
// the tensors, and the scratch of the 2K inversions that are in flight together.
// The order here is the order prove_core carves in.
static size_t prove_ws_bytes_shapes(const size_t* D, const size_t* N, size_t K) {
    Carver cv(nullptr, 0);
    for (size_t i = 0; i < K; ++i) {
        ProveWs w;
        carve_prove(w, cv, D[i], N[i]);
    }
    for (size_t i = 0; i < K; ++i) {
        bool seen = false;
        for (size_t j = 0; j < i; ++j) seen = seen || D[j] == D[i];
        if (seen) continue;
        cv.limbs(EqPool::entries(log2_floor(D[i])));
        cv.take(EqPool::entries29(log2_floor(D[i])) * 36);
    }
    for (size_t i = 0; i < K; ++i) {
        size_t apart = batch_inverse_scratch_bytes(D[i]) + batch_inverse_scratch_bytes(N[i]),
               joined = batch_inverse_scratch_bytes(D[i] + N[i]);
        cv.take(apart > joined ? apart : joined);
    }
    return cv.used();
}

static size_t prove_ws_bytes(size_t D, size_t N, size_t K = 1) {
    size_t Ds[kMailboxMaxInstances], Ns[kMailboxMaxInstances];
    if (K > kMailboxMaxInstances) K = kMailboxMaxInstances;
    for (size_t i = 0; i < K; ++i) {
        Ds[i] = D;
        Ns[i] = N;
    }
    return prove_ws_bytes_shapes(Ds, Ns, K);
}

// Multiplicities into w.m (and the digest leaves into w.leaves).  Returns
// ZK_E_NOT_IN_TABLE with *bad_index set if some S_i is not in T.
// With defer_check (hints given, workgroup histograms in use) the hints are
// only range-checked here; S_i = T[idx_i] is then checked by the caller.
static bool can_defer_check(const ProveWs& w, const uint32_t* idx, size_t D) { return w.hist && idx && D > (size_t)kBlock; }

static int count_rows(ProveWs& w, fr_vec S, const uint32_t* idx, fr_vec T, size_t D, size_t N, uint64_t* bad_index,
                      Mailbox* mb, hipStream_t stream, bool defer_check = false, bool counts_as_fr = false) {
    if (defer_check && !can_defer_check(w, idx, D)) return ZK_E_BADARG;
    uint32_t cap = w.cap_mask + 1;
    hipLaunchKernelGGL(k_count_init, dim3(grid_for((size_t)cap + N + 4)), dim3(kBlock), 0, stream, w.slots, (size_t)cap, w.m,
                       N, w.flags);
    hipLaunchKernelGGL(k_hash_build, dim3(grid_for(N)), dim3(kBlock), 0, stream, w.slots, w.cap_mask, T.limbs, T.stride,
                       (uint32_t)N, w.flags);
    hipLaunchKernelGGL(k_canon_rows, dim3(grid_for(N)), dim3(kBlock), 0, stream, w.canon, w.rows, w.slots, w.cap_mask,
                       T.limbs, T.stride, (uint32_t)N);
    if (w.hist) {
        // LDS histograms: every workgroup takes a contiguous share of S
        static thread_local bool lds_limit_raised = false;
        const size_t lds_bytes = ((N + 1) / 2) * 4;
        if (!lds_limit_raised) {
            ZK_HIP_TRY(hipFuncSetAttribute((const void*)k_count_lds<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)(((kLdsHistMaxRows + 1) / 2) * 4)));
            ZK_HIP_TRY(hipFuncSetAttribute((const void*)k_count_lds<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)(((kLdsHistMaxRows + 1) / 2) * 4)));
            lds_limit_raised = true;
        }
        // equal chunks, as few passes per workgroup as the 16-bit counters allow
        const size_t passes = div_up(div_up(D, w.hist_parts), (size_t)kHistPass);
        const size_t per_block = align_up(div_up(D, w.hist_parts * passes), kHistThreads);
        if (defer_check)
            hipLaunchKernelGGL(k_count_lds<false>, dim3(w.hist_parts), dim3(kHistThreads), lds_bytes, stream, w.m, w.hist,
                               S.limbs, S.stride, D, per_block, idx, T.limbs, T.stride, w.rows, (uint32_t)N, w.slots,
                               w.cap_mask, w.canon, w.flags, (unsigned long long*)(w.flags + 2));
        else
            hipLaunchKernelGGL(k_count_lds<true>, dim3(w.hist_parts), dim3(kHistThreads), lds_bytes, stream, w.m, w.hist,
                               S.limbs, S.stride, D, per_block, idx, T.limbs, T.stride, w.rows, (uint32_t)N, w.slots,
                               w.cap_mask, w.canon, w.flags, (unsigned long long*)(w.flags + 2));
        const uint32_t group = 16;
        hipLaunchKernelGGL(k_hist_reduce, dim3((unsigned)div_up(N, kBlock), (unsigned)div_up(w.hist_parts, group)),
                           dim3(kBlock), 0, stream, w.m, w.hist, w.hist_parts, group, (uint32_t)N);
    } else {
        hipLaunchKernelGGL(k_count, dim3(grid_for(D, kBlock, 8192)), dim3(kBlock), 0, stream, w.m, S.limbs, S.stride, D,
                           idx, T.limbs, T.stride, w.rows, (uint32_t)N, w.slots, w.cap_mask, w.canon, w.flags,
                           (unsigned long long*)(w.flags + 2));
    }
    hipLaunchKernelGGL(k_leaf_digests, dim3((unsigned)div_up(w.nleaves, 64)), dim3(64), 0, stream, w.leaves, w.m,
                       (uint32_t)N, w.nleaves);
    // the counts as field elements (w.M), while the host is busy with the digest
    if (counts_as_fr) hipLaunchKernelGGL(k_counts_to_fr, dim3(grid_for(N)), dim3(kBlock), 0, stream, w.M, N, w.m, N);
    ZK_HIP_TRY(hipGetLastError());
    ZK_TRY(mailbox_bulk(mb, (size_t)w.nleaves * 32 + 16));
    ZK_HIP_TRY(hipMemcpyAsync(mb->bulk, w.flags, 16, hipMemcpyDeviceToHost, stream));
    ZK_HIP_TRY(hipMemcpyAsync(mb->bulk + 16, w.leaves, (size_t)w.nleaves * 32, hipMemcpyDeviceToHost, stream));
    ZK_HIP_TRY(hipStreamSynchronize(stream));
    uint64_t bad;
    memcpy(&bad, mb->bulk + 8, 8);
    if (bad != UINT64_MAX) {
        if (bad_index) *bad_index = bad;
        return ZK_E_NOT_IN_TABLE;
    }
    return ZK_OK;
}

// Smallest i with S_i != row idx_i of the table (w.rows), or all ones.
static int find_bad_row(ProveWs& w, fr_vec S, const SmallSource& ints, const uint32_t* idx, size_t D, size_t N,
                        uint64_t* bad, hipStream_t stream) {
    if (!S.limbs && !ints.x) return ZK_E_BADARG;
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(kBlock), 0, stream, w.flags + 2, (size_t)2, 0xffffffffu);
    hipLaunchKernelGGL(k_check_rows, dim3(grid_for(D, kBlock, 16384)), dim3(kBlock), 0, stream, S.limbs, S.stride, D, idx,
                       w.rows, (uint32_t)N, (unsigned long long*)(w.flags + 2), ints);
    ZK_HIP_TRY(hipGetLastError());
    ZK_HIP_TRY(hipMemcpyAsync(bad, w.flags + 2, 8, hipMemcpyDeviceToHost, stream));
    ZK_HIP_TRY(hipStreamSynchronize(stream));
    return ZK_OK;
}

static void digest_of_leaves(uint8_t out[32], const uint8_t* leaves, uint32_t nleaves) {
    host::Sha256 h;
    h.update(leaves, (size_t)nleaves * 32);
    h.finish(out);
}

// ---- prover --------------------------------------------------------------------------------------
//
// One routine proves K instances with a single sumcheck over
//   f = sum_i lambda^i f_i,   claim_0 = (sum_i lambda^i)(alpha + alpha^2),
// f_i the tlookup summand of instance i; beta, alpha, u and the round challenges
// are shared.  tlookup_prove is K = 1 without lambda and with its own transcript
// label and proof header.  Per instance the device work is exactly that of a
// single proof: every round launches the instance's kernels one after the other
// on the stream, each instance's sums land in its own part of the mailbox, only
// the last launch of a round publishes, and the host adds the instances' round
// polynomials weighted by lambda^i.
//
// Shapes may differ (tlookup_prove_multi).  The sumcheck then has n = max_i n_i
// variables, instance i lives on the last n_i of them (skip_i = n - n_i) and
//   f = sum_i lambda^i 2^-skip_i f_i(x_[skip_i:]),  f_i built with u_[skip_i:]:
// in a round k < skip_i the instance is a constant, (alpha + alpha^2) 2^(skip_i-k-1)
// before its weight, which the host adds without any device work; from round
// skip_i on it runs the rounds of a proof of its own ("local round" k - skip_i)
// with the shared challenges, and all instances reach their last round together.

struct Instance {
    ProveWs w;
    fr_vec S, T;
    size_t D = 0, N = 0;             // its shape: n = log2 D, l = log2 N, h = n - l;
    int n = 0, l = 0, h = 0, skip = 0;  // skip: the rounds of the whole proof before its own first
    const EqPool* ep = nullptr;      // weight tables for u_[skip:]
    host::F cD, cT;                  // products of e~(u_t, r_t) over its bound variables (all / the table's)
    host::F half_pow;                // 2^-(local round + 1)
    host::F scale;                   // 2^-h
    int lazy_rounds = 0;             // how many of its rounds in a row have left the data arrays in 29-bit planes
    host::F inv_den;                 // what the one-sided round's other side is divided by (this round)
    host::F pass01[9];               // kRoundFirstTwo's sums: c20, c21, qd, T, qe, then the sums of A_00, A_01, A_10, A_11
    const uint32_t* idx = nullptr;
    uint32_t* b_cur = nullptr;  // where B lives at the moment (it ping-pongs while folding)
    size_t b_cur_stride = 0;
    uint32_t* words = nullptr;  // this instance's round sums in the mailbox
    uint32_t* inv_words = nullptr;    // totals of its two inversions (B, then A)
    uint32_t* const_words = nullptr;  // its two table-side constants
    uint32_t* dig_words = nullptr;    // hash-state words of digest(A), then of digest(B)
    host::F c1, c2, cB, sum_A, lam;
    host::F claim;       // the running claim of this instance's own sumcheck: f_i's round polynomial at 0 plus at 1
    host::F fX[4];       // its last round polynomial at X = 0..3
    host::F sA_prev[2];  // its last round's sums of A at X = 0, 1
    uint8_t md[32], dA[32], dB[32];
    BatchInverseJob job_a, job_b;
    bool deferred = false;  // S_i = T[idx_i] is checked through sum A = sum m B after the first round, not while counting
};

struct ProveCall {
    const uint8_t* seed = nullptr;
    size_t K = 1;
    const fr_vec* S = nullptr;
    const uint32_t* const* idx = nullptr;  // may be null, entries may be null
    const fr_vec* T = nullptr;
    bool batch = false;                    // batched transcript and proof layout
    bool multi = false;                    // batched, and the instances' shapes may differ (S[i].n, T[i].n)
    const fr_t* forced_beta = nullptr;
    bool by_rows = false;                  // A as B[idx_i] instead of inverting beta + S_i
    bool check_upfront = false;            // compare every S_i with its hinted row while counting (no deferred check)
    // S_0 given as small integers x + rho y (K = 1, hints required, S ignored): see tlookup_prove_small
    const int32_t* ints_x = nullptr;
    const int32_t* ints_y = nullptr;
    const fr_t* ints_rho = nullptr;
    size_t ints_D = 0;
    uint8_t* proof = nullptr;
    size_t cap = 0;
    size_t* len = nullptr;
    tlookup_aux* aux = nullptr;            // single proof
    tlookup_batch_aux* baux = nullptr;     // batched proof
    void* ws = nullptr;
    size_t ws_bytes = 0;
    void* stream = nullptr;
};

// ---- which kernel runs a round, and where it finds S ---------------------------------
//
// Decided in one place, by a function of the shape alone, so that it can be
// walked on the host without a GPU (zkmi_selftest_tlookup_plan) and checked
// against the pointers actually handed to a kernel before it is launched.
enum RoundKernel {
    kRoundFirst = 0,     // k_round_data0: the first round, nothing to fold
    kRound29 = 1,        // k_round_data29: large folding rounds on 29-bit limbs
    kRoundBoth = 2,      // k_round_both: data and table side, the table's variables being bound
    kRoundOneGroup = 3,  // k_round_small: at most 256 pairs, one workgroup, one round per launch (batched proofs)
    kRoundResident = 4,  // k_tlookup_tail: at most 256 pairs, one resident kernel over these rounds (until kRoundHost)
    kRoundFirstTwo = 5,  // k_round_data01: the first pass, which yields the sums of the first two rounds
    kRoundNoPass = 6,    // the second round after kRoundFirstTwo: the host has everything, nothing is launched
    kRoundHost = 7       // at most kHostPairs pairs of a single proof: the resident kernel has handed the arrays to the
                         // host, which runs the round itself (HostTail)
};
enum SSource {
    kSFromCaller = 0,  // the caller's vector of field elements
    kSFromInts = 1,    // the caller's integer columns (tlookup_prove_small)
    kSFromWords = 2,   // the folded copy in the workspace, 32-bit words
    kSFromPlanes = 3,  // the folded copy in the workspace, 29-bit limb planes
    kSNowhere = -1     // a plan this library has no kernel for: never launched
};

struct RoundPlan {
    int kernel;
    int s_source;
    bool table_round;  // the variable being bound is one of the table's
    bool tiny;         // at most kSmallPairs pairs
    bool use29;
    bool in32, out32;  // kRound29: the data arrays arrive as / leave as 32-bit words
    bool fold2;        // kRound29: binds the two previous variables at once (after kRoundFirstTwo, kRoundNoPass)
    int lazy_after;    // folds since the data arrays were last fully reduced, if they are in 29-bit planes now
};

// The last rounds of a single proof on the host.  A round of the resident kernel costs a trip to the host and back
// (about thirty microseconds) whatever it computes; a round of 32 pairs is some six hundred multiplications, which
// the host does in a fraction of that.  So once a round has at most kHostPairs pairs, the resident kernel binds the
// last challenge, writes the five arrays (at most 64 elements each) into the mailbox and ends, and the host computes
// the remaining rounds' sums, folds and final claims from them: the same sums over the same arrays (Section 3.3's
// sumcheck, Section 4's summand), exact arithmetic, so the same bytes.
static const size_t kHostPairs = kMailboxShipEntries / 2;

struct HostTail {
    host::F A[kMailboxShipEntries], S[kMailboxShipEntries], B[kMailboxShipEntries], M[kMailboxShipEntries],
        T[kMailboxShipEntries];
    host::F W[kHostPairs];  // this round's weights e~(u_rest, p), p < half
    bool on = false;
    int first = 0;  // the first round the host runs

    // e~((u_0 .. u_{m-1}), p) for p < 2^m, u_0 belonging to the top bit of p
    void weights(const host::F* u, int m) {
        using namespace host;
        W[0] = one();
        for (int t = 0; t < m; ++t) {
            for (size_t e = (size_t)1 << t; e-- > 0;) {
                const F hi = mul(W[e], u[t]);
                W[2 * e] = sub(W[e], hi);
                W[2 * e + 1] = hi;
            }
        }
    }
    // the round's eleven sums in the order the kernels report them: q0, q1, qinf, sA0, sA1, then the table side's
    // t0, t1, tinf, m0, m1, minf (zero unless a table variable is being bound)
    void sums(size_t half, bool table_round, const host::F& beta, host::F out[11]) const {
        using namespace host;
        for (int q = 0; q < 11; ++q) out[q] = zero();
        for (size_t p = 0; p < half; ++p) {
            const F wa0 = mul(W[p], A[p]), wa1 = mul(W[p], A[p + half]);
            out[0] = add(out[0], mul(wa0, add(S[p], beta)));
            out[1] = add(out[1], mul(wa1, add(S[p + half], beta)));
            out[2] = add(out[2], mul(sub(wa1, wa0), sub(S[p + half], S[p])));
            out[3] = add(out[3], A[p]);
            out[4] = add(out[4], A[p + half]);
            if (!table_round) continue;
            const F wb0 = mul(W[p], B[p]), wb1 = mul(W[p], B[p + half]);
            out[5] = add(out[5], mul(wb0, add(T[p], beta)));
            out[6] = add(out[6], mul(wb1, add(T[p + half], beta)));
            out[7] = add(out[7], mul(sub(wb1, wb0), sub(T[p + half], T[p])));
            out[8] = add(out[8], mul(B[p], M[p]));
            out[9] = add(out[9], mul(B[p + half], M[p + half]));
            out[10] = add(out[10], mul(sub(B[p + half], B[p]), sub(M[p + half], M[p])));
        }
    }
    // binds the round's variable to r and moves the weights on to the next round
    void fold(size_t half, bool table_round, const host::F& r) {
        using namespace host;
        auto bind = [&](F* x) {
            for (size_t p = 0; p < half; ++p) x[p] = add(x[p], mul(r, sub(x[p + half], x[p])));
        };
        bind(A);
        bind(S);
        if (table_round) {
            bind(B);
            bind(M);
            bind(T);
        }
        for (size_t p = 0; p < half / 2; ++p) W[p] = add(W[p], W[p + half / 2]);  // the next variable summed out
    }
};

static bool round_on_29_bits(int n, int h, int k) {
    return k >= 1 && k < h && ((size_t)1 << (n - k - 1)) > kSmallPairs;
}

// Whether the first pass over the data serves the first two rounds (round01_dev.h)
// and the third round's kernel binds two variables at once: the three rounds must
// all bind data variables only, and the third must be one of the 29-bit kernel's.
static bool first_two_rounds_share_a_pass(int n, int h, bool from_ints) {
    return !from_ints && h >= 3 && round_on_29_bits(n, h, 2);
}

// n = log2 D, h = log2(D/N); lazy_rounds: lazy_after of the round before;
// resident_running: an earlier round has started the resident kernel.
static RoundPlan plan_round(int n, int h, int k, size_t K, bool from_ints, int lazy_rounds, bool resident_running) {
    RoundPlan pl;
    const size_t half = (size_t)1 << (n - k - 1);
    pl.table_round = k >= h;
    pl.tiny = k > 0 && half <= kSmallPairs;
    pl.use29 = round_on_29_bits(n, h, k);
    pl.in32 = lazy_rounds == 0;
    pl.out32 = pl.use29 && (!round_on_29_bits(n, h, k + 1) || lazy_rounds + 1 == kMaxLazyRounds);
    pl.lazy_after = pl.use29 && !pl.out32 ? lazy_rounds + 1 : 0;
    pl.fold2 = false;
    if (first_two_rounds_share_a_pass(n, h, from_ints) && k <= 2) {
        // rounds 0 and 1 from one pass that folds nothing, round 2 binds both their variables
        pl.kernel = k == 0 ? kRoundFirstTwo : k == 1 ? kRoundNoPass : kRound29;
        pl.use29 = k == 2;
        pl.in32 = true;
        pl.out32 = k == 2 && !round_on_29_bits(n, h, 3);
        pl.fold2 = k == 2;
        pl.lazy_after = k == 2 && !pl.out32 ? 2 : 0;
        pl.s_source = kSFromCaller;
        return pl;
    }
    if (resident_running && K == 1 && half <= kHostPairs) pl.kernel = kRoundHost;
    else if (resident_running || (pl.tiny && K == 1 && n - k <= kTailRoundsMax)) pl.kernel = kRoundResident;
    else if (pl.tiny) pl.kernel = kRoundOneGroup;
    else if (pl.table_round && k > 0) pl.kernel = kRoundBoth;
    else if (pl.use29) pl.kernel = kRound29;
    else pl.kernel = kRoundFirst;
    if (k <= 1) {
        // S has not been folded yet (round 0) or is folded by this round's kernel (round 1): it is read where the
        // caller left it.  Integers are read by the first round's kernel and by the 29-bit kernel only.
        pl.s_source = from_ints ? kSFromInts : kSFromCaller;
        if (from_ints && !((k == 0 && pl.kernel == kRoundFirst) || (k == 1 && pl.kernel == kRound29 && pl.in32)))
            pl.s_source = kSNowhere;
    } else {
        pl.s_source = pl.kernel == kRound29 && !pl.in32 ? kSFromPlanes : kSFromWords;
    }
    return pl;
}

// Whether a lookup of this shape can read S as small integers all the way: the
// multiplicities come from the hints alone (workgroup histograms), the first
// round and the first fold are kernels of their own that read integers.
static bool small_source_shape_ok(size_t D, size_t N) {
    if (!is_pow2(D) || !is_pow2(N) || N > D || N > kLdsHistMaxRows || D <= (size_t)kBlock) return false;
    const int n = log2_floor(D), h = n - log2_floor(N);
    if (n < 2) return false;
    const RoundPlan p0 = plan_round(n, h, 0, 1, true, 0, false);
    const RoundPlan p1 = plan_round(n, h, 1, 1, true, p0.lazy_after, p0.kernel == kRoundResident);
    return p0.s_source == kSFromInts && p1.s_source == kSFromInts;
}

static __global__ void k_store_fold4(SmallFold4 v, SmallFold4* dst) {
    ((uint32_t*)dst)[threadIdx.x] = ((const uint32_t*)&v)[threadIdx.x];  // 64 words
}

static size_t batch_proof_bytes(size_t D, size_t K) {
    return 32 + 96 * K + (size_t)log2_floor(D ? D : 1) * 128 + 160 * K;
}

// "ZKTM" | u32 1 | LE64 K | K x (LE64 D_i, LE64 N_i) | K digests of m | K x [digest(A) digest(B)] | rounds | K x 5 claims
static size_t multi_proof_bytes(int n_max, size_t K) { return 16 + 16 * K + 96 * K + (size_t)n_max * 128 + 160 * K; }

static int prove_core(const ProveCall& c) {
    using namespace host;
    const size_t K = c.K;
    const bool from_ints = c.ints_x != nullptr;
    if (!c.seed || (!c.S && !from_ints) || !c.T || K == 0 || K > kMailboxMaxInstances) return ZK_E_BADARG;
    if (!c.batch && (K != 1 || c.multi)) return ZK_E_BADARG;
    if (from_ints && (K != 1 || c.batch || c.by_rows || !c.idx || !c.idx[0])) return ZK_E_BADARG;
    // shapes: one for all, unless the call says they may differ
    size_t Ds[kMailboxMaxInstances], Ns[kMailboxMaxInstances];
    int n = 0;  // variables of the sumcheck: those of the longest instance
    for (size_t i = 0; i < K; ++i) {
        Ds[i] = from_ints ? c.ints_D : c.S[c.multi ? i : 0].n;
        Ns[i] = c.T[c.multi ? i : 0].n;
        if (!is_pow2(Ds[i]) || !is_pow2(Ns[i]) || Ns[i] > Ds[i] || Ds[i] > ((size_t)1 << 31)) return ZK_E_BADARG;
        if (c.T[i].n != Ns[i] || !vec_ok(c.T[i], Ns[i])) return ZK_E_BADARG;
        if (!from_ints && (c.S[i].n != Ds[i] || !vec_ok(c.S[i], Ds[i]))) return ZK_E_BADARG;
        if (c.by_rows && !(c.idx && c.idx[i])) return ZK_E_BADARG;
        if (log2_floor(Ds[i]) > n) n = log2_floor(Ds[i]);
    }
    if (from_ints && !small_source_shape_ok(Ds[0], Ns[0])) return ZK_E_BADARG;
    if (from_ints && ((c.ints_y != nullptr) != (c.ints_rho != nullptr))) return ZK_E_BADARG;
    if (from_ints && c.ints_rho && !canonical_in_range(*c.ints_rho)) return ZK_E_BADARG;
    // the tensor as small integers, if it came that way
    SmallSource ints_src;
    memset(&ints_src, 0, sizeof ints_src);
    F ints_rho = zero();
    const F two64 = mul(from_u64((uint64_t)1 << 32), from_u64((uint64_t)1 << 32));
    if (from_ints) {
        if (c.ints_rho) ints_rho = from_canonical(*c.ints_rho);
        ints_src.x = c.ints_x;
        ints_src.y = c.ints_y;
        to_device_limbs(ints_src.plus_one, two64);
        to_device_limbs(ints_src.minus_one, neg(two64));
        to_device_limbs(ints_src.plus_rho, mul(ints_rho, two64));
        to_device_limbs(ints_src.minus_rho, neg(mul(ints_rho, two64)));
    }
    if (c.forced_beta && !canonical_in_range(*c.forced_beta)) return ZK_E_BADARG;
    const size_t need = c.multi ? multi_proof_bytes(n, K) : c.batch ? batch_proof_bytes(Ds[0], K) : tlookup_proof_bytes(Ds[0]);
    if (c.len) *c.len = need;
    if (!c.proof || c.cap < need) return ZK_E_BUFSZ;
    if (!c.ws || c.ws_bytes < prove_ws_bytes_shapes(Ds, Ns, K)) return ZK_E_BUFSZ;
    hipStream_t stream = as_stream(c.stream);
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(c.ws, c.ws_bytes);
    Instance inst[kMailboxMaxInstances];
    const F inv2 = inv(from_u64(2));
    for (size_t i = 0; i < K; ++i) {
        Instance& I = inst[i];
        I.D = Ds[i];
        I.N = Ns[i];
        I.n = log2_floor(I.D);
        I.l = log2_floor(I.N);
        I.h = I.n - I.l;
        I.skip = n - I.n;
        carve_prove(I.w, cv, I.D, I.N);
        I.S = from_ints ? fr_vec{nullptr, I.D, I.D} : c.S[i];  // with integers there is no vector: every reader of I.S.limbs
        I.T = c.T[i];                                           // is gated by the round's plan (s_source)
        I.idx = c.idx ? c.idx[i] : nullptr;
        I.b_cur = I.w.B;
        I.b_cur_stride = I.N;
        I.words = mb->words + kMailboxSlot * i;
        I.inv_words = mb->words + kMailboxInvB + 16 * i;
        I.const_words = mb->words + kMailboxTableC + 16 * i;
        I.dig_words = mb->words + kMailboxDigest + 16 * i;
        I.c1 = I.c2 = I.cB = I.sum_A = zero();
        I.cD = I.cT = I.half_pow = one();
        I.inv_den = zero();
        I.scale = one();
        for (int t = 0; t < I.h; ++t) I.scale = mul(I.scale, inv2);
    }
    if (cv.overflow()) return ZK_E_BUFSZ;

    ProfileScope prof_total(kProfTotal, stream);

    // -- Prep: multiplicities and their digests -------------------------------------------------
    bool defer_all = !c.by_rows && !c.check_upfront;
    for (size_t i = 0; i < K; ++i) defer_all = defer_all && can_defer_check(inst[i].w, inst[i].idx, inst[i].D);
    if (from_ints && !defer_all) return ZK_E_BADARG;  // counting would read S as a vector
    for (size_t i = 0; i < K; ++i) {
        uint64_t bad = 0;
        int rc;
        {
            ProfileScope prof(kProfCount, stream);
            // with hints, the inverse vectors themselves tell whether S_i = T[idx_i] everywhere (see the first round);
            // all instances or none, so that the first instance at fault is the one reported
            inst[i].deferred = defer_all;
            rc = count_rows(inst[i].w, inst[i].S, inst[i].idx, inst[i].T, inst[i].D, inst[i].N, &bad, mb, stream,
                            inst[i].deferred, true);
        }
        if (rc == ZK_E_NOT_IN_TABLE) {
            if (c.aux) c.aux->bad_index = bad;
            if (c.baux) {
                c.baux->bad_instance = i;
                c.baux->bad_index = bad;
            }
        }
        ZK_TRY(rc);
        digest_of_leaves(inst[i].md, mb->bulk + 16, inst[i].w.nleaves);
    }

    uint64_t dims[1 + 2 * kMailboxMaxInstances];
    int ndims;
    if (c.multi) {
        dims[0] = K;
        for (size_t i = 0; i < K; ++i) {
            dims[1 + 2 * i] = inst[i].D;
            dims[2 + 2 * i] = inst[i].N;
        }
        ndims = 1 + 2 * (int)K;
    } else {
        dims[0] = inst[0].D;
        dims[1] = inst[0].N;
        dims[2] = K;
        ndims = c.batch ? 3 : 2;
    }
    Transcript tr(c.multi ? "zkmi/tlookup-multi/v1" : c.batch ? "zkmi/tlookup-batch/v2" : "zkmi/tlookup/v2", c.seed, dims, ndims);
    for (size_t i = 0; i < K; ++i) tr.absorb("m", inst[i].md, 32);

    // -- Prove: beta, inverse vectors ---------------------------------------------------------------
    F beta = tr.challenge("beta");
    if (c.forced_beta) beta = from_canonical(*c.forced_beta);
    if (!c.by_rows) {
        // all inversions share one wait: the down passes, one round trip, one host
        // inversion (of the product of all grand totals), the up passes.  The table
        // is inverted together with the tensor, as one vector, whenever the tensor's
        // length allows (its small passes then cost nothing of their own).
        ProfileScope prof(kProfInverse, stream);
        Carver inv_cv = cv;
        const uint32_t seq = mb->next_seq();
        BatchInverseJob* jobs[2 * kMailboxMaxInstances];
        const uint32_t* totals[2 * kMailboxMaxInstances];
        size_t njobs = 0;
        for (size_t i = 0; i < K; ++i) {
            Instance& I = inst[i];
            const size_t D = I.D, N = I.N;
            const uint32_t last = i + 1 == K ? seq : 0;
            const bool joined = batch_inverse_can_join(D) && D > (size_t)kBlock;
            if (joined) {
                ZK_TRY(batch_inverse_begin(I.job_a, I.w.A, D, I.S.limbs, I.S.stride, D, beta, inv_cv, I.inv_words + 8,
                                           mb->words, last, stream, I.w.B, N, I.T.limbs, I.T.stride, N,
                                           from_ints ? &ints_src : nullptr));
            } else {
                ZK_TRY(batch_inverse_begin(I.job_b, I.w.B, N, I.T.limbs, I.T.stride, N, beta, inv_cv, I.inv_words, mb->words,
                                           0, stream, nullptr, 0, nullptr, 0, 0));
                jobs[njobs] = &I.job_b;
                totals[njobs++] = I.inv_words;
                ZK_TRY(batch_inverse_begin(I.job_a, I.w.A, D, I.S.limbs, I.S.stride, D, beta, inv_cv, I.inv_words + 8,
                                           mb->words, last, stream, nullptr, 0, nullptr, 0, 0,
                                           from_ints ? &ints_src : nullptr));
            }
            jobs[njobs] = &I.job_a;
            totals[njobs++] = I.inv_words + 8;
        }
        ZK_TRY(mailbox_wait(mb, seq, stream));
        // inverse of each total from one inversion of their product
        F tot[2 * kMailboxMaxInstances], pre[2 * kMailboxMaxInstances + 1];
        pre[0] = one();
        for (size_t q = 0; q < njobs; ++q) {
            tot[q] = from_dev(totals[q]);
            if (is_zero(tot[q])) return ZK_E_ZERO_DENOM;
            pre[q + 1] = mul(pre[q], tot[q]);
        }
        F suffix_inv = inv(pre[njobs]);  // 1 / (tot_0 ... tot_q) while walking down
        for (size_t q = njobs; q-- > 0;) {
            F inv_q = mul(suffix_inv, pre[q]);
            suffix_inv = mul(suffix_inv, tot[q]);
            ZK_TRY(batch_inverse_end(*jobs[q], inv_q, stream));
        }
    } else {
        // every S_i has been checked to equal T[idx_i]: invert the table side only
        // and read A off it (a zero beta + S_i is a zero beta + T[idx_i])
        ProfileScope prof(kProfInverse, stream);
        for (size_t i = 0; i < K; ++i) {
            Instance& I = inst[i];
            const size_t D = I.D, N = I.N;
            Carver inv_cv = cv;
            ZK_TRY(batch_inverse_run(I.w.B, N, I.T.limbs, I.T.stride, N, beta, inv_cv, mb, stream));
            hipLaunchKernelGGL(k_rows_of, dim3(grid_for(N)), dim3(kBlock), 0, stream, I.w.rows, I.w.B, N, (uint32_t)N);
            hipLaunchKernelGGL(k_gather_rows, dim3(grid_for(D, kBlock, 16384)), dim3(kBlock), 0, stream, I.w.A, D, D, I.idx,
                               I.w.rows);
            ZK_HIP_TRY(hipGetLastError());
        }
    }

    // The prover sends A and B before the sumcheck (Protocol 1, tlookup-Prove): their
    // digests, standing in for the commitments, enter the transcript before alpha
    // and u are drawn.
    {
        ProfileScope prof(kProfDigest, stream);
        const uint32_t seq = mb->next_seq();
        for (size_t i = 0; i < K; ++i) {
            Instance& I = inst[i];
            const VecDigestJob ja{I.w.A, I.D, I.D, I.w.dig_rows, I.dig_words}, jb{I.w.B, I.N, I.N, I.w.dig_rows_b, I.dig_words + 8};
            vec_digest_launch(ja, &jb, I.w.dig_leaves, mb->words, i + 1 == K ? seq : 0, I.w.flags + 1, stream);
        }
        ZK_HIP_TRY(hipGetLastError());
        ZK_TRY(mailbox_wait(mb, seq, stream));
        for (size_t i = 0; i < K; ++i) {
            digest_bytes(inst[i].dA, inst[i].dig_words);
            digest_bytes(inst[i].dB, inst[i].dig_words + 8);
            tr.absorb("A", inst[i].dA, 32);
            tr.absorb("B", inst[i].dB, 32);
        }
    }

    F alpha = tr.challenge("alpha");
    F alpha2 = sqr(alpha);
    F u[32];
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");
    F lambda = one();
    if (c.batch) lambda = tr.challenge("lambda");
    // an instance's weight in f: lambda^i, times 2^-skip when it is shorter than the longest
    {
        F lam_pow = one();
        for (size_t i = 0; i < K; ++i) {
            inst[i].lam = lam_pow;
            for (int t = 0; t < inst[i].skip; ++t) inst[i].lam = mul(inst[i].lam, inv2);
            lam_pow = mul(lam_pow, lambda);
        }
    }

    // weight tables: instance i uses u_[skip_i:], so instances of one length share a pool
    EqPool pools[kMailboxMaxInstances];
    for (size_t i = 0; i < K; ++i) {
        for (size_t j = 0; j < i && !inst[i].ep; ++j)
            if (inst[j].D == inst[i].D) inst[i].ep = inst[j].ep;
        if (inst[i].ep) continue;
        ZK_TRY(eq_pool_build(pools[i], u + inst[i].skip, inst[i].n, cv, stream));
        inst[i].ep = &pools[i];
    }

    // -- table-side constants ---------------------------------------------------------------------
    // c1 = sum_j e'_j B_j (T_j+beta), c2 = sum_j m_j B_j.  e' = e~(u_[h:], .) is the
    // weight table of "round h-1" (remaining variables h .. n-1); with h = 0 no
    // round needs the constant, only c2 is reported.
    for (size_t i = 0; i < K; ++i) {
        Instance& I = inst[i];
        const size_t N = I.N;
        const int h = I.h;
        const EqPool& ep = *I.ep;
        TableConstArgs a;
        a.B = I.w.B; a.bs = N;
        a.T = I.T.limbs; a.ts = I.T.stride;
        a.M = I.w.M; a.ms = N;
        a.N = N;
        a.beta = to_dev(beta);
        if (h >= 1) {
            a.eq = ep.round(h - 1);
        } else {
            // weights unused for the reported sum; point at the one-entry table
            a.eq = EqSplit{ep.pool, ep.stride, ep.suffix_off[0], 0, 0, 0};
        }
        a.partials = I.w.partT;
        a.pstride = I.w.part_blocks * 6;
        unsigned blocks = grid_for(N, kBlock * 4, kMaxPartialBlocks);
        hipLaunchKernelGGL(k_table_const, dim3(blocks), dim3(kBlock), 0, stream, a);
        // read back together with the first round's sums (or the final values)
        launch_final_sum(I.w.partT, a.pstride, blocks, 2, I.const_words, mb->words, 0, I.w.flags + 1, stream);
        ZK_HIP_TRY(hipGetLastError());
    }
    bool table_consts_read = false;
    auto read_table_consts = [&]() {
        if (table_consts_read) return;
        for (size_t i = 0; i < K; ++i) {
            inst[i].c1 = from_dev(inst[i].const_words);
            inst[i].c2 = from_dev(inst[i].const_words + 8);
            inst[i].cB = sub(mul(alpha2, inst[i].c1), inst[i].c2);
        }
        table_consts_read = true;
    };

    // -- header -----------------------------------------------------------------------------------------
    uint8_t* out = c.proof;
    if (c.multi) {
        memcpy(out, "ZKTM", 4);
        out[4] = 1; out[5] = out[6] = out[7] = 0;
        put_le64(out + 8, K);
        out += 16;
        for (size_t i = 0; i < K; ++i) {
            put_le64(out, inst[i].D);
            put_le64(out + 8, inst[i].N);
            out += 16;
        }
    } else {
        memcpy(out, c.batch ? "ZKTB" : "ZKTL", 4);
        out[4] = 2; out[5] = out[6] = out[7] = 0;
        put_le64(out + 8, inst[0].D);
        put_le64(out + 16, inst[0].N);
        out += 24;
        if (c.batch) {
            put_le64(out, K);
            out += 8;
        }
    }
    for (size_t i = 0; i < K; ++i) {
        memcpy(out, inst[i].md, 32);
        out += 32;
    }
    for (size_t i = 0; i < K; ++i) {
        memcpy(out, inst[i].dA, 32);
        memcpy(out + 32, inst[i].dB, 32);
        out += 64;
    }

    // -- rounds -----------------------------------------------------------------------------------------
    // Below, k counts the rounds of the whole proof and kk = k - skip those of one
    // instance ("local"): an instance's kernels, plan and arrays only ever see kk.
    F r_prev = zero(), r_prev2 = zero();  // the challenges of the last round and of the one before it
    // Rounds that fold the data arrays only and are large run on 29-bit limbs
    // (tlookup_round29.h).  Between two of them the arrays stay in 29-bit planes,
    // unreduced, for at most kMaxLazyRounds rounds in a row.
    const F29 beta29 = f29_unpack(to_dev(beta).l);
    // Where local round kk reads and writes the arrays that change place: S comes from
    // the caller's vector until it has been folded once, T likewise, and B alternates
    // between its two buffers on every fold (it has two readers).  b_cur: where B is
    // before the round; returns where it is afterwards.
    struct Moving {
        PairArray S, B, T;
    };
    auto moving_arrays = [&](int kk, const Instance& I, uint32_t*& b_cur, size_t& b_stride, bool s_unfolded) {
        const ProveWs& w = I.w;
        const size_t D = I.D, N = I.N;
        const int h = I.h;
        Moving m;
        if (s_unfolded) m.S = PairArray{I.S.limbs, I.S.stride, w.Sf, D / 2};
        else m.S = PairArray{w.Sf, D / 2, w.Sf, D / 2};
        if (kk > h) {
            uint32_t* other = b_cur == w.B ? w.Bf : w.B;
            size_t other_stride = b_cur == w.B ? N / 2 : N;
            m.B = PairArray{b_cur, b_stride, other, other_stride};
            b_cur = other;
            b_stride = other_stride;
        } else {
            m.B = PairArray{b_cur, b_stride, b_cur, b_stride};
        }
        if (kk <= h + 1) m.T = PairArray{I.T.limbs, I.T.stride, w.Tf, N / 2};
        else m.T = PairArray{w.Tf, N / 2, w.Tf, N / 2};
        return m;
    };
    auto final_arrays = [&](const Instance& I, const uint32_t* b_cur, size_t b_stride) {
        const ProveWs& w = I.w;
        const size_t D = I.D, N = I.N;
        FinalArgs f;
        memset(&f, 0, sizeof f);
        f.count = 5;
        const bool d_fold = I.n >= 1, t_fold = I.l >= 1;
        // A, S, B, m, T in the order of the proof
        f.p[0] = w.A; f.stride[0] = D; f.fold[0] = d_fold;
        if (I.n <= 1) { f.p[1] = I.S.limbs; f.stride[1] = I.S.stride; }
        else { f.p[1] = w.Sf; f.stride[1] = D / 2; }
        f.fold[1] = d_fold;
        f.p[2] = b_cur; f.stride[2] = b_stride; f.fold[2] = t_fold;
        f.p[3] = w.M; f.stride[3] = N; f.fold[3] = t_fold;
        if (I.l <= 1) { f.p[4] = I.T.limbs; f.stride[4] = I.T.stride; }
        else { f.p[4] = w.Tf; f.stride[4] = N / 2; }
        f.fold[4] = t_fold;
        return f;
    };
    // A single proof runs its small rounds in one resident kernel (k_tlookup_tail) and the very last on the host.
    TlookupTailArgs tail;
    int tail_first = -1;  // the round the resident kernel was launched for, if it is running
    TailGuard tail_guard{mb, stream};
    HostTail host_tail;
    for (int k = 0; k < n; ++k) {
        // The 29-bit kernel sums one side of the round only (X = 0, or X = 1 with side1); the other side's two sums
        // follow from what the prover has already sent: sA0 + sA1 is the previous round's sum of A at its challenge,
        // g(0) + g(1) the running claim.  The second needs a division by alpha c e~(u_k, X) of the side that was not
        // summed, so the side is chosen by which of the two is not zero (alternating otherwise, both being equally
        // good); if alpha c itself is zero, q carries no weight in g and is not needed.
        const F e_side[2] = {sub(one(), u[k]), u[k]};
        bool side1 = (k & 1) != 0;
        if (is_zero(e_side[0])) side1 = false;  // u_k = 1: only g(1) can tell q1, so sum the X = 0 side
        if (is_zero(e_side[1])) side1 = true;
        // the last instance that has kernels in this round publishes it; a round in which no instance has any (every
        // active one is in the second round of a pass that served two) is answered by the host alone
        RoundPlan plans[kMailboxMaxInstances] = {};
        size_t last_launch = K;
        for (size_t i = 0; i < K; ++i) {
            const Instance& I = inst[i];
            if (k < I.skip) continue;
            plans[i] = plan_round(I.n, I.h, k - I.skip, K, from_ints, I.lazy_rounds, tail_first >= 0);
            if (plans[i].s_source == kSNowhere) return ZK_E_BADARG;  // cannot happen: small_source_shape_ok has walked these rounds
            if (plans[i].kernel != kRoundNoPass) last_launch = i;
        }
        const bool any_launch = last_launch < K || tail_first >= 0;

        if (K == 1 && plans[0].kernel == kRoundResident && tail_first < 0) {
            // this and every later round in one launch (K = 1, so k is the instance's own count)
            Instance& I = inst[0];
            const size_t D = I.D, N = I.N;
            const int h = I.h;
            memset(&tail, 0, sizeof tail);
            tail.A = PairArray{I.w.A, D, I.w.A, D};
            tail.M = PairArray{I.w.M, N, I.w.M, N};
            tail.beta = to_dev(beta);
            tail.r_prev = to_dev(r_prev);
            // the kernel's rounds: up to the first one short enough for the host (kRoundHost), if there is one
            int k_host = k + 1;
            while (k_host < n && ((size_t)1 << (n - k_host - 1)) > kHostPairs) ++k_host;
            tail.nrounds = k_host - k;
            uint32_t* b_at = I.b_cur;
            size_t b_at_stride = I.b_cur_stride;
            for (int j = k; j < k_host; ++j) {
                TailRound& rd = tail.round[j - k];
                Moving m = moving_arrays(j, I, b_at, b_at_stride, j <= 1);
                rd.S = m.S;
                rd.B = m.B;
                rd.T = m.T;
                rd.eq = I.ep->round(j);
                rd.half = (size_t)1 << (n - j - 1);
                rd.table = j < h ? 0 : j == h ? 1 : 2;
            }
            tail.fin = final_arrays(I, b_at, b_at_stride);
            if (k_host < n) {
                // what the kernel hands over after round k_host - 1: the data arrays with that round's variable still
                // to bind, the table's arrays likewise once its variables are being bound, as they came before that
                const int j_last = k_host - 1;
                const uint32_t n_data = (uint32_t)1 << (n - k_host);
                const bool table_bound = j_last >= h;
                const uint32_t n_table = table_bound ? n_data : (uint32_t)N;
                if (n_data > kMailboxShipEntries || n_table > kMailboxShipEntries) return ZK_E_BADARG;  // cannot happen: N <= 2^(n - h)
                TailShip& sh = tail.ship;
                sh.out = mb->words + kMailboxShip;
                sh.p[0] = I.w.A; sh.stride[0] = D; sh.n_out[0] = n_data; sh.fold[0] = 1;
                sh.p[1] = I.w.Sf; sh.stride[1] = D / 2; sh.n_out[1] = n_data; sh.fold[1] = 1;
                sh.p[2] = b_at; sh.stride[2] = b_at_stride; sh.n_out[2] = n_table; sh.fold[2] = table_bound;
                sh.p[3] = I.w.M; sh.stride[3] = N; sh.n_out[3] = n_table; sh.fold[3] = table_bound;
                if (j_last >= h + 1) { sh.p[4] = I.w.Tf; sh.stride[4] = N / 2; }
                else { sh.p[4] = I.T.limbs; sh.stride[4] = I.T.stride; }
                sh.n_out[4] = n_table; sh.fold[4] = table_bound;
                host_tail.on = true;
                host_tail.first = k_host;
            }
            tail.out_words = I.words;
            tail.words = mb->words;
            tail.cmd = mb->cmd;
            for (int j = 0; j <= tail.nrounds; ++j) tail.out_seq[j] = mb->next_seq();
            for (int j = 0; j < tail.nrounds; ++j) tail.cmd_seq[j] = mb->next_cmd_seq();
            tail.spin_limit = device_spin_limit();
            mailbox_channel_reset(mb);
            {
                ProfileScope prof(kProfRoundSmall, stream);
                hipLaunchKernelGGL(k_tlookup_tail, dim3(1), dim3(kSmallThreads), 0, stream, tail);
            }
            ZK_HIP_TRY(hipGetLastError());
            tail_guard.armed = true;
            tail_first = k;
        }
        const bool host_round = host_tail.on && k >= host_tail.first;
        if (host_round && k == host_tail.first) {
            // the resident kernel's last message: the arrays, from here on the host's
            ZK_TRY(mailbox_wait(mb, tail.out_seq[tail.nrounds], stream));
            tail_guard.armed = false;
            const uint32_t* at = mb->words + kMailboxShip;
            F* const arrays[5] = {host_tail.A, host_tail.S, host_tail.B, host_tail.M, host_tail.T};
            for (int q = 0; q < 5; ++q)
                for (uint32_t j = 0; j < tail.ship.n_out[q]; ++j, at += 8) arrays[q][j] = from_dev(at);
            host_tail.weights(u + k + 1, n - k - 1);
        }
        const uint32_t seq = host_round ? 0 : tail_first >= 0 ? tail.out_seq[k - tail_first] : any_launch ? mb->next_seq() : 0;
        for (size_t i = 0; i < K && tail_first < 0; ++i) {
            Instance& I = inst[i];
            if (k < I.skip || plans[i].kernel == kRoundNoPass) continue;
            ProveWs& w = I.w;
            const size_t D = I.D, N = I.N;
            const int h = I.h, kk = k - I.skip;
            const RoundPlan& plan = plans[i];
            const size_t half = (size_t)1 << (I.n - kk - 1);
            const EqSplit eq = I.ep->round(kk);
            const EqPool& ep = *I.ep;
            const bool table_round = plan.table_round;
            const bool in32 = plan.in32, out32 = plan.out32;
            // pairs per workgroup: a workgroup's pairs must share the high factor of
            // their weights (at most 2^kLoBits pairs, 16 per thread).  As many as that
            // allows, since a thread's closing reduction costs about as much as two
            // pairs, but at least 512 workgroups while the round is large enough;
            // small rounds get one pair per thread
            size_t span = half / 512;
            if (span < (size_t)kBlock) span = (size_t)kBlock;
            if (span > ((size_t)1 << kLoBits)) span = (size_t)1 << kLoBits;
            if (span > half) span = half;
            const unsigned blocks = (unsigned)(half / span);
            if (blocks > w.part_blocks) return ZK_E_BUFSZ;  // cannot happen: see round_blocks_max
            const uint32_t my_seq = i == last_launch ? seq : 0;  // the last instance's last launch publishes the round
            const Moving mv = moving_arrays(kk, I, I.b_cur, I.b_cur_stride, kk <= 1 || plan.fold2);
            DataRoundArgs d;
            d.A = PairArray{w.A, D, w.A, D};
            d.S = mv.S;
            d.half = half;
            d.block_span = span;
            d.r_prev = to_dev(r_prev);
            d.beta = to_dev(beta);
            d.eq = eq;
            d.partials = w.partD;
            d.pstride = w.part_blocks * 5;
            memset(&d.ints, 0, sizeof d.ints);
            if (plan.s_source == kSFromInts && plan.kernel == kRoundFirst) d.ints = ints_src;
            // every kernel below reads S through d.S.src unless the plan says otherwise: no launch with nothing behind it
            if ((plan.s_source == kSFromCaller || plan.s_source == kSFromWords) && !d.S.src) return ZK_E_BADARG;
            if (plan.s_source == kSFromInts && !ints_src.x) return ZK_E_BADARG;
            if (!d.A.src || !d.partials) return ZK_E_BADARG;
            TableRoundArgs t;
            t.B = mv.B;
            t.T = mv.T;
            t.M = PairArray{w.M, N, w.M, N};
            t.half = half;
            t.block_span = span;
            t.r_prev = d.r_prev;
            t.beta = d.beta;
            t.eq = eq;
            t.partials = w.partT;
            t.pstride = w.part_blocks * 6;

            if (plan.kernel == kRoundFirstTwo) {
                // one pass for this round and the next: nothing is folded, the weights are the next round's
                const size_t quarter = half / 2;
                const EqSplit eq1 = ep.round(kk + 1);
                size_t span01 = quarter / 512;
                if (span01 < (size_t)kBlock) span01 = (size_t)kBlock;
                if (span01 > (size_t)kBlock * kRound01MaxQuads) span01 = (size_t)kBlock * kRound01MaxQuads;
                if (span01 > quarter) span01 = quarter;
                const unsigned blocks01 = (unsigned)(quarter / span01);
                if (blocks01 > w.part_blocks || span01 > ((size_t)1 << eq1.lbits) || !I.S.limbs) return ZK_E_BADARG;  // cannot happen
                DataRound01Args d01;
                d01.A = w.A;
                d01.as = D;
                d01.S = I.S.limbs;
                d01.ss = I.S.stride;
                d01.quarter = quarter;
                d01.block_span = span01;
                d01.weights = Planes29{ep.pool29, ep.count29};
                d01.lo_off = ep.suffix29_off[eq1.lbits];
                d01.lbits = eq1.lbits;
                d01.has_hi = eq1.has_hi;
                d01.hi_pool = ep.pool;
                d01.hi_stride = ep.stride;
                d01.hi_off = eq1.hi_off;
                d01.partD = w.partD;
                d01.pstrideD = w.part_blocks * 5;
                d01.partT = w.partT;
                d01.pstrideT = w.part_blocks * 6;
                {
                    ProfileScope prof(kProfRoundData, stream);
                    hipLaunchKernelGGL(k_round_data01, dim3(blocks01), dim3(kBlock), 0, stream, d01);
                }
                launch_final_sum2(w.partD, d01.pstrideD, 5, w.partT, d01.pstrideT, 6, blocks01, I.words, mb->words, my_seq,
                                  w.flags + 1, stream);
            } else if (plan.kernel == kRoundOneGroup) {
                // one workgroup, one launch, sums straight to the host
                ProfileScope prof(kProfRoundSmall, stream);
                if (!table_round)
                    hipLaunchKernelGGL(k_round_small<0>, dim3(1), dim3(kSmallThreads), 0, stream, d, t, I.words, mb->words,
                                       my_seq);
                else if (kk == h)
                    hipLaunchKernelGGL(k_round_small<1>, dim3(1), dim3(kSmallThreads), 0, stream, d, t, I.words, mb->words,
                                       my_seq);
                else
                    hipLaunchKernelGGL(k_round_small<2>, dim3(1), dim3(kSmallThreads), 0, stream, d, t, I.words, mb->words,
                                       my_seq);
            } else if (plan.kernel == kRoundBoth) {
                {
                    ProfileScope prof(kProfRoundSmall, stream);
                    if (kk > h) hipLaunchKernelGGL(k_round_both<true>, dim3(blocks, 3), dim3(kBlock), 0, stream, d, t);
                    else hipLaunchKernelGGL(k_round_both<false>, dim3(blocks, 3), dim3(kBlock), 0, stream, d, t);
                }
                launch_final_sum2(w.partD, d.pstride, 5, w.partT, t.pstride, 6, blocks, I.words, mb->words, my_seq,
                                  w.flags + 1, stream);
            } else if (plan.kernel == kRound29) {
                // as many pairs per workgroup as its weights' shared factor allows, but at least 512 workgroups while the
                // round is large enough (measured: 1024 workgroups do the same, 2048 and workgroups of three or two
                // wavefronts are slower)
                const unsigned threads29 = (unsigned)kBlock;
                const size_t span29 = span;
                const unsigned blocks29 = blocks;
                if (span29 > (size_t)threads29 * kRound29MaxPairs) return ZK_E_BUFSZ;  // cannot happen
                DataRound29Args d29;
                // 32-bit words: A in place (stride D), S from the caller's vector or Sf; 29-bit limbs: A29, S29
                d29.A = Array29{w.A, D, Planes29{w.A29, D / 2}, w.A, D};
                d29.S = Array29{d.S.src, d.S.ss, Planes29{w.S29, D / 2}, w.Sf, D / 2};
                d29.half = half;
                d29.block_span = span29;
                d29.off0 = side1 ? half : 0;
                d29.off1 = side1 ? 0 : half;
                d29.r_prev = f29_unpack(to_dev(mul(r_prev, from_u64(32))).l);
                d29.r_first = f29_unpack(to_dev(mul(r_prev2, from_u64(32))).l);
                d29.r_both = f29_unpack(to_dev(mul(mul(r_prev2, r_prev), from_u64(32))).l);
                d29.beta = beta29;
                d29.weights = Planes29{ep.pool29, ep.count29};
                d29.lo_off = ep.suffix29_off[eq.lbits];
                d29.lbits = eq.lbits;
                d29.has_hi = eq.has_hi;
                d29.hi_pool = ep.pool;
                d29.hi_stride = ep.stride;
                d29.hi_off = eq.hi_off;
                d29.partials = d.partials;
                d29.pstride = d.pstride;
                d29.sx = nullptr;
                d29.sy = nullptr;
                d29.sf = w.fold4;
                const bool ints_round = plan.s_source == kSFromInts;
                if (ints_round) {
                    // constants of x0 + r (x1 - x0) + rho y0 + rho r (y1 - y0), r the first challenge
                    d29.sx = c.ints_x;
                    d29.sy = c.ints_y;
                    SmallFold4 f4;
                    const F cr = mul(r_prev, two64), crho = mul(ints_rho, two64), crr = mul(crho, r_prev);
                    to_device_limbs(f4.plus_one, two64);
                    to_device_limbs(f4.minus_one, neg(two64));
                    to_device_limbs(f4.plus_c, cr);
                    to_device_limbs(f4.minus_c, neg(cr));
                    to_device_limbs(f4.plus_rho, crho);
                    to_device_limbs(f4.minus_rho, neg(crho));
                    to_device_limbs(f4.plus_rho_c, crr);
                    to_device_limbs(f4.minus_rho_c, neg(crr));
                    hipLaunchKernelGGL(k_store_fold4, dim3(1), dim3(64), 0, stream, f4, w.fold4);
                }
                {
                    ProfileScope prof(kProfRound29, stream);
                    if (plan.fold2 && (ints_round || !in32)) return ZK_E_BADARG;  // cannot happen: see plan_round
                    if (plan.fold2 && out32) hipLaunchKernelGGL((k_round_data29<true, true, false, true>), dim3(blocks29), dim3(threads29), 0, stream, d29);
                    else if (plan.fold2) hipLaunchKernelGGL((k_round_data29<true, false, false, true>), dim3(blocks29), dim3(threads29), 0, stream, d29);
                    else if (ints_round && out32) hipLaunchKernelGGL((k_round_data29<true, true, true>), dim3(blocks29), dim3(threads29), 0, stream, d29);
                    else if (ints_round) hipLaunchKernelGGL((k_round_data29<true, false, true>), dim3(blocks29), dim3(threads29), 0, stream, d29);
                    else if (in32 && out32) hipLaunchKernelGGL((k_round_data29<true, true>), dim3(blocks29), dim3(threads29), 0, stream, d29);
                    else if (in32) hipLaunchKernelGGL((k_round_data29<true, false>), dim3(blocks29), dim3(threads29), 0, stream, d29);
                    else if (out32) hipLaunchKernelGGL((k_round_data29<false, true>), dim3(blocks29), dim3(threads29), 0, stream, d29);
                    else hipLaunchKernelGGL((k_round_data29<false, false>), dim3(blocks29), dim3(threads29), 0, stream, d29);
                }
                launch_final_sum2(w.partD, d.pstride, 5, w.partT, t.pstride, 0, blocks29, I.words, mb->words, my_seq,
                                  w.flags + 1, stream);
            } else {
                {  // the first round (every later one is small, binds a table variable, or runs on 29-bit limbs)
                    ProfileScope prof(kProfRoundData, stream);
                    hipLaunchKernelGGL(k_round_data0, dim3(blocks), dim3(kBlock), 0, stream, d);
                }
                if (table_round) {  // only with kk == 0, i.e. D == N
                    ProfileScope prof(kProfRoundTable, stream);
                    hipLaunchKernelGGL(k_round_table<false>, dim3(blocks), dim3(kBlock), 0, stream, t);
                }
                launch_final_sum2(w.partD, d.pstride, 5, w.partT, t.pstride, table_round ? 6 : 0, blocks, I.words,
                                  mb->words, my_seq, w.flags + 1, stream);
            }
            ZK_HIP_TRY(hipGetLastError());
        }
        // while the device works: each instance's running claim, and the inverse the 29-bit round's other side needs
        // (instances of one length share it)
        for (size_t i = 0; i < K; ++i) {
            Instance& I = inst[i];
            if (k < I.skip) continue;
            I.lazy_rounds = plans[i].lazy_after;
            I.claim = k == I.skip ? add(alpha, alpha2) : interpolate_at(I.fX, 4, r_prev);
            I.inv_den = zero();
            const F wD = mul(alpha, I.cD);
            if (plans[i].kernel != kRound29 || tail_first >= 0 || is_zero(wD)) continue;
            bool shared = false;
            for (size_t j = 0; j < i && !shared; ++j)
                if (k >= inst[j].skip && inst[j].skip == I.skip && plans[j].kernel == kRound29) {
                    I.inv_den = inst[j].inv_den;  // same bound variables, same product of weights
                    shared = true;
                }
            if (!shared) I.inv_den = inv(mul(wD, e_side[side1 ? 0 : 1]));
        }
        if (any_launch && !host_round) ZK_TRY(mailbox_wait(mb, seq, stream));
        if (k > 0 || any_launch) read_table_consts();

        F e[4], g[4];
        line_values(e, e_side[0], e_side[1]);
        for (int X = 0; X < 4; ++X) g[X] = zero();
        for (size_t i = 0; i < K; ++i) {
            Instance& I = inst[i];
            if (k < I.skip) {
                // not one of this instance's variables: its summand is the same at every X, and over the rest of the
                // cube it sums to 2^(skip - k - 1) times its whole sum alpha + alpha^2 (before its weight 2^-skip)
                F f = add(alpha, alpha2);
                for (int t = 0; t < I.skip - k - 1; ++t) f = add(f, f);
                for (int X = 0; X < 4; ++X) g[X] = add(g[X], mul(I.lam, f));
                continue;
            }
            const int kk = k - I.skip;
            const RoundPlan& plan = plans[i];
            const bool table_round = plan.table_round;
            const F wD = mul(alpha, I.cD);
            const F wT = table_round ? mul(alpha2, I.cT) : zero();
            I.half_pow = mul(I.half_pow, inv2);
            const uint32_t* sums = I.words;
            F q0, q1, qi, sA0, sA1;
            F hs[11];  // kRoundHost: the round's sums, computed here
            if (plan.kernel == kRoundHost) {
                host_tail.sums((size_t)1 << (I.n - kk - 1), table_round, beta, hs);
                q0 = hs[0];
                q1 = hs[1];
                qi = hs[2];
                sA0 = hs[3];
                sA1 = hs[4];
            } else if (plan.kernel == kRoundFirstTwo) {
                // the pass has summed, with the NEXT round's weights, what this round and the next are made of
                // (round01_dev.h): this round's leading coefficient splits by the next variable
                for (int q = 0; q < 9; ++q) I.pass01[q] = from_dev(sums + 8 * q);
                q0 = q1 = one();
                qi = add(mul(sub(one(), u[k + 1]), I.pass01[0]), mul(u[k + 1], I.pass01[1]));
                sA0 = add(I.pass01[5], I.pass01[6]);
                sA1 = add(I.pass01[7], I.pass01[8]);
            } else if (plan.kernel == kRoundNoPass) {
                // every sum of this round is a polynomial of degree two in the challenge r before it
                const F& r = r_prev;
                const F t = mul(r, sub(one(), r));
                const F* P = I.pass01;
                q0 = sub(one(), mul(t, P[0]));
                q1 = sub(one(), mul(t, P[1]));
                qi = add(P[2], mul(r, add(sub(sub(P[3], P[2]), P[4]), mul(r, P[4]))));  // qd + r (T - qd - qe) + r^2 qe
                sA0 = add(P[5], mul(r, sub(P[7], P[5])));
                sA1 = add(P[6], mul(r, sub(P[8], P[6])));
            } else {
                q0 = from_dev(sums);
                q1 = from_dev(sums + 8);
                qi = from_dev(sums + 16);
                if (kk == 0) q0 = q1 = one();  // A (S + beta) = 1 everywhere and the weights sum to 1
                sA0 = from_dev(sums + 24);
                sA1 = from_dev(sums + 32);
            }
            const F table_const = mul(I.cB, I.half_pow);
            if (plan.kernel == kRound29 && tail_first < 0) {
                // the kernel has summed one side: (q0, sA0) hold that side's q and sum of A; the other side from
                // sA(0) + sA(1) = sA_prev(r_prev) and g(0) + g(1) = claim (never a table round: the table side is a constant)
                const int a = side1 ? 1 : 0;
                const F sA_b = sub(add(I.sA_prev[0], mul(r_prev, sub(I.sA_prev[1], I.sA_prev[0]))), sA0);
                const F g_a = add(add(mul(mul(wD, e_side[a]), q0), sA0), table_const);
                const F q_b = mul(sub(sub(sub(I.claim, g_a), sA_b), table_const), I.inv_den);
                const F q_a = q0, sA_a = sA0;
                q0 = a == 0 ? q_a : q_b;
                q1 = a == 0 ? q_b : q_a;
                sA0 = a == 0 ? sA_a : sA_b;
                sA1 = a == 0 ? sA_b : sA_a;
            }
            I.sA_prev[0] = sA0;
            I.sA_prev[1] = sA1;
            if (kk == 0) I.sum_A = add(sA0, sA1);
            if (kk == 0 && I.deferred && !equal(I.sum_A, I.c2)) {
                // The counts were taken from the hints without looking at S.  Had every
                // S_i been the hinted row, sum_i 1/(beta+S_i) = sum_j m_j/(beta+T_j) would hold
                // (Section 4, first form of the identity); it does not, so some S_i differs
                // from its row: find the smallest such i by comparing them all.
                uint64_t bad = UINT64_MAX;
                ZK_TRY(find_bad_row(I.w, I.S, ints_src, I.idx, I.D, I.N, &bad, stream));
                if (bad == UINT64_MAX) return ZK_E_HIP;  // the sums disagree although every row matches
                if (c.aux) c.aux->bad_index = bad;
                if (c.baux) {
                    c.baux->bad_instance = i;
                    c.baux->bad_index = bad;
                }
                return ZK_E_NOT_IN_TABLE;
            }
            F q[4], sa[4], tq[4], tm[4];
            quad_values(q, q0, q1, qi);
            line_values(sa, sA0, sA1);
            if (table_round && plan.kernel == kRoundHost) {
                quad_values(tq, hs[5], hs[6], hs[7]);
                quad_values(tm, hs[8], hs[9], hs[10]);
            } else if (table_round) {
                quad_values(tq, from_dev(sums + 40), from_dev(sums + 48), from_dev(sums + 56));
                quad_values(tm, from_dev(sums + 64), from_dev(sums + 72), from_dev(sums + 80));
            }
            for (int X = 0; X < 4; ++X) {
                F data = add(mul(mul(wD, e[X]), q[X]), sa[X]);
                F table = table_round ? mul(I.scale, sub(mul(mul(wT, e[X]), tq[X]), tm[X])) : table_const;
                F f = add(data, table);
                I.fX[X] = f;
                g[X] = add(g[X], !c.batch ? f : mul(I.lam, f));
            }
        }
        for (int X = 0; X < 4; ++X) to_bytes(out + 32 * X, g[X]);
        tr.absorb("g", out, 128);
        out += 128;
        F r = tr.challenge("r");
        F er = add(mul(sub(one(), u[k]), sub(one(), r)), mul(u[k], r));
        for (size_t i = 0; i < K; ++i) {
            Instance& I = inst[i];
            if (k < I.skip) continue;
            I.cD = mul(I.cD, er);
            if (plans[i].table_round) I.cT = mul(I.cT, er);
        }
        r_prev2 = r_prev;
        r_prev = r;
        if (tail_first >= 0 && k - tail_first < tail.nrounds) mailbox_send_challenge(mb, tail.cmd_seq[k - tail_first], to_dev(r).l);
        if (host_round) host_tail.fold((size_t)1 << (n - k - 1), plans[0].table_round, r);
    }

    // -- final claims -------------------------------------------------------------------------------------
    {
        if (host_tail.on) {
            // the host has bound the last variable itself: each array's first element is its claim
            const F* const arrays[5] = {host_tail.A, host_tail.S, host_tail.B, host_tail.M, host_tail.T};
            for (int q = 0; q < 5; ++q) to_device_limbs(inst[0].words + 8 * q, arrays[q][0]);
        } else if (tail_first >= 0) {
            // the resident kernel writes them after the last challenge
            ZK_TRY(mailbox_wait(mb, tail.out_seq[tail.nrounds], stream));
            tail_guard.armed = false;
        } else {
            const uint32_t seq = mb->next_seq();
            for (size_t i = 0; i < K; ++i) {
                Instance& I = inst[i];
                FinalArgs f = final_arrays(I, I.b_cur, I.b_cur_stride);
                f.r = to_dev(r_prev);
                hipLaunchKernelGGL(k_final_values, dim3(1), dim3(64), 0, stream, f, I.words, mb->words, i + 1 == K ? seq : 0);
            }
            ZK_HIP_TRY(hipGetLastError());
            ZK_TRY(mailbox_wait(mb, seq, stream));
        }
        ZK_HIP_TRY(hipStreamSynchronize(stream));  // everything of this call has left the device
        read_table_consts();
        uint8_t* first = out;
        for (size_t i = 0; i < K; ++i) {
            for (int q = 0; q < 5; ++q) {
                F v = from_dev(inst[i].words + 8 * q);
                if (q == 0 && inst[i].n == 0) inst[i].sum_A = v;
                to_bytes(out, v);
                out += 32;
            }
        }
        tr.absorb("final", first, 160 * K);
    }
    if (c.aux) {
        c.aux->beta = to_canonical(beta);
        c.aux->alpha = to_canonical(alpha);
        c.aux->sum_A = to_canonical(inst[0].sum_A);
        c.aux->sum_mB = to_canonical(inst[0].c2);
        c.aux->bad_index = 0;
    }
    if (c.baux) {
        memset(c.baux, 0, sizeof *c.baux);
        c.baux->beta = to_canonical(beta);
        c.baux->alpha = to_canonical(alpha);
        c.baux->lambda = to_canonical(lambda);
        for (size_t i = 0; i < K; ++i) {
            c.baux->sum_A[i] = to_canonical(inst[i].sum_A);
            c.baux->sum_mB[i] = to_canonical(inst[i].c2);
        }
    }
    return ZK_OK;
}

// ---- verifier ----------------------------------------------------------------------------------

static size_t verify_ws_bytes(size_t D, size_t N) {
    Carver cv(nullptr, 0);
    cv.limbs(N);                                   // m as field elements
    cv.take(div_up(N, kLeafCounts) * 32);          // leaf digests
    cv.take(vec_digest_leaves(D) * 32);            // hash tree over a witness vector
    cv.take(vec_digest_row_digests(D) * 32);
    cv.take(256);                                  // its ticket
    cv.take(mle_scratch_bytes(log2_floor(D)));
    return cv.used();
}

struct VerifyCall {
    const uint8_t* seed = nullptr;
    const uint8_t* proof = nullptr;
    size_t len = 0;
    size_t K = 1;
    const fr_vec* T = nullptr;
    size_t D = 0;
    bool batch = false;
    bool multi = false;            // shapes may differ: lengths of the tensors in Ds, of the tables in T[i].n
    const size_t* Ds = nullptr;
    const tlookup_witness* wit = nullptr;  // K entries, or null
    tlookup_claims* claims = nullptr;      // single proof
    tlookup_batch_claims* bclaims = nullptr;
    void* ws = nullptr;
    size_t ws_bytes = 0;
    void* stream = nullptr;
};

static int verify_core(const VerifyCall& c) {
    using namespace host;
    const size_t K = c.K;
    if (!c.seed || !c.proof || !c.T || K == 0 || K > kMailboxMaxInstances || (!c.batch && (K != 1 || c.multi))) return ZK_E_BADARG;
    if (c.multi && !c.Ds) return ZK_E_BADARG;
    // shapes: n variables in all; instance i has n_i of them, the last ones (skip_i = n - n_i)
    size_t Ds[kMailboxMaxInstances], Ns[kMailboxMaxInstances];
    int ns[kMailboxMaxInstances], ls[kMailboxMaxInstances], hs[kMailboxMaxInstances], skips[kMailboxMaxInstances];
    int n = 0;
    size_t D_max = 1, N_max = 1;
    for (size_t i = 0; i < K; ++i) {
        Ds[i] = c.multi ? c.Ds[i] : c.D;
        Ns[i] = c.T[c.multi ? i : 0].n;
        if (!is_pow2(Ds[i]) || !is_pow2(Ns[i]) || Ns[i] > Ds[i] || Ds[i] > ((size_t)1 << 31)) return ZK_E_BADARG;
        if (c.T[i].n != Ns[i] || !vec_ok(c.T[i], Ns[i])) return ZK_E_BADARG;
        ns[i] = log2_floor(Ds[i]);
        ls[i] = log2_floor(Ns[i]);
        hs[i] = ns[i] - ls[i];
        if (ns[i] > n) n = ns[i];
        if (Ds[i] > D_max) D_max = Ds[i];
        if (Ns[i] > N_max) N_max = Ns[i];
    }
    for (size_t i = 0; i < K; ++i) skips[i] = n - ns[i];
    if (!c.ws || c.ws_bytes < verify_ws_bytes(D_max, N_max)) return ZK_E_BUFSZ;
    const uint8_t* proof = c.proof;
    const uint8_t* digests;
    if (c.multi) {
        if (c.len != multi_proof_bytes(n, K)) return ZK_E_REJECT;
        if (memcmp(proof, "ZKTM\x01\0\0\0", 8) != 0) return ZK_E_REJECT;
        if (get_le64(proof + 8) != K) return ZK_E_REJECT;
        for (size_t i = 0; i < K; ++i)
            if (get_le64(proof + 16 + 16 * i) != Ds[i] || get_le64(proof + 24 + 16 * i) != Ns[i]) return ZK_E_REJECT;
        digests = proof + 16 + 16 * K;
    } else if (c.batch) {
        if (c.len != batch_proof_bytes(Ds[0], K)) return ZK_E_REJECT;
        if (memcmp(proof, "ZKTB\x02\0\0\0", 8) != 0) return ZK_E_REJECT;
        if (get_le64(proof + 8) != Ds[0] || get_le64(proof + 16) != Ns[0] || get_le64(proof + 24) != K) return ZK_E_REJECT;
        digests = proof + 32;
    } else {
        if (c.len != tlookup_proof_bytes(Ds[0])) return ZK_E_REJECT;
        if (memcmp(proof, "ZKTL\x02\0\0\0", 8) != 0) return ZK_E_REJECT;
        if (get_le64(proof + 8) != Ds[0] || get_le64(proof + 16) != Ns[0]) return ZK_E_REJECT;
        digests = proof + 24;
    }
    const uint8_t* ab_digests = digests + 32 * K;  // per instance: digest(A), digest(B)
    const uint8_t* body = ab_digests + 64 * K;
    F el[4 * 32 + 5 * kMailboxMaxInstances];
    const int nel = 4 * n + 5 * (int)K;
    for (int i = 0; i < nel; ++i)
        if (!from_bytes(&el[i], body + 32 * i)) return ZK_E_REJECT;

    uint64_t dims[1 + 2 * kMailboxMaxInstances];
    int ndims;
    if (c.multi) {
        dims[0] = K;
        for (size_t i = 0; i < K; ++i) {
            dims[1 + 2 * i] = Ds[i];
            dims[2 + 2 * i] = Ns[i];
        }
        ndims = 1 + 2 * (int)K;
    } else {
        dims[0] = Ds[0];
        dims[1] = Ns[0];
        dims[2] = K;
        ndims = c.batch ? 3 : 2;
    }
    Transcript tr(c.multi ? "zkmi/tlookup-multi/v1" : c.batch ? "zkmi/tlookup-batch/v2" : "zkmi/tlookup/v2", c.seed, dims, ndims);
    for (size_t i = 0; i < K; ++i) tr.absorb("m", digests + 32 * i, 32);
    F beta = tr.challenge("beta");
    for (size_t i = 0; i < K; ++i) {
        tr.absorb("A", ab_digests + 64 * i, 32);
        tr.absorb("B", ab_digests + 64 * i + 32, 32);
    }
    F alpha = tr.challenge("alpha");
    F alpha2 = sqr(alpha);
    F u[32], v[32];
    for (int t = 0; t < n; ++t) u[t] = tr.challenge("u");
    F lambda = one();
    if (c.batch) lambda = tr.challenge("lambda");
    F lam[kMailboxMaxInstances], lam_sum = zero();
    for (size_t i = 0; i < K; ++i) {
        lam[i] = i == 0 ? one() : mul(lam[i - 1], lambda);
        lam_sum = add(lam_sum, lam[i]);
    }
    F claim = mul(lam_sum, add(alpha, alpha2));
    for (int k = 0; k < n; ++k) {
        const F* g = &el[4 * k];
        if (!equal(add(g[0], g[1]), claim)) return ZK_E_REJECT;
        tr.absorb("g", body + 128 * k, 128);
        v[k] = tr.challenge("r");
        claim = interpolate_at(g, 4, v[k]);
    }
    const F* fin = &el[4 * n];
    tr.absorb("final", body + 128 * n, 160 * K);
    const F inv2 = inv(from_u64(2));
    F total = zero();
    for (size_t i = 0; i < K; ++i) {
        const F* f = fin + 5 * i;
        const int skip = skips[i], h = hs[i];
        F scale = one(), weight = lam[i];  // 2^-h; lambda^i 2^-skip
        for (int t = 0; t < h; ++t) scale = mul(scale, inv2);
        for (int t = 0; t < skip; ++t) weight = mul(weight, inv2);
        const F e_full = eq_point(u + skip, v + skip, ns[i]), e_tab = eq_point(u + skip + h, v + skip + h, ls[i]);
        F lhs = mul(f[0], add(mul(mul(alpha, e_full), add(f[1], beta)), one()));
        F rhs = mul(scale, mul(f[2], sub(mul(mul(alpha2, e_tab), add(f[4], beta)), f[3])));
        total = add(total, mul(weight, add(lhs, rhs)));
    }
    if (!equal(total, claim)) return ZK_E_REJECT;

    // claims against tensors
    hipStream_t stream = as_stream(c.stream);
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(c.ws, c.ws_bytes);
    uint32_t* Mfr = cv.limbs(N_max);
    uint32_t* leaves = (uint32_t*)cv.take(div_up(N_max, kLeafCounts) * 32);
    uint32_t* dig_leaves = (uint32_t*)cv.take(vec_digest_leaves(D_max) * 32);
    uint32_t* dig_rows = (uint32_t*)cv.take(vec_digest_row_digests(D_max) * 32);
    uint32_t* dig_ticket = (uint32_t*)cv.take(256);
    // a witness vector must be the one whose digest the proof carries
    auto check_digest = [&](const fr_vec& vec, size_t count, const uint8_t* want, int* ok) -> int {
        const uint32_t seq = mb->next_seq();
        const VecDigestJob job{vec.limbs, vec.stride, count, dig_rows, mb->words + kMailboxDigest};
        launch_fill_u32(dig_ticket, 1, 0u, stream);
        vec_digest_launch(job, nullptr, dig_leaves, mb->words, seq, dig_ticket, stream);
        ZK_HIP_TRY(hipGetLastError());
        ZK_TRY(mailbox_wait(mb, seq, stream));
        ZK_HIP_TRY(hipStreamSynchronize(stream));
        uint8_t got[32];
        digest_bytes(got, mb->words + kMailboxDigest);
        *ok = memcmp(got, want, 32) == 0 ? 1 : 0;
        return ZK_OK;
    };
    auto check = [&](const uint32_t* a, size_t stride, int nv, const F* pt, const F& want, int* ok) -> int {
        Carver scratch = cv;
        uint32_t seq = mb->next_seq();
        ZK_TRY(mle_eval_run(a, stride, nv, pt, scratch, mb, seq, stream));
        ZK_TRY(mailbox_wait(mb, seq, stream));
        ZK_HIP_TRY(hipStreamSynchronize(stream));
        *ok = equal(from_dev(mb->words), want) ? 1 : 0;
        return ZK_OK;
    };
    for (size_t i = 0; i < K; ++i) {
        const F* f = fin + 5 * i;
        const size_t D = Ds[i], N = Ns[i];
        const int ni = ns[i], l = ls[i];
        const F* vd = v + skips[i];          // the instance's point
        const F* vt = vd + hs[i];            // its table's
        const uint32_t nleaves = (uint32_t)div_up(N, kLeafCounts);
        int ok = 0;
        ZK_TRY(check(c.T[i].limbs, c.T[i].stride, l, vt, f[4], &ok));
        if (!ok) return ZK_E_REJECT;
        if (!c.wit) continue;
        const tlookup_witness* wit = c.wit + i;
        if (wit->S.limbs) {
            if (!vec_ok(wit->S, D)) return ZK_E_BADARG;
            ZK_TRY(check(wit->S.limbs, wit->S.stride, ni, vd, f[1], &ok));
            if (!ok) return ZK_E_REJECT;
        }
        if (wit->A.limbs) {
            if (!vec_ok(wit->A, D)) return ZK_E_BADARG;
            ZK_TRY(check(wit->A.limbs, wit->A.stride, ni, vd, f[0], &ok));
            if (!ok) return ZK_E_REJECT;
            ZK_TRY(check_digest(wit->A, D, ab_digests + 64 * i, &ok));
            if (!ok) return ZK_E_REJECT;
        }
        if (wit->B.limbs) {
            if (!vec_ok(wit->B, N)) return ZK_E_BADARG;
            ZK_TRY(check(wit->B.limbs, wit->B.stride, l, vt, f[2], &ok));
            if (!ok) return ZK_E_REJECT;
            ZK_TRY(check_digest(wit->B, N, ab_digests + 64 * i + 32, &ok));
            if (!ok) return ZK_E_REJECT;
        }
        if (wit->m) {
            hipLaunchKernelGGL(k_counts_to_fr, dim3(grid_for(N)), dim3(kBlock), 0, stream, Mfr, N, wit->m, N);
            hipLaunchKernelGGL(k_leaf_digests, dim3((unsigned)div_up(nleaves, 64)), dim3(64), 0, stream, leaves, wit->m,
                               (uint32_t)N, nleaves);
            ZK_TRY(mailbox_bulk(mb, (size_t)nleaves * 32));
            ZK_HIP_TRY(hipMemcpyAsync(mb->bulk, leaves, (size_t)nleaves * 32, hipMemcpyDeviceToHost, stream));
            ZK_TRY(check(Mfr, N, l, vt, f[3], &ok));
            if (!ok) return ZK_E_REJECT;
            uint8_t md[32];
            digest_of_leaves(md, mb->bulk, nleaves);
            if (memcmp(md, digests + 32 * i, 32) != 0) return ZK_E_REJECT;
        }
    }
    if (c.claims) {
        memset(c.claims, 0, sizeof *c.claims);
        c.claims->A_v = to_canonical(fin[0]);
        c.claims->S_v = to_canonical(fin[1]);
        c.claims->B_vp = to_canonical(fin[2]);
        c.claims->m_vp = to_canonical(fin[3]);
        c.claims->T_vp = to_canonical(fin[4]);
        c.claims->nvars = n;
        for (int t = 0; t < n; ++t) c.claims->v[t] = to_canonical(v[t]);
    }
    if (c.bclaims) {
        memset(c.bclaims, 0, sizeof *c.bclaims);
        c.bclaims->nvars = n;
        c.bclaims->count = (int)K;
        c.bclaims->lambda = to_canonical(lambda);
        for (int t = 0; t < n; ++t) c.bclaims->v[t] = to_canonical(v[t]);
        for (size_t i = 0; i < K; ++i)
            for (int q = 0; q < 5; ++q) c.bclaims->value[i][q] = to_canonical(fin[5 * i + q]);
    }
    return ZK_OK;
}

}  // namespace zkmi

using namespace zkmi;

extern "C" {

size_t tlookup_proof_bytes(size_t D) { return 120 + (size_t)log2_floor(D ? D : 1) * 128 + 160; }

size_t tlookup_workspace_bytes(size_t D, size_t N) {
    if (!is_pow2(D) || !is_pow2(N) || N > D) return 0;
    return prove_ws_bytes(D, N);
}

int tlookup_multiplicities(uint32_t* m, fr_vec S, const uint32_t* idx, fr_vec T, void* ws, size_t ws_bytes,
                           uint64_t* bad_index, void* stream) {
    const size_t D = S.n, N = T.n;
    if (!m || D == 0 || N == 0 || N > ((size_t)1 << 31) || !vec_ok(S, D) || !vec_ok(T, N)) return ZK_E_BADARG;
    if (!is_pow2(D) || !is_pow2(N) || N > D) return ZK_E_BADARG;
    if (!ws || ws_bytes < prove_ws_bytes(D, N)) return ZK_E_BUFSZ;
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(ws, ws_bytes);
    ProveWs w;
    carve_prove(w, cv, D, N);
    ZK_TRY(count_rows(w, S, idx, T, D, N, bad_index, mb, as_stream(stream)));
    ZK_HIP_TRY(hipMemcpyAsync(m, w.m, N * 4, hipMemcpyDeviceToDevice, as_stream(stream)));
    ZK_HIP_TRY(hipStreamSynchronize(as_stream(stream)));
    return ZK_OK;
}

static int prove_single(const uint8_t seed[32], fr_vec S, const uint32_t* idx, fr_vec T, const fr_t* forced_beta,
                        bool by_rows, uint8_t* proof, size_t cap, size_t* len, tlookup_aux* aux, void* ws,
                        size_t ws_bytes, void* stream, bool check_upfront = false) {
    ProveCall c;
    c.check_upfront = check_upfront;
    c.seed = seed;
    c.K = 1;
    c.S = &S;
    c.idx = &idx;
    c.T = &T;
    c.forced_beta = forced_beta;
    c.by_rows = by_rows;
    c.proof = proof;
    c.cap = cap;
    c.len = len;
    c.aux = aux;
    c.ws = ws;
    c.ws_bytes = ws_bytes;
    c.stream = stream;
    return prove_core(c);
}

int tlookup_prove(const uint8_t seed[32], fr_vec S, const uint32_t* idx, fr_vec T, uint8_t* proof, size_t cap,
                  size_t* len, tlookup_aux* aux, void* ws, size_t ws_bytes, void* stream) {
    return prove_single(seed, S, idx, T, nullptr, false, proof, cap, len, aux, ws, ws_bytes, stream);
}

static __global__ void __launch_bounds__(kBlock) k_small_materialize(uint32_t* __restrict__ dst, size_t ds, size_t n,
                                                                     SmallSource ints) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        Fr v;
        small_source_load(v.l, ints, i);
        fr_store(dst, ds, i, v);
    }
}

size_t tlookup_small_workspace_bytes(size_t D, size_t N) {
    if (!is_pow2(D) || !is_pow2(N) || N > D) return 0;
    size_t base = align_up(prove_ws_bytes(D, N), 256);
    return small_source_shape_ok(D, N) ? base : base + D * 32;  // other shapes: S is written out as field elements first
}

int tlookup_prove_small(const uint8_t seed[32], const int32_t* X, const int32_t* Y, const fr_t* rho, size_t D,
                        const uint32_t* idx, fr_vec T, uint8_t* proof, size_t cap, size_t* len, tlookup_aux* aux, void* ws,
                        size_t ws_bytes, void* stream) {
    using namespace host;
    const size_t N = T.n;
    if (!seed || !X || !idx || (Y != nullptr) != (rho != nullptr)) return ZK_E_BADARG;
    if (!is_pow2(D) || !is_pow2(N) || N > D || D > ((size_t)1 << 31) || !vec_ok(T, N)) return ZK_E_BADARG;
    if (rho && !canonical_in_range(*rho)) return ZK_E_BADARG;
    if (len) *len = tlookup_proof_bytes(D);
    if (!ws || ws_bytes < tlookup_small_workspace_bytes(D, N)) return ZK_E_BUFSZ;
    if (small_source_shape_ok(D, N)) {
        ProveCall c;
        c.seed = seed;
        c.K = 1;
        c.idx = &idx;
        c.T = &T;
        c.ints_x = X;
        c.ints_y = Y;
        c.ints_rho = rho;
        c.ints_D = D;
        c.proof = proof;
        c.cap = cap;
        c.len = len;
        c.aux = aux;
        c.ws = ws;
        c.ws_bytes = ws_bytes;
        c.stream = stream;
        return prove_core(c);
    }
    // a shape whose first fold is not a kernel of its own: the tensor as field elements, then the usual path
    const size_t base = align_up(prove_ws_bytes(D, N), 256);
    SmallSource src;
    memset(&src, 0, sizeof src);
    const F two64 = mul(from_u64((uint64_t)1 << 32), from_u64((uint64_t)1 << 32));
    const F r = rho ? from_canonical(*rho) : zero();
    src.x = X;
    src.y = Y;
    to_device_limbs(src.plus_one, two64);
    to_device_limbs(src.minus_one, neg(two64));
    to_device_limbs(src.plus_rho, mul(r, two64));
    to_device_limbs(src.minus_rho, neg(mul(r, two64)));
    fr_vec S = {(uint32_t*)((uint8_t*)ws + base), D, D};
    hipLaunchKernelGGL(k_small_materialize, dim3(grid_for(D, kBlock, 16384)), dim3(kBlock), 0, as_stream(stream), S.limbs,
                       S.stride, D, src);
    ZK_HIP_TRY(hipGetLastError());
    return prove_single(seed, S, idx, T, nullptr, false, proof, cap, len, aux, ws, base, stream);
}

// The per-round plan of a proof of this shape, walked on the host (no GPU is
// touched): four integers per round -- kernel, source of S, arrays arrive as
// 32-bit words, arrays leave as 32-bit words.
int zkmi_selftest_tlookup_plan(size_t D, size_t N, size_t K, int from_ints, int32_t* out, size_t cap_rounds) {
    if (!out || !is_pow2(D) || !is_pow2(N) || N > D || D > ((size_t)1 << 31) || K == 0 || K > kMailboxMaxInstances) return ZK_E_BADARG;
    const int n = log2_floor(D), h = n - log2_floor(N);
    if ((size_t)n > cap_rounds) return ZK_E_BUFSZ;
    if (from_ints && (K != 1 || !small_source_shape_ok(D, N))) return ZK_E_BADARG;
    int lazy = 0;
    bool resident = false;
    for (int k = 0; k < n; ++k) {
        const RoundPlan pl = plan_round(n, h, k, K, from_ints != 0, lazy, resident);
        out[4 * k] = pl.kernel;
        out[4 * k + 1] = pl.s_source;
        out[4 * k + 2] = pl.in32 ? 1 : 0;
        out[4 * k + 3] = pl.out32 ? 1 : 0;
        lazy = pl.lazy_after;
        resident = resident || pl.kernel == kRoundResident;
    }
    return n;
}

// The host's rounds (HostTail) on arrays and challenges of the caller's choosing: no GPU is touched.
int zkmi_selftest_host_rounds(const fr_t* A, const fr_t* S, const fr_t* B, const fr_t* M, const fr_t* T, size_t n_data,
                              size_t n_table, const fr_t* u_rest, const fr_t* beta, const fr_t* challenges, fr_t* sums,
                              fr_t* finals) {
    using namespace host;
    if (!A || !S || !B || !M || !T || !beta || !sums || !finals) return ZK_E_BADARG;
    if (!is_pow2(n_data) || !is_pow2(n_table) || n_data < 2 || n_data > kMailboxShipEntries || n_table > n_data) return ZK_E_BADARG;
    const int d = log2_floor(n_data);
    if (d > 1 && !u_rest) return ZK_E_BADARG;
    if (!challenges) return ZK_E_BADARG;
    for (int t = 0; t < d - 1; ++t)
        if (!canonical_in_range(u_rest[t])) return ZK_E_BADARG;
    for (int t = 0; t < d; ++t)
        if (!canonical_in_range(challenges[t])) return ZK_E_BADARG;
    if (!canonical_in_range(*beta)) return ZK_E_BADARG;
    HostTail ht;
    const fr_t* const src[5] = {A, S, B, M, T};
    F* const dst[5] = {ht.A, ht.S, ht.B, ht.M, ht.T};
    for (int q = 0; q < 5; ++q)
        for (size_t j = 0; j < (q < 2 ? n_data : n_table); ++j) {
            if (!canonical_in_range(src[q][j])) return ZK_E_BADARG;
            dst[q][j] = from_canonical(src[q][j]);
        }
    F us[8];
    for (int t = 0; t < d - 1; ++t) us[t] = from_canonical(u_rest[t]);
    ht.weights(us, d - 1);
    const F b = from_canonical(*beta);
    int round = 0;
    for (size_t half = n_data / 2; half >= 1; half >>= 1, ++round) {
        const bool table_round = 2 * half <= n_table;
        F out[11];
        ht.sums(half, table_round, b, out);
        for (int q = 0; q < 11; ++q) sums[11 * round + q] = to_canonical(out[q]);
        ht.fold(half, table_round, from_canonical(challenges[round]));
    }
    for (int q = 0; q < 5; ++q) finals[q] = to_canonical(dst[q][0]);
    return d;
}

int tlookup_prove_checked(const uint8_t seed[32], fr_vec S, const uint32_t* idx, fr_vec T, uint8_t* proof, size_t cap,
                          size_t* len, tlookup_aux* aux, void* ws, size_t ws_bytes, void* stream) {
    return prove_single(seed, S, idx, T, nullptr, false, proof, cap, len, aux, ws, ws_bytes, stream, true);
}

int tlookup_prove_by_rows(const uint8_t seed[32], fr_vec S, const uint32_t* idx, fr_vec T, uint8_t* proof, size_t cap,
                          size_t* len, tlookup_aux* aux, void* ws, size_t ws_bytes, void* stream) {
    if (!idx) return ZK_E_BADARG;
    return prove_single(seed, S, idx, T, nullptr, true, proof, cap, len, aux, ws, ws_bytes, stream);
}

int tlookup_prove_with_beta(const uint8_t seed[32], fr_vec S, const uint32_t* idx, fr_vec T, const fr_t* forced_beta,
                            uint8_t* proof, size_t cap, size_t* len, tlookup_aux* aux, void* ws, size_t ws_bytes,
                            void* stream) {
    if (!forced_beta) return ZK_E_BADARG;
    return prove_single(seed, S, idx, T, forced_beta, false, proof, cap, len, aux, ws, ws_bytes, stream);
}

size_t tlookup_verify_workspace_bytes(size_t D, size_t N) {
    if (!is_pow2(D) || !is_pow2(N) || N > D) return 0;
    return verify_ws_bytes(D, N);
}

int tlookup_verify(const uint8_t seed[32], const uint8_t* proof, size_t len, fr_vec T, size_t D,
                   const tlookup_witness* witness, tlookup_claims* claims, void* ws, size_t ws_bytes, void* stream) {
    VerifyCall c;
    c.seed = seed;
    c.proof = proof;
    c.len = len;
    c.K = 1;
    c.T = &T;
    c.D = D;
    c.wit = witness;
    c.claims = claims;
    c.ws = ws;
    c.ws_bytes = ws_bytes;
    c.stream = stream;
    return verify_core(c);
}

size_t tlookup_batch_proof_bytes(size_t D, size_t K) { return batch_proof_bytes(D, K); }

size_t tlookup_batch_workspace_bytes(size_t D, size_t N, size_t K) {
    if (!is_pow2(D) || !is_pow2(N) || N > D || K == 0 || K > TLOOKUP_BATCH_MAX) return 0;
    return prove_ws_bytes(D, N, K);
}

int tlookup_prove_batch(const uint8_t seed[32], const fr_vec* S, const uint32_t* const* idx, const fr_vec* T, size_t K,
                        uint8_t* proof, size_t cap, size_t* len, tlookup_batch_aux* aux, void* ws, size_t ws_bytes,
                        void* stream) {
    ProveCall c;
    c.seed = seed;
    c.K = K;
    c.S = S;
    c.idx = idx;
    c.T = T;
    c.batch = true;
    c.proof = proof;
    c.cap = cap;
    c.len = len;
    c.baux = aux;
    c.ws = ws;
    c.ws_bytes = ws_bytes;
    c.stream = stream;
    return prove_core(c);
}

int tlookup_verify_batch(const uint8_t seed[32], const uint8_t* proof, size_t len, const fr_vec* T, size_t K, size_t D,
                         const tlookup_witness* witness, tlookup_batch_claims* claims, void* ws, size_t ws_bytes,
                         void* stream) {
    VerifyCall c;
    c.seed = seed;
    c.proof = proof;
    c.len = len;
    c.K = K;
    c.T = T;
    c.D = D;
    c.batch = true;
    c.wit = witness;
    c.bclaims = claims;
    c.ws = ws;
    c.ws_bytes = ws_bytes;
    c.stream = stream;
    return verify_core(c);
}

static bool multi_shapes_ok(const size_t* D, const size_t* N, size_t K) {
    if (!D || !N || K == 0 || K > TLOOKUP_BATCH_MAX) return false;
    for (size_t i = 0; i < K; ++i)
        if (!is_pow2(D[i]) || !is_pow2(N[i]) || N[i] > D[i] || D[i] > ((size_t)1 << 31)) return false;
    return true;
}

size_t tlookup_multi_proof_bytes(const size_t* D, size_t K) {
    if (!D || K == 0 || K > TLOOKUP_BATCH_MAX) return 0;
    int n = 0;
    for (size_t i = 0; i < K; ++i) {
        if (!is_pow2(D[i])) return 0;
        if (log2_floor(D[i]) > n) n = log2_floor(D[i]);
    }
    return multi_proof_bytes(n, K);
}

size_t tlookup_multi_workspace_bytes(const size_t* D, const size_t* N, size_t K) {
    if (!multi_shapes_ok(D, N, K)) return 0;
    return prove_ws_bytes_shapes(D, N, K);
}

int tlookup_prove_multi(const uint8_t seed[32], const fr_vec* S, const uint32_t* const* idx, const fr_vec* T, size_t K,
                        uint8_t* proof, size_t cap, size_t* len, tlookup_batch_aux* aux, void* ws, size_t ws_bytes,
                        void* stream) {
    ProveCall c;
    c.seed = seed;
    c.K = K;
    c.S = S;
    c.idx = idx;
    c.T = T;
    c.batch = true;
    c.multi = true;
    c.proof = proof;
    c.cap = cap;
    c.len = len;
    c.baux = aux;
    c.ws = ws;
    c.ws_bytes = ws_bytes;
    c.stream = stream;
    return prove_core(c);
}

size_t tlookup_multi_verify_workspace_bytes(const size_t* D, const size_t* N, size_t K) {
    if (!multi_shapes_ok(D, N, K)) return 0;
    size_t D_max = 1, N_max = 1;
    for (size_t i = 0; i < K; ++i) {
        if (D[i] > D_max) D_max = D[i];
        if (N[i] > N_max) N_max = N[i];
    }
    return verify_ws_bytes(D_max, N_max);
}

int tlookup_verify_multi(const uint8_t seed[32], const uint8_t* proof, size_t len, const fr_vec* T, const size_t* D,
                         size_t K, const tlookup_witness* witness, tlookup_batch_claims* claims, void* ws,
                         size_t ws_bytes, void* stream) {
    VerifyCall c;
    c.seed = seed;
    c.proof = proof;
    c.len = len;
    c.K = K;
    c.T = T;
    c.Ds = D;
    c.batch = true;
    c.multi = true;
    c.wit = witness;
    c.bclaims = claims;
    c.ws = ws;
    c.ws_bytes = ws_bytes;
    c.stream = stream;
    return verify_core(c);
}

}  // extern "C"
