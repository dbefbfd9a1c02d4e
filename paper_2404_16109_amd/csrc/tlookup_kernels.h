// Kernels of the tlookup prover (Section 4 of the paper, Protocol 1): table
// hashing and multiplicity counting, the leaf digests of m, pooled eq tables,
// and the sumcheck round kernels for the data side (A, S) and the table side
// (B, T, m) of the tlookup identity.
#pragma once
#include "common.h"
#include "reduce_dev.h"
#include "fr29_dev.h"
#include "sha256_dev.h"
#include "small_dev.h"

namespace zkmi {

// ---- table rows by value: open-addressing hash of T -----------------------------

static const uint32_t kEmptySlot = 0xffffffffu;

__device__ __forceinline__ uint32_t fr_hash(const Fr& a) {
    uint32_t h = a.l[0] * 0x9e3779b1u;
    h = (h ^ a.l[1]) * 0x85ebca77u;
    h = (h ^ a.l[2]) * 0xc2b2ae3du;
    h = (h ^ a.l[3]) * 0x27d4eb2fu;
    h = (h ^ a.l[4]) * 0x165667b1u;
    h = (h ^ a.l[5]) * 0x9e3779b1u;
    h = (h ^ a.l[6]) * 0x85ebca77u;
    h = (h ^ a.l[7]) * 0xc2b2ae3du;
    return h ^ (h >> 15);
}

// Every row j claims the first slot of its probe sequence that is empty or holds
// a row with the same value; equal values meet in one slot and the lowest row
// wins.  Slots never empty again and the value class of a slot never changes, so
// all rows of one value walk the same sequence to the same slot.
static __global__ void __launch_bounds__(kBlock) k_hash_build(uint32_t* slots, uint32_t cap_mask,
                                                       const uint32_t* __restrict__ T, size_t ts, uint32_t N,
                                                       uint32_t* dup_flag) {
    for (uint32_t j = blockIdx.x * kBlock + threadIdx.x; j < N; j += gridDim.x * kBlock) {
        Fr v = fr_load(T, ts, j);
        uint32_t pos = fr_hash(v) & cap_mask;
        for (uint32_t step = 0; step <= cap_mask; ++step) {
            uint32_t cur = atomicCAS(&slots[pos], kEmptySlot, j);
            if (cur == kEmptySlot) break;  // claimed
            if (fr_equal(fr_load(T, ts, cur), v)) {
                atomicMin(&slots[pos], j);
                atomicOr(dup_flag, 1u);
                break;
            }
            pos = (pos + 1) & cap_mask;
        }
    }
}

// Row of the table holding value v (lowest row of equal ones), or kEmptySlot.
__device__ __forceinline__ uint32_t hash_find(const uint32_t* __restrict__ slots, uint32_t cap_mask,
                                              const uint32_t* __restrict__ T, size_t ts, const Fr& v) {
    uint32_t pos = fr_hash(v) & cap_mask;
    for (uint32_t step = 0; step <= cap_mask; ++step) {
        uint32_t cur = slots[pos];
        if (cur == kEmptySlot) return kEmptySlot;
        if (fr_equal(fr_load(T, ts, cur), v)) return cur;
        pos = (pos + 1) & cap_mask;
    }
    return kEmptySlot;
}

// The same through the row-major copy of the table (k_canon_rows): a candidate row
// is one 32-byte access instead of eight words from eight limb planes.
__device__ __forceinline__ uint32_t hash_find_rows(const uint32_t* __restrict__ slots, uint32_t cap_mask,
                                                   const uint4* __restrict__ rows, const Fr& v) {
    uint32_t pos = fr_hash(v) & cap_mask;
    for (uint32_t step = 0; step <= cap_mask; ++step) {
        uint32_t cur = slots[pos];
        if (cur == kEmptySlot) return kEmptySlot;
        const uint4 lo = rows[2 * (size_t)cur], hi = rows[2 * (size_t)cur + 1];
        const uint32_t diff = (lo.x ^ v.l[0]) | (lo.y ^ v.l[1]) | (lo.z ^ v.l[2]) | (lo.w ^ v.l[3]) |
                              (hi.x ^ v.l[4]) | (hi.y ^ v.l[5]) | (hi.z ^ v.l[6]) | (hi.w ^ v.l[7]);
        if (diff == 0) return cur;
        pos = (pos + 1) & cap_mask;
    }
    return kEmptySlot;
}

// canon[j] = lowest row with the value of row j; rows[j] = row j of T as eight
// consecutive words, so that a lookup by row number is one 32-byte access
// instead of eight accesses to eight limb planes.
static __global__ void __launch_bounds__(kBlock) k_canon_rows(uint32_t* __restrict__ canon, uint4* __restrict__ rows,
                                                       const uint32_t* __restrict__ slots, uint32_t cap_mask,
                                                       const uint32_t* __restrict__ T, size_t ts, uint32_t N) {
    for (uint32_t j = blockIdx.x * kBlock + threadIdx.x; j < N; j += gridDim.x * kBlock) {
        Fr v = fr_load(T, ts, j);
        canon[j] = hash_find(slots, cap_mask, T, ts, v);
        rows[2 * j] = make_uint4(v.l[0], v.l[1], v.l[2], v.l[3]);
        rows[2 * j + 1] = make_uint4(v.l[4], v.l[5], v.l[6], v.l[7]);
    }
}

// A wavefront's running total for the row it keeps meeting (wave-uniform).
// Long runs of one row (padding, saturated activations) would otherwise become
// a stream of atomics to a single address, which the memory system serialises.
struct HotRun {
    uint32_t row = kEmptySlot;
    uint32_t count = 0;
    __device__ __forceinline__ void add(uint32_t* m, uint32_t r, uint32_t c) {
        if (r == row) {
            count += c;
        } else {
            flush(m);
            row = r;
            count = c;
        }
    }
    __device__ __forceinline__ void flush(uint32_t* m) {
        if (count && (threadIdx.x & 63) == 0) atomicAdd(&m[row], count);
        count = 0;
    }
};

// Adds one to m[row] for every active lane with a valid row.  Lanes of a
// wavefront that hit the same row are merged first: a few rounds of "take the
// first pending lane's row, count the lanes that share it", runs of half a
// wavefront or more going to the wavefront's running total and shorter ones to
// one atomic each, then plain atomics for whatever rows are left.
__device__ __forceinline__ void count_merged(uint32_t* m, uint32_t row, bool valid, HotRun& hot) {
    bool pending = valid;
#pragma unroll 1
    for (int round = 0; round < 8; ++round) {
        unsigned long long todo = __ballot(pending);
        if (todo == 0) return;
        int leader = __ffsll((long long)todo) - 1;
        uint32_t lead_row = (uint32_t)__builtin_amdgcn_readlane((int)row, leader);  // leader is wave-uniform: no trip through LDS
        bool mine = pending && row == lead_row;
        uint32_t run = (uint32_t)__popcll(__ballot(mine));
        if (run >= 32) hot.add(m, lead_row, run);
        else if ((int)(threadIdx.x & 63) == leader) atomicAdd(&m[lead_row], run);
        pending = pending && !mine;
    }
    if (pending) atomicAdd(&m[row], 1u);
}

// m[row(S_i)] += 1.  With idx the row is given and only checked; without, it is
// found through the hash.  The smallest offending i ends up in *bad.
static __global__ void __launch_bounds__(kBlock) k_count(uint32_t* m, const uint32_t* __restrict__ S, size_t ss, size_t D,
                                                  const uint32_t* __restrict__ idx, const uint32_t* __restrict__ T,
                                                  size_t ts, const uint4* __restrict__ rows, uint32_t N,
                                                  const uint32_t* __restrict__ slots,
                                                  uint32_t cap_mask, const uint32_t* __restrict__ canon,
                                                  const uint32_t* __restrict__ dup_flag, unsigned long long* bad) {
    const bool dups = *dup_flag != 0;
    // every lane of a wavefront runs the same number of iterations, so the
    // cross-lane steps in count_merged see whole wavefronts
    const size_t per_pass = (size_t)gridDim.x * kBlock;
    const size_t passes = (D + per_pass - 1) / per_pass;
    HotRun hot;
    for (size_t pass = 0; pass < passes; ++pass) {
        size_t i = pass * per_pass + blockIdx.x * (size_t)kBlock + threadIdx.x;
        bool in_range = i < D;
        uint32_t row = kEmptySlot;
        if (in_range) {
            Fr v = fr_load(S, ss, i);
            if (idx) {
                row = idx[i];
                if (row < N) {
                    uint4 lo = rows[2 * (size_t)row], hi = rows[2 * (size_t)row + 1];
                    uint32_t diff = (lo.x ^ v.l[0]) | (lo.y ^ v.l[1]) | (lo.z ^ v.l[2]) | (lo.w ^ v.l[3]) |
                                    (hi.x ^ v.l[4]) | (hi.y ^ v.l[5]) | (hi.z ^ v.l[6]) | (hi.w ^ v.l[7]);
                    if (diff) row = kEmptySlot;
                    else if (dups) row = canon[row];
                } else {
                    row = kEmptySlot;
                }
            } else {
                row = hash_find_rows(slots, cap_mask, rows, v);
            }
            if (row == kEmptySlot) atomicMin(bad, (unsigned long long)i);
        }
        count_merged(m, row, in_range && row != kEmptySlot, hot);
    }
    hot.flush(m);
}

// ---- multiplicities through workgroup-private histograms in LDS ---------------------
//
// For tables of up to 2^16 rows the counters of a workgroup fit in LDS as packed
// 16-bit pairs (128 KiB at 2^16 rows, of the 160 KiB a gfx950 compute unit has),
// which takes the counting off the device-wide atomics.  A workgroup walks its
// share of S in passes (chunks of at most kHistPass elements, handed out round
// robin) short enough that no 16-bit counter can overflow, and
// after each pass adds its counters into a 32-bit histogram of its own in HBM
// (plain loads and stores, nobody else touches it); a second kernel adds the
// workgroups' histograms up.  Runs of one row that fill half a wavefront or more
// (padding, saturated activations) are kept in a per-wavefront running total and
// go straight to the result, so they do not eat into the 16-bit budget.
static const int kHistThreads = 1024;
static const uint32_t kHistPass = 60 * 1024;  // elements per pass, < 2^16

// CHECK_S = false: rows are taken from the hints unchecked (an out-of-range hint
// still counts as a failure); the comparison of every S_i with its row is then
// the caller's business (it rides on the inversion's first pass over S).
template <bool CHECK_S>
static __global__ void __launch_bounds__(kHistThreads)
k_count_lds(uint32_t* m, uint32_t* __restrict__ part, const uint32_t* __restrict__ S, size_t ss, size_t D,
            size_t chunk, const uint32_t* __restrict__ idx, const uint32_t* __restrict__ T, size_t ts,
            const uint4* __restrict__ rows, uint32_t N, const uint32_t* __restrict__ slots, uint32_t cap_mask,
            const uint32_t* __restrict__ canon, const uint32_t* __restrict__ dup_flag, unsigned long long* bad) {
    extern __shared__ uint32_t hist[];  // (N+1)/2 words, two 16-bit counters each
    const uint32_t words = (N + 1) / 2;
    const bool dups = *dup_flag != 0;
    uint32_t* mine_part = part + (size_t)blockIdx.x * N;
    bool first = true;
    HotRun hot;
    // pass p of this workgroup covers chunk p * gridDim.x + blockIdx.x of S: stretches
    // that are cheap to count (padding) are spread over all workgroups that way
    for (size_t pass_begin = blockIdx.x * chunk; pass_begin < D || first; pass_begin += (size_t)gridDim.x * chunk) {
        for (uint32_t w = threadIdx.x; w < words; w += kHistThreads) hist[w] = 0;
        __syncthreads();
        const size_t pass_end = pass_begin + chunk < D ? pass_begin + chunk : D;
        // whole wavefronts iterate together so that the cross-lane merge sees all 64
        // lanes; several elements per thread per trip keep more loads in flight
        // (four when S is read as well, eight when only the hints are)
        constexpr int E = 8;
        for (size_t base = pass_begin; base < pass_end; base += E * kHistThreads) {
            size_t i[E];
            bool in_range[E];
            uint32_t row[E];
            Fr v[CHECK_S ? E : 1];
#pragma unroll
            for (int e = 0; e < E; ++e) {
                i[e] = base + (size_t)e * kHistThreads + threadIdx.x;
                in_range[e] = i[e] < pass_end;
                row[e] = kEmptySlot;
                if (in_range[e]) {
                    if (idx) row[e] = idx[i[e]];
                    if constexpr (CHECK_S) v[e] = fr_load(S, ss, i[e]);
                }
            }
#pragma unroll
            for (int e = 0; e < E; ++e) {
                if (!in_range[e]) continue;
                if (idx) {
                    uint32_t r = row[e];
                    if (r < N) {
                        uint32_t diff = 0;
                        if constexpr (CHECK_S) {
                            uint4 lo = rows[2 * (size_t)r], hi = rows[2 * (size_t)r + 1];
                            diff = (lo.x ^ v[e].l[0]) | (lo.y ^ v[e].l[1]) | (lo.z ^ v[e].l[2]) | (lo.w ^ v[e].l[3]) |
                                   (hi.x ^ v[e].l[4]) | (hi.y ^ v[e].l[5]) | (hi.z ^ v[e].l[6]) | (hi.w ^ v[e].l[7]);
                        }
                        if (diff) r = kEmptySlot;
                        else if (dups) r = canon[r];
                    } else {
                        r = kEmptySlot;
                    }
                    row[e] = r;
                } else {
                    if constexpr (CHECK_S) row[e] = hash_find_rows(slots, cap_mask, rows, v[e]);
                }
                // without the comparison a hint out of range is left for the caller's check to report
                if (CHECK_S && row[e] == kEmptySlot) atomicMin(bad, (unsigned long long)i[e]);
            }
#pragma unroll
            for (int e = 0; e < E; ++e) {
                bool pending = in_range[e] && row[e] != kEmptySlot;
#pragma unroll 1
                for (int round = 0; round < 4; ++round) {
                    unsigned long long todo = __ballot(pending);
                    if (todo == 0) break;
                    int leader = __ffsll((long long)todo) - 1;
                    uint32_t lead_row = (uint32_t)__builtin_amdgcn_readlane((int)row[e], leader);  // wave-uniform lane: no trip through LDS
                    bool same_row = pending && row[e] == lead_row;
                    uint32_t run = (uint32_t)__popcll(__ballot(same_row));
                    // A long run goes to the wavefront's running total and a run of a few
                    // lanes is added once by its first lane (lanes on one address are
                    // served one after the other).  A run of one to three lanes says that
                    // the wavefront's rows are mostly different: the remaining lanes then
                    // go in one instruction, because the LDS pipeline, which every
                    // instruction occupies for about as long whatever it carries, is what
                    // bounds this kernel.
                    if (run >= 32) hot.add(m, lead_row, run);
                    else if (run < 4) break;
                    else if ((int)(threadIdx.x & 63) == leader)
                        atomicAdd(&hist[lead_row >> 1], run << (16 * (lead_row & 1)));
                    pending = pending && !same_row;
                }
                if (pending) atomicAdd(&hist[row[e] >> 1], 1u << (16 * (row[e] & 1)));
            }
        }
        __syncthreads();
        // Flush into this workgroup's 32-bit histogram, eight words per thread at a
        // time so that the loads of a group are in flight together (one word after
        // the other this flush cost more than the counting).
        if ((N & 1u) == 0) {
            uint2* mine2 = reinterpret_cast<uint2*>(mine_part);
            for (uint32_t w0 = threadIdx.x; w0 < words; w0 += 8 * kHistThreads) {
                uint32_t v[8];
                uint2 old[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const uint32_t w = w0 + k * kHistThreads;
                    v[k] = w < words ? hist[w] : 0;
                    old[k] = make_uint2(0, 0);
                    if (!first && v[k]) old[k] = mine2[w];
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const uint32_t w = w0 + k * kHistThreads;
                    if (w < words && (first || v[k])) mine2[w] = make_uint2(old[k].x + (v[k] & 0xffffu), old[k].y + (v[k] >> 16));
                }
            }
        } else {  // a table of one row
            for (uint32_t w = threadIdx.x; w < words; w += kHistThreads) {
                uint32_t v = hist[w];
                uint32_t c0 = v & 0xffffu, c1 = v >> 16;
                if (first) {
                    mine_part[2 * w] = c0;
                    if (2 * w + 1 < N) mine_part[2 * w + 1] = c1;
                } else if (v) {
                    mine_part[2 * w] += c0;
                    if (2 * w + 1 < N) mine_part[2 * w + 1] += c1;
                }
            }
        }
        __syncthreads();
        first = false;
    }
    hot.flush(m);
}

// m[j] += sum over workgroups of their histograms; blockIdx.y selects a group of
// `group` histograms, so that the additions of one row are spread over several
// threads.
static __global__ void __launch_bounds__(kBlock) k_hist_reduce(uint32_t* __restrict__ m, const uint32_t* __restrict__ part,
                                                        uint32_t nparts, uint32_t group, uint32_t N) {
    uint32_t j = blockIdx.x * kBlock + threadIdx.x;
    if (j >= N) return;
    uint32_t b0 = blockIdx.y * group, b1 = b0 + group < nparts ? b0 + group : nparts;
    uint32_t acc = 0;
    for (uint32_t b = b0; b < b1; ++b) acc += part[(size_t)b * N + j];
    if (acc) atomicAdd(&m[j], acc);
}

// Smallest index i whose S_i is not row idx_i of the table (or whose hint is out
// of range) into *bad.  Only runs after the prover's sums have shown that there
// is such an index.
static __global__ void __launch_bounds__(kBlock) k_check_rows(const uint32_t* __restrict__ S, size_t ss, size_t D,
                                                       const uint32_t* __restrict__ idx, const uint4* __restrict__ rows,
                                                       uint32_t N, unsigned long long* bad, SmallSource ints) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < D; i += (size_t)gridDim.x * kBlock) {
        const uint32_t r = idx[i];
        bool ok = r < N;
        if (ok) {
            Fr x;
            if (ints.x) small_source_load(x.l, ints, i);
            else x = fr_load(S, ss, i);
            const uint4 lo = rows[2 * (size_t)r], hi = rows[2 * (size_t)r + 1];
            ok = ((lo.x ^ x.l[0]) | (lo.y ^ x.l[1]) | (lo.z ^ x.l[2]) | (lo.w ^ x.l[3]) | (hi.x ^ x.l[4]) | (hi.y ^ x.l[5]) |
                  (hi.z ^ x.l[6]) | (hi.w ^ x.l[7])) == 0;
        }
        if (!ok) atomicMin(bad, (unsigned long long)i);
    }
}

// A_i = B[row_i]: with the row of every S_i known and checked, 1/(beta + S_i) is
// the table-side inverse of that row.  B is read row-major (one 32-byte access per
// element) from a copy written by k_rows_of.
static __global__ void __launch_bounds__(kBlock) k_rows_of(uint4* __restrict__ rows, const uint32_t* __restrict__ B,
                                                    size_t bs, uint32_t N) {
    for (uint32_t j = blockIdx.x * kBlock + threadIdx.x; j < N; j += gridDim.x * kBlock) {
        Fr v = fr_load(B, bs, j);
        rows[2 * j] = make_uint4(v.l[0], v.l[1], v.l[2], v.l[3]);
        rows[2 * j + 1] = make_uint4(v.l[4], v.l[5], v.l[6], v.l[7]);
    }
}

static __global__ void __launch_bounds__(kBlock) k_gather_rows(uint32_t* __restrict__ A, size_t as, size_t D,
                                                        const uint32_t* __restrict__ idx,
                                                        const uint4* __restrict__ rows) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < D; i += (size_t)gridDim.x * kBlock) {
        size_t r = idx[i];
        uint4 lo = rows[2 * r], hi = rows[2 * r + 1];
        Fr v = Fr{{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w}};
        fr_store(A, as, i, v);
    }
}

static __global__ void __launch_bounds__(kBlock) k_fill_u32(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) p[i] = v;
}

// What counting starts from, in one launch: empty hash slots, zero counts, and the
// four flag words (duplicate flag and ticket zero, smallest bad index all ones).
static __global__ void __launch_bounds__(kBlock) k_count_init(uint32_t* __restrict__ slots, size_t cap,
                                                       uint32_t* __restrict__ m, size_t N, uint32_t* __restrict__ flags) {
    const size_t total = cap + N + 4;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < total; i += (size_t)gridDim.x * kBlock) {
        if (i < cap) slots[i] = kEmptySlot;
        else if (i < cap + N) m[i - cap] = 0;
        else flags[i - cap - N] = i - cap - N < 2 ? 0u : 0xffffffffu;
    }
}

static __global__ void __launch_bounds__(kBlock) k_counts_to_fr(uint32_t* __restrict__ dst, size_t ds,
                                                         const uint32_t* __restrict__ m, size_t N) {
    for (size_t j = blockIdx.x * (size_t)kBlock + threadIdx.x; j < N; j += (size_t)gridDim.x * kBlock)
        fr_store(dst, ds, j, fr_from_u32(m[j]));
}

// ---- SHA-256 of the leaves of m ---------------------------------------------------

static const uint32_t kLeafCounts = 128;

// One thread per leaf: SHA-256 of up to 128 counts as 4-byte little-endian
// words.  Digest bytes go out in order, 32 per leaf.
static __global__ void __launch_bounds__(64) k_leaf_digests(uint32_t* __restrict__ out, const uint32_t* __restrict__ m,
                                                     uint32_t N, uint32_t nleaves) {
    uint32_t leaf = blockIdx.x * 64 + threadIdx.x;
    if (leaf >= nleaves) return;
    uint32_t base = leaf * kLeafCounts;
    uint32_t cnt = N - base < kLeafCounts ? N - base : kLeafCounts;
    uint32_t nblk = (cnt + 3 + 15) / 16;
    uint32_t h[8];
    sha256_init(h);
    for (uint32_t b = 0; b < nblk; ++b) {
        uint32_t w[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            uint32_t pos = b * 16 + i;
            uint32_t v = 0;
            if (pos < cnt) v = __builtin_bswap32(m[base + pos]);
            else if (pos == cnt) v = 0x80000000u;
            else if (pos == nblk * 16 - 1) v = cnt * 32;  // message length in bits
            w[i] = v;
        }
        sha256_compress(h, w);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) out[leaf * 8 + i] = __builtin_bswap32(h[i]);
}

// ---- digest of a vector of field elements (stand-in for its commitment) ----------
//
// A hash tree over the canonical bytes of the elements: with L = max(1, n/128)
// leaves, leaf i is the SHA-256 of elements i, i+L, i+2L, ... (so that lane i of a
// wavefront reads element i + tL in step t: one limb plane of 64 consecutive
// elements is 256 contiguous bytes); rows of digests are then hashed in
// consecutive fours (a last pair in twos) down to one.  Digests travel between
// the kernels as the eight state words of the hash (big-endian words of the
// digest's bytes).
static const uint32_t kVecLeaf = 128;

// Up to two vectors are hashed by one launch (the table-side vector's few leaves
// are chains of 65 dependent blocks: next to the tensor-side vector's they cost
// nothing, on their own a quarter of a millisecond).
struct VecLeavesJob {
    const uint32_t* v;
    size_t stride, n, L;  // L = 0: no such vector
    uint32_t* out;        // L digests
};

static __global__ void __launch_bounds__(kBlock) k_vec_leaves(VecLeavesJob first, VecLeavesJob second) {
    size_t leaf = blockIdx.x * (size_t)kBlock + threadIdx.x;
    const bool in_first = leaf < first.L;
    const VecLeavesJob& job = in_first ? first : second;
    if (!in_first) leaf -= first.L;
    if (leaf >= job.L) return;
    const uint32_t* v = job.v;
    const size_t stride = job.stride, L = job.L;
    const size_t cnt = job.n / L;  // elements per leaf: kVecLeaf, or all n (a power of two) when n < kVecLeaf
    uint32_t h[8];
    sha256_init(h);
    // the next two elements are asked for before the current two are hashed: one block is some 1400 instructions
    // during which their loads can be on the way
    Fr next_a = fr_zero(), next_b = fr_zero();
    if (cnt >= 2) {
        next_a = fr_load(v, stride, leaf);
        next_b = fr_load(v, stride, leaf + L);
    }
    for (size_t t = 0; t + 1 < cnt; t += 2) {
        const Fr raw_a = next_a, raw_b = next_b;
        if (t + 3 < cnt) {
            next_a = fr_load(v, stride, leaf + (t + 2) * L);
            next_b = fr_load(v, stride, leaf + (t + 3) * L);
        }
        const Fr a = fr_from_mont(raw_a);
        const Fr b = fr_from_mont(raw_b);
        uint32_t w[16];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            w[k] = __builtin_bswap32(a.l[k]);
            w[8 + k] = __builtin_bswap32(b.l[k]);
        }
        sha256_compress(h, w);
    }
    if (cnt == 1) {  // a vector of one element: 32 bytes and the padding in one block
        const Fr a = fr_from_mont(fr_load(v, stride, leaf));
        uint32_t w[16];
#pragma unroll
        for (int k = 0; k < 8; ++k) w[k] = __builtin_bswap32(a.l[k]);
        w[8] = 0x80000000u;
#pragma unroll
        for (int k = 9; k < 15; ++k) w[k] = 0;
        w[15] = 256;
        sha256_compress(h, w);
    } else {
        sha256_finish_aligned(h, (uint64_t)cnt * 32);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) job.out[leaf * 8 + k] = h[k];
}

// One step up the tree, again for up to two rows at once: workgroup b of a job
// reduces digests [b*chunk, (b+1)*chunk) of `in` to one (chunk a power of two, at
// most kTreeChunk, and a power of four unless it is the whole row) and writes it
// to out[8b..8b+8).  The launch's last workgroup publishes `seq` if it is not zero
// (then the launch is the last one writing results into the mailbox `words`).
static const uint32_t kTreeChunk = 1024;

struct DigestTreeJob {
    const uint32_t* in;
    uint32_t* out;
    uint32_t chunk;
    uint32_t blocks;  // 0: no such row
};

static __global__ void __launch_bounds__(kBlock) k_digest_tree(DigestTreeJob first, DigestTreeJob second, uint32_t* words,
                                                        uint32_t seq, uint32_t* ticket) {
    __shared__ uint32_t rows[2][kTreeChunk / 4 * 8];  // the row being read and the one being written (at most chunk/4 digests)
    const bool in_first = blockIdx.x < first.blocks;
    const DigestTreeJob& job = in_first ? first : second;
    const uint32_t b = in_first ? blockIdx.x : blockIdx.x - first.blocks;
    // the first row comes from memory; every later one from LDS
    const uint32_t* base = job.in + (size_t)b * job.chunk * 8;
    uint32_t cnt = job.chunk;
    int cur = 0;
    bool from_lds = false;
    while (cnt > 1) {
        const uint32_t group = cnt >= 4 ? 4 : 2;
        const uint32_t nodes = cnt / group;
        for (uint32_t node = threadIdx.x; node < nodes; node += kBlock) {
            uint32_t h[8];
            sha256_init(h);
            for (uint32_t part = 0; part < group; part += 2) {
                uint32_t w[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const uint32_t at = (node * group + part) * 8 + k;
                    w[k] = from_lds ? rows[cur][at] : base[at];
                }
                sha256_compress(h, w);
            }
            sha256_finish_aligned(h, (uint64_t)group * 32);
#pragma unroll
            for (int k = 0; k < 8; ++k) rows[cur ^ 1][node * 8 + k] = h[k];
        }
        __syncthreads();
        cur ^= 1;
        from_lds = true;
        cnt = nodes;
    }
    if (threadIdx.x < 8) {
        const uint32_t v = from_lds ? rows[cur][threadIdx.x] : base[threadIdx.x];
        job.out[(size_t)b * 8 + threadIdx.x] = v;
        mailbox_written();
    }
    __syncthreads();
    if (seq != 0 && threadIdx.x == 0) {
        const unsigned done = atomicAdd(ticket, 1u);
        if (done == gridDim.x - 1) {
            *ticket = 0;
            mailbox_publish(words, seq);
        }
    }
}

// ---- pooled eq tables ----------------------------------------------------------------

// Table q covers variables [var0, var0 + nvars) of the point and occupies
// elements [offset, offset + 2^nvars) of the pool.  Tables marked `scaled` are
// the weights of the rounds on 29-bit limbs: their entries are multiplied by
// `scale` and go, as nine 29-bit limbs, into a pool of their own (three planes of
// `count29` elements, see Planes29 in tlookup_round29.h) at offset - first29.
struct EqPoolArgs {
    Fr u[32];
    uint32_t offset[64];
    uint8_t var0[64];
    uint8_t nvars[64];
    uint8_t scaled[64];
    Fr scale;
    int ntables;
    uint32_t total;
    uint4* pool29;
    size_t count29;
    uint32_t first29;
};

static __global__ void __launch_bounds__(kBlock) k_eq_pool(uint32_t* __restrict__ pool, size_t stride, EqPoolArgs args) {
    const Fr one = fr_one();
    for (uint32_t g = blockIdx.x * kBlock + threadIdx.x; g < args.total; g += gridDim.x * kBlock) {
        int q = 0;
        while (q + 1 < args.ntables && args.offset[q + 1] <= g) ++q;
        uint32_t x = g - args.offset[q];
        int nv = args.nvars[q], v0 = args.var0[q];
        Fr acc = one;
        for (int t = 0; t < nv; ++t) {
            unsigned bit = (x >> (nv - 1 - t)) & 1u;
            Fr f = bit ? args.u[v0 + t] : fr_sub(one, args.u[v0 + t]);
            acc = t == 0 ? f : fr_mul(acc, f);
        }
        if (args.scaled[q]) {
            acc = fr_mul(acc, args.scale);
            const F29 v = f29_unpack(acc.l);
            const size_t i = g - args.first29;
            args.pool29[i] = make_uint4(v.l[0], v.l[1], v.l[2], v.l[3]);
            args.pool29[args.count29 + i] = make_uint4(v.l[4], v.l[5], v.l[6], v.l[7]);
            reinterpret_cast<uint32_t*>(args.pool29 + 2 * args.count29)[i] = v.l[8];
        } else {
            fr_store(pool, stride, g, acc);
        }
    }
}

// ---- sumcheck rounds ---------------------------------------------------------------------

// Weights of a round: the pair with index p (the remaining variables after the
// one being bound) has weight lo[p & (2^lbits - 1)] * hi[p >> lbits]; `hi` is
// null when the low table covers every remaining variable.
struct EqSplit {
    const uint32_t* pool;
    size_t stride;
    uint32_t lo_off;
    uint32_t hi_off;
    int lbits;
    int has_hi;
};

struct PairArray {
    const uint32_t* src;
    size_t ss;
    uint32_t* dst;
    size_t ds;
};

// Loads the pair (x0, x1) of index p for this round.  Without folding the
// array has 2*half entries.  With folding it has 4*half: the previous variable
// is bound to r first (r is wave-uniform), the folded entries are written back
// (to dst) and returned.
template <bool FOLD, bool STORE = true>
__device__ __forceinline__ void load_pair(const PairArray& a, size_t p, size_t half, const Fr& r, Fr& x0, Fr& x1) {
    if constexpr (!FOLD) {
        x0 = fr_load(a.src, a.ss, p);
        x1 = fr_load(a.src, a.ss, p + half);
    } else {
        {
            Fr y0 = fr_load(a.src, a.ss, p), y2 = fr_load(a.src, a.ss, p + 2 * half);
            x0 = fr_fold(y0, y2, r);
        }
        if constexpr (STORE) fr_store(a.dst, a.ds, p, x0);
        {
            Fr y1 = fr_load(a.src, a.ss, p + half), y3 = fr_load(a.src, a.ss, p + 3 * half);
            x1 = fr_fold(y1, y3, r);
        }
        if constexpr (STORE) fr_store(a.dst, a.ds, p + half, x1);
    }
}

struct DataRoundArgs {
    PairArray A, S;
    size_t half;        // pairs in this round
    size_t block_span;  // pairs per workgroup (power of two, at most 2^eq.lbits when eq.has_hi)
    Fr r_prev, beta;
    EqSplit eq;
    uint32_t* partials;  // 5 values per workgroup
    size_t pstride;
    SmallSource ints;    // ints.x not null (first round only): S is given as small integers
};

// Data side of one round.  With w the weight of a pair and (A0, A1), (S0, S1)
// its entries, the sums are
//   q0 = w A0 (S0+beta), q1 = w A1 (S1+beta), qinf = w (A1-A0)(S1-S0), sA0 = A0, sA1 = A1,
// from which the host forms  alpha c e~(u_k, X) q(X) + sA(X).
//
// FOLD = false is the first round, straight after the inversion: there
// A_i (S_i + beta) = 1 for every i, so q0 = q1 = sum of the weights = 1 and only
// qinf and the sums of A are computed (q0 and q1 stay zero and are set by the
// host).
// The three weighted sums are sums of products: they are accumulated as
// unreduced 512-bit integers and reduced once per thread.  In the streaming
// kernels the three 16-limb accumulators of a thread live in LDS (48 KiB per
// workgroup, limb-major so that lanes hit distinct banks) and only pass through
// registers while one product is added: holding them in registers would cost a
// third of the kernel's occupancy.
struct WideInLds {
    // volatile: the accesses stay where they are written, so that at most one
    // accumulator is in registers at a time
    volatile uint32_t* base;  // [3][16][kBlock]
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int k = 0; k < 48; ++k) base[k * kBlock + threadIdx.x] = 0;
    }
    __device__ __forceinline__ FrWide load(int which) const {
        FrWide w;
#pragma unroll
        for (int k = 0; k < 16; ++k) w.l[k] = base[(which * 16 + k) * kBlock + threadIdx.x];
        return w;
    }
    __device__ __forceinline__ void mac(int which, const Fr& a, const Fr& b) {
        FrWide w = load(which);
        fr_wide_mac(w, a, b);
#pragma unroll
        for (int k = 0; k < 16; ++k) base[(which * 16 + k) * kBlock + threadIdx.x] = w.l[k];
    }
    __device__ __forceinline__ Fr finish(int which) const { return fr_wide_reduce(load(which)); }
};

// The same three accumulators in registers, for kernels with one pair per thread.
struct WideInRegs {
    FrWide w[3];
    __device__ __forceinline__ void clear() {
        w[0] = fr_wide_zero();
        w[1] = fr_wide_zero();
        w[2] = fr_wide_zero();
    }
    __device__ __forceinline__ void mac(int which, const Fr& a, const Fr& b) { fr_wide_mac(w[which], a, b); }
    __device__ __forceinline__ Fr finish(int which) const { return fr_wide_reduce(w[which]); }
};

template <bool FOLD, class Wide>
__device__ __forceinline__ void data_pair(const DataRoundArgs& g, size_t p, size_t lo_mask, Wide& wide, Fr& sA0, Fr& sA1) {
    Fr a0, a1, s0, s1;
    load_pair<FOLD>(g.A, p, g.half, g.r_prev, a0, a1);
    if (!FOLD && g.ints.x) {
        small_source_load(s0.l, g.ints, p);
        small_source_load(s1.l, g.ints, p + g.half);
    } else {
        load_pair<FOLD>(g.S, p, g.half, g.r_prev, s0, s1);
    }
    Fr w = fr_load(g.eq.pool, g.eq.stride, g.eq.lo_off + (p & lo_mask));
    sA0 = fr_add(sA0, a0);
    sA1 = fr_add(sA1, a1);
    if constexpr (FOLD) {
        Fr wa0 = fr_mul(w, a0), wa1 = fr_mul(w, a1);
        wide.mac(0, wa0, fr_add(s0, g.beta));
        wide.mac(1, wa1, fr_add(s1, g.beta));
        wide.mac(2, fr_sub(wa1, wa0), fr_sub(s1, s0));
    } else {
        wide.mac(2, w, fr_mul(fr_sub(a1, a0), fr_sub(s1, s0)));
    }
}

// One workgroup's share of the data side: block_span consecutive pairs, which
// all share the high-variable factor of their weight; it is applied once to the
// workgroup's sums.
template <bool FOLD>
__device__ __forceinline__ void round_data_block(const DataRoundArgs& g, unsigned block, uint32_t* lds,
                                                 uint32_t* wide_lds) {
    (void)wide_lds;
    WideInRegs wide;
    wide.clear();
    Fr tot[5];
    tot[3] = fr_zero();
    tot[4] = fr_zero();
    const size_t start = block * g.block_span;
    const size_t lo_mask = ((size_t)1 << g.eq.lbits) - 1;
    for (size_t p = start + threadIdx.x; p < start + g.block_span; p += kBlock)
        data_pair<FOLD>(g, p, lo_mask, wide, tot[3], tot[4]);
    tot[0] = FOLD ? wide.finish(0) : fr_zero();
    tot[1] = FOLD ? wide.finish(1) : fr_zero();
    tot[2] = wide.finish(2);
    block_sum<5, 4>(tot, lds);
    if (threadIdx.x == 0) {
        if (g.eq.has_hi) {
            Fr hf = fr_load(g.eq.pool, g.eq.stride, g.eq.hi_off + (start >> g.eq.lbits));
            if constexpr (FOLD) {
                tot[0] = fr_mul(tot[0], hf);
                tot[1] = fr_mul(tot[1], hf);
            }
            tot[2] = fr_mul(tot[2], hf);
        }
#pragma unroll
        for (int q = 0; q < 5; ++q) fr_store(g.partials, g.pstride, (size_t)block * 5 + q, tot[q]);
    }
}

// The first round: 128 bytes per pair for two multiplications, bound by HBM.  (The
// large folding rounds after it are in tlookup_round29.h; round_data_block<true>
// serves the rounds that also bind a table variable.)
static __global__ void __launch_bounds__(kBlock) k_round_data0(DataRoundArgs g) {
    __shared__ uint32_t lds[4 * 6 * 8];
    round_data_block<false>(g, blockIdx.x, lds, nullptr);
}

struct TableRoundArgs {
    PairArray B, T, M;
    size_t half;
    size_t block_span;
    Fr r_prev, beta;
    EqSplit eq;
    uint32_t* partials;  // 6 values per workgroup
    size_t pstride;
};

// Table side of one round (once the table's own variables are being bound):
//   t0 = w B0 (T0+beta), t1 = w B1 (T1+beta), tinf = w (B1-B0)(T1-T0),
//   m0 = B0 M0, m1 = B1 M1, minf = (B1-B0)(M1-M0).
// The two groups of sums share only B, so they can be computed by different
// threads (PART 1: the T sums, PART 2: the m sums, PART 0: both), which halves the
// dependent chain of multiplications in the rounds that are bound by latency.
// For that B is folded from one buffer into another (both parts read the
// unfolded entries; only PART 0 and PART 1 store the folded ones).
template <bool FOLD, int PART>
__device__ __forceinline__ void table_pair(const TableRoundArgs& g, size_t p, size_t lo_mask, Fr (&tot)[6]) {
    Fr b0, b1;
    load_pair<FOLD, PART != 2>(g.B, p, g.half, g.r_prev, b0, b1);
    if constexpr (PART != 1) {
        Fr m0, m1;
        load_pair<FOLD>(g.M, p, g.half, g.r_prev, m0, m1);
        tot[3] = fr_add(tot[3], fr_mul(b0, m0));
        tot[4] = fr_add(tot[4], fr_mul(b1, m1));
        tot[5] = fr_add(tot[5], fr_mul(fr_sub(b1, b0), fr_sub(m1, m0)));
    }
    if constexpr (PART != 2) {
        Fr t0, t1;
        load_pair<FOLD>(g.T, p, g.half, g.r_prev, t0, t1);
        Fr w = fr_load(g.eq.pool, g.eq.stride, g.eq.lo_off + (p & lo_mask));
        Fr wb0 = fr_mul(w, b0), wb1 = fr_mul(w, b1);
        tot[0] = fr_add(tot[0], fr_mul(wb0, fr_add(t0, g.beta)));
        tot[1] = fr_add(tot[1], fr_mul(wb1, fr_add(t1, g.beta)));
        tot[2] = fr_add(tot[2], fr_mul(fr_sub(wb1, wb0), fr_sub(t1, t0)));
    }
}

template <bool FOLD, int PART>
__device__ __forceinline__ void round_table_block(const TableRoundArgs& g, unsigned block, uint32_t* lds) {
    Fr tot[6];
#pragma unroll
    for (int q = 0; q < 6; ++q) tot[q] = fr_zero();
    const size_t start = block * g.block_span;
    const size_t lo_mask = ((size_t)1 << g.eq.lbits) - 1;
    for (size_t p = start + threadIdx.x; p < start + g.block_span; p += kBlock)
        table_pair<FOLD, PART>(g, p, lo_mask, tot);
    block_sum<6, 4>(tot, lds);
    if (threadIdx.x == 0) {
        if (PART != 2 && g.eq.has_hi) {
            Fr hf = fr_load(g.eq.pool, g.eq.stride, g.eq.hi_off + (start >> g.eq.lbits));
            tot[0] = fr_mul(tot[0], hf);
            tot[1] = fr_mul(tot[1], hf);
            tot[2] = fr_mul(tot[2], hf);
        }
#pragma unroll
        for (int q = 0; q < 6; ++q) {
            const bool mine = PART == 0 || (PART == 1 ? q < 3 : q >= 3);
            if (mine) fr_store(g.partials, g.pstride, (size_t)block * 6 + q, tot[q]);
        }
    }
}

template <bool FOLD>
static __global__ void __launch_bounds__(kBlock) k_round_table(TableRoundArgs g) {
    __shared__ uint32_t lds[4 * 6 * 8];
    round_table_block<FOLD, 0>(g, blockIdx.x, lds);
}

// A round that binds one of the table's variables, all of it in one launch:
// workgroups with blockIdx.y = 0 do the data side, 1 the T sums and 2 the m sums
// of the table side.  The data arrays have been folded at least once by then.
template <bool FOLD_T>
static __global__ void __launch_bounds__(kBlock) k_round_both(DataRoundArgs d, TableRoundArgs t) {
    __shared__ uint32_t lds[4 * 6 * 8];
    if (blockIdx.y == 0) round_data_block<true>(d, blockIdx.x, lds, nullptr);
    else if (blockIdx.y == 1) round_table_block<FOLD_T, 1>(t, blockIdx.x, lds);
    else round_table_block<FOLD_T, 2>(t, blockIdx.x, lds);
}

// The last rounds (at most 256 pairs): one workgroup does the whole round, data
// pairs on threads 0..255, the T sums of the table side on threads 256..511 and
// its m sums on threads 512..767, and writes the eleven sums straight to
// out_words (value q at words 8q..8q+7, data sums first; `words` is the mailbox
// the flag lives in), so the round costs a single launch.  TABLE: 0 = the table is not being bound yet, 1 = first table
// round (nothing to fold), 2 = fold.
static const int kSmallThreads = 768;
static const size_t kSmallPairs = 256;

template <int TABLE>
static __global__ void __launch_bounds__(kSmallThreads) k_round_small(DataRoundArgs d, TableRoundArgs t,
                                                                     uint32_t* out_words, uint32_t* words,
                                                                     uint32_t seq) {
    __shared__ uint32_t lds[12 * 6 * 8];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int group = threadIdx.x >> 8;  // 0 data, 1 table T sums, 2 table m sums
    const size_t p = threadIdx.x & 255;
    const size_t lo_mask = ((size_t)1 << d.eq.lbits) - 1;
    Fr tot[6];
#pragma unroll
    for (int q = 0; q < 6; ++q) tot[q] = fr_zero();
    if (group == 0) {
        if (p < d.half) {
            WideInRegs wide;
            wide.clear();
            data_pair<true>(d, p, lo_mask, wide, tot[3], tot[4]);
            tot[0] = wide.finish(0);
            tot[1] = wide.finish(1);
            tot[2] = wide.finish(2);
        }
    } else if (TABLE != 0 && p < t.half) {
        if (group == 1) table_pair<TABLE == 2, 1>(t, p, lo_mask, tot);
        else table_pair<TABLE == 2, 2>(t, p, lo_mask, tot);
    }
#pragma unroll
    for (int q = 0; q < 6; ++q) {
        tot[q] = wave_sum(tot[q]);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < 8; ++k) lds[(wave * 6 + q) * 8 + k] = tot[q].l[k];
        }
    }
    __syncthreads();
    // thread `slot` adds up output value `slot` over the four wavefronts of its group:
    // 0..4 data sums, 5..7 the T sums (accumulators 0..2 of group 1), 8..10 the m sums
    // (accumulators 3..5 of group 2)
    const int slot = threadIdx.x;
    if (slot < (TABLE != 0 ? 11 : 5)) {
        const int g = slot < 5 ? 0 : slot < 8 ? 1 : 2;
        const int q = slot < 5 ? slot : slot - 5;
        Fr acc = fr_zero();
        for (int w = 4 * g; w < 4 * g + 4; ++w) {
            Fr o;
#pragma unroll
            for (int k = 0; k < 8; ++k) o.l[k] = lds[(w * 6 + q) * 8 + k];
            acc = fr_add(acc, o);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) out_words[8 * slot + k] = acc.l[k];
        mailbox_written();
    }
    __syncthreads();
    if (threadIdx.x == 0) mailbox_publish(words, seq);
}

// Final values: each of up to five arrays is either a single entry or a pair
// still to be bound to the last challenge.  Value q goes to out_words[8q..8q+8);
// `words` is the mailbox the flag lives in.
struct FinalArgs {
    const uint32_t* p[8];
    size_t stride[8];
    int fold[8];
    int count;
    Fr r;
};

// All the last rounds of one proof in one resident kernel: what k_round_small
// does for one round, repeated, with each round's challenge received over the
// host's command channel (a bounded wait) instead of as a launch argument, and
// the five final values at the end.  What changes from round to round comes in
// a small record per round.  Every thread takes every barrier; a wait that
// fails ends the kernel for all of them.
static const int kTailRoundsMax = 9;  // pairs go 256, 128, .., 1

struct TailRound {
    PairArray S, B, T;  // this round's sources and destinations (A and M fold in place)
    EqSplit eq;
    size_t half;
    int table;          // as k_round_small's TABLE
};

// What the resident kernel hands to the host after its last round, if the host runs the remaining rounds itself:
// the five arrays A, S, B, m, T as they stand then, each with its pending variable (if it has one) bound to the
// last challenge, n_out[q] elements of array q one after the other, eight Montgomery words per element.
struct TailShip {
    uint32_t* out;  // pinned host memory; null: the kernel runs every round and writes the final claims
    const uint32_t* p[5];
    size_t stride[5];
    uint32_t n_out[5];
    int fold[5];
};

struct TlookupTailArgs {
    PairArray A, M;
    Fr beta, r_prev;
    TailRound round[kTailRoundsMax];
    int nrounds;
    FinalArgs fin;      // where the five arrays end up (fin.r is not used)
    TailShip ship;
    uint32_t* out_words;   // this proof's slot in the mailbox
    uint32_t* words;       // the mailbox (flag)
    const uint32_t* cmd;
    uint32_t out_seq[kTailRoundsMax + 1];
    uint32_t cmd_seq[kTailRoundsMax];
    uint32_t spin_limit;
};

static __global__ void __launch_bounds__(kSmallThreads) k_tlookup_tail(TlookupTailArgs g) {
    __shared__ uint32_t lds[12 * 6 * 8];
    __shared__ uint32_t sh_r[8];
    __shared__ int sh_ok;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int group = threadIdx.x >> 8;  // 0 data, 1 table T sums, 2 table m sums
    const size_t p = threadIdx.x & 255;
    Fr r = g.r_prev;
    bool ok = true;
    for (int i = 0; i < g.nrounds; ++i) {
        const TailRound& rd = g.round[i];
        const size_t lo_mask = ((size_t)1 << rd.eq.lbits) - 1;
        Fr tot[6];
#pragma unroll
        for (int q = 0; q < 6; ++q) tot[q] = fr_zero();
        if (group == 0) {
            if (p < rd.half) {
                DataRoundArgs d;
                d.A = g.A;
                d.S = rd.S;
                d.half = rd.half;
                d.block_span = 0;
                d.r_prev = r;
                d.beta = g.beta;
                d.eq = rd.eq;
                d.partials = nullptr;
                d.pstride = 0;
                WideInRegs wide;
                wide.clear();
                data_pair<true>(d, p, lo_mask, wide, tot[3], tot[4]);
                tot[0] = wide.finish(0);
                tot[1] = wide.finish(1);
                tot[2] = wide.finish(2);
            }
        } else if (rd.table != 0 && p < rd.half) {
            TableRoundArgs t;
            t.B = rd.B;
            t.T = rd.T;
            t.M = g.M;
            t.half = rd.half;
            t.block_span = 0;
            t.r_prev = r;
            t.beta = g.beta;
            t.eq = rd.eq;
            t.partials = nullptr;
            t.pstride = 0;
            if (rd.table == 2) {
                if (group == 1) table_pair<true, 1>(t, p, lo_mask, tot);
                else table_pair<true, 2>(t, p, lo_mask, tot);
            } else {
                if (group == 1) table_pair<false, 1>(t, p, lo_mask, tot);
                else table_pair<false, 2>(t, p, lo_mask, tot);
            }
        }
#pragma unroll
        for (int q = 0; q < 6; ++q) {
            tot[q] = wave_sum(tot[q]);
            if (lane == 0) {
#pragma unroll
                for (int k = 0; k < 8; ++k) lds[(wave * 6 + q) * 8 + k] = tot[q].l[k];
            }
        }
        __syncthreads();
        // thread `slot` adds up output value `slot` over the four wavefronts of its group
        // (see k_round_small)
        const int slot = threadIdx.x;
        if (slot < (rd.table != 0 ? 11 : 5)) {
            const int gq = slot < 5 ? 0 : slot < 8 ? 1 : 2;
            const int q = slot < 5 ? slot : slot - 5;
            Fr acc = fr_zero();
            for (int w = 4 * gq; w < 4 * gq + 4; ++w) {
                Fr o;
#pragma unroll
                for (int k = 0; k < 8; ++k) o.l[k] = lds[(w * 6 + q) * 8 + k];
                acc = fr_add(acc, o);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) g.out_words[8 * slot + k] = acc.l[k];
            mailbox_written();
        }
        __syncthreads();
        if (threadIdx.x == 0) {
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
        __syncthreads();
        if (!ok) break;  // the same for every thread
    }
    if (ok && g.ship.out) {
        // the host takes over: the arrays with the last challenge bound (at most 64 elements each)
        const uint32_t total = g.ship.n_out[0] + g.ship.n_out[1] + g.ship.n_out[2] + g.ship.n_out[3] + g.ship.n_out[4];
        for (uint32_t t = threadIdx.x; t < total; t += kSmallThreads) {
            int q = 0;
            uint32_t j = t;
            while (q < 4 && j >= g.ship.n_out[q]) {
                j -= g.ship.n_out[q];
                ++q;
            }
            Fr v = fr_load(g.ship.p[q], g.ship.stride[q], j);
            if (g.ship.fold[q]) v = fr_fold(v, fr_load(g.ship.p[q], g.ship.stride[q], j + g.ship.n_out[q]), r);
#pragma unroll
            for (int k = 0; k < 8; ++k) g.ship.out[8 * (size_t)t + k] = v.l[k];
            mailbox_written();
        }
    } else if (ok && threadIdx.x < (unsigned)g.fin.count) {
        const int q = threadIdx.x;
        Fr v = fr_load(g.fin.p[q], g.fin.stride[q], 0);
        if (g.fin.fold[q]) v = fr_fold(v, fr_load(g.fin.p[q], g.fin.stride[q], 1), r);
#pragma unroll
        for (int k = 0; k < 8; ++k) g.out_words[8 * q + k] = v.l[k];
        mailbox_written();
    }
    __syncthreads();
    if (ok && threadIdx.x == 0) mailbox_publish(g.words, g.out_seq[g.nrounds]);
}

// Sums over the whole table, before any of its variables is bound:
//   c1 = sum_j e'_j B_j (T_j + beta),  c2 = sum_j B_j M_j,
// with e'_j = lo[j & mask] * hi[j >> lbits].
struct TableConstArgs {
    const uint32_t* B; size_t bs;
    const uint32_t* T; size_t ts;
    const uint32_t* M; size_t ms;
    size_t N;
    Fr beta;
    EqSplit eq;
    uint32_t* partials;  // 2 values per workgroup
    size_t pstride;
};

static __global__ void __launch_bounds__(kBlock) k_table_const(TableConstArgs g) {
    __shared__ uint32_t lds[4 * 2 * 8];
    Fr tot[2] = {fr_zero(), fr_zero()};
    const size_t lo_mask = ((size_t)1 << g.eq.lbits) - 1;
    for (size_t j = blockIdx.x * (size_t)kBlock + threadIdx.x; j < g.N; j += (size_t)gridDim.x * kBlock) {
        Fr b = fr_load(g.B, g.bs, j), t = fr_load(g.T, g.ts, j), m = fr_load(g.M, g.ms, j);
        Fr w = fr_load(g.eq.pool, g.eq.stride, g.eq.lo_off + (j & lo_mask));
        if (g.eq.has_hi) w = fr_mul(w, fr_load(g.eq.pool, g.eq.stride, g.eq.hi_off + (j >> g.eq.lbits)));
        tot[0] = fr_add(tot[0], fr_mul(fr_mul(w, b), fr_add(t, g.beta)));
        tot[1] = fr_add(tot[1], fr_mul(b, m));
    }
    block_sum<2, 4>(tot, lds);
    if (threadIdx.x == 0) {
        fr_store(g.partials, g.pstride, (size_t)blockIdx.x * 2, tot[0]);
        fr_store(g.partials, g.pstride, (size_t)blockIdx.x * 2 + 1, tot[1]);
    }
}

static __global__ void k_final_values(FinalArgs g, uint32_t* out_words, uint32_t* words, uint32_t seq) {
    int q = threadIdx.x;
    if (q < g.count) {
        Fr v = fr_load(g.p[q], g.stride[q], 0);
        if (g.fold[q]) v = fr_fold(v, fr_load(g.p[q], g.stride[q], 1), g.r);
#pragma unroll
        for (int k = 0; k < 8; ++k) out_words[8 * q + k] = v.l[k];
        mailbox_written();
    }
    __syncthreads();
    if (threadIdx.x == 0) mailbox_publish(words, seq);
}

}  // namespace zkmi
