// Batched inversion by the product trick, arranged for a GPU:
//
//   down pass  : every thread multiplies up its K elements (stride 256 within a
//                block, so loads stay coalesced), storing the running products,
//                and emits its total into the next, K times smaller, level;
//   top        : one workgroup scans the last level (<= 256 values); the host
//                inverts the single grand total (the only field inversion);
//   up pass    : each thread receives the inverse of its own total and walks
//                back over its elements: out_j = inv * prefix_{j-1}, inv *= x_j.
//
// A level after the first that is short enough (<= 2^20 elements) is reduced by
// whole workgroups instead: the threads' totals are multiplied up within the
// workgroup (a scan in LDS), so the next level is 256*K times smaller and fits
// the top.  That saves dependent launches, which is all the small levels cost:
// eight for 2^25 elements instead of twelve.  (Longer levels stay with the
// threads: there the scans cost more than the launches they save.)
//
// Cost: about 3 multiplications per element plus a geometric tail.  A zero
// anywhere makes the grand total zero, which is how it is detected.
#include "internal.h"
#include "small_dev.h"

namespace zkmi {

static const int kBiK = 16;  // elements per thread per level

// A level can be the concatenation of two vectors (the tensor and the table of a
// lookup, inverted in one go): elements from n1 on belong to the second, which
// has its own source and its own prefix/result buffer.  n1 is a multiple of the
// elements one workgroup covers, so a workgroup lies in one of them.
struct BiSecond {
    const uint32_t* src;
    size_t ss;
    uint32_t* p;
    size_t ps;
    size_t n1;  // SIZE_MAX: no second vector
};

__device__ __forceinline__ Fr bi_load(const uint32_t* __restrict__ src, size_t ss, size_t i, bool shifted,
                                      const Fr& shift) {
    Fr x = fr_load(src, ss, i);
    return shifted ? fr_add(x, shift) : x;
}

// The first vector of the first level given as small integers (SmallSource, see
// small_dev.h) instead of field elements.
__device__ __forceinline__ Fr bi_load_small(const SmallSource& small, size_t i, bool shifted, const Fr& shift) {
    Fr x;
    small_source_load(x.l, small, i);
    return shifted ? fr_add(x, shift) : x;
}

// prefix_i = product of this thread's elements up to and including i; the
// thread's total goes to next[tid].
__global__ void __launch_bounds__(kBlock) k_bi_down(const uint32_t* __restrict__ src, size_t ss, size_t n, int shifted,
                                                    Fr shift, uint32_t* __restrict__ prefix, size_t ps,
                                                    uint32_t* __restrict__ next, size_t ns, BiSecond second,
                                                    SmallSource small) {
    size_t tid = blockIdx.x * (size_t)kBlock + threadIdx.x;
    size_t base = blockIdx.x * (size_t)kBlock * kBiK + threadIdx.x;
    bool from_small = small.x != nullptr;
    if (blockIdx.x * (size_t)kBlock * kBiK >= second.n1) {  // the whole workgroup is in the second vector
        src = second.src;
        ss = second.ss;
        prefix = second.p;
        ps = second.ps;
        base -= second.n1;
        n -= second.n1;
        from_small = false;
    } else if (n > second.n1) {
        n = second.n1;
    }
    Fr acc = fr_one();
    bool first = true;
    for (int j = 0; j < kBiK; ++j) {
        size_t i = base + (size_t)j * kBlock;
        if (i < n) {
            Fr x = from_small ? bi_load_small(small, i, shifted, shift) : bi_load(src, ss, i, shifted, shift);
            acc = first ? x : fr_mul(acc, x);
            first = false;
            fr_store(prefix, ps, i, acc);
        }
    }
    fr_store(next, ns, tid, acc);
}

// inv_next[tid] = inverse of this thread's total.  out may be the prefix buffer.
__global__ void __launch_bounds__(kBlock) k_bi_up(const uint32_t* __restrict__ src, size_t ss, size_t n, int shifted,
                                                  Fr shift, const uint32_t* prefix, size_t ps,
                                                  const uint32_t* __restrict__ inv_next, size_t is, uint32_t* out,
                                                  size_t os, BiSecond second, SmallSource small) {
    size_t tid = blockIdx.x * (size_t)kBlock + threadIdx.x;
    size_t base = blockIdx.x * (size_t)kBlock * kBiK + threadIdx.x;
    bool from_small = small.x != nullptr;
    if (blockIdx.x * (size_t)kBlock * kBiK >= second.n1) {  // prefix and out are the same buffer (see batch_inverse_end)
        src = second.src;
        ss = second.ss;
        prefix = second.p;
        ps = second.ps;
        out = second.p;
        os = second.ps;
        base -= second.n1;
        n -= second.n1;
        from_small = false;
    } else if (n > second.n1) {
        n = second.n1;
    }
    Fr inv = fr_load(inv_next, is, tid);
    for (int j = kBiK - 1; j >= 0; --j) {
        size_t i = base + (size_t)j * kBlock;
        if (i < n) {
            if (j > 0) {
                Fr before = fr_load(prefix, ps, i - kBlock);
                Fr x = from_small ? bi_load_small(small, i, shifted, shift) : bi_load(src, ss, i, shifted, shift);
                fr_store(out, os, i, fr_mul(inv, before));
                inv = fr_mul(inv, x);
            } else {
                fr_store(out, os, i, inv);
            }
        }
    }
}

// Inclusive scan of products over one workgroup of THREADS threads (Hillis-Steele in LDS, 8*THREADS words).
template <int THREADS>
__device__ __forceinline__ Fr block_scan_mul(Fr v, uint32_t* lds, bool reverse) {
    const int t = threadIdx.x;
    for (int off = 1; off < THREADS; off <<= 1) {
#pragma unroll
        for (int k = 0; k < 8; ++k) lds[k * THREADS + t] = v.l[k];
        __syncthreads();
        int partner = reverse ? t + off : t - off;
        if (partner >= 0 && partner < THREADS) {
            Fr o;
#pragma unroll
            for (int k = 0; k < 8; ++k) o.l[k] = lds[k * THREADS + partner];
            v = fr_mul(v, o);
        }
        __syncthreads();
    }
    return v;
}

// The scanned value of the thread before (reverse: after) this one, or one at the end of the line.
template <int THREADS>
__device__ __forceinline__ Fr block_neighbour(const Fr& scanned, uint32_t* lds, bool reverse) {
    const int t = threadIdx.x;
#pragma unroll
    for (int k = 0; k < 8; ++k) lds[k * THREADS + t] = scanned.l[k];
    __syncthreads();
    Fr o = fr_one();
    const int partner = reverse ? t + 1 : t - 1;
    if (partner >= 0 && partner < THREADS) {
#pragma unroll
        for (int k = 0; k < 8; ++k) o.l[k] = lds[k * THREADS + partner];
    }
    __syncthreads();
    return o;
}

// A level reduced by whole workgroups, down: as k_bi_down, then the product of the
// workgroup's thread totals goes to next[blockIdx.x].
template <int kPer>
__global__ void __launch_bounds__(kBlock) k_bi_down_wg(const uint32_t* __restrict__ src, size_t ss, size_t n,
                                                       uint32_t* __restrict__ prefix, size_t ps,
                                                       uint32_t* __restrict__ next, size_t ns) {
    __shared__ uint32_t lds[8 * kBlock];
    const size_t base = blockIdx.x * (size_t)kBlock * kPer + threadIdx.x;
    Fr x[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const size_t i = base + (size_t)j * kBlock;
        x[j] = i < n ? fr_load(src, ss, i) : fr_one();
    }
    Fr acc = x[0];
    if (base < n) fr_store(prefix, ps, base, acc);
#pragma unroll
    for (int j = 1; j < kPer; ++j) {
        const size_t i = base + (size_t)j * kBlock;
        if (i < n) {
            acc = fr_mul(acc, x[j]);
            fr_store(prefix, ps, i, acc);
        }
    }
    const Fr total = block_scan_mul<kBlock>(acc, lds, false);
    if (threadIdx.x == kBlock - 1) fr_store(next, ns, blockIdx.x, total);
}

// Up: inv_next[blockIdx.x] is the inverse of the workgroup's product; a thread's
// own inverse is that times the totals of all other threads of the workgroup.
template <int kPer>
__global__ void __launch_bounds__(kBlock) k_bi_up_wg(const uint32_t* __restrict__ src, size_t ss, size_t n,
                                                     const uint32_t* prefix, size_t ps,
                                                     const uint32_t* __restrict__ inv_next, size_t is, uint32_t* out,
                                                     size_t os) {
    __shared__ uint32_t lds[8 * kBlock];
    const size_t base = blockIdx.x * (size_t)kBlock * kPer + threadIdx.x;
    // how many elements this thread has; its total is the last of its running products
    int count = 0;
    if (base < n) {
        const size_t left = (n - base + kBlock - 1) / kBlock;
        count = left < (size_t)kPer ? (int)left : kPer;
    }
    const Fr total = count ? fr_load(prefix, ps, base + (size_t)(count - 1) * kBlock) : fr_one();
    const Fr pre = block_scan_mul<kBlock>(total, lds, false);
    const Fr suf = block_scan_mul<kBlock>(total, lds, true);
    const Fr others = fr_mul(block_neighbour<kBlock>(pre, lds, false), block_neighbour<kBlock>(suf, lds, true));
    Fr inv = fr_mul(fr_load(inv_next, is, blockIdx.x), others);
    // back over the elements, at most eight at a time: their loads do not depend on the chain of products
    constexpr int kStep = kPer < 8 ? kPer : 8;
#pragma unroll
    for (int part = kPer / kStep - 1; part >= 0; --part) {
        Fr x[kStep], before[kStep];
#pragma unroll
        for (int q = 0; q < kStep; ++q) {
            const int j = part * kStep + q;
            const size_t i = base + (size_t)j * kBlock;
            x[q] = j > 0 && j < count ? fr_load(src, ss, i) : fr_one();
            before[q] = j > 0 && j < count ? fr_load(prefix, ps, i - kBlock) : fr_one();
        }
#pragma unroll
        for (int q = kStep - 1; q >= 0; --q) {
            const int j = part * kStep + q;
            if (j < count) {
                const size_t i = base + (size_t)j * kBlock;
                if (j > 0) {
                    fr_store(out, os, i, fr_mul(inv, before[q]));
                    inv = fr_mul(inv, x[q]);
                } else {
                    fr_store(out, os, i, inv);
                }
            }
        }
    }
}

// Grand total of the last level (n <= THREADS) to total_words (Montgomery limbs).
template <int THREADS>
__global__ void __launch_bounds__(THREADS) k_bi_top_total(const uint32_t* __restrict__ src, size_t ss, size_t n,
                                                          int shifted, Fr shift, uint32_t* total_words,
                                                          uint32_t* flag_words, uint32_t seq) {
    __shared__ uint32_t lds[8 * THREADS];
    Fr x = threadIdx.x < n ? bi_load(src, ss, threadIdx.x, shifted, shift) : fr_one();
    Fr p = block_scan_mul<THREADS>(x, lds, false);
    if (threadIdx.x == THREADS - 1) {
#pragma unroll
        for (int k = 0; k < 8; ++k) total_words[k] = p.l[k];
        mailbox_written();
        mailbox_publish(flag_words, seq);
    }
}

// out_t = inv_total * (product of the others) for the last level.
template <int THREADS>
__global__ void __launch_bounds__(THREADS) k_bi_top_finish(const uint32_t* __restrict__ src, size_t ss, size_t n,
                                                           int shifted, Fr shift, Fr inv_total, uint32_t* out,
                                                           size_t os) {
    __shared__ uint32_t lds[8 * THREADS];
    const int t = threadIdx.x;
    Fr x = (size_t)t < n ? bi_load(src, ss, t, shifted, shift) : fr_one();
    Fr pre = block_scan_mul<THREADS>(x, lds, false);  // x_0 .. x_t
    Fr suf = block_scan_mul<THREADS>(x, lds, true);   // x_t .. x_last
    Fr before = block_neighbour<THREADS>(pre, lds, false);
    Fr after = block_neighbour<THREADS>(suf, lds, true);
    if ((size_t)t < n) fr_store(out, os, t, fr_mul(inv_total, fr_mul(before, after)));
}

static const size_t kBiTopMax = kBlock;  // values the top kernels take

// Whether level `depth` of length n is reduced by whole workgroups, how many
// elements a thread then takes (as few as still leave the top at most kBiTopMax
// values: the chain of products is what such a level costs), and the next level's length.
static bool bi_by_workgroups(int depth, size_t n) { return depth >= 1 && n <= kBiTopMax * kBlock * kBiK; }
static int bi_wg_per_thread(size_t n) {
    int per = 2;
    while (per < kBiK && div_up(n, (size_t)kBlock * per) > kBiTopMax) per *= 2;
    return per;
}
static size_t bi_next_size(int depth, size_t n) {
    if (bi_by_workgroups(depth, n)) return div_up(n, (size_t)kBlock * bi_wg_per_thread(n));
    return div_up(n, (size_t)kBlock * kBiK) * kBlock;
}

template <int kPer>
static void bi_launch_wg(bool down, unsigned blocks, hipStream_t stream, const uint32_t* x, size_t xs, size_t n, uint32_t* p,
                         size_t ps, uint32_t* next_or_inv, size_t ns) {
    if (down) hipLaunchKernelGGL(k_bi_down_wg<kPer>, dim3(blocks), dim3(kBlock), 0, stream, x, xs, n, p, ps, next_or_inv, ns);
    else hipLaunchKernelGGL(k_bi_up_wg<kPer>, dim3(blocks), dim3(kBlock), 0, stream, x, xs, n, p, ps, next_or_inv, ns, p, ps);
}
static void bi_launch_wg_level(bool down, hipStream_t stream, const uint32_t* x, size_t xs, size_t n, uint32_t* p, size_t ps,
                               uint32_t* next_or_inv, size_t ns) {
    const int per = bi_wg_per_thread(n);
    const unsigned blocks = (unsigned)div_up(n, (size_t)kBlock * per);
    if (per == 2) bi_launch_wg<2>(down, blocks, stream, x, xs, n, p, ps, next_or_inv, ns);
    else if (per == 4) bi_launch_wg<4>(down, blocks, stream, x, xs, n, p, ps, next_or_inv, ns);
    else if (per == 8) bi_launch_wg<8>(down, blocks, stream, x, xs, n, p, ps, next_or_inv, ns);
    else bi_launch_wg<16>(down, blocks, stream, x, xs, n, p, ps, next_or_inv, ns);
}

size_t batch_inverse_scratch_bytes(size_t n) {
    Carver cv(nullptr, 0);
    size_t m = n;
    for (int depth = 0; m > kBiTopMax; ++depth) {
        m = bi_next_size(depth, m);
        cv.limbs(m);  // level values
        cv.limbs(m);  // level prefixes, then inverses
    }
    return cv.used();
}

static BiSecond bi_second_of(const BatchInverseJob& job, int depth) {
    if (depth == 0 && job.n2) return BiSecond{job.src2, job.src2_stride, job.dst2, job.dst2_stride, job.lv[0].n - job.n2};
    return BiSecond{nullptr, 0, nullptr, 0, SIZE_MAX};
}

static SmallSource bi_small_of(const BatchInverseJob& job, int depth) {
    SmallSource none;
    memset(&none, 0, sizeof none);
    return depth == 0 && job.small.x ? job.small : none;
}

bool batch_inverse_can_join(size_t n1) { return n1 % ((size_t)kBlock * kBiK) == 0; }

int batch_inverse_begin(BatchInverseJob& job, uint32_t* dst, size_t dst_stride, const uint32_t* src, size_t src_stride,
                        size_t n, const host::F& shift, Carver& cv, uint32_t* total_words, uint32_t* flag_words,
                        uint32_t seq, hipStream_t stream, uint32_t* dst2, size_t dst2_stride, const uint32_t* src2,
                        size_t src2_stride, size_t n2, const SmallSource* small) {
    typedef BatchInverseJob::Level Level;
    if (n2 && !batch_inverse_can_join(n)) return ZK_E_BADARG;
    if (small && n <= kBiTopMax) return ZK_E_BADARG;  // the top kernels read field elements
    memset(&job.small, 0, sizeof job.small);
    if (small) job.small = *small;
    job.depth = 0;
    job.shift = to_dev(shift);
    job.n2 = n2;
    job.src2 = src2;
    job.src2_stride = src2_stride;
    job.dst2 = dst2;
    job.dst2_stride = dst2_stride;
    int shifted0 = host::is_zero(shift) ? 0 : 1;
    job.lv[0] = Level{src, src_stride, dst, dst_stride, n + n2, shifted0};
    if (n2 && n + n2 <= kBiTopMax) return ZK_E_BADARG;  // a joined vector is longer than the top kernels take
    while (job.lv[job.depth].n > kBiTopMax) {
        const Level& cur = job.lv[job.depth];
        const size_t m = bi_next_size(job.depth, cur.n);
        const unsigned blocks = (unsigned)div_up(cur.n, (size_t)kBlock * kBiK);
        uint32_t* x = cv.limbs(m);
        uint32_t* p = cv.limbs(m);
        if (!x || !p) return ZK_E_BUFSZ;
        if (bi_by_workgroups(job.depth, cur.n))
            bi_launch_wg_level(true, stream, cur.x, cur.xs, cur.n, cur.p, cur.ps, x, m);
        else
            hipLaunchKernelGGL(k_bi_down, dim3(blocks), dim3(kBlock), 0, stream, cur.x, cur.xs, cur.n, cur.shifted,
                               job.shift, cur.p, cur.ps, x, m, bi_second_of(job, job.depth), bi_small_of(job, job.depth));
        ++job.depth;
        job.lv[job.depth] = Level{x, m, p, m, m, 0};
    }
    const Level& top = job.lv[job.depth];
    hipLaunchKernelGGL(k_bi_top_total<kBlock>, dim3(1), dim3(kBlock), 0, stream, top.x, top.xs, top.n, top.shifted,
                       job.shift, total_words, flag_words, seq);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

int batch_inverse_end(const BatchInverseJob& job, const host::F& inv_total, hipStream_t stream) {
    typedef BatchInverseJob::Level Level;
    const Level& top = job.lv[job.depth];
    hipLaunchKernelGGL(k_bi_top_finish<kBlock>, dim3(1), dim3(kBlock), 0, stream, top.x, top.xs, top.n, top.shifted,
                       job.shift, to_dev(inv_total), top.p, top.ps);
    for (int d = job.depth - 1; d >= 0; --d) {
        const Level& cur = job.lv[d];
        const Level& up = job.lv[d + 1];
        const unsigned blocks = (unsigned)div_up(cur.n, (size_t)kBlock * kBiK);
        if (bi_by_workgroups(d, cur.n))
            bi_launch_wg_level(false, stream, cur.x, cur.xs, cur.n, cur.p, cur.ps, up.p, up.ps);
        else
            hipLaunchKernelGGL(k_bi_up, dim3(blocks), dim3(kBlock), 0, stream, cur.x, cur.xs, cur.n, cur.shifted, job.shift,
                               cur.p, cur.ps, up.p, up.ps, cur.p, cur.ps, bi_second_of(job, d), bi_small_of(job, d));
    }
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

int batch_inverse_run(uint32_t* dst, size_t dst_stride, const uint32_t* src, size_t src_stride, size_t n,
                      const host::F& shift, Carver& cv, Mailbox* mb, hipStream_t stream) {
    if (n == 0) return ZK_OK;
    BatchInverseJob job;
    uint32_t seq = mb->next_seq();
    ZK_TRY(batch_inverse_begin(job, dst, dst_stride, src, src_stride, n, shift, cv, mb->words + kMailboxInvA, mb->words,
                               seq, stream, nullptr, 0, nullptr, 0, 0, nullptr));
    ZK_TRY(mailbox_wait(mb, seq, stream));
    host::F total = from_dev(mb->words + kMailboxInvA);
    if (host::is_zero(total)) return ZK_E_ZERO_DENOM;
    return batch_inverse_end(job, host::inv(total), stream);
}

}  // namespace zkmi

using namespace zkmi;

extern "C" {

size_t fr_batch_inverse_workspace_bytes(size_t n) { return batch_inverse_scratch_bytes(n); }

int fr_batch_inverse(fr_vec dst, fr_vec src, void* ws, size_t ws_bytes, void* stream) {
    size_t n = dst.n;
    if (!vec_ok(dst, n) || !vec_ok(src, n)) return ZK_E_BADARG;
    if (n == 0) return ZK_OK;
    if (dst.limbs == src.limbs) return ZK_E_BADARG;
    if (!ws || ws_bytes < batch_inverse_scratch_bytes(n)) return ZK_E_BUFSZ;
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(ws, ws_bytes);
    ZK_TRY(batch_inverse_run(dst.limbs, dst.stride, src.limbs, src.stride, n, host::zero(), cv, mb, as_stream(stream)));
    ZK_HIP_TRY(hipStreamSynchronize(as_stream(stream)));
    return ZK_OK;
}

}  // extern "C"
