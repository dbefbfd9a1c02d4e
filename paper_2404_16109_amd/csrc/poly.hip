// Sums, eq tables, folding and multilinear evaluation (Section 3.3 of the paper:
// tensors as functions on the Boolean cube and their multilinear extensions).
#include <mutex>

#include "internal.h"
#include "reduce_dev.h"

namespace zkmi {

// ---- sums -------------------------------------------------------------------

__global__ void k_fill_words(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

void launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t stream) {
    if (n == 0) return;
    hipLaunchKernelGGL(k_fill_words, dim3(grid_for(n)), dim3(kBlock), 0, stream, p, n, v);
}

__global__ void __launch_bounds__(kBlock) k_sum_partial(const uint32_t* __restrict__ a, size_t stride, size_t n,
                                                        uint32_t* __restrict__ partials, size_t pstride) {
    __shared__ uint32_t lds[4 * 8];
    Fr acc[1] = {fr_zero()};
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
        acc[0] = fr_add(acc[0], fr_load(a, stride, i));
    block_sum<1, 4>(acc, lds);
    if (threadIdx.x == 0) fr_store(partials, pstride, blockIdx.x, acc[0]);
}

// Adds up the per-workgroup partial values of a round, one workgroup per value
// (the first nv1 values come from the first array, the rest from the second;
// value v of workgroup b sits at element b*nv + v of its array).  Totals go out as
// raw Montgomery limbs, value q at out_words[8q..8q+7].  The workgroup that
// finishes last (a ticket counter in device memory, left at zero again) publishes
// completion.
static const int kFinalThreads = 1024;

__global__ void __launch_bounds__(kFinalThreads) k_final_sum2(const uint32_t* __restrict__ part1, size_t pstride1, int nv1,
                                                              const uint32_t* __restrict__ part2, size_t pstride2, int nv2,
                                                              unsigned nblocks, uint32_t* out_words, uint32_t* words,
                                                              uint32_t seq, uint32_t* ticket) {
    __shared__ uint32_t lds[16 * 8];
    const int q = blockIdx.x;
    const bool first = q < nv1;
    const uint32_t* part = first ? part1 : part2;
    const size_t pstride = first ? pstride1 : pstride2;
    const int nv = first ? nv1 : nv2, qq = first ? q : q - nv1;
    Fr acc[1] = {fr_zero()};
    for (unsigned b = threadIdx.x; b < nblocks; b += kFinalThreads)
        acc[0] = fr_add(acc[0], fr_load(part, pstride, (size_t)b * nv + qq));
    block_sum<1, 16>(acc, lds);
    if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) out_words[8 * q + k] = acc[0].l[k];
        mailbox_written();
        if (seq != 0) {
            unsigned done = atomicAdd(ticket, 1u);
            if (done == gridDim.x - 1) {
                *ticket = 0;
                mailbox_publish(words, seq);
            }
        }
    }
}

void launch_final_sum2(const uint32_t* part1, size_t pstride1, int nv1, const uint32_t* part2, size_t pstride2, int nv2,
                       unsigned nblocks, uint32_t* out_words, uint32_t* words, uint32_t seq, uint32_t* ticket,
                       hipStream_t stream) {
    hipLaunchKernelGGL(k_final_sum2, dim3(nv1 + nv2), dim3(kFinalThreads), 0, stream, part1, pstride1, nv1, part2, pstride2,
                       nv2, nblocks, out_words, words, seq, ticket);
}

void launch_final_sum(const uint32_t* partials, size_t pstride, unsigned nblocks, int nv, uint32_t* out_words,
                      uint32_t* words, uint32_t seq, uint32_t* ticket, hipStream_t stream) {
    launch_final_sum2(partials, pstride, nv, nullptr, 0, 0, nblocks, out_words, words, seq, ticket, stream);
}

size_t sum_scratch_bytes(size_t) {
    Carver cv(nullptr, 0);
    cv.limbs(kMaxPartialBlocks);
    cv.take(256);  // ticket
    return cv.used();
}

int sum_run(const uint32_t* a, size_t stride, size_t n, Carver& cv, Mailbox* mb, uint32_t seq, hipStream_t stream) {
    uint32_t* partials = cv.limbs(kMaxPartialBlocks);
    uint32_t* ticket = (uint32_t*)cv.take(256);
    if (!partials || !ticket) return ZK_E_BUFSZ;
    launch_fill_u32(ticket, 1, 0u, stream);
    unsigned blocks = grid_for(n, kBlock * 8, kMaxPartialBlocks);
    hipLaunchKernelGGL(k_sum_partial, dim3(blocks), dim3(kBlock), 0, stream, a, stride, n, partials,
                       (size_t)kMaxPartialBlocks);
    launch_final_sum(partials, kMaxPartialBlocks, blocks, 1, mb->words, mb->words, seq, ticket, stream);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

// ---- the sum for callers that cannot allocate ---------------------------------------
//
// fr_sum_noalloc keeps its per-workgroup partial sums in an array that is part of
// the library's image on every GPU instead of in a workspace.  The array's name
// is only a handle on the host: the address kernels can use is asked for once per
// device (hipGetSymbolAddress with that device current) and kept.

static const unsigned kStaticSumBlocks = 1024;
static __device__ __align__(256) uint32_t scratch[kStaticSumBlocks * 8];  // 32 KiB on every GPU the library runs on

static const int kStaticMaxDevices = 64;
static std::mutex g_scratch_mutex;
static uint32_t* g_scratch_ptr[kStaticMaxDevices];  // device address of `scratch`, per device

static int scratch_of_current_device(uint32_t** out) {
    int dev = -1;
    ZK_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticMaxDevices) return ZK_E_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ZK_E_HIP;
        g_scratch_ptr[dev] = (uint32_t*)p;
    }
    *out = g_scratch_ptr[dev];
    return ZK_OK;
}

// Adds up nblocks partial sums (limb-major, stride pstride) and writes the total
// as the canonical integer, eight little-endian words, to out (device memory).
__global__ void __launch_bounds__(kFinalThreads) k_sum_finish_canonical(const uint32_t* __restrict__ partials,
                                                                        size_t pstride, unsigned nblocks,
                                                                        uint32_t* __restrict__ out) {
    __shared__ uint32_t lds[16 * 8];
    Fr acc[1] = {fr_zero()};
    for (unsigned b = threadIdx.x; b < nblocks; b += kFinalThreads) acc[0] = fr_add(acc[0], fr_load(partials, pstride, b));
    block_sum<1, 16>(acc, lds);
    if (threadIdx.x == 0) {
        const Fr c = fr_from_mont(acc[0]);
#pragma unroll
        for (int k = 0; k < 8; ++k) out[k] = c.l[k];
    }
}

// ---- eq tables ----------------------------------------------------------------

struct EqArgs {
    Fr u[32];    // the point, Montgomery
    Fr top[16];  // e~ over the first `ntop` variables, computed on the host
};

// Thread x_lo computes the product over the low nvars-ntop variables once and
// writes one entry per value of the top bits.
__global__ void __launch_bounds__(kBlock) k_eq_table(uint32_t* __restrict__ dst, size_t stride, EqArgs args, int nvars,
                                                     int ntop) {
    const int nlow = nvars - ntop;
    const size_t low_count = (size_t)1 << nlow;
    const Fr one = fr_one();
    for (size_t x = blockIdx.x * (size_t)kBlock + threadIdx.x; x < low_count; x += (size_t)gridDim.x * kBlock) {
        Fr acc = one;
        for (int t = ntop; t < nvars; ++t) {
            unsigned bit = (unsigned)(x >> (nvars - 1 - t)) & 1u;
            Fr f = bit ? args.u[t] : fr_sub(one, args.u[t]);
            acc = (t == ntop) ? f : fr_mul(acc, f);
        }
        for (int hi = 0; hi < (1 << ntop); ++hi) {
            Fr v = nlow ? fr_mul(acc, args.top[hi]) : args.top[hi];
            fr_store(dst, stride, ((size_t)hi << nlow) + x, v);
        }
    }
}

int eq_table_run(uint32_t* dst, size_t stride, const host::F* u, int nvars, hipStream_t stream) {
    if (nvars < 0 || nvars > 31) return ZK_E_BADARG;
    EqArgs args;
    int ntop = nvars < 4 ? nvars : 4;
    host::F top[16];
    top[0] = host::one();
    for (int t = 0; t < ntop; ++t) {
        // append variable t below the ones already in the table
        for (int x = (1 << t) - 1; x >= 0; --x) {
            host::F hi = host::mul(top[x], u[t]);
            top[2 * x + 1] = hi;
            top[2 * x] = host::sub(top[x], hi);
        }
    }
    for (int i = 0; i < 16; ++i) args.top[i] = to_dev(i < (1 << ntop) ? top[i] : host::zero());
    for (int t = 0; t < 32; ++t) args.u[t] = to_dev(t < nvars ? u[t] : host::zero());
    size_t low_count = (size_t)1 << (nvars - ntop);
    hipLaunchKernelGGL(k_eq_table, dim3(grid_for(low_count)), dim3(kBlock), 0, stream, dst, stride, args, nvars, ntop);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

// ---- copy / fold / evaluation ----------------------------------------------------

__global__ void __launch_bounds__(kBlock) k_copy(uint32_t* __restrict__ dst, size_t ds,
                                                 const uint32_t* __restrict__ src, size_t ss, size_t n) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
#pragma unroll
        for (int k = 0; k < 8; ++k) dst[k * ds + i] = src[k * ss + i];
    }
}

void launch_copy(uint32_t* dst, size_t ds, const uint32_t* src, size_t ss, size_t n, hipStream_t stream) {
    if (n == 0) return;
    hipLaunchKernelGGL(k_copy, dim3(grid_for(n)), dim3(kBlock), 0, stream, dst, ds, src, ss, n);
}

__global__ void __launch_bounds__(kBlock) k_fold(uint32_t* dst, size_t ds, const uint32_t* src, size_t ss, size_t half,
                                                 Fr r) {
    for (size_t p = blockIdx.x * (size_t)kBlock + threadIdx.x; p < half; p += (size_t)gridDim.x * kBlock) {
        Fr a0 = fr_load(src, ss, p), a1 = fr_load(src, ss, p + half);
        fr_store(dst, ds, p, fr_fold(a0, a1, r));
    }
}

void launch_fold(uint32_t* dst, size_t ds, const uint32_t* src, size_t ss, size_t half, const host::F& r,
                 hipStream_t stream) {
    if (half == 0) return;
    hipLaunchKernelGGL(k_fold, dim3(grid_for(half)), dim3(kBlock), 0, stream, dst, ds, src, ss, half, to_dev(r));
}

__global__ void k_emit(const uint32_t* __restrict__ a, size_t stride, size_t index, uint32_t* words, uint32_t seq) {
    if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) words[k] = a[k * stride + index];
        mailbox_written();
        mailbox_publish(words, seq);
    }
}

size_t mle_scratch_bytes(int nvars) {
    Carver cv(nullptr, 0);
    if (nvars >= 1) cv.limbs((size_t)1 << (nvars - 1));
    return cv.used();
}

int mle_eval_run(const uint32_t* a, size_t stride, int nvars, const host::F* point, Carver& cv, Mailbox* mb,
                 uint32_t seq, hipStream_t stream) {
    if (nvars == 0) {
        hipLaunchKernelGGL(k_emit, dim3(1), dim3(64), 0, stream, a, stride, (size_t)0, mb->words, seq);
        ZK_HIP_TRY(hipGetLastError());
        return ZK_OK;
    }
    size_t half = (size_t)1 << (nvars - 1);
    uint32_t* buf = cv.limbs(half);
    if (!buf) return ZK_E_BUFSZ;
    launch_fold(buf, half, a, stride, half, point[0], stream);
    for (int t = 1; t < nvars; ++t) {
        half >>= 1;
        launch_fold(buf, (size_t)1 << (nvars - 1), buf, (size_t)1 << (nvars - 1), half, point[t], stream);
    }
    hipLaunchKernelGGL(k_emit, dim3(1), dim3(64), 0, stream, buf, (size_t)1 << (nvars - 1), (size_t)0, mb->words, seq);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

}  // namespace zkmi

using namespace zkmi;

extern "C" {

size_t fr_sum_workspace_bytes(size_t n) { return sum_scratch_bytes(n); }

int fr_sum(fr_t* out, fr_vec a, void* ws, size_t ws_bytes, void* stream) {
    if (!out || (a.n && !vec_ok(a, a.n))) return ZK_E_BADARG;
    if (a.n == 0) {
        memset(out, 0, sizeof *out);
        return ZK_OK;
    }
    if (!ws || ws_bytes < sum_scratch_bytes(a.n)) return ZK_E_BUFSZ;
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(ws, ws_bytes);
    uint32_t seq = mb->next_seq();
    ZK_TRY(sum_run(a.limbs, a.stride, a.n, cv, mb, seq, as_stream(stream)));
    ZK_TRY(mailbox_wait(mb, seq, as_stream(stream)));
    ZK_HIP_TRY(hipStreamSynchronize(as_stream(stream)));
    *out = host::to_canonical(from_dev(mb->words));
    return ZK_OK;
}

int fr_sum_noalloc(uint32_t* out, fr_vec a, void* stream) {
    if (!out || a.n > FR_SUM_NOALLOC_MAX || (a.n && !vec_ok(a, a.n))) return ZK_E_BADARG;
    uint32_t* partials = nullptr;
    ZK_TRY(scratch_of_current_device(&partials));
    // every workgroup writes its partial sum before the closing kernel reads exactly
    // that many: nothing in the array has to start at zero
    unsigned blocks = 0;
    if (a.n) {
        blocks = grid_for(a.n, kBlock * 8, kStaticSumBlocks);
        hipLaunchKernelGGL(k_sum_partial, dim3(blocks), dim3(kBlock), 0, as_stream(stream), a.limbs, a.stride, a.n, partials,
                           (size_t)kStaticSumBlocks);
    }
    hipLaunchKernelGGL(k_sum_finish_canonical, dim3(1), dim3(kFinalThreads), 0, as_stream(stream), partials,
                       (size_t)kStaticSumBlocks, blocks, out);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

int fr_eq_table(fr_vec dst, const fr_t* u, int nvars, void* stream) {
    if (nvars < 0 || nvars > 31 || (nvars && !u) || !vec_ok(dst, (size_t)1 << nvars)) return ZK_E_BADARG;
    host::F um[32];
    for (int t = 0; t < nvars; ++t) {
        if (!host::canonical_in_range(u[t])) return ZK_E_BADARG;
        um[t] = host::from_canonical(u[t]);
    }
    return eq_table_run(dst.limbs, dst.stride, um, nvars, as_stream(stream));
}

size_t fr_mle_eval_workspace_bytes(int nvars) { return mle_scratch_bytes(nvars); }

int fr_mle_eval(fr_t* out, fr_vec a, const fr_t* point, int nvars, void* ws, size_t ws_bytes, void* stream) {
    if (!out || nvars < 0 || nvars > 31 || (nvars && !point) || !vec_ok(a, (size_t)1 << nvars)) return ZK_E_BADARG;
    if (nvars && (!ws || ws_bytes < mle_scratch_bytes(nvars))) return ZK_E_BUFSZ;
    host::F pm[32];
    for (int t = 0; t < nvars; ++t) {
        if (!host::canonical_in_range(point[t])) return ZK_E_BADARG;
        pm[t] = host::from_canonical(point[t]);
    }
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    Carver cv(ws, ws_bytes);
    uint32_t seq = mb->next_seq();
    ZK_TRY(mle_eval_run(a.limbs, a.stride, nvars, pm, cv, mb, seq, as_stream(stream)));
    ZK_TRY(mailbox_wait(mb, seq, as_stream(stream)));
    ZK_HIP_TRY(hipStreamSynchronize(as_stream(stream)));
    *out = host::to_canonical(from_dev(mb->words));
    return ZK_OK;
}

}  // extern "C"
