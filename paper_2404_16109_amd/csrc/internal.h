// Launchers shared between the translation units of the library.
#pragma once
#include "common.h"
#include "small_dev.h"

namespace zkmi {

// ---- batch inversion ------------------------------------------------------
// dst_i = 1 / (src_i + shift) for i < n (shift in Montgomery form; pass zero for
// a plain inverse).  dst must not overlap src.  Scratch comes from `cv`.
// Synchronises the stream once (the single field inversion is done on the host).
size_t batch_inverse_scratch_bytes(size_t n);
int batch_inverse_run(uint32_t* dst, size_t dst_stride, const uint32_t* src, size_t src_stride, size_t n,
                      const host::F& shift, Carver& cv, Mailbox* mb, hipStream_t stream);

// The same in two halves, so that several inversions can share one wait:
// `begin` runs the down passes and leaves the grand total (Montgomery limbs) at
// total_words, publishing `seq` if it is not zero; `end` takes the inverse of
// that total and runs the up passes.
struct BatchInverseJob {
    struct Level {
        const uint32_t* x;
        size_t xs;
        uint32_t* p;
        size_t ps;
        size_t n;
        int shifted;
    };
    Level lv[16];
    int depth = 0;
    Fr shift;
    // a second vector inverted together with the first (its elements follow the first's)
    size_t n2 = 0;
    const uint32_t* src2 = nullptr;
    size_t src2_stride = 0;
    uint32_t* dst2 = nullptr;
    size_t dst2_stride = 0;
    SmallSource small;  // small.x not null: the first vector's entries are these integers, not src
};
// src2 (n2 elements, may be none: n2 = 0) is inverted into dst2 by the same passes,
// shifted like src; needs batch_inverse_can_join(n) and scratch for n + n2 elements.
// small (may be null): src is ignored and the n entries are small integers (small_dev.h).
bool batch_inverse_can_join(size_t n);
int batch_inverse_begin(BatchInverseJob& job, uint32_t* dst, size_t dst_stride, const uint32_t* src, size_t src_stride,
                        size_t n, const host::F& shift, Carver& cv, uint32_t* total_words, uint32_t* flag_words,
                        uint32_t seq, hipStream_t stream, uint32_t* dst2, size_t dst2_stride, const uint32_t* src2,
                        size_t src2_stride, size_t n2, const SmallSource* small = nullptr);
int batch_inverse_end(const BatchInverseJob& job, const host::F& inv_total, hipStream_t stream);

// ---- sums -----------------------------------------------------------------
// Partial sums buffer for reductions: up to kMaxPartialBlocks blocks.
static const unsigned kMaxPartialBlocks = 4096;

// Adds up `nv` interleaved per-block partial values (block b, value q at
// element b*nv + q of `partials`, limb-major with stride pstride) and writes
// the nv totals, Montgomery limbs, to out_words (device-visible host memory
// or device memory): value q at out_words[8q .. 8q+8).
// `words` is the mailbox the flag lives in; seq != 0 publishes completion, for
// which `ticket` (one zeroed word of device memory, left zero) is needed.
void launch_final_sum(const uint32_t* partials, size_t pstride, unsigned nblocks, int nv, uint32_t* out_words,
                      uint32_t* words, uint32_t seq, uint32_t* ticket, hipStream_t stream);

// Same for two partial arrays at once: nv1 values per block from the first, then
// nv2 from the second (nv2 may be 0); totals at out_words[8q..], first array first.
void launch_final_sum2(const uint32_t* part1, size_t pstride1, int nv1, const uint32_t* part2, size_t pstride2, int nv2,
                       unsigned nblocks, uint32_t* out_words, uint32_t* words, uint32_t seq, uint32_t* ticket,
                       hipStream_t stream);

// sum_i a_i into mailbox words [0, 8).
size_t sum_scratch_bytes(size_t n);
int sum_run(const uint32_t* a, size_t stride, size_t n, Carver& cv, Mailbox* mb, uint32_t seq, hipStream_t stream);

// ---- eq tables --------------------------------------------------------------
// dst_x = prod_{t < nvars} (u_t x_t + (1-u_t)(1-x_t)), x in {0,1}^nvars, first
// variable = top bit.  u: host, Montgomery.
int eq_table_run(uint32_t* dst, size_t stride, const host::F* u, int nvars, hipStream_t stream);

// ---- multilinear evaluation ---------------------------------------------------
// a~(point) into out_words[0, 8) (Montgomery); a is not modified.
size_t mle_scratch_bytes(int nvars);
int mle_eval_run(const uint32_t* a, size_t stride, int nvars, const host::F* point, Carver& cv, Mailbox* mb,
                 uint32_t seq, hipStream_t stream);

// p[0..n) = v (a kernel, so that it can sit in a captured graph).
void launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t stream);

// Copies the leading `n` elements of a limb-major vector.
void launch_copy(uint32_t* dst, size_t ds, const uint32_t* src, size_t ss, size_t n, hipStream_t stream);

// One folding pass: dst_p = src_p + r (src_{p+half} - src_p), p < half.
void launch_fold(uint32_t* dst, size_t ds, const uint32_t* src, size_t ss, size_t half, const host::F& r,
                 hipStream_t stream);

// ---- product sumcheck rounds (shared by sumcheck_prove_product and matmul) ----
// Runs d rounds over a, b (2^d elements each, folded in place), writing 3 values
// per round and the two final values to `out` (canonical bytes) and driving the
// transcript.  Needs product_rounds_scratch_bytes(n) of scratch.
}  // namespace zkmi
