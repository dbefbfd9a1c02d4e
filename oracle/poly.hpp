// CPU oracle -- TEST INFRASTRUCTURE, not the product.
//
// Tensors as functions on the Boolean cube and their multilinear extensions
// (Section 3.3).  Conventions (the paper fixes PyTorch-style flattening and
// 0-based indices in Section 3.1; the bit order is this build's reading):
//
//   * a tensor of 2^n entries is indexed by x = sum_t b_t 2^t;
//   * a point is written (w_0, ..., w_{n-1}) and w_0 belongs to the MOST
//     significant bit b_{n-1}, so "i (+) j" with j in [N] is x = i*N + j and
//     u_[h:] are the coordinates of the low bits;
//   * e~(u, x) = prod_t ( u_t x_t + (1-u_t)(1-x_t) ).  Section 3.3 prints a
//     sum sign there; only the product restricts to the equality indicator on
//     bits, which the same sentence requires, so the product is implemented.
#pragma once
#include <algorithm>
#include <functional>
#include <thread>
#include <vector>

#include "fr.hpp"

namespace oracle {

// Runs fn(lo, hi, worker) over a partition of [0, n) on up to `threads` threads.
inline void parallel_ranges(size_t n, int threads,
                            const std::function<void(size_t, size_t, int)>& fn) {
    if (threads < 1) threads = 1;
    if ((size_t)threads > n) threads = n ? (int)n : 1;
    if (threads == 1) {
        fn(0, n, 0);
        return;
    }
    std::vector<std::thread> pool;
    size_t chunk = (n + threads - 1) / threads;
    for (int w = 0; w < threads; ++w) {
        size_t lo = std::min(n, (size_t)w * chunk), hi = std::min(n, lo + chunk);
        pool.emplace_back([=, &fn] { fn(lo, hi, w); });
    }
    for (auto& th : pool) th.join();
}

inline int log2_exact(uint64_t v) {  // -1 unless v is a power of two
    if (v == 0 || (v & (v - 1))) return -1;
    int n = 0;
    while ((v >> n) != 1) ++n;
    return n;
}

// One factor of e~: u*b + (1-u)*(1-b) for a bit b.
inline Fr eq_factor_bit(const Fr& u, unsigned b) { return b ? u : fr_sub(fr_one(), u); }

// e~(u, x) for an index x of nvars bits, straight from the product formula.
inline Fr eq_at_index(const Fr* u, int nvars, uint64_t x) {
    Fr acc = fr_one();
    for (int t = 0; t < nvars; ++t) acc = fr_mul(acc, eq_factor_bit(u[t], (x >> (nvars - 1 - t)) & 1));
    return acc;
}

// e~(u, v) for two field points.
inline Fr eq_at_point(const Fr* u, const Fr* v, int nvars) {
    Fr acc = fr_one();
    for (int t = 0; t < nvars; ++t) {
        Fr both = fr_mul(u[t], v[t]);
        Fr neither = fr_mul(fr_sub(fr_one(), u[t]), fr_sub(fr_one(), v[t]));
        acc = fr_mul(acc, fr_add(both, neither));
    }
    return acc;
}

inline std::vector<Fr> eq_table(const Fr* u, int nvars, int threads) {
    size_t n = (size_t)1 << nvars;
    std::vector<Fr> e(n);
    parallel_ranges(n, threads, [&](size_t lo, size_t hi, int) {
        for (size_t x = lo; x < hi; ++x) e[x] = eq_at_index(u, nvars, x);
    });
    return e;
}

// S~(point) = sum_x e~(point, x) S_x, the definition in Section 3.3.
inline Fr mle_eval(const Fr* s, int nvars, const Fr* point, int threads) {
    size_t n = (size_t)1 << nvars;
    int workers = std::max(1, threads);
    std::vector<Fr> partial(workers, fr_zero());
    parallel_ranges(n, workers, [&](size_t lo, size_t hi, int w) {
        Fr acc = fr_zero();
        for (size_t x = lo; x < hi; ++x) acc = fr_add(acc, fr_mul(eq_at_index(point, nvars, x), s[x]));
        partial[w] = acc;
    });
    Fr total = fr_zero();
    for (const Fr& p : partial) total = fr_add(total, p);
    return total;
}

// Value at `at` of the polynomial of degree <= npts-1 that takes y[j] at X = j,
// by the Lagrange formula.
inline Fr lagrange_eval(const Fr* y, int npts, const Fr& at) {
    Fr total = fr_zero();
    for (int j = 0; j < npts; ++j) {
        Fr num = fr_one(), den = fr_one();
        for (int m = 0; m < npts; ++m) {
            if (m == j) continue;
            num = fr_mul(num, fr_sub(at, fr_from_u64(m)));
            den = fr_mul(den, fr_sub(fr_from_u64(j), fr_from_u64(m)));
        }
        total = fr_add(total, fr_mul(y[j], fr_mul(num, fr_inv(den))));
    }
    return total;
}

// a(r, .) = a0 + r (a1 - a0), binding the current first variable (top bit):
// entries p and p + half of `a` (length 2*half) merge into entry p.
inline void fold_top(std::vector<Fr>& a, const Fr& r, int threads) {
    size_t half = a.size() / 2;
    parallel_ranges(half, threads, [&](size_t lo, size_t hi, int) {
        for (size_t p = lo; p < hi; ++p) a[p] = fr_add(a[p], fr_mul(r, fr_sub(a[p + half], a[p])));
    });
    a.resize(half);
}

}  // namespace oracle
