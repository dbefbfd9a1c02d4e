// Elementwise field kernels and their C entry points: embedding of integers,
// conversions between canonical and Montgomery limb-major form, add/sub/mul and
// the scalar variants.
#include <string.h>

#include <atomic>
#include <chrono>
#include <thread>
#include <vector>

#include "common.h"
#include "transcript.h"

namespace zkmi {

static thread_local Mailbox t_mailbox;  // this host thread's pinned state

int mailbox_get(Mailbox** out) {
    Mailbox& mb = t_mailbox;
    if (!mb.words) {
        void* p = nullptr;
        ZK_HIP_TRY(hipHostMalloc(&p, kMailboxWords * sizeof(uint32_t), hipHostMallocDefault));
        mb.words = (uint32_t*)p;
        memset(mb.words, 0, kMailboxWords * sizeof(uint32_t));
        void* q = nullptr;
        ZK_HIP_TRY(hipHostMalloc(&q, kCmdWords * sizeof(uint32_t), hipHostMallocCoherent));
        mb.cmd = (uint32_t*)q;
        memset(mb.cmd, 0, kCmdWords * sizeof(uint32_t));
    }
    *out = &mb;
    return ZK_OK;
}

static std::atomic<uint32_t> g_spin_limit{1u << 20};  // about two seconds
uint32_t device_spin_limit() { return g_spin_limit.load(); }

int mailbox_wait(Mailbox* mb, uint32_t seq, hipStream_t stream) {
    volatile uint32_t* flag = mb->words + kMailboxFlag;
    // About 20 ms of pure spinning covers every kernel of the library at its usual
    // sizes.  Beyond that the flag is still what is waited for, but the stream is
    // asked now and then whether it has run dry or failed: a stream that has
    // finished without the flag showing means the kernel that should have set it
    // is gone.  The stream is never blocked on: a resident kernel may be waiting,
    // inside that stream, for the very answer this wait stands before.
    const auto start = std::chrono::steady_clock::now();
    bool patient = false;
    for (;;) {
        for (int spin = 0; spin < 2048; ++spin) {
            if (*flag == seq) {
                std::atomic_thread_fence(std::memory_order_acquire);
                return ZK_OK;
            }
            __builtin_ia32_pause();
        }
        if (!patient && std::chrono::steady_clock::now() - start > std::chrono::milliseconds(20)) patient = true;
        if (patient) {
            const hipError_t q = hipStreamQuery(stream);
            if (q == hipSuccess) {
                std::atomic_thread_fence(std::memory_order_acquire);
                return *flag == seq ? ZK_OK : ZK_E_HIP;
            }
            if (q != hipErrorNotReady) return ZK_E_HIP;
            std::this_thread::yield();
        }
    }
}

int mailbox_bulk(Mailbox* mb, size_t bytes) {
    if (mb->bulk_bytes >= bytes) return ZK_OK;
    if (mb->bulk) (void)hipHostFree(mb->bulk);
    mb->bulk = nullptr;
    mb->bulk_bytes = 0;
    void* p = nullptr;
    size_t want = align_up(bytes, 1 << 16);
    ZK_HIP_TRY(hipHostMalloc(&p, want, hipHostMallocDefault));
    mb->bulk = (uint8_t*)p;
    mb->bulk_bytes = want;
    return ZK_OK;
}

// ---- phase timing ----------------------------------------------------------------------

namespace {
struct ProfileRecord {
    int phase;
    hipEvent_t start, stop;
};
struct ProfileState {
    bool on = false;
    std::vector<hipEvent_t> pool;  // events created so far
    size_t used = 0;
    std::vector<ProfileRecord> open_records;
    double ms[kProfPhases] = {0};
    uint64_t count[kProfPhases] = {0};
};
ProfileState& profile_state() {
    static thread_local ProfileState st;
    return st;
}
hipEvent_t profile_event(ProfileState& st) {
    if (st.used == st.pool.size()) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        st.pool.push_back(e);
    }
    return st.pool[st.used++];
}
void profile_resolve(ProfileState& st) {
    for (const ProfileRecord& r : st.open_records) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            st.ms[r.phase] += ms;
            st.count[r.phase] += 1;
        }
    }
    st.open_records.clear();
    st.used = 0;
}
}  // namespace

int profile_open(int phase, hipStream_t stream) {
    ProfileState& st = profile_state();
    if (!st.on) return -1;
    hipEvent_t a = profile_event(st), b = profile_event(st);
    if (!a || !b) return -1;
    if (hipEventRecord(a, stream) != hipSuccess) return -1;
    st.open_records.push_back(ProfileRecord{phase, a, b});
    return (int)st.open_records.size() - 1;
}

void profile_close(int handle, hipStream_t stream) {
    if (handle < 0) return;
    ProfileState& st = profile_state();
    if ((size_t)handle < st.open_records.size()) (void)hipEventRecord(st.open_records[handle].stop, stream);
}

// x >= 0 -> x, x < 0 -> r - |x|, in Montgomery form.
__global__ void __launch_bounds__(kBlock) k_from_i32(uint32_t* __restrict__ dst, size_t stride,
                                                     const int32_t* __restrict__ src, size_t n) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        int32_t x = src[i];
        uint32_t mag = x < 0 ? (0u - (uint32_t)x) : (uint32_t)x;
        Fr m = fr_from_u32(mag);
        if (x < 0) m = fr_neg(m);
        fr_store(dst, stride, i, m);
    }
}

__global__ void __launch_bounds__(kBlock) k_from_canonical(uint32_t* __restrict__ dst, size_t stride,
                                                           const uint32_t* __restrict__ aos, size_t n) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        Fr c;
#pragma unroll
        for (int k = 0; k < 8; ++k) c.l[k] = aos[i * 8 + k];
        fr_store(dst, stride, i, fr_to_mont(c));
    }
}

__global__ void __launch_bounds__(kBlock) k_to_canonical(uint32_t* __restrict__ aos, const uint32_t* __restrict__ src,
                                                         size_t stride, size_t n) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        Fr c = fr_from_mont(fr_load(src, stride, i));
#pragma unroll
        for (int k = 0; k < 8; ++k) aos[i * 8 + k] = c.l[k];
    }
}

enum { OP_ADD = 0, OP_SUB = 1, OP_MUL = 2 };

template <int OP>
__global__ void __launch_bounds__(kBlock) k_binary(uint32_t* dst, size_t ds, const uint32_t* a, size_t as,
                                                   const uint32_t* b, size_t bs, size_t n) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        Fr x = fr_load(a, as, i), y = fr_load(b, bs, i);
        Fr z = OP == OP_ADD ? fr_add(x, y) : OP == OP_SUB ? fr_sub(x, y) : fr_mul(x, y);
        fr_store(dst, ds, i, z);
    }
}

enum { SC_ADD = 0, SC_MUL = 1, SC_AXPY = 2 };

template <int OP>
__global__ void __launch_bounds__(kBlock) k_scalar(uint32_t* dst, size_t ds, const uint32_t* x, size_t xs, Fr s,
                                                   const uint32_t* y, size_t ys, size_t n) {
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) {
        Fr a = fr_load(x, xs, i);
        Fr z;
        if (OP == SC_ADD) z = fr_add(a, s);
        else if (OP == SC_MUL) z = fr_mul(a, s);
        else z = fr_add(a, fr_mul(s, fr_load(y, ys, i)));
        fr_store(dst, ds, i, z);
    }
}

template <int OP>
static int launch_binary(fr_vec dst, fr_vec a, fr_vec b, void* stream) {
    size_t n = dst.n;
    if (!vec_ok(dst, n) || !vec_ok(a, n) || !vec_ok(b, n)) return ZK_E_BADARG;
    if (n == 0) return ZK_OK;
    hipLaunchKernelGGL(k_binary<OP>, dim3(grid_for(n)), dim3(kBlock), 0, as_stream(stream), dst.limbs, dst.stride,
                       a.limbs, a.stride, b.limbs, b.stride, n);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

template <int OP>
static int launch_scalar(fr_vec dst, fr_vec x, const fr_t* s, const fr_vec* y, void* stream) {
    size_t n = dst.n;
    if (!s || !vec_ok(dst, n) || !vec_ok(x, n) || (y && !vec_ok(*y, n))) return ZK_E_BADARG;
    if (!host::canonical_in_range(*s)) return ZK_E_BADARG;
    if (n == 0) return ZK_OK;
    Fr sm = to_dev(host::from_canonical(*s));
    hipLaunchKernelGGL(k_scalar<OP>, dim3(grid_for(n)), dim3(kBlock), 0, as_stream(stream), dst.limbs, dst.stride,
                       x.limbs, x.stride, sm, y ? y->limbs : nullptr, y ? y->stride : 0, n);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

}  // namespace zkmi

using namespace zkmi;

extern "C" {

int zkmi_version(void) { return 100; }

int zkmi_sha256(const uint8_t* data, size_t len, uint8_t out[32], int use_sha_instructions) {
    if ((!data && len) || !out) return ZK_E_BADARG;
    bool& flag = host::Sha256::use_sha_instructions();
    const bool available = flag;
    flag = available && use_sha_instructions != 0;
    const int used = flag ? 1 : 0;
    host::Sha256 h;
    h.update(data, len);
    h.finish(out);
    flag = available;
    return used;
}

int zkmi_thread_init(size_t max_table_rows) {
    Mailbox* mb;
    ZK_TRY(mailbox_get(&mb));
    // the staging buffer holds a table's leaf digests (one per 128 rows, 32 bytes each) and two status words
    return mailbox_bulk(mb, div_up(max_table_rows ? max_table_rows : 1, (size_t)128) * 32 + 16);
}

int zkmi_thread_release(void) {
    Mailbox& mb = t_mailbox;
    hipError_t first = hipSuccess;
    void* blocks[3] = {mb.words, mb.cmd, mb.bulk};
    for (void* p : blocks) {
        if (!p) continue;
        const hipError_t e = hipHostFree(p);
        if (first == hipSuccess) first = e;
    }
    mb = Mailbox();
    return first == hipSuccess ? ZK_OK : ZK_E_HIP;
}

int zkmi_profile_enable(int on) {
    profile_state().on = on != 0;
    return ZK_OK;
}

int zkmi_profile_reset(void) {
    ProfileState& st = profile_state();
    profile_resolve(st);
    for (int p = 0; p < kProfPhases; ++p) {
        st.ms[p] = 0;
        st.count[p] = 0;
    }
    return ZK_OK;
}

int zkmi_profile_query(const char* phase, uint64_t* records, double* total_ms) {
    static const char* names[kProfPhases] = {"total", "count", "inverse", "round_data", "round_table", "round_data29", "digest", "round_small"};
    if (!phase || !records || !total_ms) return ZK_E_BADARG;
    ProfileState& st = profile_state();
    profile_resolve(st);
    for (int p = 0; p < kProfPhases; ++p) {
        if (strcmp(phase, names[p]) == 0) {
            *records = st.count[p];
            *total_ms = st.ms[p];
            return ZK_OK;
        }
    }
    return ZK_E_BADARG;
}

int fr_constants(fr_t* modulus, fr_t* mont_r, fr_t* mont_r2, uint32_t* neg_inv32) {
    if (!modulus || !mont_r || !mont_r2 || !neg_inv32) return ZK_E_BADARG;
    const uint32_t r[8] = {ZK_R0, ZK_R1, ZK_R2, ZK_R3, ZK_R4, ZK_R5, ZK_R6, ZK_R7};
    const uint32_t one[8] = {ZK_ONE0, ZK_ONE1, ZK_ONE2, ZK_ONE3, ZK_ONE4, ZK_ONE5, ZK_ONE6, ZK_ONE7};
    const uint32_t rr[8] = {ZK_RR0, ZK_RR1, ZK_RR2, ZK_RR3, ZK_RR4, ZK_RR5, ZK_RR6, ZK_RR7};
    for (int k = 0; k < 8; ++k) {
        modulus->l[k] = r[k];
        mont_r->l[k] = one[k];
        mont_r2->l[k] = rr[k];
    }
    *neg_inv32 = 0xffffffffu;
    // the host glue carries its own copies; they must agree
    for (int k = 0; k < 4; ++k) {
        if (host::kMod[k] != ((uint64_t)r[2 * k] | ((uint64_t)r[2 * k + 1] << 32))) return ZK_E_BADARG;
        if (host::kOne[k] != ((uint64_t)one[2 * k] | ((uint64_t)one[2 * k + 1] << 32))) return ZK_E_BADARG;
        if (host::kRR[k] != ((uint64_t)rr[2 * k] | ((uint64_t)rr[2 * k + 1] << 32))) return ZK_E_BADARG;
    }
    return ZK_OK;
}

int fr_from_i32(fr_vec dst, const int32_t* src, size_t n, void* stream) {
    if (!src || !vec_ok(dst, n)) return ZK_E_BADARG;
    if (n == 0) return ZK_OK;
    hipLaunchKernelGGL(k_from_i32, dim3(grid_for(n)), dim3(kBlock), 0, as_stream(stream), dst.limbs, dst.stride, src, n);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

int fr_from_canonical(fr_vec dst, const uint32_t* aos, size_t n, void* stream) {
    if (!aos || !vec_ok(dst, n)) return ZK_E_BADARG;
    if (n == 0) return ZK_OK;
    hipLaunchKernelGGL(k_from_canonical, dim3(grid_for(n)), dim3(kBlock), 0, as_stream(stream), dst.limbs, dst.stride,
                       aos, n);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

int fr_to_canonical(uint32_t* aos, fr_vec src, size_t n, void* stream) {
    if (!aos || !vec_ok(src, n)) return ZK_E_BADARG;
    if (n == 0) return ZK_OK;
    hipLaunchKernelGGL(k_to_canonical, dim3(grid_for(n)), dim3(kBlock), 0, as_stream(stream), aos, src.limbs,
                       src.stride, n);
    ZK_HIP_TRY(hipGetLastError());
    return ZK_OK;
}

int fr_add(fr_vec dst, fr_vec a, fr_vec b, void* stream) { return launch_binary<OP_ADD>(dst, a, b, stream); }
int fr_sub(fr_vec dst, fr_vec a, fr_vec b, void* stream) { return launch_binary<OP_SUB>(dst, a, b, stream); }
int fr_mul(fr_vec dst, fr_vec a, fr_vec b, void* stream) { return launch_binary<OP_MUL>(dst, a, b, stream); }

int fr_add_scalar(fr_vec dst, fr_vec x, const fr_t* s, void* stream) {
    return launch_scalar<SC_ADD>(dst, x, s, nullptr, stream);
}
int fr_mul_scalar(fr_vec dst, fr_vec x, const fr_t* s, void* stream) {
    return launch_scalar<SC_MUL>(dst, x, s, nullptr, stream);
}
int fr_axpy(fr_vec dst, fr_vec x, const fr_t* s, fr_vec y, void* stream) {
    return launch_scalar<SC_AXPY>(dst, x, s, &y, stream);
}

}  // extern "C"
