// Shared host-side plumbing of the library: error handling, argument checks,
// workspace carving and the pinned "mailbox" through which kernels hand small
// results (sums, round values, flags) to the host.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/zkmi.h"
#include "fr_dev.h"
#include "host_fr.h"

#define ZK_HIP_TRY(expr)                         \
    do {                                         \
        if ((expr) != hipSuccess) return ZK_E_HIP; \
    } while (0)

#define ZK_TRY(expr)              \
    do {                          \
        int zk_rc_ = (expr);      \
        if (zk_rc_ != ZK_OK) return zk_rc_; \
    } while (0)

namespace zkmi {

static const int kBlock = 256;  // threads per workgroup: four wavefronts

inline bool vec_ok(const fr_vec& v, size_t n) { return v.limbs != nullptr && v.n >= n && v.stride >= v.n; }
inline bool is_pow2(size_t v) { return v != 0 && (v & (v - 1)) == 0; }
inline int log2_floor(size_t v) {
    int n = 0;
    while ((v >> n) > 1) ++n;
    return n;
}
inline int log2_ceil(size_t v) {
    int n = 0;
    while (((size_t)1 << n) < v) ++n;
    return n;
}
inline size_t div_up(size_t a, size_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t a, size_t b) { return div_up(a, b) * b; }

// Bump allocator over the caller's workspace; every block is 256-byte aligned.
// With base == nullptr it only measures.
class Carver {
public:
    Carver(void* base, size_t bytes) : base_((uint8_t*)base), cap_(bytes), used_(0) {
        // the caller's pointer need not be aligned
        size_t mis = (size_t)((uintptr_t)base_ & 255);
        if (base_ && mis) used_ = 256 - mis;
    }
    void* take(size_t bytes) {
        size_t off = used_;
        used_ = align_up(used_ + bytes, 256);
        if (!base_) return nullptr;
        if (used_ > cap_) return nullptr;
        return base_ + off;
    }
    uint32_t* limbs(size_t n_elements) { return (uint32_t*)take(n_elements * 32); }
    size_t used() const { return used_ + 256; }  // slack for an unaligned base
    bool overflow() const { return base_ != nullptr && used_ > cap_; }

private:
    uint8_t* base_;
    size_t cap_, used_;
};

// Pinned, device-visible host memory, one per host thread, allocated on first
// use and kept: kernels write small results into it directly and the host reads
// them after synchronising the stream.
//
// Completion is signalled through the mailbox too: the kernel that writes the
// last result of a step stores a sequence number into the flag word after a
// system-scope fence, and the host spins on that word.  This hands a round's
// sums to the host a few microseconds after they are computed instead of after
// the stream's completion signal has made its way through the runtime.
struct Mailbox {
    uint32_t* words = nullptr;  // kMailboxWords uint32_t
    uint8_t* bulk = nullptr;    // staging for larger copies (leaf digests)
    size_t bulk_bytes = 0;
    uint32_t seq = 0;           // last sequence number handed out
    uint32_t next_seq() {
        seq = seq == 0xfffffffeu ? 1 : seq + 1;
        return seq;
    }
    // The other direction: a kernel that stays resident over several sumcheck
    // rounds reads each round's challenge from here.  Word 0 is the sequence
    // number of the challenge in words 1..8 (the host writes it last); kCmdAbort
    // tells a waiting kernel to give up.
    uint32_t* cmd = nullptr;    // kCmdWords uint32_t, coherent pinned memory
    uint32_t cmd_seq = 0;
    uint32_t next_cmd_seq() {
        cmd_seq = cmd_seq >= 0xfffffff0u ? 1 : cmd_seq + 1;
        return cmd_seq;
    }
};
static const size_t kCmdWords = 16;
static const uint32_t kCmdAbort = 0xffffffffu;

// Host side of the command channel: the challenge, then (release) its number.
inline void mailbox_send_challenge(Mailbox* mb, uint32_t seq, const uint32_t limbs[8]) {
    volatile uint32_t* c = mb->cmd;
    for (int k = 0; k < 8; ++k) c[1 + k] = limbs[k];
    __atomic_store_n(&mb->cmd[0], seq, __ATOMIC_RELEASE);
}
inline void mailbox_send_abort(Mailbox* mb) { __atomic_store_n(&mb->cmd[0], kCmdAbort, __ATOMIC_RELEASE); }
// Before a resident kernel is launched: an abort left behind by an earlier call
// that ended early must not reach it.  (No kernel of this thread's is listening
// then: a call that aborts waits for its stream before it returns.)
inline void mailbox_channel_reset(Mailbox* mb) { __atomic_store_n(&mb->cmd[0], 0u, __ATOMIC_RELEASE); }

// Ends a resident kernel that is still waiting when the host leaves early.
struct TailGuard {
    Mailbox* mb;
    hipStream_t stream;
    bool armed = false;
    ~TailGuard() {
        if (!armed) return;
        mailbox_send_abort(mb);
        (void)hipStreamSynchronize(stream);
    }
};

// How many times a resident kernel polls for a challenge before it gives up
// (every poll crosses PCIe, about a microsecond): bounded so that a kernel can
// never outlive a host that has stopped talking to it by more than a fraction
// of a second.
uint32_t device_spin_limit();
static const size_t kMailboxFlag = 2040;    // the flag word
// Behind the result words: the arrays a single proof hands to the host once they are short enough for the host to
// finish the sumcheck by itself (five arrays of at most kMailboxShipEntries elements, eight words each).
static const size_t kMailboxShip = 2048;
static const size_t kMailboxShipEntries = 64;
static const size_t kMailboxWords = kMailboxShip + 5 * kMailboxShipEntries * 8;
// A tlookup instance's round sums (eleven values) and final claims start at
// kMailboxSlot * instance; up to eight instances share the mailbox.
static const size_t kMailboxSlot = 96;
static const size_t kMailboxMaxInstances = 8;
static const size_t kMailboxInvB = 1024;    // grand total of the table-side inversion (+16 per instance)
static const size_t kMailboxInvA = 1032;    // grand total of the data-side inversion (+16 per instance)
static const size_t kMailboxTableC = 1280;  // the two table-side constants (+16 per instance)
static const size_t kMailboxDigest = 1536;  // digests of A and B, eight hash-state words each (+16 per instance)

int mailbox_get(Mailbox** out);
int mailbox_bulk(Mailbox* mb, size_t bytes);
// Waits until the flag shows `seq` (spinning, then falling back to
// synchronising the stream).
int mailbox_wait(Mailbox* mb, uint32_t seq, hipStream_t stream);

inline hipStream_t as_stream(void* s) { return (hipStream_t)s; }

// Optional timing of phases with HIP events on the caller's stream (see
// zkmi_profile_* in the public header).  A scope records one start/stop pair.
enum ProfilePhase { kProfTotal = 0, kProfCount, kProfInverse, kProfRoundData, kProfRoundTable, kProfRound29, kProfDigest, kProfRoundSmall, kProfPhases };
int profile_open(int phase, hipStream_t stream);   // returns a record handle or -1 when profiling is off
void profile_close(int handle, hipStream_t stream);
struct ProfileScope {
    ProfileScope(int phase, hipStream_t stream) : stream_(stream), handle_(profile_open(phase, stream)) {}
    ~ProfileScope() { profile_close(handle_, stream_); }
    hipStream_t stream_;
    int handle_;
};

// Montgomery scalar as a kernel argument.
inline Fr to_dev(const host::F& a) {
    Fr o;
    host::to_device_limbs(o.l, a);
    return o;
}
inline host::F from_dev(const uint32_t limbs[8]) { return host::from_device_limbs(limbs); }

// Device side of the completion protocol.  Every thread that writes result words
// calls mailbox_written() after its stores; one thread calls mailbox_publish()
// once all writers are known to be done (same thread, or after a barrier).
__device__ __forceinline__ void mailbox_written() { __threadfence_system(); }
__device__ __forceinline__ void mailbox_publish(uint32_t* words, uint32_t seq) {
    if (seq == 0) return;
    __threadfence_system();
    __hip_atomic_store(&words[kMailboxFlag], seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Device side of the command channel, for one thread: waits until the host has
// published challenge number `want` and reads it.  False on abort or when the
// bound on polls is reached; the caller then winds the kernel down.
__device__ __forceinline__ bool mailbox_receive_challenge(const uint32_t* cmd, uint32_t want, uint32_t spin_limit,
                                                          uint32_t (&limbs)[8]) {
    uint32_t polls = 0;
    for (;;) {
        uint32_t v = __hip_atomic_load(&cmd[0], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
        if (v == want) break;
        if (v == kCmdAbort || ++polls >= spin_limit) return false;
        __builtin_amdgcn_s_sleep(4);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) limbs[k] = __hip_atomic_load(&cmd[1 + k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    return true;
}

// Launch geometry for an elementwise pass over n items.
inline unsigned grid_for(size_t n, size_t per_block = kBlock, size_t max_blocks = (size_t)1 << 20) {
    size_t g = div_up(n, per_block);
    if (g > max_blocks) g = max_blocks;
    if (g == 0) g = 1;
    return (unsigned)g;
}

}  // namespace zkmi
