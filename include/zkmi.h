/*
 * zkmi -- tlookup / sumcheck prover hot path of zkLLM on one AMD MI355X (gfx950).
 *
 * C boundary of the device library.  Every entry point is plain C: pointers
 * (each comment says host or device), sizes, no C++ or framework types.
 *
 * Field.  All arithmetic is in the BLS12-381 scalar field Fr (the paper's
 * implementation field, Section 7.2), r = z^4 - z^2 + 1, z = -0xd201000000010000.
 *
 * Host scalars   : fr_t, eight 32-bit limbs, least significant first, the
 *                  canonical integer in [0, r).  Not Montgomery form.
 * Device vectors : fr_vec, limb-major structure of arrays in MONTGOMERY form
 *                  (x * 2^256 mod r, always fully reduced): limb k of element i
 *                  is limbs[k * stride + i], stride >= n.  A wavefront reading
 *                  one limb of 64 consecutive elements reads 256 contiguous bytes.
 *
 * Ownership.  The caller owns every buffer: inputs, outputs and workspace.  No
 * entry point allocates device memory; `*_workspace_bytes` says how much
 * workspace a call needs.  The library does keep a little state of its own PER
 * HOST THREAD, allocated by that thread's first call that needs it and kept until
 * the process ends: 18 KiB of pinned host memory into which kernels write the
 * handful of sums a step returns (and, at the end of a single tlookup proof, the
 * five arrays of at most 64 elements from which the host finishes the rounds),
 * 64 bytes of coherent pinned memory through which a kernel that stays resident
 * over several sumcheck rounds receives each round's challenge, a pinned staging buffer for digest leaves that grows to the
 * largest table seen, and the event pool of zkmi_profile_*.  Calls from
 * different host threads share nothing; a thread's calls must not overlap.
 * zkmi_thread_init makes that allocation at a time of the caller's choosing and
 * zkmi_thread_release gives the pinned memory back (both are optional).
 * (fr_sum_noalloc touches none of this.)  Inputs are not modified unless the comment says "in
 * place".  `stream` is a hipStream_t passed as void* (NULL = the null stream);
 * all device work of a call is enqueued on it.  Calls that return host values
 * (proofs, sums, error codes that depend on data) synchronise that stream
 * before returning; the others only enqueue.
 *
 * Errors.  Every function returns ZK_OK or a negative code; nothing is thrown.
 * On error the contents of output buffers are unspecified.
 *
 * Index and variable order (the paper fixes PyTorch flattening and 0-based
 * indices in Section 3.1; the bit order is this library's reading): element x
 * of a vector of 2^n entries has bits x = sum b_t 2^t; a point is written
 * (w_0, ..., w_{n-1}) with w_0 belonging to the TOP bit b_{n-1}.  Sumcheck
 * rounds bind w_0 first.
 *
 * Fiat-Shamir.  The paper's protocols are interactive; here verifier messages
 * come from a SHA-256 transcript:
 *   absorb(tag, data): state <- SHA256(state || tag || LE64(len) || data)
 *   challenge(tag)   : c = (SHA256(state||tag||0x00) || SHA256(state||tag||0x01))
 *                          as a 512-bit big-endian integer, mod r;
 *                      state <- SHA256(state || tag || 0x02)
 * Field elements enter the transcript and the proofs as 32 little-endian bytes
 * of the canonical integer.
 */
#ifndef ZKMI_H
#define ZKMI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ZK_OK = 0,
    ZK_E_BADARG = -1,       /* null pointer, bad size, D or N not a power of two, N > D */
    ZK_E_NOT_IN_TABLE = -2, /* some S_i is not an entry of T */
    ZK_E_ZERO_DENOM = -3,   /* an element to invert is zero (beta + S_i = 0 or beta + T_j = 0) */
    ZK_E_REJECT = -4,       /* verifiers: the proof does not verify; zkattn_link_prove*: the tensors break a relation */
    ZK_E_BUFSZ = -5,        /* proof buffer or workspace too small */
    ZK_E_HIP = -6           /* a HIP runtime call failed */
};

typedef struct {
    uint32_t l[8];
} fr_t;

typedef struct {
    uint32_t* limbs; /* device */
    size_t n;        /* number of elements */
    size_t stride;   /* distance, in uint32_t, between consecutive limb planes */
} fr_vec;

/* ---- field library ------------------------------------------------------- */

/* Constants of the field as the library uses them, for checking against an
 * independent computation: modulus r, 2^256 mod r, 2^512 mod r (canonical
 * limbs) and -r^-1 mod 2^32.  All host pointers. */
int fr_constants(fr_t* modulus, fr_t* mont_r, fr_t* mont_r2, uint32_t* neg_inv32);

/* dst_i = src_i embedded in Fr: x >= 0 is x, x < 0 is r - |x| (fixed-point
 * tensors are "discretized into a finite field", Section 3.3).  src: device. */
int fr_from_i32(fr_vec dst, const int32_t* src, size_t n, void* stream);

/* Conversion between device vectors and canonical array-of-structures form
 * (element i = 8 consecutive little-endian uint32_t, value < r).  aos: device.
 * fr_from_canonical does not check that the input is < r. */
int fr_from_canonical(fr_vec dst, const uint32_t* aos, size_t n, void* stream);
int fr_to_canonical(uint32_t* aos, fr_vec src, size_t n, void* stream);

/* Elementwise dst = a (op) b over dst.n elements; dst may alias a or b. */
int fr_add(fr_vec dst, fr_vec a, fr_vec b, void* stream);
int fr_sub(fr_vec dst, fr_vec a, fr_vec b, void* stream);
int fr_mul(fr_vec dst, fr_vec a, fr_vec b, void* stream);

/* dst = x + s, dst = x * s, dst = x + s * y with a host scalar s.  fr_axpy is
 * the pair-table combination X + rho Y of Section 4 (last paragraph). */
int fr_add_scalar(fr_vec dst, fr_vec x, const fr_t* s, void* stream);
int fr_mul_scalar(fr_vec dst, fr_vec x, const fr_t* s, void* stream);
int fr_axpy(fr_vec dst, fr_vec x, const fr_t* s, fr_vec y, void* stream);

/* dst_i = 1 / src_i for all i (the inverse vectors A and B of Section 4 are
 * this applied to beta + S and beta + T).  One field inversion in total, on the
 * host; everything else is products on the device.  dst must not overlap src.
 * Returns ZK_E_ZERO_DENOM if any src_i is zero.  Synchronises the stream. */
size_t fr_batch_inverse_workspace_bytes(size_t n);
int fr_batch_inverse(fr_vec dst, fr_vec src, void* ws, size_t ws_bytes, void* stream);

/* *out = sum_i a_i (host, canonical).  Synchronises the stream. */
size_t fr_sum_workspace_bytes(size_t n);
int fr_sum(fr_t* out, fr_vec a, void* ws, size_t ws_bytes, void* stream);

/* fr_sum for callers that cannot allocate or wait: code under HIP graph capture,
 * serving loops that must not call hipMalloc, harnesses that forbid it.  Takes
 * no workspace and allocates nothing, on the device or on the host, in any call:
 * the per-workgroup partial sums live in an array of 32 KiB that is part of the
 * library's image on every GPU it runs on (held until the process ends).  It only
 * enqueues two kernels on `stream` and returns; the sum arrives in out (DEVICE
 * memory, 8 uint32_t: the canonical integer, least significant word first) when
 * the stream reaches that point.  a.n may be 0 (the sum is zero) and at most
 * FR_SUM_NOALLOC_MAX, else ZK_E_BADARG.  All calls on one GPU share the one
 * array (nothing in it needs clearing between calls: a call only reads what it
 * has written), so calls that overlap on one GPU, on different streams or from
 * different threads, race; calls on one stream are ordered and safe. */
#define FR_SUM_NOALLOC_MAX ((size_t)1 << 28)
int fr_sum_noalloc(uint32_t* out, fr_vec a, void* stream);

/* dst_x = e~(u, x) = prod_t (u_t x_t + (1-u_t)(1-x_t)) for all x in
 * {0,1}^nvars (Section 3.3; the product, which restricts to the equality
 * indicator on bits).  u: host, nvars elements; dst.n = 2^nvars. */
int fr_eq_table(fr_vec dst, const fr_t* u, int nvars, void* stream);

/* *out = a~(point), the multilinear extension of a (2^nvars elements) at a host
 * point (Section 3.3).  Synchronises the stream. */
size_t fr_mle_eval_workspace_bytes(int nvars);
int fr_mle_eval(fr_t* out, fr_vec a, const fr_t* point, int nvars, void* ws, size_t ws_bytes, void* stream);

/* ---- tlookup (Section 4, Protocol 1) ---------------------------------------- */

/* What the prover also reports, for checks: the challenges and the two sides of
 * the log-derivative identity sum_i A_i = sum_j m_j B_j at beta. */
typedef struct {
    fr_t beta, alpha;
    fr_t sum_A, sum_mB;
    uint64_t bad_index; /* on ZK_E_NOT_IN_TABLE: the smallest i with S_i outside T */
} tlookup_aux;

/* Tensors standing in for the openings of the commitments in tlookup_verify.
 * Any member may be empty (limbs == NULL / m == NULL): that claim is then not
 * checked against its tensor. */
typedef struct {
    fr_vec S;          /* D elements, device */
    fr_vec A;          /* D elements, device */
    fr_vec B;          /* N elements, device */
    const uint32_t* m; /* N counts, device */
} tlookup_witness;

typedef struct {
    fr_t A_v, S_v, B_vp, m_vp, T_vp; /* claimed values at v and v' = v_[log2(D/N):] */
    fr_t v[32];                      /* the sumcheck point, log2 D entries used */
    int nvars;
} tlookup_claims;

/* m_j = |{i : S_i = T_j}| as 32-bit counts (Section 4).  If T has equal entries
 * an S_i is counted at the lowest such j.  idx (device, D entries) may give the
 * table row of every S_i; S_i == T[idx_i] is still checked.  With idx == NULL
 * rows are found through a hash table of T built in the workspace.
 * m: device, N counters, overwritten.  *bad_index (host, may be NULL) receives
 * the smallest offending i on ZK_E_NOT_IN_TABLE.  Synchronises the stream. */
size_t tlookup_workspace_bytes(size_t D, size_t N);
int tlookup_multiplicities(uint32_t* m, fr_vec S, const uint32_t* idx, fr_vec T, void* ws, size_t ws_bytes,
                           uint64_t* bad_index, void* stream);

/* Proof that every element of S (D elements) is an entry of T (N elements);
 * D, N powers of two, N <= D <= 2^31 (Protocol 1, "Require").  Steps: multiplicities,
 * beta, A = 1/(beta+S), B = 1/(beta+T), alpha, u, then the sumcheck of
 *   alpha + alpha^2 = sum_{x = i (+) j} A(x)(alpha e~(u,x)(S(x)+beta) + 1)
 *                     + (N/D) B(j)(alpha^2 e~(u_[h:],j)(T(j)+beta) - m(j)),  h = log2(D/N),
 * round polynomials sent as their values at X = 0,1,2,3, and the five final
 * claims A~(v), S~(v), B~(v'), m~(v'), T~(v').
 *
 * The commitments of Protocol 1 are outside this library; digests stand in for
 * them and enter the transcript where Protocol 1 sends the commitments: `seed`
 * (host, 32 bytes) for those of T and S, digest(m) before beta is drawn, and
 * digest(A), digest(B) after beta and BEFORE alpha and u, so that the sumcheck's
 * randomness depends on the inverse vectors (tlookup-Prove: "P -> V: commitments
 * of A and B", then the sumcheck).
 *
 * Transcript: SHA256("zkmi/tlookup/v2" || seed || LE64 D || LE64 N); absorb("m",
 * digest(m)); beta = challenge("beta"); absorb("A", digest(A)); absorb("B",
 * digest(B)); alpha = challenge("alpha"); u_t = challenge("u"), t = 0..n-1; per
 * round absorb("g", 4 values), r = challenge("r"); absorb("final", 5 claims).
 * digest(m) = SHA256 of the concatenated SHA256 digests of the leaves of 128
 * counts, each count 4 little-endian bytes.  digest of a vector of n field
 * elements (n a power of two): with L = max(1, n/128) leaves, leaf i = SHA256 of
 * the canonical bytes of elements i, i+L, i+2L, ...; rows of digests are then
 * hashed in consecutive groups of four (a last pair as a group of two) until one
 * digest remains.
 *
 * Proof (host buffer, tlookup_proof_bytes(D) bytes):
 *   "ZKTL" | u32 2 | LE64 D | LE64 N | digest(m) | digest(A) | digest(B)
 *   | n x 4 elements | 5 elements.
 * *len (host) receives the size, also on ZK_E_BUFSZ.  aux: host, may be NULL.
 * ws: device, at least tlookup_workspace_bytes(D, N).  Synchronises the stream.
 *
 * S not in T is ZK_E_NOT_IN_TABLE with aux->bad_index the smallest such i, as in
 * tlookup_multiplicities.  With idx given (and D > 256, N <= 2^16) the prover does
 * not compare every S_i with T[idx_i] up front: it counts from idx alone and then
 * applies the identity the protocol itself rests on, sum_i 1/(beta+S_i) =
 * sum_j m_j/(beta+T_j) (Section 4), to the sums it has after the first round;
 * only if they differ are all S_i compared with their rows to find bad_index.  A
 * tensor with S_i != T[idx_i] slips through with probability at most (D+N)/|F|
 * over beta (the identity cleared of its denominators is a polynomial identity of
 * degree below D+N; this is the step the soundness proof of Appendix C takes),
 * and the proof it then yields is one the verifier accepts for the same reason. */
size_t tlookup_proof_bytes(size_t D);
int tlookup_prove(const uint8_t seed[32], fr_vec S, const uint32_t* idx, fr_vec T, uint8_t* proof, size_t cap,
                  size_t* len, tlookup_aux* aux, void* ws, size_t ws_bytes, void* stream);

/* tlookup_prove with every S_i compared with its hinted row T[idx_i] before
 * anything else is done (while counting), as tlookup_multiplicities does, instead
 * of through the identity after the first round: the same proof, byte for byte,
 * for callers who want the membership check to be exact rather than sound up to
 * (D+N)/|F|.  Costs one more pass over S (36 instead of 4 bytes per element while
 * counting); timed beside the headline by the benchmark.  Without idx it is
 * tlookup_prove. */
int tlookup_prove_checked(const uint8_t seed[32], fr_vec S, const uint32_t* idx, fr_vec T, uint8_t* proof, size_t cap,
                          size_t* len, tlookup_aux* aux, void* ws, size_t ws_bytes, void* stream);

/* tlookup_prove from the tensor as the integers it is quantised from:
 * S_i = X_i + rho Y_i for signed 32-bit device arrays X and Y of D entries (the
 * pair-table reduction of Section 4, last paragraph: a function table becomes a
 * set by combining its two columns with a random rho; T is then T_X + rho T_Y as
 * field elements, as for tlookup_prove), or S_i = X_i with Y and rho both NULL (a
 * range check).  rho: host, canonical.  The proof is tlookup_prove's for that S,
 * byte for byte; S is never written out: the inversion and the first round read
 * eight bytes per entry instead of thirty-two and build beta + S_i from them (two
 * 32x256-bit products and a two-step reduction), the first fold takes the four
 * integers of an entry pair straight to a reduced field element.  Row hints idx
 * are required (for a range check idx_i = X_i - min T).  Shapes with N > 2^16,
 * D < 4 N or D <= 1024 have no such path: S is written out first, into D * 32
 * further bytes of workspace (tlookup_small_workspace_bytes accounts for them).
 * Errors as for tlookup_prove. */
size_t tlookup_small_workspace_bytes(size_t D, size_t N);
int tlookup_prove_small(const uint8_t seed[32], const int32_t* X, const int32_t* Y, const fr_t* rho, size_t D,
                        const uint32_t* idx, fr_vec T, uint8_t* proof, size_t cap, size_t* len, tlookup_aux* aux, void* ws,
                        size_t ws_bytes, void* stream);

/* The same proof, byte for byte, for callers that know the table row of every
 * element (idx is required): once S_i = T[idx_i] has been checked, A_i = 1/(beta + S_i)
 * is the table-side inverse B[idx_i], so only the N table entries are inverted and
 * A is gathered from them instead of inverting D elements.  Not what the
 * benchmark's headline times (that is tlookup_prove, with the D-element
 * inversion); reported beside it. */
int tlookup_prove_by_rows(const uint8_t seed[32], fr_vec S, const uint32_t* idx, fr_vec T, uint8_t* proof, size_t cap,
                          size_t* len, tlookup_aux* aux, void* ws, size_t ws_bytes, void* stream);

/* As tlookup_prove with beta replaced by *forced_beta (host) after the
 * transcript has produced its own: the only way to reach the completeness
 * failure of Protocol 1 (beta + S_i = 0, Section 6.3) deliberately.  For tests. */
int tlookup_prove_with_beta(const uint8_t seed[32], fr_vec S, const uint32_t* idx, fr_vec T, const fr_t* forced_beta,
                            uint8_t* proof, size_t cap, size_t* len, tlookup_aux* aux, void* ws, size_t ws_bytes,
                            void* stream);

/* Verifier: replays the transcript, checks g_k(0) + g_k(1) against the running
 * claim in every round and the final identity, recomputes T~(v') from the public
 * table (device), and, for each tensor given in *witness, recomputes that claim
 * from the tensor (standing in for the proofs of evaluation on commitments,
 * which are outside this library) and, for m, A and B, the digest the proof
 * carries for it.  Returns ZK_OK (accept) or ZK_E_REJECT.
 * claims: host, may be NULL.  ws: device, tlookup_verify_workspace_bytes(D, N). */
size_t tlookup_verify_workspace_bytes(size_t D, size_t N);
int tlookup_verify(const uint8_t seed[32], const uint8_t* proof, size_t len, fr_vec T, size_t D,
                   const tlookup_witness* witness, tlookup_claims* claims, void* ws, size_t ws_bytes, void* stream);

/* ---- several tlookup instances under one sumcheck ---------------------------- */

/* The paper proves each lookup of an attention layer on its own (Section 5.2,
 * Protocol 2) and does not describe batching; this is the standard random
 * linear combination applied to Protocol 1.  K instances (S_i, T_i) of one shape
 * (D, N) share beta, alpha, u and all round challenges, and ONE sumcheck runs on
 *   f = sum_i lambda^i f_i,   claim = (sum_i lambda^i)(alpha + alpha^2),
 * f_i being the summand of tlookup_prove for instance i and lambda one more
 * challenge.  It ends in 5 K claims: A_i~(v), S_i~(v), B_i~(v'), m_i~(v'), T_i~(v').
 *
 * Transcript: SHA256("zkmi/tlookup-batch/v2" || seed || LE64 D || LE64 N || LE64 K);
 * absorb("m", digest(m_i)) for i = 0..K-1; beta; absorb("A", digest(A_i)),
 * absorb("B", digest(B_i)) for i = 0..K-1; alpha, u_0..u_{n-1} as in
 * tlookup_prove; lambda = challenge("lambda"); per round absorb("g", 4 values),
 * r = challenge("r"); absorb("final", 5 K claims).
 *
 * Proof (host, tlookup_batch_proof_bytes(D, K) bytes):
 *   "ZKTB" | u32 2 | LE64 D | LE64 N | LE64 K | K x digest(m_i)
 *   | K x [digest(A_i) digest(B_i)] | n x 4 elements | K x 5 elements. */
#define TLOOKUP_BATCH_MAX 8

typedef struct {
    fr_t beta, alpha, lambda;
    fr_t sum_A[TLOOKUP_BATCH_MAX], sum_mB[TLOOKUP_BATCH_MAX]; /* per instance, as in tlookup_aux */
    uint64_t bad_instance, bad_index; /* on ZK_E_NOT_IN_TABLE: first offending instance, smallest i in it */
} tlookup_batch_aux;

typedef struct {
    fr_t value[TLOOKUP_BATCH_MAX][5]; /* per instance: A~(v), S~(v), B~(v'), m~(v'), T~(v') */
    fr_t v[32];
    fr_t lambda;
    int nvars, count;
} tlookup_batch_claims;

/* S, T: host arrays of K descriptors of device vectors (all S_i of D elements,
 * all T_i of N).  idx: NULL, or a host array of K device pointers, each NULL or
 * the rows of that instance as in tlookup_multiplicities.  1 <= K <=
 * TLOOKUP_BATCH_MAX.  ws: device, tlookup_batch_workspace_bytes(D, N, K) (K times
 * the single-instance buffers; the weight tables are shared).  Other arguments
 * and error behaviour as tlookup_prove.  Synchronises the stream. */
size_t tlookup_batch_proof_bytes(size_t D, size_t K);
size_t tlookup_batch_workspace_bytes(size_t D, size_t N, size_t K);
int tlookup_prove_batch(const uint8_t seed[32], const fr_vec* S, const uint32_t* const* idx, const fr_vec* T, size_t K,
                        uint8_t* proof, size_t cap, size_t* len, tlookup_batch_aux* aux, void* ws, size_t ws_bytes,
                        void* stream);

/* Verifier of the batched proof.  witness: NULL or a host array of K entries
 * (members may be empty, as in tlookup_verify).  ws: device,
 * tlookup_verify_workspace_bytes(D, N). */
int tlookup_verify_batch(const uint8_t seed[32], const uint8_t* proof, size_t len, const fr_vec* T, size_t K, size_t D,
                         const tlookup_witness* witness, tlookup_batch_claims* claims, void* ws, size_t ws_bytes,
                         void* stream);

/* ---- lookups of different shapes under one sumcheck ---------------------------- */

/* Some layers look one tensor up in two tables in a row whose lengths differ, and
 * the tensors' lengths with them (LayerNorm, Section 6.1.3: first the scaling
 * down of the per-row statistic, then the table of 1/sqrt).  The paper proves
 * such lookups one by one, which ends them at unrelated points; here K instances
 * (S_i, T_i) of ANY shapes (D_i, N_i) run under ONE sumcheck, so that all 5 K
 * claims are at (suffixes of) one point.  With n_i = log2 D_i, n = max_i n_i and
 * skip_i = n - n_i, instance i lives on the LAST n_i of the n variables and its
 * summand does not depend on the first skip_i:
 *   f(x) = sum_i lambda^i 2^-skip_i f_i(x_[skip_i:]),   claim = (sum_i lambda^i)(alpha + alpha^2),
 * f_i the summand of tlookup_prove built with u_[skip_i:].  The claims of
 * instance i are A_i~, S_i~ at v_[skip_i:] and B_i~, m_i~, T_i~ at
 * v_[skip_i + log2(D_i/N_i):].
 *
 * Transcript: SHA256("zkmi/tlookup-multi/v1" || seed || LE64 K || K x (LE64 D_i, LE64 N_i)),
 * then exactly as tlookup_prove_batch (digests of all m_i; beta; digests of all
 * A_i, B_i; alpha; u_0..u_{n-1}; lambda; rounds; final).
 *
 * Proof (host, tlookup_multi_proof_bytes(D, K) bytes):
 *   "ZKTM" | u32 1 | LE64 K | K x (LE64 D_i, LE64 N_i) | K x digest(m_i)
 *   | K x [digest(A_i) digest(B_i)] | n x 4 elements | K x 5 elements.
 *
 * S, T: host arrays of K descriptors of device vectors; S[i].n = D_i and
 * T[i].n = N_i give the shapes (powers of two, N_i <= D_i <= 2^31).  idx, aux,
 * errors, stream: as tlookup_prove_batch.  ws: device,
 * tlookup_multi_workspace_bytes(D, N, K) with D, N host arrays of the K lengths.
 * In claims (tlookup_verify_multi) nvars = n and v holds the n challenges. */
size_t tlookup_multi_proof_bytes(const size_t* D, size_t K);
size_t tlookup_multi_workspace_bytes(const size_t* D, const size_t* N, size_t K);
int tlookup_prove_multi(const uint8_t seed[32], const fr_vec* S, const uint32_t* const* idx, const fr_vec* T, size_t K,
                        uint8_t* proof, size_t cap, size_t* len, tlookup_batch_aux* aux, void* ws, size_t ws_bytes,
                        void* stream);

/* Its verifier.  D: host array of the K tensor lengths (the tables' lengths are
 * T[i].n).  witness as in tlookup_verify_batch.  ws: device,
 * tlookup_multi_verify_workspace_bytes(D, N, K). */
size_t tlookup_multi_verify_workspace_bytes(const size_t* D, const size_t* N, size_t K);
int tlookup_verify_multi(const uint8_t seed[32], const uint8_t* proof, size_t len, const fr_vec* T, const size_t* D,
                         size_t K, const tlookup_witness* witness, tlookup_batch_claims* claims, void* ws,
                         size_t ws_bytes, void* stream);

/* ---- product sumcheck and matrix multiplication (Sections 3.3, 6.1.1) -------- */

/* Sumcheck of sum_{x in {0,1}^d} a(x) b(x) = claim over vectors of 2^d elements
 * (device, both folded IN PLACE: they are the prover's scratch, their contents
 * on return are unspecified; the final values are in the proof).  Round polynomials (degree 2) are sent as values
 * at X = 0,1,2.  Transcript: SHA256("zkmi/sumcheck-product/v1" || seed || LE64 d);
 * absorb("claim", claim); per round absorb("g", 3 values), r = challenge("r");
 * absorb("final", a~(r), b~(r)).
 * Proof: "ZKSP" | u32 1 | LE64 d | claim | d x 3 elements | a~(r) | b~(r). */
size_t sumcheck_product_proof_bytes(size_t n);
size_t sumcheck_product_workspace_bytes(size_t n);
int sumcheck_prove_product(const uint8_t seed[32], fr_vec a, fr_vec b, const fr_t* claim, uint8_t* proof, size_t cap,
                           size_t* len, void* ws, size_t ws_bytes, void* stream);

/* Host-only verifier of the above: round consistency and last claim =
 * a~(r) b~(r) as stated in the proof.  final_claims (host, may be NULL)
 * receives a~(r), b~(r); point (host, may be NULL) the d challenges. */
int sumcheck_verify_product(const uint8_t seed[32], const uint8_t* proof, size_t len, size_t n, fr_t final_claims[2],
                            fr_t* point);

/* Proof of Y = X W for X (D0 x D1) and W (D1 x D2), row-major device vectors
 * (element (i,k) of X at index i*D1 + k), following Section 6.1.1:
 *   Y~(u,v) = sum_{k in {0,1}^ceil(log2 D1)} X~(u,k) W~(k,v).
 * Dimensions need not be powers of two (zero padding, Section 3.3).  Transcript:
 * SHA256("zkmi/matmul/v1" || seed || LE64 D0 || LE64 D1 || LE64 D2); u_t =
 * challenge("u") x ceil(log2 D0), v_t = challenge("v") x ceil(log2 D2); the
 * library forms a_k = X~(u,k), b_k = W~(k,v) and the claim sum_k a_k b_k, then
 * absorb("claim") and the product-sumcheck rounds.
 * Proof: "ZKMM" | u32 1 | LE64 D0 | LE64 D1 | LE64 D2 | claim | d x 3 elements
 *        | X~(u,r) | W~(r,v),  d = ceil(log2 D1). */
size_t matmul_proof_bytes(size_t D1);
size_t matmul_workspace_bytes(size_t D0, size_t D1, size_t D2);
int matmul_sumcheck_prove(const uint8_t seed[32], fr_vec X, size_t D0, size_t D1, fr_vec W, size_t D2, uint8_t* proof,
                          size_t cap, size_t* len, void* ws, size_t ws_bytes, void* stream);

/* The same proof, byte for byte, from matrices of 16-bit integers (device,
 * row-major, D0*D1 and D1*D2 entries; an entry x stands for the field element x,
 * negative x for r - |x|): quantised activations and weights need not be expanded
 * to field vectors, and the partial evaluations a_k, b_k cost eight 32-bit
 * multiply-adds and two bytes of traffic per matrix entry instead of a field
 * multiplication and 32 bytes.  D0 <= 2^21 and D2 <= 2^15 (the unreduced sums
 * must fit their accumulators), else ZK_E_BADARG. */
int matmul_sumcheck_prove_i16(const uint8_t seed[32], const int16_t* X, size_t D0, size_t D1, const int16_t* W, size_t D2,
                              uint8_t* proof, size_t cap, size_t* len, void* ws, size_t ws_bytes, void* stream);

/* Verifier of the above: rounds and last claim as in sumcheck_verify_product;
 * for each of Y (D0 x D2), X, W given (device, may be empty) the corresponding
 * claim Y~(u,v), X~(u,r), W~(r,v) is recomputed from the tensor. */
size_t matmul_verify_workspace_bytes(size_t D0, size_t D1, size_t D2);
int matmul_sumcheck_verify(const uint8_t seed[32], const uint8_t* proof, size_t len, size_t D0, size_t D1, size_t D2,
                           fr_vec Y, fr_vec X, fr_vec W, void* ws, size_t ws_bytes, void* stream);

/* ---- zkAttn: the sumcheck linking the tensors of an attention layer ------------
 *
 * Last step of zkAttn-Prove (Protocol 2): after the lookups of the K segments
 * have been proved, one sumcheck shows the arithmetic relations between the
 * tensors (Section 5.1): for a rows x cols matrix of shifted scores Z' (row-major,
 * rows and cols powers of two, rows * cols <= 2^31), digits X^(k) of -Z' to the
 * public bases B^(k), segment outputs Y^(k), their product Y and its row sums yhat,
 *     Z'_x + sum_k B^(k) X^(k)_x = 0,   Y_x = prod_k Y^(k)_x,   yhat_i = sum_j Y_(i,j).
 * (Z' = Z - zhat 1^T, also part of that step, is linear in committed tensors and
 * left to the caller: Z'~(v) = Z~(v) - zhat~(v_rows).  Segments without an output
 * table are the case Y^(k) = 1.)  The paper leaves the batching of the relations
 * open; with u in F^n, n = log2(rows cols), and alpha from the transcript the
 * identity proved is
 *   alpha^2 yhat~(u_rows) = sum_x [ e~(u,x) (Z'(x) + sum_k B^(k) X^(k)(x))
 *                                  + alpha e~(u,x) (Y(x) - prod_k Y^(k)(x))
 *                                  + alpha^2 e~(u_rows, x_rows) Y(x) ],
 * degree K+1 per variable, round polynomials sent as values at X = 0..K+1, row
 * variables bound first.  1 <= K <= ZKATTN_LINK_MAX_K.  (Z' and the X^(k) are read
 * by the first round and once more at the end: their combination is the zero
 * polynomial once the first round has passed, so the later rounds do without them
 * and their values at the final point are evaluated from the tensors directly.)
 *
 * Transcript: SHA256("zkmi/zkattn-link/v1" || seed || LE64 rows || LE64 cols ||
 * LE64 K || B^(0..K-1)); u_t = challenge("u"); absorb("yhat", yhat~(u_rows));
 * alpha = challenge("alpha"); per round absorb("g", K+2 values), r =
 * challenge("r"); absorb("final", 2K+2 claims).
 * Proof: "ZKAL" | u32 1 | LE64 rows | LE64 cols | LE64 K | yhat~(u_rows)
 *        | n x (K+2) elements | Z'~(v) X^(0..K-1)~(v) Y~(v) Y^(0..K-1)~(v).
 *
 * X, Yk: host arrays of K device vectors of rows*cols elements; yhat: rows
 * elements; bases: host, K canonical non-zero elements.  Inputs are not
 * modified.  ZK_E_REJECT if the tensors do not satisfy the relations (seen in the
 * first round, where the sum differs from the claim).  ws: device,
 * zkattn_link_workspace_bytes.  Synchronises the stream. */
#define ZKATTN_LINK_MAX_K 3

typedef struct {
    fr_vec Zp, Y, yhat;
    fr_vec X[ZKATTN_LINK_MAX_K], Yk[ZKATTN_LINK_MAX_K];
} zkattn_link_witness; /* device tensors; a member with limbs == NULL is skipped */

typedef struct {
    fr_t yhat_u;                     /* yhat~(u_rows) */
    fr_t Zp_v, Y_v;                  /* claimed values at v */
    fr_t X_v[ZKATTN_LINK_MAX_K], Yk_v[ZKATTN_LINK_MAX_K];
    fr_t u[32], v[32];               /* the random point and the sumcheck point, nvars entries used */
    int nvars, K;
} zkattn_link_claims;

size_t zkattn_link_proof_bytes(size_t rows, size_t cols, size_t K);
size_t zkattn_link_workspace_bytes(size_t rows, size_t cols, size_t K);
int zkattn_link_prove(const uint8_t seed[32], fr_vec Zp, const fr_vec* X, fr_vec Y, const fr_vec* Yk, fr_vec yhat,
                      const fr_t* bases, size_t rows, size_t cols, size_t K, uint8_t* proof, size_t cap, size_t* len,
                      void* ws, size_t ws_bytes, void* stream);

/* The same proof, byte for byte, from the tensors as the integers they are
 * quantised to (Section 3.3: tensors enter the field by scaling and rounding;
 * until the first challenge binds a variable they are still small): Zp int64,
 * X^(k) and Y^(k) uint32, Y uint64, row-major device arrays of rows*cols entries;
 * X, Yk: host arrays of K device pointers; bases: host, K integers in [1, 2^32).
 * The first round checks the relations entry by entry as integers and multiplies
 * weights by integers (16 multiply-adds, no reduction until the end of a sum);
 * the second folds integers straight into reduced field elements; from the third
 * round on the path is zkattn_link_prove's.  Ranges: |Zp|, Y < 2^62; Y^(k) below
 * 2^32 - 1, 2^30, 2^18 for K = 1, 2, 3 (so that products of K extrapolated
 * factors fit 63 bits); rows*cols >= 4.  ZK_E_BADARG if an entry is out of range,
 * ZK_E_REJECT if one breaks a relation or yhat is not the row sums.  Workspace
 * and proof size as for zkattn_link_prove.  Synchronises the stream. */
int zkattn_link_prove_small(const uint8_t seed[32], const int64_t* Zp, const uint32_t* const* X, const uint64_t* Y,
                            const uint32_t* const* Yk, fr_vec yhat, const uint64_t* bases, size_t rows, size_t cols,
                            size_t K, uint8_t* proof, size_t cap, size_t* len, void* ws, size_t ws_bytes, void* stream);

/* Verifier: replays the transcript, checks every round and the last claim against
 * the summand at the final point built from the stated values, and recomputes
 * from each tensor given in *witness (may be NULL) the value stated for it.
 * claims: host, may be NULL.  ws: device, zkattn_link_verify_workspace_bytes
 * (only needed with a witness). */
size_t zkattn_link_verify_workspace_bytes(size_t rows, size_t cols);
int zkattn_link_verify(const uint8_t seed[32], const uint8_t* proof, size_t len, size_t rows, size_t cols, size_t K,
                       const fr_t* bases, const zkattn_link_witness* witness, zkattn_link_claims* claims, void* ws,
                       size_t ws_bytes, void* stream);

/* The calling host thread's pinned state (see Ownership), for callers that want no
 * allocation inside their first proof: zkmi_thread_init allocates it now, with
 * the staging buffer sized for tables of up to max_table_rows rows (a longer
 * table later makes it grow once more); zkmi_thread_release frees it (a later
 * call allocates it again).  Neither may overlap another call of the same
 * thread.  Errors: ZK_E_HIP if the runtime refuses. */
int zkmi_thread_init(size_t max_table_rows);
int zkmi_thread_release(void);

/* ---- measurement support ------------------------------------------------------
 * For benchmarks: the library can time its own phases with HIP events recorded
 * on the caller's stream (so that kernels are timed where they are launched).
 * State is per host thread.  Phases: "total" (a whole tlookup_prove call),
 * "count" (multiplicities and digest leaves), "inverse" (both batch inversions),
 * "digest" (the hash trees over A and B), "round_small" (the kernels of the rounds
 * that are bound by latency: those that also bind a table variable and those of at
 * most 256 pairs, the resident kernel included),
 * "round_data29" (the large folding rounds, which run on 29-bit limbs: one
 * record per launch of that kernel), "round_data" (the first round's kernel),
 * "round_table" (the table-side round kernel alone, which only runs when D = N).
 * A phase that waits for the host in its middle (count, inverse, digest) is
 * timed from its first launch to its last, the wait included.
 * zkmi_profile_query returns the number of records and their summed duration in
 * milliseconds; call it after the stream has been synchronised.  Unknown phase:
 * ZK_E_BADARG. */
int zkmi_profile_enable(int on);
int zkmi_profile_reset(void);
int zkmi_profile_query(const char* phase, uint64_t* records, double* total_ms);

/* Self-test of the bounded wait in the kernels that stay resident over the last
 * sumcheck rounds and receive each round's challenge from the host: such a kernel
 * is started on a tiny input with a bound of a few polls and never answered.  It
 * must publish its first round, then give up by itself and publish nothing more.
 * Then an abort is left in the channel, as a call that ends early leaves one, and
 * the kernel is started again and answered: it must run to its end.  ZK_OK if
 * both hold, ZK_E_HIP otherwise.  ws: device, at least 1 KiB. */
int zkmi_selftest_resident_wait(void* ws, size_t ws_bytes, void* stream);

/* Which kernel runs each sumcheck round of a tlookup proof of K instances of shape
 * (D, N), and where it reads S from, decided exactly as the prover decides it but
 * walked on the host alone: no GPU is touched.  from_ints != 0: the plan of
 * tlookup_prove_small (K = 1; ZK_E_BADARG for shapes that path does not take).
 * out (host): four integers per round -- kernel (0 first round, 1 large folding
 * round on 29-bit limbs, 2 data and table side together, 3 one workgroup per
 * round, 4 resident kernel, 5 the first pass when it serves the first two rounds,
 * 6 the second of those two: no kernel, 7 no kernel either: the resident kernel
 * has handed the arrays, at most 64 elements each, to the host, which runs the
 * round itself), source of S (0 the caller's
 * vector, 1 the caller's integer columns, 2 folded 32-bit words in the workspace,
 * 3 folded 29-bit limb planes in the workspace), arrays arrive as 32-bit words,
 * arrays leave as 32-bit words (both only meaningful for kernel 1).  Returns the
 * number of rounds, ZK_E_BUFSZ if cap_rounds is below it. */
int zkmi_selftest_tlookup_plan(size_t D, size_t N, size_t K, int from_ints, int32_t* out, size_t cap_rounds);

/* The rounds a single tlookup proof leaves to the host (kernel code 7 above), on
 * arrays and challenges of the caller's choosing; no GPU is touched.  All
 * pointers are host memory, all elements canonical.  A, S: n_data elements
 * (2..64, a power of two); B, M, T: n_table elements (a power of two, at most
 * n_data).  The rounds bind log2(n_data) variables, the top bit of the index
 * first; the table's arrays take part from the round on in which as many
 * variables are left as they have.  u_rest: the log2(n_data) - 1 coordinates
 * of u that belong to the variables after the first of these rounds (weights
 * e~(u_rest, p) for its pairs p).  challenges: one per round.  sums: eleven per
 * round (q0, q1, qinf, sA0, sA1, then the table side's t0, t1, tinf, m0, m1, minf,
 * zero while the table's arrays take no part), as the kernels report them
 * (Section 4's summand split into its sums over a round's pairs).  finals: what
 * is left of A, S, B, m, T.  Returns the number of rounds. */
int zkmi_selftest_host_rounds(const fr_t* A, const fr_t* S, const fr_t* B, const fr_t* M, const fr_t* T, size_t n_data,
                              size_t n_table, const fr_t* u_rest, const fr_t* beta, const fr_t* challenges, fr_t* sums,
                              fr_t* finals);

/* SHA-256 of `len` bytes at `data` (host) into out (host, 32 bytes): the hash
 * the transcript is built on, exported so that it can be checked on its own.
 * use_sha_instructions: 0 = the portable compression function, 1 = the x86 SHA
 * extensions if the processor has them (what the library uses by default),
 * else the portable one.  Returns 1 if the instruction path was used, 0 if not,
 * ZK_E_BADARG on null pointers. */
int zkmi_sha256(const uint8_t* data, size_t len, uint8_t out[32], int use_sha_instructions);

/* Library version (major * 100 + minor). */
int zkmi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ZKMI_H */
