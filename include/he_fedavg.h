/*
 * he_fedavg.h -- C ABI of the MI355X (gfx950) library for HE-based federated aggregation.
 *
 * The library implements the data path of Algorithm 1 ("HE-Based Federated Aggregation")
 * of the FedML-HE paper with an RNS-CKKS scheme over 31-bit primes:
 *
 *   key authority : (pk, sk) <- HE.KeyGen                                   he_keygen
 *   client        : [W_i] <- HE.Enc(pk, M . W_i) + (1-M) . W_i              he_encrypt_masked
 *   server        : [W_glob] <- sum_i a_i [[M . W_i]] + sum_i a_i (1-M).W_i he_aggregate
 *   client        : W <- HE.Dec(sk, M . [W_glob]) + (1-M) . [W_glob]        he_decrypt_merge
 *
 * (Section "Algorithm for HE-Based Federated Aggregation"; the call names follow the table
 * "HE Framework APIs": key_gen, enc, he_aggregate, dec.  flatten/reshape are the caller's.)
 *
 * Conventions
 * -----------
 *  - Every function returns he_status: 0 on success, negative on error.  Nothing throws,
 *    aborts or prints.  he_last_error() returns a thread-local, library-owned message for
 *    the most recent failing call of the calling thread.
 *  - "dev" pointers are device (HBM) pointers on the context's GPU, "host" pointers are
 *    ordinary host memory.  All data buffers are allocated by the caller and are never
 *    retained after the call returns; host arrays are consumed before the call returns.
 *  - All GPU work is enqueued on the given stream (a hipStream_t passed as void*; NULL is
 *    the default stream).  Calls are asynchronous with respect to the host except where a
 *    function says otherwise.  A context owns scratch memory: calls that share a context
 *    must be issued on one stream (or be externally ordered).  The scratch grows on demand:
 *    the FIRST call on a context that needs more of it than any call before (a larger model,
 *    more than 64 clients) waits for the whole device (hipDeviceSynchronize), frees the old
 *    block and allocates a larger one; every later call of that size or smaller is fully
 *    asynchronous.  The calls of the round (he_encrypt_masked, he_aggregate*, he_decrypt_merge*)
 *    can be recorded into a HIP graph by stream capture once such a first eager call with the
 *    same sizes has been made: after that they allocate nothing, synchronise nothing and clear
 *    memory with kernels.  The set-up calls (contexts, keys, masks) cannot.
 *  - Ring: R = Z[X]/(X^N+1), N = 2^log2_n, n = N/2 slots per ciphertext (the paper's
 *    "packing batch size").  Modulus chain q_0 > ... > q_{L-1}, primes < 2^31, q = 1 mod 2N.
 *  - Ciphertext layout: uint32 [n_ct][2][level][N], coefficient domain, residues in [0,q_j),
 *    poly 0 = c0, poly 1 = c1; a fresh ciphertext has level L, an aggregated one L-1.
 *    Ciphertext buffers must be 16-byte aligned (HE_ERR_INVALID_ARG otherwise).  While
 *    he_encrypt_masked runs, rows of its output buffer hold intermediate values.
 *  - Masked parameters are packed in parameter order, n per ciphertext, the last ciphertext
 *    zero padded (a vector shorter than the packing batch still takes a whole ciphertext,
 *    Section "Results on Different Scales of Models").  The plaintext remainder (1-M).W is
 *    kept compacted in parameter order: float32 [P - P_enc].
 *  - Randomness: Philox4x32-10, key = seed, counter = (block, ciphertext index, client id,
 *    stream tag); outputs are a pure function of (params, seed, client id, inputs).
 *    SECURITY: the encryption randomness (u, e0, e1) of a ciphertext is a function of
 *    (seed, client id, ciphertext index) ONLY.  Algorithm 1 keeps one key pair for all T rounds,
 *    so every he_encrypt_masked* call under one key must get a (seed, client id) pair that was
 *    never used before -- a fresh seed per round -- and that is unrelated to the he_keygen seed.
 *    Two calls with the same pair yield ciphertexts with identical c1 and c0 - c0' = m - m':
 *    whoever sees both reads the difference of the two updates without any key.  The library
 *    keeps no state between calls and cannot detect the reuse.
 *  - Ciphertext inputs of the server calls (he_aggregate*, and he_decrypt_merge*) must hold
 *    canonical residues, every word of limb j in [0, q_j): the aggregation accumulates four
 *    products w * x in 64 bits before it reduces, which is exact only for x < 2^31.  Buffers from
 *    he_encrypt_masked* and he_aggregate* satisfy this by construction; a buffer from elsewhere
 *    (the network) can be checked with he_debug_count_noncanonical.
 *  - Input parameters must be finite with |x| * 2^scale_bits < 2^31 (not checked on the
 *    hot path).
 */
#ifndef HE_FEDAVG_H
#define HE_FEDAVG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t he_status;
enum {
  HE_OK = 0,
  HE_ERR_INVALID_ARG = -1,   /* null pointer, bad size, unsorted/overlapping runs, bad weights */
  HE_ERR_LEVEL = -2,         /* ciphertext level does not fit the operation                     */
  HE_ERR_HIP = -3,           /* a HIP runtime call failed; message carries hipGetErrorString     */
  HE_ERR_NOMEM = -4,         /* host or device allocation failed                                 */
  HE_ERR_UNIMPLEMENTED = -5
};

#define HE_MAX_LIMBS 8
#define HE_MAX_CLIENTS_PER_CALL 4096

typedef struct he_ctx he_ctx;    /* public crypto context: N, chain, scale, tables (device)     */
typedef struct he_pk he_pk;      /* public key (b, a), transform domain, device                  */
typedef struct he_sk he_sk;      /* secret key s, transform domain, device                       */
typedef struct he_mask he_mask;  /* selective-encryption mask M as sorted runs, host + device    */

typedef struct {
  uint32_t log2_n;        /* 3..14; 11 ... 14 run on the specialised kernels                    */
  uint32_t n_limbs;       /* L, 2..HE_MAX_LIMBS                                                 */
  uint32_t scale_bits;    /* log2 of the CKKS scale Delta, 1..30                                */
  uint32_t cbd_eta;       /* centred-binomial parameter of the error, 0..32 (0 = no error)      */
  const uint32_t* primes; /* host, L entries descending, or NULL: the L largest primes < 2^31
                             with q = 1 (mod 2N)                                                */
} he_params;

const char* he_last_error(void);

/* ---- context (the public "crypto context" that also the server receives) -------------- */

/* Creates the context on GPU `device`: derives the chain, the 2N-th roots (smallest
   primitive root per prime), transform and encoder tables, and uploads them.  Synchronous. */
he_status he_ctx_create(const he_params* params, int device, he_ctx** out);
void he_ctx_destroy(he_ctx* ctx);
/* Copies the L primes to primes_host[L]. */
he_status he_ctx_primes(const he_ctx* ctx, uint32_t* primes_host);
uint32_t he_ctx_ring_degree(const he_ctx* ctx);                 /* N                          */
uint32_t he_ctx_n_limbs(const he_ctx* ctx);                     /* L                          */
uint64_t he_ct_bytes(const he_ctx* ctx, uint32_t level);        /* 2 * level * N * 4          */

/* ---- HE.KeyGen (Algorithm 1, "Key Authority Generate Key") ---------------------------- */

/* s ternary, a_j uniform, e centred binomial; b_j = -(a_j * s) + e mod q_j.  Keys live on
   the device in the transform domain.  Set-up call: allocates the key tables and a temporary,
   enqueues on `stream` and waits for it (hipStreamSynchronize) before it returns. */
he_status he_keygen(he_ctx* ctx, uint64_t seed, he_pk** pk, he_sk** sk, void* stream);
void he_pk_destroy(he_pk* pk);
void he_sk_destroy(he_sk* sk);

/* ---- mask M ("Selective Parameter Encryption": which entries are encrypted) ----------- */

/* starts/lens: host arrays of n_runs sorted, disjoint, non-empty runs inside [0, P).
   n_runs = 0 is the empty mask (everything stays plaintext).  Synchronous.
   The mask object holds 32 bytes of device memory per run (masked and complement runs); a
   mask whose unencrypted runs average under 4096 parameters also holds a bit per parameter
   and a word per 64 encrypted parameters (P / 8 + P_enc / 16 bytes): under such a mask
   he_encrypt_masked and he_decrypt_merge go through the model once in parameter order, with a
   packed copy of the encrypted parameters (4 bytes each) in the context's scratch. */
he_status he_mask_create(he_ctx* ctx, uint64_t P, const uint64_t* starts_host,
                         const uint64_t* lens_host, uint64_t n_runs, he_mask** out);
/* Builds the mask from a device byte mask (non-zero = encrypted).  The mask object's device
   tables are written on the GPU and a handful of words travel to the host (set-up path,
   synchronous on `stream`, allocates temporaries of about 36 bytes per 2048 entries).  Any
   alignment of mask_dev is accepted; 8-byte alignment is faster. */
he_status he_mask_from_bytes(he_ctx* ctx, uint64_t P, const uint8_t* mask_dev, he_mask** out,
                             void* stream);
/* Select(global privacy map, p) of Algorithm 1 ("Server Encryption Mask Aggregation"; Section
   "Selective Parameter Encryption", Step 2: the ratio p is the share of parameters, the most
   sensitive ones, that gets encrypted).  s_dev float32[P] is the aggregated sensitivity map (decrypted:
   the selection itself is not homomorphic); the mask takes the k = rint(ratio * P) largest
   entries (ties to even in k; equal sensitivities go to the lower parameter index; -0 = +0;
   entries must not be NaN).  Radix select and the mask object's tables on the GPU (set-up path,
   synchronous on `stream`, allocates temporaries of about P + 48 KiB bytes).  Any 4-byte
   alignment of s_dev is accepted; 16-byte alignment is faster. */
he_status he_mask_select_top(he_ctx* ctx, uint64_t P, const float* s_dev, double ratio,
                             he_mask** out, void* stream);
/* Copies the run list to the host: starts_host / lens_host hold he_mask_n_runs entries.
   For a mask built on the GPU (the two calls above) the first he_mask_runs fetches the list from
   the device with a blocking copy; he_mask_runs on one mask is not safe from several threads. */
uint64_t he_mask_n_runs(const he_mask* mask);
he_status he_mask_runs(const he_mask* mask, uint64_t* starts_host, uint64_t* lens_host);
void he_mask_destroy(he_mask* mask);
uint64_t he_mask_n_params(const he_mask* mask);                 /* P                          */
uint64_t he_mask_n_enc(const he_mask* mask);                    /* P_enc                      */
uint64_t he_n_ct(const he_ctx* ctx, const he_mask* mask);       /* ceil(P_enc / n)            */

/* ---- client: [W_i] <- HE.Enc(pk, M . W_i) + (1-M) . W_i (Algorithm 1, training loop) --- */

/* w_dev float32[P]; ct_out_dev uint32[n_ct][2][L][N]; plain_out_dev float32[P-P_enc]
   (may be NULL when P == P_enc).  Gathers the masked entries, encodes each block of n into
   a plaintext polynomial at scale Delta, encrypts it under pk with the randomness stream
   (seed, client_id, ciphertext index), and compacts the unmasked entries. */
he_status he_encrypt_masked(he_ctx* ctx, const he_pk* pk, const he_mask* mask, uint64_t seed,
                            uint32_t client_id, const float* w_dev, uint32_t* ct_out_dev,
                            float* plain_out_dev, void* stream);

/* he_encrypt_masked for callers that cannot allocate device memory: code under HIP graph capture, tight
   serving loops, harnesses that forbid hipMalloc.  Same arguments, same output bytes.  The per-ciphertext
   scratch (plaintext polynomial int32[N] and the randomness u, e0, e1 as int8[N] each: 7 * N bytes per
   ciphertext) lives in a fixed array of HE_STATIC_SCRATCH_BYTES inside the library's code object instead of
   the context's grown-on-demand block, so the call allocates and frees nothing and never synchronises.
   Limit: n_ct * N * 7 <= HE_STATIC_SCRATCH_BYTES (292 ciphertexts at N = 2^14, 585 at N = 2^13);
   HE_ERR_INVALID_ARG beyond it, with nothing enqueued.  Every GPU the library runs on holds the array until the
   process ends, and ALL calls on one GPU, from any context or stream, share it: calls that overlap in time
   on one GPU race (order them on one stream or with events).  Nothing in it has to start at zero: every
   byte a call reads was written by that call.  Per-kernel timing (he_debug_timing_enable) skips this call. */
#define HE_STATIC_SCRATCH_BYTES (32u << 20)
he_status he_encrypt_masked_static(he_ctx* ctx, const he_pk* pk, const he_mask* mask, uint64_t seed,
                                   uint32_t client_id, const float* w_dev, uint32_t* ct_out_dev,
                                   float* plain_out_dev, void* stream);

/* ---- server: [W_glob] <- sum_i a_i [[M.W_i]] + sum_i a_i (1-M).W_i ---------------------
   ("Server Model Aggregation"; plaintext weights, one multiplicative depth.)
   alpha_host double[K]: alpha_i > 0, |sum - 1| <= 1e-9.  Each weight becomes the integer
   w_i = rint(alpha_i * q_{L-1}) (ties to even); ciphertexts are multiplied by w_i, summed
   over clients, and rescaled by q_{L-1} (round to nearest), which returns the scale to
   Delta and drops one limb.  The plaintext remainders are averaged in float64 in client
   order (product and sum rounded separately) and rounded once to float32.
   ct_in_dev / plain_in_dev: host arrays of K device pointers (plain_in_dev may be NULL when
   n_plain == 0).  ct_out_dev uint32[n_ct][2][L-1][N]; plain_out_dev float32[n_plain].
   Needs only the public context -- no key. */
he_status he_aggregate(he_ctx* ctx, uint32_t K, const double* alpha_host,
                       const uint32_t* const* ct_in_dev, const float* const* plain_in_dev,
                       uint64_t n_ct, uint64_t n_plain, uint32_t* ct_out_dev,
                       float* plain_out_dev, void* stream);

/* Streaming form of the same sum for client sets that do not fit in memory at once.
   acc_ct_dev uint32[n_ct][2][L][N] (residues), acc_plain_dev double[n_plain]; both caller
   owned.  begin zeroes them; add folds K_chunk more clients in (alpha_host holds their
   globally normalised weights; clients must be added in the same order as the one-shot
   call would see them for bit-identical plaintext sums); finalize rescales / rounds. */
he_status he_aggregate_begin(he_ctx* ctx, uint64_t n_ct, uint64_t n_plain, uint32_t* acc_ct_dev,
                             double* acc_plain_dev, void* stream);
he_status he_aggregate_add(he_ctx* ctx, uint32_t K_chunk, const double* alpha_host,
                           const uint32_t* const* ct_in_dev, const float* const* plain_in_dev,
                           uint64_t n_ct, uint64_t n_plain, uint32_t* acc_ct_dev,
                           double* acc_plain_dev, void* stream);
he_status he_aggregate_finalize(he_ctx* ctx, uint64_t n_ct, uint64_t n_plain,
                                const uint32_t* acc_ct_dev, const double* acc_plain_dev,
                                uint32_t* ct_out_dev, float* plain_out_dev, void* stream);
/* The same stream of folds with two passes over the accumulators fewer (they are the extra
   memory traffic of the streaming form: 8 bytes per plaintext parameter and pass).
   he_aggregate_add_first is begin + add in one: the accumulators are written, never read, and need
   no begin.  he_aggregate_add_last is add + finalize in one: the last K_chunk clients are folded
   in and the rescaled / rounded result goes straight to ct_out_dev / plain_out_dev; the
   accumulators are read (and, for K_chunk above 64, used for partial sums) and hold nothing
   defined afterwards.  Results are bit-identical to begin, add ..., finalize. */
he_status he_aggregate_add_first(he_ctx* ctx, uint32_t K_chunk, const double* alpha_host,
                                 const uint32_t* const* ct_in_dev, const float* const* plain_in_dev,
                                 uint64_t n_ct, uint64_t n_plain, uint32_t* acc_ct_dev,
                                 double* acc_plain_dev, void* stream);
he_status he_aggregate_add_last(he_ctx* ctx, uint32_t K_chunk, const double* alpha_host,
                                const uint32_t* const* ct_in_dev, const float* const* plain_in_dev,
                                uint64_t n_ct, uint64_t n_plain, uint32_t* acc_ct_dev,
                                double* acc_plain_dev, uint32_t* ct_out_dev, float* plain_out_dev,
                                void* stream);

/* ---- client: W <- HE.Dec(sk, M . [W_glob]) + (1-M) . [W_glob] -------------------------- */

/* ct_glob_dev uint32[n_ct][2][L-1][N] (level L-1); plain_glob_dev float32[P-P_enc] (may be
   NULL when P == P_enc); w_out_dev float32[P].  Decrypts, lifts the residues to the centred
   integer, decodes the slots, and scatters masked and unmasked entries back to their
   parameter positions. */
he_status he_decrypt_merge(he_ctx* ctx, const he_sk* sk, const he_mask* mask,
                           const uint32_t* ct_glob_dev, const float* plain_glob_dev,
                           float* w_out_dev, void* stream);

/* ---- variant: weighing on the client (Section "Comparison with Other FL Frameworks" describes a
   system whose learners multiply their parameters by their weight before encrypting).
   The client encodes alpha_i * W_i, the server only adds ciphertexts: no ciphertext-scalar
   product, no rescale, and the level never drops, so a context with one limb fewer serves the
   same plaintext range.  The paper notes the price: every client learns its own weight.
   (A second price shows in the noise: K fresh encryption noises add up unweighted, so the slot
   error grows like sqrt(K) instead of sqrt(sum alpha_i^2).) ------------------------------- */

/* As he_encrypt_masked, but slot j carries alpha * w (product in float64, before encoding) and
   the plaintext remainder holds float32(alpha * w).  0 < alpha <= 1. */
he_status he_encrypt_masked_weighted(he_ctx* ctx, const he_pk* pk, const he_mask* mask,
                                     uint64_t seed, uint32_t client_id, double alpha,
                                     const float* w_dev, uint32_t* ct_out_dev,
                                     float* plain_out_dev, void* stream);
/* ct_out = sum_i ct_i (mod q_j) in all L limbs: uint32[n_ct][2][L][N], level L.  plain_out =
   float32 of the float64 sum of the K remainders in client order.  Pointer arrays as in
   he_aggregate.  Needs only the public context. */
he_status he_aggregate_sum(he_ctx* ctx, uint32_t K, const uint32_t* const* ct_in_dev,
                           const float* const* plain_in_dev, uint64_t n_ct, uint64_t n_plain,
                           uint32_t* ct_out_dev, float* plain_out_dev, void* stream);
/* he_decrypt_merge for a global ciphertext at any level 1..L: uint32[n_ct][2][level][N]. */
he_status he_decrypt_merge_level(he_ctx* ctx, const he_sk* sk, const he_mask* mask, uint32_t level,
                                 const uint32_t* ct_glob_dev, const float* plain_glob_dev,
                                 float* w_out_dev, void* stream);

/* ---- test / measurement exports (single steps of the calls above) ---------------------- */

/* Slot encoding only: slots_dev float32[n_ct][n] -> m_out_dev int32[n_ct][N],
   m_k = rint((2*Delta/N) * sum_j z_j cos(pi * 5^j * k / N)). */
he_status he_debug_encode(he_ctx* ctx, const float* slots_dev, uint64_t n_ct, int32_t* m_out_dev,
                          void* stream);
/* Encryption of given integer plaintexts m_dev int32[n_ct][N], |m| <= 2^31 - 33 so that
   m + e0 fits 32 bits (ciphertext indices first_ct .. first_ct + n_ct - 1 of client
   `client_id`) -> ct_out_dev uint32[n_ct][2][L][N]. */
he_status he_debug_encrypt_plain(he_ctx* ctx, const he_pk* pk, uint64_t seed, uint32_t client_id,
                                 uint64_t first_ct, const int32_t* m_dev, uint64_t n_ct,
                                 uint32_t* ct_out_dev, void* stream);
/* Decryption without decoding: ct_dev uint32[n_ct][2][level][N] -> d_out_dev
   uint32[n_ct][level][N], d_j = c0_j + c1_j * s mod q_j. */
he_status he_debug_decrypt_residues(he_ctx* ctx, const he_sk* sk, const uint32_t* ct_dev,
                                    uint64_t n_ct, uint32_t level, uint32_t* d_out_dev,
                                    void* stream);
/* Lift + decode only: d_dev uint32[n_ct][level][N] -> slots_out_dev float64[n_ct][n]. */
he_status he_debug_decode(he_ctx* ctx, const uint32_t* d_dev, uint64_t n_ct, uint32_t level,
                          double* slots_out_dev, void* stream);
/* In-place negacyclic transform of polys_dev uint32[batch][N] modulo q_limb.  Forward:
   coefficients -> evaluations, entry i = a(psi^(2*bitrev(i)+1)); inverse undoes it
   (including the 1/N factor). */
he_status he_debug_ntt(he_ctx* ctx, int inverse, uint32_t limb, uint32_t* polys_dev,
                       uint64_t batch, void* stream);
/* Keys in the coefficient domain for comparison with a reference: pk_coeff_dev
   uint32[2][L][N] (b then a), sk_coeff_dev int32[N] in {-1,0,1}.  Either may be NULL. */
he_status he_debug_export_keys(he_ctx* ctx, const he_pk* pk, const he_sk* sk,
                               uint32_t* pk_coeff_dev, int32_t* sk_coeff_dev, void* stream);

/* Precondition check for he_encrypt_masked (which does not validate on the hot path): counts the
   entries of w_dev float32[n] that are not finite or whose magnitude times Delta reaches
   2^31 - 32, so that plaintext plus error would leave 32 bits.  Synchronous on `stream`; uses the
   context's scratch like every other call. */
he_status he_debug_count_out_of_range(he_ctx* ctx, const float* w_dev, uint64_t n,
                                      uint64_t* count_host, void* stream);

/* Precondition check for the server calls: counts the words of ct_dev uint32[n_ct][2][level][N]
   that are not canonical residues (word >= q_j in limb j).  Synchronous on `stream`; uses the
   context's scratch. */
he_status he_debug_count_noncanonical(he_ctx* ctx, const uint32_t* ct_dev, uint64_t n_ct,
                                      uint32_t level, uint64_t* count_host, void* stream);

/* Per-kernel device timing for benchmarks: while enabled, every kernel launch of this
   context is bracketed by a pair of HIP events on its stream.  he_debug_timing_read waits
   for the recorded events, writes the summed milliseconds and the launch count of each
   kernel id (0 .. he_debug_timing_kernels()-1, named by he_debug_timing_name) to the host
   arrays, and clears the record. */
he_status he_debug_timing_enable(he_ctx* ctx, int on);
uint32_t he_debug_timing_kernels(void);
const char* he_debug_timing_name(uint32_t kernel_id);
he_status he_debug_timing_read(he_ctx* ctx, double* ms_host, uint64_t* launches_host);

#ifdef __cplusplus
}
#endif
#endif /* HE_FEDAVG_H */
