/*
 * haflo.h - C boundary of the MI355X Paillier operator library.
 *
 * The library implements the homomorphic operators that federated logistic
 * regression runs every iteration under additive Paillier encryption (the
 * operator set of the paper's Table 1 and Table 2: encoding, decoding,
 * encryption, decryption, ciphertext addition, ciphertext-by-plaintext
 * multiplication, summation and matrix multiplication), over arrays that stay
 * resident in GPU memory between calls (the paper's "cached results" workflow,
 * Section 3.3): the caller keeps the device pointers, or lets a haflo_store
 * manage them behind handles (end of this file).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Return value: 0 on success, a negative HAFLO_E* code otherwise. No exception
 *   crosses the boundary and there is no global state besides loaded code.
 * "host" pointers are ordinary process memory; "device" pointers are HIP device
 *   memory on the current device. The caller owns every buffer it passes; the
 *   library owns only the haflo_ctx (which holds small per-key constant tables
 *   in device memory) and frees it in haflo_ctx_destroy.
 * Streams: `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *   Device work is enqueued on it and the call returns without synchronising.
 *   Operator calls enqueue kernels only (no allocation, no memset, no copy,
 *   no read-back of device data), so a sequence of them can be captured into
 *   a HIP graph and replayed on new contents of the same buffers; the
 *   staging calls and the store's upload / download copy and may wait.
 * Workspace: operators that need temporary device memory take a caller-supplied
 *   workspace pointer and its size; haflo_workspace_bytes says how much is
 *   needed. The library never allocates device memory inside an operator call.
 *   Contents of the workspace are undefined afterwards; two calls that share a
 *   workspace must be ordered on one stream.
 *
 * Interchange format (what a framework serialises, the paper's Section 3.2):
 *   a big integer is an array of little-endian uint32 limbs, item-major:
 *   element i of an array occupies words [i*L, (i+1)*L).
 *   - plaintext residue: Lp = n_bits/32 limbs, value in [0, n).
 *   - canonical ciphertext: Lc = n_bits/16 limbs, value in [0, n^2).
 * Internal ciphertext format ("cipher" below): opaque, fixed size per element
 *   (haflo_ctx_info reports it); it is the Montgomery form modulo n^2 held in
 *   29-bit limbs. Every operator consumes and produces this format, so chains
 *   of operators need no conversion; haflo_import_cipher / haflo_export_cipher
 *   convert from / to the canonical interchange format.
 * Ciphertexts that are not units modulo n^2 are the caller's error: they give
 *   an unspecified plaintext, never a fault.
 */
#ifndef HAFLO_H
#define HAFLO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HAFLO_OK 0
#define HAFLO_EINVAL (-1)  /* null pointer, bad count / size / scale, workspace too small */
#define HAFLO_EKEY (-2)    /* unusable key material */
#define HAFLO_ENOPRIV (-3) /* private-key operation on a public-only context */
#define HAFLO_EHIP (-4)    /* the HIP runtime reported an error */
#define HAFLO_ENOMEM (-5)  /* host or device allocation failed, or a store's arena is exhausted */
#define HAFLO_ETOOBIG (-6) /* haflo_decrypt_static: the batch needs more than HAFLO_STATIC_SCRATCH_BYTES */

/* Per-element status bits written by encode / decode / import. */
#define HAFLO_ST_OK 0u
#define HAFLO_ST_RANGE 1u /* value not representable: non-finite or out of range */

typedef struct haflo_ctx haflo_ctx;

/* Operator selector for haflo_workspace_bytes. */
enum haflo_op {
  HAFLO_OP_ENCRYPT = 1,
  HAFLO_OP_DECRYPT = 2,
  HAFLO_OP_SCALAR_MUL = 3,
  HAFLO_OP_MATVEC_XT_D = 4, /* orientation 0 */
  HAFLO_OP_MATVEC_X_W = 5,  /* orientation 1 */
  HAFLO_OP_FORE_GRADIENT = 6,
  HAFLO_OP_TAYLOR_LOSS = 7,
  HAFLO_OP_ENCRYPT_OBFUSCATOR = 8,
  HAFLO_OP_SUM_SEGMENTS = 9 /* rows = elements, cols = segments */
};

/* Text for an error code; never NULL. */
const char* haflo_strerror(int code);

/*
 * Deterministic key generation (host only). The paper takes the Paillier key
 * pair as given (Section 2.1); this is the seeded procedure the benchmark
 * configurations ask for: one SplitMix64 stream seeded with `seed`; a prime
 * candidate is n_bits/128 stream words (first word least significant) with the
 * two top bits and the low bit set; candidates divisible by a prime below 2000
 * are dropped; survivors take up to 40 Miller-Rabin rounds with bases
 * (words mod (cand-3)) + 2 drawn from the same stream; the first survivor is p,
 * the stream continues for q until q != p and gcd(pq,(p-1)(q-1)) = 1.
 * n_bits must be 512, 1024, 2048 or 4096. p_le and q_le are host buffers of
 * n_bits/16 bytes each (little-endian bytes).
 */
int haflo_keygen(uint32_t n_bits, uint64_t seed, uint8_t* p_le, uint8_t* q_le);

/*
 * Key contexts. g = n + 1 always. A private context (p, q given) can run every
 * operator; a public one (n only) everything except haflo_decrypt.
 * p_le / q_le: host, n_bits/16 little-endian bytes each; n_le: host, n_bits/8
 * bytes. p and q must be distinct odd numbers of exactly n_bits/2 bits whose
 * product has exactly n_bits bits and is coprime to (p-1)(q-1); primality is
 * the caller's responsibility. n_bits in {512, 1024, 2048, 4096}.
 * Context creation synchronises with the device (it uploads constant tables).
 * A context belongs to the device that is current when it is created and is
 * read-only afterwards: operator calls on one context may run from several
 * host threads as long as each uses its own workspace and stream.
 */
int haflo_ctx_create_private(const uint8_t* p_le, const uint8_t* q_le, uint32_t n_bits, haflo_ctx** out);
int haflo_ctx_create_public(const uint8_t* n_le, uint32_t n_bits, haflo_ctx** out);
int haflo_ctx_destroy(haflo_ctx* ctx);

/* Sizes for a context: key bits, canonical ciphertext limbs Lc, plaintext
 * limbs Lp, bytes of one internal ciphertext element, bytes of one plaintext
 * element (= 4*Lp). Any output pointer may be NULL. */
int haflo_ctx_info(const haflo_ctx* ctx, uint32_t* n_bits, uint32_t* cipher_limbs, uint32_t* plain_limbs,
                   size_t* cipher_bytes_internal, size_t* plain_bytes);

/* Row count from which X^T [[d]] (haflo_cipher_matvec, orientation 0) takes
 * the bucket method instead of per-base power tables; both give the same
 * ciphertext bits. The setting belongs to the context and is read by the
 * matvec itself and by every workspace query that contains one
 * (haflo_workspace_bytes for the matvec and the Taylor loss, the store's
 * calls), so change it only between a query and the call it sizes if both are
 * repeated. min_rows = 0 restores HAFLO_XTD_BUCKET_MIN_ROWS_DEFAULT; 1 forces
 * buckets wherever the shape allows them; SIZE_MAX forces tables. Not
 * synchronised: do not call it while another thread uses the context. */
#define HAFLO_XTD_BUCKET_MIN_ROWS_DEFAULT 4096
int haflo_ctx_set_xtd_bucket_min_rows(haflo_ctx* ctx, size_t min_rows);

/* Arithmetic cost of one element of an operator, for throughput accounting:
 * the number of Montgomery products the library's schedule executes per
 * element (exponentiation windows and table building included) and the size,
 * in 32-bit limbs, of the modulus they run on. Defined for HAFLO_OP_ENCRYPT
 * (modulus n^2 on a public context; on a private one the key owner's route
 * through p^2 and q^2, with its products on smaller and larger moduli
 * converted to products of the size of p^2 by their multiplication counts)
 * and HAFLO_OP_DECRYPT (the sum over both prime-power branches, modulus size
 * of p^2). Either output may be NULL. */
int haflo_op_cost(const haflo_ctx* ctx, int op, uint64_t* montmuls, uint32_t* modulus_limbs);

/* The multiply-adds (32x32+64-bit, on 29-bit limbs) the kernels really execute
 * for one element of an operator on the path a chip-filling batch takes, all
 * lanes together: the squarings leave out the symmetric half of their limb
 * products and the arithmetic modulo n^2 (p^2, q^2) runs on pairs of half-length
 * residues, so this is well below haflo_op_cost's products times (2 L^2 + L).
 * Defined for HAFLO_OP_ENCRYPT on a public context and HAFLO_OP_DECRYPT. */
int haflo_op_work(const haflo_ctx* ctx, int op, uint64_t* mads_executed);

/* Workspace needed by an operator call of the given shape. For element-wise
 * operators `rows` is the element count and `cols` is ignored; for the matvecs
 * they are the matrix shape. Returns 0 for operators that need none and
 * (size_t)-1 on bad arguments. */
size_t haflo_workspace_bytes(const haflo_ctx* ctx, int op, size_t rows, size_t cols);

/*
 * Serialisation boundary (paper Section 3.2, "Data Preprocessing" /
 * "Postprocessing"): canonical ciphertexts <-> internal ciphertexts.
 * d_canon: device, count*Lc uint32. d_cipher: device, count internal elements.
 * d_status: device, one uint32 OR-ed with HAFLO_ST_RANGE when any imported
 * value is >= n^2 (that element is imported as 0); may be NULL.
 */
int haflo_import_cipher(const haflo_ctx* ctx, const uint32_t* d_canon, void* d_cipher, uint32_t* d_status,
                        size_t count, void* stream);
int haflo_export_cipher(const haflo_ctx* ctx, const void* d_cipher, uint32_t* d_canon, size_t count, void* stream);

/*
 * "Encoding" (paper Table 2, first row; defined by the benchmark
 * configurations as signed fixed point): q = rint(v * 2^scale_bits) with ties
 * to even, computed in binary64; the plaintext residue is q mod n (a negative
 * q is stored as n - |q|). d_v: device float[count]; d_plain: device
 * count*Lp uint32; d_status: device uint32[count] or NULL, HAFLO_ST_RANGE
 * (and residue 0) when v is not finite or q leaves int64. scale_bits <= 62.
 */
int haflo_encode_f32(const haflo_ctx* ctx, const float* d_v, uint32_t scale_bits, uint32_t* d_plain,
                     uint32_t* d_status, size_t count, void* stream);

/* The same quantisation for matrix entries, kept as signed 32-bit exponents
 * for the matvecs. d_x: device float[count]; d_e: device int32[count];
 * d_status as above (HAFLO_ST_RANGE and exponent 0 when q leaves int32). */
int haflo_encode_exponents_f32(const float* d_x, uint32_t scale_bits, int32_t* d_e, uint32_t* d_status,
                               size_t count, void* stream);

/*
 * "Decoding" (paper Table 2, second row): signed lift (m > floor(n/2) means
 * m - n) to q, then value = q / 2^scale_bits in binary64 (q converted with
 * round-to-nearest-even). d_plain: device count*Lp uint32; d_q: device
 * int64[count] or NULL; d_v: device double[count] or NULL; d_status: device
 * uint32[count] or NULL, HAFLO_ST_RANGE (q = 0, value = 0) when the lifted
 * integer leaves int64. scale_bits <= 1000.
 */
int haflo_decode(const haflo_ctx* ctx, const uint32_t* d_plain, uint32_t scale_bits, int64_t* d_q, double* d_v,
                 uint32_t* d_status, size_t count, void* stream);

/*
 * "Homomorphic Encryption" (paper Table 1): E(m) = g^m * r^n mod n^2.
 * d_plain: device count*Lp uint32, residues in [0, n). d_r: device count*Lp
 * uint32, the caller's random units in [1, n) (the library draws no random
 * numbers). d_cipher: device, count internal elements (may not alias inputs).
 * Workspace: haflo_workspace_bytes(ctx, HAFLO_OP_ENCRYPT, count, 0).
 * A private context computes r^n through p^2 and q^2 (about three times the
 * rate of a public one); the ciphertexts are the same bit for bit.
 */
int haflo_encrypt(const haflo_ctx* ctx, const uint32_t* d_plain, const uint32_t* d_r, void* d_cipher, size_t count,
                  void* d_workspace, size_t workspace_bytes, void* stream);

/*
 * Encryption with a precomputed obfuscator (the usual split of Paillier
 * encryption into an offline and an online part; paper Table 1, "Homomorphic
 * Encryption": E(m) = g^m r^n mod n^2): d_obfuscator holds count internal
 * elements r_i^n mod n^2, i.e. encryptions of zero made ahead of time with
 * haflo_encrypt (plaintext 0); out[i] = (1 + m_i n) * obfuscator[i] mod n^2,
 * two products per element. Each obfuscator may be used once. d_cipher may
 * alias d_obfuscator. Workspace: HAFLO_OP_ENCRYPT_OBFUSCATOR.
 * With any ciphertext array in place of the obfuscators the same call adds the
 * plaintexts to it without an exponentiation: out[i] = c[i] * g^(m_i) mod n^2
 * encrypts D(c[i]) + m_i (and is as randomised as c[i] was, no more).
 */
int haflo_encrypt_with_obfuscator(const haflo_ctx* ctx, const uint32_t* d_plain, const void* d_obfuscator,
                                  void* d_cipher, size_t count, void* d_workspace, size_t workspace_bytes,
                                  void* stream);

/*
 * "Homomorphic Decryption" (paper Table 2; the scheme of the paper's reference
 * for Paillier): m = L(c^lambda mod n^2) * mu mod n, L(x) = (x-1)/n, evaluated
 * through the factors p^2 and q^2 and recombined (same plaintext). Private
 * context only. d_cipher: device, count internal elements; d_plain: device
 * count*Lp uint32. Workspace: HAFLO_OP_DECRYPT.
 */
int haflo_decrypt(const haflo_ctx* ctx, const void* d_cipher, uint32_t* d_plain, size_t count, void* d_workspace,
                  size_t workspace_bytes, void* stream);

/* "Homomorphic Addition" (paper Table 1): out = c1 * c2 mod n^2, element-wise.
 * All three device arrays hold count internal elements; out may alias c1 or c2. */
/*
 * haflo_decrypt for callers that cannot allocate or bring a workspace: code
 * under HIP graph capture, tight serving loops (the handful of gradient entries
 * decrypted every iteration), harnesses that forbid hipMalloc. Same arguments
 * and results as haflo_decrypt without the workspace pair; the temporaries live
 * in a fixed array of HAFLO_STATIC_SCRATCH_BYTES inside the library's device
 * image (one copy per GPU, held until the process ends; its address is
 * resolved when a context is created). No allocation of any kind happens in
 * the call. Limit: haflo_workspace_bytes(ctx, HAFLO_OP_DECRYPT, count, 0) <=
 * HAFLO_STATIC_SCRATCH_BYTES (about 5000 / 1400 / 600 elements at 1024 / 2048 /
 * 4096-bit keys), otherwise HAFLO_ETOOBIG and nothing is launched. All calls on
 * one GPU share the array: calls that overlap (different streams, threads or
 * contexts on the same GPU) race; order them on one stream.
 */
#define HAFLO_STATIC_SCRATCH_BYTES (16u << 20)
int haflo_decrypt_static(const haflo_ctx* ctx, const void* d_cipher, uint32_t* d_plain, size_t count, void* stream);

int haflo_add(const haflo_ctx* ctx, const void* d_c1, const void* d_c2, void* d_out, size_t count, void* stream);

/*
 * "Homomorphic Multiplication" (paper Table 1): out = c^k mod n^2.
 * _u64: one unsigned 64-bit scalar per element (d_k: device uint64[count]).
 * _i64_bcast: one signed scalar for the whole array; k < 0 raises the inverse
 * of c to |k|. d_out may alias d_c. Workspace: HAFLO_OP_SCALAR_MUL.
 */
int haflo_scalar_mul_u64(const haflo_ctx* ctx, const void* d_c, const uint64_t* d_k, void* d_out, size_t count,
                         void* d_workspace, size_t workspace_bytes, void* stream);
int haflo_scalar_mul_i64_bcast(const haflo_ctx* ctx, const void* d_c, int64_t k, void* d_out, size_t count,
                               void* d_workspace, size_t workspace_bytes, void* stream);

/*
 * "Homomorphic Matrix Multiplication" (paper Table 2; multiplication followed
 * by summation, Table 1) with a plaintext matrix of signed 32-bit exponents,
 * row-major X[rows][cols]; a negative exponent is a power of the inverse.
 *   orientation 0, the encrypted gradient X^T [[d]] (paper Section 2.1):
 *     d_c holds `rows` elements, d_out receives `cols` elements,
 *     out[j] = prod_i c[i]^X[i][j] mod n^2.
 *   orientation 1, the encrypted forward pass X [[w]]:
 *     d_c holds `cols` elements, d_out receives `rows` elements,
 *     out[i] = prod_j c[j]^X[i][j] mod n^2.
 * An empty or all-zero product is an encryption-free 1. d_out may not alias
 * d_c. Workspace: HAFLO_OP_MATVEC_XT_D / HAFLO_OP_MATVEC_X_W with the shape.
 * Orientation 0 has two implementations with identical results: per-base
 * power tables for matrices of fewer than 4096 rows (or more than 1024
 * columns), the bucket method above that; the row threshold is a setting of
 * the context (haflo_ctx_set_xtd_bucket_min_rows).
 */
int haflo_cipher_matvec(const haflo_ctx* ctx, int orientation, const void* d_c, const int32_t* d_X, size_t rows,
                        size_t cols, void* d_out, void* d_workspace, size_t workspace_bytes, void* stream);

/*
 * The guest's fore gradient of heterogeneous logistic regression as one call
 * (paper section 3.4 and the workflow figure there: [[0.25 (logits_host +
 * logits_guest) - 0.5 label]], eight operator calls in the framework the paper
 * accelerates), with every intermediate kept on the device:
 *   out[i] = c_host[i] * E(q(logits_guest[i]) - 2 q(label[i]) mod n; r[i]) mod n^2,
 * q(v) = rint(v * 2^scale_bits) as in haflo_encode_f32. With c_host[i] an
 * encryption of q(logits_host[i]) at the same scale, out[i] encrypts
 * q_host + q_guest - 2 q_label, which is the fore gradient at scale
 * 2^(scale_bits + 2): the factor 0.25 is a change of scale, not a ciphertext
 * operation. d_c_host, d_out: count internal elements (d_out may alias
 * d_c_host); d_logits_guest, d_label: device float[count]; d_r: device
 * count*Lp uint32 as for haflo_encrypt; d_status: device uint32[count] or
 * NULL, HAFLO_ST_RANGE (and plaintext part 0) when an input is not finite or
 * a quantised input reaches 2^61 in magnitude. scale_bits <= 60.
 * Workspace: HAFLO_OP_FORE_GRADIENT with rows = count.
 */
int haflo_fore_gradient(const haflo_ctx* ctx, const void* d_c_host, const float* d_logits_guest,
                        const float* d_label, const uint32_t* d_r, uint32_t scale_bits, void* d_out,
                        uint32_t* d_status, size_t count, void* d_workspace, size_t workspace_bytes, void* stream);

/*
 * Encrypted second-order Taylor loss (paper section 2.1, the approximated loss
 * l_H): sum_i ( -1/2 y_i u_i + 1/8 u_i^2 ) with u_i = u_host,i + u_guest,i, as
 * one ciphertext; the constant log 2 per instance and the factor 1/h are
 * public and left to the caller. With q(v) = rint(v * 2^scale_bits),
 * c_u[i] an encryption of m1_i = q(u_host,i) and c_u2[i] of m2_i = m1_i^2,
 *   out = prod_i c_u2[i] * prod_i c_u[i]^(k_i) * E(P; r)  mod n^2,
 *   k_i = 2 q(u_guest,i) - 4 q(y_i),
 *   P   = sum_i q(u_guest,i) (q(u_guest,i) - 4 q(y_i))  mod n,
 * which encrypts sum_i ( m2_i + k_i m1_i ) + P = 8 * 2^(2 scale_bits) times
 * the sum above: the result is read at scale 2^(2 scale_bits + 3).
 * d_c_u, d_c_u2: count internal elements; d_u_guest, d_label: device
 * float[count]; d_r: device Lp uint32 (one r), or NULL for r = 1 without the
 * exponentiation (the result is then randomised by the host's ciphertexts
 * only, which suffices when it goes straight to the key owner);
 * d_out: one internal element;
 * d_status: device uint32 (one word) or NULL, OR-ed with HAFLO_ST_RANGE when
 * an element is not finite or too large (|q(u_guest)| >= 2^28 or
 * |q(y)| >= 2^27; such an element contributes m2_i only). scale_bits <= 27,
 * count < 2^32. Workspace: HAFLO_OP_TAYLOR_LOSS with rows = count.
 */
int haflo_taylor_loss(const haflo_ctx* ctx, const void* d_c_u, const void* d_c_u2, const float* d_u_guest,
                      const float* d_label, const uint32_t* d_r, uint32_t scale_bits, void* d_out,
                      uint32_t* d_status, size_t count, void* d_workspace, size_t workspace_bytes, void* stream);

/* "Homomorphic Summation" (paper Table 1): out[0] = prod_i c[i] mod n^2 over
 * count internal elements (1 for count = 0). Workspace: the same as
 * HAFLO_OP_MATVEC_XT_D with rows = count, cols = 1. */
int haflo_cipher_sum(const haflo_ctx* ctx, const void* d_c, size_t count, void* d_out, void* d_workspace,
                     size_t workspace_bytes, void* stream);

/* "Homomorphic Summation" (paper Table 1) over consecutive slices of one
 * array: out[k] = prod of c[offsets[k] .. offsets[k+1]) mod n^2 for k < nseg
 * (1 for an empty slice); one slice over everything is haflo_cipher_sum.
 * d_c: count internal elements, count < 2^32. d_offsets: nseg + 1 device
 * uint32, non-decreasing, last <= count; nseg < 2^24. Slices may be of any
 * length, from empty to the whole array: every slice is spread over the chip
 * in chunks of 16 or 32 elements and reduced in rounds. An offset that runs
 * backwards or past count is the caller's error: that slice is clipped or
 * empty and HAFLO_ST_RANGE is OR-ed into d_status (one device uint32, or
 * NULL); nothing outside the array is read. d_out: nseg internal elements, may
 * not alias d_c. Workspace: HAFLO_OP_SUM_SEGMENTS with rows = count,
 * cols = nseg. */
int haflo_cipher_sum_segments(const haflo_ctx* ctx, const void* d_c, size_t count, const uint32_t* d_offsets,
                              size_t nseg, void* d_out, uint32_t* d_status, void* d_workspace, size_t workspace_bytes,
                              void* stream);

/*
 * Host staging (paper section 3.2, "Operator-level Storage Optimizer": page-locked
 * buffers reused by size, serialised arrays moved in bulk, transfers overlapped
 * with computation). A stager moves arrays in the interchange format between
 * ordinary host memory and device arrays in chunks of `chunk_elems` elements:
 * while one chunk is converted by the import / export kernel on the caller's
 * stream, the next is copied through a page-locked buffer on the stager's own
 * copy stream. The page-locked buffers come from a pool keyed by size; idle
 * buffers beyond `pool_cap_bytes` are released, least recently used first.
 * A stager belongs to one context and one host thread at a time; it owns two
 * device staging buffers of chunk_elems canonical ciphertexts.
 * The calls return when the host buffer may be reused (in) or is filled (out);
 * device-side work of the "in" calls is ordered on `stream`.
 */
typedef struct haflo_stager haflo_stager;
int haflo_stager_create(const haflo_ctx* ctx, size_t chunk_elems, size_t pool_cap_bytes, haflo_stager** out);
int haflo_stager_destroy(haflo_stager* s);
/* Page-locked bytes currently held, buffers allocated so far, requests served from the pool. */
int haflo_stager_stats(const haflo_stager* s, size_t* pinned_bytes, size_t* pinned_allocs, size_t* pinned_reuses);
/* h_canon: host, count*Lc uint32 canonical ciphertexts -> d_cipher: count internal elements
 * (d_status as for haflo_import_cipher). */
int haflo_stage_in_cipher(haflo_stager* s, const uint32_t* h_canon, void* d_cipher, uint32_t* d_status, size_t count,
                          void* stream);
/* h_plain: host, count*Lp uint32 -> d_plain: device, the same words. */
int haflo_stage_in_plain(haflo_stager* s, const uint32_t* h_plain, uint32_t* d_plain, size_t count, void* stream);
/* d_cipher: count internal elements (produced on `stream`) -> h_canon: host, count*Lc uint32. */
int haflo_stage_out_cipher(haflo_stager* s, const void* d_cipher, uint32_t* h_canon, size_t count, void* stream);
/* d_plain: device, count*Lp uint32 (produced on `stream`) -> h_plain: host. */
int haflo_stage_out_plain(haflo_stager* s, const uint32_t* d_plain, uint32_t* h_plain, size_t count, void* stream);

/*
 * Managed device-resident operands (paper section 3.3, "Operator-level
 * Computation Optimizer": results stay in GPU memory, the framework holds a
 * handle for each and passes handles back as operands; the workflow figure of
 * that section chains eight operators this way, and an allocator of the
 * library's own serves the cached results).
 * A store sub-allocates one device arena supplied by the caller (d_arena:
 * device, 256-byte aligned, arena_bytes long; it stays the caller's and must
 * outlive the store). Objects are typed arrays (enum haflo_kind) named by a
 * haflo_handle; 0 is never a valid handle and a handle dies with its object.
 * `uses` is the number of operator calls that will consume the object: the
 * call that consumes it last frees it (haflo_h_add and the scalar
 * multiplications then write their result into its block instead of a new
 * one); uses = 0 keeps the object until haflo_store_release. A call that fails
 * consumes nothing and leaves no new object. An operand that appears twice in
 * one call gives up two uses. When the arena cannot hold a result or the
 * call's temporary workspace the call fails with HAFLO_ENOMEM (nothing is
 * moved to the host).
 * All device work of a store is enqueued on the stream given at creation, and
 * calls return without synchronising (haflo_h_download to host memory
 * excepted). A store belongs to one host thread at a time.
 * haflo_store_info gives the device address of an object, so that any
 * pointer-based entry point above can read or fill it on the same stream.
 */
typedef struct haflo_store haflo_store;
typedef uint64_t haflo_handle;
enum haflo_kind {
  HAFLO_KIND_CIPHER = 1, /* internal ciphertext elements */
  HAFLO_KIND_PLAIN = 2,  /* plaintext residues, Lp uint32 each (also the random r of encryption) */
  HAFLO_KIND_F32 = 3,
  HAFLO_KIND_F64 = 4,
  HAFLO_KIND_I32 = 5, /* matrix exponents */
  HAFLO_KIND_U32 = 6, /* status words */
  HAFLO_KIND_I64 = 7,
  HAFLO_KIND_U64 = 8 /* per-element scalars */
};
int haflo_store_create(const haflo_ctx* ctx, void* d_arena, size_t arena_bytes, void* stream, haflo_store** out);
/* Forgets every object; the arena is untouched and remains the caller's. */
int haflo_store_destroy(haflo_store* s);
/* Bytes in use now (objects, 256-byte granules), the highest value that figure has
 * reached (temporaries included), live objects, the largest free block. Outputs may be NULL. */
int haflo_store_stats(const haflo_store* s, size_t* live_bytes, size_t* peak_bytes, size_t* live_objects,
                      size_t* largest_free);
/* An uninitialised object of `count` elements. */
int haflo_store_new(haflo_store* s, int kind, size_t count, uint32_t uses, haflo_handle* out);
/* Kind, element count, device address and uses left of an object; outputs may be NULL.
 * HAFLO_EINVAL for a handle that is not (or no longer) valid. */
int haflo_store_info(const haflo_store* s, haflo_handle h, int* kind, size_t* count, void** d_ptr,
                     uint32_t* uses_left);
/* Frees an object whatever uses it has left. */
int haflo_store_release(haflo_store* s, haflo_handle h);
/* A new object filled with `count` elements from src (host memory when src_on_host is
 * non-zero, else device memory). Pageable host memory is copied before the call returns. */
int haflo_h_upload(haflo_store* s, int kind, const void* src, int src_on_host, size_t count, uint32_t uses,
                   haflo_handle* out);
/* Copies an object out (one use); to host memory the call waits for the stream. */
int haflo_h_download(haflo_store* s, haflo_handle h, void* dst, int dst_on_host);
/* The operators of the paper's Table 2 over handles; semantics, value ranges and status bits
 * are those of the pointer-based entry point each one wraps. `status`, where present, may be
 * NULL; otherwise it receives a HAFLO_KIND_U32 object (one word per element) with one use. */
/* haflo_encode_f32: F32 -> PLAIN */
int haflo_h_encode(haflo_store* s, haflo_handle values, uint32_t scale_bits, uint32_t uses, haflo_handle* plain,
                   haflo_handle* status);
/* haflo_encode_exponents_f32: F32 -> I32 */
int haflo_h_encode_exponents(haflo_store* s, haflo_handle values, uint32_t scale_bits, uint32_t uses,
                             haflo_handle* exponents, haflo_handle* status);
/* haflo_decode: PLAIN -> F64 */
int haflo_h_decode(haflo_store* s, haflo_handle plain, uint32_t scale_bits, uint32_t uses, haflo_handle* values,
                   haflo_handle* status);
/* haflo_encrypt: PLAIN, PLAIN (r) -> CIPHER */
int haflo_h_encrypt(haflo_store* s, haflo_handle plain, haflo_handle r, uint32_t uses, haflo_handle* cipher);
/* haflo_decrypt: CIPHER -> PLAIN */
int haflo_h_decrypt(haflo_store* s, haflo_handle cipher, uint32_t uses, haflo_handle* plain);
/* haflo_add: CIPHER, CIPHER -> CIPHER */
int haflo_h_add(haflo_store* s, haflo_handle a, haflo_handle b, uint32_t uses, haflo_handle* out);
/* haflo_scalar_mul_i64_bcast: CIPHER -> CIPHER */
int haflo_h_scalar_mul(haflo_store* s, haflo_handle cipher, int64_t k, uint32_t uses, haflo_handle* out);
/* haflo_scalar_mul_u64: CIPHER, U64 -> CIPHER */
int haflo_h_scalar_mul_each(haflo_store* s, haflo_handle cipher, haflo_handle scalars, uint32_t uses,
                            haflo_handle* out);
/* haflo_cipher_matvec: CIPHER, I32 (rows*cols, row-major) -> CIPHER */
int haflo_h_matvec(haflo_store* s, int orientation, haflo_handle cipher, haflo_handle exponents, size_t rows,
                   size_t cols, uint32_t uses, haflo_handle* out);
/* haflo_cipher_sum: CIPHER -> CIPHER (one element) */
int haflo_h_sum(haflo_store* s, haflo_handle cipher, uint32_t uses, haflo_handle* out);

#ifdef __cplusplus
}
#endif
#endif /* HAFLO_H */
