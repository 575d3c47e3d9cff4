/*
 * hcnn.h -- C ABI of the MI355X (gfx950) library for the hot path of HCNN's
 * encrypted CNN inference: RNS-form FV/BFV ciphertext arithmetic.
 *
 * Citations name sections, tables and equations of the HCNN paper
 * (arXiv 1811.00778).
 *
 * Data model (Sec. 2.1): R = Z[X]/(X^n+1), ciphertext modulus q = q_0*...*q_{k-1}
 * (distinct primes, 2^29 < q_i < 2^30, q_i = 1 mod 2n), plaintext modulus t (prime,
 * t = 1 mod 2n for slot packing, Sec. 4.2 end).  A polynomial of R_q is stored as
 * k rows of n uint32 residues ("limb-major"): row l holds the coefficients mod q_l,
 * canonical in [0, q_l).  A ciphertext is uint32[2][k][n]; a batch is
 * uint32[n_ct][2][k][n].  Unless an entry point says otherwise, ciphertexts cross
 * this boundary in the coefficient domain.
 *
 * Pointers named *_dev are DEVICE pointers (HBM), 16-byte aligned, owned by the
 * caller; *_host are host pointers.  Input and output buffers must not overlap
 * unless "in place" is stated.  The library owns the context, its tables and its
 * scratch memory.  Every call enqueues work on the context's HIP stream and
 * returns without synchronising (hcnn_get_stat synchronises).  Return value: 0 on
 * success, a negative HCNN_ERR_* code for rejected arguments (nothing was
 * enqueued), or a positive hipError_t value when the HIP runtime failed.  No
 * exception or abort crosses this boundary.  No randomness is drawn inside the
 * library: every random polynomial is an argument.
 *
 * Conventions the paper leaves open:
 *   - psi_l, the primitive 2n-th root of unity mod q_l used by the transforms, is
 *     x^((q_l-1)/2n) for the smallest x >= 2 for which that power has order 2n;
 *   - NTT-domain index j holds the value of the polynomial at psi_l^(2*brev(j)+1),
 *     brev = bit reversal on log2(n) bits;
 *   - before the tensor product residues are lifted to the centred interval
 *     [-(q-1)/2, (q-1)/2];
 *   - relinearisation digits are the RNS residues: digit i of c2 is the polynomial
 *     with coefficients (c2 mod q_i) in [0, q_i), and evaluation-key component i
 *     encrypts g_i*s^2 with g_i = (q/q_i)*((q/q_i)^-1 mod q_i).
 */
#ifndef HCNN_H
#define HCNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hcnn_ctx hcnn_ctx;

enum {
  HCNN_OK = 0,
  HCNN_ERR_NULL = -1,     /* a required pointer is null                                     */
  HCNN_ERR_N = -2,        /* n is not a power of two in [2^10, 2^15]                        */
  HCNN_ERR_PRIME = -3,    /* a modulus is not a prime in (2^29, 2^30), not 1 mod 2n, or repeated */
  HCNN_ERR_T = -4,        /* t is not a prime below 2^47, equals a ciphertext or auxiliary prime,
                             or the call's plaintext word size does not match t            */
  HCNN_ERR_AUX = -5,      /* auxiliary basis too small: needs p_0*...*p_{k'-1} > t*n*q + 1    */
  HCNN_ERR_ARG = -6,      /* a count or size is zero, too large, or inconsistent            */
  HCNN_ERR_NOKEY = -7,    /* hcnn_ct_square_relin before hcnn_set_relin_key                 */
  HCNN_ERR_ALIGN = -8,    /* a device pointer is not 16-byte aligned                        */
  HCNN_ERR_NODEVICE = -9, /* no usable gfx950 device / LDS too small for this n             */
  HCNN_ERR_SCRATCH = -10  /* hcnn_ct_square_relin_noalloc: the parameter set needs more than
                             HCNN_STATIC_SCRATCH_BYTES for one ciphertext                   */
};

/* Limits. */
#define HCNN_MAX_LIMBS 32u        /* k <= 32 and k' <= 32 */
#define HCNN_MAX_FILTERS 16u      /* F of hcnn_ct_scalar_mac */
#define HCNN_STATIC_SCRATCH_BYTES (128u << 20)   /* work array of hcnn_ct_square_relin_noalloc, per device */

/* ---- parameter helpers (host only, no device needed) ------------------------------- */

/* Writes to primes_host[0..count) the `count` largest primes below 2^30 that are
 * 1 mod 2n, in descending order.  The usual choice is: the first k are q_0..q_{k-1},
 * the next k' the auxiliary basis. */
int hcnn_gen_primes(uint32_t n, uint32_t count, uint32_t* primes_host);

/* Smallest k' such that candidates_host[0..k') (distinct primes as above, none among
 * q) has product > t*n*q + 1: the range needed to hold the scaled tensor product
 * round(t*c*c'/q) of Sec. 2.1 (HMult step 2) exactly.  HCNN_ERR_AUX if n_candidates
 * do not suffice. */
int hcnn_min_aux_count(uint32_t n, uint32_t k, const uint32_t* q_primes_host, uint64_t t,
                       const uint32_t* candidates_host, uint32_t n_candidates, uint32_t* k_aux_out);

/* ---- context ------------------------------------------------------------------------ */

/* Builds all tables (roots of unity, base-conversion constants) for ring degree n,
 * ciphertext primes q_primes_host[0..k), auxiliary primes p_primes_host[0..k_aux) and
 * plaintext modulus t, uploads them to the current HIP device and binds the context
 * to hip_stream (a hipStream_t passed as void*; NULL = the default stream).
 * k_aux may be 0 when hcnn_ct_square_relin is not used.
 * t is any prime below 2^47 that is none of the primes above (the parameter table of Sec. 4.2 uses a
 * 43-bit t for MNIST and ten 22/23-bit moduli, one context each, for CIFAR-10).  Plaintext polynomials
 * cross the boundary in 32-bit words when t < 2^32 (hcnn_encrypt / hcnn_decrypt) and in 64-bit words
 * otherwise (hcnn_encrypt_wide / hcnn_decrypt_wide); the other entry points do not depend on the size of t. */
int hcnn_ctx_create(hcnn_ctx** out, uint32_t n, uint32_t k, const uint32_t* q_primes_host,
                    uint32_t k_aux, const uint32_t* p_primes_host, uint64_t t, void* hip_stream);
int hcnn_ctx_destroy(hcnn_ctx* ctx);
int hcnn_set_stream(hcnn_ctx* ctx, void* hip_stream);

/* Evaluation key of Sec. 2.1 (KeyGen), one component per RNS prime:
 * evk_dev = uint32[k][2][k][n], evk[i][0] = g_i*s^2 - (a_i*s + e_i), evk[i][1] = a_i,
 * coefficient domain.  The library keeps its own NTT-domain copy; the caller's
 * buffer is free again once the stream has passed this call. */
int hcnn_set_relin_key(hcnn_ctx* ctx, const uint32_t* evk_dev);

/* ---- hot path ----------------------------------------------------------------------- */

/* Batched negacyclic number-theoretic transform, in place, on n_polys polynomials:
 * polys_dev = uint32[n_polys][k][n].  Forward: row l becomes the values at
 * psi_l^(2*brev(j)+1), j = 0..n-1 -- the CRT decomposition of Sec. 2.1.1 applied to a
 * ciphertext prime; products in R_q (Sec. 2.1) become slot-wise products.  Inverse:
 * the exact inverse map (includes the factor n^-1).  Residues in and out are canonical. */
int hcnn_ntt_fwd(hcnn_ctx* ctx, uint32_t* polys_dev, size_t n_polys);
int hcnn_ntt_inv(hcnn_ctx* ctx, uint32_t* polys_dev, size_t n_polys);

/* Convolution-type layer (Sec. 3.2 "Convolution-Type Layers", Sec. 4.3): every output
 * node is sum_tau w_tau * z_tau over ciphertexts, i.e. HMultPlain by the constant
 * integer w_tau (same weight in every slot) followed by HAdd; no bias.
 *   in_cts_dev  uint32[n_in][2][k][n]
 *   idx_dev     uint32[n_grp][T]      input ciphertext index of term tau of group g
 *   w_dev       int32 [n_grp][F][T]   signed integer weights
 *   out_cts_dev uint32[F][n_grp][2][k][n]
 *   out[f][g] = sum_{tau<T} w[g][f][tau] * in[idx[g][tau]]   (mod q, both polynomials)
 * F outputs share one gather row: F = number of filters of a convolution (g runs over
 * the filter placements f_jk = j*s_h*i_w + k*s_w of Sec. 4.4.1) or the number of
 * outputs of a fully connected layer (n_grp = 1); F = 1 gives independent rows.
 * w_abs_max >= 0 is the caller's bound on |w| (it sets how often partial sums are reduced).
 * Works in either domain (the map is linear) as long as in and out use the same one.
 * An index >= n_in or a weight beyond the bound is skipped and counted in
 * HCNN_STAT_BAD_INPUT; the outputs touched are then unspecified.
 * 1 <= F <= HCNN_MAX_FILTERS. */
int hcnn_ct_scalar_mac(hcnn_ctx* ctx, const uint32_t* in_cts_dev, size_t n_in,
                       const uint32_t* idx_dev, const int32_t* w_dev, int32_t w_abs_max,
                       size_t n_grp, size_t F, size_t T, uint32_t* out_cts_dev);

/* Square activation (Sec. 3.2, "Square layer"; HSquare of Table "FHE primitives
 * benchmarks") on n_ct ciphertexts: HMult(c, c) of Sec. 2.1 --
 *   tensor (c0*c0, 2*c0*c1, c1*c1) over the integers on centred lifts,
 *   scaling round(t/q * .) of each coefficient (exact; ties cannot occur),
 *   relinearisation c'_b = y_b + sum_i evk[i][b] * digit_i(y_2) in R_q.
 * in_cts_dev, out_cts_dev = uint32[n_ct][2][k][n]; may be the same buffer (in place).
 * Needs k_aux auxiliary primes and hcnn_set_relin_key. */
int hcnn_ct_square_relin(hcnn_ctx* ctx, const uint32_t* in_cts_dev, size_t n_ct,
                         uint32_t* out_cts_dev);

/* hcnn_ct_square_relin for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result, same kernels; the intermediate
 * polynomials live in a static device array of HCNN_STATIC_SCRATCH_BYTES (128 MiB) inside the library instead of a
 * buffer from hipMalloc, and the call makes no hipMalloc / hipFree (no first-call warm-up is needed for that).
 * The batch is processed in internal batches of as many ciphertexts as fit the array:
 *   5(k+k') + 3k + k^2 + 2k polynomial rows of 4n bytes per ciphertext (5.9 MiB at n = 8192, k = 8;
 *   118 MiB at n = 32768, k = 24); any n_ct is accepted.
 * A parameter set whose single ciphertext exceeds the array (e.g. n = 32768 with 30 primes) is refused with
 * HCNN_ERR_SCRATCH before anything is enqueued.  Launches of this call are not recorded by HCNN_OPT_PROFILE.
 * Every device that loads the library holds one such array until the process ends, and all contexts on a device
 * share it: calls of this entry point that overlap in time on one device (two streams, two threads) race on it and
 * must be serialised by the caller.  Calls on one stream are ordered and safe; nothing has to be cleared between
 * calls (every word that is read was written earlier in the same call). */
int hcnn_ct_square_relin_noalloc(hcnn_ctx* ctx, const uint32_t* in_cts_dev, size_t n_ct,
                                 uint32_t* out_cts_dev);

/* General HMult of Sec. 2.1 (Table "FHE primitives benchmarks", not used by the paper's networks):
 * out_i = Relinearize(round(t/q * a_i (x) b_i)) with the tensor (c0 c0', c0 c1' + c1 c0', c1 c1') over
 * the integers on centred lifts.  a, b, out = uint32[n_ct][2][k][n]; out may be a or b. */
int hcnn_ct_mul_relin(hcnn_ctx* ctx, const uint32_t* a_cts_dev, const uint32_t* b_cts_dev, size_t n_ct,
                      uint32_t* out_cts_dev);

/* ---- test helpers (same kernels, not tuned) ------------------------------------------- */

/* KeyGen of Sec. 2.1 with the randomness passed in:
 *   s_dev int32[n] (secret, small), a_dev uint32[k][n], e_dev int32[n],
 *   a_evk_dev uint32[k][k][n] (a_i of component i), e_evk_dev int32[k][n];
 *   pk_out_dev uint32[2][k][n] = (e - a*s, a);  evk_out_dev uint32[k][2][k][n] as in
 *   hcnn_set_relin_key.  evk_out_dev may be NULL (public key only). */
int hcnn_keygen(hcnn_ctx* ctx, const int32_t* s_dev, const uint32_t* a_dev, const int32_t* e_dev,
                const uint32_t* a_evk_dev, const int32_t* e_evk_dev,
                uint32_t* pk_out_dev, uint32_t* evk_out_dev);

/* Encrypt of Sec. 2.1: c = (pk0*u + e1 + floor(q/t)*m, pk1*u + e2).
 *   pk_dev uint32[2][k][n]; m_dev uint32[n_ct][n] with entries in [0,t);
 *   u_dev, e1_dev, e2_dev int32[n_ct][n] (small); ct_out_dev uint32[n_ct][2][k][n]. */
int hcnn_encrypt(hcnn_ctx* ctx, const uint32_t* pk_dev, const uint32_t* m_dev, const int32_t* u_dev,
                 const int32_t* e1_dev, const int32_t* e2_dev, size_t n_ct, uint32_t* ct_out_dev);

/* Decrypt of Sec. 2.1: m = round(t/q * (c0 + c1*s mod q)) mod t, exact.
 *   sk_dev int32[n]; ct_dev uint32[n_ct][2][k][n]; m_out_dev uint32[n_ct][n]. */
int hcnn_decrypt(hcnn_ctx* ctx, const int32_t* sk_dev, const uint32_t* ct_dev, size_t n_ct,
                 uint32_t* m_out_dev);

/* The same two operations for a context whose t is 2^32 or more: the plaintext polynomials are
 * uint64[n_ct][n] with entries in [0,t).  (hcnn_encrypt / hcnn_decrypt return HCNN_ERR_T on such a
 * context, and these return HCNN_ERR_T on a context with t < 2^32.) */
int hcnn_encrypt_wide(hcnn_ctx* ctx, const uint32_t* pk_dev, const uint64_t* m_dev, const int32_t* u_dev,
                      const int32_t* e1_dev, const int32_t* e2_dev, size_t n_ct, uint32_t* ct_out_dev);
int hcnn_decrypt_wide(hcnn_ctx* ctx, const int32_t* sk_dev, const uint32_t* ct_dev, size_t n_ct,
                      uint64_t* m_out_dev);

/* ---- deterministic sampling (test helpers) ------------------------------------------------
 * The randomness of KeyGen and Encrypt (Sec. 2.1) always enters the library as explicit inputs.  These three calls
 * produce such inputs on the device: every element is a fixed function of (seed, stream, element index), so the
 * result does not depend on launch shapes and can be reproduced elsewhere.  Word source: Philox4x32 with 10 rounds
 * (Salmon, Moraes, Dror, Shaw, SC'11), key = (seed low word, seed high word), counter = (index low word, index
 * high word, low word of stream, kind * 2^24 + attempt); the four words of a call are used in order, then
 * attempt + 1.  Element index = poly * n + coeff, and (poly * k + limb) * n + coeff for the uniform sampler.
 *   hcnn_sample_ternary  (kind 1): out_dev int32[n_polys][n], uniform on {-1, 0, 1}: a word w is accepted unless
 *                         w = 2^32 - 1; value = w mod 3 - 1.
 *   hcnn_sample_gaussian (kind 2): out_dev int32[n_polys][n], round(N(0, 3.2^2)) with |value| <= 19 (larger values
 *                         are redrawn): words in pairs (a, b); magnitude = number of thresholds T[0..19] that are
 *                         <= a, T[v] = floor(2^32 * P(|X| <= v)); a pair with a >= T[19] is rejected; the sign is
 *                         minus when the lowest bit of b is set.
 *   hcnn_sample_uniform  (kind 3): out_dev uint32[n_polys][k][n], row l uniform in [0, q_l): a word w is accepted
 *                         when w < q_l * floor(2^32 / q_l); value = w mod q_l.
 * They return HCNN_OK, HCNN_ERR_NULL, HCNN_ERR_ARG (too many elements) or a HIP error code. */
int hcnn_sample_ternary(hcnn_ctx* ctx, uint64_t seed, uint64_t stream, int32_t* out_dev, size_t n_polys);
int hcnn_sample_gaussian(hcnn_ctx* ctx, uint64_t seed, uint64_t stream, int32_t* out_dev, size_t n_polys);
int hcnn_sample_uniform(hcnn_ctx* ctx, uint64_t seed, uint64_t stream, uint32_t* out_dev, size_t n_polys);

/* Noise read-out (the quantity behind the noise-budget figure of Sec. 5.5): with x = [c0 + c1*s]_q,
 * t*x = q*(m + t*a) + r for the centred remainder r = [t*x]_q; r/q is the invariant noise and Decrypt
 * returns m while |r/q| < 1/2.  bits_out_dev[i] = bit length of max_j |r_j| of ciphertext i (0 when every
 * r_j is 0), computed exactly; the noise budget in bits is log2(q) - 1 - bits (within one bit).
 *   sk_dev int32[n]; ct_dev uint32[n_ct][2][k][n] (16-byte aligned); bits_out_dev uint32[n_ct] (device,
 *   overwritten; cleared with a memset on the context's stream, so the call is not for graph capture).
 *   Returns HCNN_OK, HCNN_ERR_NULL, HCNN_ERR_ALIGN, or a HIP error code. */
int hcnn_noise_bits(hcnn_ctx* ctx, const int32_t* sk_dev, const uint32_t* ct_dev, size_t n_ct,
                    uint32_t* bits_out_dev);

/* ---- diagnostics ---------------------------------------------------------------------- */
enum {
  HCNN_STAT_EXACT_FALLBACKS = 0, /* coefficients whose base conversion needed the exact
                                    mixed-radix comparison instead of the fixed-point estimate */
  HCNN_STAT_BAD_INPUT = 1,       /* out-of-range indices / weights seen by hcnn_ct_scalar_mac   */
  HCNN_STAT_SCRATCH_BYTES = 2,   /* device work buffer currently held by the context            */
  HCNN_STAT_RELIN_FUSED_WGS = 3, /* workgroups of the one-kernel relinearisation that the device holds at a time
                                    (compute units x the occupancy the runtime reports for the compiled kernel);
                                    the default policy of HCNN_OPT_FUSION sizes its rounds from it: a round is
                                    8 * floor(this / 8 / k) ciphertexts                         */
  HCNN_STAT_TENSOR_FUSED_WGS = 4 /* the same for the one-kernel squaring tensor, taken for internal batches of
                                    at least 6 * this (ciphertext, limb) pairs                  */
};
/* Synchronises the context's stream, then reads the counter. */
int hcnn_get_stat(hcnn_ctx* ctx, int which, uint64_t* out);
int hcnn_reset_stats(hcnn_ctx* ctx);

enum {
  HCNN_OPT_AMBIGUITY_BAND = 0,  /* width (in units of 2^-26 of the modulus) of the band around
                                   the rounding boundary inside which the exact comparison is
                                   used; 128 (default) .. 2^26 (always); raising it only costs
                                   time (for tests) */
  HCNN_OPT_SQUARE_CHUNK = 1,    /* ciphertexts per internal batch of hcnn_ct_square_relin;
                                   0 = choose from the scratch budget */
  HCNN_OPT_PROFILE = 2,         /* non-zero: record a HIP event pair around every kernel launch */
  HCNN_OPT_RELIN_ORDER = 3,     /* workgroup order of the evaluation-key inner product: 0 = chosen from
                                   the key size (default), 1 = ciphertext-major, 2 = key-major (needs
                                   n >= 8192).  Same results either way; for tests and tuning. */
  HCNN_OPT_FUSION = 4           /* one-kernel forms of two parts of HMult that keep their intermediate
                                   polynomials in registers: the squaring tensor (step 1 with equal operands:
                                   both forward transforms, the three products and inverse transforms; rings
                                   n <= 16384) and the relinearisation (step 3: digit transforms, inner product
                                   with the key, inverse transforms; n <= 8192, and n = 16384 with at most 16
                                   primes).  0 (default) = chosen per internal batch: the tensor kernel for
                                   batches of several rounds of its workgroups, the relinearisation kernel for
                                   as many ciphertexts as fill whole rounds, the separate kernels for the rest
                                   and for small batches; 1 = always the separate kernels; 2 = always the
                                   one-kernel forms where the ring allows them.  Same results either way; for
                                   tests and tuning. */
};
int hcnn_set_option(hcnn_ctx* ctx, int which, uint64_t value);

/* Per-kernel timing collected while HCNN_OPT_PROFILE is on.  One class per kernel of the hot
 * path (the classes follow the steps of HMult in Sec. 2.1 and the layer sum of Sec. 4.3).
 * `blocks` is the number of workgroups launched: one (polynomial, limb) row of n residues per
 * workgroup for the two NTT classes, 256 coefficient positions (1024 for RELIN_MAC and
 * SCALAR_MAC) per workgroup for the others; for RELIN_FUSED it is the number of rows the launch
 * transforms (k forward + 2 inverse per workgroup).
 * hcnn_profile_read synchronises the stream; hcnn_reset_stats clears the accumulators. */
enum {
  HCNN_PROF_NTT_FWD = 0,
  HCNN_PROF_NTT_INV = 1,
  HCNN_PROF_BASE_EXT = 2,    /* centred lift q -> q u p                              */
  HCNN_PROF_TENSOR = 3,      /* the squaring tensor in one kernel (2 forward + 3 inverse transforms per workgroup;
                                `blocks` counts transformed rows); 0 where the separate transforms run */
  HCNN_PROF_SCALE = 4,       /* round(t/q .) and return to basis q                   */
  HCNN_PROF_DIGIT = 5,       /* RNS digits of c2 mod every prime: fused into NTT_FWD, stays 0 */
  HCNN_PROF_RELIN_MAC = 6,   /* inner product with the evaluation key                */
  HCNN_PROF_RELIN_ADD = 7,   /* final addition: fused into NTT_INV, stays 0           */
  HCNN_PROF_SCALAR_MAC = 8,
  HCNN_PROF_OTHER = 9,
  HCNN_PROF_RELIN_FUSED = 10, /* relinearisation in one kernel (digit transforms, inner product, inverse
                                 transforms and final addition); DIGIT-side NTT_FWD rows, RELIN_MAC and the
                                 adding NTT_INV rows are then not launched */
  HCNN_PROF_COUNT = 11
};
int hcnn_profile_read(hcnn_ctx* ctx, int kernel_class, uint64_t* launches, uint64_t* blocks,
                      double* total_ms);

/* Measured ceilings of the device the context lives on, for reading the timings above against: the rate that a
 * plain streaming kernel of this library reaches on 512 MiB buffers (HCNN_CEIL_COPY: bytes read + bytes written
 * per second of a device-to-device copy; _READ: a read-only pass; _WRITE: a fill), and the issue rate of the
 * integer instructions that the transforms (32-bit low / high multiply, add) and the multiply-accumulate (32 x 32
 * + 64-bit multiply-add, unsigned and signed) are made of, eight independent chains per lane at full occupancy.
 * value_out: GB/s for the three streaming cases, 10^12 lane-instructions per second for the others.
 * Allocates and frees its own buffers, launches on the context's stream and synchronises it: a diagnostic, not
 * for the hot path. */
enum {
  HCNN_CEIL_COPY = 0, HCNN_CEIL_READ = 1, HCNN_CEIL_WRITE = 2,
  HCNN_CEIL_MUL_LO = 3, HCNN_CEIL_MUL_HI = 4, HCNN_CEIL_MAD_U64 = 5, HCNN_CEIL_MAD_I64 = 6, HCNN_CEIL_ADD = 7,
  HCNN_CEIL_COUNT = 8
};
int hcnn_measure_ceiling(hcnn_ctx* ctx, int which, double* value_out);

const char* hcnn_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* HCNN_H */
