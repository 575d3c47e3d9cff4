/*
 * Oracle inner loops (TEST INFRASTRUCTURE ONLY -- never part of the product path).
 *
 * Plain C for the O(n^2) loops of the CPU oracle.  Everything here is the
 * textbook definition written out, with no blocking, no fast transform and no
 * lazy modular tricks: a reader can check each loop against the definition it
 * cites.  Big-integer CRT, centring, rounding and all parameter generation
 * live in oracle/fv.py (Python integers); this file only supplies
 *
 *   orc_ntt_eval        direct evaluation of a polynomial at given roots
 *   orc_ntt_interp      the inverse of the above (inverse-DFT sum)
 *   orc_negacyclic_mod  schoolbook product in Z_p[X]/(X^n+1)   (Sec. 2.1, ring R_q)
 *   orc_negacyclic_int  schoolbook product in Z[X]/(X^n+1) on multiword integers
 *                       (the tensor step of HMult is over the integers, Sec. 2.1)
 *   orc_scalar_mac      sum_i w_i * z_i mod p  (convolution-type layer, Sec. 3.2 / 4.3)
 *
 * OpenMP only splits the outermost loop over output coefficients.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef unsigned __int128 u128;

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static inline uint32_t mulmod(uint32_t a, uint32_t b, uint32_t p) {
  return (uint32_t)(((uint64_t)a * (uint64_t)b) % p);
}

/* out[j] = sum_i a[i] * psi^(expo[j]*i) mod p, psi a primitive 2n-th root of unity
 * mod p given through its power table psipow[e] = psi^e (e < 2n).
 * With expo[j] = 2*brev(j)+1 this is the negacyclic NTT in bit-reversed
 * evaluation order: the image of a under R_p -> prod_j Z_p[X]/(X - psi^expo[j])
 * (the same decomposition Sec. 2.1.1 states for the plaintext modulus). */
void orc_ntt_eval(uint32_t n, uint32_t p, const uint32_t* psipow, const uint32_t* expo,
                  const uint32_t* a, uint32_t* out) {
#pragma omp parallel for schedule(static)
  for (int64_t j = 0; j < (int64_t)n; ++j) {
    uint64_t acc = 0;
    for (uint64_t i = 0; i < n; ++i) {
      uint64_t e = ((uint64_t)expo[j] * i) % (2ull * n);
      acc = (acc + (uint64_t)mulmod(a[i] % p, psipow[e], p)) % p;
    }
    out[j] = (uint32_t)acc;
  }
}

/* a[i] = n^-1 * sum_j ahat[j] * psi^(-expo[j]*i) mod p : the unique polynomial of
 * degree < n whose values at the n distinct roots psi^expo[j] are ahat. */
void orc_ntt_interp(uint32_t n, uint32_t p, const uint32_t* psipow, const uint32_t* expo,
                    uint32_t n_inv, const uint32_t* ahat, uint32_t* a) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i) {
    uint64_t acc = 0;
    for (uint64_t j = 0; j < n; ++j) {
      uint64_t e = ((uint64_t)expo[j] * (uint64_t)i) % (2ull * n);
      uint64_t einv = (2ull * n - e) % (2ull * n);       /* psi^-e = psi^(2n-e) */
      acc = (acc + (uint64_t)mulmod(ahat[j] % p, psipow[einv], p)) % p;
    }
    a[i] = mulmod((uint32_t)acc, n_inv, p);
  }
}

/* c = a*b in Z_p[X]/(X^n+1): c_m = sum_{i+j=m} a_i b_j - sum_{i+j=m+n} a_i b_j. */
void orc_negacyclic_mod(uint32_t n, uint32_t p, const uint32_t* a, const uint32_t* b, uint32_t* c) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < (int64_t)n; ++m) {
    u128 pos = 0, neg = 0;
    for (int64_t i = 0; i < (int64_t)n; ++i) {
      int64_t j = m - i;
      if (j >= 0) pos += (u128)((uint64_t)a[i] * (uint64_t)b[j]);
      else        neg += (u128)((uint64_t)a[i] * (uint64_t)b[j + n]);
    }
    uint32_t ps = (uint32_t)(pos % p), ng = (uint32_t)(neg % p);
    c[m] = (uint32_t)(((uint64_t)ps + p - ng) % p);
  }
}

/* acc (wo words) += x (w words) * y (w words), all unsigned little-endian 64-bit words. */
static void mw_mul_acc(uint64_t* acc, int wo, const uint64_t* x, const uint64_t* y, int w) {
  for (int i = 0; i < w; ++i) {
    uint64_t xi = x[i];
    if (!xi) continue;
    uint64_t carry = 0;
    int k = i;
    for (int j = 0; j < w; ++j, ++k) {
      u128 t = (u128)xi * y[j] + acc[k] + carry;
      acc[k] = (uint64_t)t;
      carry = (uint64_t)(t >> 64);
    }
    for (; carry && k < wo; ++k) {
      u128 t = (u128)acc[k] + carry;
      acc[k] = (uint64_t)t;
      carry = (uint64_t)(t >> 64);
    }
  }
}

/* Integer negacyclic product.  Inputs are sign-magnitude: a_mag[i*w .. i*w+w) is
 * |a_i| and a_neg[i] is 1 when a_i < 0.  For every output coefficient m the sum
 * of the positive products (after applying X^n = -1 and the operand signs) goes
 * to pos[m*wo ..] and the sum of the negative ones to neg[m*wo ..]; the caller
 * forms c_m = pos_m - neg_m with Python integers.  wo must hold n * max|a| * max|b|. */
void orc_negacyclic_int(uint32_t n, int w, int wo,
                        const uint64_t* a_mag, const uint8_t* a_neg,
                        const uint64_t* b_mag, const uint8_t* b_neg,
                        uint64_t* pos, uint64_t* neg) {
  memset(pos, 0, (size_t)n * wo * sizeof(uint64_t));
  memset(neg, 0, (size_t)n * wo * sizeof(uint64_t));
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < (int64_t)n; ++m) {
    uint64_t* P = pos + (size_t)m * wo;
    uint64_t* N = neg + (size_t)m * wo;
    for (int64_t i = 0; i < (int64_t)n; ++i) {
      int64_t j = m - i;
      int wrap = 0;
      if (j < 0) { j += n; wrap = 1; }          /* X^(i+j) = -X^(i+j-n) */
      int negative = (a_neg[i] ^ b_neg[j] ^ wrap) & 1;
      mw_mul_acc(negative ? N : P, wo, a_mag + (size_t)i * w, b_mag + (size_t)j * w, w);
    }
  }
}

/* out[c] = sum_{tau<T} w[tau] * z[tau][c] mod p, w signed.  z rows are given by pointer. */
void orc_scalar_mac(uint32_t n, uint32_t p, uint32_t T, const uint32_t* const* z, const int32_t* w,
                    uint32_t* out) {
#pragma omp parallel for schedule(static)
  for (int64_t c = 0; c < (int64_t)n; ++c) {
    uint64_t acc = 0;
    for (uint32_t tau = 0; tau < T; ++tau) {
      int64_t ww = (int64_t)w[tau] % (int64_t)p;
      if (ww < 0) ww += p;
      acc = (acc + ((uint64_t)ww * (uint64_t)(z[tau][c] % p)) % p) % p;
    }
    out[c] = (uint32_t)acc;
  }
}
