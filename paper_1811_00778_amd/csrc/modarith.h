// Modular arithmetic on 32-bit residues for primes 2^29 < p < 2^30.
// Products are 64-bit; constant multiplications use Shoup's precomputed quotient,
// 64-bit accumulators are reduced with a two-word Barrett step.
#pragma once
#include "platform.h"

namespace hcnn {

// Per-prime constants (16 bytes).
struct Mod {
  uint32_t p;     // the prime
  uint32_t c32;   // 2^32 mod p
  uint32_t c32s;  // floor(c32 * 2^32 / p)
  uint32_t mu;    // floor(2^61 / p)  (fits 32 bits because p > 2^29)
};

// A constant w < p with its Shoup companion floor(w * 2^32 / p).
struct ShoupConst {
  uint32_t w, ws;
};

HCNN_HD uint32_t mulhi32(uint32_t a, uint32_t b) {
#if defined(HCNN_HOSTEMU)
  return (uint32_t)(((uint64_t)a * b) >> 32);
#else
  return __umulhi(a, b);
#endif
}

// x * w mod p up to one extra p: result in [0, 2p) for ANY x < 2^32.
HCNN_HD uint32_t shoup_lazy(uint32_t x, uint32_t w, uint32_t ws, uint32_t p) {
  uint32_t q = mulhi32(x, ws);
  return x * w - q * p;
}

HCNN_HD uint32_t csub(uint32_t x, uint32_t p) { return x >= p ? x - p : x; }

// x * w mod p, canonical.
HCNN_HD uint32_t shoup_mul(uint32_t x, ShoupConst c, uint32_t p) {
  return csub(shoup_lazy(x, c.w, c.ws, p), p);
}

// x mod p for any x < 2^64, canonical.
HCNN_HD uint32_t reduce64(uint64_t x, const Mod& m) {
  uint32_t hi = (uint32_t)(x >> 32), lo = (uint32_t)x;
  uint32_t y = shoup_lazy(hi, m.c32, m.c32s, m.p);        // hi * 2^32 mod p, in [0, 2p)
  uint32_t qb = mulhi32(lo, m.mu) >> 29;                  // floor(lo/p) or one less
  uint32_t b = lo - qb * m.p;                             // in [0, 2p)
  uint32_t s = y + b;                                     // < 4p < 2^32
  s = csub(s, 2 * m.p);
  return csub(s, m.p);
}

// x mod p up to one extra p: result in [0, 2p) for any x < 2^64.
HCNN_HD uint32_t reduce64_2p(uint64_t x, const Mod& m) {
  uint32_t hi = (uint32_t)(x >> 32), lo = (uint32_t)x;
  uint32_t y = shoup_lazy(hi, m.c32, m.c32s, m.p);
  uint32_t qb = mulhi32(lo, m.mu) >> 29;
  return csub(y + (lo - qb * m.p), 2 * m.p);
}

// Montgomery reduction: x * 2^-32 mod p up to one extra p, for x < p * 2^32 (in particular for the
// product of two values below 2p).  pinv = -p^-1 mod 2^32; result in [0, 2p).
HCNN_HD uint32_t redc_2p(uint64_t x, uint32_t p, uint32_t pinv) {
  const uint32_t mm = (uint32_t)x * pinv;              // x + mm*p = 0 mod 2^32
  return (uint32_t)((x + (uint64_t)mm * p) >> 32);     // below 2^62 + 2^62: no overflow
}

// x mod p for x < 2^32, canonical.
HCNN_HD uint32_t reduce32(uint32_t x, const Mod& m) {
  uint32_t qb = mulhi32(x, m.mu) >> 29;
  return csub(x - qb * m.p, m.p);
}

// x * 2^-32 mod p, canonical, for any x < 3 * 2^62: a Montgomery step (result below 2^32) followed by a
// one-word Barrett step.  Used for sums of products whose constant factors carry an extra 2^32.
HCNN_HD uint32_t mont_reduce(uint64_t x, const Mod& m, uint32_t pinv) {
  const uint32_t mm = (uint32_t)x * pinv;
  const uint32_t u = (uint32_t)((x + (uint64_t)mm * m.p) >> 32);     // x + mm*p < 3*2^62 + 2^62
  return reduce32(u, m);
}
// The Montgomery step alone: x * 2^-32 mod p as a value below 2^32 (not reduced further), x < 3 * 2^62.
HCNN_HD uint32_t mont_step(uint64_t x, uint32_t p, uint32_t pinv) {
  const uint32_t mm = (uint32_t)x * pinv;
  return (uint32_t)((x + (uint64_t)mm * p) >> 32);
}
// such a sum may hold kMontRoom products of two values below 2^30 (11 * 2^60 plus small terms < 3 * 2^62)
constexpr uint32_t kMontRoom = 11;

// x mod p up to three extra p: result in [0, 4p) for any x < 2^64.
HCNN_HD uint32_t reduce64_lazy(uint64_t x, const Mod& m) {
  uint32_t hi = (uint32_t)(x >> 32), lo = (uint32_t)x;
  uint32_t y = shoup_lazy(hi, m.c32, m.c32s, m.p);
  uint32_t qb = mulhi32(lo, m.mu) >> 29;
  return y + (lo - qb * m.p);
}

HCNN_HD uint32_t mul_mod(uint32_t a, uint32_t b, const Mod& m) { return reduce64((uint64_t)a * b, m); }

HCNN_HD uint32_t add_mod(uint32_t a, uint32_t b, uint32_t p) { return csub(a + b, p); }
HCNN_HD uint32_t sub_mod(uint32_t a, uint32_t b, uint32_t p) { return a >= b ? a - b : a + p - b; }

// signed small integer -> canonical residue
HCNN_HD uint32_t small_to_res(int32_t v, const Mod& m) {
  uint32_t a = v < 0 ? (uint32_t)(-(int64_t)v) : (uint32_t)v;
  uint32_t r = reduce32(a, m);
  return (v < 0 && r != 0) ? m.p - r : r;
}

}  // namespace hcnn
