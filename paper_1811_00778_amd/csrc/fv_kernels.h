// Element-wise and base-conversion kernels of the FV hot path.
//
// All of them are streaming kernels: a thread owns one coefficient position (or
// four consecutive ones) and walks over limbs / terms, so every global access is
// unit-stride across the lanes of a wavefront.
#pragma once
#include "modarith.h"

namespace hcnn {

constexpr int kEwThreads = 256;   // threads per workgroup of the element-wise kernels
constexpr int kEwVec = 4;         // coefficients per thread where 16-byte accesses are used
constexpr uint32_t kXcds = 8;     // accelerator dies (each with its own L2); workgroup i runs on die i % 8

// ===================================================================================
// Exact centred base conversion.
//
// Source basis m_0..m_{ks-1} (product M), destination moduli m'_0..m'_{kd-1}.
// For an integer x given by residues x_i, |x| <= (M-1)/2:
//     z_i = [x_i * (M/m_i)^-1]_{m_i},   sum_i z_i * (M/m_i) = x + v*M,
//     v   = round(sum_i z_i / m_i)                      (because |x|/M < 1/2),
//     x mod m'_j = sum_i z_i * [(M/m_i)]_{m'_j} - v * [M]_{m'_j}.
// The tables hold the destination constants in "positive form", Bp and Vp, so that
//     out_j = ( sum_i z_i * Bp[i][j] + v * Vp[j] (+ caller's extra term) ) mod m'_j
// is one lazy 64-bit accumulation and one reduction (Vp = m' - [M]_{m'}; callers may fold
// further constant factors into zmul, Bp and Vp).
//
// sum_i z_i/m_i is estimated in fixed point with 26 fractional bits: every term
// floor(4 z_i * floor(2^56/m_i) / 2^32) is low by less than 2 units, so the estimate S
// satisfies S <= exact*2^26 < S + 2*ks.  When frac(S/2^31 + 1/2) is within `band`
// units of wrapping the estimate cannot decide the rounding; the decision is then taken
// exactly by comparing the mixed-radix (Garner) digits of the non-negative lift of x
// with those of (M-1)/2.  With the default band (128) that happens for about one
// coefficient in 2^19.
// ===================================================================================
struct BConvDev {
  uint32_t ks, kd;
  const Mod* src_mod;        // [ks]
  const ShoupConst* zmul;    // [ks]   z_i = in_i * zmul_i mod m_i
  const ShoupConst* xmul;    // [ks]   residue of the converted integer = in_i * xmul_i mod m_i
  const uint32_t* ginv;      // [ks][ks] ginv[i*ks + l] = m_l^-1 mod m_i, l < i
  const uint32_t* half;      // [ks]   mixed-radix digits of (M-1)/2
  const Mod* dst_mod;        // [kd]
  const uint32_t* dst_pinv;  // [kd]   -m'_j^-1 mod 2^32 (destinations that are RNS primes)
  uint32_t mont;             // 1: the destination constants carry an extra factor 2^32 (Montgomery form), which the
                             // reduction of the accumulated sum takes out again (mont_reduce); see bconv_use_mont
  const uint32_t* Bp;        // [ks][kd]
  const uint32_t* BpT;       // [kd][ks]  the same constants, transposed
  const uint32_t* Vp;        // [kd]
};

// Montgomery form is used where the whole sum of a destination residue (ks products plus `extra` more of the same
// size) fits the 64-bit accumulator without an intermediate fold; longer sums keep plain constants and the
// two-word Barrett reduction, which leaves room for 15 products between folds.
HCNN_HOSTDEV constexpr bool bconv_use_mont(uint32_t ks, uint32_t extra) { return ks + extra <= kMontRoom; }

constexpr uint32_t kFracBits = 26;
constexpr uint32_t kFracOne = 1u << kFracBits;

// Fixed-point estimate of z/m with 26 fractional bits (low by less than 2 units).  The sum of up
// to 32 such terms plus one half stays below 2^32.
HCNN_HD uint32_t frac_est(uint32_t z, const Mod& m) { return mulhi32(z << 2, m.mu >> 5); }

// col[i*stride] holds the residues x_i of a non-negative integer X < M on entry; they are replaced
// by its mixed-radix digits.  Returns 1 when X > (M-1)/2.
HCNN_HD uint32_t garner_gt_half(const BConvDev& bc, uint32_t* col, int stride) {
  for (uint32_t i = 1; i < bc.ks; ++i) {
    const Mod m = ldc(bc.src_mod, i);
    uint32_t t = col[i * stride];
    for (uint32_t l = 0; l < i; ++l) {
      const uint32_t al = reduce32(col[l * stride], m);
      t = sub_mod(t, al, m.p);
      t = mul_mod(t, ldc(bc.ginv, i * bc.ks + l), m);
    }
    col[i * stride] = t;
  }
  for (int i = (int)bc.ks - 1; i >= 0; --i) {
    const uint32_t a = col[i * stride], h = ldc(bc.half, i);
    if (a > h) return 1;
    if (a < h) return 0;
  }
  return 0;
}

// Rounding decision from the estimate S (sum of frac_est terms).  `exact` is called only when the
// estimate is not trustworthy AND the true fraction is near 1/2; it must return 1 when the
// non-negative lift exceeds (M-1)/2.
template <class Exact>
HCNN_HD uint32_t bconv_round(uint32_t S, uint32_t band, Exact exact, unsigned long long* fallback_counter) {
  const uint32_t w = S + (kFracOne >> 1);
  uint32_t v = w >> kFracBits;
  const uint32_t wf = w & (kFracOne - 1);
  if (wf >= kFracOne - band) {
    const uint32_t sf = S & (kFracOne - 1);
    if (sf >= (kFracOne >> 2) && sf < 3u * (kFracOne >> 2)) {   // only then can the estimate be off
      v = (S >> kFracBits) + exact();
      atomic_inc64(fallback_counter);
    }
  }
  return v;
}

// ---- generic (run-time ks, kd) helpers: per-thread columns in LDS -----------------------------
// Computes z_i (stored to zcol) and returns v.  gcol is a second private column for the exact path.
template <class In>
HCNN_HD uint32_t bconv_prepare(const BConvDev& bc, In in, uint32_t* zcol, uint32_t* gcol, int stride,
                               uint32_t band, unsigned long long* fallback_counter) {
  uint32_t S = 0;
  for (uint32_t i = 0; i < bc.ks; ++i) {
    const Mod m = ldc(bc.src_mod, i);
    const uint32_t z = shoup_mul(in(i), ldc(bc.zmul, i), m.p);
    zcol[i * stride] = z;
    S += frac_est(z, m);
  }
  auto exact = [&]() {
    for (uint32_t i = 0; i < bc.ks; ++i) gcol[i * stride] = shoup_mul(in(i), ldc(bc.xmul, i), ldc(bc.src_mod, i).p);
    return garner_gt_half(bc, gcol, stride);
  };
  return bconv_round(S, band, exact, fallback_counter);
}

// Residue of the converted integer modulo destination j; `extra` (below 2^60, in the form of the table's constants)
// is added before reducing.
HCNN_HD uint32_t bconv_output(const BConvDev& bc, const uint32_t* zcol, int stride, uint32_t v, uint32_t j,
                              uint64_t extra = 0) {
  const Mod dm = ldc(bc.dst_mod, j);
  uint64_t acc = extra + (uint64_t)v * ldc(bc.Vp, j);
  if (bc.mont) {
    for (uint32_t i = 0; i < bc.ks; ++i) acc += (uint64_t)zcol[i * stride] * ldc(bc.Bp, i * bc.kd + j);
    return mont_reduce(acc, dm, ldc(bc.dst_pinv, j));
  }
  for (uint32_t i = 0; i < bc.ks; ++i) {
    acc += (uint64_t)zcol[i * stride] * ldc(bc.Bp, i * bc.kd + j);
    if ((i & 7u) == 7u) acc = reduce64(acc, dm);
  }
  return reduce64(acc, dm);
}

// ---------------------------------------------------------------- q -> q u p extension
// in  [n_ct][2][k][n]  ->  out [n_ct][2][k+kd][n]; rows 0..k-1 are copies, rows k.. are
// the residues of the centred lift modulo the auxiliary primes.
struct ExtArgs {
  const uint32_t* in;
  uint32_t* out;
  BConvDev bc;
  uint32_t n;
  uint32_t band;
  unsigned long long* fallback_counter;
};
struct ExtKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  static size_t lds_bytes(uint32_t ks) { return (size_t)2 * ks * kThreads * 4; }
  template <int PH>
  HCNN_HD static void phase(const ExtArgs& a, unsigned bid, int tid, uint32_t* lds, Regs&) {
    const uint32_t ks = a.bc.ks, kd = a.bc.kd, n = a.n;
    const uint32_t blocks_per_poly = n / kThreads;
    const size_t poly = bid / blocks_per_poly;
    const uint32_t c = (bid % blocks_per_poly) * kThreads + tid;
    const uint32_t* src = a.in + poly * ks * n + c;
    uint32_t* dst = a.out + poly * (size_t)(ks + kd) * n + c;
    uint32_t* zcol = lds + tid;
    uint32_t* gcol = lds + (size_t)ks * kThreads + tid;
    auto in = [&](uint32_t i) { return src[(size_t)i * n]; };
    const uint32_t v = bconv_prepare(a.bc, in, zcol, gcol, kThreads, a.band, a.fallback_counter);
    // (rows 0..ks-1 of `out` are not written: the forward transform reads those limbs from the ciphertext itself)
    for (uint32_t j = 0; j < kd; ++j) dst[(size_t)(ks + j) * n] = bconv_output(a.bc, zcol, kThreads, v, j);
  }
};

// Register-resident variant for compile-time basis sizes: z_i stay in VGPRs, every table index is a
// compile-time constant (scalar loads), the LDS column is touched only by the exact path.
template <int K, int KP>
struct ExtKernelT {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  static size_t lds_bytes() { return (size_t)K * kThreads * 4; }
  template <int PH>
  HCNN_HD static void phase(const ExtArgs& a, unsigned bid, int tid, uint32_t* lds, Regs&) {
    const uint32_t n = a.n;
    const uint32_t blocks_per_poly = n / kThreads;
    const size_t poly = bid / blocks_per_poly;
    const uint32_t c = (bid % blocks_per_poly) * kThreads + tid;
    const uint32_t* src = a.in + poly * K * n + c;
    uint32_t* dst = a.out + poly * (size_t)(K + KP) * n + c;
    uint32_t x[K], z[K];
    uint32_t S = 0;
#pragma unroll
    for (int i = 0; i < K; ++i) x[i] = src[(size_t)i * n];
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const Mod m = ldc(a.bc.src_mod, i);
      z[i] = shoup_mul(x[i], ldc(a.bc.zmul, i), m.p);
      S += frac_est(z[i], m);
    }
    auto exact = [&]() {
      uint32_t* col = lds + tid;
#pragma unroll
      for (int i = 0; i < K; ++i) col[i * kThreads] = shoup_mul(x[i], ldc(a.bc.xmul, i), ldc(a.bc.src_mod, i).p);
      return garner_gt_half(a.bc, col, kThreads);
    };
    const uint32_t v = bconv_round(S, a.band, exact, a.fallback_counter);
    // (rows 0..K-1 of `out` are not written: the forward transform reads those limbs from the ciphertext itself)
    // rolled loop over the destination primes: row j of the transposed table is one contiguous scalar load
#pragma unroll 1
    for (uint32_t j = 0; j < (uint32_t)KP; ++j) {
      const Mod dm = ldc(a.bc.dst_mod, j);
      const uint32_t* bt = a.bc.BpT + (size_t)j * K;
      uint64_t acc = (uint64_t)v * ldc(a.bc.Vp, j);
      if constexpr (bconv_use_mont(K, 0)) {
#pragma unroll
        for (int i = 0; i < K; ++i) acc += (uint64_t)z[i] * ldc(bt, i);
        // The forward transform that reads these rows takes any value below 4p.  A sum of K products leaves the
        // Montgomery step below K*2^28 + p; for K <= 9 one conditional subtraction of 2p brings that under
        // max(2p, 9*2^28 - p) < 4p for every p > 2^29.
        if constexpr (K <= 9) dst[(size_t)(K + j) * n] = csub(mont_step(acc, dm.p, ldc(a.bc.dst_pinv, j)), 2 * dm.p);
        else                  dst[(size_t)(K + j) * n] = mont_reduce(acc, dm, ldc(a.bc.dst_pinv, j));
      } else {
#pragma unroll
        for (int i = 0; i < K; ++i) {
          acc += (uint64_t)z[i] * ldc(bt, i);
          if ((i % 14) == 12 && i + 1 < K) acc = reduce64(acc, dm);
        }
        dst[(size_t)(K + j) * n] = reduce64(acc, dm);
      }
    }
  }
};

// ---------------------------------------------------------------- scale-and-round (HMult step 2)
// d [n_ct][3][k+kp][n] (coefficient domain, integer tensor known mod q and mod p)
//   -> y [n_ct][3][k][n],  y = round(t*d/q) mod q.
// With r = [t*d]_q (centred): y = (t*d - r)/q exactly.  Modulo p_j:
//     y = d'_j * (t q^-1) - sum_i z_i * q_i^-1 + v          (z_i = [t d_i (q/q_i)^-1]_{q_i})
// (table to_p: Bp = p_j - q_i^-1, Vp = 1, extra term d'_j * tq_inv_j), then y, which satisfies
// |y| < p/2 by the choice of the auxiliary basis, is converted p -> q (table to_q).
struct ScaleArgs {
  const uint32_t* d;
  uint32_t* y;
  BConvDev to_p;              // src q (zmul = t*(q/q_i)^-1, xmul = t), dst p
  BConvDev to_q;              // src p (zmul = (p/p_j)^-1, xmul = 1), dst q
  const uint32_t* tq_inv;     // [kp]  t * q^-1 mod p_j
  uint32_t n;
  uint32_t band;
  unsigned long long* fallback_counter;
};
struct ScaleKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  static size_t lds_bytes(uint32_t k, uint32_t kp) { return (size_t)(2 * (k > kp ? k : kp) + kp) * kThreads * 4; }
  template <int PH>
  HCNN_HD static void phase(const ScaleArgs& a, unsigned bid, int tid, uint32_t* lds, Regs&) {
    const uint32_t k = a.to_p.ks, kp = a.to_p.kd, n = a.n, L = k + kp;
    const uint32_t kmax = k > kp ? k : kp;
    const uint32_t blocks_per_poly = n / kThreads;
    const size_t poly = bid / blocks_per_poly;             // (ct, component)
    const uint32_t c = (bid % blocks_per_poly) * kThreads + tid;
    const uint32_t* src = a.d + poly * (size_t)L * n + c;
    uint32_t* dst = a.y + poly * (size_t)k * n + c;
    uint32_t* zcol = lds + tid;
    uint32_t* gcol = lds + (size_t)kmax * kThreads + tid;
    uint32_t* ycol = lds + (size_t)2 * kmax * kThreads + tid;

    auto in_q = [&](uint32_t i) { return src[(size_t)i * n]; };
    const uint32_t v = bconv_prepare(a.to_p, in_q, zcol, gcol, kThreads, a.band, a.fallback_counter);
    for (uint32_t j = 0; j < kp; ++j) {
      // d'_j arrives in [0, 2p): made canonical so that its product takes the room of one
      const uint64_t extra = (uint64_t)csub(src[(size_t)(k + j) * n], ldc(a.to_p.dst_mod, j).p) * ldc(a.tq_inv, j);
      ycol[j * kThreads] = bconv_output(a.to_p, zcol, kThreads, v, j, extra);
    }
    auto in_p = [&](uint32_t j) { return ycol[j * kThreads]; };
    const uint32_t v2 = bconv_prepare(a.to_q, in_p, zcol, gcol, kThreads, a.band, a.fallback_counter);
    for (uint32_t i = 0; i < k; ++i) dst[(size_t)i * n] = bconv_output(a.to_q, zcol, kThreads, v2, i);
  }
};

// Register-resident variant (see ExtKernelT) with a rolled loop over the auxiliary primes: y_j is produced, used at once for the
// p -> q conversion (k running 64-bit sums) and parked in the LDS column for the exact path, so
// the register footprint is 3k + O(1) and the code size does not grow with k*k'.
template <int K, int KP>
struct ScaleKernelR {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  static size_t lds_bytes() { return (size_t)(K > KP ? K : KP) * kThreads * 4; }
  template <int PH>
  HCNN_HD static void phase(const ScaleArgs& a, unsigned bid, int tid, uint32_t* lds, Regs&) {
    const uint32_t n = a.n;
    constexpr int L = K + KP;
    const uint32_t blocks_per_poly = n / kThreads;
    const size_t poly = bid / blocks_per_poly;             // (ct, component)
    const uint32_t c = (bid % blocks_per_poly) * kThreads + tid;
    const uint32_t* src = a.d + poly * (size_t)L * n + c;
    uint32_t* dst = a.y + poly * (size_t)K * n + c;
    uint32_t* col = lds + tid;

    uint32_t z[K];
    uint32_t S = 0;
    {
      uint32_t dq[K];
#pragma unroll
      for (int i = 0; i < K; ++i) dq[i] = src[(size_t)i * n];
#pragma unroll
      for (int i = 0; i < K; ++i) {
        const Mod m = ldc(a.to_p.src_mod, i);
        z[i] = shoup_mul(dq[i], ldc(a.to_p.zmul, i), m.p);
        S += frac_est(z[i], m);
      }
    }
    auto exact_q = [&]() {
      for (uint32_t i = 0; i < (uint32_t)K; ++i)
        col[i * kThreads] = shoup_mul(src[(size_t)i * n], ldc(a.to_p.xmul, i), ldc(a.to_p.src_mod, i).p);
      return garner_gt_half(a.to_p, col, kThreads);
    };
    const uint32_t v = bconv_round(S, a.band, exact_q, a.fallback_counter);

    // to_p sums K products and the term of d'_j (which arrives in [0, 2p): it takes the room of two unless it is made
    // canonical first); to_q sums KP products.  Each uses Montgomery-form constants iff the host built them so.
    constexpr bool kMontP = bconv_use_mont(K, 1), kCanonDp = !bconv_use_mont(K, 2);
    constexpr bool kMontQ = bconv_use_mont(KP, 0);
    constexpr int kCadence = 14;             // plain form: products below 2^60 between two-word reductions
    uint64_t out_acc[K];
#pragma unroll
    for (int i = 0; i < K; ++i) out_acc[i] = 0;
    uint32_t S2 = 0;
    uint32_t dp_next = src[(size_t)K * n];
#pragma unroll 1
    for (uint32_t j = 0; j < (uint32_t)KP; ++j) {
      uint32_t dpj = dp_next;
      if (j + 1 < (uint32_t)KP) dp_next = src[(size_t)(K + j + 1) * n];
      const Mod dm = ldc(a.to_p.dst_mod, j);
      if constexpr (kCanonDp) dpj = csub(dpj, dm.p);
      uint64_t acc = (uint64_t)dpj * ldc(a.tq_inv, j) + (uint64_t)v * ldc(a.to_p.Vp, j);
      const uint32_t* bt = a.to_p.BpT + (size_t)j * K;
      uint32_t yj;
      if constexpr (kMontP) {
#pragma unroll
        for (int i = 0; i < K; ++i) acc += (uint64_t)z[i] * ldc(bt, i);
        yj = mont_step(acc, dm.p, ldc(a.to_p.dst_pinv, j));     // any 32-bit value is a valid operand of the Shoup product below
      } else {
#pragma unroll
        for (int i = 0; i < K; ++i) {
          acc += (uint64_t)z[i] * ldc(bt, i);
          if ((i % kCadence) == kCadence - 2 && i + 1 < K) acc = reduce64(acc, dm);   // the term of d'_j came first
        }
        yj = reduce64_lazy(acc, dm);
      }
      col[j * kThreads] = yj;                                     // made canonical by the exact path if it runs
      const Mod sm = ldc(a.to_q.src_mod, j);
      const uint32_t z2 = shoup_mul(yj, ldc(a.to_q.zmul, j), sm.p);
      S2 += frac_est(z2, sm);
      const uint32_t* b2 = a.to_q.Bp + (size_t)j * K;
#pragma unroll
      for (int i = 0; i < K; ++i) out_acc[i] += (uint64_t)z2 * ldc(b2, i);
      if constexpr (!kMontQ) {
        if ((j % kCadence) == kCadence - 1) {
#pragma unroll
          for (int i = 0; i < K; ++i) out_acc[i] = reduce64(out_acc[i], ldc(a.to_q.dst_mod, i));
        }
      }
    }
    auto exact_p = [&]() {
      for (uint32_t j = 0; j < (uint32_t)KP; ++j) {
        const Mod sm = ldc(a.to_q.src_mod, j);
        col[j * kThreads] = reduce32(col[j * kThreads], sm);
      }
      return garner_gt_half(a.to_q, col, kThreads);
    };
    const uint32_t v2 = bconv_round(S2, a.band, exact_p, a.fallback_counter);
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const Mod dm = ldc(a.to_q.dst_mod, i);
      const uint64_t sum = out_acc[i] + (uint64_t)v2 * ldc(a.to_q.Vp, i);      // v2*Vp < 2^36
      dst[(size_t)i * n] = kMontQ ? mont_reduce(sum, dm, ldc(a.to_q.dst_pinv, i)) : reduce64(sum, dm);
    }
  }
};

// ---------------------------------------------------------------- relinearisation inner product
// (the digit reduction and the final addition are fused into the transforms, see ntt_kernels.h)
// acc[ct][b][j] = sum_i evk_hat[i][b][j] * dig_hat[ct][i][j]   (all NTT domain)
struct RelinMacArgs {
  const uint32_t* dig;   // [n_ct][k][k][n]
  const uint32_t* evk;   // [k][2][k][n]
  uint32_t* acc;         // [n_ct][2][k][n]
  const Mod* mods;
  uint32_t k, n;
  uint32_t n_grp;        // groups of CT ciphertexts in this launch
  uint32_t ct_base;      // first ciphertext of the launch
  uint32_t key_major;    // workgroup order, see the kernel
};
// A workgroup takes one (limb j, coefficient tile) for CT consecutive ciphertexts: every evaluation-key tile
// is loaded once and multiplied with the digits of all CT ciphertexts from registers.  (The key is read from
// L2; with one ciphertext per workgroup it makes up two thirds of what flows from L2 into the compute units,
// and that flow, not HBM, then bounds the kernel.)
template <int CT>
struct RelinMacKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  template <int PH>
  HCNN_HD static void phase(const RelinMacArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    const uint32_t per_row = a.n / (kThreads * kEwVec);
    size_t grp;
    uint32_t j, tile;
    if (a.key_major) {
      // (chosen by the host when the evaluation key outgrows an L2 in the plain order)
      // die x takes the coefficient tiles x, x+8, ... ; for one (limb, tile) it sweeps the ciphertexts of
      // the batch back to back, so the 2k evaluation-key tiles they all multiply with stay in that die's L2
      const uint32_t xcd = bid % kXcds, local = bid / kXcds;
      grp = local % a.n_grp;
      const uint32_t rest = local / a.n_grp;
      tile = (rest % (per_row / kXcds)) * kXcds + xcd;
      j = rest / (per_row / kXcds);
    } else {
      const size_t row = bid / per_row;                     // (group, j)
      tile = bid % per_row;
      grp = row / a.k;
      j = (uint32_t)(row % a.k);
    }
    const size_t ct0 = a.ct_base + grp * CT;
    const uint32_t c = (tile * kThreads + tid) * kEwVec;
    const Mod m = ldc(a.mods, j);
    const size_t rn = a.n;
    uint64_t s0[CT][4], s1[CT][4];
#pragma unroll
    for (int t = 0; t < CT; ++t)
      for (int q = 0; q < 4; ++q) { s0[t][q] = 0; s1[t][q] = 0; }
    // 15 products below 2^60 (+ a residue) fit 64 bits; inside a run of 15 the loop is unrolled so that the
    // loads of several digits are in flight together
    for (uint32_t i0 = 0; i0 < a.k; i0 += 15) {
      const uint32_t i1 = i0 + 15 < a.k ? i0 + 15 : a.k;
#pragma unroll 2
      for (uint32_t i = i0; i < i1; ++i) {
        const U4 e0 = *reinterpret_cast<const U4*>(a.evk + (((size_t)i * 2 + 0) * a.k + j) * rn + c);
        const U4 e1 = *reinterpret_cast<const U4*>(a.evk + (((size_t)i * 2 + 1) * a.k + j) * rn + c);
        U4 d[CT];
#pragma unroll
        for (int t = 0; t < CT; ++t)
          d[t] = *reinterpret_cast<const U4*>(a.dig + (((ct0 + t) * a.k + i) * a.k + j) * rn + c);
#pragma unroll
        for (int t = 0; t < CT; ++t) {
          s0[t][0] += (uint64_t)d[t].x * e0.x; s0[t][1] += (uint64_t)d[t].y * e0.y;
          s0[t][2] += (uint64_t)d[t].z * e0.z; s0[t][3] += (uint64_t)d[t].w * e0.w;
          s1[t][0] += (uint64_t)d[t].x * e1.x; s1[t][1] += (uint64_t)d[t].y * e1.y;
          s1[t][2] += (uint64_t)d[t].z * e1.z; s1[t][3] += (uint64_t)d[t].w * e1.w;
        }
      }
      if (i1 < a.k) {
#pragma unroll
        for (int t = 0; t < CT; ++t)
          for (int q = 0; q < 4; ++q) { s0[t][q] = reduce64(s0[t][q], m); s1[t][q] = reduce64(s1[t][q], m); }
      }
    }
#pragma unroll
    for (int t = 0; t < CT; ++t) {
      U4 r0, r1;
      r0.x = reduce64(s0[t][0], m); r0.y = reduce64(s0[t][1], m); r0.z = reduce64(s0[t][2], m); r0.w = reduce64(s0[t][3], m);
      r1.x = reduce64(s1[t][0], m); r1.y = reduce64(s1[t][1], m); r1.z = reduce64(s1[t][2], m); r1.w = reduce64(s1[t][3], m);
      *reinterpret_cast<U4*>(a.acc + (((ct0 + t) * 2 + 0) * a.k + j) * rn + c) = r0;
      *reinterpret_cast<U4*>(a.acc + (((ct0 + t) * 2 + 1) * a.k + j) * rn + c) = r1;
    }
  }
};

// ---------------------------------------------------------------- scalar multiply-accumulate
// out[f][g] = sum_tau w[g][f][tau] * in[idx[g][tau]]  per residue (HMultPlain by an integer + HAdd).
struct MacArgs {
  const uint32_t* in;     // [n_in][2][k][n]
  const uint32_t* idx;    // [G][T]
  const int32_t* w;       // [G][F][T]
  uint32_t* out;          // [F][G][2][k][n]
  const Mod* mods;        // [k]
  uint32_t k, n;
  uint32_t n_in, G, F, T;
  int32_t w_abs_max;
  uint32_t chunk;         // terms between reductions of the signed 64-bit accumulators
  unsigned long long* bad_counter;
};
// Fallback for gather rows too long to stage in LDS: indices and weights are read from global
// memory inside the term loop.
template <int FT>
struct MacKernelDirect {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  HCNN_HD static int64_t fold(int64_t s, const Mod& m) {
    const uint64_t mag = s < 0 ? (uint64_t)(-s) : (uint64_t)s;
    const uint32_t r = reduce64(mag, m);
    return (s < 0 && r != 0) ? (int64_t)(m.p - r) : (int64_t)r;
  }
  template <int PH>
  HCNN_HD static void phase(const MacArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    const uint32_t ct_words32 = 2u * a.k * a.n;                       // at most 2^22
    const size_t ct_words = ct_words32;
    const uint32_t tiles = ct_words32 / (kThreads * kEwVec);
    const uint32_t g = bid / tiles;
    const uint32_t tile = bid % tiles;
    const uint32_t pos = (tile * kThreads + tid) * kEwVec;            // word offset inside a ciphertext
    const uint32_t row = tile / (a.n / (kThreads * kEwVec));          // (poly, limb) row; uniform in the block
    const uint32_t limb = row % a.k;
    const Mod m = ldc(a.mods, limb);
    const uint32_t* idx = a.idx + (size_t)g * a.T;
    const int32_t* w = a.w + (size_t)g * a.F * a.T;
    int64_t s[FT][4];
#pragma unroll
    for (int f = 0; f < FT; ++f) { s[f][0] = 0; s[f][1] = 0; s[f][2] = 0; s[f][3] = 0; }
    uint32_t since = 0;
    for (uint32_t tau = 0; tau < a.T; ++tau) {
      const uint32_t src = idx[tau];
      if (src >= a.n_in) {
        if (tid == 0 && tile == 0) atomic_inc64(a.bad_counter);
        continue;
      }
      const U4 x = *reinterpret_cast<const U4*>(a.in + (size_t)src * ct_words + pos);
#pragma unroll
      for (int f = 0; f < FT; ++f) {
        int32_t wf = w[(size_t)f * a.T + tau];
        if (wf > a.w_abs_max || wf < -a.w_abs_max) {
          if (tid == 0 && tile == 0) atomic_inc64(a.bad_counter);
          wf = 0;
        }
        // residues are below 2^30, so they are valid signed 32-bit operands: one 32x32+64 multiply-add each
        s[f][0] += (int64_t)wf * (int64_t)(int32_t)x.x;
        s[f][1] += (int64_t)wf * (int64_t)(int32_t)x.y;
        s[f][2] += (int64_t)wf * (int64_t)(int32_t)x.z;
        s[f][3] += (int64_t)wf * (int64_t)(int32_t)x.w;
      }
      if (++since == a.chunk) {
        since = 0;
#pragma unroll
        for (int f = 0; f < FT; ++f)
          for (int q = 0; q < 4; ++q) s[f][q] = fold(s[f][q], m);
      }
    }
#pragma unroll
    for (int f = 0; f < FT; ++f) {
      U4 r;
      r.x = (uint32_t)fold(s[f][0], m); r.y = (uint32_t)fold(s[f][1], m);
      r.z = (uint32_t)fold(s[f][2], m); r.w = (uint32_t)fold(s[f][3], m);
      *reinterpret_cast<U4*>(a.out + ((size_t)f * a.G + g) * ct_words + pos) = r;
    }
  }
};

// Main variant: the gather row and the F*T weights of the group are staged in LDS once per
// workgroup (validated while staging: a bad index or weight becomes a zero-weight term on input 0;
// the row is padded to a multiple of kMacBatch with zero-weight terms on its last input), so the
// term loop reads them with broadcast LDS reads and carries no data-dependent branches.  Inputs are fetched kMacBatch terms
// ahead of their use (double buffering in registers) to keep HBM requests in flight during the
// multiply-adds.  Requires chunk % kMacBatch == 0.
// SKIP: the multiply-adds of the padding terms are skipped (a branch in the term loop, uniform over the workgroup).
// Measured: 6 % faster at 8 filters x 27 terms, nothing at 5 x 25, 14 % slower at 16 filters and hundreds of
// terms (where nothing is padded); the host picks the form by filter count and row length.
constexpr uint32_t kMacBatch = 4;
template <int FT, bool SKIP = false>
struct MacKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 2;
  struct Regs {};
  static size_t padded_terms(size_t T) { return (T + kMacBatch - 1) / kMacBatch * kMacBatch; }
  static size_t lds_bytes(size_t F, size_t T) { return ((1 + F) * padded_terms(T) + 2 * kMacBatch) * 4; }
  static size_t grid(size_t tiles, size_t G) { return kXcds * ((tiles + kXcds - 1) / kXcds) * G; }
  template <int PH>
  HCNN_HD static void phase(const MacArgs& a, unsigned bid, int tid, uint32_t* lds, Regs&) {
    const uint32_t ct_words32 = 2u * a.k * a.n;                       // at most 2^22
    const size_t ct_words = ct_words32;
    const uint32_t tiles = ct_words32 / (kThreads * kEwVec);
    // Workgroups go to the 8 XCDs round-robin by index, and each XCD has its own L2.  XCD x sweeps
    // the coefficient tiles x, x+8, ... and, inside a tile, the groups in order: the blocks that are
    // resident on one XCD at a time then share their gather rows' inputs (neighbouring filter
    // placements overlap), so every input tile is fetched from HBM about once.
    const uint32_t xcd = bid % kXcds, local = bid / kXcds;
    const uint32_t tile = (local / a.G) * kXcds + xcd;
    const uint32_t g = local % a.G;
    if (tile >= tiles) return;                                        // padding blocks (whole block)
    const uint32_t Tpad = (a.T + kMacBatch - 1) / kMacBatch * kMacBatch;
    uint32_t* l_idx = lds;                                            // [Tpad + 2*kMacBatch]
    int32_t* l_w = reinterpret_cast<int32_t*>(lds + Tpad + 2 * kMacBatch);   // [F][Tpad]
    if constexpr (PH == 0) {
      const uint32_t* idx = a.idx + (size_t)g * a.T;
      const int32_t* w = a.w + (size_t)g * a.F * a.T;
      for (uint32_t tau = tid; tau < Tpad + 2 * kMacBatch; tau += kThreads) {
        // the padding terms and the read-ahead slots of the last batches fetch the row's last input once more
        // (the compute unit's cache has just seen it); padding terms carry weight zero, read-ahead slots are never
        // consumed
        const bool pad = tau >= a.T;
        uint32_t src = idx[pad ? a.T - 1 : tau];
        const bool bad_src = src >= a.n_in;
        if (bad_src) {
          src = 0;
          if (tile == 0 && !pad) atomic_inc64(a.bad_counter);
        }
        l_idx[tau] = src * (ct_words32 / 4);   // offset of the input in 16-byte units (the host checked that it fits)
        if (tau >= Tpad) continue;
#pragma unroll
        for (int f = 0; f < FT; ++f) {
          int32_t wf = pad ? 0 : w[(size_t)f * a.T + tau];
          if (wf > a.w_abs_max || wf < -a.w_abs_max) {
            wf = 0;
            if (tile == 0) atomic_inc64(a.bad_counter);
          }
          l_w[(size_t)f * Tpad + tau] = bad_src ? 0 : wf;
        }
      }
    } else {
      const uint32_t pos = (tile * kThreads + tid) * kEwVec;          // word offset inside a ciphertext
      const uint32_t row = tile / (a.n / (kThreads * kEwVec));        // (poly, limb) row; uniform in the block
      const Mod m = ldc(a.mods, row % a.k);
      const U4* in = reinterpret_cast<const U4*>(a.in + pos);
      // accumulators carry the bias p*2^33 (a multiple of p above 2^62), so they stay positive while
      // the signed partial sums stay inside (-2^62, 2^62) and one unsigned reduction folds them
      const uint64_t bias = (uint64_t)m.p << 33;
      uint64_t s[FT][4];
#pragma unroll
      for (int f = 0; f < FT; ++f) { s[f][0] = bias; s[f][1] = bias; s[f][2] = bias; s[f][3] = bias; }
      auto fetch = [&](U4 (&buf)[kMacBatch], uint32_t t) {
#pragma unroll
        for (uint32_t b = 0; b < kMacBatch; ++b)
          buf[b] = in[(size_t)l_idx[t + b]];
      };
      auto consume = [&](const U4 (&buf)[kMacBatch], uint32_t t) {
#pragma unroll
        for (uint32_t b = 0; b < kMacBatch; ++b) {
          if constexpr (SKIP) {
            if (t + b >= a.T) break;            // padding terms of the last batch
          }
#pragma unroll
          for (int f = 0; f < FT; ++f) {
            const int64_t wf = l_w[(size_t)f * Tpad + t + b];
            // residues are below 2^30, so they are valid signed 32-bit operands: one 32x32+64 multiply-add each
            s[f][0] += (uint64_t)(wf * (int64_t)(int32_t)buf[b].x);
            s[f][1] += (uint64_t)(wf * (int64_t)(int32_t)buf[b].y);
            s[f][2] += (uint64_t)(wf * (int64_t)(int32_t)buf[b].z);
            s[f][3] += (uint64_t)(wf * (int64_t)(int32_t)buf[b].w);
          }
        }
      };
      auto refold = [&]() {
#pragma unroll
        for (int f = 0; f < FT; ++f)
          for (int q = 0; q < 4; ++q) s[f][q] = bias + reduce64(s[f][q], m);
      };
      // two register buffers used alternately: the loads of the next batch are in flight while the
      // current one is consumed.  Every fetch is unconditional (the gather row is followed by 2*kMacBatch
      // entries that name its last input again) so that the number of loads in flight is the same on every path
      // and the compiler can wait for exactly the older batch.
      U4 buf_a[kMacBatch], buf_b[kMacBatch];
      fetch(buf_a, 0);
      uint32_t since = 0;
      for (uint32_t tau = 0; tau < Tpad; tau += 2 * kMacBatch) {
        fetch(buf_b, tau + kMacBatch);
        if (since >= a.chunk) { since = 0; refold(); }
        since += kMacBatch;
        consume(buf_a, tau);
        fetch(buf_a, tau + 2 * kMacBatch);
        if (tau + kMacBatch < Tpad) {
          if (since >= a.chunk) { since = 0; refold(); }
          since += kMacBatch;
          consume(buf_b, tau + kMacBatch);
        }
      }
#pragma unroll
      for (int f = 0; f < FT; ++f) {
        U4 r;
        r.x = reduce64(s[f][0], m); r.y = reduce64(s[f][1], m);
        r.z = reduce64(s[f][2], m); r.w = reduce64(s[f][3], m);
        *reinterpret_cast<U4*>(a.out + ((size_t)f * a.G + g) * ct_words + pos) = r;
      }
    }
  }
};

// ---------------------------------------------------------------- helpers for KeyGen / Encrypt / Decrypt
// small signed polynomial(s) [count][n] -> residues [count][k][n]
struct SmallToRnsArgs {
  const int32_t* small;
  uint32_t* out;
  const Mod* mods;
  uint32_t k, n;
};
struct SmallToRnsKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  template <int PH>
  HCNN_HD static void phase(const SmallToRnsArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    const uint32_t per_poly = a.n / kThreads;
    const size_t poly = bid / per_poly;
    const uint32_t c = (bid % per_poly) * kThreads + tid;
    const int32_t v = a.small[poly * a.n + c];
    for (uint32_t l = 0; l < a.k; ++l) a.out[(poly * a.k + l) * a.n + c] = small_to_res(v, ldc(a.mods, l));
  }
};

// Pointwise c = a (*) b over rows; row r of a is a_rows[r % a_cycle], likewise b; limb = r % k.
// mode: 0 -> c = a*b ; 1 -> c = -(a*b)
struct PointMulArgs {
  const uint32_t* a;
  const uint32_t* b;
  uint32_t* c;
  const Mod* mods;
  uint32_t k, n;
  uint32_t a_cycle, b_cycle;   // in rows
  uint32_t negate;
};
struct PointMulKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  template <int PH>
  HCNN_HD static void phase(const PointMulArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    const uint32_t per_row = a.n / kThreads;
    const size_t row = bid / per_row;
    const uint32_t c = (bid % per_row) * kThreads + tid;
    const Mod m = ldc(a.mods, row % a.k);
    const uint32_t x = a.a[(row % a.a_cycle) * a.n + c];
    const uint32_t y = a.b[(row % a.b_cycle) * a.n + c];
    uint32_t r = mul_mod(x, y, m);
    if (a.negate && r != 0) r = m.p - r;
    a.c[row * a.n + c] = r;
  }
};

// out[row] = x[row] + small[poly(row)] (+ scale_l * msg[poly(row)]) ; rows are [count][k][n]
struct AddSmallArgs {
  const uint32_t* x;
  const int32_t* small;        // [count][n]
  const uint32_t* msg;         // [count][n] or null
  const uint64_t* msg64;       // [count][n] or null: the plaintext in 64-bit words (plaintext modulus above 2^32)
  const ShoupConst* scale;     // [k] (floor(q/t) mod q_l) or null
  uint32_t* out;
  const Mod* mods;
  uint32_t k, n;
  uint32_t subtract_small;     // 1: out = x - small
  uint32_t out_poly_rows, out_row0;   // output row = poly*out_poly_rows + out_row0 + l
};
struct AddSmallKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  template <int PH>
  HCNN_HD static void phase(const AddSmallArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    const uint32_t per_row = a.n / kThreads;
    const size_t row = bid / per_row;                  // (poly, l)
    const uint32_t c = (bid % per_row) * kThreads + tid;
    const size_t poly = row / a.k;
    const uint32_t l = (uint32_t)(row % a.k);
    const Mod m = ldc(a.mods, l);
    const uint32_t sv = small_to_res(a.small[poly * a.n + c], m);
    uint32_t r = a.subtract_small ? sub_mod(a.x[row * a.n + c], sv, m.p) : add_mod(a.x[row * a.n + c], sv, m.p);
    if (a.msg) r = add_mod(r, shoup_mul(reduce32(a.msg[poly * a.n + c], m), ldc(a.scale, l), m.p), m.p);
    if (a.msg64) r = add_mod(r, shoup_mul(reduce64(a.msg64[poly * a.n + c], m), ldc(a.scale, l), m.p), m.p);
    a.out[(poly * a.out_poly_rows + a.out_row0 + l) * a.n + c] = r;
  }
};

// evk[i][0][i] += s2[i] for i < k  (g_i = 1 mod q_i and 0 mod every other prime)
struct AddDiagArgs {
  uint32_t* evk;          // [k][2][k][n]
  const uint32_t* s2;     // [k][n]
  const Mod* mods;
  uint32_t k, n;
};
struct AddDiagKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  template <int PH>
  HCNN_HD static void phase(const AddDiagArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    const uint32_t per_row = a.n / kThreads;
    const uint32_t i = bid / per_row;
    const uint32_t c = (bid % per_row) * kThreads + tid;
    uint32_t* dst = a.evk + (((size_t)i * 2 + 0) * a.k + i) * a.n + c;
    *dst = add_mod(*dst, a.s2[(size_t)i * a.n + c], ldc(a.mods, i).p);
  }
};

// c = a + b over `rows` rows [..][k][n]
struct AddRowsArgs {
  const uint32_t* a;
  const uint32_t* b;
  uint32_t* c;
  const Mod* mods;
  uint32_t k, n;
  uint32_t a_poly_rows, a_row0;   // a row = (poly*a_poly_rows + a_row0 + l); b and c are dense [poly][k]
};
struct AddRowsKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  template <int PH>
  HCNN_HD static void phase(const AddRowsArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    const uint32_t per_row = a.n / kThreads;
    const size_t row = bid / per_row;
    const uint32_t c = (bid % per_row) * kThreads + tid;
    const size_t poly = row / a.k;
    const uint32_t l = (uint32_t)(row % a.k);
    const uint32_t p = ldc(a.mods, l).p;
    a.c[row * a.n + c] = add_mod(a.a[(poly * a.a_poly_rows + a.a_row0 + l) * a.n + c], a.b[row * a.n + c], p);
  }
};

// Decrypt rounding: x [count][k][n] (c0 + c1*s mod q) -> m = round(t*x/q) mod t.
// r = [t*x]_q centred is converted to the single modulus t; m = -r * q^-1 mod t.
struct DecRoundArgs {
  const uint32_t* x;
  uint32_t* m_out;
  BConvDev bc;             // src q (zmul = t*(q/q_i)^-1, xmul = t), dst {t}: Bp = q/q_i mod t, Vp = t - (q mod t)
  uint32_t t, neg_qinv_t;  // -q^-1 mod t
  uint32_t n;
  uint32_t band;
  unsigned long long* fallback_counter;
};
struct DecRoundKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  static size_t lds_bytes(uint32_t ks) { return (size_t)2 * ks * kThreads * 4; }
  template <int PH>
  HCNN_HD static void phase(const DecRoundArgs& a, unsigned bid, int tid, uint32_t* lds, Regs&) {
    const uint32_t ks = a.bc.ks, n = a.n;
    const uint32_t per_poly = n / kThreads;
    const size_t poly = bid / per_poly;
    const uint32_t c = (bid % per_poly) * kThreads + tid;
    const uint32_t* src = a.x + poly * ks * n + c;
    uint32_t* zcol = lds + tid;
    uint32_t* gcol = lds + (size_t)ks * kThreads + tid;
    auto in = [&](uint32_t i) { return src[(size_t)i * n]; };
    const uint32_t v = bconv_prepare(a.bc, in, zcol, gcol, kThreads, a.band, a.fallback_counter);
    // the destination modulus t is small: plain 64-bit remainder (test helper, not tuned)
    uint64_t acc = ((uint64_t)v * ldc(a.bc.Vp, 0)) % a.t;
    for (uint32_t i = 0; i < ks; ++i) acc = (acc + (uint64_t)zcol[i * kThreads] * ldc(a.bc.Bp, i)) % a.t;
    a.m_out[poly * n + c] = (uint32_t)((acc * a.neg_qinv_t) % a.t);
  }
};

// Decrypt rounding for a plaintext modulus of up to 47 bits (64-bit plaintext words).  Same conversion as above
// with the destination arithmetic done modulo t in 64-bit words: a 32-bit by 47-bit product is formed from
// two 16-bit halves, each partial product below 2^63.
struct DecRoundWideArgs {
  const uint32_t* x;
  uint64_t* m_out;
  BConvDev bc;             // source side only (zmul = t*(q/q_i)^-1, xmul = t)
  const uint64_t* tab;     // [ks + 2]: (q/q_i) mod t for i < ks, then t - (q mod t), then -q^-1 mod t
  uint64_t t;
  uint32_t n;
  uint32_t band;
  unsigned long long* fallback_counter;
};
HCNN_HD uint64_t mul32_mod_wide(uint32_t a, uint64_t b, uint64_t t) {     // a*b mod t for b < t < 2^47
  uint64_t r = ((uint64_t)(a >> 16) * b) % t;
  r = (r << 16) % t;
  return (r + ((uint64_t)(a & 0xffffu) * b) % t) % t;
}
HCNN_HD uint64_t mul_mod_wide(uint64_t a, uint64_t b, uint64_t t) {       // a*b mod t for a, b < t < 2^47
  uint64_t r = mul32_mod_wide((uint32_t)(a >> 32), b, t);                  // a = hi*2^32 + lo
  r = (r << 16) % t;
  r = (r << 16) % t;
  return (r + mul32_mod_wide((uint32_t)a, b, t)) % t;
}
struct DecRoundWideKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  static size_t lds_bytes(uint32_t ks) { return (size_t)2 * ks * kThreads * 4; }
  template <int PH>
  HCNN_HD static void phase(const DecRoundWideArgs& a, unsigned bid, int tid, uint32_t* lds, Regs&) {
    const uint32_t ks = a.bc.ks, n = a.n;
    const uint32_t per_poly = n / kThreads;
    const size_t poly = bid / per_poly;
    const uint32_t c = (bid % per_poly) * kThreads + tid;
    const uint32_t* src = a.x + poly * ks * n + c;
    uint32_t* zcol = lds + tid;
    uint32_t* gcol = lds + (size_t)ks * kThreads + tid;
    auto in = [&](uint32_t i) { return src[(size_t)i * n]; };
    const uint32_t v = bconv_prepare(a.bc, in, zcol, gcol, kThreads, a.band, a.fallback_counter);
    uint64_t acc = mul32_mod_wide(v, a.tab[ks], a.t);
    for (uint32_t i = 0; i < ks; ++i) acc = (acc + mul32_mod_wide(zcol[i * kThreads], a.tab[i], a.t)) % a.t;
    a.m_out[poly * n + c] = mul_mod_wide(acc, a.tab[ks + 1], a.t);
  }
};

// ---------------------------------------------------------------- counter-based sampling
// Every output element is a fixed function of (seed, stream, element index): the word source is Philox4x32 with
// 10 rounds (Salmon et al., SC'11) keyed by the seed, with counter (index low, index high, stream, kind*2^24 +
// attempt); a call gives four words, used in order, and a sampler that needs more moves on to attempt + 1.
struct PhiloxWords { uint32_t w[4]; };
HCNN_HD PhiloxWords philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)c0 * 0xD2511F53u, p1 = (uint64_t)c2 * 0xCD9E8D57u;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  PhiloxWords r; r.w[0] = c0; r.w[1] = c1; r.w[2] = c2; r.w[3] = c3;
  return r;
}
enum { kSampleTernary = 1, kSampleGaussian = 2, kSampleUniform = 3 };
constexpr uint32_t kSampleMaxAttempts = 256;   // 1024 words: no sampler comes anywhere near (rejection odds <= 2^-29 per try,
                                               // or 1 - 4p/2^32 for a prime p > 2^29 that is not close to 2^30)
struct SampleArgs {
  void* out;                 // int32 [count][n] (ternary, Gaussian) or uint32 [count][k][n] (uniform)
  const Mod* mods;           // uniform: [k]
  const uint32_t* gauss_t;   // Gaussian: 20 thresholds, T[v] = floor(2^32 * P(|X| <= v))
  uint64_t seed, total;      // total elements
  uint32_t stream, kind, k, n;
};
struct SampleKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  template <int PH>
  HCNN_HD static void phase(const SampleArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    const uint64_t idx = (uint64_t)bid * kThreads + (uint64_t)tid;
    if (idx >= a.total) return;
    const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
    uint32_t p = 0, lim = 0;
    if (a.kind == kSampleUniform) {
      p = ldc(a.mods, (uint32_t)((idx / a.n) % a.k)).p;
      lim = p * (uint32_t)(0x100000000ull / p);                    // accepted words: below the largest multiple of p
    }
    for (uint32_t attempt = 0; attempt < kSampleMaxAttempts; ++attempt) {
      const PhiloxWords r = philox4x32_10((uint32_t)idx, (uint32_t)(idx >> 32), a.stream, (a.kind << 24) + attempt, k0, k1);
      if (a.kind == kSampleGaussian) {
        for (int s = 0; s < 4; s += 2) {
          const uint32_t x = r.w[s], y = r.w[s + 1];
          if (x >= ldc(a.gauss_t, 19)) continue;                    // beyond the cut: redraw
          int32_t mag = 0;
          for (uint32_t v = 0; v < 20; ++v) mag += ldc(a.gauss_t, v) <= x ? 1 : 0;
          reinterpret_cast<int32_t*>(a.out)[idx] = (y & 1u) ? -mag : mag;
          return;
        }
      } else {
        for (int s = 0; s < 4; ++s) {
          const uint32_t x = r.w[s];
          if (a.kind == kSampleTernary) {
            if (x == 0xFFFFFFFFu) continue;                         // 2^32 - 1 words split evenly over three values
            reinterpret_cast<int32_t*>(a.out)[idx] = (int32_t)(x % 3u) - 1;
          } else {
            if (x >= lim) continue;
            reinterpret_cast<uint32_t*>(a.out)[idx] = x % p;
          }
          return;
        }
      }
    }
    reinterpret_cast<uint32_t*>(a.out)[idx] = 0;                    // not reached in practice (see kSampleMaxAttempts)
  }
};

// Noise read-out: x [count][k][n] (c0 + c1*s mod q) -> bits[count] = bit length of max_j |r_j|, r = [t*x]_q centred.
// Exact: the residues of the non-negative remainder R = t*x mod q are turned into mixed-radix digits, R > (q-1)/2
// is decided on the digits, |r| = R or q - R is rebuilt as a multiword integer by Horner's rule on the digits, and its
// bit length is folded into the ciphertext's maximum.  bits[] must be zero on entry.
struct NoiseArgs {
  const uint32_t* x;
  uint32_t* bits;
  BConvDev bc;             // src q with xmul = t (the table of the decrypt rounding)
  uint32_t n;
};
struct NoiseKernel {
  static constexpr int kThreads = kEwThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  static size_t lds_bytes(uint32_t ks) { return (size_t)2 * ks * kThreads * 4; }
  template <int PH>
  HCNN_HD static void phase(const NoiseArgs& a, unsigned bid, int tid, uint32_t* lds, Regs&) {
    const uint32_t ks = a.bc.ks, n = a.n;
    const uint32_t per_poly = n / kThreads;
    const size_t poly = bid / per_poly;
    const uint32_t c = (bid % per_poly) * kThreads + tid;
    const uint32_t* src = a.x + poly * ks * n + c;
    uint32_t* dig = lds + tid;                                   // mixed-radix digits
    uint32_t* word = lds + (size_t)ks * kThreads + tid;          // multiword |r|, least significant first
    for (uint32_t i = 0; i < ks; ++i)
      dig[i * kThreads] = shoup_mul(src[(size_t)i * n], ldc(a.bc.xmul, i), ldc(a.bc.src_mod, i).p);
    if (garner_gt_half(a.bc, dig, kThreads)) {
      // digits of q - R: zero while the lower digits of R are zero, q_i - d_i at the first non-zero digit,
      // q_i - 1 - d_i above it
      bool low_zero = true;
      for (uint32_t i = 0; i < ks; ++i) {
        const uint32_t d = dig[i * kThreads], qi = ldc(a.bc.src_mod, i).p;
        if (low_zero) {
          if (d != 0) { dig[i * kThreads] = qi - d; low_zero = false; }
        } else {
          dig[i * kThreads] = qi - 1 - d;
        }
      }
    }
    // value = d_0 + q_0*(d_1 + q_1*(d_2 + ...)): Horner from the top digit; it stays below q < 2^(30 ks)
    for (uint32_t w = 0; w < ks; ++w) word[w * kThreads] = 0;
    for (int i = (int)ks - 1; i >= 0; --i) {
      uint64_t carry = dig[i * kThreads];
      const uint64_t qi = ldc(a.bc.src_mod, (uint32_t)i).p;
      for (uint32_t w = 0; w < ks; ++w) {
        const uint64_t v = (uint64_t)word[w * kThreads] * qi + carry;
        word[w * kThreads] = (uint32_t)v;
        carry = v >> 32;
      }
    }
    uint32_t bits = 0;
    for (int w = (int)ks - 1; w >= 0; --w) {
      uint32_t v = word[w * kThreads];
      if (v != 0) {
        uint32_t len = 0;
        while (v) { ++len; v >>= 1; }
        bits = 32u * (uint32_t)w + len;
        break;
      }
    }
    if (bits) atomic_max32(a.bits + poly, bits);
  }
};

}  // namespace hcnn
