// Batched negacyclic NTT over 30-bit primes, one workgroup per (polynomial, limb) row.
//
// Forward: Cooley-Tukey butterflies with the powers of psi merged into the
// twiddles, natural order in, bit-reversed order out (index j holds the value at
// psi^(2*brev(j)+1)).  Inverse: Gentleman-Sande butterflies with the inverse
// twiddles in the reverse stage order, n^-1 merged into the last stage.
//
// The log2(n) stages are cut into passes of at most LOGR stages.  In a pass every
// thread keeps R = 2^LOGR residues in registers and runs complete radix-2^NS
// butterfly networks on them; between passes the row lives in LDS (one barrier per
// pass).  The first pass reads HBM with unit stride across lanes, the last pass
// writes HBM.  Residues stay lazily reduced (forward: [0,4p), inverse: [0,2p)) and
// are made canonical only on the way out.
//
// Twiddle table layout: tw[limb][node], node in [1, n): the butterflies of the stage
// with m groups use nodes m .. 2m-1 (node m+i = psi^brev_{log n}(m+i)); a radix-2^NS
// network rooted at node r uses the sub-tree r, 2r, 2r+1, 4r, ...
#pragma once
#include "modarith.h"

namespace hcnn {

struct NttLimb {
  Mod m;
  ShoupConst ninv;    // n^-1 mod p
  ShoupConst w1ninv;  // (inverse twiddle of node 1) * n^-1 mod p
  // the tensor-forming loads multiply with a Montgomery reduction, which leaves a factor 2^-32 on every
  // product; their transforms scale by n^-1 * 2^32 at the end instead of n^-1
  ShoupConst ninv_r;    // n^-1 * 2^32 mod p
  ShoupConst w1ninv_r;  // (inverse twiddle of node 1) * n^-1 * 2^32 mod p
  uint32_t pinv;        // -p^-1 mod 2^32
  uint32_t pneg;        // -p mod 2^32.  The compiler folds a 32-bit product into a following addition (one multiply-add)
                        // but not into a subtraction: written x*w + q*pneg, the lazy product x*w - q*p is a
                        // multiplication and a multiply-add.  The word has to come from memory for that: a negation
                        // the compiler can see is turned back into the subtraction.
  uint32_t zero;        // 0, unknown to the compiler: zero - w is the negated twiddle and stays one (see the inverse butterfly)
  uint32_t pad;
};

// Row r (= workgroup index) belongs to group r / limb_cycle and limb limb_base + r % limb_cycle.
// Its data sits at row (group * group_rows + row0 + r % limb_cycle) of the in / out arrays, so a
// launch can pick one polynomial out of every ciphertext of a batch.
// Fused input / output stages (template parameter IO of the kernels):
//   kNttPlain       rows are read and written as they are
//   kNttLoadDigit   forward only: row (ct, i, j) reads digit i of y2, i.e. row (ct*3+2)*k + i of `in`
//                   = y[n_ct][3][k][n], taken as it is (every prime lies in (2^29, 2^30), so a digit is below
//                   2*q_j, which the lazy butterflies accept); output rows dense [ct][i][j]
//   kNttLoadTensor  inverse only: row (ct, b, l) reads c0^ = in[(ct*2)*L + l], c1^ = in[(ct*2+1)*L + l]
//                   and transforms c0^*c0^, 2*c0^*c1^ or c1^*c1^ for b = 0, 1, 2 (HMult step 1, c = c')
//   kNttLoadTensorMul  inverse only: the general tensor of HMult step 1 for two different operands;
//                   `in` holds the first, `aux` the second (same [ct][2][L][n] layout):
//                   c0^*c0'^, c0^*c1'^ + c1^*c0'^, c1^*c1'^
//   kNttStoreAdd    inverse only: row (ct, b, j) adds aux row (ct*3+b)*k + j (aux = y) on the way out
//   kNttStoreLazy   forward only: the output is left lazily reduced in [0, 2p) (for rows whose only reader is
//                   the tensor-forming load: products of two such values are below p * 2^32, the range of
//                   its Montgomery reduction)
// The tensor-forming loads also leave their output lazily reduced, in [0, 2p): its only reader multiplies it
// by a constant with Shoup's method, which takes any 32-bit operand.
//   kNttFusedMac    forward only, inside RelinFused: workgroup (ct, j) transforms digit `iter` of y2 modulo q_j
//                   (loaded like kNttLoadDigit) and, instead of storing, adds its products with the two key
//                   rows evk^[iter][0][j], evk^[iter][1][j] (`aux`) to 64-bit sums held in registers
//   kNttFromRegs0/1 inverse only, inside RelinFused: the input is the register-held sum of component 0 / 1;
//                   the output adds y row (ct, b, j) (`aux`) like kNttStoreAdd and goes to out row (ct, b, j)
enum NttIo { kNttPlain = 0, kNttLoadDigit = 1, kNttLoadTensor = 2, kNttStoreAdd = 3, kNttLoadTensorMul = 4,
             kNttStoreLazy = 5, kNttFusedMac = 6, kNttFromRegs0 = 7, kNttFromRegs1 = 8,
             kNttFusedMac16 = 9, kNttFusedMacAny = 10,     // the fused inner product for k <= 8, k <= 16, any k
             kNttToRegs0 = 11, kNttToRegs1 = 12,           // forward, inside TensorFused: c0 / c1 of workgroup (ct, limb); the
                                                           // transformed row stays in registers, lazily reduced in [0, 2p)
             kNttTensorRegs0 = 13, kNttTensorRegs1 = 14, kNttTensorRegs2 = 15 };   // inverse, inside TensorFused: component
                                                           // b of the tensor formed from those registers (as kNttLoadTensor)

// Per-thread state of TensorFused: the two transformed polynomials of the ciphertext, one limb.
template <int R>
struct TensorRegs {
  uint32_t c0[R], c1[R];
};

// Per-thread state of RelinFused: the iteration (digit) and the two inner-product sums of every residue the
// thread holds after the last forward pass.
template <int R>
struct RelinRegs {
  uint32_t iter;
  uint64_t s0[R], s1[R];
};
struct NoRegs {};

struct NttArgs {
  const uint32_t* in;
  uint32_t* out;            // may equal `in`
  const uint32_t* aux;      // kNttStoreAdd: the addend; kNttLoadTensorMul: the second operand
  const ShoupConst* tw;     // [L][n] node table (forward: {-w mod 2^32, w'}; inverse: {w, w'})
  const NttLimb* limbs;     // [L]
  uint32_t limb_cycle;
  uint32_t limb_base;
  uint32_t in_group_rows, in_row0;
  uint32_t out_group_rows, out_row0;
  uint32_t n_rows;          // rows of this launch (the grid may be padded, see ntt_logical_row)
  uint32_t own_limbs;       // kNttStoreLazy with `aux` set: rows of the first own_limbs limbs of every group are read from
                            // aux, laid out [group][own_limbs][n] (a ciphertext's own limbs), the others from `in`
};

// Workgroups are handed to the 8 accelerator dies round-robin by index, and each die has its own
// L2.  The fused loads read one source row from several workgroups (a digit row feeds k transforms,
// a c0^/c1^ row feeds two tensor components); this maps the workgroup index to a row so that the
// `share` rows that read the same source run on the same die, next to each other in time.
// Rows are numbered unit*share + within for the digit load (within = j) and the caller converts
// for the tensor load.  Returns n_rows or more for the padding workgroups of the last round.
constexpr uint32_t kNttXcds = 8;
HCNN_HD uint32_t ntt_grouped_index(uint32_t bid, uint32_t share) {
  const uint32_t xcd = bid % kNttXcds, local = bid / kNttXcds;
  return ((local / share) * kNttXcds + xcd) * share + local % share;
}
inline size_t ntt_grouped_grid(size_t rows, size_t share) {
  const size_t units = rows / share;
  return (units + kNttXcds - 1) / kNttXcds * kNttXcds * share;
}

HCNN_HD size_t ntt_row(uint32_t r, uint32_t cycle, uint32_t group_rows, uint32_t row0) {
  return (size_t)(r / cycle) * group_rows + row0 + r % cycle;
}

// LDS layout: one unused word after every 32, which spreads the power-of-two strides of the passes
// over the 32 banks.  The map a -> a + a/32 is additive over operands with disjoint bit fields (no
// carries), and the element e of a network sits at base | (e << LOG_TLAST) with those bits of base
// clear: its LDS word is pad(base) + pad(e << LOG_TLAST), a register plus a compile-time offset.
HCNN_HD constexpr uint32_t lds_swz(uint32_t i) { return i + (i >> 5); }
template <int LOG_TLAST>
HCNN_HD constexpr uint32_t lds_elem(uint32_t sbase, int e) {
  return sbase + lds_swz((uint32_t)e << LOG_TLAST);
}

template <int LOGN, int LOGR>
struct NttGeom {
  static constexpr int N = 1 << LOGN;
  static constexpr int R = 1 << LOGR;
  static constexpr int kThreads = N / R;
  static constexpr int kPhases = (LOGN + LOGR - 1) / LOGR;
  static constexpr size_t kLdsBytes = (size_t)(N + N / 32) * 4;
  // forward pass PH covers stages [s0(PH), s0(PH)+ns(PH))
  static constexpr int s0(int ph) { return ph * LOGR; }
  static constexpr int ns(int ph) { return ph < kPhases - 1 ? LOGR : LOGN - LOGR * (kPhases - 1); }
};

// n = 32768: four passes of 5 + 4 + 4 + 2 stages.  The last forward pass (the first inverse one) has every thread store
// (load) 2^ns consecutive residues; with five stages there that is 128 bytes per lane, one cache line per lane and
// access, eight times the line accesses the bytes need.  Two stages there make it one 16-byte word per lane: the lanes of
// a wave touch consecutive words.  Measured against 5 + 5 + 5: whole-row forward 119 -> 98 ns per row, the inverse
// transforms of a squaring 123 -> 103, although the row makes one more trip through the LDS (5 + 5 + 3 + 2 and
// 4 + 5 + 4 + 2 are within 2 % of it; 5 + 5 + 4 + 1, eight bytes per lane, gains nothing).  The half-row network of
// that ring's two-workgroup forward transform (14 stages, 32 residues per thread) takes 5 + 4 + 3 + 2 for the same
// reason (2 % faster than 5 + 5 + 4).  At n = 8192 the three passes 5 + 5 + 3 (32 bytes per lane) stay: 5 + 4 + 2 + 2,
// 5 + 3 + 3 + 2 and 5 + 4 + 4 were each 3-5 % slower.
#define HCNN_GEOM_SPEC(LOGN_, LOGR_, NP_, ...)                                                        \
  template <>                                                                                          \
  struct NttGeom<LOGN_, LOGR_> {                                                                       \
    static constexpr int N = 1 << LOGN_;                                                               \
    static constexpr int R = 1 << LOGR_;                                                               \
    static constexpr int kThreads = N / R;                                                             \
    static constexpr int kPhases = NP_;                                                                \
    static constexpr size_t kLdsBytes = (size_t)(N + N / 32) * 4;                                      \
    static constexpr int kNs[NP_] = {__VA_ARGS__};                                                     \
    static constexpr int s0(int ph) { int s = 0; for (int i = 0; i < ph; ++i) s += kNs[i]; return s; } \
    static constexpr int ns(int ph) { return kNs[ph]; }                                                \
  };
HCNN_GEOM_SPEC(15, 5, 4, 5, 4, 4, 2)
HCNN_GEOM_SPEC(14, 5, 4, 5, 4, 3, 2)
HCNN_GEOM_SPEC(13, 4, 4, 4, 3, 4, 2)
#undef HCNN_GEOM_SPEC

// ------------------------------------------------------------------------- forward
// SPLIT = 1: two workgroups per row.  The first stage of the forward transform pairs element i with element
// i + n/2 and leaves two halves that never meet again; workgroup (row, half) computes its half of that stage while
// loading (it reads both halves of the row, the second reader out of L2) and then runs the remaining log2(n) - 1
// stages on n/2 residues.  Half the LDS and half the threads per workgroup: for the largest ring, whose whole row
// fills the LDS of a compute unit, two workgroups fit where one did, and they are out of step with each other.
template <int LOGN, int LOGR, int IO = kNttPlain, int SPLIT = 0>
struct NttFwd {
  static constexpr bool kFused = IO == kNttFusedMac || IO == kNttFusedMac16 || IO == kNttFusedMacAny;
  static constexpr bool kToRegs = IO == kNttToRegs0 || IO == kNttToRegs1;
  static_assert(IO == kNttPlain || IO == kNttLoadDigit || IO == kNttStoreLazy || kFused || kToRegs,
                "forward NTT: plain, digit load, lazy store, fused inner product or register output");
  static_assert(SPLIT == 0 || (SPLIT == 1 && !kFused && !kToRegs), "the split form stores its rows");
  using G = NttGeom<LOGN - SPLIT, LOGR>;      // the stages after the split one
  static constexpr int kThreads = G::kThreads;
  static constexpr int kPhases = G::kPhases;
  static constexpr bool kDigitIn = IO == kNttLoadDigit || kFused;
  using Regs = std::conditional_t<kFused, RelinRegs<G::R>, std::conditional_t<kToRegs, TensorRegs<G::R>, NoRegs>>;
  // workgroups of a launch over `slots` row positions (a multiple of the die count for the split form)
  static size_t grid(size_t slots) { return SPLIT ? 2 * ((slots + kNttXcds - 1) / kNttXcds * kNttXcds) : slots; }

  template <int PH>
  HCNN_HD static void phase(const NttArgs& a, unsigned bid, int tid, uint32_t* lds, Regs& regs) {
    constexpr int N = 1 << LOGN, R = G::R;                 // N: residues of a row in memory
    constexpr int LOGM = LOGN - SPLIT;                     // stages S0 .. of this workgroup run on 2^LOGM residues
    constexpr int S0 = G::s0(PH), NS = G::ns(PH), NET = 1 << NS, C = R / NET;
    constexpr int LOG_TLAST = LOGM - S0 - NS, TLAST = 1 << LOG_TLAST;
    constexpr bool kFirst = PH == 0, kLast = PH == kPhases - 1;
    if constexpr (kFused || kToRegs) tid = opaque(tid);

    uint32_t half = 0;
    if constexpr (SPLIT) {
      // both halves of a row on one die, next to each other in time
      half = (bid / kNttXcds) & 1u;
      bid = (bid / (2 * kNttXcds)) * kNttXcds + bid % kNttXcds;
      if constexpr (!kDigitIn) {
        if (bid >= a.n_rows) return;                       // padding workgroups of the last round
      }
    }
    if constexpr (kDigitIn) {
      bid = ntt_grouped_index(bid, a.limb_cycle);      // the k transforms of one digit row share a die
      if (bid >= a.n_rows) return;
    }
    const uint32_t limb = a.limb_base + bid % a.limb_cycle;
    const NttLimb L = ldc(a.limbs, limb);
    const uint32_t p = L.m.p, two_p = 2 * L.m.p;
    const ShoupConst* tw = a.tw + (size_t)limb * N;
    const uint32_t* gin;
    uint32_t* gout = nullptr;
    const uint32_t* key0 = nullptr;       // kNttFusedMac: evk^[iter][0][j]; component 1 lies k rows further
    if constexpr (kFused) {
      const uint32_t kk = a.limb_cycle;                // rows are (ct, j)
      gin = a.in + ((size_t)(bid / kk) * 3 * kk + 2 * kk + regs.iter) * N;
      key0 = a.aux + ((size_t)regs.iter * 2 * kk + limb) * N;
      if (kFirst && regs.iter == 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) { regs.s0[r] = 0; regs.s1[r] = 0; }
      }
    } else if constexpr (IO == kNttLoadDigit) {
      const uint32_t kk = a.limb_cycle;
      gin = a.in + ((size_t)(bid / (kk * kk)) * 3 * kk + 2 * kk + (bid / kk) % kk) * N;
    } else if constexpr (kToRegs) {
      // workgroup (ct, l): polynomial c0 or c1 of the ciphertext; its own limbs come from the ciphertext (`aux`,
      // [ct][2][own_limbs][n]), the auxiliary limbs from the extension buffer (`in`, [ct][2][L][n])
      const uint32_t LL = a.limb_cycle, poly = IO == kNttToRegs1 ? 1u : 0u;
      const size_t grp = (size_t)(bid / LL) * 2 + poly;
      if (bid >= a.n_rows) return;
      gin = limb < a.own_limbs ? a.aux + (grp * a.own_limbs + limb) * N : a.in + (grp * LL + limb) * N;
    } else {
      gin = a.in + ntt_row(bid, a.limb_cycle, a.in_group_rows, a.in_row0) * N;
      if constexpr (IO == kNttStoreLazy) {
        if (a.aux != nullptr && bid % a.limb_cycle < a.own_limbs)
          gin = a.aux + ((size_t)(bid / a.limb_cycle) * a.own_limbs + bid % a.limb_cycle) * N;
      }
    }
    if constexpr (!kFused && !kToRegs)
      gout = a.out + ntt_row(bid, a.limb_cycle, a.out_group_rows, a.out_row0) * N + (size_t)half * (N / 2);
    // split form: the butterfly of the first stage (node 1) on the way in -- this half's output of the pair
    // (i, i + n/2).  X is brought below 2p first (rows may arrive lazily reduced below 4p), the product T lies in
    // [0, 2p): X + T and X - T + 2p are valid inputs of the stages that follow.
    [[maybe_unused]] const ShoupConst w_split = SPLIT ? ldc(tw, 1) : ShoupConst{0, 0};
    auto load_first = [&](uint32_t idx) -> uint32_t {
      if constexpr (SPLIT) {
        const uint32_t X = csub(gin[idx], two_p), Y = gin[idx + N / 2];
        const uint32_t negT = mulhi32(Y, w_split.ws) * p + Y * w_split.w;
        return half ? X + two_p + negT : X - negT;
      } else {
        return gin[idx];
      }
    };

#pragma unroll
    for (int c = 0; c < C; ++c) {
      const uint32_t nu = (uint32_t)tid + (uint32_t)kThreads * c;   // network id
      const uint32_t o = nu & (TLAST - 1), i = nu >> LOG_TLAST;
      const uint32_t base = i * (uint32_t)(NET * TLAST) + o;        // element e at base + e*TLAST
      const uint32_t sbase = lds_swz(base);
      uint32_t v[NET];
#pragma unroll
      for (int e = 0; e < NET; ++e)
        v[e] = kFirst ? load_first(base + (uint32_t)e * TLAST) : lds[lds_elem<LOG_TLAST>(sbase, e)];
      // (kNttLoadDigit: a digit lies in [0, q_i) and every prime in (2^29, 2^30), so it is below 2p for this
      // row's prime p: a valid lazily reduced input of the butterflies as it stands)
      // node of the twiddle tree over the whole row: the half's own sub-tree in the split form
      const uint32_t root = SPLIT ? ((2u + half) << S0) + i : (1u << S0) + i;
#pragma unroll
      for (int l = 0; l < NS; ++l) {
        const int half = NET >> (l + 1);
#pragma unroll
        for (int h = 0; h < (1 << l); ++h) {
          const ShoupConst w = ldc(tw, (root << l) + h);
#pragma unroll
          for (int x = 0; x < half; ++x) {
            const int ia = h * 2 * half + x, ib = ia + half;
            const uint32_t X = csub(v[ia], two_p);                          // [0, 2p)
            // the forward table holds -w (mod 2^32): q*p - y*w is then a multiplication and a multiply-add
            const uint32_t negT = mulhi32(v[ib], w.ws) * p + v[ib] * w.w;   // -(y*w mod p) - {0,p}  (mod 2^32)
            v[ia] = X - negT;                                              // X + T        in [0, 4p)
            v[ib] = X + two_p + negT;                                      // X - T + 2p   in (0, 4p)
          }
        }
      }
      if constexpr (kLast && kFused) {
        // The transformed digit times the key rows (below p < 2^30), added to the 64-bit sums.  With the digit only
        // brought into [0, 2p), 8 products stay below 16 p^2 < 2^64 (kNttFusedMac, k <= 8); with the digit made
        // canonical, 16 products do, or 15 and a residue (kNttFusedMac16, k <= 16), and
        // kNttFusedMacAny folds the sums before digits 16, 31, 46, ...
        const uint32_t* key1 = key0 + (size_t)a.limb_cycle * N;
        uint32_t e0[NET], e1[NET];
#pragma unroll
        for (int e = 0; e < NET; ++e) { e0[e] = key0[base + (uint32_t)e]; e1[e] = key1[base + (uint32_t)e]; }
        if constexpr (IO == kNttFusedMacAny) {
          if (regs.iter >= 16 && (regs.iter - 16) % 15 == 0) {
#pragma unroll
            for (int e = 0; e < NET; ++e) {
              regs.s0[c * NET + e] = reduce64(regs.s0[c * NET + e], L.m);
              regs.s1[c * NET + e] = reduce64(regs.s1[c * NET + e], L.m);
            }
          }
        }
#pragma unroll
        for (int e = 0; e < NET; ++e) {
          uint32_t d = csub(v[e], two_p);
          if constexpr (IO != kNttFusedMac) d = csub(d, p);
          regs.s0[c * NET + e] += (uint64_t)d * e0[e];
          regs.s1[c * NET + e] += (uint64_t)d * e1[e];
        }
      } else if constexpr (kLast && kToRegs) {
#pragma unroll
        for (int e = 0; e < NET; ++e) {
          if constexpr (IO == kNttToRegs1) regs.c1[c * NET + e] = csub(v[e], two_p);
          else                             regs.c0[c * NET + e] = csub(v[e], two_p);
        }
      } else if constexpr (kLast && NET >= 4) {
        // TLAST == 1: the network is NET consecutive coefficients -> 16-byte stores
        U4* g4 = reinterpret_cast<U4*>(gout + base);
#pragma unroll
        for (int e = 0; e < NET; e += 4) {
          U4 t;
          if constexpr (IO == kNttStoreLazy) {
            t.x = csub(v[e + 0], two_p); t.y = csub(v[e + 1], two_p); t.z = csub(v[e + 2], two_p); t.w = csub(v[e + 3], two_p);
          } else {
            t.x = csub(csub(v[e + 0], two_p), p);
            t.y = csub(csub(v[e + 1], two_p), p);
            t.z = csub(csub(v[e + 2], two_p), p);
            t.w = csub(csub(v[e + 3], two_p), p);
          }
          g4[e / 4] = t;
        }
      } else {
#pragma unroll
        for (int e = 0; e < NET; ++e) {
          if (kLast) gout[base + (uint32_t)e * TLAST] = IO == kNttStoreLazy ? csub(v[e], two_p) : csub(csub(v[e], two_p), p);
          else       lds[lds_elem<LOG_TLAST>(sbase, e)] = v[e];
        }
      }
    }
  }
};

// ------------------------------------------------------------------------- inverse
template <int LOGN, int LOGR, int IO = kNttPlain>
struct NttInv {
  static_assert(IO == kNttPlain || IO == kNttLoadTensor || IO == kNttStoreAdd || IO == kNttLoadTensorMul ||
                IO == kNttFromRegs0 || IO == kNttFromRegs1 || IO == kNttTensorRegs0 || IO == kNttTensorRegs1 ||
                IO == kNttTensorRegs2, "inverse NTT io mode");
  using G = NttGeom<LOGN, LOGR>;
  static constexpr int kThreads = G::kThreads;
  static constexpr int kPhases = G::kPhases;
  // a 1024-thread workgroup whose row leaves LDS for a second one: keep the registers within what two of them need
  // (the plain transform of n = 16384 took 68 and ran alone on its compute unit, a third slower per row)
  static constexpr int kMinWavesPerSimd = (G::kThreads == 1024 && 2 * G::kLdsBytes <= 160 * 1024) ? 8 : 1;
  static constexpr bool kFromRegs = IO == kNttFromRegs0 || IO == kNttFromRegs1;
  static constexpr bool kTensorRegs = IO == kNttTensorRegs0 || IO == kNttTensorRegs1 || IO == kNttTensorRegs2;
  using Regs = std::conditional_t<kFromRegs, RelinRegs<G::R>, std::conditional_t<kTensorRegs, TensorRegs<G::R>, NoRegs>>;

  template <int PHI>
  HCNN_HD static void phase(const NttArgs& a, unsigned bid, int tid, uint32_t* lds, Regs& regs) {
    constexpr int PH = kPhases - 1 - PHI;   // mirrors forward pass PH
    constexpr int N = G::N, R = G::R;
    constexpr int S0 = G::s0(PH), NS = G::ns(PH), NET = 1 << NS, C = R / NET;
    constexpr int LOG_TLAST = LOGN - S0 - NS, TLAST = 1 << LOG_TLAST;
    constexpr bool kFirst = PHI == 0, kLast = PHI == kPhases - 1;   // kLast <=> S0 == 0

    if constexpr (IO == kNttLoadTensor || IO == kNttLoadTensorMul) {
      // the three components of one (ciphertext, limb) pair read the same c0^ / c1^ rows: same die
      const uint32_t LL = a.limb_cycle;
      const uint32_t g = ntt_grouped_index(bid, 3);            // unit = ct*L + l, within = component
      const uint32_t unit = g / 3, b = g % 3;
      bid = ((unit / LL) * 3 + b) * LL + unit % LL;            // row (ct, b, l)
      if (unit >= a.n_rows / 3) return;
    }
    if constexpr (kFromRegs) {
      bid = ntt_grouped_index(bid, a.limb_cycle);      // the same workgroup -> (ct, j) map as kNttFusedMac
      if (bid >= a.n_rows) return;
    }
    if constexpr (kTensorRegs) {
      tid = opaque(tid);
      if (bid >= a.n_rows) return;
    }
    const uint32_t limb = a.limb_base + bid % a.limb_cycle;
    const NttLimb L = ldc(a.limbs, limb);
    const uint32_t p = L.m.p, two_p = 2 * L.m.p;
    const ShoupConst* tw = a.tw + (size_t)limb * N;
    const uint32_t* gin = nullptr;
    const uint32_t* gin2 = nullptr;       // kNttLoadTensor: the c1^ row
    uint32_t comp = 0;                    // kNttLoadTensor: tensor component b
    const uint32_t* gmul0 = nullptr;      // kNttLoadTensorMul: rows c0^, c1^ of the first operand and
    const uint32_t* gmul1 = nullptr;      // c0'^, c1'^ of the second
    if constexpr (IO == kNttLoadTensor) {
      const uint32_t LL = a.limb_cycle;
      const uint32_t ct = bid / (3 * LL);
      comp = (bid / LL) % 3;
      gin2 = a.in + ((size_t)(ct * 2 + 1) * LL + bid % LL) * N;     // c1^
      gin = comp == 2 ? gin2 : gin2 - (size_t)LL * N;                 // c0^ unless b = 2
    } else if constexpr (IO == kNttLoadTensorMul) {
      const uint32_t LL = a.limb_cycle;
      const uint32_t ct = bid / (3 * LL);
      comp = (bid / LL) % 3;
      const size_t row0 = ((size_t)ct * 2 * LL + bid % LL) * N;        // component 0 of this limb
      gmul0 = a.in + row0;
      gmul1 = a.aux + row0;
      // b = 0: c0*c0' ; b = 2: c1*c1' ; b = 1: c0*c1' + c1*c0'
      gin = gmul0 + (comp == 2 ? (size_t)LL * N : 0);
      gin2 = gmul1 + (comp == 0 ? 0 : (size_t)LL * N);
    } else if constexpr (!kFromRegs && !kTensorRegs) {
      gin = a.in + ntt_row(bid, a.limb_cycle, a.in_group_rows, a.in_row0) * N;
    }
    uint32_t* gout;
    const uint32_t* gaux = nullptr;
    if constexpr (kFromRegs) {
      const uint32_t kk = a.limb_cycle, ct = bid / kk, b = IO == kNttFromRegs1 ? 1u : 0u;
      gout = a.out + ((size_t)(ct * 2 + b) * kk + bid % kk) * N;
      gaux = a.aux + ((size_t)(ct * 3 + b) * kk + bid % kk) * N;
    } else if constexpr (kTensorRegs) {
      const uint32_t LL = a.limb_cycle, b = IO == kNttTensorRegs0 ? 0u : (IO == kNttTensorRegs1 ? 1u : 2u);
      gout = a.out + ((size_t)((bid / LL) * 3 + b) * LL + bid % LL) * N;       // d row (ct, b, l)
    } else {
      gout = a.out + ntt_row(bid, a.limb_cycle, a.out_group_rows, a.out_row0) * N;
    }
    if constexpr (IO == kNttStoreAdd) {
      const uint32_t kk = a.limb_cycle, grp = bid / kk;
      gaux = a.aux + ((size_t)(grp / 2) * 3 * kk + (size_t)(grp % 2) * kk + bid % kk) * N;
    }

#pragma unroll
    for (int c = 0; c < C; ++c) {
      const uint32_t nu = (uint32_t)tid + (uint32_t)kThreads * c;
      const uint32_t o = nu & (TLAST - 1), i = nu >> LOG_TLAST;
      const uint32_t base = i * (uint32_t)(NET * TLAST) + o;
      const uint32_t sbase = lds_swz(base);
      uint32_t v[NET];
      if constexpr (kFirst && kFromRegs) {
        // the sums sit where the last forward pass left its residues, which is where this pass takes them
#pragma unroll
        for (int e = 0; e < NET; ++e)
          v[e] = reduce64(IO == kNttFromRegs1 ? regs.s1[c * NET + e] : regs.s0[c * NET + e], L.m);
      } else if constexpr (kFirst && kTensorRegs) {
        // c0^*c0^, 2*c0^*c1^ or c1^*c1^ from the registers of the two forward transforms (values in [0, 2p)); products
        // carry the factor 2^-32 of the reduction and stay in [0, 2p)
#pragma unroll
        for (int e = 0; e < NET; ++e) {
          const uint32_t x = IO == kNttTensorRegs2 ? regs.c1[c * NET + e] : regs.c0[c * NET + e];
          const uint32_t y = IO == kNttTensorRegs0 ? regs.c0[c * NET + e] : regs.c1[c * NET + e];
          uint32_t t = redc_2p((uint64_t)x * y, p, L.pinv);
          if constexpr (IO == kNttTensorRegs1) t = csub(2 * t, two_p);
          v[e] = t;
        }
      } else if constexpr (kFirst && NET >= 4) {
        // TLAST == 1: NET consecutive coefficients -> 16-byte loads
        const U4* g4 = reinterpret_cast<const U4*>(gin + base);
#pragma unroll
        for (int e = 0; e < NET; e += 4) {
          U4 t = g4[e / 4];
          if constexpr (IO == kNttLoadTensorMul) {
            // t = c0^ (b = 0, 1) or c1^ (b = 2);  y = c0'^ (b = 0) or c1'^ (b = 1, 2); all in [0, 2p)
            const U4 y = reinterpret_cast<const U4*>(gin2 + base)[e / 4];
            t.x = redc_2p((uint64_t)t.x * y.x, p, L.pinv); t.y = redc_2p((uint64_t)t.y * y.y, p, L.pinv);
            t.z = redc_2p((uint64_t)t.z * y.z, p, L.pinv); t.w = redc_2p((uint64_t)t.w * y.w, p, L.pinv);
            if (comp == 1) {                 // + c1^ * c0'^
              const U4 u = reinterpret_cast<const U4*>(gmul0 + (size_t)a.limb_cycle * N + base)[e / 4];
              const U4 w = reinterpret_cast<const U4*>(gmul1 + base)[e / 4];
              t.x = csub(t.x + redc_2p((uint64_t)u.x * w.x, p, L.pinv), two_p);
              t.y = csub(t.y + redc_2p((uint64_t)u.y * w.y, p, L.pinv), two_p);
              t.z = csub(t.z + redc_2p((uint64_t)u.z * w.z, p, L.pinv), two_p);
              t.w = csub(t.w + redc_2p((uint64_t)u.w * w.w, p, L.pinv), two_p);
            }
          }
          if constexpr (IO == kNttLoadTensor) {
            // gin was pointed at c0^ (b = 0, 1) or c1^ (b = 2); only b = 1 needs the second row.  Products (with
            // the factor 2^-32 of the reduction) and the doubled cross term stay in [0, 2p), which is what the
            // first butterflies of the inverse transform take
            U4 y = t;
            if (comp == 1) y = reinterpret_cast<const U4*>(gin2 + base)[e / 4];
            t.x = redc_2p((uint64_t)t.x * y.x, p, L.pinv); t.y = redc_2p((uint64_t)t.y * y.y, p, L.pinv);
            t.z = redc_2p((uint64_t)t.z * y.z, p, L.pinv); t.w = redc_2p((uint64_t)t.w * y.w, p, L.pinv);
            if (comp == 1) { t.x = csub(2 * t.x, two_p); t.y = csub(2 * t.y, two_p); t.z = csub(2 * t.z, two_p); t.w = csub(2 * t.w, two_p); }
          }
          v[e + 0] = t.x; v[e + 1] = t.y; v[e + 2] = t.z; v[e + 3] = t.w;
        }
      } else {
#pragma unroll
        for (int e = 0; e < NET; ++e) {
          if constexpr (kFirst) {
            uint32_t t = gin[base + (uint32_t)e * TLAST];
            if constexpr (IO == kNttLoadTensorMul) {
              const uint32_t idx = base + (uint32_t)e * TLAST;
              t = redc_2p((uint64_t)t * gin2[idx], p, L.pinv);
              if (comp == 1)
                t = csub(t + redc_2p((uint64_t)gmul0[(size_t)a.limb_cycle * N + idx] * gmul1[idx], p, L.pinv), two_p);
            }
            if constexpr (IO == kNttLoadTensor) {
              const uint32_t u = comp == 1 ? gin2[base + (uint32_t)e * TLAST] : t;
              t = redc_2p((uint64_t)t * u, p, L.pinv);
              if (comp == 1) t = csub(2 * t, two_p);
            }
            v[e] = t;
          } else {
            v[e] = lds[lds_elem<LOG_TLAST>(sbase, e)];   // [0, 2p)
          }
        }
      }
      const uint32_t root = (1u << S0) + i;
      const uint32_t pn = L.pneg;
#pragma unroll
      for (int l = NS - 1; l >= 0; --l) {
        const int half = NET >> (l + 1);
        const bool top = kLast && l == 0;                 // node 1: fold in n^-1
#pragma unroll
        for (int h = 0; h < (1 << l); ++h) {
          constexpr bool kMont = IO == kNttLoadTensor || IO == kNttLoadTensorMul || kTensorRegs;
          const ShoupConst w = top ? (kMont ? L.w1ninv_r : L.w1ninv) : ldc(tw, (root << l) + h);
          const ShoupConst nv = kMont ? L.ninv_r : L.ninv;
          // Both forms of the lazy product are a multiplication and a multiply-add: x*w + q*(-p), and negated
          // x*(-w) + q*p.  -p and the zero that -w is taken from come out of the table, so that the compiler
          // keeps the sums (it would turn a visible negation back into two multiplications and a subtraction).
          const uint32_t wn = L.zero - w.w;
#pragma unroll
          for (int x = 0; x < half; ++x) {
            const int ia = h * 2 * half + x, ib = ia + half;
            // A product that the next level subtracts (its position is a right operand there) is kept
            // negated mod 2^32: the difference then is one three-operand addition.
            const bool y_neg = l < NS - 1 && (x & (half >> 1)) != 0;    // v[ib] was stored negated by level l + 1
            const bool out_neg = l > 0 && (h & 1) != 0;                 // v[ib] is a right operand of level l - 1
            const uint32_t X = v[ia], Y = v[ib];
            const uint32_t S = y_neg ? X - Y : X + Y;                   // [0, 4p)
            const uint32_t D = y_neg ? X + two_p + Y : X + two_p - Y;   // (0, 4p)
            v[ia] = top ? S * nv.w + mulhi32(S, nv.ws) * pn : csub(S, two_p);
            v[ib] = out_neg ? D * wn + mulhi32(D, w.ws) * p             // -(D * w mod p) - {0, p}  (mod 2^32)
                            : D * w.w + mulhi32(D, w.ws) * pn;          // D * w mod p + {0, p}: [0, 2p)
          }
        }
      }
      if constexpr (kLast && (IO == kNttStoreAdd || kFromRegs)) {
        // all loads of the addend before the first store (the compiler must assume the buffers alias)
        uint32_t addend[NET];
#pragma unroll
        for (int e = 0; e < NET; ++e) addend[e] = gaux[base + (uint32_t)e * TLAST];
#pragma unroll
        for (int e = 0; e < NET; ++e) gout[base + (uint32_t)e * TLAST] = add_mod(csub(v[e], p), addend[e], p);
      } else if constexpr (kLast) {
        constexpr bool kLazyOut = IO == kNttLoadTensor || IO == kNttLoadTensorMul || kTensorRegs;
#pragma unroll
        for (int e = 0; e < NET; ++e) gout[base + (uint32_t)e * TLAST] = kLazyOut ? v[e] : csub(v[e], p);
      } else {
#pragma unroll
        for (int e = 0; e < NET; ++e) lds[lds_elem<LOG_TLAST>(sbase, e)] = v[e];
      }
    }
  }
};

// ------------------------------------------------------------------------- relinearisation in one kernel
// Workgroup (ct, j): for every digit i of y2[ct] -- forward transform modulo q_j, products with the two key rows
// added to register-held sums -- then the two sums go back through the inverse transform and leave as
// c'_b = y_b + sum_i evk[i][b] * digit_i (HMult step 3).  Neither the transformed digits nor the sums touch memory.
struct RelinFusedArgs {
  const uint32_t* y;        // [n_ct][3][k][n]
  const uint32_t* evk;      // [k][2][k][n], transformed
  uint32_t* out;            // [n_ct][2][k][n]
  const ShoupConst* tw_fwd;
  const ShoupConst* tw_inv;
  const NttLimb* limbs;
  uint32_t k;
  uint32_t n_rows;          // n_ct * k
};

template <int LOGN, int LOGR, int MAC = kNttFusedMacAny>
struct RelinFused {
  using G = NttGeom<LOGN, LOGR>;
  using Fwd = NttFwd<LOGN, LOGR, MAC>;
  using Inv0 = NttInv<LOGN, LOGR, kNttFromRegs0>;
  using Inv1 = NttInv<LOGN, LOGR, kNttFromRegs1>;
  static constexpr int P = G::kPhases;
  static constexpr int kThreads = G::kThreads;
  static constexpr int kLoopPhases = P;
  // room for two workgroups per compute unit (one of 1024 threads)
  static constexpr int kMinWavesPerSimd = G::kThreads >= 1024 ? 4 : (G::kThreads / 256 * 2 > 0 ? G::kThreads / 256 * 2 : 1);
  static constexpr int kPhases = 3 * P;
  using Regs = RelinRegs<G::R>;
  HCNN_HD static uint32_t loop_count(const RelinFusedArgs& a) { return a.k; }

  template <int PH>
  HCNN_HD static void phase(const RelinFusedArgs& a, unsigned bid, int tid, uint32_t* lds, Regs& regs) {
    NttArgs na{};
    na.limbs = a.limbs; na.limb_cycle = a.k; na.limb_base = 0; na.n_rows = a.n_rows;
    if constexpr (PH < P) {
      na.in = a.y; na.aux = a.evk; na.tw = a.tw_fwd;
      Fwd::template phase<PH>(na, bid, tid, lds, regs);
    } else {
      na.aux = a.y; na.out = a.out; na.tw = a.tw_inv;
      if constexpr (PH < 2 * P) Inv0::template phase<PH - P>(na, bid, tid, lds, regs);
      else Inv1::template phase<PH - 2 * P>(na, bid, tid, lds, regs);
    }
  }
};

// ------------------------------------------------------------------------- squaring tensor in one kernel
// Workgroup (ct, l): forward transforms of c0 and c1 modulo limb l (l < k: read from the ciphertext; else from the
// extension buffer), kept in registers, then the three tensor components c0^2, 2 c0 c1, c1^2 through the inverse
// transform into d[ct][b][l] (HMult step 1 with both operands equal).  The transformed operands never touch memory.
struct TensorFusedArgs {
  const uint32_t* cts;      // [n_ct][2][k][n]
  const uint32_t* ext;      // [n_ct][2][L][n], rows k..L-1 of every polynomial valid
  uint32_t* d;              // [n_ct][3][L][n]
  const ShoupConst* tw_fwd;
  const ShoupConst* tw_inv;
  const NttLimb* limbs;
  uint32_t k, L;
  uint32_t n_rows;          // n_ct * L
};

template <int LOGN, int LOGR>
struct TensorFused {
  using G = NttGeom<LOGN, LOGR>;
  static constexpr int P = G::kPhases;
  static constexpr int kThreads = G::kThreads;
  static constexpr int kPhases = 5 * P;
  static constexpr int kMinWavesPerSimd = 4;     // 128 registers: two 512-thread or four 256-thread workgroups per compute unit
  using Regs = TensorRegs<G::R>;

  template <int PH>
  HCNN_HD static void phase(const TensorFusedArgs& a, unsigned bid, int tid, uint32_t* lds, Regs& regs) {
    NttArgs na{};
    na.limbs = a.limbs; na.limb_cycle = a.L; na.limb_base = 0; na.n_rows = a.n_rows;
    if constexpr (PH < 2 * P) {
      na.in = a.ext; na.aux = a.cts; na.own_limbs = a.k; na.tw = a.tw_fwd;
      if constexpr (PH < P) NttFwd<LOGN, LOGR, kNttToRegs0>::template phase<PH>(na, bid, tid, lds, regs);
      else NttFwd<LOGN, LOGR, kNttToRegs1>::template phase<PH - P>(na, bid, tid, lds, regs);
    } else {
      na.out = a.d; na.tw = a.tw_inv;
      if constexpr (PH < 3 * P) NttInv<LOGN, LOGR, kNttTensorRegs0>::template phase<PH - 2 * P>(na, bid, tid, lds, regs);
      else if constexpr (PH < 4 * P) NttInv<LOGN, LOGR, kNttTensorRegs1>::template phase<PH - 3 * P>(na, bid, tid, lds, regs);
      else NttInv<LOGN, LOGR, kNttTensorRegs2>::template phase<PH - 4 * P>(na, bid, tid, lds, regs);
    }
  }
};

}  // namespace hcnn
