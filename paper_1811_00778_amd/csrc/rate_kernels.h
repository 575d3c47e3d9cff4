// Measured ceilings of the device: streaming kernels (copy, read, fill) and instruction-issue probes for the
// integer operations the transforms and the multiply-accumulate are made of.  They give the denominators that
// the benchmark reports next to the vendor's peak figures; nothing on the hot path uses them.
#pragma once
#include "modarith.h"

namespace hcnn {

constexpr int kRateThreads = 256;
constexpr int kStreamUnroll = 8;          // 16-byte accesses per thread of the streaming kernels
constexpr uint32_t kRateIters = 4096;     // iterations of the issue probes
constexpr int kRateChains = 8;            // independent dependency chains per lane

// mode 0: dst = src; mode 1: read src only (the sum is stored by no thread unless it hits a value it cannot have);
// mode 2: fill dst.  A workgroup handles kStreamUnroll consecutive runs of 256 x 16 bytes.
struct StreamArgs {
  const U4* src;
  U4* dst;
  uint32_t mode;
  uint32_t fill;
};
struct StreamKernel {
  static constexpr int kThreads = kRateThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  template <int PH>
  HCNN_HD static void phase(const StreamArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    const size_t base = (size_t)bid * kStreamUnroll * kThreads + (size_t)tid;
    if (a.mode == 2) {
      U4 v;
      v.x = a.fill; v.y = a.fill; v.z = a.fill; v.w = a.fill;
#pragma unroll
      for (int u = 0; u < kStreamUnroll; ++u) a.dst[base + (size_t)u * kThreads] = v;
      return;
    }
    U4 v[kStreamUnroll];
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) v[u] = a.src[base + (size_t)u * kThreads];
    if (a.mode == 0) {
#pragma unroll
      for (int u = 0; u < kStreamUnroll; ++u) a.dst[base + (size_t)u * kThreads] = v[u];
    } else {
      uint32_t r = 0;
#pragma unroll
      for (int u = 0; u < kStreamUnroll; ++u) r ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
      if (r == a.fill) a.dst[base] = v[0];        // the caller fills src so that this cannot happen
    }
  }
};

// Issue probes: kRateIters x kRateChains operations per lane, each chain depending on its own previous value.
enum { kRateMulLo = 0, kRateMulHi = 1, kRateMadU64 = 2, kRateMadI64 = 3, kRateAdd = 4, kRateOps = 5 };
struct RateArgs {
  uint32_t* out;
  uint32_t seed;
};
template <int OP>
struct RateKernel {
  static constexpr int kThreads = kRateThreads;
  static constexpr int kPhases = 1;
  struct Regs {};
  template <int PH>
  HCNN_HD static void phase(const RateArgs& a, unsigned bid, int tid, uint32_t*, Regs&) {
    uint32_t v[kRateChains];
    uint64_t w[kRateChains];
    const uint32_t x = a.seed + (uint32_t)tid + bid, y = a.seed * 2u + 1u, big = 0xfffffff1u - a.seed;
#pragma unroll
    for (int i = 0; i < kRateChains; ++i) { v[i] = x + (uint32_t)i; w[i] = (uint64_t)x * 7u + (uint32_t)i; }
    for (uint32_t it = 0; it < kRateIters; ++it) {
#pragma unroll
      for (int i = 0; i < kRateChains; ++i) {
#if defined(__HIP_DEVICE_COMPILE__)
        // the instruction itself, so that the compiler can neither merge iterations nor pick another opcode
        if constexpr (OP == kRateMulLo) asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(v[i]) : "v"(y));
        if constexpr (OP == kRateMulHi) asm volatile("v_mul_hi_u32 %0, %0, %1" : "+v"(v[i]) : "v"(big));
        if constexpr (OP == kRateMadU64) asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, %0" : "+v"(w[i]) : "v"(v[i]), "v"(y) : "vcc");
        if constexpr (OP == kRateMadI64) asm volatile("v_mad_i64_i32 %0, vcc, %1, %2, %0" : "+v"(w[i]) : "v"(v[i]), "v"(y) : "vcc");
        if constexpr (OP == kRateAdd) asm volatile("v_add_u32 %0, %0, %1" : "+v"(v[i]) : "v"(y));
#else
        if constexpr (OP == kRateMulLo) v[i] = v[i] * y;
        if constexpr (OP == kRateMulHi) v[i] = mulhi32(v[i], big);
        if constexpr (OP == kRateMadU64) w[i] = (uint64_t)v[i] * y + w[i];
        if constexpr (OP == kRateMadI64) w[i] = (uint64_t)((int64_t)(int32_t)v[i] * (int64_t)(int32_t)y + (int64_t)w[i]);
        if constexpr (OP == kRateAdd) v[i] = v[i] + y;
#endif
      }
    }
    uint32_t r = 0;
#pragma unroll
    for (int i = 0; i < kRateChains; ++i) r ^= v[i] ^ (uint32_t)w[i] ^ (uint32_t)(w[i] >> 32);
    if (r == 0x12345678u) a.out[tid] = r;         // keeps the chains alive; practically never taken
  }
};

}  // namespace hcnn
