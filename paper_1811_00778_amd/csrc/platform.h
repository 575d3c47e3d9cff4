// Launch and memory shims.
//
// Every kernel of this library is written as a struct with
//   kThreads                      threads per workgroup
//   kPhases                       number of barrier-separated phases
//   struct Regs                   per-thread state that lives across barriers
//   template<int PH> phase(args, block, tid, lds, regs)
// and, optionally, a repeated prefix:
//   kLoopPhases, loop_count(args) phases [0, kLoopPhases) run loop_count times (Regs::iter = the iteration, a
//                                 barrier after every one of them), then the remaining phases once
// The HIP build runs the phases of one workgroup inside one __global__ function
// with __syncthreads() between phases.  The HCNN_HOSTEMU build (used only by the
// CPU test-suite to check kernel indexing and arithmetic before anything touches
// a GPU) runs the same phase bodies as plain loops over blocks and threads; it is
// a checker for the kernel sources, not a product path, and the Python binding
// never loads it.
#pragma once
#include <cstddef>
#include <cstdint>
#include <cstdlib>
#include <atomic>
#include <cstring>
#include <type_traits>
#include <vector>

#ifdef HCNN_HOSTEMU
#define HCNN_HD inline
#define HCNN_HOSTDEV inline
#define HCNN_DEVICE_CODE 0
typedef int hcnn_hip_error_t;
typedef void* hcnn_stream_t;
#else
#include <hip/hip_runtime.h>
#define HCNN_HD __device__ __forceinline__
#define HCNN_HOSTDEV __host__ __device__ inline
typedef hipError_t hcnn_hip_error_t;
typedef hipStream_t hcnn_stream_t;
#endif

namespace hcnn {

#ifdef HCNN_HOSTEMU
struct alignas(16) U4 { uint32_t x, y, z, w; };
#else
typedef uint4 U4;
#endif

// opaque(x): x again, but as a value the compiler cannot trace back.  Used inside the repeated phases of a looped
// kernel on the thread index, so that the per-thread addresses derived from it are recomputed in every iteration
// (a few instructions) rather than computed once, kept across the whole loop and spilled.
HCNN_HD int opaque(int x) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("" : "+v"(x));
#endif
  return x;
}

// ldc(table, i): element i of a read-only table (moduli, twiddles, base-conversion constants).
// In device code the words are read through the constant address space: with a wave-uniform
// index the compiler then issues scalar loads instead of one vector load per lane.  The tables
// are written once, before any kernel runs, and never by a kernel.
#if defined(__HIP_DEVICE_COMPILE__)
template <class T>
__device__ __forceinline__ T ldc(const T* table, size_t i) {
  static_assert(sizeof(T) % 4 == 0 && alignof(T) >= 4, "tables are made of 32-bit words");
  typedef const uint32_t __attribute__((address_space(4))) * cptr;
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
  cptr w = (cptr)(table + i);
#pragma clang diagnostic pop
  T out;
  uint32_t* o = reinterpret_cast<uint32_t*>(&out);
#pragma unroll
  for (unsigned k = 0; k < sizeof(T) / 4; ++k) o[k] = w[k];
  return out;
}
#elif defined(HCNN_HOSTEMU)
template <class T> inline T ldc(const T* table, size_t i) { return table[i]; }
#else
template <class T> __device__ __forceinline__ T ldc(const T* table, size_t i) { return table[i]; }
#endif

// kMinWavesPerSimd (optional): occupancy the register allocation of the kernel must allow
template <class K, class = void> struct MinWavesPerSimd { static constexpr int value = 1; };
template <class K> struct MinWavesPerSimd<K, std::void_t<decltype(K::kMinWavesPerSimd)>> { static constexpr int value = K::kMinWavesPerSimd; };
template <class K, class = void> struct LoopPhases { static constexpr int value = 0; };
template <class K> struct LoopPhases<K, std::void_t<decltype(K::kLoopPhases)>> { static constexpr int value = K::kLoopPhases; };

#ifdef HCNN_HOSTEMU
// ------------------------------------------------------------------ host emulation
inline int dev_malloc(void** p, size_t bytes) {
  *p = std::malloc(bytes ? bytes : 1);
  return *p ? 0 : 2;
}
inline int dev_free(void* p) { std::free(p); return 0; }
inline int dev_memset(void* p, int v, size_t bytes, hcnn_stream_t) { std::memset(p, v, bytes); return 0; }
inline int copy_h2d(void* d, const void* h, size_t bytes, hcnn_stream_t) { std::memcpy(d, h, bytes); return 0; }
inline int copy_d2h(void* h, const void* d, size_t bytes, hcnn_stream_t) { std::memcpy(h, d, bytes); return 0; }
inline int copy_d2d(void* d, const void* s, size_t bytes, hcnn_stream_t) { std::memmove(d, s, bytes); return 0; }
inline int stream_sync(hcnn_stream_t) { return 0; }
typedef int hcnn_event_t;
inline int event_create(hcnn_event_t* e) { *e = 0; return 0; }
inline int event_destroy(hcnn_event_t) { return 0; }
inline int event_record(hcnn_event_t, hcnn_stream_t) { return 0; }
inline int event_elapsed_ms(float* ms, hcnn_event_t, hcnn_event_t) { *ms = 0.f; return 0; }
inline size_t max_lds_bytes() { return 160 * 1024; }
inline uint32_t compute_unit_count() { return 1; }   // small rounds: the checker's little batches reach every batch-splitting path
HCNN_HD void atomic_inc64(unsigned long long* p) { *p += 1; }
HCNN_HD void atomic_max32(uint32_t* p, uint32_t v) { if (v > *p) *p = v; }
// Workgroups of kernel K that one compute unit holds at a time.  The checker has no device to ask: it counts 16
// wavefronts per compute unit (8 for workgroups of 256 threads, the shape whose register use halves the occupancy
// on the device), which with its single compute unit gives rounds of a few workgroups.
template <class K, class Args>
int resident_workgroups_per_cu(size_t, int* out) {
  const int waves = K::kThreads / 64 > 0 ? K::kThreads / 64 : 1;
  *out = (K::kThreads == 256 ? 8 : 16) / waves;
  if (*out < 1) *out = 1;
  return 0;
}

template <class K, int PH, int END>
struct EmuPhases {
  template <class Args>
  static void run(const Args& a, unsigned bid, uint32_t* lds, std::vector<typename K::Regs>& regs) {
    for (int tid = 0; tid < K::kThreads; ++tid) K::template phase<PH>(a, bid, tid, lds, regs[tid]);
    if constexpr (PH + 1 < END) EmuPhases<K, PH + 1, END>::run(a, bid, lds, regs);
  }
};

template <class K, class Args>
int launch(hcnn_stream_t, size_t grid, size_t lds_bytes, const Args& a) {
  if (lds_bytes > max_lds_bytes()) return 1;
  std::vector<uint32_t> lds(lds_bytes / 4 + 4);
  std::vector<typename K::Regs> regs(K::kThreads);
  constexpr int LP = LoopPhases<K>::value;
  for (size_t bid = 0; bid < grid; ++bid) {
    if constexpr (LP > 0) {
      const uint32_t count = K::loop_count(a);
      for (uint32_t it = 0; it < count; ++it) {
        for (auto& r : regs) r.iter = it;
        EmuPhases<K, 0, LP>::run(a, (unsigned)bid, lds.data(), regs);
      }
    }
    if constexpr (LP < K::kPhases) EmuPhases<K, LP, K::kPhases>::run(a, (unsigned)bid, lds.data(), regs);
  }
  return 0;
}

#else
// ------------------------------------------------------------------ HIP
inline int dev_malloc(void** p, size_t bytes) { return (int)hipMalloc(p, bytes ? bytes : 1); }
inline int dev_free(void* p) { return (int)hipFree(p); }
inline int dev_memset(void* p, int v, size_t bytes, hcnn_stream_t s) { return (int)hipMemsetAsync(p, v, bytes, s); }
inline int copy_h2d(void* d, const void* h, size_t bytes, hcnn_stream_t s) {
  // tables are tiny and built once: a synchronous copy keeps the host vector's lifetime simple
  (void)s;
  return (int)hipMemcpy(d, h, bytes, hipMemcpyHostToDevice);
}
inline int copy_d2h(void* h, const void* d, size_t bytes, hcnn_stream_t s) {
  int e = (int)hipStreamSynchronize(s);
  if (e) return e;
  return (int)hipMemcpy(h, d, bytes, hipMemcpyDeviceToHost);
}
inline int copy_d2d(void* d, const void* s_, size_t bytes, hcnn_stream_t s) {
  return (int)hipMemcpyAsync(d, s_, bytes, hipMemcpyDeviceToDevice, s);
}
inline int stream_sync(hcnn_stream_t s) { return (int)hipStreamSynchronize(s); }
typedef hipEvent_t hcnn_event_t;
inline int event_create(hcnn_event_t* e) { return (int)hipEventCreate(e); }
inline int event_destroy(hcnn_event_t e) { return (int)hipEventDestroy(e); }
inline int event_record(hcnn_event_t e, hcnn_stream_t s) { return (int)hipEventRecord(e, s); }
inline int event_elapsed_ms(float* ms, hcnn_event_t a, hcnn_event_t b) { return (int)hipEventElapsedTime(ms, a, b); }
inline size_t max_lds_bytes() {
  int dev = 0, v = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return 0;
  return (size_t)v;
}
inline uint32_t compute_unit_count() {
  int dev = 0, v = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 256;
  return (uint32_t)v;
}
HCNN_HD void atomic_inc64(unsigned long long* p) { atomicAdd(p, 1ull); }
HCNN_HD void atomic_max32(uint32_t* p, uint32_t v) { atomicMax(p, v); }

template <class K, int PH, int END, class Args>
__device__ __forceinline__ void run_phases(const Args& a, unsigned bid, int tid, uint32_t* lds,
                                           typename K::Regs& regs) {
  K::template phase<PH>(a, bid, tid, lds, regs);
  if constexpr (PH + 1 < END) {
    __syncthreads();
    run_phases<K, PH + 1, END, Args>(a, bid, tid, lds, regs);
  }
}

template <class K, class Args>
__global__ void __launch_bounds__(K::kThreads, MinWavesPerSimd<K>::value) kernel_entry(const Args a) {
  extern __shared__ __align__(16) uint32_t hcnn_lds[];
  typename K::Regs regs;
  constexpr int LP = LoopPhases<K>::value;
  if constexpr (LP > 0) {
    const uint32_t count = K::loop_count(a);
    for (uint32_t it = 0; it < count; ++it) {
      regs.iter = it;
      run_phases<K, 0, LP, Args>(a, blockIdx.x, (int)threadIdx.x, hcnn_lds, regs);
      __syncthreads();
    }
  }
  if constexpr (LP < K::kPhases) run_phases<K, LP, K::kPhases, Args>(a, blockIdx.x, (int)threadIdx.x, hcnn_lds, regs);
}

template <class K, class Args>
int launch(hcnn_stream_t s, size_t grid, size_t lds_bytes, const Args& a) {
  if (grid == 0) return 0;
  if (grid > 0x7fffffffull) return (int)hipErrorInvalidConfiguration;
  if (lds_bytes > 48 * 1024) {
    // raised once per kernel and size (not on every launch, and so not while a caller records a graph after its
    // warm-up call)
    static std::atomic<size_t> allowed{0};
    if (lds_bytes > allowed.load(std::memory_order_relaxed)) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&kernel_entry<K, Args>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
      if (e != hipSuccess) return (int)e;
      allowed.store(lds_bytes, std::memory_order_relaxed);
    }
  }
  hipLaunchKernelGGL((kernel_entry<K, Args>), dim3((unsigned)grid), dim3(K::kThreads), lds_bytes, s, a);
  return (int)hipGetLastError();
}

// Workgroups of kernel K (with lds_bytes of dynamic LDS each) that one compute unit holds at a time, as the runtime
// derives it from the compiled kernel's register and LDS use.
template <class K, class Args>
int resident_workgroups_per_cu(size_t lds_bytes, int* out) {
  if (lds_bytes > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&kernel_entry<K, Args>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return (int)e;
  }
  int n = 0;
  hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel_entry<K, Args>, K::kThreads, lds_bytes);
  if (e != hipSuccess) return (int)e;
  *out = n > 0 ? n : 1;
  return 0;
}
#endif

}  // namespace hcnn
