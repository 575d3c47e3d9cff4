// C ABI, context, table generation and kernel orchestration.
// Compiled as HIP for gfx950 (the product) or, with -DHCNN_HOSTEMU, as plain C++
// for the CPU checker of the kernel sources.
#include "../../include/hcnn.h"

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "fv_kernels.h"
#include "ntt_kernels.h"
#include "rate_kernels.h"

using namespace hcnn;

namespace {

typedef unsigned __int128 u128;

// ---------------------------------------------------------------- host number theory
uint32_t h_mulmod(uint32_t a, uint32_t b, uint32_t m) { return (uint32_t)(((uint64_t)a * b) % m); }
uint32_t h_powmod(uint32_t a, uint64_t e, uint32_t m) {
  uint64_t r = 1, b = a % m;
  while (e) {
    if (e & 1) r = r * b % m;
    b = b * b % m;
    e >>= 1;
  }
  return (uint32_t)r;
}
uint32_t h_inv(uint32_t a, uint32_t prime) { return h_powmod(a % prime, (uint64_t)prime - 2, prime); }

bool h_is_prime(uint32_t x) {
  if (x < 2) return false;
  for (uint32_t sp : {2u, 3u, 5u, 7u, 11u, 13u}) {
    if (x % sp == 0) return x == sp;
  }
  uint32_t d = x - 1;
  int r = 0;
  while ((d & 1) == 0) { d >>= 1; ++r; }
  for (uint32_t a : {2u, 3u, 5u, 7u}) {          // decides every x < 3,215,031,751
    uint64_t y = h_powmod(a, d, x);
    if (y == 1 || y == x - 1) continue;
    bool comp = true;
    for (int i = 1; i < r; ++i) {
      y = y * y % x;
      if (y == x - 1) { comp = false; break; }
    }
    if (comp) return false;
  }
  return true;
}

// 64-bit variants for the plaintext modulus (up to 47 bits)
uint64_t h_mulmod64(uint64_t a, uint64_t b, uint64_t m) { return (uint64_t)((unsigned __int128)a * b % m); }
uint64_t h_powmod64(uint64_t b, uint64_t e, uint64_t m) {
  uint64_t r = 1 % m;
  b %= m;
  while (e) {
    if (e & 1) r = h_mulmod64(r, b, m);
    b = h_mulmod64(b, b, m);
    e >>= 1;
  }
  return r;
}
bool h_is_prime64(uint64_t x) {
  if (x < 2) return false;
  for (uint64_t sp : {2ull, 3ull, 5ull, 7ull, 11ull, 13ull, 17ull, 19ull, 23ull, 29ull, 31ull, 37ull}) {
    if (x % sp == 0) return x == sp;
  }
  uint64_t d = x - 1;
  int r = 0;
  while ((d & 1) == 0) { d >>= 1; ++r; }
  for (uint64_t a : {2ull, 3ull, 5ull, 7ull, 11ull, 13ull, 17ull, 19ull, 23ull, 29ull, 31ull, 37ull}) {   // decides every x < 2^64
    uint64_t y = h_powmod64(a, d, x);
    if (y == 1 || y == x - 1) continue;
    bool comp = true;
    for (int i = 1; i < r; ++i) {
      y = h_mulmod64(y, y, x);
      if (y == x - 1) { comp = false; break; }
    }
    if (comp) return false;
  }
  return true;
}
// product of all `ms` except index `skip` (skip < 0: all), modulo a 64-bit m
uint64_t h_prod_mod64(const std::vector<uint32_t>& ms, int skip, uint64_t m) {
  uint64_t r = 1 % m;
  for (int i = 0; i < (int)ms.size(); ++i)
    if (i != skip) r = h_mulmod64(r, ms[i] % m, m);
  return r;
}

// psi = x^((p-1)/2n) for the smallest x >= 2 giving order exactly 2n
uint32_t h_root_of_unity(uint32_t n, uint32_t p) {
  const uint64_t e = ((uint64_t)p - 1) / (2ull * n);
  for (uint32_t x = 2;; ++x) {
    uint32_t psi = h_powmod(x, e, p);
    if (h_powmod(psi, n, p) == p - 1) return psi;
  }
}

uint32_t h_brev(uint32_t v, int bits) {
  uint32_t r = 0;
  for (int i = 0; i < bits; ++i) { r = (r << 1) | (v & 1); v >>= 1; }
  return r;
}

// -p^-1 mod 2^32 for odd p (Newton iteration, doubling the number of correct bits each step)
uint32_t h_neg_inv32(uint32_t p) {
  uint32_t inv = 1;
  for (int it = 0; it < 5; ++it) inv *= 2u - p * inv;
  return 0u - inv;
}

ShoupConst h_shoup(uint32_t w, uint32_t p) {
  ShoupConst c;
  c.w = w;
  c.ws = (uint32_t)(((uint64_t)w << 32) / p);
  return c;
}

Mod h_mod(uint32_t p) {
  Mod m;
  m.p = p;
  m.c32 = (uint32_t)((1ull << 32) % p);
  m.c32s = (uint32_t)(((uint64_t)m.c32 << 32) / p);
  m.mu = (uint32_t)((1ull << 61) / p);
  return m;
}

// product of all `ms` except index `skip` (skip < 0: all), modulo m
uint32_t h_prod_mod(const std::vector<uint32_t>& ms, int skip, uint32_t m) {
  uint64_t r = 1 % m;
  for (int i = 0; i < (int)ms.size(); ++i)
    if (i != skip) r = r * (ms[i] % m) % m;
  return (uint32_t)r;
}

// little-endian multiword natural numbers, only for the size check of the auxiliary basis
typedef std::vector<uint32_t> Big;
void big_mul_small(Big& a, uint32_t f) {
  uint64_t carry = 0;
  for (auto& w : a) {
    uint64_t t = (uint64_t)w * f + carry;
    w = (uint32_t)t;
    carry = t >> 32;
  }
  if (carry) a.push_back((uint32_t)carry);
}
void big_add_small(Big& a, uint32_t v) {
  uint64_t carry = v;
  for (auto& w : a) {
    uint64_t t = (uint64_t)w + carry;
    w = (uint32_t)t;
    carry = t >> 32;
    if (!carry) break;
  }
  if (carry) a.push_back((uint32_t)carry);
}
int big_cmp(Big a, Big b) {
  while (!a.empty() && a.back() == 0) a.pop_back();
  while (!b.empty() && b.back() == 0) b.pop_back();
  if (a.size() != b.size()) return a.size() < b.size() ? -1 : 1;
  for (size_t i = a.size(); i-- > 0;)
    if (a[i] != b[i]) return a[i] < b[i] ? -1 : 1;
  return 0;
}

bool valid_n(uint32_t n) { return n >= 1024 && n <= 32768 && (n & (n - 1)) == 0; }
bool valid_rns_prime(uint32_t p, uint32_t n) {
  return p > (1u << 29) && p < (1u << 30) && (p - 1) % (2 * n) == 0 && h_is_prime(p);
}

int check_primes(uint32_t n, const uint32_t* q, uint32_t k, const uint32_t* p, uint32_t kp) {
  std::vector<uint32_t> all(q, q + k);
  if (kp) all.insert(all.end(), p, p + kp);
  for (uint32_t v : all)
    if (!valid_rns_prime(v, n)) return HCNN_ERR_PRIME;
  std::sort(all.begin(), all.end());
  if (std::adjacent_find(all.begin(), all.end()) != all.end()) return HCNN_ERR_PRIME;
  return HCNN_OK;
}

// is prod(p[0..kp)) > t*n*prod(q) + 1 ?
bool aux_sufficient(uint32_t n, const uint32_t* q, uint32_t k, uint64_t t, const uint32_t* p, uint32_t kp) {
  Big lhs{1}, rhs{1};
  for (uint32_t j = 0; j < kp; ++j) big_mul_small(lhs, p[j]);
  for (uint32_t i = 0; i < k; ++i) big_mul_small(rhs, q[i]);
  // t < 2^47 = (t >> 24) * 2^24 + (t & 0xffffff): two small factors and a sum
  {
    Big hi = rhs;
    big_mul_small(hi, (uint32_t)(t >> 24));
    big_mul_small(hi, 1u << 24);
    big_mul_small(rhs, (uint32_t)(t & 0xffffffu));
    if (rhs.size() < hi.size()) rhs.resize(hi.size(), 0);
    uint64_t carry = 0;
    for (size_t w = 0; w < rhs.size(); ++w) {
      const uint64_t sum = (uint64_t)rhs[w] + (w < hi.size() ? hi[w] : 0) + carry;
      rhs[w] = (uint32_t)sum;
      carry = sum >> 32;
    }
    if (carry) rhs.push_back((uint32_t)carry);
  }
  big_mul_small(rhs, n);
  big_add_small(rhs, 1);
  return big_cmp(lhs, rhs) > 0;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

// ---------------------------------------------------------------- scratch of the entry point that allocates nothing
// hcnn_ct_square_relin_noalloc keeps the intermediate polynomials of its internal batch in this array instead of a
// buffer from hipMalloc.  Every device that loads the library holds its own copy (at its own address) until the
// process ends; every call on a device shares that copy.
constexpr size_t kStaticScratchBytes = (size_t)128 << 20;
#ifdef HCNN_HOSTEMU
alignas(256) static uint32_t scratch[kStaticScratchBytes / 4];
#else
static __device__ __align__(256) uint32_t scratch[kStaticScratchBytes / 4];
#endif

namespace {
#ifndef HCNN_HOSTEMU
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint32_t* g_scratch_addr[kMaxDevices] = {};
#endif

// Device address of `scratch` on the current device, looked up once per device.  (In host code the array's name is
// only a handle for the lookup: kernels and copies take the address returned here.)
int static_scratch_of_current_device(uint32_t** out) {
#ifdef HCNN_HOSTEMU
  *out = scratch;
  return 0;
#else
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return HCNN_ERR_NODEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_addr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!ptr) return HCNN_ERR_NODEVICE;
    g_scratch_addr[dev] = (uint32_t*)ptr;
  }
  *out = g_scratch_addr[dev];
  return 0;
#endif
}
}  // namespace

// ---------------------------------------------------------------- context
struct BConvHost {
  uint32_t ks = 0, kd = 0;
  std::vector<Mod> src_mod, dst_mod;
  std::vector<ShoupConst> zmul, xmul;
  std::vector<uint32_t> ginv, half, Bp, BpT, Vp, dst_pinv;
  uint32_t mont = 0;
};

struct hcnn_ctx {
  uint32_t n = 0, logn = 0, k = 0, kp = 0;
  uint64_t t = 0;
  std::vector<uint32_t> q, p;
  hcnn_stream_t stream = nullptr;
  std::vector<void*> owned;

  Mod* d_mods = nullptr;            // [k + kp]
  NttLimb* d_limbs = nullptr;       // [k + kp]
  ShoupConst* d_tw_fwd = nullptr;   // [k + kp][n]
  ShoupConst* d_tw_inv = nullptr;
  ShoupConst* d_delta = nullptr;    // [k] floor(q/t) mod q_l
  uint32_t* d_tq_inv = nullptr;     // [kp] t * q^-1 mod p_j
  BConvDev ext{}, to_p{}, to_q{}, dec{};
  uint32_t neg_qinv_t = 0;
  uint32_t* d_gauss_t = nullptr;    // thresholds of the Gaussian sampler (uploaded on first use)
  uint64_t* d_dec_wide = nullptr;   // plaintext modulus above 2^32: [k + 2] constants of the decrypt rounding
  unsigned long long* d_counters = nullptr;   // [2]

  uint32_t* d_evk_hat = nullptr;
  bool has_key = false;

  uint32_t* work = nullptr;       // device work buffer of the entry points that may allocate (grown on demand)
  size_t work_bytes = 0;
  uint32_t* static_scratch = nullptr;   // this device's copy of the file-scope array `scratch` (kStaticScratchBytes)

  uint32_t band = 128;
  uint64_t square_chunk = 0;
  uint64_t relin_order = 0;   // 0 = by key size, 1 = ciphertext-major, 2 = key-major
  uint64_t fusion = 0;   // one-kernel tensor / relinearisation: 0 = chosen per batch, 1 = never, 2 = always where available
  size_t max_lds = 0;
  uint32_t compute_units = 256;
  uint32_t relin_fused_wgs = 1, tensor_fused_wgs = 1;   // resident workgroups per compute unit of the one-kernel forms

  // optional per-kernel timing (HCNN_OPT_PROFILE): an event pair around every launch
  struct Pending { int cls; uint64_t blocks; hcnn_event_t start, stop; };
  bool profile = false;
  std::vector<Pending> pending;
  std::vector<hcnn_event_t> free_events;
  uint64_t prof_launches[HCNN_PROF_COUNT] = {};
  uint64_t prof_blocks[HCNN_PROF_COUNT] = {};
  double prof_ms[HCNN_PROF_COUNT] = {};
};

namespace {

template <class T>
int upload(hcnn_ctx* c, const std::vector<T>& h, T** d) {
  void* ptr = nullptr;
  int e = dev_malloc(&ptr, h.size() * sizeof(T));
  if (e) return e;
  c->owned.push_back(ptr);
  if (!h.empty()) {
    e = copy_h2d(ptr, h.data(), h.size() * sizeof(T), c->stream);
    if (e) return e;
  }
  *d = (T*)ptr;
  return 0;
}

template <class K> struct KernelClass { static constexpr int id = HCNN_PROF_OTHER; };
template <int A, int B, int C, int D> struct KernelClass<NttFwd<A, B, C, D>> { static constexpr int id = HCNN_PROF_NTT_FWD; };
template <int A, int B, int C> struct KernelClass<NttInv<A, B, C>> { static constexpr int id = HCNN_PROF_NTT_INV; };
template <> struct KernelClass<ExtKernel> { static constexpr int id = HCNN_PROF_BASE_EXT; };
template <int A, int B> struct KernelClass<ExtKernelT<A, B>> { static constexpr int id = HCNN_PROF_BASE_EXT; };
template <int A, int B> struct KernelClass<ScaleKernelR<A, B>> { static constexpr int id = HCNN_PROF_SCALE; };
template <> struct KernelClass<ScaleKernel> { static constexpr int id = HCNN_PROF_SCALE; };
template <int A> struct KernelClass<RelinMacKernel<A>> { static constexpr int id = HCNN_PROF_RELIN_MAC; };
template <int A, int B, int C> struct KernelClass<RelinFused<A, B, C>> { static constexpr int id = HCNN_PROF_RELIN_FUSED; };
template <int A, int B> struct KernelClass<TensorFused<A, B>> { static constexpr int id = HCNN_PROF_TENSOR; };
template <int F, bool S> struct KernelClass<MacKernel<F, S>> { static constexpr int id = HCNN_PROF_SCALAR_MAC; };
template <int F> struct KernelClass<MacKernelDirect<F>> { static constexpr int id = HCNN_PROF_SCALAR_MAC; };

int take_event(hcnn_ctx* c, hcnn_event_t* ev) {
  if (!c->free_events.empty()) {
    *ev = c->free_events.back();
    c->free_events.pop_back();
    return 0;
  }
  return event_create(ev);
}

// Launch on the context's stream; with profiling on, bracket the launch with two events.
// `units` (default: the grid) is what the profile counts: the rows of an NTT launch whose grid is padded.
template <class K, class Args>
int run(hcnn_ctx* c, size_t grid, size_t lds_bytes, const Args& a, size_t units = 0) {
  const hcnn_stream_t stream = c->stream;
  if (!c->profile || grid == 0) return launch<K>(stream, grid, lds_bytes, a);
  hcnn_ctx::Pending pd;
  pd.cls = KernelClass<K>::id;
  pd.blocks = units ? units : grid;
  int e;
  if ((e = take_event(c, &pd.start))) return e;
  if ((e = take_event(c, &pd.stop))) return e;
  if ((e = event_record(pd.start, stream))) return e;
  if ((e = launch<K>(stream, grid, lds_bytes, a))) return e;
  if ((e = event_record(pd.stop, stream))) return e;
  c->pending.push_back(pd);
  return 0;
}

int fold_profile(hcnn_ctx* c) {
  if (c->pending.empty()) return 0;
  int e = stream_sync(c->stream);
  if (e) return e;
  for (auto& pd : c->pending) {
    float ms = 0.f;
    if ((e = event_elapsed_ms(&ms, pd.start, pd.stop))) return e;
    c->prof_launches[pd.cls] += 1;
    c->prof_blocks[pd.cls] += pd.blocks;
    c->prof_ms[pd.cls] += ms;
    c->free_events.push_back(pd.start);
    c->free_events.push_back(pd.stop);
  }
  c->pending.clear();
  return 0;
}

// Tables of an exact centred base conversion src -> dst.
//   zfac[i]   extra factor folded into z_i (1 or t), also used as xmul
//   fold_inv  when true the tables give -(x * M^-1): Bp = m'_j - m_i^-1, Vp = 1
//             otherwise they give x:                 Bp = M/m_i mod m'_j, Vp = m'_j - M mod m'_j
//   dst_is_rns_prime  the destinations are ciphertext / auxiliary primes (dst_pinv holds -m'_j^-1 mod 2^32)
//   extra_terms       further products of the same size that the kernels add to each destination sum; when the
//             whole sum fits (bconv_use_mont) Bp and Vp are stored with an extra factor 2^32 mod m'_j (Montgomery form)
BConvHost make_bconv(const std::vector<uint32_t>& src, const std::vector<uint32_t>& dst, uint64_t zfac,
                     bool fold_inv, bool dst_is_rns_prime, uint32_t extra_terms = 0) {
  BConvHost h;
  h.ks = (uint32_t)src.size();
  h.kd = (uint32_t)dst.size();
  for (uint32_t i = 0; i < h.ks; ++i) {
    const uint32_t m = src[i];
    h.src_mod.push_back(h_mod(m));
    const uint32_t Mi_inv = h_inv(h_prod_mod(src, (int)i, m), m);        // (M/m_i)^-1 mod m_i
    h.zmul.push_back(h_shoup(h_mulmod(Mi_inv, (uint32_t)(zfac % m), m), m));
    h.xmul.push_back(h_shoup((uint32_t)(zfac % m), m));
  }
  h.ginv.assign((size_t)h.ks * h.ks, 0);
  for (uint32_t i = 0; i < h.ks; ++i)
    for (uint32_t l = 0; l < i; ++l) h.ginv[(size_t)i * h.ks + l] = h_inv(src[l] % src[i], src[i]);
  // mixed-radix digits of (M-1)/2, whose residue mod m_i is (m_i-1)/2
  h.half.assign(h.ks, 0);
  for (uint32_t i = 0; i < h.ks; ++i) {
    uint32_t tt = (src[i] - 1) / 2;
    for (uint32_t l = 0; l < i; ++l) {
      uint32_t al = h.half[l] % src[i];
      tt = (tt + src[i] - al) % src[i];
      tt = h_mulmod(tt, h.ginv[(size_t)i * h.ks + l], src[i]);
    }
    h.half[i] = tt;
  }
  h.Bp.assign((size_t)h.ks * h.kd, 0);
  h.Vp.assign(h.kd, 0);
  for (uint32_t j = 0; j < h.kd; ++j) {
    const uint32_t mj = dst[j];
    if (dst_is_rns_prime) h.dst_mod.push_back(h_mod(mj));
    else { Mod dm{}; dm.p = mj; h.dst_mod.push_back(dm); }
    for (uint32_t i = 0; i < h.ks; ++i)
      h.Bp[(size_t)i * h.kd + j] = fold_inv ? mj - h_inv(src[i] % mj, mj) : h_prod_mod(src, (int)i, mj);
    h.Vp[j] = fold_inv ? 1u : (mj - h_prod_mod(src, -1, mj)) % mj;
    h.mont = (dst_is_rns_prime && bconv_use_mont(h.ks, extra_terms)) ? 1u : 0u;
    if (h.mont) {
      const uint32_t r32 = (uint32_t)((1ull << 32) % mj);
      for (uint32_t i = 0; i < h.ks; ++i) h.Bp[(size_t)i * h.kd + j] = h_mulmod(h.Bp[(size_t)i * h.kd + j], r32, mj);
      h.Vp[j] = h_mulmod(h.Vp[j], r32, mj);
    }
    h.dst_pinv.push_back(dst_is_rns_prime ? h_neg_inv32(mj) : 0u);
  }
  h.BpT.assign((size_t)h.ks * h.kd, 0);
  for (uint32_t i = 0; i < h.ks; ++i)
    for (uint32_t j = 0; j < h.kd; ++j) h.BpT[(size_t)j * h.ks + i] = h.Bp[(size_t)i * h.kd + j];
  return h;
}

int upload_bconv(hcnn_ctx* c, const BConvHost& h, BConvDev* d) {
  int e;
  Mod* sm; Mod* dm; ShoupConst* zm; ShoupConst* xm; uint32_t* gi; uint32_t* hf; uint32_t* B; uint32_t* BT; uint32_t* Mm; uint32_t* pi;
  if ((e = upload(c, h.src_mod, &sm))) return e;
  if ((e = upload(c, h.dst_mod, &dm))) return e;
  if ((e = upload(c, h.zmul, &zm))) return e;
  if ((e = upload(c, h.xmul, &xm))) return e;
  if ((e = upload(c, h.ginv, &gi))) return e;
  if ((e = upload(c, h.half, &hf))) return e;
  if ((e = upload(c, h.Bp, &B))) return e;
  if ((e = upload(c, h.BpT, &BT))) return e;
  if ((e = upload(c, h.Vp, &Mm))) return e;
  if ((e = upload(c, h.dst_pinv, &pi))) return e;
  d->ks = h.ks; d->kd = h.kd;
  d->src_mod = sm; d->dst_mod = dm; d->zmul = zm; d->xmul = xm;
  d->ginv = gi; d->half = hf; d->Bp = B; d->BpT = BT; d->Vp = Mm; d->dst_pinv = pi; d->mont = h.mont;
  return 0;
}

int build_tables(hcnn_ctx* c) {
  const uint32_t n = c->n, L = c->k + c->kp;
  std::vector<uint32_t> all = c->q;
  all.insert(all.end(), c->p.begin(), c->p.end());

  std::vector<Mod> mods;
  std::vector<NttLimb> limbs;
  std::vector<ShoupConst> twf((size_t)L * n), twi((size_t)L * n);
  std::vector<uint32_t> pw(2 * (size_t)n);
  for (uint32_t l = 0; l < L; ++l) {
    const uint32_t p = all[l];
    const uint32_t psi = h_root_of_unity(n, p);
    uint64_t v = 1;
    for (uint32_t e = 0; e < 2 * n; ++e) { pw[e] = (uint32_t)v; v = v * psi % p; }
    twf[(size_t)l * n] = h_shoup(0, p);
    twi[(size_t)l * n] = h_shoup(0, p);
    for (uint32_t node = 1; node < n; ++node) {
      const uint32_t e = h_brev(node, (int)c->logn);
      twf[(size_t)l * n + node] = h_shoup(pw[e], p);
      // the forward butterflies use the twiddle negated modulo 2^32 (their product is kept negated)
      twf[(size_t)l * n + node].w = 0u - twf[(size_t)l * n + node].w;
      twi[(size_t)l * n + node] = h_shoup(pw[2 * n - e], p);
    }
    NttLimb nl;
    nl.m = h_mod(p);
    const uint32_t ninv = h_inv(n % p, p);
    nl.ninv = h_shoup(ninv, p);
    nl.w1ninv = h_shoup(h_mulmod(twi[(size_t)l * n + 1].w, ninv, p), p);
    const uint32_t ninv_r = h_mulmod(ninv, nl.m.c32, p);                     // c32 = 2^32 mod p
    nl.ninv_r = h_shoup(ninv_r, p);
    nl.w1ninv_r = h_shoup(h_mulmod(twi[(size_t)l * n + 1].w, ninv_r, p), p);
    nl.pinv = h_neg_inv32(p);
    nl.pneg = 0u - p;
    nl.zero = 0;
    nl.pad = 0;
    mods.push_back(nl.m);
    limbs.push_back(nl);
  }
  int e;
  if ((e = upload(c, mods, &c->d_mods))) return e;
  if ((e = upload(c, limbs, &c->d_limbs))) return e;
  if ((e = upload(c, twf, &c->d_tw_fwd))) return e;
  if ((e = upload(c, twi, &c->d_tw_inv))) return e;

  // floor(q/t) mod q_l = -(q mod t) * t^-1 mod q_l   (q = 0 mod q_l)
  const uint64_t q_mod_t = h_prod_mod64(c->q, -1, c->t);
  std::vector<ShoupConst> delta;
  for (uint32_t l = 0; l < c->k; ++l) {
    const uint32_t ql = c->q[l];
    const uint32_t v = h_mulmod((ql - (uint32_t)(q_mod_t % ql)) % ql, h_inv((uint32_t)(c->t % ql), ql), ql);
    delta.push_back(h_shoup(v, ql));
  }
  if ((e = upload(c, delta, &c->d_delta))) return e;

  // decryption: r = [t*x]_q converted to the modulus t
  if (c->t < (1ull << 32)) {
    const uint32_t t32 = (uint32_t)c->t;
    BConvHost h = make_bconv(c->q, std::vector<uint32_t>{t32}, c->t, false, false);
    if ((e = upload_bconv(c, h, &c->dec))) return e;
    const uint32_t qinv_t = h_inv((uint32_t)q_mod_t, t32);
    c->neg_qinv_t = (t32 - qinv_t) % t32;
  } else {
    // source side of the same conversion; the destination constants modulo the wide t live in 64-bit words
    BConvHost h = make_bconv(c->q, std::vector<uint32_t>{}, c->t, false, false);
    if ((e = upload_bconv(c, h, &c->dec))) return e;
    std::vector<uint64_t> tab;
    for (uint32_t i = 0; i < c->k; ++i) tab.push_back(h_prod_mod64(c->q, (int)i, c->t));
    tab.push_back((c->t - q_mod_t) % c->t);
    tab.push_back((c->t - h_powmod64(q_mod_t, c->t - 2, c->t)) % c->t);
    if ((e = upload(c, tab, &c->d_dec_wide))) return e;
  }
  if (c->kp) {
    BConvHost h_ext = make_bconv(c->q, c->p, 1, false, true);
    BConvHost h_to_p = make_bconv(c->q, c->p, c->t, true, true, 1);      // + the term of d'_j
    BConvHost h_to_q = make_bconv(c->p, c->q, 1, false, true);
    if ((e = upload_bconv(c, h_ext, &c->ext))) return e;
    if ((e = upload_bconv(c, h_to_p, &c->to_p))) return e;
    if ((e = upload_bconv(c, h_to_q, &c->to_q))) return e;
    std::vector<uint32_t> tq;
    for (uint32_t j = 0; j < c->kp; ++j) {
      const uint32_t pj = c->p[j];
      // t * q^-1 mod p_j, in the form of the constants it is summed with
      uint32_t v = h_mulmod((uint32_t)(c->t % pj), h_inv(h_prod_mod(c->q, -1, pj), pj), pj);
      if (h_to_p.mont) v = h_mulmod(v, (uint32_t)((1ull << 32) % pj), pj);
      tq.push_back(v);
    }
    if ((e = upload(c, tq, &c->d_tq_inv))) return e;
  }
  std::vector<unsigned long long> zeros(2, 0);
  if ((e = upload(c, zeros, &c->d_counters))) return e;
  return 0;
}

int ensure_work(hcnn_ctx* c, size_t bytes) {
  if (bytes <= c->work_bytes) return 0;
  if (c->work) {
    int e = stream_sync(c->stream);
    if (e) return e;
    dev_free(c->work);
    c->work = nullptr;
    c->work_bytes = 0;
  }
  void* ptr = nullptr;
  int e = dev_malloc(&ptr, bytes);
  if (e) return e;
  c->work = (uint32_t*)ptr;
  c->work_bytes = bytes;
  return 0;
}

// ---------------------------------------------------------------- NTT dispatch
struct NttRows {
  const uint32_t* in;
  uint32_t* out;
  size_t rows;
  uint32_t cycle, limb_base;
  uint32_t in_group_rows, in_row0, out_group_rows, out_row0;
  const uint32_t* aux = nullptr;
  uint32_t own_limbs = 0;
};

template <int LOGN, int LOGR>
int ntt_launch(hcnn_ctx* c, const NttRows& r, bool inverse, int io) {
  NttArgs a;
  a.in = r.in; a.out = r.out; a.aux = r.aux;
  a.tw = inverse ? c->d_tw_inv : c->d_tw_fwd;
  a.limbs = c->d_limbs;
  a.limb_cycle = r.cycle; a.limb_base = r.limb_base;
  a.in_group_rows = r.in_group_rows; a.in_row0 = r.in_row0;
  a.out_group_rows = r.out_group_rows; a.out_row0 = r.out_row0;
  a.n_rows = (uint32_t)r.rows;
  a.own_limbs = r.own_limbs;
  const size_t lds = NttGeom<LOGN, LOGR>::kLdsBytes;
  if (inverse) {
    const size_t g3 = ntt_grouped_grid(r.rows, 3);
    if (io == kNttLoadTensor) return run<NttInv<LOGN, LOGR, kNttLoadTensor>>(c, g3, lds, a, r.rows);
    if (io == kNttLoadTensorMul) return run<NttInv<LOGN, LOGR, kNttLoadTensorMul>>(c, g3, lds, a, r.rows);
    if (io == kNttStoreAdd) return run<NttInv<LOGN, LOGR, kNttStoreAdd>>(c, r.rows, lds, a);
    return run<NttInv<LOGN, LOGR>>(c, r.rows, lds, a);
  }
  // The largest ring runs its forward transforms as two workgroups per row (first stage folded into the load):
  // a whole row of it takes the LDS of a compute unit, half a row leaves room for two workgroups.  Each of the two
  // reads the whole row, so the form needs an output that is not its input.
  if constexpr (LOGN == 15) {
    if (r.in != r.out) {
      const size_t lds_h = NttGeom<LOGN - 1, LOGR>::kLdsBytes;
      if (io == kNttLoadDigit) {
        using K = NttFwd<LOGN, LOGR, kNttLoadDigit, 1>;
        return run<K>(c, K::grid(ntt_grouped_grid(r.rows, r.cycle)), lds_h, a, r.rows);
      }
      if (io == kNttStoreLazy) {
        using K = NttFwd<LOGN, LOGR, kNttStoreLazy, 1>;
        return run<K>(c, K::grid(r.rows), lds_h, a, r.rows);
      }
      using K = NttFwd<LOGN, LOGR, kNttPlain, 1>;
      return run<K>(c, K::grid(r.rows), lds_h, a, r.rows);
    }
  }
  if (io == kNttLoadDigit)
    return run<NttFwd<LOGN, LOGR, kNttLoadDigit>>(c, ntt_grouped_grid(r.rows, r.cycle), lds, a, r.rows);
  if (io == kNttStoreLazy) return run<NttFwd<LOGN, LOGR, kNttStoreLazy>>(c, r.rows, lds, a);
  return run<NttFwd<LOGN, LOGR>>(c, r.rows, lds, a);
}

int ntt_rows(hcnn_ctx* c, const NttRows& r, bool inverse, int io = kNttPlain) {
  switch (c->logn) {
    case 10: return ntt_launch<10, 4>(c, r, inverse, io);
    case 11: return ntt_launch<11, 4>(c, r, inverse, io);
    case 12: return ntt_launch<12, 4>(c, r, inverse, io);
    case 13: return ntt_launch<13, 5>(c, r, inverse, io);
    // n = 2^14: 16 residues per thread (1024 threads, four passes) give twice the waves per compute unit of the
    // 32-residue shape, whose 66 KiB of LDS per row allow only two workgroups; measured 8-10 % faster per row
    case 14: return ntt_launch<14, 4>(c, r, inverse, io);
    case 15: return ntt_launch<15, 5>(c, r, inverse, io);
  }
  return HCNN_ERR_N;
}

// dense rows [rows][n], limb = base + r % cycle
int ntt_dense(hcnn_ctx* c, const uint32_t* in, uint32_t* out, size_t rows, uint32_t cycle, bool inverse,
              int io = kNttPlain, const uint32_t* aux = nullptr, uint32_t own_limbs = 0) {
  NttRows r{in, out, rows, cycle, 0, cycle, 0, cycle, 0, aux, own_limbs};
  return ntt_rows(c, r, inverse, io);
}

// Base-conversion kernels: register-resident variants for the basis sizes of the standard
// parameter sets, the generic LDS-column kernels otherwise (about four times slower in the scaling step).
// k' = k + 1 covers t = 65537 up to n = 8192, k' = k + 2 the larger rings and the larger plaintext moduli.
#define HCNN_REGISTER_BASES(X)                                                                          \
  X(2, 3) X(3, 4) X(4, 5) X(5, 6) X(6, 7) X(7, 8) X(8, 9) X(9, 10) X(10, 11) X(11, 12) X(12, 13)        \
  X(4, 6) X(6, 8) X(8, 10) X(10, 12) X(11, 13) X(12, 14) X(14, 16) X(16, 18) X(24, 26)
int ext_dispatch(hcnn_ctx* c, size_t grid, const ExtArgs& a) {
  const uint32_t k = c->k, kp = c->kp;
#define HCNN_EXT_CASE(K, KP) \
  if (k == K && kp == KP) return run<ExtKernelT<K, KP>>(c, grid, ExtKernelT<K, KP>::lds_bytes(), a);
  HCNN_REGISTER_BASES(HCNN_EXT_CASE)
#undef HCNN_EXT_CASE
  return run<ExtKernel>(c, grid, ExtKernel::lds_bytes(k), a);
}

int scale_dispatch(hcnn_ctx* c, size_t grid, const ScaleArgs& a) {
  const uint32_t k = c->k, kp = c->kp;
#define HCNN_SCALE_CASE(K, KP) \
  if (k == K && kp == KP) return run<ScaleKernelR<K, KP>>(c, grid, ScaleKernelR<K, KP>::lds_bytes(), a);
  HCNN_REGISTER_BASES(HCNN_SCALE_CASE)
#undef HCNN_SCALE_CASE
  return run<ScaleKernel>(c, grid, ScaleKernel::lds_bytes(k, kp), a);
}

template <int FT>
int mac_launch(hcnn_ctx* c, size_t grid, const MacArgs& a) {
  const size_t lds = MacKernel<FT>::lds_bytes(a.F, a.T);
  const size_t tiles = grid / a.G;
  const bool offsets_fit = (uint64_t)a.n_in * 2 * a.k * a.n / 4 <= 0xffffffffull;   // 16-byte offsets kept in 32 bits
  if (lds <= 64 * 1024 && lds <= c->max_lds && a.chunk >= kMacBatch && a.T >= kMacBatch && offsets_fit) {
    MacArgs b = a;
    b.chunk = a.chunk / kMacBatch * kMacBatch;      // the staged kernel reduces at batch boundaries
    // At most four workgroups per compute unit (requested through the LDS size): the inputs that the resident
    // workgroups of a die gather from then stay within its L2 (measured: 5-10 % faster on convolution shapes).
    const size_t lds_req = std::max<size_t>(lds, 36 * 1024);
    if (FT <= 8 && a.T % kMacBatch != 0)        // padded rows at few filters: skip the padding terms' multiply-adds
      return run<MacKernel<FT, true>>(c, MacKernel<FT>::grid(tiles, a.G), lds_req, b);
    return run<MacKernel<FT>>(c, MacKernel<FT>::grid(tiles, a.G), lds_req, b);
  }
  return run<MacKernelDirect<FT>>(c, grid, 0, a);
}

int mac_dispatch(hcnn_ctx* c, size_t grid, const MacArgs& a) {
  switch (a.F) {
    case 1: return mac_launch<1>(c, grid, a);
    case 2: return mac_launch<2>(c, grid, a);
    case 3: return mac_launch<3>(c, grid, a);
    case 4: return mac_launch<4>(c, grid, a);
    case 5: return mac_launch<5>(c, grid, a);
    case 6: return mac_launch<6>(c, grid, a);
    case 7: return mac_launch<7>(c, grid, a);
    case 8: return mac_launch<8>(c, grid, a);
    case 9: return mac_launch<9>(c, grid, a);
    case 10: return mac_launch<10>(c, grid, a);
    case 11: return mac_launch<11>(c, grid, a);
    case 12: return mac_launch<12>(c, grid, a);
    case 13: return mac_launch<13>(c, grid, a);
    case 14: return mac_launch<14>(c, grid, a);
    case 15: return mac_launch<15>(c, grid, a);
    case 16: return mac_launch<16>(c, grid, a);
  }
  return HCNN_ERR_ARG;
}

// Occupancy of the two long-running one-kernel forms for this ring and basis, asked of the runtime once.
int query_fused_occupancy(hcnn_ctx* c) {
  if (c->logn > 14) return 0;                       // neither form exists for the largest ring
  const uint32_t k = c->k;
  int e = 0, r = 1, t = 1;
#define HCNN_OCC(LOGN, LOGR)                                                                                          \
  {                                                                                                                   \
    const size_t lds = NttGeom<LOGN, LOGR>::kLdsBytes;                                                                \
    e = k <= 8    ? resident_workgroups_per_cu<RelinFused<LOGN, LOGR, kNttFusedMac>, RelinFusedArgs>(lds, &r)         \
        : k <= 16 ? resident_workgroups_per_cu<RelinFused<LOGN, LOGR, kNttFusedMac16>, RelinFusedArgs>(lds, &r)       \
                  : resident_workgroups_per_cu<RelinFused<LOGN, LOGR, kNttFusedMacAny>, RelinFusedArgs>(lds, &r);     \
  }
  switch (c->logn) {
    case 10: HCNN_OCC(10, 4) break;
    case 11: HCNN_OCC(11, 4) break;
    case 12: HCNN_OCC(12, 4) break;
    case 13: HCNN_OCC(13, 5) break;
    case 14: HCNN_OCC(14, 4) break;
  }
#undef HCNN_OCC
  if (e) return e;
  switch (c->logn) {
    case 10: e = resident_workgroups_per_cu<TensorFused<10, 4>, TensorFusedArgs>(NttGeom<10, 4>::kLdsBytes, &t); break;
    case 11: e = resident_workgroups_per_cu<TensorFused<11, 4>, TensorFusedArgs>(NttGeom<11, 4>::kLdsBytes, &t); break;
    case 12: e = resident_workgroups_per_cu<TensorFused<12, 4>, TensorFusedArgs>(NttGeom<12, 4>::kLdsBytes, &t); break;
    case 13: e = resident_workgroups_per_cu<TensorFused<13, 4>, TensorFusedArgs>(NttGeom<13, 4>::kLdsBytes, &t); break;
    case 14: e = resident_workgroups_per_cu<TensorFused<14, 4>, TensorFusedArgs>(NttGeom<14, 4>::kLdsBytes, &t); break;
  }
  if (e) return e;
  c->relin_fused_wgs = (uint32_t)r;
  c->tensor_fused_wgs = (uint32_t)t;
  return 0;
}

// Median duration in milliseconds of `reps` launches of one kernel on the context's stream, one event pair each.
template <class K, class Args>
int timed_launches(hcnn_ctx* c, size_t grid, const Args& a, int reps, double* ms_out) {
  hcnn_event_t e0, e1;
  int e;
  if ((e = event_create(&e0))) return e;
  if ((e = event_create(&e1))) { event_destroy(e0); return e; }
  std::vector<float> ms;
  e = launch<K>(c->stream, grid, 0, a);                     // warm-up
  for (int r = 0; r < reps && !e; ++r) {
    float t = 0.f;
    if ((e = event_record(e0, c->stream))) break;
    if ((e = launch<K>(c->stream, grid, 0, a))) break;
    if ((e = event_record(e1, c->stream))) break;
    if ((e = stream_sync(c->stream))) break;
    if ((e = event_elapsed_ms(&t, e0, e1))) break;
    ms.push_back(t);
  }
  event_destroy(e0);
  event_destroy(e1);
  if (e) return e;
  std::sort(ms.begin(), ms.end());
  *ms_out = ms[ms.size() / 2];
  return 0;
}

}  // namespace

// ================================================================= C ABI
extern "C" {

int hcnn_gen_primes(uint32_t n, uint32_t count, uint32_t* primes_host) {
  if (!primes_host) return HCNN_ERR_NULL;
  if (!valid_n(n)) return HCNN_ERR_N;
  if (count == 0 || count > 2 * HCNN_MAX_LIMBS) return HCNN_ERR_ARG;
  const uint32_t step = 2 * n;
  uint32_t c = ((1u << 30) - 2) / step * step + 1;
  uint32_t found = 0;
  while (found < count) {
    if (c <= (1u << 29)) return HCNN_ERR_ARG;
    if (h_is_prime(c)) primes_host[found++] = c;
    c -= step;
  }
  return HCNN_OK;
}

int hcnn_min_aux_count(uint32_t n, uint32_t k, const uint32_t* q, uint64_t t, const uint32_t* cand,
                       uint32_t n_cand, uint32_t* k_aux_out) {
  if (!q || !cand || !k_aux_out) return HCNN_ERR_NULL;
  if (!valid_n(n)) return HCNN_ERR_N;
  if (k == 0 || k > HCNN_MAX_LIMBS || n_cand == 0 || n_cand > 2 * HCNN_MAX_LIMBS) return HCNN_ERR_ARG;
  int e = check_primes(n, q, k, cand, n_cand);
  if (e) return e;
  if (t < 2 || t >= (1ull << 47)) return HCNN_ERR_T;
  for (uint32_t kp = 1; kp <= n_cand && kp <= HCNN_MAX_LIMBS; ++kp) {
    if (aux_sufficient(n, q, k, t, cand, kp)) {
      *k_aux_out = kp;
      return HCNN_OK;
    }
  }
  return HCNN_ERR_AUX;
}

int hcnn_ctx_create(hcnn_ctx** out, uint32_t n, uint32_t k, const uint32_t* q, uint32_t k_aux,
                    const uint32_t* p, uint64_t t, void* hip_stream) {
  if (!out || !q || (k_aux && !p)) return HCNN_ERR_NULL;
  *out = nullptr;
  if (!valid_n(n)) return HCNN_ERR_N;
  if (k == 0 || k > HCNN_MAX_LIMBS || k_aux > HCNN_MAX_LIMBS) return HCNN_ERR_ARG;
  int e = check_primes(n, q, k, p, k_aux);
  if (e) return e;
  if (t < 2 || t >= (1ull << 47) || !h_is_prime64(t)) return HCNN_ERR_T;
  for (uint32_t i = 0; i < k; ++i)
    if (q[i] == t) return HCNN_ERR_T;
  for (uint32_t j = 0; j < k_aux; ++j)
    if (p[j] == t) return HCNN_ERR_T;
  if (k_aux && !aux_sufficient(n, q, k, t, p, k_aux)) return HCNN_ERR_AUX;

  hcnn_ctx* c = new (std::nothrow) hcnn_ctx();
  if (!c) return HCNN_ERR_ARG;
  c->n = n;
  while ((1u << c->logn) < n) ++c->logn;
  c->k = k; c->kp = k_aux; c->t = t;
  c->q.assign(q, q + k);
  if (k_aux) c->p.assign(p, p + k_aux);
  c->stream = (hcnn_stream_t)hip_stream;
  c->max_lds = max_lds_bytes();
  c->compute_units = compute_unit_count();
  if (c->max_lds < (size_t)(n + n / 32) * 4) {
    delete c;
    return HCNN_ERR_NODEVICE;
  }
  e = build_tables(c);
  if (!e) e = static_scratch_of_current_device(&c->static_scratch);
  if (!e) e = query_fused_occupancy(c);
  if (e) {
    hcnn_ctx_destroy(c);
    return e;
  }
  *out = c;
  return HCNN_OK;
}

int hcnn_ctx_destroy(hcnn_ctx* c) {
  if (!c) return HCNN_ERR_NULL;
  stream_sync(c->stream);
  fold_profile(c);
  for (auto ev : c->free_events) event_destroy(ev);
  for (void* p : c->owned) dev_free(p);
  if (c->d_evk_hat) dev_free(c->d_evk_hat);
  if (c->work) dev_free(c->work);
  delete c;
  return HCNN_OK;
}

int hcnn_set_stream(hcnn_ctx* c, void* hip_stream) {
  if (!c) return HCNN_ERR_NULL;
  int e = stream_sync(c->stream);
  if (e) return e;
  c->stream = (hcnn_stream_t)hip_stream;
  return HCNN_OK;
}

int hcnn_set_relin_key(hcnn_ctx* c, const uint32_t* evk_dev) {
  if (!c || !evk_dev) return HCNN_ERR_NULL;
  if (!aligned16(evk_dev)) return HCNN_ERR_ALIGN;
  const size_t rows = (size_t)c->k * 2 * c->k;
  if (!c->d_evk_hat) {
    void* ptr = nullptr;
    int e = dev_malloc(&ptr, rows * c->n * 4);
    if (e) return e;
    c->d_evk_hat = (uint32_t*)ptr;
  }
  int e = ntt_dense(c, evk_dev, c->d_evk_hat, rows, c->k, false);
  if (e) return e;
  c->has_key = true;
  return HCNN_OK;
}

int hcnn_ntt_fwd(hcnn_ctx* c, uint32_t* polys_dev, size_t n_polys) {
  if (!c) return HCNN_ERR_NULL;
  if (n_polys == 0) return HCNN_OK;
  if (!polys_dev) return HCNN_ERR_NULL;
  if (!aligned16(polys_dev)) return HCNN_ERR_ALIGN;
  if (n_polys > (size_t)0x7fffffff / c->k) return HCNN_ERR_ARG;
  return ntt_dense(c, polys_dev, polys_dev, n_polys * c->k, c->k, false);
}

int hcnn_ntt_inv(hcnn_ctx* c, uint32_t* polys_dev, size_t n_polys) {
  if (!c) return HCNN_ERR_NULL;
  if (n_polys == 0) return HCNN_OK;
  if (!polys_dev) return HCNN_ERR_NULL;
  if (!aligned16(polys_dev)) return HCNN_ERR_ALIGN;
  if (n_polys > (size_t)0x7fffffff / c->k) return HCNN_ERR_ARG;
  return ntt_dense(c, polys_dev, polys_dev, n_polys * c->k, c->k, true);
}

int hcnn_ct_scalar_mac(hcnn_ctx* c, const uint32_t* in, size_t n_in, const uint32_t* idx, const int32_t* w,
                       int32_t w_abs_max, size_t G, size_t F, size_t T, uint32_t* out) {
  if (!c) return HCNN_ERR_NULL;
  if (G == 0) return HCNN_OK;
  if (!in || !idx || !w || !out) return HCNN_ERR_NULL;
  if (!aligned16(in) || !aligned16(out)) return HCNN_ERR_ALIGN;
  if (n_in == 0 || n_in > 0xffffffffull || F == 0 || F > HCNN_MAX_FILTERS || T == 0 || T > 0xffffffffull ||
      w_abs_max < 0)
    return HCNN_ERR_ARG;
  if (G == 0) return HCNN_OK;
  const size_t ct_words = (size_t)2 * c->k * c->n;
  const size_t tiles = ct_words / (kEwThreads * kEwVec);
  if (G > (size_t)0x7fffffff / tiles) return HCNN_ERR_ARG;
  MacArgs a;
  a.in = in; a.idx = idx; a.w = w; a.out = out;
  a.mods = c->d_mods; a.k = c->k; a.n = c->n;
  a.n_in = (uint32_t)n_in; a.G = (uint32_t)G; a.F = (uint32_t)F; a.T = (uint32_t)T;
  a.w_abs_max = w_abs_max;
  // partial sums stay below 2^62 in magnitude: chunk * w_abs_max * 2^30 + 2^30 <= 2^62
  const uint64_t wm = w_abs_max > 0 ? (uint64_t)w_abs_max : 1;
  uint64_t chunk = ((1ull << 32) - 1) / wm;
  if (chunk > (1u << 30)) chunk = 1u << 30;          // a row shorter than the chunk is never folded midway
  a.chunk = (uint32_t)chunk;
  a.bad_counter = c->d_counters + 1;
  return mac_dispatch(c, G * tiles, a);
}

// Workgroups of the one-kernel relinearisation / of the one-kernel squaring tensor that the device holds at a time:
// compute units x the per-compute-unit figure that the runtime reported for the compiled kernel when the context
// was created (query_fused_occupancy).  The rounds of these long-running kernels are sized from it.
static size_t relin_fused_slots(const hcnn_ctx* c) { return (size_t)c->compute_units * c->relin_fused_wgs; }
static size_t tensor_fused_slots(const hcnn_ctx* c) { return (size_t)c->compute_units * c->tensor_fused_wgs; }

// HMult of Sec. 2.1 on n_ct pairs (a_i, b_i); b == nullptr squares a (HSquare).
// static_ws: the intermediate polynomials go to this device's copy of the file-scope array `scratch` and nothing is
// allocated; a parameter set whose single ciphertext does not fit that array is refused.
static int mul_relin_impl(hcnn_ctx* c, const uint32_t* in, const uint32_t* in_b, size_t n_ct, uint32_t* out,
                          bool static_ws = false) {
  if (!c) return HCNN_ERR_NULL;
  if (n_ct == 0) return HCNN_OK;
  if (!in || !out) return HCNN_ERR_NULL;
  if (!aligned16(in) || !aligned16(out) || !aligned16(in_b)) return HCNN_ERR_ALIGN;
  if (c->kp == 0) return HCNN_ERR_AUX;
  const uint32_t k = c->k, kp = c->kp, L = k + kp, n = c->n;
  const size_t rn = n;
  const size_t ext_rows = in_b ? 4 * (size_t)L : 2 * (size_t)L;
  if (static_ws && (ext_rows + 3 * L + 3 * k + (size_t)k * k + 2 * k) * rn * 4 > kStaticScratchBytes)
    return HCNN_ERR_SCRATCH;
  if (!c->has_key) return HCNN_ERR_NOKEY;
  // n <= 16384: relinearisation runs as one kernel that needs no buffers for the transformed digits and the sums.
  // (At n = 16384 its 1024-thread workgroup fills a compute unit alone: measured +5..8 % up to 16 primes, no gain
  // with the in-loop folds of longer bases, which stay with the separate kernels; at n = 32768 a row and its sums
  // do not fit the registers of 1024 threads.)
  // Its workgroups are long (k + 2 transforms each), so it only takes whole rounds of resident workgroups; what is
  // left of a batch (all of a small batch) goes through the three separate kernels, which spread k^2 rows per
  // ciphertext over the chip.
  const bool fused = c->fusion != 1 && (c->logn <= 13 || (c->logn == 14 && k <= 16));
  // (the k workgroups of a ciphertext share a die, for its L2: a round is counted per die)
  const size_t fused_round = fused ? relin_fused_slots(c) / kXcds / k * kXcds : 0;   // ciphertexts per round (0: never)
  const size_t words_main = (ext_rows + 3 * L + 3 * k) * rn;
  const size_t words_split = ((size_t)k * k + 2 * k) * rn;
  const size_t words_per_ct = words_main + words_split;
  size_t C = c->square_chunk;
  // 6 GiB of work buffer (of 288 GB): enough rows per launch at every n
  const size_t budget = static_ws ? kStaticScratchBytes : (size_t)6 << 30;
  if (static_ws && C > budget / (words_per_ct * 4)) C = 0;
  if (C == 0) {
    C = budget / (words_per_ct * 4);
    // measured: up to n = 8192 batches of 512 are 3-4 % faster than 256 (the long workgroups of the one-kernel
    // relinearisation leave a longer tail per launch), at n = 16384 128-256 is best; small rings need more
    // ciphertexts to fill the chip at all
    const size_t cap = std::max<size_t>(c->logn <= 13 ? 512 : 256, fused_round);
    if (C > cap) C = cap;
    if (fused_round && C > fused_round) C = C / fused_round * fused_round;   // whole rounds of the one-kernel relinearisation
  }
  if (C < 1) C = 1;
  if (C > n_ct) C = n_ct;
  const size_t need_lds_scale = ScaleKernel::lds_bytes(k, kp);
  if (need_lds_scale > c->max_lds) return HCNN_ERR_NODEVICE;
  // ciphertexts of one internal batch that can take the separate kernels
  const size_t C_split = (fused && fused_round) ? std::min(C, fused_round) : C;
  int e;
  e = static_ws ? 0 : ensure_work(c, (C * words_main + C_split * words_split) * 4);
  if (e) return e;
  uint32_t* ext = static_ws ? c->static_scratch : c->work;
  uint32_t* ext_b = ext + C * 2 * L * rn;                 // used only by the two-operand product
  uint32_t* d = ext + C * ext_rows * rn;
  uint32_t* y = d + C * 3 * L * rn;
  uint32_t* dig = y + C * 3 * k * rn;
  uint32_t* acc = dig + C_split * k * k * rn;
  const size_t ct_words = (size_t)2 * k * rn;
  const size_t bpp = n / kEwThreads;                 // blocks per polynomial, 1 coefficient / thread
  const size_t bpr = n / (kEwThreads * kEwVec);      // blocks per row, 4 coefficients / thread

  // How many ciphertexts of an internal batch of cc take the one-kernel relinearisation (steps 6-8 in one kernel
  // for whole rounds of its workgroups: a row and its two 64-bit sums stay in registers).
  auto fused_count = [&](size_t cc) -> size_t {
    size_t nf = 0;
    if (fused && fused_round) {
      nf = cc / fused_round * fused_round;
      // a last round joins when it is at least 3/8 full (3/4 if it is the only one): measured break-even points
      const size_t rest = cc - nf;
      if (nf ? rest * 8 >= fused_round * 3 : rest * 4 >= fused_round * 3) nf = cc;
      if (c->fusion == 2) nf = cc;
    }
    return nf;
  };
  // Steps 2+3 in one kernel for squarings: its workgroups are long (five transforms) and two fit a compute unit at
  // n = 8192 (one at n = 16384), so it pays from several rounds of workgroups on (measured: +3-5 % from 6 rounds,
  // nothing below).
  auto takes_tensor_fused = [&](size_t cc) {
    return !in_b && c->logn <= 14 && c->fusion != 1 && (c->fusion == 2 || cc * L >= 6 * tensor_fused_slots(c));
  };

  // One internal batch: ciphertexts [c0, c0 + cc) of the call, kept in slots [s0, s0 + cc) of the work arrays, nf of
  // them through the one-kernel relinearisation.
  auto one_batch = [&](size_t c0, size_t cc, size_t s0, size_t nf) -> int {
    int e;
    uint32_t* const b_ext = ext + s0 * 2 * L * rn;
    uint32_t* const b_ext_b = ext_b + s0 * 2 * L * rn;
    uint32_t* const b_d = d + s0 * 3 * L * rn;
    uint32_t* const b_y = y + s0 * 3 * k * rn;
    uint32_t* const b_dig = dig + s0 * k * k * rn;
    uint32_t* const b_acc = acc + s0 * 2 * k * rn;
    // 1. centred lift of c0, c1 extended to the auxiliary primes (only the new rows are written);
    // 2. forward NTT over all k + k' limbs, the first k read from the ciphertext itself
    // (n = 32768: the new rows are staged in the array of the tensor, free until step 3, because the two-workgroup
    // transform of that ring cannot work in place)
    uint32_t* const b_new = c->logn == 15 ? b_d : b_ext;
    ExtArgs ea;
    ea.in = in + c0 * ct_words; ea.out = b_new; ea.bc = c->ext; ea.n = n; ea.band = c->band;
    ea.fallback_counter = c->d_counters;
    if ((e = ext_dispatch(c, cc * 2 * bpp, ea))) return e;
    const bool tensor_fused = takes_tensor_fused(cc);
    if (tensor_fused) {
      TensorFusedArgs ta{in + c0 * ct_words, b_ext, b_d, c->d_tw_fwd, c->d_tw_inv, c->d_limbs, k, L, (uint32_t)(cc * L)};
      const size_t rows = cc * L * 5;
      switch (c->logn) {
        case 10: e = run<TensorFused<10, 4>>(c, cc * L, NttGeom<10, 4>::kLdsBytes, ta, rows); break;
        case 11: e = run<TensorFused<11, 4>>(c, cc * L, NttGeom<11, 4>::kLdsBytes, ta, rows); break;
        case 12: e = run<TensorFused<12, 4>>(c, cc * L, NttGeom<12, 4>::kLdsBytes, ta, rows); break;
        // 16 residues per thread also at n = 8192: with the two transformed operands (2 x 16 registers) the kernel
        // needs 120 registers; at 32 residues per thread it spills
        case 13: e = run<TensorFused<13, 4>>(c, cc * L, NttGeom<13, 4>::kLdsBytes, ta, rows); break;
        case 14: e = run<TensorFused<14, 4>>(c, cc * L, NttGeom<14, 4>::kLdsBytes, ta, rows); break;
        default: e = HCNN_ERR_N; break;
      }
      if (e) return e;
    } else if ((e = ntt_dense(c, b_new, b_ext, cc * 2 * L, L, false, kNttStoreLazy, in + c0 * ct_words, k))) {
      return e;
    }
    if (in_b) {
      uint32_t* const b_new_b = c->logn == 15 ? b_d : b_ext_b;
      ea.in = in_b + c0 * ct_words; ea.out = b_new_b;
      if ((e = ext_dispatch(c, cc * 2 * bpp, ea))) return e;
      if ((e = ntt_dense(c, b_new_b, b_ext_b, cc * 2 * L, L, false, kNttStoreLazy, in_b + c0 * ct_words, k))) return e;
    }
    // 3+4. tensor formed while loading, then back to coefficients: the integer tensor, known mod q*p
    if (in_b) {
      if ((e = ntt_dense(c, b_ext, b_d, cc * 3 * L, L, true, kNttLoadTensorMul, b_ext_b))) return e;
    } else if (!tensor_fused) {
      if ((e = ntt_dense(c, b_ext, b_d, cc * 3 * L, L, true, kNttLoadTensor))) return e;
    }
    // 5. y = round(t/q * d) mod q
    ScaleArgs sa;
    sa.d = b_d; sa.y = b_y; sa.to_p = c->to_p; sa.to_q = c->to_q; sa.tq_inv = c->d_tq_inv; sa.n = n;
    sa.band = c->band; sa.fallback_counter = c->d_counters;
    if ((e = scale_dispatch(c, cc * 3 * bpp, sa))) return e;
    // 6-8 in one kernel
    if (nf) {
      RelinFusedArgs fa{b_y, c->d_evk_hat, out + c0 * ct_words, c->d_tw_fwd, c->d_tw_inv, c->d_limbs, k, (uint32_t)(nf * k)};
      const size_t grid = ntt_grouped_grid(nf * k, k), rows = nf * k * (k + 2);
#define HCNN_FUSED(LOGN, LOGR)                                                                                      \
  (k <= 8 ? run<RelinFused<LOGN, LOGR, kNttFusedMac>>(c, grid, NttGeom<LOGN, LOGR>::kLdsBytes, fa, rows)             \
          : k <= 16 ? run<RelinFused<LOGN, LOGR, kNttFusedMac16>>(c, grid, NttGeom<LOGN, LOGR>::kLdsBytes, fa, rows) \
                    : run<RelinFused<LOGN, LOGR, kNttFusedMacAny>>(c, grid, NttGeom<LOGN, LOGR>::kLdsBytes, fa, rows))
      switch (c->logn) {
        case 10: e = HCNN_FUSED(10, 4); break;
        case 11: e = HCNN_FUSED(11, 4); break;
        case 12: e = HCNN_FUSED(12, 4); break;
        // n = 8192: 32 residues per thread (three passes, 8 waves per compute unit) when the launch holds several
        // rounds of workgroups; a single round runs 5 % shorter at 16 residues per thread (four passes, 16 waves per
        // compute unit hide more of what no other round overlaps).  Both forms hold two workgroups per compute unit.
        case 13: e = nf > std::max<size_t>(fused_round, 1) ? HCNN_FUSED(13, 5) : HCNN_FUSED(13, 4); break;
        case 14: e = HCNN_FUSED(14, 4); break;
        default: e = HCNN_ERR_N; break;
      }
#undef HCNN_FUSED
      if (e) return e;
    }
    const size_t ns = cc - nf;                                // ciphertexts left for the separate kernels
    if (ns == 0) return 0;
    const uint32_t* y_s = b_y + nf * 3 * k * rn;
    uint32_t* out_s = out + (c0 + nf) * ct_words;
    // 6. RNS digits of y2, each reduced modulo every q_j while loading, transformed
    if ((e = ntt_dense(c, y_s, b_dig, ns * k * k, k, false, kNttLoadDigit))) return e;
    // 7. inner product with the evaluation key
    RelinMacArgs ra;
    ra.dig = b_dig; ra.evk = c->d_evk_hat; ra.acc = b_acc; ra.mods = c->d_mods; ra.k = k; ra.n = n;
    // in the plain (ciphertext-major) order every die touches the key tiles of all limbs: 2*k*k*(tiles/8) * 4 KiB
    ra.key_major = (bpr % kXcds == 0 && (size_t)2 * k * k * (bpr / kXcds) * 4096 > ((size_t)1 << 20)) ? 1u : 0u;
    if (c->relin_order == 1) ra.key_major = 0;
    if (c->relin_order == 2 && bpr % kXcds == 0) ra.key_major = 1;
    // groups of kRelinCts ciphertexts share their loads of the key; the remainder goes one by one
    constexpr int kRelinCts = 4;
    const size_t full = ns / kRelinCts;
    if (full) {
      ra.n_grp = (uint32_t)full; ra.ct_base = 0;
      if ((e = run<RelinMacKernel<kRelinCts>>(c, full * k * bpr, 0, ra))) return e;
    }
    if (ns % kRelinCts) {
      ra.n_grp = (uint32_t)(ns % kRelinCts); ra.ct_base = (uint32_t)(full * kRelinCts);
      if ((e = run<RelinMacKernel<1>>(c, (ns % kRelinCts) * k * bpr, 0, ra))) return e;
    }
    // 8. c'_b = y_b + sum_i evk[i][b] * digit_i : inverse transform with the addition on the way out
    return ntt_dense(c, b_acc, out_s, ns * 2 * k, k, true, kNttStoreAdd, y_s);
  };

  for (size_t c0 = 0; c0 < n_ct; c0 += C) {
    const size_t cc = std::min(C, n_ct - c0);
    const size_t nf = fused_count(cc);
    if ((e = one_batch(c0, cc, 0, nf))) return e;
  }
  return HCNN_OK;
}

int hcnn_ct_square_relin(hcnn_ctx* c, const uint32_t* in, size_t n_ct, uint32_t* out) {
  return mul_relin_impl(c, in, nullptr, n_ct, out);
}

int hcnn_ct_mul_relin(hcnn_ctx* c, const uint32_t* a, const uint32_t* b, size_t n_ct, uint32_t* out) {
  if (n_ct != 0 && c && !b) return HCNN_ERR_NULL;
  return mul_relin_impl(c, a, b, n_ct, out);
}

int hcnn_ct_square_relin_noalloc(hcnn_ctx* c, const uint32_t* in, size_t n_ct, uint32_t* out) {
  if (!c) return HCNN_ERR_NULL;
  // no event pair around the launches of this call: an event may have to be created
  const bool profile = c->profile;
  c->profile = false;
  const int e = mul_relin_impl(c, in, nullptr, n_ct, out, true);
  c->profile = profile;
  return e;
}

// ---------------------------------------------------------------- test helpers
int hcnn_keygen(hcnn_ctx* c, const int32_t* s, const uint32_t* a, const int32_t* e_small, const uint32_t* a_evk,
                const int32_t* e_evk, uint32_t* pk_out, uint32_t* evk_out) {
  if (!c || !s || !a || !e_small || !pk_out) return HCNN_ERR_NULL;
  if (evk_out && (!a_evk || !e_evk)) return HCNN_ERR_NULL;
  if (!aligned16(a) || !aligned16(pk_out) || !aligned16(a_evk) || !aligned16(evk_out)) return HCNN_ERR_ALIGN;
  const uint32_t k = c->k, n = c->n;
  const size_t rn = n, poly = (size_t)k * rn;
  const size_t bpp = n / kEwThreads;
  // scratch: s_hat [k][n] | s2 [k][n] | tmp [k*k][n]
  int e = ensure_work(c, (2 * poly + (size_t)k * poly) * 4);
  if (e) return e;
  uint32_t* s_hat = c->work;
  uint32_t* s2 = s_hat + poly;
  uint32_t* tmp = s2 + poly;

  SmallToRnsArgs sr{s, s_hat, c->d_mods, k, n};
  if ((e = run<SmallToRnsKernel>(c, bpp, 0, sr))) return e;
  if ((e = ntt_dense(c, s_hat, s_hat, k, k, false))) return e;

  // pk = (e - a*s, a)
  if ((e = ntt_dense(c, a, tmp, k, k, false))) return e;
  PointMulArgs pm{tmp, s_hat, tmp, c->d_mods, k, n, k, k, 1u};
  if ((e = run<PointMulKernel>(c, (size_t)k * bpp, 0, pm))) return e;
  if ((e = ntt_dense(c, tmp, tmp, k, k, true))) return e;
  AddSmallArgs as{tmp, e_small, nullptr, nullptr, nullptr, pk_out, c->d_mods, k, n, 0u, 2 * k, 0u};
  if ((e = run<AddSmallKernel>(c, (size_t)k * bpp, 0, as))) return e;
  if ((e = copy_d2d(pk_out + poly, a, poly * 4, c->stream))) return e;
  if (!evk_out) return HCNN_OK;

  // s^2, coefficient domain
  PointMulArgs p2{s_hat, s_hat, s2, c->d_mods, k, n, k, k, 0u};
  if ((e = run<PointMulKernel>(c, (size_t)k * bpp, 0, p2))) return e;
  if ((e = ntt_dense(c, s2, s2, k, k, true))) return e;
  // evk[i][0] = g_i*s^2 - (a_i*s + e_i), evk[i][1] = a_i, all components at once
  if ((e = ntt_dense(c, a_evk, tmp, (size_t)k * k, k, false))) return e;
  PointMulArgs pe{tmp, s_hat, tmp, c->d_mods, k, n, k * k, k, 1u};
  if ((e = run<PointMulKernel>(c, (size_t)k * k * bpp, 0, pe))) return e;
  if ((e = ntt_dense(c, tmp, tmp, (size_t)k * k, k, true))) return e;
  AddSmallArgs ae{tmp, e_evk, nullptr, nullptr, nullptr, evk_out, c->d_mods, k, n, 1u, 2 * k, 0u};
  if ((e = run<AddSmallKernel>(c, (size_t)k * k * bpp, 0, ae))) return e;
  AddDiagArgs ad{evk_out, s2, c->d_mods, k, n};
  if ((e = run<AddDiagKernel>(c, (size_t)k * bpp, 0, ad))) return e;
  for (uint32_t i = 0; i < k; ++i)
    if ((e = copy_d2d(evk_out + ((size_t)i * 2 + 1) * poly, a_evk + (size_t)i * poly, poly * 4, c->stream))) return e;
  return HCNN_OK;
}

static int encrypt_impl(hcnn_ctx* c, const uint32_t* pk, const uint32_t* m, const uint64_t* m64, const int32_t* u,
                        const int32_t* e1, const int32_t* e2, size_t n_ct, uint32_t* ct_out) {
  if (!c || !pk || (!m && !m64) || !u || !e1 || !e2 || !ct_out) return HCNN_ERR_NULL;
  if ((m != nullptr) != (c->t < (1ull << 32))) return HCNN_ERR_T;     // word size of the plaintext follows t
  if (!aligned16(pk) || !aligned16(ct_out)) return HCNN_ERR_ALIGN;
  if (n_ct == 0) return HCNN_OK;
  const uint32_t k = c->k, n = c->n;
  const size_t rn = n, poly = (size_t)k * rn;
  const size_t bpp = n / kEwThreads;
  const size_t C = std::min<size_t>(n_ct, 64);
  // scratch: pk_hat [2][k][n] | u_hat [C][k][n] | prod [C][k][n]
  int e = ensure_work(c, (2 * poly + 2 * C * poly) * 4);
  if (e) return e;
  uint32_t* pk_hat = c->work;
  uint32_t* u_hat = pk_hat + 2 * poly;
  uint32_t* prod = u_hat + C * poly;
  if ((e = ntt_dense(c, pk, pk_hat, 2 * (size_t)k, k, false))) return e;
  for (size_t c0 = 0; c0 < n_ct; c0 += C) {
    const size_t cc = std::min(C, n_ct - c0);
    SmallToRnsArgs sr{u + c0 * rn, u_hat, c->d_mods, k, n};
    if ((e = run<SmallToRnsKernel>(c, cc * bpp, 0, sr))) return e;
    if ((e = ntt_dense(c, u_hat, u_hat, cc * k, k, false))) return e;
    for (uint32_t b = 0; b < 2; ++b) {
      PointMulArgs pm{u_hat, pk_hat + b * poly, prod, c->d_mods, k, n, (uint32_t)(cc * k), k, 0u};
      if ((e = run<PointMulKernel>(c, cc * k * bpp, 0, pm))) return e;
      if ((e = ntt_dense(c, prod, prod, cc * k, k, true))) return e;
      AddSmallArgs as{prod, (b == 0 ? e1 : e2) + c0 * rn, (b == 0 && m) ? m + c0 * rn : nullptr,
                      (b == 0 && m64) ? m64 + c0 * rn : nullptr,
                      b == 0 ? c->d_delta : nullptr, ct_out + c0 * 2 * poly, c->d_mods, k, n, 0u, 2 * k, b * k};
      if ((e = run<AddSmallKernel>(c, cc * k * bpp, 0, as))) return e;
    }
  }
  return HCNN_OK;
}

int hcnn_encrypt(hcnn_ctx* c, const uint32_t* pk, const uint32_t* m, const int32_t* u, const int32_t* e1,
                 const int32_t* e2, size_t n_ct, uint32_t* ct_out) {
  if (!m) return HCNN_ERR_NULL;
  return encrypt_impl(c, pk, m, nullptr, u, e1, e2, n_ct, ct_out);
}

int hcnn_encrypt_wide(hcnn_ctx* c, const uint32_t* pk, const uint64_t* m, const int32_t* u, const int32_t* e1,
                      const int32_t* e2, size_t n_ct, uint32_t* ct_out) {
  if (!m) return HCNN_ERR_NULL;
  return encrypt_impl(c, pk, nullptr, m, u, e1, e2, n_ct, ct_out);
}

static int decrypt_impl(hcnn_ctx* c, const int32_t* sk, const uint32_t* ct, size_t n_ct, uint32_t* m_out,
                        uint64_t* m_out64) {
  if (!c || !sk || !ct || (!m_out && !m_out64)) return HCNN_ERR_NULL;
  if ((m_out != nullptr) != (c->t < (1ull << 32))) return HCNN_ERR_T;
  if (!aligned16(ct)) return HCNN_ERR_ALIGN;
  if (n_ct == 0) return HCNN_OK;
  const uint32_t k = c->k, n = c->n;
  const size_t rn = n, poly = (size_t)k * rn;
  const size_t bpp = n / kEwThreads;
  const size_t C = std::min<size_t>(n_ct, 64);
  // scratch: s_hat [k][n] | x [C][k][n]
  int e = ensure_work(c, (poly + C * poly) * 4);
  if (e) return e;
  uint32_t* s_hat = c->work;
  uint32_t* x = s_hat + poly;
  SmallToRnsArgs sr{sk, s_hat, c->d_mods, k, n};
  if ((e = run<SmallToRnsKernel>(c, bpp, 0, sr))) return e;
  if ((e = ntt_dense(c, s_hat, s_hat, k, k, false))) return e;
  for (size_t c0 = 0; c0 < n_ct; c0 += C) {
    const size_t cc = std::min(C, n_ct - c0);
    const uint32_t* cts = ct + c0 * 2 * poly;
    // x = NTT(c1) picked out of every ciphertext
    NttRows r{cts, x, cc * k, k, 0, 2 * k, k, k, 0};
    if ((e = ntt_rows(c, r, false))) return e;
    PointMulArgs pm{x, s_hat, x, c->d_mods, k, n, (uint32_t)(cc * k), k, 0u};
    if ((e = run<PointMulKernel>(c, cc * k * bpp, 0, pm))) return e;
    if ((e = ntt_dense(c, x, x, cc * k, k, true))) return e;
    AddRowsArgs ar{cts, x, x, c->d_mods, k, n, 2 * k, 0u};
    if ((e = run<AddRowsKernel>(c, cc * k * bpp, 0, ar))) return e;
    if (m_out) {
      DecRoundArgs da;
      da.x = x; da.m_out = m_out + c0 * rn; da.bc = c->dec; da.t = (uint32_t)c->t; da.neg_qinv_t = c->neg_qinv_t; da.n = n;
      da.band = c->band; da.fallback_counter = c->d_counters;
      if ((e = run<DecRoundKernel>(c, cc * bpp, DecRoundKernel::lds_bytes(k), da))) return e;
    } else {
      DecRoundWideArgs da;
      da.x = x; da.m_out = m_out64 + c0 * rn; da.bc = c->dec; da.tab = c->d_dec_wide; da.t = c->t; da.n = n;
      da.band = c->band; da.fallback_counter = c->d_counters;
      if ((e = run<DecRoundWideKernel>(c, cc * bpp, DecRoundWideKernel::lds_bytes(k), da))) return e;
    }
  }
  return HCNN_OK;
}

int hcnn_decrypt(hcnn_ctx* c, const int32_t* sk, const uint32_t* ct, size_t n_ct, uint32_t* m_out) {
  if (!m_out) return HCNN_ERR_NULL;
  return decrypt_impl(c, sk, ct, n_ct, m_out, nullptr);
}

int hcnn_decrypt_wide(hcnn_ctx* c, const int32_t* sk, const uint32_t* ct, size_t n_ct, uint64_t* m_out) {
  if (!m_out) return HCNN_ERR_NULL;
  return decrypt_impl(c, sk, ct, n_ct, nullptr, m_out);
}

int hcnn_noise_bits(hcnn_ctx* c, const int32_t* sk, const uint32_t* ct, size_t n_ct, uint32_t* bits_out) {
  if (!c || !sk || !ct || !bits_out) return HCNN_ERR_NULL;
  if (!aligned16(ct)) return HCNN_ERR_ALIGN;
  if (n_ct == 0) return HCNN_OK;
  const uint32_t k = c->k, n = c->n;
  const size_t rn = n, poly = (size_t)k * rn;
  const size_t bpp = n / kEwThreads;
  const size_t C = std::min<size_t>(n_ct, 64);
  // scratch: s_hat [k][n] | x [C][k][n]
  int e = ensure_work(c, (poly + C * poly) * 4);
  if (e) return e;
  uint32_t* s_hat = c->work;
  uint32_t* x = s_hat + poly;
  if ((e = dev_memset(bits_out, 0, n_ct * sizeof(uint32_t), c->stream))) return e;
  SmallToRnsArgs sr{sk, s_hat, c->d_mods, k, n};
  if ((e = run<SmallToRnsKernel>(c, bpp, 0, sr))) return e;
  if ((e = ntt_dense(c, s_hat, s_hat, k, k, false))) return e;
  for (size_t c0 = 0; c0 < n_ct; c0 += C) {
    const size_t cc = std::min(C, n_ct - c0);
    const uint32_t* cts = ct + c0 * 2 * poly;
    NttRows r{cts, x, cc * k, k, 0, 2 * k, k, k, 0};            // x = NTT(c1) of every ciphertext
    if ((e = ntt_rows(c, r, false))) return e;
    PointMulArgs pm{x, s_hat, x, c->d_mods, k, n, (uint32_t)(cc * k), k, 0u};
    if ((e = run<PointMulKernel>(c, cc * k * bpp, 0, pm))) return e;
    if ((e = ntt_dense(c, x, x, cc * k, k, true))) return e;
    AddRowsArgs ar{cts, x, x, c->d_mods, k, n, 2 * k, 0u};
    if ((e = run<AddRowsKernel>(c, cc * k * bpp, 0, ar))) return e;
    NoiseArgs na;
    na.x = x; na.bits = bits_out + c0; na.bc = c->dec; na.n = n;
    if ((e = run<NoiseKernel>(c, cc * bpp, NoiseKernel::lds_bytes(k), na))) return e;
  }
  return HCNN_OK;
}

// ---------------------------------------------------------------- sampling
namespace {
// T[v] = floor(2^32 * P(|X| <= v)), X = round(N(0, 3.2^2)), v = 0..19: a format constant of the samplers
const uint32_t kGaussT[20] = {533280463u, 1549416568u, 2428136261u, 3117868636u, 3609276189u, 3927060812u, 4113592370u,
                              4212972233u, 4261030606u, 4282124752u, 4290528529u, 4293567340u, 4294564687u, 4294861785u,
                              4294942112u, 4294961823u, 4294966213u, 4294967101u, 4294967264u, 4294967291u};

int sample_impl(hcnn_ctx* c, uint32_t kind, uint64_t seed, uint64_t stream, void* out, size_t count) {
  if (!c) return HCNN_ERR_NULL;
  if (count == 0) return HCNN_OK;
  if (!out) return HCNN_ERR_NULL;
  int e;
  if (!c->d_gauss_t) {
    std::vector<uint32_t> tab(kGaussT, kGaussT + 20);
    if ((e = upload(c, tab, &c->d_gauss_t))) return e;
  }
  SampleArgs a;
  a.out = out; a.mods = c->d_mods; a.gauss_t = c->d_gauss_t; a.seed = seed;
  a.stream = (uint32_t)stream; a.kind = kind; a.k = c->k; a.n = c->n;
  a.total = (uint64_t)count * c->n * (kind == kSampleUniform ? c->k : 1u);
  const uint64_t blocks = (a.total + kEwThreads - 1) / kEwThreads;
  if (blocks > 0x7fffffffull) return HCNN_ERR_ARG;
  return run<SampleKernel>(c, (size_t)blocks, 0, a);
}
}  // namespace

int hcnn_sample_ternary(hcnn_ctx* c, uint64_t seed, uint64_t stream, int32_t* out, size_t n_polys) {
  return sample_impl(c, kSampleTernary, seed, stream, out, n_polys);
}
int hcnn_sample_gaussian(hcnn_ctx* c, uint64_t seed, uint64_t stream, int32_t* out, size_t n_polys) {
  return sample_impl(c, kSampleGaussian, seed, stream, out, n_polys);
}
int hcnn_sample_uniform(hcnn_ctx* c, uint64_t seed, uint64_t stream, uint32_t* out, size_t n_polys) {
  return sample_impl(c, kSampleUniform, seed, stream, out, n_polys);
}

// ---------------------------------------------------------------- diagnostics
int hcnn_get_stat(hcnn_ctx* c, int which, uint64_t* out) {
  if (!c || !out) return HCNN_ERR_NULL;
  if (which == HCNN_STAT_SCRATCH_BYTES) {
    *out = c->work_bytes;
    return HCNN_OK;
  }
  if (which == HCNN_STAT_RELIN_FUSED_WGS || which == HCNN_STAT_TENSOR_FUSED_WGS) {
    *out = which == HCNN_STAT_RELIN_FUSED_WGS ? relin_fused_slots(c) : tensor_fused_slots(c);
    return HCNN_OK;
  }
  if (which != HCNN_STAT_EXACT_FALLBACKS && which != HCNN_STAT_BAD_INPUT) return HCNN_ERR_ARG;
  unsigned long long v[2] = {0, 0};
  int e = copy_d2h(v, c->d_counters, sizeof(v), c->stream);
  if (e) return e;
  *out = v[which];
  return HCNN_OK;
}

int hcnn_measure_ceiling(hcnn_ctx* c, int which, double* value_out) {
  if (!c || !value_out) return HCNN_ERR_NULL;
  if (which < 0 || which >= HCNN_CEIL_COUNT) return HCNN_ERR_ARG;
  int e;
  double ms = 0.0;
  if (which <= HCNN_CEIL_WRITE) {
    const size_t bytes = (size_t)512 << 20;                                       // per buffer
    const size_t grid = bytes / ((size_t)kRateThreads * kStreamUnroll * 16);
    void* src = nullptr;
    void* dst = nullptr;
    if ((e = dev_malloc(&src, bytes))) return e;
    if ((e = dev_malloc(&dst, bytes))) { dev_free(src); return e; }
    StreamArgs a;
    a.src = (const U4*)src; a.dst = (U4*)dst; a.fill = 0x01010101u;
    a.mode = 2;                                                                  // defined contents for both buffers
    e = launch<StreamKernel>(c->stream, grid, 0, a);
    if (!e) { a.dst = (U4*)src; e = launch<StreamKernel>(c->stream, grid, 0, a); a.dst = (U4*)dst; }
    a.mode = which == HCNN_CEIL_COPY ? 0u : (which == HCNN_CEIL_READ ? 1u : 2u);
    a.fill = 0x5a5a5a5au;                              // read mode: the xor of equal words is 0, never this
    if (!e) e = timed_launches<StreamKernel>(c, grid, a, 9, &ms);
    const int es = stream_sync(c->stream);
    dev_free(src);
    dev_free(dst);
    if (e || es) return e ? e : es;
    // (a build that does not time its launches -- the host emulation -- reports 0)
    *value_out = ms > 0.0 ? (which == HCNN_CEIL_COPY ? 2.0 : 1.0) * (double)bytes / (ms * 1e-3) / 1e9 : 0.0;
    return HCNN_OK;
  }
  void* out = nullptr;
  if ((e = dev_malloc(&out, kRateThreads * 4))) return e;
  RateArgs a;
  a.out = (uint32_t*)out; a.seed = 12345u;
  const size_t grid = (size_t)c->compute_units * 8;          // 8 workgroups of 256 per compute unit: full occupancy
  switch (which) {
    case HCNN_CEIL_MUL_LO: e = timed_launches<RateKernel<kRateMulLo>>(c, grid, a, 5, &ms); break;
    case HCNN_CEIL_MUL_HI: e = timed_launches<RateKernel<kRateMulHi>>(c, grid, a, 5, &ms); break;
    case HCNN_CEIL_MAD_U64: e = timed_launches<RateKernel<kRateMadU64>>(c, grid, a, 5, &ms); break;
    case HCNN_CEIL_MAD_I64: e = timed_launches<RateKernel<kRateMadI64>>(c, grid, a, 5, &ms); break;
    default: e = timed_launches<RateKernel<kRateAdd>>(c, grid, a, 5, &ms); break;
  }
  dev_free(out);
  if (e) return e;
  *value_out = ms > 0.0 ? (double)grid * kRateThreads * kRateIters * kRateChains / (ms * 1e-3) / 1e12 : 0.0;
  return HCNN_OK;
}

int hcnn_profile_read(hcnn_ctx* c, int cls, uint64_t* launches, uint64_t* blocks, double* total_ms) {
  if (!c || !launches || !blocks || !total_ms) return HCNN_ERR_NULL;
  if (cls < 0 || cls >= HCNN_PROF_COUNT) return HCNN_ERR_ARG;
  int e = fold_profile(c);
  if (e) return e;
  *launches = c->prof_launches[cls];
  *blocks = c->prof_blocks[cls];
  *total_ms = c->prof_ms[cls];
  return HCNN_OK;
}

int hcnn_reset_stats(hcnn_ctx* c) {
  if (!c) return HCNN_ERR_NULL;
  int pe = fold_profile(c);
  if (pe) return pe;
  for (int i = 0; i < HCNN_PROF_COUNT; ++i) { c->prof_launches[i] = 0; c->prof_blocks[i] = 0; c->prof_ms[i] = 0.0; }
  return dev_memset(c->d_counters, 0, 2 * sizeof(unsigned long long), c->stream);
}

int hcnn_set_option(hcnn_ctx* c, int which, uint64_t value) {
  if (!c) return HCNN_ERR_NULL;
  switch (which) {
    case HCNN_OPT_AMBIGUITY_BAND:
      // never below the error bound 2*ks of the estimate, at most "always ask the exact comparison"
      if (value < 4ull * HCNN_MAX_LIMBS || value > (1ull << 26)) return HCNN_ERR_ARG;
      c->band = (uint32_t)value;
      return HCNN_OK;
    case HCNN_OPT_SQUARE_CHUNK:
      c->square_chunk = value;
      return HCNN_OK;
    case HCNN_OPT_PROFILE:
      c->profile = value != 0;
      return HCNN_OK;
    case HCNN_OPT_RELIN_ORDER:
      if (value > 2) return HCNN_ERR_ARG;
      c->relin_order = value;
      return HCNN_OK;
    case HCNN_OPT_FUSION:
      if (value > 2) return HCNN_ERR_ARG;
      c->fusion = value;
      return HCNN_OK;
      if (value > 2) return HCNN_ERR_ARG;
      return HCNN_OK;
  }
  return HCNN_ERR_ARG;
}

const char* hcnn_strerror(int code) {
  switch (code) {
    case HCNN_OK: return "ok";
    case HCNN_ERR_NULL: return "null pointer";
    case HCNN_ERR_N: return "n must be a power of two in [1024, 32768]";
    case HCNN_ERR_PRIME: return "modulus is not a distinct prime in (2^29, 2^30) congruent to 1 mod 2n";
    case HCNN_ERR_T: return "t must be a prime below 2^47 other than the ciphertext primes (and the plaintext word size must match it)";
    case HCNN_ERR_AUX: return "auxiliary basis missing or too small (need prod p > t*n*q + 1)";
    case HCNN_ERR_ARG: return "invalid count, size or option";
    case HCNN_ERR_NOKEY: return "relinearisation key not set";
    case HCNN_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case HCNN_ERR_NODEVICE: return "no usable device or LDS too small";
    case HCNN_ERR_SCRATCH: return "one ciphertext's intermediate polynomials exceed the 128 MiB static scratch array";
  }
#ifndef HCNN_HOSTEMU
  if (code > 0) return hipGetErrorString((hipError_t)code);
#endif
  return "unknown error";
}

}  // extern "C"
