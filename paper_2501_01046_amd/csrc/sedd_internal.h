// Internal declarations shared by the HIP translation units of libsedd.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sedd.h"
#include "sedd_debug.h"

namespace sedd {

// ---- constants of the method (Section 3.2 Eq. 1; readings fixed in include/sedd.h) ----
constexpr uint64_t P61 = 2305843009213693951ull;     // 2^61 - 1
constexpr uint64_t Q_BAND = 1687994237021934823ull;  // base of the band-key polynomial
constexpr uint64_t G_A = 1425089352415399810ull;
constexpr uint64_t G_B = 955111447119501601ull;

// ---- arithmetic mod 2^61-1 (device) ----------------------------------------------------

// canonical residue of r < 2^63
__device__ __forceinline__ uint64_t fold61(uint64_t r) {
  r = (r & P61) + (r >> 61);
  return r >= P61 ? r - P61 : r;
}
__device__ __forceinline__ uint64_t addmod(uint64_t a, uint64_t b) {
  uint64_t r = a + b;  // < 2^62
  return r >= P61 ? r - P61 : r;
}
// a, b < 2^61.  2^64 = 8 (mod p), so hi*2^64 + lo = (lo & p) + (lo >> 61) + 8*hi.
__device__ __forceinline__ uint64_t mulmod(uint64_t a, uint64_t b) {
  uint64_t lo = a * b;
  uint64_t hi = __umul64hi(a, b);  // < 2^58
  return fold61((lo & P61) + (lo >> 61) + (hi << 3));
}
// Same product through 31-bit limbs and the 32x32+64 multiply-add (fewer instructions than the
// 64x64 high/low pair): a = a1 2^31 + a0, x = x1 2^31 + x0, 2^61 = 1, 2^62 = 2 (mod p):
//   a x = a0 x0 + 2 a1 x1 + 2^31 M,  M = a0 x1 + a1 x0,  2^31 M = (M >> 30) + 2^31 (M mod 2^30).
// N = 4M keeps M >> 30 in its high word and 4 (M mod 2^30) in its low word.
__device__ __forceinline__ uint64_t mulmod31(uint64_t a, uint64_t x) {
  const uint32_t a0 = (uint32_t)a & 0x7FFFFFFFu, a12 = (uint32_t)(a >> 31) << 1;
  const uint32_t x0 = (uint32_t)x & 0x7FFFFFFFu, x1 = (uint32_t)(x >> 31);
  const uint64_t N = (uint64_t)a0 * (x1 << 2) + (uint64_t)a12 * (x0 << 1);
  const uint64_t U = (uint64_t)a12 * x1 + (uint64_t)a0 * x0;           // < 2^61 + 2^62
  return fold61(((uint64_t)(uint32_t)N << 29) + U + (N >> 32));         // < 2^63 + 2^33
}
// x * 257 for x < p: 257 = 2^8 + 1 and a shift by 8 is a rotation of the 61-bit residue
__device__ __forceinline__ uint64_t mul257(uint64_t x) {
  uint64_t rot = ((x << 8) & P61) | (x >> 53);
  return fold61(rot + x);
}
__device__ __forceinline__ uint64_t powmod(uint64_t g, uint64_t e) {
  uint64_t r = 1;
  while (e) {
    if (e & 1) r = mulmod(r, g);
    g = mulmod(g, g);
    e >>= 1;
  }
  return r;
}
// true if p is a multiple of `align` bytes (the kernels use naturally aligned accesses and atomics)
inline bool aligned_to(const void *p, uintptr_t align) { return ((uintptr_t)p & (align - 1)) == 0; }

__device__ __forceinline__ bool is_ws(uint32_t c) { return c == 0x20u || (c - 0x09u) <= 4u; }

// ---- block-level scan (device) ------------------------------------------------------------

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (no LDS traffic):
// shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0 / rows 0-1 is
// broadcast into the following rows.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  // update_dpp(old, src, dpp_ctrl, row_mask, bank_mask, bound_ctrl): lanes without a source keep `old`
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);  // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15 -> rows 1, 3
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);  // row_bcast:31 -> rows 2, 3
  return v;
}

// Exclusive scan across the block of one value per thread; returns the exclusive prefix and
// the block total in *total.  Must be called by all THREADS threads of the block.
template <int THREADS>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *total) {
  __shared__ uint32_t wave_sum[THREADS / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t inc = wave_inclusive_scan(v);
  __syncthreads();  // protects wave_sum across repeated calls
  if (lane == 63) wave_sum[wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; w++) {
    uint32_t s = wave_sum[w];
    if (w < wave) base += s;
    tot += s;
  }
  *total = tot;
  return base + inc - v;
}

// ---- host runtime ------------------------------------------------------------------------

int set_device_error(hipError_t e, const char *what);
#define SEDD_HIP(expr)                                            \
  do {                                                            \
    hipError_t _e = (expr);                                       \
    if (_e != hipSuccess) return sedd::set_device_error(_e, #expr); \
  } while (0)
#define SEDD_LAUNCH_CHECK() SEDD_HIP(hipGetLastError())

// Grow-only device arena.  ensure() may synchronise the device and reallocate.
int scratch_ensure(uint64_t bytes, uint8_t **base);
// Grow-only pinned host buffer.
int pinned_ensure(uint64_t bytes, void **ptr);
// Frees the device staging buffers of sedd_minhash_host_chunked (the device must be idle).
int release_host_feed();
// Frees the coefficient sets and probe records of the streaming min-hash path (device idle).
int release_stream_state();

// The fallback flag of the most recent clustering call (inside its workspace; debug read-out).
// Forgotten when the arena it may point into is freed.
extern uint32_t *g_last_gate;

// Device counters that persist for the life of the process (SEDD_STAT_* indices).
int stats_ensure(unsigned long long **p);

// Times the work enqueued during its lifetime under `label` when profiling is enabled.
struct ProfScope {
  ProfScope(int label, hipStream_t st);
  ~ProfScope();
  ProfScope(const ProfScope &) = delete;
  ProfScope &operator=(const ProfScope &) = delete;

 private:
  hipStream_t st_;
  int idx_;
};

struct Carver {  // carves 256-byte aligned sub-buffers out of the arena
  uint64_t off = 0;
  template <typename T> uint64_t take(uint64_t count) {
    uint64_t o = off;
    off += (count * sizeof(T) + 255) & ~uint64_t(255);
    return o;
  }
};

// Exclusive prefix sum of n uint32 (out may alias in).  tmp must hold scan_tmp_count(n) uint32.
// With a gate (device pointer) the kernels are still launched but do nothing unless *gate != 0.
uint64_t scan_tmp_count(uint64_t n);
int scan_exclusive_u32(const uint32_t *in, uint32_t *out, uint64_t n, uint32_t *tmp,
                       hipStream_t s, const uint32_t *gate = nullptr);

}  // namespace sedd
