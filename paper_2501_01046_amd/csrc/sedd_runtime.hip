// Host runtime of libsedd: error reporting, the grow-only scratch arena, and the
// exclusive-scan primitive the work-list builders use.
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "sedd_internal.h"

namespace sedd {

static thread_local char g_dev_err[512] = "";

int set_device_error(hipError_t e, const char *what) {
  snprintf(g_dev_err, sizeof(g_dev_err), "%s: %s (%s)", hipGetErrorName(e), hipGetErrorString(e),
           what);
  (void)hipGetLastError();  // clear the sticky last-error slot
  return e == hipErrorOutOfMemory ? SEDD_ENOMEM : SEDD_EDEVICE;
}

uint32_t *g_last_gate = nullptr;
static uint8_t *g_arena = nullptr;
static uint64_t g_arena_bytes = 0;
static void *g_pinned = nullptr;
static uint64_t g_pinned_bytes = 0;

static uint64_t g_scratch_cap = 0;  // debug: arena sizes above this fail as if the device were full

int scratch_ensure(uint64_t bytes, uint8_t **base) {
  if (g_scratch_cap && bytes > g_scratch_cap) {
    snprintf(g_dev_err, sizeof(g_dev_err), "scratch of %llu bytes exceeds the debug cap of %llu",
             (unsigned long long)bytes, (unsigned long long)g_scratch_cap);
    return SEDD_ENOMEM;
  }
  if (bytes > g_arena_bytes) {
    // earlier calls may still be using the old arena
    SEDD_HIP(hipDeviceSynchronize());
    if (g_arena) {
      SEDD_HIP(hipFree(g_arena));
      g_arena = nullptr;
      g_arena_bytes = 0;
      g_last_gate = nullptr;
    }
    uint64_t want = (bytes + (uint64_t(1) << 21)) & ~((uint64_t(1) << 21) - 1);
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, want);
    if (e != hipSuccess) {
      set_device_error(e, "hipMalloc(scratch)");
      return SEDD_ENOMEM;
    }
    g_arena = (uint8_t *)p;
    g_arena_bytes = want;
  }
  *base = g_arena;
  return SEDD_OK;
}

int pinned_ensure(uint64_t bytes, void **ptr) {
  if (bytes > g_pinned_bytes) {
    if (g_pinned) {
      SEDD_HIP(hipHostFree(g_pinned));
      g_pinned = nullptr;
      g_pinned_bytes = 0;
    }
    uint64_t want = (bytes + 4095) & ~uint64_t(4095);
    void *p = nullptr;
    hipError_t e = hipHostMalloc(&p, want, hipHostMallocDefault);
    if (e != hipSuccess) {
      set_device_error(e, "hipHostMalloc(offsets)");
      return SEDD_ENOMEM;
    }
    g_pinned = p;
    g_pinned_bytes = want;
  }
  *ptr = g_pinned;
  return SEDD_OK;
}

// ---- persistent device counters ------------------------------------------------------------

static unsigned long long *g_stats = nullptr;
static std::mutex g_small_state_mutex;  // the counters' allocation and the list of timed spans

int stats_ensure(unsigned long long **p) {
  std::lock_guard<std::mutex> lock(g_small_state_mutex);
  if (!g_stats) {
    void *q = nullptr;
    hipError_t e = hipMalloc(&q, SEDD_STAT_N * sizeof(unsigned long long));
    if (e != hipSuccess) {
      set_device_error(e, "hipMalloc(stats)");
      return SEDD_ENOMEM;
    }
    SEDD_HIP(hipMemset(q, 0, SEDD_STAT_N * sizeof(unsigned long long)));
    g_stats = (unsigned long long *)q;
  }
  *p = g_stats;
  return SEDD_OK;
}

// ---- per-stage timing with HIP events (off unless enabled) -------------------------------

struct ProfSpan {
  int label;
  hipEvent_t e0, e1;
};
static bool g_prof_on = false;
static std::vector<ProfSpan> g_spans;
static std::vector<hipEvent_t> g_event_pool;

static hipEvent_t prof_event() {
  if (!g_event_pool.empty()) {
    hipEvent_t e = g_event_pool.back();
    g_event_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

ProfScope::ProfScope(int label, hipStream_t st) : st_(st), idx_(-1) {
  if (!g_prof_on || label < 0) return;  // a negative label: this scope is not timed
  std::lock_guard<std::mutex> lock(g_small_state_mutex);
  ProfSpan sp{label, prof_event(), prof_event()};
  if (!sp.e0 || !sp.e1) return;
  (void)hipEventRecord(sp.e0, st);
  g_spans.push_back(sp);
  idx_ = (int)g_spans.size() - 1;
}
ProfScope::~ProfScope() {
  if (idx_ < 0) return;
  std::lock_guard<std::mutex> lock(g_small_state_mutex);
  if (idx_ < (int)g_spans.size()) (void)hipEventRecord(g_spans[idx_].e1, st_);
}

// ---- exclusive scan ----------------------------------------------------------------------
//
// Blocks of 256 threads x 4 values.  Level 0 reduces each block to one partial; then each block
// rescans its values on top of the sum of the partials before it.  Up to SCAN_DIRECT partials
// every block adds those up itself (a few coalesced loads), which saves the launch that would
// scan them; beyond that the partials are scanned recursively first.

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_PER_THREAD = 4;
constexpr int SCAN_BLOCK = SCAN_THREADS * SCAN_PER_THREAD;
constexpr uint64_t SCAN_DIRECT = 2048;

// `gate` (optional, in every scan kernel): the launch does nothing unless *gate is non-zero.
__global__ void __launch_bounds__(SCAN_THREADS)
k_scan_reduce(const uint32_t *__restrict__ in, uint32_t *__restrict__ partial, uint64_t n,
              const uint32_t *__restrict__ gate) {
  if (gate && *gate == 0) return;
  uint64_t i0 = (uint64_t)blockIdx.x * SCAN_BLOCK + (uint64_t)threadIdx.x * SCAN_PER_THREAD;
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < SCAN_PER_THREAD; j++)
    if (i0 + j < n) s += in[i0 + j];
  uint32_t tot;
  block_exclusive_scan<SCAN_THREADS>(s, &tot);
  if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

// partial_is_sum: partial[b] is the sum of block b (the block adds up partial[0 .. b) itself);
// otherwise partial[b] already is the exclusive prefix of block b.
__global__ void __launch_bounds__(SCAN_THREADS)
k_scan_down(const uint32_t *in, uint32_t *out, uint64_t n, const uint32_t *__restrict__ partial,
            int partial_is_sum, const uint32_t *__restrict__ gate) {
  if (gate && *gate == 0) return;
  uint64_t i0 = (uint64_t)blockIdx.x * SCAN_BLOCK + (uint64_t)threadIdx.x * SCAN_PER_THREAD;
  uint32_t v[SCAN_PER_THREAD];
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < SCAN_PER_THREAD; j++) {
    v[j] = (i0 + j < n) ? in[i0 + j] : 0u;
    s += v[j];
  }
  uint32_t before = 0;
  if (partial) {
    if (partial_is_sum) {
      uint32_t mine = 0;
      for (uint32_t b = threadIdx.x; b < blockIdx.x; b += SCAN_THREADS) mine += partial[b];
      uint32_t tot_before;
      block_exclusive_scan<SCAN_THREADS>(mine, &tot_before);
      before = tot_before;
    } else {
      before = partial[blockIdx.x];
    }
  }
  uint32_t tot;
  uint32_t ex = block_exclusive_scan<SCAN_THREADS>(s, &tot) + before;
#pragma unroll
  for (int j = 0; j < SCAN_PER_THREAD; j++) {
    if (i0 + j < n) out[i0 + j] = ex;
    ex += v[j];
  }
}

uint64_t scan_tmp_count(uint64_t n) {
  uint64_t total = 0;
  while (n > SCAN_BLOCK) {
    n = (n + SCAN_BLOCK - 1) / SCAN_BLOCK;
    total += (n + 63) & ~uint64_t(63);
  }
  return total + 64;
}

int scan_exclusive_u32(const uint32_t *in, uint32_t *out, uint64_t n, uint32_t *tmp,
                       hipStream_t s, const uint32_t *gate) {
  if (n == 0) return SEDD_OK;
  uint64_t nb = (n + SCAN_BLOCK - 1) / SCAN_BLOCK;
  if (nb == 1) {
    hipLaunchKernelGGL(k_scan_down, dim3(1), dim3(SCAN_THREADS), 0, s, in, out, n,
                       (const uint32_t *)nullptr, 0, gate);
    SEDD_LAUNCH_CHECK();
    return SEDD_OK;
  }
  hipLaunchKernelGGL(k_scan_reduce, dim3((uint32_t)nb), dim3(SCAN_THREADS), 0, s, in, tmp, n, gate);
  SEDD_LAUNCH_CHECK();
  const int direct = nb <= SCAN_DIRECT ? 1 : 0;
  if (!direct) {
    uint32_t *next_tmp = tmp + ((nb + 63) & ~uint64_t(63));
    int rc = scan_exclusive_u32(tmp, tmp, nb, next_tmp, s, gate);
    if (rc) return rc;
  }
  hipLaunchKernelGGL(k_scan_down, dim3((uint32_t)nb), dim3(SCAN_THREADS), 0, s, in, out, n,
                     (const uint32_t *)tmp, direct, gate);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

}  // namespace sedd

using namespace sedd;

extern "C" {

const char *sedd_strerror(int code) {
  switch (code) {
    case SEDD_OK: return "success";
    case SEDD_EINVAL: return "invalid argument";
    case SEDD_ENOMEM: return "scratch allocation failed";
    case SEDD_EDEVICE: return "HIP call failed (see sedd_last_device_error)";
    case SEDD_ELIMIT: return "input exceeds a fixed limit of this entry point";
    default: return "unknown error code";
  }
}

const char *sedd_last_device_error(void) { return g_dev_err; }

int32_t sedd_min_match(uint64_t theta_num, uint64_t theta_den, int32_t K) {
  if (theta_den == 0 || K < 0) return SEDD_EINVAL;
  const unsigned __int128 t = (unsigned __int128)theta_num * (uint64_t)K;
  const unsigned __int128 m = (t + theta_den - 1) / theta_den;  // ceiling of theta * K
  if (m > (unsigned __int128)INT32_MAX) return SEDD_EINVAL;
  return (int32_t)m;
}

uint64_t sedd_dense_bucket_count(uint64_t n_docs, uint32_t k) {
  const unsigned __int128 v = (unsigned __int128)n_docs * k * k;  // below 2^128
  // largest s with s * s <= v, bit by bit (s < 2^64)
  uint64_t s = 0;
  for (int bit = 63; bit >= 0; bit--) {
    const uint64_t c = s | (uint64_t(1) << bit);
    if ((unsigned __int128)c * c <= v) s = c;
  }
  return s ? s : 1;
}

int sedd_version(void) { return 100; }

int sedd_release_scratch(void) {
  SEDD_HIP(hipDeviceSynchronize());
  if (g_arena) {
    SEDD_HIP(hipFree(g_arena));
    g_arena = nullptr;
    g_arena_bytes = 0;
    g_last_gate = nullptr;
  }
  if (g_pinned) {
    SEDD_HIP(hipHostFree(g_pinned));
    g_pinned = nullptr;
    g_pinned_bytes = 0;
  }
  int rc = release_host_feed();
  if (rc) return rc;
  return release_stream_state();
}

uint64_t sedd_scratch_bytes(void) { return g_arena_bytes; }

int sedd_profile_enable(int on) {
  g_prof_on = on != 0;
  return SEDD_OK;
}

int sedd_profile_read(double *ms, uint64_t *spans) {
  if (!ms || !spans) return SEDD_EINVAL;
  for (int i = 0; i < SEDD_PROF_N; i++) {
    ms[i] = 0.0;
    spans[i] = 0;
  }
  std::lock_guard<std::mutex> lock(g_small_state_mutex);
  for (ProfSpan &sp : g_spans) {
    SEDD_HIP(hipEventSynchronize(sp.e1));
    float t = 0.f;
    SEDD_HIP(hipEventElapsedTime(&t, sp.e0, sp.e1));
    if (sp.label >= 0 && sp.label < SEDD_PROF_N) {
      ms[sp.label] += t;
      spans[sp.label] += 1;
    }
    g_event_pool.push_back(sp.e0);
    g_event_pool.push_back(sp.e1);
  }
  g_spans.clear();
  return SEDD_OK;
}

const char *sedd_profile_label(int label) {
  switch (label) {
    case SEDD_PROF_MINHASH: return "minhash";
    case SEDD_PROF_TOKENIZE: return "tokenize";
    case SEDD_PROF_WORKLIST: return "worklist";
    case SEDD_PROF_LSH_KEYS: return "lsh_keys";
    case SEDD_PROF_SORT: return "sort";
    case SEDD_PROF_UNION: return "union_find";
    case SEDD_PROF_VERIFY: return "verify";
    default: return "";
  }
}

int sedd_debug_stats(uint64_t *out) {
  if (!out) return SEDD_EINVAL;
  unsigned long long *p = nullptr;
  int rc = stats_ensure(&p);
  if (rc) return rc;
  SEDD_HIP(hipDeviceSynchronize());
  SEDD_HIP(hipMemcpy(out, p, SEDD_STAT_N * sizeof(uint64_t), hipMemcpyDeviceToHost));
  return SEDD_OK;
}

int sedd_debug_set_scratch_cap(uint64_t bytes) {
  g_scratch_cap = bytes;
  return SEDD_OK;
}

int sedd_debug_scan_u32(const uint32_t *in, uint32_t *out, uint64_t n, void *stream) {
  if (n == 0) return SEDD_OK;
  if (!in || !out || n >= (uint64_t(1) << 32)) return SEDD_EINVAL;
  uint8_t *base;
  int rc = scratch_ensure(scan_tmp_count(n) * 4, &base);
  if (rc) return rc;
  return scan_exclusive_u32(in, out, n, (uint32_t *)base, (hipStream_t)stream);
}

}  // extern "C"
