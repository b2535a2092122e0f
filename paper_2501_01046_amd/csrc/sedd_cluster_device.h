// What the translation units of the clustering calls share: the constants of the grouping sort,
// the union-find of the device side, the buffers of one call, and the host routines and small
// kernels that one unit defines and the other uses.
//   sedd_lsh_cluster.hip       band keys, grouping sort, sedd_cluster and its variants
//   sedd_cluster_verified.hip  the count-match step: sedd_cluster_verified and its variant
#ifndef SEDD_CLUSTER_DEVICE_H
#define SEDD_CLUSTER_DEVICE_H

#include "sedd_internal.h"

namespace sedd {

constexpr int SORT_THREADS = 256;
constexpr int SORT_ITEMS = 16;
constexpr uint32_t SORT_TILE = SORT_THREADS * SORT_ITEMS;
constexpr int RADIX_BITS = 8;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int KEY_BITS = 61;
constexpr uint32_t XCDS = 8;  // accelerator dies of the chip; consecutive workgroups go to them in turn

// ---- union-find --------------------------------------------------------------------------
//
// parent[] only ever points to smaller ids: a root is hooked under a smaller root with a
// compare-and-swap, so the root of a finished tree is the smallest id of its component,
// whatever order the links arrive in.

__device__ __forceinline__ uint32_t ld_parent(const uint32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint32_t uf_find(uint32_t *parent, uint32_t x) {
  uint32_t p = ld_parent(parent + x);
  while (p != x) {
    uint32_t gp = ld_parent(parent + p);
    if (gp != p) atomicMin(parent + x, gp);  // path halving; ancestors have smaller ids
    x = p;
    p = gp;
  }
  return x;
}

__device__ __forceinline__ void uf_unite(uint32_t *parent, uint32_t a, uint32_t b) {
  for (;;) {
    a = uf_find(parent, a);
    b = uf_find(parent, b);
    if (a == b) return;
    const uint32_t hi = max(a, b), lo = min(a, b);
    const uint32_t old = atomicCAS(parent + hi, hi, lo);
    if (old == hi) return;
    a = old;  // hi was hooked meanwhile: continue from its new parent
    b = lo;
  }
}

struct BigGroup {  // a group of more than BIG_GROUP records (verified path)
  uint32_t start, size;
};
constexpr uint32_t BIG_GROUP = 64;

// sketch words per document
__host__ __device__ static inline uint32_t sketch_words(int K) { return (uint32_t)((K + 31) / 32); }

struct SortBufs {
  uint64_t *ka, *kb;
  uint32_t *da, *db, *hist, *tmp, *parent;
  uint32_t *gate;      // raised by the linking / marking kernel when the sorted bits are too few
  uint32_t *high;      // raised by k_to_band_major when some key reaches into the last two digits sorted
  uint32_t *counts;    // verified path: lengths of the follower, outsider and large-group lists
  uint32_t *sketch;    // one-bit signature sketches (verified path): n * sketch_words(K) words
  BigGroup *big;       // capacity big_cap
  uint64_t *tile_pre;  // 2 * (big_cap + 1) prefix sums of tile counts
  uint64_t big_cap;
  uint32_t nblk;
};

// Where the buffers of one clustering call sit inside its workspace (256-byte aligned pieces).
struct SortPlan {
  uint64_t o_ka, o_kb, o_da, o_db, o_h, o_t, o_p, o_gate, o_counts, o_big, o_pre, o_sk;
  uint64_t big_cap, bytes;
  uint32_t nblk;
};

// ---- defined in sedd_lsh_cluster.hip -----------------------------------------------------------

__global__ void k_fill_small_u32(uint32_t *p, uint32_t n, uint32_t v, const uint32_t *gate);
__global__ void k_iota_u32(uint32_t *p, uint32_t n);
__global__ void k_write_roots(uint32_t *parent, uint32_t n, int64_t *__restrict__ cluster_id);

// K_sketch = 0: the buffers of sedd_cluster; K_sketch = K: those of sedd_cluster_verified as well
SortPlan plan_sort(uint64_t n, uint32_t b, int K_sketch);
void bind_sort(const SortPlan &pl, uint8_t *A, SortBufs *sb);
// the buffers carved out of the library's own arena
int sort_layout(uint64_t n, uint32_t b, SortBufs *sb, int K_sketch = 0);
// the caller's workspace, aligned up to 256 bytes, if it is large enough for the plan
int bind_workspace(const SortPlan &pl, void *workspace, uint64_t workspace_bytes, SortBufs *sb);
// number of low key bits the grouping sort orders by: whole digits with 2^bits >= slack * n
int grouping_bits(uint64_t n_docs, uint64_t slack);
// leaves the records, sorted by the low key_bits bits, in sb->ka / sb->da (see the definition)
int sort_bands(const uint64_t *keys, uint64_t n_docs, uint32_t b, int key_bits, SortBufs *sb,
               hipStream_t st, bool skip_empty_digits = false);
// the passes over the key bits the grouping sort left out, executed only when *sb->gate is non-zero
int sort_rest_if_gated(uint64_t n_docs, uint32_t b, int key_bits, SortBufs *sb, hipStream_t st);
// argument checks of the clustering calls
int check_cluster_args(const void *keys, uint64_t n_docs, int32_t b, const void *out);

}  // namespace sedd

#endif
