// sedd_lsh_keys and sedd_cluster: band keys, per-band radix sort, run detection, union-find.
#include <algorithm>

#include "sedd_internal.h"

namespace sedd {

// ---- band keys ---------------------------------------------------------------------------

// key = sum_i sig[i] * Q^i mod p, by Horner from the last row.  One thread per (doc, band).
__global__ void __launch_bounds__(256)
k_lsh_keys(const uint32_t *__restrict__ sig, uint64_t n_docs, int K, int b, int r,
           uint64_t *__restrict__ keys) {
  uint64_t idx = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_docs * (uint64_t)b) return;
  uint64_t d = idx / (uint32_t)b;
  uint32_t j = (uint32_t)(idx - d * (uint32_t)b);
  const uint32_t *src = sig + d * (uint64_t)K + (uint64_t)j * r;
  uint64_t acc = src[r - 1];
  for (int i = r - 2; i >= 0; i--) acc = addmod(mulmod31(acc, Q_BAND), (uint64_t)src[i]);
  keys[idx] = acc;
}

// ---- radix sort of (key, doc) per band ---------------------------------------------------
//
// Records of band j live in [j*n, (j+1)*n) of band-major arrays.  Stable passes over 8-bit
// digits of the low `key_bits` bits of the key.  Per pass: per-block digit histograms, one
// exclusive scan over [band][digit][block] (every band holds exactly n records, so the scan of
// the whole array already yields band-major positions), then a stable scatter.
//
// Grouping does not need a full sort.  Band keys are residues of a polynomial hash, so their low
// bits are uniform: sorting by the low B bits with 2^B >= 16 n leaves, on average, less than 1/16
// foreign record inside a group of records that agree in those bits.  sedd_cluster therefore
// sorts by B = 24 or 32 bits (3 or 4 passes instead of 8) and the linking kernel walks back over
// the records that share the low B bits until it meets one with the same full key.

constexpr int SORT_THREADS = 256;
constexpr int SORT_ITEMS = 16;
constexpr uint32_t SORT_TILE = SORT_THREADS * SORT_ITEMS;
constexpr int RADIX_BITS = 8;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int KEY_BITS = 61;

// keys[d*b + j] -> bk[j*n + d], bd[j*n + d] = d
__global__ void __launch_bounds__(256)
k_to_band_major(const uint64_t *__restrict__ keys, uint32_t n, uint32_t b,
                uint64_t *__restrict__ bk, uint32_t *__restrict__ bd) {
  uint32_t d = blockIdx.x * blockDim.x + threadIdx.x;
  if (d >= n) return;
  const uint64_t *row = keys + (uint64_t)d * b;
  for (uint32_t j = 0; j < b; j++) {
    bk[(uint64_t)j * n + d] = row[j];
    bd[(uint64_t)j * n + d] = d;
  }
}

__global__ void __launch_bounds__(SORT_THREADS)
k_radix_hist(const uint64_t *__restrict__ bk, uint32_t n, uint32_t nblk, int shift,
             uint32_t *__restrict__ hist) {
  __shared__ uint32_t h[RADIX];
  const uint32_t blk = blockIdx.x, band = blockIdx.y;
  h[threadIdx.x] = 0;
  __syncthreads();
  const uint64_t *src = bk + (uint64_t)band * n;
  for (int it = 0; it < SORT_ITEMS; it++) {
    uint32_t e = blk * SORT_TILE + it * SORT_THREADS + threadIdx.x;
    if (e < n) atomicAdd(&h[(uint32_t)(src[e] >> shift) & (RADIX - 1)], 1u);
  }
  __syncthreads();
  hist[((uint64_t)band * RADIX + threadIdx.x) * nblk + blk] = h[threadIdx.x];
}

__global__ void __launch_bounds__(SORT_THREADS)
k_radix_scatter(const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd, uint32_t n,
                uint32_t nblk, int shift, const uint32_t *__restrict__ pos,
                uint64_t *__restrict__ ok, uint32_t *__restrict__ od) {
  __shared__ uint32_t running[RADIX];
  __shared__ uint32_t wcnt[SORT_THREADS / 64][RADIX];
  const uint32_t blk = blockIdx.x, band = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  running[threadIdx.x] = pos[((uint64_t)band * RADIX + threadIdx.x) * nblk + blk];
  const uint64_t *sk = bk + (uint64_t)band * n;
  const uint32_t *sd = bd + (uint64_t)band * n;
  for (int it = 0; it < SORT_ITEMS; it++) {
#pragma unroll
    for (int w = 0; w < SORT_THREADS / 64; w++) wcnt[w][threadIdx.x] = 0;
    __syncthreads();
    const uint32_t e = blk * SORT_TILE + it * SORT_THREADS + threadIdx.x;
    const bool valid = e < n;
    uint64_t key = 0;
    uint32_t doc = 0, digit = 0;
    if (valid) {
      key = sk[e];
      doc = sd[e];
      digit = (uint32_t)(key >> shift) & (RADIX - 1);
    }
    // lanes of this wavefront holding the same digit
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int bit = 0; bit < RADIX_BITS; bit++) {
      const bool set = (digit >> bit) & 1;
      const uint64_t bb = __ballot(valid && set);
      peers &= set ? bb : ~bb;
    }
    const uint32_t below = __popcll(peers & ((uint64_t(1) << lane) - 1));
    if (valid && below == 0) wcnt[wave][digit] = __popcll(peers);
    __syncthreads();
    if (valid) {
      uint32_t o = running[digit] + below;
      for (int w = 0; w < wave; w++) o += wcnt[w][digit];
      ok[o] = key;
      od[o] = doc;
    }
    __syncthreads();
    uint32_t add = 0;
#pragma unroll
    for (int w = 0; w < SORT_THREADS / 64; w++) add += wcnt[w][threadIdx.x];
    running[threadIdx.x] += add;
    __syncthreads();
  }
}

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

__global__ void k_iota_u32(uint32_t *p, uint32_t n) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i;
}

// Records sorted by the low bits selected by `mask`: every record is linked to the nearest
// earlier record of its band with the same full key; the walk stops at the first record that
// differs in the sorted bits.  (With a full sort the walk is one step.)
__global__ void __launch_bounds__(256)
k_link_runs(const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd, uint32_t n,
            uint32_t b, uint64_t mask, uint32_t *parent) {
  uint64_t idx = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (uint64_t)n * b) return;
  const uint32_t i = (uint32_t)(idx % n);
  const uint64_t key = bk[idx];
  for (uint32_t back = 1; back <= i; back++) {
    const uint64_t other = bk[idx - back];
    if ((other ^ key) & mask) break;
    if (other == key) {
      uf_unite(parent, bd[idx - back], bd[idx]);
      break;
    }
  }
}

__global__ void k_write_roots(uint32_t *parent, uint32_t n, int64_t *__restrict__ cluster_id) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) cluster_id[i] = (int64_t)uf_find(parent, i);
}

__global__ void k_copy_sorted(const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd,
                              uint64_t total, uint64_t *__restrict__ ok,
                              uint32_t *__restrict__ od) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) {
    ok[i] = bk[i];
    od[i] = bd[i];
  }
}

struct SortBufs {
  uint64_t *ka, *kb;
  uint32_t *da, *db, *hist, *tmp, *parent;
  uint32_t nblk;
};

static int sort_layout(uint64_t n, uint32_t b, SortBufs *sb) {
  const uint64_t total = n * b;
  const uint32_t nblk = (uint32_t)((n + SORT_TILE - 1) / SORT_TILE);
  const uint64_t nh = (uint64_t)b * RADIX * nblk;
  Carver cv;
  const uint64_t o_ka = cv.take<uint64_t>(total), o_kb = cv.take<uint64_t>(total);
  const uint64_t o_da = cv.take<uint32_t>(total), o_db = cv.take<uint32_t>(total);
  const uint64_t o_h = cv.take<uint32_t>(nh), o_t = cv.take<uint32_t>(scan_tmp_count(nh));
  const uint64_t o_p = cv.take<uint32_t>(n);
  uint8_t *A = nullptr;
  int rc = scratch_ensure(cv.off, &A);
  if (rc) return rc;
  sb->ka = (uint64_t *)(A + o_ka);
  sb->kb = (uint64_t *)(A + o_kb);
  sb->da = (uint32_t *)(A + o_da);
  sb->db = (uint32_t *)(A + o_db);
  sb->hist = (uint32_t *)(A + o_h);
  sb->tmp = (uint32_t *)(A + o_t);
  sb->parent = (uint32_t *)(A + o_p);
  sb->nblk = nblk;
  return SEDD_OK;
}

// number of low key bits sedd_cluster sorts by: a multiple of 16 (an even number of passes, so
// the result lands in the first buffer) with 2^bits >= 16 n where that is possible
static int grouping_bits(uint64_t n_docs) {
  int bits = 16;
  while (bits < 48 && (uint64_t(1) << bits) < 16 * n_docs) bits += 16;
  return bits;
}

// leaves the records, sorted by the low key_bits bits (a multiple of 16, or KEY_BITS for a full
// sort), in sb->ka / sb->da
static int sort_bands(const uint64_t *keys, uint64_t n_docs, uint32_t b, int key_bits, SortBufs *sb,
                      hipStream_t st) {
  const uint32_t n = (uint32_t)n_docs;
  hipLaunchKernelGGL(k_to_band_major, dim3((n + 255) / 256), dim3(256), 0, st, keys, n, b, sb->ka,
                     sb->da);
  SEDD_LAUNCH_CHECK();
  const uint64_t nh = (uint64_t)b * RADIX * sb->nblk;
  uint64_t *src_k = sb->ka, *dst_k = sb->kb;
  uint32_t *src_d = sb->da, *dst_d = sb->db;
  static_assert(((KEY_BITS + RADIX_BITS - 1) / RADIX_BITS) % 2 == 0, "even pass count");
  for (int shift = 0; shift < key_bits; shift += RADIX_BITS) {
    dim3 grid(sb->nblk, b);
    hipLaunchKernelGGL(k_radix_hist, grid, dim3(SORT_THREADS), 0, st, src_k, n, sb->nblk, shift,
                       sb->hist);
    SEDD_LAUNCH_CHECK();
    int rc = scan_exclusive_u32(sb->hist, sb->hist, nh, sb->tmp, st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_radix_scatter, grid, dim3(SORT_THREADS), 0, st, src_k, src_d, n,
                       sb->nblk, shift, sb->hist, dst_k, dst_d);
    SEDD_LAUNCH_CHECK();
    std::swap(src_k, dst_k);
    std::swap(src_d, dst_d);
  }
  return SEDD_OK;
}

}  // namespace sedd

using namespace sedd;

extern "C" {

int sedd_lsh_keys(const uint32_t *sig, uint64_t n_docs, int32_t K, int32_t b, int32_t r,
                  uint64_t *keys, void *stream) {
  if (K < 1 || K > SEDD_MAX_K || b < 1 || r < 1 || (int64_t)b * r > K) return SEDD_EINVAL;
  if (n_docs == 0) return SEDD_OK;
  if (!sig || !keys || n_docs >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  const uint64_t total = n_docs * (uint64_t)b;
  if ((total + 255) / 256 >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  ProfScope prof(SEDD_PROF_LSH_KEYS, (hipStream_t)stream);
  hipLaunchKernelGGL(k_lsh_keys, dim3((uint32_t)((total + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, sig, n_docs, (int)K, (int)b, (int)r, keys);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

static int check_cluster_args(const void *keys, uint64_t n_docs, int32_t b, const void *out) {
  if (b < 1 || b > SEDD_MAX_BANDS) return SEDD_EINVAL;
  if (n_docs == 0) return SEDD_OK;
  if (!keys || !out) return SEDD_EINVAL;
  if (n_docs >= (uint64_t(1) << 31) || n_docs * (uint64_t)b >= (uint64_t(1) << 32))
    return SEDD_EINVAL;
  return SEDD_OK;
}

int sedd_cluster(const uint64_t *keys, uint64_t n_docs, int32_t b, int64_t *cluster_id,
                 void *stream) {
  int rc = check_cluster_args(keys, n_docs, b, cluster_id);
  if (rc || n_docs == 0) return rc;
  hipStream_t st = (hipStream_t)stream;
  SortBufs sb;
  rc = sort_layout(n_docs, (uint32_t)b, &sb);
  if (rc) return rc;
  const int bits = grouping_bits(n_docs);
  {
    ProfScope prof(SEDD_PROF_SORT, st);
    rc = sort_bands(keys, n_docs, (uint32_t)b, bits, &sb, st);
    if (rc) return rc;
  }
  ProfScope prof(SEDD_PROF_UNION, st);
  const uint32_t n = (uint32_t)n_docs;
  hipLaunchKernelGGL(k_iota_u32, dim3((n + 255) / 256), dim3(256), 0, st, sb.parent, n);
  SEDD_LAUNCH_CHECK();
  const uint64_t total = n_docs * (uint64_t)b;
  hipLaunchKernelGGL(k_link_runs, dim3((uint32_t)((total + 255) / 256)), dim3(256), 0, st, sb.ka,
                     sb.da, n, (uint32_t)b, (uint64_t(1) << bits) - 1, sb.parent);
  SEDD_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_write_roots, dim3((n + 255) / 256), dim3(256), 0, st, sb.parent, n,
                     cluster_id);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

int sedd_debug_sort_bands(const uint64_t *keys, uint64_t n_docs, int32_t b,
                          uint64_t *keys_sorted, uint32_t *docs_sorted, void *stream) {
  int rc = check_cluster_args(keys, n_docs, b, keys_sorted);
  if (rc || n_docs == 0) return rc;
  if (!docs_sorted) return SEDD_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  SortBufs sb;
  rc = sort_layout(n_docs, (uint32_t)b, &sb);
  if (rc) return rc;
  rc = sort_bands(keys, n_docs, (uint32_t)b, KEY_BITS, &sb, st);
  if (rc) return rc;
  const uint64_t total = n_docs * (uint64_t)b;
  hipLaunchKernelGGL(k_copy_sorted, dim3((uint32_t)((total + 255) / 256)), dim3(256), 0, st, sb.ka,
                     sb.da, total, keys_sorted, docs_sorted);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

}  // extern "C"
