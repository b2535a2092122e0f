// sedd_lsh_keys and sedd_cluster: band keys, per-band radix sort, run detection, union-find.
#include <algorithm>

#include "sedd_cluster_device.h"

namespace sedd {

// ---- band keys ---------------------------------------------------------------------------

// key = sum_i sig[i] * Q^i mod p, by Horner from the last row.  One thread per (doc, band).
__global__ void __launch_bounds__(256)
k_lsh_keys(const uint32_t *__restrict__ sig, uint64_t n_docs, int K, int b, int r, int vec4,
           uint64_t *__restrict__ keys) {
  uint64_t idx = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_docs * (uint64_t)b) return;
  uint64_t d = idx / (uint32_t)b;
  uint32_t j = (uint32_t)(idx - d * (uint32_t)b);
  const uint32_t *src = sig + d * (uint64_t)K + (uint64_t)j * r;
  uint64_t acc = 0;
  if (vec4) {
    // r and K are multiples of 4 and sig is 16-byte aligned: the band is read as 16-byte vectors
    for (int i = r - 4; i >= 0; i -= 4) {
      const uint4 q = *reinterpret_cast<const uint4 *>(src + i);
      acc = addmod(mulmod31(acc, Q_BAND), (uint64_t)q.w);
      acc = addmod(mulmod31(acc, Q_BAND), (uint64_t)q.z);
      acc = addmod(mulmod31(acc, Q_BAND), (uint64_t)q.y);
      acc = addmod(mulmod31(acc, Q_BAND), (uint64_t)q.x);
    }
  } else {
    acc = src[r - 1];
    for (int i = r - 2; i >= 0; i--) acc = addmod(mulmod31(acc, Q_BAND), (uint64_t)src[i]);
  }
  keys[idx] = acc;
}

// Dense bucket id (Section 3.2): sum of the band's r values modulo the number of buckets.
__global__ void __launch_bounds__(256)
k_lsh_dense_keys(const uint32_t *__restrict__ sig, uint64_t n_docs, int K, int b, int r, int vec4,
                 uint64_t n_buckets, uint64_t *__restrict__ keys) {
  uint64_t idx = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_docs * (uint64_t)b) return;
  uint64_t d = idx / (uint32_t)b;
  uint32_t j = (uint32_t)(idx - d * (uint32_t)b);
  const uint32_t *src = sig + d * (uint64_t)K + (uint64_t)j * r;
  uint64_t sum = 0;  // r <= SEDD_MAX_K values below 2^32: no overflow
  if (vec4) {
    for (int i = 0; i < r; i += 4) {
      const uint4 q = *reinterpret_cast<const uint4 *>(src + i);
      sum += (uint64_t)q.x + q.y + q.z + q.w;
    }
  } else {
    for (int i = 0; i < r; i++) sum += src[i];
  }
  keys[idx] = sum % n_buckets;
}

// ---- radix sort of (key, doc) per band ---------------------------------------------------
//
// Records of band j live in [j*n, (j+1)*n) of band-major arrays.  Stable passes over 8-bit
// digits of the low `key_bits` bits of the key.  Per pass: per-block digit histograms, one
// exclusive scan over [band][digit][block] (every band holds exactly n records, so the scan of
// the whole array already yields band-major positions), then a stable scatter.
//
// Grouping does not need a full sort.  Band keys are residues of a polynomial hash, so their low
// bits are uniform: sorting by the low B bits with 2^B >= n leaves, on average, less than one
// foreign record inside a group of records that agree in those bits.  sedd_cluster therefore
// sorts by B = 16, 24 or 32 bits (2 to 4 passes instead of 8) and the linking kernel walks back
// over the records that share the low B bits until it meets one with the same full key.

// keys[d*b + j] -> bk[j*n + d], bd[j*n + d] = d.  With `high`: *high is raised if some key has a
// bit set at or above high_shift (the word must be zero before the launch).
// A block moves 64 documents, 32 bands at a time, through LDS: rows of the document-major input
// are read whole (32 keys = 256 contiguous bytes per document), columns of the band-major output
// are written 64 documents = 512 contiguous bytes at a time.
constexpr uint32_t TBM_DOCS = 64, TBM_BANDS = 32;
__global__ void __launch_bounds__(256)
k_to_band_major(const uint64_t *__restrict__ keys, uint32_t n, uint32_t b,
                uint64_t *__restrict__ bk, uint32_t *__restrict__ bd, int high_shift,
                uint32_t *high) {
  __shared__ uint64_t tile[TBM_DOCS][TBM_BANDS + 1];  // one key of padding per row: no bank conflicts
  const uint32_t d0 = blockIdx.x * TBM_DOCS, nd = min(TBM_DOCS, n - d0);
  uint64_t seen = 0;
  for (uint32_t j0 = 0; j0 < b; j0 += TBM_BANDS) {
    const uint32_t nb = min(TBM_BANDS, b - j0);
    for (uint32_t e = threadIdx.x; e < nd * nb; e += blockDim.x) {
      const uint32_t doc = e / nb, band = e - doc * nb;
      const uint64_t key = keys[(uint64_t)(d0 + doc) * b + j0 + band];
      seen |= key;
      tile[doc][band] = key;
    }
    __syncthreads();
    for (uint32_t e = threadIdx.x; e < nb * TBM_DOCS; e += blockDim.x) {
      const uint32_t band = e / TBM_DOCS, doc = e % TBM_DOCS;
      if (doc < nd) {
        const uint64_t o = (uint64_t)(j0 + band) * n + d0 + doc;
        bk[o] = tile[doc][band];
        bd[o] = d0 + doc;
      }
    }
    __syncthreads();
  }
  // every writer stores the same value; a block that already sees the flag up leaves it alone, so
  // that keys which all reach that high do not queue a write per block on one address
  if (high && __syncthreads_or((seen >> high_shift) != 0) && threadIdx.x == 0 &&
      __hip_atomic_load(high, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0)
    *high = 1u;
}

__global__ void __launch_bounds__(SORT_THREADS)
k_radix_hist(const uint64_t *__restrict__ bk, uint32_t n, uint32_t nblk, int shift,
             uint32_t *__restrict__ hist, const uint32_t *__restrict__ gate) {
  __shared__ uint32_t h[RADIX];
  if (gate && *gate == 0) return;  // a pass of the full-key fallback that is not needed
  // tiles to XCDs as in k_radix_scatter: the counts of 32 consecutive tiles share a cache line
  const uint32_t per_xcd = gridDim.x / XCDS;
  const uint32_t blk = (blockIdx.x % XCDS) * per_xcd + blockIdx.x / XCDS, band = blockIdx.y;
  if (blk >= nblk) return;
  h[threadIdx.x] = 0;
  __syncthreads();
  const uint64_t *src = bk + (uint64_t)band * n;
  uint64_t key[SORT_ITEMS];  // all loads before the first count
#pragma unroll
  for (int it = 0; it < SORT_ITEMS; it++) {
    const uint32_t e = blk * SORT_TILE + it * SORT_THREADS + threadIdx.x;
    key[it] = e < n ? src[e] : 0;
  }
#pragma unroll
  for (int it = 0; it < SORT_ITEMS; it++) {
    const uint32_t e = blk * SORT_TILE + it * SORT_THREADS + threadIdx.x;
    if (e < n) atomicAdd(&h[(uint32_t)(key[it] >> shift) & (RADIX - 1)], 1u);
  }
  __syncthreads();
  hist[((uint64_t)band * RADIX + threadIdx.x) * nblk + blk] = h[threadIdx.x];
}

// Stable scatter of one tile.  Wavefront w owns the tile's records [w*1024, (w+1)*1024), 16 per
// lane, all loaded before the first is used.  Ranking needs no block barrier: the lanes of a
// wavefront that hold the same digit find each other with ballots, the first of them advances the
// wavefront's own counter of that digit in LDS.  The records are then put in digit order in LDS
// and written out from there, so that consecutive threads write consecutive addresses of a
// digit's run (writing straight from the ranking order leaves cache lines half written for long
// enough that they go to memory more than once).
__global__ void __launch_bounds__(SORT_THREADS)
k_radix_scatter(const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd, uint32_t n,
                uint32_t nblk, int shift, const uint32_t *__restrict__ pos,
                uint64_t *__restrict__ ok, uint32_t *__restrict__ od,
                const uint32_t *__restrict__ gate) {
  constexpr int WAVES = SORT_THREADS / 64;
  if (gate && *gate == 0) return;
  __shared__ uint32_t wc[WAVES][RADIX];  // per wavefront: digit count, later its offset in the tile
  __shared__ uint32_t s_lstart[RADIX];   // first position of the digit in the sorted tile
  __shared__ uint32_t s_gbase[RADIX];    // where the tile's run of the digit starts in the output
  __shared__ uint64_t s_key[SORT_TILE];
  __shared__ uint32_t s_doc[SORT_TILE];
  // Workgroups go to the chip's eight XCDs in turn, each with an L2 of its own.  Tile t and tile
  // t + 1 of a band write adjoining stretches of every digit's run, so the cache lines where
  // they meet are completed only if both tiles pass through the same L2: XCD x takes the tiles
  // [x * per_xcd, (x + 1) * per_xcd) (the grid is padded to 8 * per_xcd).
  const uint32_t per_xcd = gridDim.x / XCDS;
  const uint32_t blk = (blockIdx.x % XCDS) * per_xcd + blockIdx.x / XCDS, band = blockIdx.y;
  if (blk >= nblk) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t *sk = bk + (uint64_t)band * n;
  const uint32_t *sd = bd + (uint64_t)band * n;
#pragma unroll
  for (int w = 0; w < WAVES; w++) wc[w][threadIdx.x] = 0;
  uint64_t key[SORT_ITEMS];
  uint32_t doc[SORT_ITEMS];
  const uint32_t e0 = blk * SORT_TILE + wave * (SORT_TILE / WAVES) + lane;
#pragma unroll
  for (int it = 0; it < SORT_ITEMS; it++) {
    const uint32_t e = e0 + it * 64;
    key[it] = 0;
    doc[it] = 0;
    if (e < n) {
      key[it] = sk[e];
      doc[it] = sd[e];
    }
  }
  __syncthreads();  // counters cleared
  uint32_t rank[SORT_ITEMS];  // rank among the wavefront's records of the same digit
  const uint64_t lt_mask = (uint64_t(1) << lane) - 1;
#pragma unroll
  for (int it = 0; it < SORT_ITEMS; it++) {
    const bool valid = e0 + it * 64 < n;
    const uint32_t digit = (uint32_t)(key[it] >> shift) & (RADIX - 1);
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int bit = 0; bit < RADIX_BITS; bit++) {
      const bool set = (digit >> bit) & 1;
      const uint64_t bb = __ballot(valid && set);
      peers &= set ? bb : ~bb;
    }
    const uint32_t below = __popcll(peers & lt_mask);
    volatile uint32_t *ctr = &wc[wave][digit];
    uint32_t old = 0;
    if (valid) old = *ctr;                                  // every peer reads the count ...
    if (valid && below == 0) *ctr = old + __popcll(peers);  // ... before the first one advances it
    rank[it] = old + below;
  }
  __syncthreads();
  {
    // this thread's digit: its records of the four wavefronts follow each other in the tile
    uint32_t c[WAVES], tot = 0;
#pragma unroll
    for (int w = 0; w < WAVES; w++) {
      c[w] = wc[w][threadIdx.x];
      tot += c[w];
    }
    uint32_t all;
    uint32_t at = block_exclusive_scan<SORT_THREADS>(tot, &all);
    s_lstart[threadIdx.x] = at;
    s_gbase[threadIdx.x] = pos[((uint64_t)band * RADIX + threadIdx.x) * nblk + blk];
#pragma unroll
    for (int w = 0; w < WAVES; w++) {
      wc[w][threadIdx.x] = at;
      at += c[w];
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < SORT_ITEMS; it++) {
    if (e0 + it * 64 < n) {
      const uint32_t digit = (uint32_t)(key[it] >> shift) & (RADIX - 1);
      const uint32_t lp = wc[wave][digit] + rank[it];
      s_key[lp] = key[it];
      s_doc[lp] = doc[it];
    }
  }
  __syncthreads();
  const uint32_t n_valid = min(SORT_TILE, n - blk * SORT_TILE);
#pragma unroll
  for (int it = 0; it < SORT_ITEMS; it++) {
    const uint32_t i = it * SORT_THREADS + threadIdx.x;
    if (i < n_valid) {
      const uint64_t k = s_key[i];
      const uint32_t digit = (uint32_t)(k >> shift) & (RADIX - 1);
      const uint32_t o = s_gbase[digit] + (i - s_lstart[digit]);
      ok[o] = k;
      od[o] = s_doc[i];
    }
  }
}

// ---- small kernels of the union-find (the device functions are in sedd_cluster_device.h) ------

__global__ void k_fill_small_u32(uint32_t *p, uint32_t n, uint32_t v, const uint32_t *gate) {
  if (gate && *gate == 0) return;
  if (threadIdx.x < n) p[threadIdx.x] = v;
}

__global__ void k_iota_u32(uint32_t *p, uint32_t n) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i;
}

// Records sorted by the low bits selected by `mask`: every record is linked to the nearest
// earlier record of its band with the same full key; the walk stops at the first record that
// differs in the sorted bits.  (With a full sort the walk is one step.)
//
// The walk is capped: a record that has not met its key, nor the end of its group, after
// WALK_CAP records raises *gate.  Keys whose sorted bits are uniform (the band keys of
// sedd_lsh_keys are) never do; keys that agree in the sorted bits and differ above them
// would otherwise make every record walk over all earlier ones.  When the gate is up the
// remaining radix passes run (they are always enqueued, and return at once while it is down)
// and a second launch of this kernel (retry = 1, mask = all ones) links the fully sorted records.
// Links made by the first launch stay valid: it only ever unites records with equal keys.
constexpr uint32_t WALK_CAP = 64;
constexpr int LINK_ITEMS = 4;  // records per thread: their keys and left neighbours are loaded together
__global__ void __launch_bounds__(256)
k_link_runs(const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd, uint32_t n,
            uint64_t mask, uint32_t *parent, uint32_t *gate, int retry) {
  if (retry && *gate == 0) return;
  // grid: x over the records of a band (256 * LINK_ITEMS per block), y = band
  const uint64_t band0 = (uint64_t)blockIdx.y * n;
  const uint32_t i0 = blockIdx.x * (256u * LINK_ITEMS) + threadIdx.x;
  uint64_t key[LINK_ITEMS], left[LINK_ITEMS];
#pragma unroll
  for (int it = 0; it < LINK_ITEMS; it++) {
    const uint32_t i = i0 + it * 256u;
    key[it] = i < n ? bk[band0 + i] : 0;
    left[it] = i < n && i > 0 ? bk[band0 + i - 1] : 0;
  }
  bool open = false;
#pragma unroll
  for (int it = 0; it < LINK_ITEMS; it++) {
    const uint32_t i = i0 + it * 256u;
    if (i >= n) continue;
    const uint64_t idx = band0 + i;
    uint64_t other = left[it];
    for (uint32_t back = 1; back <= i; back++) {
      if (back > WALK_CAP) {
        open = true;
        break;
      }
      if (back > 1) other = bk[idx - back];
      if ((other ^ key[it]) & mask) break;
      if (other == key[it]) {
        uf_unite(parent, bd[idx - back], bd[idx]);
        break;
      }
    }
  }
  // with mask = all ones the first step always ends the walk, so a retry never gets here
  // (raised by whoever still sees it down: thousands of atomics on one word would queue up)
  if (__any(open) && (threadIdx.x & 63) == 0 &&
      __hip_atomic_load(gate, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0)
    atomicOr(gate, 1u);
}

__global__ void k_write_roots(uint32_t *parent, uint32_t n, int64_t *__restrict__ cluster_id) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) cluster_id[i] = (int64_t)uf_find(parent, i);
}

__global__ void k_copy_sorted(const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd,
                              uint64_t total, uint64_t *__restrict__ ok,
                              uint32_t *__restrict__ od, const uint32_t *__restrict__ gate) {
  if (gate && *gate == 0) return;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    ok[i] = bk[i];
    od[i] = bd[i];
  }
}
// a grid that fills the chip a few times over: a gated launch that has nothing to do costs little
static uint32_t copy_grid(uint64_t total) {
  return (uint32_t)std::min<uint64_t>((total + 255) / 256, 256 * 64);
}

// K_sketch = 0: the buffers of sedd_cluster; K_sketch = K: those of sedd_cluster_verified as well
SortPlan plan_sort(uint64_t n, uint32_t b, int K_sketch) {
  SortPlan pl;
  const uint64_t total = n * b;
  pl.nblk = (uint32_t)((n + SORT_TILE - 1) / SORT_TILE);
  const uint64_t nh = (uint64_t)b * RADIX * pl.nblk;
  Carver cv;
  pl.o_ka = cv.take<uint64_t>(total);
  pl.o_kb = cv.take<uint64_t>(total);
  pl.o_da = cv.take<uint32_t>(total);
  pl.o_db = cv.take<uint32_t>(total);
  pl.o_h = cv.take<uint32_t>(nh);
  pl.o_t = cv.take<uint32_t>(scan_tmp_count(nh));
  pl.o_p = cv.take<uint32_t>(n);
  pl.o_gate = cv.take<uint32_t>(2);
  pl.o_counts = cv.take<uint32_t>(4);
  pl.big_cap = K_sketch ? total / BIG_GROUP + 1 : 0;
  pl.o_big = cv.take<BigGroup>(pl.big_cap + 1);
  pl.o_pre = cv.take<uint64_t>(2 * (pl.big_cap + 1));
  pl.o_sk = cv.take<uint32_t>(K_sketch ? n * sketch_words(K_sketch) : 1);
  pl.bytes = cv.off;
  return pl;
}

void bind_sort(const SortPlan &pl, uint8_t *A, SortBufs *sb) {
  sb->ka = (uint64_t *)(A + pl.o_ka);
  sb->kb = (uint64_t *)(A + pl.o_kb);
  sb->da = (uint32_t *)(A + pl.o_da);
  sb->db = (uint32_t *)(A + pl.o_db);
  sb->hist = (uint32_t *)(A + pl.o_h);
  sb->tmp = (uint32_t *)(A + pl.o_t);
  sb->parent = (uint32_t *)(A + pl.o_p);
  sb->gate = (uint32_t *)(A + pl.o_gate);
  sb->high = sb->gate + 1;
  sb->counts = (uint32_t *)(A + pl.o_counts);
  sb->big = (BigGroup *)(A + pl.o_big);
  sb->tile_pre = (uint64_t *)(A + pl.o_pre);
  sb->sketch = (uint32_t *)(A + pl.o_sk);
  sb->big_cap = pl.big_cap;
  sb->nblk = pl.nblk;
}

// the buffers carved out of the library's own arena
int sort_layout(uint64_t n, uint32_t b, SortBufs *sb, int K_sketch) {
  const SortPlan pl = plan_sort(n, b, K_sketch);
  uint8_t *A = nullptr;
  int rc = scratch_ensure(pl.bytes, &A);
  if (rc) return rc;
  bind_sort(pl, A, sb);
  return SEDD_OK;
}

// number of low key bits the grouping sort orders by: whole digits with 2^bits >= slack * n where
// that is possible.  A group of equal low bits then holds about 1 / slack records of other keys.
// sedd_cluster takes slack 1 (its linker walks over the few strangers, neighbours in memory: a
// step of the walk costs far less than a radix pass over all records); the verified path takes
// 256 so that a group is, nearly always, exactly one bucket.
int grouping_bits(uint64_t n_docs, uint64_t slack) {
  int bits = 2 * RADIX_BITS;
  while (bits < 56 && (uint64_t(1) << bits) < slack * n_docs) bits += RADIX_BITS;
  return bits;
}

// Stable radix passes over the digits at shift0, shift0 + 8, ... below shift1 of the records in
// sb->ka / sb->da; the result is again in sb->ka / sb->da and sb->kb / sb->db are free.
// Without a gate an odd number of passes renames the two buffer pairs.  With a gate (device word;
// every kernel returns at once while it is zero) the pairs keep their roles whatever the gate
// says, so an odd number of passes ends with a copy back.
static int sort_passes(uint32_t n, uint32_t b, int shift0, int shift1, SortBufs *sb,
                       const uint32_t *gate, hipStream_t st) {
  const uint64_t nh = (uint64_t)b * RADIX * sb->nblk;
  uint64_t *src_k = sb->ka, *dst_k = sb->kb;
  uint32_t *src_d = sb->da, *dst_d = sb->db;
  for (int shift = shift0; shift < shift1; shift += RADIX_BITS) {
    // the grid is padded to a multiple of the number of XCDs (see k_radix_scatter)
    const dim3 grid_xcd((sb->nblk + XCDS - 1) / XCDS * XCDS, b);
    hipLaunchKernelGGL(k_radix_hist, grid_xcd, dim3(SORT_THREADS), 0, st, src_k, n, sb->nblk, shift,
                       sb->hist, gate);
    SEDD_LAUNCH_CHECK();
    int rc = scan_exclusive_u32(sb->hist, sb->hist, nh, sb->tmp, st, gate);
    if (rc) return rc;
    hipLaunchKernelGGL(k_radix_scatter, grid_xcd, dim3(SORT_THREADS), 0, st, src_k, src_d, n,
                       sb->nblk, shift, sb->hist, dst_k, dst_d, gate);
    SEDD_LAUNCH_CHECK();
    std::swap(src_k, dst_k);
    std::swap(src_d, dst_d);
  }
  if (gate) {
    if (src_k != sb->ka) {
      const uint64_t total = (uint64_t)n * b;
      hipLaunchKernelGGL(k_copy_sorted, dim3(copy_grid(total)), dim3(256), 0, st, src_k,
                         src_d, total, sb->ka, sb->da, gate);
      SEDD_LAUNCH_CHECK();
    }
    return SEDD_OK;
  }
  sb->kb = dst_k;
  sb->db = dst_d;
  sb->ka = src_k;
  sb->da = src_d;
  return SEDD_OK;
}

// leaves the records, sorted by the low key_bits bits (whole digits, or KEY_BITS for a full
// sort), in sb->ka / sb->da; sb->kb / sb->db are free afterwards.
// With skip_empty_digits the last two passes run only if some key has a bit set in the digits
// they sort by (they are enqueued either way and return at once otherwise): keys that are small
// numbers, like the bucket ids of sedd_lsh_dense_keys, are sorted after the passes that matter.
int sort_bands(const uint64_t *keys, uint64_t n_docs, uint32_t b, int key_bits, SortBufs *sb,
               hipStream_t st, bool skip_empty_digits) {
  const uint32_t n = (uint32_t)n_docs;
  const bool split = skip_empty_digits && key_bits >= 3 * RADIX_BITS && key_bits < KEY_BITS;
  const int always_bits = split ? key_bits - 2 * RADIX_BITS : key_bits;
  if (split) {
    hipLaunchKernelGGL(k_fill_small_u32, dim3(1), dim3(64), 0, st, sb->high, 1u, 0u,
                       (const uint32_t *)nullptr);
    SEDD_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(k_to_band_major, dim3((n + TBM_DOCS - 1) / TBM_DOCS), dim3(256), 0, st, keys, n, b,
                     sb->ka, sb->da, always_bits, split ? sb->high : (uint32_t *)nullptr);
  SEDD_LAUNCH_CHECK();
  int rc = sort_passes(n, b, 0, always_bits, sb, nullptr, st);
  if (rc || !split) return rc;
  return sort_passes(n, b, always_bits, key_bits, sb, sb->high, st);  // two passes: no copy back
}

// The fallback of the grouping sort: the passes over the key bits it left out, enqueued always,
// executed only when *sb->gate is non-zero.
int sort_rest_if_gated(uint64_t n_docs, uint32_t b, int key_bits, SortBufs *sb, hipStream_t st) {
  return sort_passes((uint32_t)n_docs, b, key_bits, KEY_BITS, sb, sb->gate, st);
}


// sedd_cluster on the buffers of `sb` (the caller has checked the arguments)
static int run_cluster(const uint64_t *keys, uint64_t n_docs, uint32_t b, int64_t *cluster_id,
                       SortBufs &sb, bool timed, hipStream_t st) {
  const int bits = grouping_bits(n_docs, 1);
  const uint32_t n = (uint32_t)n_docs;
  const dim3 link_grid((n + 256 * LINK_ITEMS - 1) / (256 * LINK_ITEMS), b);
  g_last_gate = sb.gate;
  int rc;
  {
    ProfScope prof(timed ? SEDD_PROF_SORT : -1, st);
    rc = sort_bands(keys, n_docs, b, bits, &sb, st);
    if (rc) return rc;
  }
  {
    ProfScope prof(timed ? SEDD_PROF_UNION : -1, st);
    hipLaunchKernelGGL(k_iota_u32, dim3((n + 255) / 256), dim3(256), 0, st, sb.parent, n);
    SEDD_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_fill_small_u32, dim3(1), dim3(64), 0, st, sb.gate, 1u, 0u,
                       (const uint32_t *)nullptr);
    SEDD_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_link_runs, link_grid, dim3(256), 0, st, sb.ka, sb.da, n,
                       (uint64_t(1) << bits) - 1, sb.parent, sb.gate, 0);
    SEDD_LAUNCH_CHECK();
  }
  {
    // only if a walk hit its cap: sort by the rest of the key, link again
    ProfScope prof(timed ? SEDD_PROF_SORT : -1, st);
    rc = sort_rest_if_gated(n_docs, b, bits, &sb, st);
    if (rc) return rc;
  }
  ProfScope prof(timed ? SEDD_PROF_UNION : -1, st);
  hipLaunchKernelGGL(k_link_runs, link_grid, dim3(256), 0, st, sb.ka, sb.da, n,
                     ~uint64_t(0), sb.parent, sb.gate, 1);
  SEDD_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_write_roots, dim3((n + 255) / 256), dim3(256), 0, st, sb.parent, n,
                     cluster_id);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

// ---- scratch of the entry point that allocates nothing ---------------------------------------
//
// One fixed array in device memory, part of the code object: every GPU the library runs on holds
// its own copy from the first use of the library on it until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; the address it yields for the current
// device is what kernels and copies are given.
constexpr uint64_t STATIC_SCRATCH_BYTES = uint64_t(SEDD_STATIC_SCRATCH_MIB) << 20;
static __device__ __align__(256) uint8_t scratch[STATIC_SCRATCH_BYTES];
constexpr int STATIC_MAX_DEVICES = 64;
static uint8_t *g_static_scratch[STATIC_MAX_DEVICES];  // per device, filled on first use

static int static_scratch_for_current_device(uint8_t **out) {
  int dev = -1;
  SEDD_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return SEDD_ELIMIT;
  if (!g_static_scratch[dev]) {
    uint8_t *ptr = nullptr;
    SEDD_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return SEDD_EDEVICE;
    g_static_scratch[dev] = ptr;
  }
  *out = g_static_scratch[dev];
  return SEDD_OK;
}

// ---- argument checks and caller-provided workspaces ------------------------------------------

int check_cluster_args(const void *keys, uint64_t n_docs, int32_t b, const void *out) {
  if (b < 1 || b > SEDD_MAX_BANDS) return SEDD_EINVAL;
  if (n_docs == 0) return SEDD_OK;
  if (!keys || !out) return SEDD_EINVAL;
  if (!aligned_to(keys, 8) || !aligned_to(out, 8)) return SEDD_EINVAL;
  if (n_docs >= (uint64_t(1) << 31) || n_docs * (uint64_t)b >= (uint64_t(1) << 32))
    return SEDD_EINVAL;
  return SEDD_OK;
}

// the caller's workspace, aligned up to 256 bytes, if it is large enough for the plan
int bind_workspace(const SortPlan &pl, void *workspace, uint64_t workspace_bytes, SortBufs *sb) {
  if (!workspace) return SEDD_EINVAL;
  const uintptr_t base = ((uintptr_t)workspace + 255) & ~uintptr_t(255);
  const uint64_t lost = base - (uintptr_t)workspace;
  if (workspace_bytes < lost || workspace_bytes - lost < pl.bytes) return SEDD_ELIMIT;
  bind_sort(pl, (uint8_t *)base, sb);
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
  if (!aligned_to(sig, 4) || !aligned_to(keys, 8)) return SEDD_EINVAL;
  const uint64_t total = n_docs * (uint64_t)b;
  if ((total + 255) / 256 >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  ProfScope prof(SEDD_PROF_LSH_KEYS, (hipStream_t)stream);
  hipLaunchKernelGGL(k_lsh_keys, dim3((uint32_t)((total + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, sig, n_docs, (int)K, (int)b, (int)r,
                     (r % 4 == 0 && K % 4 == 0 && ((uintptr_t)sig & 15) == 0) ? 1 : 0, keys);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

int sedd_lsh_dense_keys(const uint32_t *sig, uint64_t n_docs, int32_t K, int32_t b, int32_t r,
                        uint64_t n_buckets, uint64_t *keys, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (K < 1 || K > SEDD_MAX_K || b < 1 || r < 1 || (int64_t)b * r > K) return SEDD_EINVAL;
  if (n_buckets < 1 || n_buckets >= (uint64_t(1) << 61)) return SEDD_EINVAL;
  if (n_docs == 0) return SEDD_OK;
  if (!sig || !keys || n_docs >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  if (!aligned_to(sig, 4) || !aligned_to(keys, 8)) return SEDD_EINVAL;
  const uint64_t total = n_docs * (uint64_t)b;
  if ((total + 255) / 256 >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  ProfScope prof(SEDD_PROF_LSH_KEYS, st);
  hipLaunchKernelGGL(k_lsh_dense_keys, dim3((uint32_t)((total + 255) / 256)), dim3(256), 0, st, sig,
                     n_docs, (int)K, (int)b, (int)r,
                     (r % 4 == 0 && K % 4 == 0 && ((uintptr_t)sig & 15) == 0) ? 1 : 0, n_buckets, keys);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

int sedd_cluster(const uint64_t *keys, uint64_t n_docs, int32_t b, int64_t *cluster_id,
                 void *stream) {
  int rc = check_cluster_args(keys, n_docs, b, cluster_id);
  if (rc || n_docs == 0) return rc;
  SortBufs sb;
  rc = sort_layout(n_docs, (uint32_t)b, &sb);
  if (rc) return rc;
  return run_cluster(keys, n_docs, (uint32_t)b, cluster_id, sb, true, (hipStream_t)stream);
}

int sedd_cluster_static(const uint64_t *keys, uint64_t n_docs, int32_t b, int64_t *cluster_id,
                        void *stream) {
  int rc = check_cluster_args(keys, n_docs, b, cluster_id);
  if (rc || n_docs == 0) return rc;
  const SortPlan pl = plan_sort(n_docs, (uint32_t)b, 0);
  if (pl.bytes > STATIC_SCRATCH_BYTES) return SEDD_ELIMIT;
  uint8_t *A = nullptr;
  rc = static_scratch_for_current_device(&A);
  if (rc) return rc;
  SortBufs sb;
  bind_sort(pl, A, &sb);
  // same kernels as sedd_cluster; no stage timing here (it would create events)
  return run_cluster(keys, n_docs, (uint32_t)b, cluster_id, sb, false, (hipStream_t)stream);
}

uint64_t sedd_cluster_workspace_bytes(uint64_t n_docs, int32_t b, int32_t K) {
  if (b < 1 || b > SEDD_MAX_BANDS || K < 0 || K > SEDD_MAX_K) return 0;
  if (n_docs >= (uint64_t(1) << 31) || n_docs * (uint64_t)b >= (uint64_t(1) << 32)) return 0;
  if (n_docs == 0) return 256;
  return plan_sort(n_docs, (uint32_t)b, (int)K).bytes + 256;  // room to align the caller's pointer
}

int sedd_cluster_ws(const uint64_t *keys, uint64_t n_docs, int32_t b, int64_t *cluster_id,
                    void *workspace, uint64_t workspace_bytes, void *stream) {
  int rc = check_cluster_args(keys, n_docs, b, cluster_id);
  if (rc || n_docs == 0) return rc;
  SortBufs sb;
  rc = bind_workspace(plan_sort(n_docs, (uint32_t)b, 0), workspace, workspace_bytes, &sb);
  if (rc) return rc;
  return run_cluster(keys, n_docs, (uint32_t)b, cluster_id, sb, true, (hipStream_t)stream);
}

int sedd_debug_last_regroup(uint32_t *out) {
  if (!out) return SEDD_EINVAL;
  *out = 0;
  if (!g_last_gate) return SEDD_OK;
  SEDD_HIP(hipDeviceSynchronize());
  SEDD_HIP(hipMemcpy(out, g_last_gate, sizeof(uint32_t), hipMemcpyDeviceToHost));
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
  hipLaunchKernelGGL(k_copy_sorted, dim3(copy_grid(total)), dim3(256), 0, st, sb.ka,
                     sb.da, total, keys_sorted, docs_sorted, (const uint32_t *)nullptr);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

}  // extern "C"
