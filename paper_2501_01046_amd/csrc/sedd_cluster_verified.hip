// sedd_cluster_verified: the count-match step of Section 3.3 on the groups the grouping sort
// leaves (first-document / outsider passes for small buckets, LDS-resident all-pairs comparison
// bounded by one-bit sketches for large ones).
#include <algorithm>
#include <cmath>

#include "sedd_cluster_device.h"

namespace sedd {

// ---- verified clusters (Section 3.3) --------------------------------------------------------
//
// A bucket is a run of records with the same key inside one band.  The grouping sort orders the
// records by their low key bits only, so a group (run of equal low bits) is a bucket or, rarely,
// a few interleaved buckets; every pair test below therefore also compares the full keys.
//
// The union graph of "pair in the same bucket with at least min_match equal signature entries"
// is built without enumerating all pairs of a large bucket whose members are alike:
//   1. every record that is not the first of its bucket is compared with the bucket's first
//      record (its head); a verified pair is united, a record that fails becomes an outsider;
//   2. every outsider is compared with all other records of its bucket.
// A pair of two non-outsiders is never compared: both are already in the head's component, so
// the edge could not change any component.  Likewise any pair found in one component is skipped.
// The components, and so the cluster ids, are exactly those of the exhaustive comparison.

constexpr int TEAM = 16;  // lanes that compare one pair of signatures

// Records that are not the first of their bucket go to list1 (one atomic per block of SORT_TILE
// records), except those that can see, BIG_GROUP records before or after them, a record of their
// own group: their group is large and is compared tile by tile instead.  The first record of a
// large group appends the group to `big`.
__global__ void __launch_bounds__(SORT_THREADS)
k_v_mark(const uint64_t *__restrict__ bk, uint32_t n, uint64_t mask,
         uint32_t *__restrict__ list1, uint32_t *__restrict__ counts,
         BigGroup *__restrict__ big, uint32_t *gate, uint32_t mixed_limit, int retry) {
  __shared__ uint32_t s_base[2];
  if (retry && *gate == 0) return;
  const uint32_t blk = blockIdx.x, band = blockIdx.y;
  const uint64_t *src = bk + (uint64_t)band * n;
  uint32_t flags = 0, heads = 0;  // bit it: item it goes to list1 / is the head of a large group
  uint32_t mixed = 0;  // records that see another key BIG_GROUP records on inside their own group
  constexpr int BATCH = 4;  // records whose three loads are issued together
  static_assert(SORT_ITEMS % BATCH == 0, "whole batches");
#pragma unroll
  for (int it0 = 0; it0 < SORT_ITEMS; it0 += BATCH) {
    uint64_t key[BATCH], before[BATCH], after[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; j++) {
      const uint32_t e = blk * SORT_TILE + (it0 + j) * SORT_THREADS + threadIdx.x;
      key[j] = e < n ? src[e] : 0;
      before[j] = e < n && e > 0 ? src[e - 1] : 0;
      after[j] = e + BIG_GROUP < n ? src[e + BIG_GROUP] : 0;
    }
#pragma unroll
    for (int j = 0; j < BATCH; j++) {
      const int it = it0 + j;
      const uint32_t e = blk * SORT_TILE + it * SORT_THREADS + threadIdx.x;
      if (e >= n) continue;
      const uint64_t low = key[j] & mask;
      const bool follower = e > 0 && (before[j] & mask) == low;
      const bool far_after = e + BIG_GROUP < n && (after[j] & mask) == low;
      mixed += far_after && after[j] != key[j];
      if (follower) {
        const bool far_before = e >= BIG_GROUP && (src[e - BIG_GROUP] & mask) == low;
        if (!far_before && !far_after) {
          // small group: listed only if an earlier record of the group has this very key (the
          // group starts fewer than BIG_GROUP records back, and is nearly always one bucket)
          bool real = before[j] == key[j];
          for (uint32_t q = e - 1; q > 0 && !real;) {
            const uint64_t other = src[--q];
            if ((other & mask) != low) break;
            real = other == key[j];
          }
          if (real) flags |= 1u << it;
        }
      } else if (far_after) {
        heads |= 1u << it;
      }
    }
  }
  // A large group with a stranger or two costs a few comparisons more (every pair test compares
  // the keys); large groups that are mixtures throughout mean the sorted bits are too few.  The
  // gate goes up when more than mixed_limit records say so (counts[3]), raised by the wavefront
  // whose addition crosses the limit.  With mask = all ones a group holds one key: a retry adds nothing.
  if (__any(mixed != 0)) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mixed += __shfl_xor(mixed, o, 64);
    if ((threadIdx.x & 63) == 0 &&
        __hip_atomic_load(gate, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
      const uint32_t before = atomicAdd(counts + 3, mixed);
      if (before <= mixed_limit && before + mixed > mixed_limit) atomicOr(gate, 1u);
    }
  }
  // both counts through one scan (at most SORT_TILE = 2^12 of either per block) and one atomic
  // each per block
  static_assert(SORT_TILE <= (1u << 15), "two counts share one 32-bit scan");
  uint32_t tot;
  const uint32_t pre = block_exclusive_scan<SORT_THREADS>(__popc(flags) | (__popc(heads) << 16), &tot);
  if (threadIdx.x == 0) {
    s_base[0] = (tot & 0xFFFFu) ? atomicAdd(counts, tot & 0xFFFFu) : 0u;
    s_base[1] = (tot >> 16) ? atomicAdd(counts + 2, tot >> 16) : 0u;
  }
  __syncthreads();
  uint32_t o = s_base[0] + (pre & 0xFFFFu), oh = s_base[1] + (pre >> 16);
#pragma unroll
  for (int it = 0; it < SORT_ITEMS; it++) {
    const uint32_t e = blk * SORT_TILE + it * SORT_THREADS + threadIdx.x;
    if (flags & (1u << it)) list1[o++] = band * n + e;
    if (heads & (1u << it)) {
      // head of a large group: its end by binary search over the rest of the band
      const uint64_t low = src[e] & mask;
      uint32_t lo = e + BIG_GROUP + 1, hi = n;
      while (lo < hi) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if ((src[mid] & mask) > low) hi = mid;
        else lo = mid + 1;
      }
      BigGroup g;
      g.start = band * n + e;
      g.size = lo - e;
      big[oh++] = g;
    }
  }
}

// number of equal entries of two signatures, computed by the TEAM lanes of one team; every
// lane of the team returns the total
__device__ __forceinline__ uint32_t team_matches(const uint32_t *__restrict__ su,
                                                 const uint32_t *__restrict__ sv, int K,
                                                 int tl) {
  uint32_t c = 0;
  if ((K & 3) == 0 && (((uintptr_t)su | (uintptr_t)sv) & 15) == 0) {
    for (int k = tl * 4; k < K; k += TEAM * 4) {
      const uint4 a = *reinterpret_cast<const uint4 *>(su + k);
      const uint4 d = *reinterpret_cast<const uint4 *>(sv + k);
      c += (a.x == d.x) + (a.y == d.y) + (a.z == d.z) + (a.w == d.w);
    }
  } else {
    for (int k = tl; k < K; k += TEAM) c += su[k] == sv[k];
  }
#pragma unroll
  for (int o = TEAM / 2; o >= 1; o >>= 1) c += __shfl_xor(c, o, TEAM);
  return c;
}

// first index in [lo, hi] whose masked key is not below `want` (the masked keys are sorted and
// bk[hi] has the masked key `want`); most groups are a few records long, so walk first
__device__ __forceinline__ uint32_t group_lower_bound(const uint64_t *__restrict__ bk, uint64_t mask,
                                                      uint32_t lo, uint32_t hi, uint64_t want) {
  for (int step = 0; step < 4; step++) {
    if (hi == lo || (bk[hi - 1] & mask) != want) return hi;
    hi--;
  }
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if ((bk[mid] & mask) >= want) hi = mid;
    else lo = mid + 1;
  }
  return lo;
}
// first index in [lo, hi) whose masked key is above `want`, or hi
__device__ __forceinline__ uint32_t group_upper_bound(const uint64_t *__restrict__ bk, uint64_t mask,
                                                      uint32_t lo, uint32_t hi, uint64_t want) {
  for (int step = 0; step < 4; step++) {
    if (lo == hi || (bk[lo] & mask) != want) return lo;
    lo++;
  }
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if ((bk[mid] & mask) > want) hi = mid;
    else lo = mid + 1;
  }
  return lo;
}

// the TEAM lanes decide one candidate pair (documents u, v of one bucket); lane 0 of the team
// unites them if they verify.  Returns whether u and v are in one component afterwards.
__device__ __forceinline__ bool team_verify_pair(const uint32_t *__restrict__ sig, int K,
                                                 int min_match, uint32_t *parent, uint32_t u,
                                                 uint32_t v, int tl) {
  uint32_t same = 0;
  if (tl == 0) same = uf_find(parent, u) == uf_find(parent, v) ? 1u : 0u;
  same = __shfl(same, 0, TEAM);
  if (same) return true;
  const uint32_t m = team_matches(sig + (uint64_t)u * K, sig + (uint64_t)v * K, K, tl);
  if ((int)m < min_match) return false;
  if (tl == 0) uf_unite(parent, u, v);
  return true;
}

// step 1: one team per follower record, against the head of its bucket.  The outsiders of a block
// collect in LDS and go to list2 every HP_FLUSH rounds, with one atomic on the list's length per
// block and flush (one per wavefront and round, all on that one word, took most of the kernel's time).
constexpr uint32_t HP_THREADS = 256, HP_FLUSH = 32;
__global__ void __launch_bounds__(HP_THREADS)
k_v_head_pairs(const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd, uint32_t n,
               uint64_t mask_lo, const uint32_t *__restrict__ gate,
               const uint32_t *__restrict__ sig, int K, int min_match,
               uint32_t *parent, const uint32_t *__restrict__ list1, uint32_t *counts,
               uint32_t *__restrict__ list2) {
  __shared__ uint32_t s_out[HP_FLUSH * (HP_THREADS / TEAM)];  // at most one outsider per team and round
  __shared__ uint32_t s_n, s_base;
  const uint64_t mask = *gate ? ~uint64_t(0) : mask_lo;  // gate up: the records are fully sorted
  const uint32_t n1 = counts[0];
  const int tl = threadIdx.x & (TEAM - 1);
  const uint32_t teams = gridDim.x * (HP_THREADS / TEAM);
  // every thread of a block runs the same number of rounds (the flush is a block operation)
  const uint32_t rounds = (n1 + teams - 1) / teams;
  if (threadIdx.x == 0) s_n = 0;
  __syncthreads();
  uint32_t e = blockIdx.x * (HP_THREADS / TEAM) + threadIdx.x / TEAM;
  for (uint32_t it = 0; it < rounds; it++, e += teams) {
    if (e < n1) {
      const uint32_t i = list1[e];
      const uint64_t key = bk[i], low = key & mask;
      const uint32_t band0 = (i / n) * n;
      const uint64_t band_end = (uint64_t)band0 + n;
      // One round of loads settles nearly every follower: lane t of the team takes the record
      // t + 1 places before i (key and document), and the record BIG_GROUP places after that one.
      const bool in_band = i >= band0 + 1u + (uint32_t)tl;
      const uint32_t back = i - 1u - (uint32_t)tl;
      const uint64_t far = (uint64_t)back + BIG_GROUP;
      const uint64_t k_back = in_band ? bk[back] : ~key;  // ~key: another group, another key
      const uint64_t k_far = in_band && far < band_end ? bk[far] : ~key;
      const uint32_t d_back = in_band ? bd[back] : 0u;
      const uint32_t d_i = bd[i];
      const uint32_t team_shift = threadIdx.x & 48u;  // the team's lanes inside the wavefront's ballot
      const uint32_t same = (uint32_t)(__ballot((k_back & mask) == low) >> team_shift) & 0xFFFFu;
      const uint32_t equal = (uint32_t)(__ballot(k_back == key) >> team_shift) & 0xFFFFu;
      const uint32_t c = (uint32_t)__ffs((int)~same) - 1u;  // records of the group right before i (16: or more)
      bool joined;
      if (c < (uint32_t)TEAM) {  // (c >= 1: k_v_mark lists records that follow one of their group)
        // the group starts at i - c; more than BIG_GROUP records: compared by k_v_groups / k_v_tiles
        const uint64_t k_over = __shfl(k_far, (int)c - 1, TEAM);  // the record at group start + BIG_GROUP
        joined = (k_over & mask) == low;
        if (!joined) {
          const uint32_t eq = equal & ((1u << c) - 1u);  // the bucket's records before i
          if (eq) {
            const int first = 31 - __clz((int)eq);  // the bucket's first record is the farthest back
            joined = team_verify_pair(sig, K, min_match, parent, __shfl(d_back, first, TEAM), d_i, tl);
          }
        }
      } else {
        const uint32_t gs = group_lower_bound(bk, mask, band0, i, low);
        joined = gs + BIG_GROUP < band_end && ((bk[gs + BIG_GROUP] ^ key) & mask) == 0;
        if (!joined) {
          uint32_t h = gs;  // the bucket's first record: k_v_mark saw one before i
          while (bk[h] != key) h++;
          joined = team_verify_pair(sig, K, min_match, parent, bd[h], d_i, tl);
        }
      }
      if (!joined && tl == 0) s_out[atomicAdd(&s_n, 1u)] = i;
    }
    if ((it + 1) % HP_FLUSH == 0 || it + 1 == rounds) {
      __syncthreads();
      const uint32_t held = s_n;
      if (held) {  // uniform over the block
        if (threadIdx.x == 0) s_base = atomicAdd(counts + 1, held);
        __syncthreads();
        for (uint32_t k = threadIdx.x; k < held; k += HP_THREADS) list2[s_base + k] = s_out[k];
        __syncthreads();
        if (threadIdx.x == 0) s_n = 0;
        __syncthreads();
      }
    }
  }
}

// step 2: one wavefront per outsider, against every other record of its group
__global__ void __launch_bounds__(256)
k_v_outsider_pairs(const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd, uint32_t n,
                   uint64_t mask_lo, const uint32_t *__restrict__ gate,
                   const uint32_t *__restrict__ sig, int K, int min_match,
                   uint32_t *parent, const uint32_t *__restrict__ list2,
                   const uint32_t *__restrict__ counts) {
  const uint64_t mask = *gate ? ~uint64_t(0) : mask_lo;
  const uint32_t n2 = counts[1];
  const int tl = threadIdx.x & (TEAM - 1);
  const uint32_t team = (threadIdx.x & 63) / TEAM;
  const uint32_t waves = gridDim.x * (blockDim.x / 64);
  for (uint32_t e = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64; e < n2; e += waves) {
    const uint32_t o = list2[e];
    const uint64_t key = bk[o];
    const uint32_t band0 = (o / n) * n;
    const uint32_t gs = group_lower_bound(bk, mask, band0, o, key & mask);
    const uint32_t ge = group_upper_bound(bk, mask, o + 1, band0 + n, key & mask);
    const uint32_t v = bd[o];
    // the bucket's first record was this record's partner in step 1 (it is the group's first
    // unless the group holds other keys; then it is merely looked at again)
    for (uint32_t j = gs + (bk[gs] == key ? 1u : 0u) + team; j < ge; j += 64 / TEAM) {
      if (j == o || bk[j] != key) continue;
      team_verify_pair(sig, K, min_match, parent, bd[j], v, tl);
    }
  }
}

// ---- large groups: all pairs, tile by tile (the count-match kernel of Section 3.3) -------------
//
// A large group is cut into tiles of VT records.  Tile (ti, tj), ti <= tj, compares the records
// of tile ti with those of tile tj: one wavefront, each lane holding an 8 x 8 block of pairs (a
// tile costs a few dependent memory round trips and little arithmetic, so many small blocks in
// flight matter more than threads per tile).
//
// The number of equal signature entries of a pair is bounded before it is counted.  Every
// document has a one-bit sketch of its signature (bit k = the lowest bit of entry k, K bits).
// Entries whose sketch bits differ are unequal, so  equal entries <= K - popcount(sketch_u xor
// sketch_v).  The tile kernel passes the sketches of its 2 x VT records through LDS (column-major,
// so that a lane reads its 8 + 8 words with four 16-byte loads), accumulates the popcounts of
// the 64 xors, and only a pair whose bound reaches min_match (and whose full keys are equal, and
// whose documents are not joined yet) has its full signatures compared, entry by entry, by its
// thread.  Unrelated documents agree on about half of the sketch bits (K/2 +- sqrt(K)/2), far
// below any useful threshold, so nearly all pairs of a coarse bucket cost two instructions per 32
// entries instead of two per entry; the pairs that are united are exactly those of the full
// comparison.
// Phase 0 runs the tiles (0, tj) of every group, phase 1 the others; a phase-1 tile whose records
// are all in the component of the group's first record already is skipped, which keeps a large
// group of alike documents (exact copies, empty documents) linear instead of quadratic.
//
// Two kernels share this scheme.  k_v_groups takes the groups whose records fit LDS: document ids,
// keys and the first `lds_words` sketch words of every record (the dense buckets of Section 3.2
// hold a few hundred records).  One block loads the group once and then runs its tiles, 32 x 64
// pairs each, from LDS, so a tile touches global memory only for the rare pair that survives.
// Groups that fit VG_SMALL_WORDS of LDS take one wavefront each (a dozen tiles, nothing to
// synchronise), larger ones a block of four.  k_v_tiles takes the groups beyond that, staging two
// tiles of 64 records' sketches at a time.
// Unrelated documents differ in about 16 sketch bits per word, so after a few words every pair
// of a tile is usually ruled out already.  `lds_words` is that number of words (chosen on the
// host from K and min_match): k_v_groups accumulates them for all pairs of a tile, drops the tile
// if no pair is left, and otherwise finishes the few pairs that are, one by one, with the
// remaining sketch words from memory.  The bound itself is exact either way: popcounts only grow.

constexpr int VT = 64;
constexpr int VWC = 8;   // sketch words per record staged at a time (256 signature entries)
constexpr int VTHREADS = 64;
constexpr uint32_t VG_LDS_WORDS = 8 * 1024;    // k_v_groups with four wavefronts: 32 KiB, five blocks
                                               // per compute unit (as many as the registers allow)
constexpr uint32_t VG_SMALL_WORDS = 2 * 1024;  // k_v_groups with one wavefront: 8 KiB

// records of a group that k_v_groups can hold: per record the sketch words it keeps in LDS, the
// key, the document id and a flag; whole tiles
__host__ __device__ static inline uint32_t group_capacity(uint32_t sketch_words_in_lds,
                                                          uint32_t lds_words = VG_LDS_WORDS) {
  return (lds_words / (sketch_words_in_lds + 4)) & ~uint32_t(VT - 1);
}

// bits[d * KW + w]: bit i = lowest bit of sig[d * K + 32 w + i] (0 past K).  A piece is 64
// consecutive entries of one document: one coalesced load, one ballot, two words.  A wavefront
// takes SKETCH_BATCH consecutive pieces at a time, all loads first.
// Does nothing when the call has no large group (counts[2] == 0).
constexpr int SKETCH_BATCH = 8;
__global__ void __launch_bounds__(256)
k_sig_sketch(const uint32_t *__restrict__ sig, uint32_t n, int K, uint32_t KW,
             const uint32_t *__restrict__ counts, uint32_t *__restrict__ bits) {
  if (counts[2] == 0) return;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t per_doc = (uint32_t)((K + 63) / 64);  // pieces per document
  const uint64_t pieces = (uint64_t)n * per_doc;
  const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const uint64_t n_waves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
  for (uint64_t pc0 = wave * SKETCH_BATCH; pc0 < pieces; pc0 += n_waves * SKETCH_BATCH) {
    const uint64_t d0 = pc0 / per_doc;
    const uint32_t part0 = (uint32_t)(pc0 - d0 * per_doc);
    uint32_t v[SKETCH_BATCH];
    uint64_t d = d0;
    uint32_t part = part0;
#pragma unroll
    for (int j = 0; j < SKETCH_BATCH; j++) {
      const uint32_t k = 64 * part + lane;
      v[j] = pc0 + j < pieces && k < (uint32_t)K ? sig[d * K + k] : 0u;
      if (++part == per_doc) {
        part = 0;
        d++;
      }
    }
    d = d0;
    part = part0;
#pragma unroll
    for (int j = 0; j < SKETCH_BATCH; j++) {
      const uint64_t m = __ballot(v[j] & 1u);
      if (pc0 + j < pieces && lane < 2 && 2 * part + lane < KW)
        bits[d * KW + 2 * part + lane] = (uint32_t)(m >> (32 * lane));
      if (++part == per_doc) {
        part = 0;
        d++;
      }
    }
  }
}

// equal entries of two signatures (one thread)
__device__ __forceinline__ int exact_matches(const uint32_t *__restrict__ sig, uint32_t u, uint32_t v,
                                             int K, bool vec_ok) {
  const uint32_t *a = sig + (uint64_t)u * K, *b = sig + (uint64_t)v * K;
  int m = 0;
  if (vec_ok) {
    for (int k = 0; k < K; k += 4) {
      const uint4 x = *reinterpret_cast<const uint4 *>(a + k);
      const uint4 y = *reinterpret_cast<const uint4 *>(b + k);
      m += (x.x == y.x) + (x.y == y.y) + (x.z == y.z) + (x.w == y.w);
    }
  } else {
    for (int k = 0; k < K; k++) m += a[k] == b[k];
  }
  return m;
}

// exclusive prefix sums over the large groups of their phase-0 and phase-1 tile counts (k_v_tiles)
__global__ void __launch_bounds__(1024)
k_v_plan_tiles(const BigGroup *__restrict__ big, const uint32_t *__restrict__ counts,
               uint64_t big_cap, uint32_t lds_capacity, uint64_t *__restrict__ pre) {
  __shared__ uint64_t s_part[1024 / 64];
  __shared__ uint64_t s_carry[2];
  const uint32_t nb = min((uint64_t)counts[2], big_cap);
  uint64_t *pre0 = pre, *pre1 = pre + big_cap + 1;
  if (threadIdx.x < 2) s_carry[threadIdx.x] = 0;
  __syncthreads();
  for (uint32_t base = 0; base < nb; base += 1024) {
    const uint32_t g = base + threadIdx.x;
    uint64_t v[2] = {0, 0};
    if (g < nb && big[g].size > lds_capacity) {  // the others are k_v_groups' work
      const uint64_t T = (big[g].size + VT - 1) / VT;
      v[0] = T;
      v[1] = T * (T - 1) / 2;
    }
    for (int which = 0; which < 2; which++) {
      // block-wide exclusive scan of v[which]
      uint64_t inc = v[which];
      const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const uint64_t o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
      }
      __syncthreads();
      if (lane == 63) s_part[wave] = inc;
      __syncthreads();
      uint64_t before = s_carry[which];
      for (int w = 0; w < wave; w++) before += s_part[w];
      if (g < nb) (which ? pre1 : pre0)[g] = before + inc - v[which];
      __syncthreads();
      if (threadIdx.x == 1023) s_carry[which] = before + inc;
      __syncthreads();
    }
  }
  if (threadIdx.x == 0) {
    pre0[nb] = s_carry[0];
    pre1[nb] = s_carry[1];
  }
}

__global__ void __launch_bounds__(VTHREADS)
k_v_tiles(int phase, const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd,
          const uint32_t *__restrict__ sig, const uint32_t *__restrict__ bits, int K, int min_match,
          uint32_t *parent, const BigGroup *__restrict__ big, const uint32_t *__restrict__ counts,
          uint64_t big_cap, const uint64_t *__restrict__ pre_all) {
  __shared__ uint32_t sm[VWC][2 * VT];  // [sketch word][record]: records 0..63 of tile ti, 64..127 of tile tj
  __shared__ uint32_t sm_doc[2 * VT];
  __shared__ uint64_t sm_key[2 * VT];
  const uint32_t nb = min((uint64_t)counts[2], big_cap);
  const uint64_t *pre = pre_all + (phase ? big_cap + 1 : 0);
  const uint64_t total = pre[nb];
  const int tid = threadIdx.x, ty = tid >> 3, tx = tid & 7;  // rows 8 ty .., columns 8 tx ..
  const bool vec_ok = (K & 3) == 0 && ((uintptr_t)sig & 15) == 0;
  const int KW = (int)sketch_words(K);
  const int max_diff = K - min_match;  // a pair whose sketches differ in more bits cannot reach min_match
  // every block takes a contiguous range of tiles: one search for the group of its first tile,
  // after that the group index only moves forward
  const uint64_t per_block = (total + gridDim.x - 1) / gridDim.x;
  const uint64_t t_begin = blockIdx.x * per_block;
  const uint64_t t_end = t_begin + per_block < total ? t_begin + per_block : total;
  uint32_t lo = 0;
  {
    uint32_t hi = nb;  // last g with pre[g] <= t_begin
    while (hi - lo > 1) {
      const uint32_t mid = (lo + hi) >> 1;
      if (pre[mid] <= t_begin) lo = mid;
      else hi = mid;
    }
  }
  const bool can_cache = KW <= VWC;  // one staging pass: the row's sketch words are not overwritten
  uint32_t cached_lo = 0xFFFFFFFFu;
  uint64_t cached_ti = 0;
  uint32_t my_doc[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};  // my_doc[0] outlives a tile while its row is cached
  for (uint64_t t = t_begin; t < t_end; t++) {
    while (lo + 1 < nb && pre[lo + 1] <= t) lo++;
    const BigGroup g = big[lo];
    const uint64_t local = t - pre[lo];
    const uint64_t T = (g.size + VT - 1) / VT;
    uint64_t ti, tj;
    if (phase == 0) {
      ti = 0;
      tj = local;
    } else {
      // tiles (ti, tj) with 1 <= ti <= tj < T in row-major order; row ti starts at
      // off(ti) = (ti - 1) T - (ti - 1) ti / 2
      uint64_t r = (uint64_t)((2.0 * (double)T - 1.0 -
                               sqrt((2.0 * (double)T - 1.0) * (2.0 * (double)T - 1.0) -
                                    8.0 * (double)local)) * 0.5) + 1;
      if (r < 1) r = 1;
      if (r > T - 1) r = T - 1;
      while (r > 1 && (r - 1) * T - (r - 1) * r / 2 > local) r--;
      while (r + 1 <= T - 1 && r * T - r * (r + 1) / 2 <= local) r++;
      ti = r;
      tj = ti + (local - ((ti - 1) * T - (ti - 1) * ti / 2));
    }
    __syncthreads();  // the previous tile's LDS reads are done
    // consecutive tiles of a block mostly share their row tile (phase 0: always tile 0 of the
    // group; phase 1: row-major order): its records, keys and sketches then stay in LDS
    const bool row_cached = can_cache && lo == cached_lo && ti == cached_ti;
    bool alike = true;
    uint32_t first_words[2][VWC];  // the records' first VWC sketch words, fetched before anything waits
#pragma unroll
    for (int h = 0; h < 2; h++) {  // lane l loads record l of tile ti and record l of tile tj
      if (h == 0 && row_cached) continue;
      const uint64_t rec = (h == 0 ? ti : tj) * VT + tid;
      uint32_t doc = 0xFFFFFFFFu;
      uint64_t key = 0;
      if (rec < g.size) {
        doc = bd[g.start + rec];
        key = bk[g.start + rec];
      }
      my_doc[h] = doc;
      sm_doc[h * VT + tid] = doc;
      sm_key[h * VT + tid] = key;
#pragma unroll
      for (int w = 0; w < VWC; w++)
        first_words[h][w] = (doc != 0xFFFFFFFFu && w < KW) ? bits[(uint64_t)doc * KW + w] : 0u;
    }
    if (phase) {
      const uint32_t head_root = uf_find(parent, bd[g.start]);
#pragma unroll
      for (int h = 0; h < 2; h++)
        if (my_doc[h] != 0xFFFFFFFFu) alike = alike && uf_find(parent, my_doc[h]) == head_root;
      if (__syncthreads_count(alike ? 0 : 1) == 0) {  // nothing left to learn here
        if (!row_cached) cached_lo = 0xFFFFFFFFu;     // the row's sketches never reached LDS
        continue;
      }
    }
    cached_lo = lo;
    cached_ti = ti;

    uint32_t diff[64];  // diff[8 i + j]: sketch bits that differ, row 8 ty + i against column 8 tx + j
#pragma unroll
    for (int i = 0; i < 64; i++) diff[i] = 0;
    for (int wc = 0; wc < KW; wc += VWC) {
      if (wc) __syncthreads();  // the previous pass has been compared
      const int wmax = min(VWC, KW - wc);
      if (wc == 0) {
#pragma unroll
        for (int w = 0; w < VWC; w++) {
          if (!row_cached) sm[w][tid] = first_words[0][w];
          sm[w][VT + tid] = first_words[1][w];
        }
      } else {
        for (int w = 0; w < wmax; w++) {
          sm[w][tid] = my_doc[0] != 0xFFFFFFFFu ? bits[(uint64_t)my_doc[0] * KW + wc + w] : 0u;
          sm[w][VT + tid] = my_doc[1] != 0xFFFFFFFFu ? bits[(uint64_t)my_doc[1] * KW + wc + w] : 0u;
        }
      }
      __syncthreads();
      for (int w = 0; w < wmax; w++) {
        const uint4 r0 = *reinterpret_cast<const uint4 *>(&sm[w][ty * 8]);
        const uint4 r1 = *reinterpret_cast<const uint4 *>(&sm[w][ty * 8 + 4]);
        const uint4 c0 = *reinterpret_cast<const uint4 *>(&sm[w][VT + tx * 8]);
        const uint4 c1 = *reinterpret_cast<const uint4 *>(&sm[w][VT + tx * 8 + 4]);
        const uint32_t rv[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
        const uint32_t cv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
        for (int i = 0; i < 8; i++)
#pragma unroll
          for (int j = 0; j < 8; j++) diff[8 * i + j] += __popc(rv[i] ^ cv[j]);
      }
    }
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
      for (int j = 0; j < 8; j++) {
        if ((int)diff[8 * i + j] > max_diff) continue;  // the bound rules the pair out
        const int ri = ty * 8 + i, cj = VT + tx * 8 + j;
        const uint32_t u = sm_doc[ri], v = sm_doc[cj];
        if (u == 0xFFFFFFFFu || v == 0xFFFFFFFFu) continue;
        if (ti == tj && ri >= cj - VT) continue;  // upper triangle of a diagonal tile
        if (sm_key[ri] != sm_key[cj]) continue;
        // a candidate: the full comparison decides (skipped for documents joined already)
        if (uf_find(parent, u) == uf_find(parent, v)) continue;
        if (min_match <= 0 || exact_matches(sig, u, v, K, vec_ok) >= min_match) uf_unite(parent, u, v);
      }
  }
}

// Pairs of documents that a block of k_v_groups puts aside (in LDS) while it runs the tiles of a
// group, and decides together afterwards: one lane finishing a pair on the spot (remaining sketch
// words, two finds, K entries) keeps its wavefront waiting on a chain of dependent loads, whereas
// the list is worked off by sixteen lanes per pair, all pairs of the block side by side.
struct PairList {
  uint2 *pairs;     // document ids
  uint32_t *count;  // pairs appended (may exceed cap: those were finished on the spot)
  uint32_t cap;
};

// A pair that the sketch words in LDS (the first lds_words of each record) have not ruled out, d
// differing bits so far: the keys; then either onto the list, or, in place, the remaining
// sketch words from memory and the full comparison.  Rare, so kept out of line.
__device__ __noinline__ void group_pair(const uint32_t *__restrict__ bits, int KW, int lds_words,
                                        uint32_t d, int max_diff, const uint32_t *__restrict__ s_doc,
                                        const uint64_t *__restrict__ s_key, uint32_t ri, uint32_t cj,
                                        const uint32_t *__restrict__ sig, int K, int min_match,
                                        bool vec_ok, uint32_t *parent, const PairList *defer) {
  const uint32_t u = s_doc[ri], v = s_doc[cj];
  if (u == 0xFFFFFFFFu || v == 0xFFFFFFFFu) return;
  if (s_key[ri] != s_key[cj]) return;
  if (defer) {
    const uint32_t slot = atomicAdd(defer->count, 1u);
    if (slot < defer->cap) {
      defer->pairs[slot] = make_uint2(u, v);
      return;
    }
  }
  const uint32_t *bu = bits + (uint64_t)u * KW, *bv = bits + (uint64_t)v * KW;
  for (int w = lds_words; w < KW && (int)d <= max_diff; w++) d += __popc(bu[w] ^ bv[w]);
  if ((int)d > max_diff) return;  // the bound rules the pair out
  // a candidate: the full comparison decides (skipped for documents joined already)
  if (uf_find(parent, u) == uf_find(parent, v)) return;
  if (min_match <= 0 || exact_matches(sig, u, v, K, vec_ok) >= min_match) uf_unite(parent, u, v);
}

// One tile of a group that sits in LDS: the 32 records from row0 on against the 64 from col0 on
// (row0 a multiple of 32, col0 of 64, row0 < col0 + 64).  sk[w * cap + rec] = sketch word w of
// record rec, w < lds_words; slots past the group's end have the document id 0xFFFFFFFF.  One wavefront, each lane a 4 x 8 block of pairs (half the registers of 8 x 8:
// five wavefronts share a SIMD).  The words in LDS are accumulated for all pairs; if some pair
// is still below the bound then, the few that are get finished one by one (s_joined, if given,
// marks the records known to be in the component of the group's first record: a pair of two such
// records has nothing to add).
__device__ __forceinline__ void group_tile(const uint32_t *__restrict__ sk, uint32_t cap, int lds_words,
                                           const uint32_t *__restrict__ bits, int KW, int max_diff,
                                           const uint32_t *__restrict__ s_doc,
                                           const uint64_t *__restrict__ s_key,
                                           const uint32_t *__restrict__ s_joined, uint32_t row0,
                                           uint32_t col0, const uint32_t *__restrict__ sig, int K,
                                           int min_match, bool vec_ok, uint32_t *parent,
                                           const PairList *defer) {
  const int lane = threadIdx.x & 63, ty = lane >> 3, tx = lane & 7;  // rows 4 ty .., columns 8 tx ..
  uint32_t diff[32];  // diff[8 i + j]: sketch bits that differ, row 4 ty + i against column 8 tx + j
  const uint32_t *rp = sk + row0 + ty * 4, *cp = sk + col0 + tx * 8;
  auto accumulate = [&](int w, bool first) {
    const uint4 r0 = *reinterpret_cast<const uint4 *>(rp + (size_t)w * cap);
    const uint4 c0 = *reinterpret_cast<const uint4 *>(cp + (size_t)w * cap);
    const uint4 c1 = *reinterpret_cast<const uint4 *>(cp + (size_t)w * cap + 4);
    const uint32_t rv[4] = {r0.x, r0.y, r0.z, r0.w};
    const uint32_t cv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 8; j++)
        diff[8 * i + j] = (first ? 0u : diff[8 * i + j]) + __popc(rv[i] ^ cv[j]);
  };
  accumulate(0, true);
  for (int w = 1; w < lds_words; w++) accumulate(w, false);
  // the smallest count among the pairs that matter: where the rows reach into the columns' range,
  // those with the row record before the column record
  const bool diagonal = row0 + 32 > col0;  // uniform: one tile in each row of tiles
  uint32_t least = diff[0];
#pragma unroll
  for (int i = 1; i < 32; i++) least = min(least, diff[i]);  // three-way minima: 16 instructions
  if (diagonal) {
    // (the empty statement keeps this a branch of its own: turned into selects inside the minima
    // above, it would cost every tile three instructions per pair)
    asm volatile("");
    least = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 8; j++)
        if (row0 + ty * 4 + i < col0 + tx * 8 + j) least = min(least, diff[8 * i + j]);
  }
  if (__all((int)least > max_diff)) return;  // no pair of the tile can reach min_match any more
  if ((int)least > max_diff) return;         // none of this lane's
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 8; j++) {
      if ((int)diff[8 * i + j] > max_diff) continue;
      const uint32_t ri = row0 + ty * 4 + i, cj = col0 + tx * 8 + j;
      if (ri >= cj) continue;  // every pair once: the earlier record is the row
      // both in the component of the group's first record already (s_joined: phase 1 only)
      if (s_joined && s_joined[ri] && s_joined[cj]) continue;
      group_pair(bits, KW, lds_words, diff[8 * i + j], max_diff, s_doc, s_key, ri, cj, sig, K, min_match,
                 vec_ok, parent, defer);
    }
}

// The large groups of more than min_size records that fit LDS_WORDS of LDS (see above): one block
// of WAVES wavefronts per group at a time.
template <int WAVES, uint32_t LDS_WORDS>
__global__ void __launch_bounds__(WAVES * 64)
k_v_groups(const uint64_t *__restrict__ bk, const uint32_t *__restrict__ bd,
           const uint32_t *__restrict__ sig, const uint32_t *__restrict__ bits, int K, int min_match,
           int lds_words, uint32_t min_size, uint32_t *parent, const BigGroup *__restrict__ big,
           const uint32_t *__restrict__ counts, uint64_t big_cap) {
  constexpr uint32_t VG_THREADS = WAVES * 64;
  constexpr uint32_t LATER_CAP = WAVES * 128;  // pairs a block can put aside per group
  __shared__ __attribute__((aligned(16))) uint32_t lds[LDS_WORDS];
  __shared__ uint2 s_later[LATER_CAP];
  __shared__ uint32_t s_later_n;
  PairList later;
  later.pairs = s_later;
  later.count = &s_later_n;
  later.cap = LATER_CAP;
  const int KW = (int)sketch_words(K);
  const uint32_t cap = group_capacity((uint32_t)lds_words, LDS_WORDS);
  // keys first (8-byte aligned), then document ids, flags, sketches [word][record]
  uint64_t *s_key = reinterpret_cast<uint64_t *>(lds);
  uint32_t *s_doc = lds + 2 * cap, *s_joined = lds + 3 * cap, *sk = lds + 4 * cap;
  const uint32_t nb = min((uint64_t)counts[2], big_cap);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform, and known to be
  const bool vec_ok = (K & 3) == 0 && ((uintptr_t)sig & 15) == 0;
  const int max_diff = K - min_match;  // a pair whose sketches differ in more bits cannot reach min_match
  for (uint32_t gi = blockIdx.x; gi < nb; gi += gridDim.x) {
    const BigGroup g = big[gi];
    if (g.size > cap || g.size <= min_size) continue;  // another launch's work (uniform over the block)
    const uint32_t T = (g.size + VT - 1) / VT;  // column blocks of 64 records; row blocks of 32: 2 T
    __syncthreads();  // the previous group's readers are done
    if (tid == 0) s_later_n = 0;
    // two sweeps, so that the loads of several records are in flight together: ids and keys
    // first, then the sketches they point to (a thread reads back what it wrote itself)
#pragma unroll 4
    for (uint32_t rec = tid; rec < T * VT; rec += VG_THREADS) {
      uint32_t doc = 0xFFFFFFFFu;
      uint64_t key = 0;
      if (rec < g.size) {
        doc = bd[g.start + rec];
        key = bk[g.start + rec];
      }
      s_doc[rec] = doc;
      s_key[rec] = key;
    }
#pragma unroll 2
    for (uint32_t rec = tid; rec < T * VT; rec += VG_THREADS) {
      const uint32_t doc = s_doc[rec];
      // a slot past the group's end gets scrambled bits, so that the bound rules it out like an
      // unrelated document instead of keeping its tile alive (its document id says what it is anyway)
      for (int w = 0; w < lds_words; w++)
        sk[(size_t)w * cap + rec] =
            doc != 0xFFFFFFFFu ? bits[(uint64_t)doc * KW + w] : 0x9E3779B9u * (rec * 8u + (uint32_t)w + 1u);
    }
    __syncthreads();
    // phase 0: the group's first 64 records (two row blocks) against every column block; pairs
    // are decided in place, so that phase 1 knows who has joined the first record
    for (uint32_t q = wave; q < 2 * T; q += WAVES) {
      const uint32_t ri = q & 1, tj = q >> 1;
      group_tile(sk, cap, lds_words, bits, KW, max_diff, s_doc, s_key, nullptr, ri * 32, tj * VT, sig, K,
                 min_match, vec_ok, parent, nullptr);
    }
    if (T < 2) continue;
    __syncthreads();
    // who is in the component of the group's first record by now (a record that joins it later
    // is merely compared once more)
    {
      const uint32_t head_root = uf_find(parent, s_doc[0]);
      for (uint32_t rec = tid; rec < T * VT; rec += VG_THREADS) {
        const uint32_t doc = s_doc[rec];
        s_joined[rec] = (doc == 0xFFFFFFFFu || uf_find(parent, doc) == head_root) ? 1u : 0u;
      }
    }
    __syncthreads();
    // phase 1: the other tiles (row block ri of 32 records against the column blocks from the one
    // that holds it on), dealt to the wavefronts in turn; surviving pairs go onto the list
    uint32_t q = 0;
    for (uint32_t ri = 2; ri < 2 * T; ri++)
      for (uint32_t tj = ri >> 1; tj < T; tj++, q++) {
        if ((q & (WAVES - 1)) != (uint32_t)wave) continue;
        const bool alike = s_joined[ri * 32 + (lane & 31)] && s_joined[tj * VT + lane];
        if (__all(alike)) continue;  // nothing left to learn here
        group_tile(sk, cap, lds_words, bits, KW, max_diff, s_doc, s_key, s_joined, ri * 32, tj * VT, sig, K,
                   min_match, vec_ok, parent, &later);
      }
    __syncthreads();
    // the pairs put aside: sixteen lanes per pair take the sketch bound over all words and, if it
    // holds, the find and the full comparison
    {
      const uint32_t n_later = min(s_later_n, LATER_CAP);
      const int tl = tid & (TEAM - 1);
      for (uint32_t e = tid / TEAM; e < n_later; e += VG_THREADS / TEAM) {
        const uint2 p = s_later[e];
        const uint32_t *bu = bits + (uint64_t)p.x * KW, *bv = bits + (uint64_t)p.y * KW;
        uint32_t d = 0;
        for (int w = tl; w < KW; w += TEAM) d += __popc(bu[w] ^ bv[w]);
#pragma unroll
        for (int o = TEAM / 2; o >= 1; o >>= 1) d += __shfl_xor(d, o, TEAM);
        if ((int)d > max_diff) continue;  // the bound rules the pair out (uniform over the team)
        team_verify_pair(sig, K, min_match, parent, p.x, p.y, tl);
      }
    }
  }
}

static int check_verified_args(const void *keys, const void *sig, uint64_t n_docs, int32_t K, int32_t b,
                               int32_t min_match, const void *out) {
  if (K < 1 || K > SEDD_MAX_K || min_match < 0) return SEDD_EINVAL;
  int rc = check_cluster_args(keys, n_docs, b, out);
  if (rc || n_docs == 0) return rc;
  if (!sig || !aligned_to(sig, 4)) return SEDD_EINVAL;
  return SEDD_OK;
}

// Sketch words that k_v_groups accumulates for every pair of a tile before it looks at the counts.
// Two unrelated documents differ in Binomial(32, 1/2) bits per word: after w words in about
// 16 w +- sqrt(8 w).  The first w where four standard deviations below that mean still exceed
// K - min_match leaves next to no unrelated pair; with a low threshold that is every word.
static int sketch_check_words(int K, int min_match) {
  const int KW = (int)sketch_words(K);
  const double max_diff = (double)K - (double)min_match;
  for (int w = 1; w < KW; w++)
    if (16.0 * w - 4.0 * std::sqrt(8.0 * w) > max_diff) return w;
  return KW;
}

// sedd_cluster_verified on the buffers of `sb` (the caller has checked the arguments)
static int run_cluster_verified(const uint64_t *keys, const uint32_t *sig, uint64_t n_docs, int32_t K,
                                uint32_t b, int32_t min_match, int64_t *cluster_id, SortBufs &sb,
                                hipStream_t st) {
  int rc;
  uint32_t *counts = sb.counts;  // list lengths (followers, outsiders, large groups), cleared by every call
  const int bits = grouping_bits(n_docs, 256);
  // records of mixed large groups the call puts up with before it sorts by the whole key
  const uint32_t mixed_limit = (uint32_t)std::min<uint64_t>(n_docs * b / 1024, 0x7FFFFFFFu);
  g_last_gate = sb.gate;
  {
    ProfScope prof(SEDD_PROF_SORT, st);
    rc = sort_bands(keys, n_docs, b, bits, &sb, st, true);
    if (rc) return rc;
  }
  const uint32_t n = (uint32_t)n_docs;
  const uint64_t mask = (uint64_t(1) << bits) - 1;
  // the sort leaves its result in the first buffer pair; the second pair holds the two lists
  uint32_t *list1 = (uint32_t *)sb.kb, *list2 = sb.db;
  {
    ProfScope prof(SEDD_PROF_VERIFY, st);
    hipLaunchKernelGGL(k_iota_u32, dim3((n + 255) / 256), dim3(256), 0, st, sb.parent, n);
    SEDD_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_fill_small_u32, dim3(1), dim3(64), 0, st, counts, 4u, 0u,
                       (const uint32_t *)nullptr);
    SEDD_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_fill_small_u32, dim3(1), dim3(64), 0, st, sb.gate, 1u, 0u,
                       (const uint32_t *)nullptr);
    SEDD_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_v_mark, dim3(sb.nblk, b), dim3(SORT_THREADS), 0, st, sb.ka, n, mask,
                       list1, counts, sb.big, sb.gate, mixed_limit, 0);
    SEDD_LAUNCH_CHECK();
  }
  {
    // only if too many records sat in large groups of mixed keys (the sorted bits were too few to separate
    // the buckets): sort by the rest of the key and mark again, now on whole keys
    ProfScope prof(SEDD_PROF_SORT, st);
    rc = sort_rest_if_gated(n_docs, b, bits, &sb, st);
    if (rc) return rc;
  }
  ProfScope prof(SEDD_PROF_VERIFY, st);
  hipLaunchKernelGGL(k_fill_small_u32, dim3(1), dim3(64), 0, st, counts, 4u, 0u,
                     (const uint32_t *)sb.gate);
  SEDD_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_v_mark, dim3(sb.nblk, b), dim3(SORT_THREADS), 0, st, sb.ka, n,
                     ~uint64_t(0), list1, counts, sb.big, sb.gate, mixed_limit, 1);
  SEDD_LAUNCH_CHECK();
  // large groups: sketches; the groups that fit LDS; for the others the tile plan, then the tiles
  // against each group's first tile, then the rest
  const uint32_t KW = sketch_words(K);
  const int check_words = sketch_check_words((int)K, (int)min_match);
  hipLaunchKernelGGL(k_v_plan_tiles, dim3(1), dim3(1024), 0, st, sb.big, counts, sb.big_cap,
                     group_capacity((uint32_t)check_words), sb.tile_pre);
  SEDD_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_sig_sketch, dim3(256 * 16), dim3(256), 0, st, sig, n, (int)K, KW, counts,
                     sb.sketch);
  SEDD_LAUNCH_CHECK();
  // many more blocks than the chip holds at once: groups differ a lot in work, and the hardware
  // hands a finished block's place to the next one; a block that finds no group of its launch exits
  hipLaunchKernelGGL((k_v_groups<1, VG_SMALL_WORDS>), dim3(256 * 512), dim3(64), 0, st, sb.ka, sb.da, sig,
                     sb.sketch, (int)K, (int)min_match, check_words, 0u, sb.parent, sb.big, counts,
                     sb.big_cap);
  SEDD_LAUNCH_CHECK();
  hipLaunchKernelGGL((k_v_groups<4, VG_LDS_WORDS>), dim3(256 * 128), dim3(256), 0, st, sb.ka, sb.da, sig,
                     sb.sketch, (int)K, (int)min_match, check_words,
                     group_capacity((uint32_t)check_words, VG_SMALL_WORDS), sb.parent, sb.big, counts,
                     sb.big_cap);
  SEDD_LAUNCH_CHECK();
  for (int phase = 0; phase < 2; phase++) {
    hipLaunchKernelGGL(k_v_tiles, dim3(256 * 24), dim3(VTHREADS), 0, st, phase, sb.ka, sb.da, sig, sb.sketch,
                       (int)K, (int)min_match, sb.parent, sb.big, counts, sb.big_cap, sb.tile_pre);
    SEDD_LAUNCH_CHECK();
  }
  // grids sized to the chip: the kernels stride over lists whose lengths only the device knows
  const uint32_t grid = 256 * 16;
  hipLaunchKernelGGL(k_v_head_pairs, dim3(grid), dim3(HP_THREADS), 0, st, sb.ka, sb.da, n, mask,
                     (const uint32_t *)sb.gate, sig, (int)K, (int)min_match, sb.parent, list1, counts,
                     list2);
  SEDD_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_v_outsider_pairs, dim3(grid), dim3(256), 0, st, sb.ka, sb.da, n, mask,
                     (const uint32_t *)sb.gate, sig, (int)K, (int)min_match, sb.parent, list2, counts);
  SEDD_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_write_roots, dim3((n + 255) / 256), dim3(256), 0, st, sb.parent, n,
                     cluster_id);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

}  // namespace sedd

using namespace sedd;

extern "C" {

int sedd_cluster_verified(const uint64_t *keys, const uint32_t *sig, uint64_t n_docs, int32_t K,
                          int32_t b, int32_t min_match, int64_t *cluster_id, void *stream) {
  int rc = check_verified_args(keys, sig, n_docs, K, b, min_match, cluster_id);
  if (rc || n_docs == 0) return rc;
  SortBufs sb;
  rc = sort_layout(n_docs, (uint32_t)b, &sb, (int)K);
  if (rc) return rc;
  return run_cluster_verified(keys, sig, n_docs, K, (uint32_t)b, min_match, cluster_id, sb,
                              (hipStream_t)stream);
}

int sedd_cluster_verified_ws(const uint64_t *keys, const uint32_t *sig, uint64_t n_docs, int32_t K,
                             int32_t b, int32_t min_match, int64_t *cluster_id, void *workspace,
                             uint64_t workspace_bytes, void *stream) {
  int rc = check_verified_args(keys, sig, n_docs, K, b, min_match, cluster_id);
  if (rc || n_docs == 0) return rc;
  SortBufs sb;
  rc = bind_workspace(plan_sort(n_docs, (uint32_t)b, (int)K), workspace, workspace_bytes, &sb);
  if (rc) return rc;
  return run_cluster_verified(keys, sig, n_docs, K, (uint32_t)b, min_match, cluster_id, sb,
                              (hipStream_t)stream);
}

}  // extern "C"
