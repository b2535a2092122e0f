// sedd_minhash: shingling, Eq. 1 base hash, K hash functions and per-document minimum.
//
// Pipeline per chunk of consecutive documents (all on the caller's stream, no host waits):
//   1. byte tiles     each non-empty document is cut into 4 KiB tiles aligned to 16-byte
//                     addresses; a scan over per-document tile counts builds the work list.
//   2. words          (word mode) one block per byte tile marks token starts from a 16-byte
//                     vector load per thread, counts them, and after a scan writes one record
//                     per token: its Eq. 1 hash W and q^len.
//   3. shingle tiles  per-document shingle counts, scanned into shingle offsets and a second
//                     work list of tiles of TS shingles.
//   4. base hash      one thread per shingle: Horner over n token records (word mode) or over
//                     n bytes (byte mode) gives x(s) of Eq. 1.
//   5. min-hash       one wavefront per shingle tile, lane = hash function: the 61-bit
//                     multiply-add mod 2^61-1, truncation to 32 bits and running minimum.
//                     This is where the time goes: K modular multiplies per shingle.
#include <algorithm>
#include <vector>

#include "sedd_internal.h"

namespace sedd {

constexpr int TB_THREADS = 256;
constexpr uint32_t TB = TB_THREADS * 16;  // bytes per byte tile
constexpr uint32_t TS = 1024;             // shingles per hash tile
constexpr int QPOW_N = 256;

// x(s) of Eq. 1 as the hot kernel wants it: x = x1 * 2^31 + x0 with x0 < 2^31, x1 < 2^30,
// stored pre-scaled as lo2 = 2 x0 and hi4 = 4 x1 (both fit 32 bits).
struct XSplit {
  uint32_t lo2, hi4;
};
__device__ __forceinline__ XSplit x_split(uint64_t x) {
  XSplit r;
  r.lo2 = ((uint32_t)x & 0x7FFFFFFFu) << 1;
  r.hi4 = (uint32_t)(x >> 31) << 2;
  return r;
}
__device__ __forceinline__ uint64_t x_join(XSplit v) {
  return ((uint64_t)(v.hi4 >> 2) << 31) | (v.lo2 >> 1);
}

// coefficients of one hash function in the same limb form: a = a1 * 2^31 + a0
struct CoefSplit {
  uint32_t a0;   // a mod 2^31
  uint32_t a12;  // 2 * (a >> 31)
};

struct WordRec {
  uint64_t w;   // Eq. 1 hash of the token's bytes
  uint64_t pw;  // 257^len mod p
};

static uint64_t g_chunk_bytes_override = 0;

// ---- small kernels -------------------------------------------------------------------------

__global__ void k_fill_u32(uint32_t *p, uint64_t n, uint32_t v) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

__global__ void k_zero_u64(uint64_t *p) { *p = 0; }

// a_k = s0 * Ga^(k+1), b_k = s0 * Gb^(k+1) (mod p), s0 = (seed mod (p-1)) + 1; qpow[i] = 257^i
__global__ void k_coeffs(uint64_t seed, int K, uint64_t *a, uint64_t *b, CoefSplit *split,
                         uint64_t *qpow) {
  int k = blockIdx.x * blockDim.x + threadIdx.x;
  uint64_t s0 = seed % (P61 - 1) + 1;
  if (k < K) {
    const uint64_t ak = mulmod(s0, powmod(G_A, (uint64_t)k + 1));
    a[k] = ak;
    b[k] = mulmod(s0, powmod(G_B, (uint64_t)k + 1));
    if (split) {
      CoefSplit c;
      c.a0 = (uint32_t)ak & 0x7FFFFFFFu;
      c.a12 = (uint32_t)(ak >> 31) << 1;
      split[k] = c;
    }
  }
  if (qpow && k < QPOW_N) qpow[k] = powmod(257, (uint64_t)k);
}

// dv[i] = position of document i's first byte in the chunk's 16-byte aligned frame;
// cnt[i] = number of 4 KiB byte tiles of document i (0 if empty); cnt[nd] = 0.
__global__ void k_doc_btiles(const uint64_t *__restrict__ off, uint64_t shift, uint32_t nd,
                             uint32_t *__restrict__ dv, uint32_t *__restrict__ cnt) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i > nd) return;
  uint32_t vs = (uint32_t)(off[i] + shift);
  dv[i] = vs;
  uint32_t c = 0;
  if (i < nd) {
    uint32_t ve = (uint32_t)(off[i + 1] + shift);
    if (ve > vs) c = (ve - (vs & ~15u) + TB - 1) / TB;
  }
  cnt[i] = c;
}

// tile_doc[t] = d for every tile t of document d
__global__ void k_fill_tile_doc(const uint32_t *__restrict__ tbase, uint32_t nd,
                                uint32_t *__restrict__ tile_doc) {
  uint32_t d = blockIdx.x * blockDim.x + threadIdx.x;
  if (d >= nd) return;
  uint32_t t1 = tbase[d + 1];
  for (uint32_t t = tbase[d]; t < t1; t++) tile_doc[t] = d;
}

// ---- tokenisation ------------------------------------------------------------------------

// Bit i of the result: byte seg+i starts a token of the document [vs, ve).  seg is 16-aligned.
__device__ __forceinline__ uint32_t token_starts(const uint8_t *__restrict__ pbase, uint32_t seg,
                                                 uint32_t vs, uint32_t ve, uint32_t *sm_last) {
  uint32_t wm = 0;
  if (seg < ve && seg + 16 > vs) {
    const uint4 q = *reinterpret_cast<const uint4 *>(pbase + seg);
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 16; i++) {
      uint32_t c = (w[i >> 2] >> (8 * (i & 3))) & 0xFFu;
      uint32_t pos = seg + i;
      if (pos >= vs && pos < ve && !is_ws(c)) wm |= 1u << i;
    }
  }
  sm_last[threadIdx.x] = wm >> 15;
  __syncthreads();
  uint32_t prev;
  if (threadIdx.x > 0) {
    prev = sm_last[threadIdx.x - 1];
  } else {
    // byte before the tile: inside the document only if seg > vs
    prev = (seg > vs && seg <= ve) ? (is_ws(pbase[seg - 1]) ? 0u : 1u) : 0u;
  }
  return wm & ~((wm << 1) | prev) & 0xFFFFu;
}

__global__ void __launch_bounds__(TB_THREADS)
k_count_words(const uint8_t *__restrict__ pbase, const uint32_t *__restrict__ dv,
              const uint32_t *__restrict__ btile_base, const uint32_t *__restrict__ tile_doc,
              uint32_t nd, uint32_t *__restrict__ wcnt) {
  __shared__ uint32_t sm_last[TB_THREADS];
  const uint32_t t = blockIdx.x;
  if (t >= btile_base[nd]) {
    if (threadIdx.x == 0) wcnt[t] = 0;
    return;
  }
  const uint32_t d = tile_doc[t];
  const uint32_t vs = dv[d], ve = dv[d + 1];
  const uint32_t seg = (vs & ~15u) + (t - btile_base[d]) * TB + threadIdx.x * 16;
  uint32_t starts = token_starts(pbase, seg, vs, ve, sm_last);
  uint32_t tot;
  block_exclusive_scan<TB_THREADS>(__popc(starts), &tot);
  if (threadIdx.x == 0) wcnt[t] = tot;
}

__global__ void __launch_bounds__(TB_THREADS)
k_emit_words(const uint8_t *__restrict__ pbase, const uint32_t *__restrict__ dv,
             const uint32_t *__restrict__ btile_base, const uint32_t *__restrict__ tile_doc,
             uint32_t nd, const uint32_t *__restrict__ wbase, const uint64_t *__restrict__ qpow,
             WordRec *__restrict__ rec) {
  __shared__ uint32_t sm_last[TB_THREADS];
  const uint32_t t = blockIdx.x;
  if (t >= btile_base[nd]) return;
  const uint32_t d = tile_doc[t];
  const uint32_t vs = dv[d], ve = dv[d + 1];
  const uint32_t seg = (vs & ~15u) + (t - btile_base[d]) * TB + threadIdx.x * 16;
  uint32_t starts = token_starts(pbase, seg, vs, ve, sm_last);
  uint32_t tot;
  uint32_t rank = wbase[t] + block_exclusive_scan<TB_THREADS>(__popc(starts), &tot);
  while (starts) {
    const uint32_t s = seg + (uint32_t)__ffs(starts) - 1;
    starts &= starts - 1;
    uint32_t e = s + 1;
    while (e < ve && !is_ws(pbase[e])) e++;
    uint64_t acc = 0;  // Horner from the last byte: W = c_0 + q (c_1 + q (...))
    for (uint32_t j = e; j-- > s;) acc = addmod(mul257(acc), (uint64_t)pbase[j]);
    const uint32_t len = e - s;
    WordRec r;
    r.w = acc;
    r.pw = len < (uint32_t)QPOW_N ? qpow[len] : powmod(257, len);
    rec[rank++] = r;
  }
}

// ---- shingle work list -------------------------------------------------------------------

// Per document: first token index, shingle count and number of TS-shingle tiles.
__global__ void k_doc_shingles(const uint32_t *__restrict__ dv,
                               const uint32_t *__restrict__ btile_base,
                               const uint32_t *__restrict__ wbase, uint32_t nd, uint32_t n,
                               int byte_mode, uint32_t *__restrict__ docw,
                               uint32_t *__restrict__ scnt, uint32_t *__restrict__ hcnt) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i > nd) return;
  uint32_t S = 0;
  if (byte_mode) {
    if (i < nd) {
      uint32_t len = dv[i + 1] - dv[i];
      S = len == 0 ? 0u : (len < n ? 1u : len - n + 1);
    }
  } else {
    uint32_t w0 = wbase[btile_base[i]];
    docw[i] = w0;
    if (i < nd) {
      uint32_t W = wbase[btile_base[i + 1]] - w0;
      S = W == 0 ? 0u : (W < n ? 1u : W - n + 1);
    }
  }
  scnt[i] = S;
  hcnt[i] = (S + TS - 1) / TS;
}

// x(s) of Eq. 1 for every shingle of the chunk: block per shingle tile, thread per shingle.
__global__ void __launch_bounds__(256)
k_shingle_hash(const uint8_t *__restrict__ pbase, const uint32_t *__restrict__ dv,
               const uint32_t *__restrict__ docw, const WordRec *__restrict__ rec,
               const uint32_t *__restrict__ sbase, const uint32_t *__restrict__ htile_base,
               const uint32_t *__restrict__ htile_doc, uint32_t nd, uint32_t n, int byte_mode,
               XSplit *__restrict__ xs) {
  const uint32_t t = blockIdx.x;
  if (t >= htile_base[nd]) return;
  const uint32_t d = htile_doc[t];
  const uint32_t s0 = sbase[d], S = sbase[d + 1] - s0;
  const uint32_t i0 = (t - htile_base[d]) * TS;
  const uint32_t i1 = min(i0 + TS, S);
  if (byte_mode) {
    const uint32_t vs = dv[d], len = dv[d + 1] - vs;
    const uint32_t per = min(len, n);
    for (uint32_t i = i0 + threadIdx.x; i < i1; i += blockDim.x) {
      const uint8_t *p = pbase + vs + i;
      uint64_t acc = 0;
      for (uint32_t j = per; j-- > 0;) acc = addmod(mul257(acc), (uint64_t)p[j]);
      xs[s0 + i] = x_split(acc);
    }
  } else {
    const uint32_t w0 = docw[d], W = docw[d + 1] - w0;
    const uint32_t per = min(W, n);
    for (uint32_t i = i0 + threadIdx.x; i < i1; i += blockDim.x) {
      const WordRec *r = rec + w0 + i;
      uint64_t acc = r[per - 1].w;
      // prepend "token 0x20": x = W + q^len * (32 + q * x_rest)
      for (uint32_t m = per - 1; m-- > 0;)
        acc = addmod(r[m].w, mulmod(r[m].pw, addmod(32, mul257(acc))));
      xs[s0 + i] = x_split(acc);
    }
  }
}

// ---- the hot kernel ------------------------------------------------------------------------
//
// One wavefront per shingle tile; lane l evaluates hash functions k0+l, k0+64+l, ... (F of them),
// the shingle value is wave-uniform (scalar registers).  Per (shingle, function) the kernel needs
// h = ((a x + b) mod p) mod 2^32 with p = 2^61-1.
//
// 31-bit limbs: a = a1 2^31 + a0, x = x1 2^31 + x0.  With 2^61 = 1 and 2^62 = 2 (mod p):
//   a x + b  =  a0 x0 + 2 a1 x1 + b  +  2^31 M,        M = a0 x1 + a1 x0  (< 2^62)
//   2^31 M   =  mh + 2^31 ml,                           mh = M >> 30, ml = M mod 2^30
// N = 4 M = a0 (4 x1) + (2 a1)(2 x0) is formed instead of M: its high word is mh and its low word
// is 4 ml, so 2^31 ml = n_lo 2^29 needs no mask.  Everything is chained through the 64-bit addend
// of the 32x32+64 multiply-add:
//   N = a0*(4x1) + (2a1)*(2x0);  S = n_lo*2^29 + a0*x0 + (2a1)*x1 + b  (< 2^64);  Z = S + mh.
// Z mod p has low word  s_lo + mh + (S >> 61)  unless bits 33..60 of S are all ones (then a carry
// may cross bit 61 or the folded value may reach p).  That case has probability 2^-28 per
// evaluation; the lane records it in `amb`, and a tile with any such lane is recomputed with the
// plain 64-bit arithmetic.  The multipliers 2^29 and 8 are passed as kernel arguments so that they
// stay multiplies (one instruction) instead of being expanded into 64-bit shift/add pairs.

struct HotConsts {
  uint32_t two29;  // 1 << 29
  uint32_t eight;  // 8
};

template <int F>
__global__ void __launch_bounds__(64)
k_minhash(const XSplit *__restrict__ xs, const uint32_t *__restrict__ sbase,
          const uint32_t *__restrict__ htile_base, const uint32_t *__restrict__ htile_doc,
          uint32_t nd, const uint64_t *__restrict__ coef_a, const uint64_t *__restrict__ coef_b,
          const CoefSplit *__restrict__ coef_split, int K,
          uint32_t *__restrict__ sig /* first document of the chunk */, HotConsts hc,
          unsigned long long *__restrict__ slow_tiles) {
  const uint32_t t = blockIdx.x;
  if (t >= htile_base[nd]) return;
  const uint32_t d = htile_doc[t];
  const uint32_t tb = htile_base[d], ntile = htile_base[d + 1] - tb;
  const uint32_t s0 = sbase[d], S = sbase[d + 1] - s0;
  const uint32_t i0 = (t - tb) * TS;
  const uint32_t cnt = min(TS, S - i0);
  const XSplit *__restrict__ xp = xs + s0 + i0;

  const int kbase = blockIdx.y * (64 * F) + threadIdx.x;
  uint64_t a[F], b[F];
  uint32_t a0[F], a12[F], m[F];
#pragma unroll
  for (int j = 0; j < F; j++) {
    int k = kbase + 64 * j;
    const int kk = k < K ? k : 0;  // lanes past K compute function 0 and store nothing
    a[j] = coef_a[kk];
    b[j] = coef_b[kk];
    const CoefSplit c = coef_split[kk];
    a0[j] = c.a0;
    a12[j] = c.a12;
    m[j] = 0xFFFFFFFFu;
  }
  uint32_t amb = 0;
#pragma unroll 4
  for (uint32_t s = 0; s < cnt; s++) {
    const XSplit xv = xp[s];
    const uint32_t x0_2 = xv.lo2, x1_4 = xv.hi4;
    const uint32_t x0 = x0_2 >> 1, x1 = x1_4 >> 2;
#pragma unroll
    for (int j = 0; j < F; j++) {
      uint64_t N = (uint64_t)a0[j] * x1_4;
      N += (uint64_t)a12[j] * x0_2;
      uint64_t U = (uint64_t)a12[j] * x1 + b[j];
      U += (uint64_t)a0[j] * x0;
      const uint64_t Sv = (uint64_t)(uint32_t)N * hc.two29 + U;
      const uint64_t W = (uint64_t)(uint32_t)(Sv >> 32) * hc.eight;  // hi: S >> 61, lo: bits 32..60
      const uint32_t h = (uint32_t)Sv + (uint32_t)(N >> 32) + (uint32_t)(W >> 32);
      amb = max(amb, (uint32_t)W);
      m[j] = min(m[j], h);
    }
  }
  if (__any(amb >= 0xFFFFFFF0u)) {
    // rare: some evaluation sat within reach of a carry across bit 61; redo the tile exactly
    if (threadIdx.x == 0 && blockIdx.y == 0) atomicAdd(slow_tiles, 1ull);
#pragma unroll
    for (int j = 0; j < F; j++) m[j] = 0xFFFFFFFFu;
    for (uint32_t s = 0; s < cnt; s++) {
      const uint64_t x = x_join(xp[s]);
#pragma unroll
      for (int j = 0; j < F; j++) m[j] = min(m[j], (uint32_t)addmod(mulmod(a[j], x), b[j]));
    }
  }
  uint32_t *out = sig + (uint64_t)d * K;
#pragma unroll
  for (int j = 0; j < F; j++) {
    int k = kbase + 64 * j;
    if (k < K) {
      if (ntile == 1) out[k] = m[j];
      else atomicMin(out + k, m[j]);
    }
  }
}

// ---- debug copies ------------------------------------------------------------------------

__global__ void k_debug_copy_x(const XSplit *__restrict__ xs, const uint32_t *__restrict__ sbase,
                               uint32_t nd, const uint64_t *__restrict__ total,
                               uint64_t *__restrict__ out_x, uint64_t cap,
                               uint64_t *__restrict__ out_off) {
  const uint64_t base = *total;
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  const uint32_t ns = sbase[nd];
  for (uint64_t j = i; j < ns; j += stride)
    if (base + j < cap) out_x[base + j] = x_join(xs[j]);
  for (uint64_t j = i; j <= nd; j += stride) out_off[j] = base + sbase[j];
}
__global__ void k_debug_add_total(uint64_t *total, const uint32_t *sbase_last) {
  *total += *sbase_last;
}

// launches the hot kernel over nht candidate tiles (tiles beyond the device-side count exit)
static int launch_minhash(const XSplit *xs, const uint32_t *sbase, const uint32_t *htb,
                          const uint32_t *htd, uint32_t nd, uint64_t nht, const uint64_t *coef_a,
                          const uint64_t *coef_b, const CoefSplit *coef_s, int K, uint32_t *csig,
                          hipStream_t st) {
  unsigned long long *stats = nullptr;
  int rc = stats_ensure(&stats);
  if (rc) return rc;
  const int F = K <= 64 ? 1 : (K <= 128 ? 2 : 4);
  const uint32_t ky = (uint32_t)((K + 64 * F - 1) / (64 * F));
  const HotConsts hc = {1u << 29, 8u};
  dim3 grid((uint32_t)nht, ky);
  ProfScope prof(SEDD_PROF_MINHASH, st);
  if (F == 1)
    hipLaunchKernelGGL(k_minhash<1>, grid, dim3(64), 0, st, xs, sbase, htb, htd, nd, coef_a,
                       coef_b, coef_s, K, csig, hc, stats + SEDD_STAT_SLOW_TILES);
  else if (F == 2)
    hipLaunchKernelGGL(k_minhash<2>, grid, dim3(64), 0, st, xs, sbase, htb, htd, nd, coef_a,
                       coef_b, coef_s, K, csig, hc, stats + SEDD_STAT_SLOW_TILES);
  else
    hipLaunchKernelGGL(k_minhash<4>, grid, dim3(64), 0, st, xs, sbase, htb, htd, nd, coef_a,
                       coef_b, coef_s, K, csig, hc, stats + SEDD_STAT_SLOW_TILES);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

// shingle_offsets (uint64, absolute) -> sbase (uint32), tile counts; x (uint64) -> split form
__global__ void k_from_x_prepare(const uint64_t *__restrict__ soff, uint32_t nd,
                                 uint32_t *__restrict__ sbase, uint32_t *__restrict__ hcnt) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i > nd) return;
  sbase[i] = (uint32_t)(soff[i] - soff[0]);
  hcnt[i] = i < nd ? (uint32_t)((soff[i + 1] - soff[i] + TS - 1) / TS) : 0u;
}
__global__ void k_from_x_split(const uint64_t *__restrict__ x, uint64_t n, XSplit *__restrict__ xs) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) xs[i] = x_split(x[i]);
}

// ---- host driver ---------------------------------------------------------------------------

struct Chunk {
  uint64_t d0, d1;
};

static int run_minhash(const uint8_t *bytes, const uint64_t *doc_offsets, uint64_t n_docs,
                       int32_t n, int32_t K, uint64_t seed, uint32_t flags, uint32_t *sig,
                       uint64_t *dbg_x, uint64_t dbg_cap, uint64_t *dbg_off, hipStream_t st) {
  const bool debug = dbg_off != nullptr;
  const int byte_mode = (flags & SEDD_FLAG_BYTE_SHINGLES) ? 1 : 0;

  // host copy of the offsets: validation and chunk planning
  void *pin = nullptr;
  int rc = pinned_ensure((n_docs + 1) * 8, &pin);
  if (rc) return rc;
  uint64_t *off = (uint64_t *)pin;
  SEDD_HIP(hipMemcpyAsync(off, doc_offsets, (n_docs + 1) * 8, hipMemcpyDeviceToHost, st));
  SEDD_HIP(hipStreamSynchronize(st));
  const uint64_t max_doc = (uint64_t(1) << 32) - (uint64_t(1) << 20);
  for (uint64_t d = 0; d < n_docs; d++) {
    if (off[d + 1] < off[d]) return SEDD_EINVAL;
    if (off[d + 1] - off[d] >= max_doc) return SEDD_EINVAL;
  }
  if (off[n_docs] > off[0] && !bytes) return SEDD_EINVAL;

  const uint64_t chunk_bytes = g_chunk_bytes_override
                                   ? g_chunk_bytes_override
                                   : (byte_mode ? (uint64_t(128) << 20) : (uint64_t(256) << 20));
  const uint64_t chunk_docs = uint64_t(1) << 22;
  std::vector<Chunk> chunks;
  uint64_t max_cv = 0, max_nd = 0;
  for (uint64_t d0 = 0; d0 < n_docs;) {
    uint64_t d1 = d0 + 1;
    while (d1 < n_docs && d1 - d0 < chunk_docs && off[d1 + 1] - off[d0] <= chunk_bytes) d1++;
    chunks.push_back({d0, d1});
    max_cv = std::max(max_cv, off[d1] - off[d0] + 16);
    max_nd = std::max(max_nd, d1 - d0);
    d0 = d1;
  }

  auto bounds = [&](uint64_t cv, uint64_t nd, uint64_t *nbt, uint64_t *nw, uint64_t *ns,
                    uint64_t *nht) {
    *nbt = nd + cv / TB + 2;
    *nw = byte_mode ? 0 : cv / 2 + nd + 2;
    *ns = byte_mode ? cv + 1 : *nw;
    *nht = nd + *ns / TS + 2;
  };
  uint64_t NBT, NW, NS, NHT;
  bounds(max_cv, max_nd, &NBT, &NW, &NS, &NHT);

  Carver cv;
  const uint64_t o_a = cv.take<uint64_t>(K), o_b = cv.take<uint64_t>(K);
  const uint64_t o_cs = cv.take<CoefSplit>(K);
  const uint64_t o_qpow = cv.take<uint64_t>(QPOW_N);
  const uint64_t o_total = cv.take<uint64_t>(1);
  const uint64_t o_dv = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_btb = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_btd = cv.take<uint32_t>(byte_mode ? 1 : NBT);
  const uint64_t o_wbase = cv.take<uint32_t>(byte_mode ? 1 : NBT + 1);
  const uint64_t o_rec = cv.take<WordRec>(byte_mode ? 1 : NW);
  const uint64_t o_docw = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_sbase = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_htb = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_htd = cv.take<uint32_t>(NHT);
  const uint64_t o_xs = cv.take<XSplit>(NS);
  const uint64_t o_tmp = cv.take<uint32_t>(scan_tmp_count(std::max(NBT + 1, max_nd + 1)));
  uint8_t *A = nullptr;
  rc = scratch_ensure(cv.off, &A);
  if (rc) return rc;
  uint64_t *coef_a = (uint64_t *)(A + o_a), *coef_b = (uint64_t *)(A + o_b);
  CoefSplit *coef_s = (CoefSplit *)(A + o_cs);
  uint64_t *qpow = (uint64_t *)(A + o_qpow), *total = (uint64_t *)(A + o_total);
  uint32_t *dv = (uint32_t *)(A + o_dv), *btb = (uint32_t *)(A + o_btb);
  uint32_t *btd = (uint32_t *)(A + o_btd), *wbase = (uint32_t *)(A + o_wbase);
  WordRec *rec = (WordRec *)(A + o_rec);
  uint32_t *docw = (uint32_t *)(A + o_docw), *sbase = (uint32_t *)(A + o_sbase);
  uint32_t *htb = (uint32_t *)(A + o_htb), *htd = (uint32_t *)(A + o_htd);
  XSplit *xs = (XSplit *)(A + o_xs);
  uint32_t *tmp = (uint32_t *)(A + o_tmp);

  {
    int nthr = std::max(K, QPOW_N);
    hipLaunchKernelGGL(k_coeffs, dim3((nthr + 255) / 256), dim3(256), 0, st, seed, (int)K, coef_a,
                       coef_b, coef_s, qpow);
    SEDD_LAUNCH_CHECK();
  }
  if (debug) {
    hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(1), 0, st, total);
    SEDD_LAUNCH_CHECK();
  } else {
    const uint64_t nsig = n_docs * (uint64_t)K;
    const uint32_t grid = (uint32_t)std::min<uint64_t>((nsig + 255) / 256, 65536);
    hipLaunchKernelGGL(k_fill_u32, dim3(grid), dim3(256), 0, st, sig, nsig, 0xFFFFFFFFu);
    SEDD_LAUNCH_CHECK();
  }

  const uint64_t align = (uint64_t)(uintptr_t)bytes & 15;
  const uint8_t *bytes16 = bytes - align;

  for (const Chunk &c : chunks) {
    const uint32_t nd = (uint32_t)(c.d1 - c.d0);
    const uint64_t origin = (align + off[c.d0]) & ~uint64_t(15);
    const uint64_t shift = align - origin;  // wraps; off[i] + shift is the aligned-frame position
    const uint8_t *pbase = bytes16 + origin;
    const uint64_t cvb = off[c.d1] - off[c.d0] + 16;
    uint64_t nbt, nw, ns, nht;
    bounds(cvb, nd, &nbt, &nw, &ns, &nht);
    const uint64_t *coff = doc_offsets + c.d0;
    const uint32_t gdoc = (nd + 1 + 255) / 256;

    {
      ProfScope prof(SEDD_PROF_WORKLIST, st);
      hipLaunchKernelGGL(k_doc_btiles, dim3(gdoc), dim3(256), 0, st, coff, shift, nd, dv, btb);
      SEDD_LAUNCH_CHECK();
      if (!byte_mode) {
        rc = scan_exclusive_u32(btb, btb, (uint64_t)nd + 1, tmp, st);
        if (rc) return rc;
        hipLaunchKernelGGL(k_fill_tile_doc, dim3(gdoc), dim3(256), 0, st, btb, nd, btd);
        SEDD_LAUNCH_CHECK();
      }
    }
    if (!byte_mode) {
      ProfScope prof(SEDD_PROF_TOKENIZE, st);
      hipLaunchKernelGGL(k_count_words, dim3((uint32_t)nbt + 1), dim3(TB_THREADS), 0, st, pbase, dv,
                         btb, btd, nd, wbase);
      SEDD_LAUNCH_CHECK();
      rc = scan_exclusive_u32(wbase, wbase, nbt + 1, tmp, st);
      if (rc) return rc;
      hipLaunchKernelGGL(k_emit_words, dim3((uint32_t)nbt), dim3(TB_THREADS), 0, st, pbase, dv, btb,
                         btd, nd, wbase, qpow, rec);
      SEDD_LAUNCH_CHECK();
    }
    {
      ProfScope prof(SEDD_PROF_WORKLIST, st);
      hipLaunchKernelGGL(k_doc_shingles, dim3(gdoc), dim3(256), 0, st, dv, btb, wbase, nd,
                         (uint32_t)n, byte_mode, docw, sbase, htb);
      SEDD_LAUNCH_CHECK();
      rc = scan_exclusive_u32(sbase, sbase, (uint64_t)nd + 1, tmp, st);
      if (rc) return rc;
      rc = scan_exclusive_u32(htb, htb, (uint64_t)nd + 1, tmp, st);
      if (rc) return rc;
      hipLaunchKernelGGL(k_fill_tile_doc, dim3(gdoc), dim3(256), 0, st, htb, nd, htd);
      SEDD_LAUNCH_CHECK();
    }
    {
      ProfScope prof(SEDD_PROF_SHINGLE_HASH, st);
      hipLaunchKernelGGL(k_shingle_hash, dim3((uint32_t)nht), dim3(256), 0, st, pbase, dv, docw,
                         rec, sbase, htb, htd, nd, (uint32_t)n, byte_mode, xs);
      SEDD_LAUNCH_CHECK();
    }
    if (debug) {
      hipLaunchKernelGGL(k_debug_copy_x, dim3(1024), dim3(256), 0, st, xs, sbase, nd, total, dbg_x,
                         dbg_cap, dbg_off + c.d0);
      SEDD_LAUNCH_CHECK();
      hipLaunchKernelGGL(k_debug_add_total, dim3(1), dim3(1), 0, st, total, sbase + nd);
      SEDD_LAUNCH_CHECK();
    } else {
      rc = launch_minhash(xs, sbase, htb, htd, nd, nht, coef_a, coef_b, coef_s, (int)K,
                          sig + c.d0 * (uint64_t)K, st);
      if (rc) return rc;
    }
  }
  return SEDD_OK;
}

}  // namespace sedd

using namespace sedd;

extern "C" {

int sedd_minhash(const uint8_t *bytes, const uint64_t *doc_offsets, uint64_t n_docs,
                 int32_t shingle_n, int32_t K, uint64_t seed, uint32_t flags, uint32_t *sig,
                 void *stream) {
  if (shingle_n < 1 || shingle_n > SEDD_MAX_SHINGLE_N || K < 1 || K > SEDD_MAX_K) return SEDD_EINVAL;
  if (flags & ~SEDD_FLAG_BYTE_SHINGLES) return SEDD_EINVAL;
  if (n_docs == 0) return SEDD_OK;
  if (!doc_offsets || !sig || n_docs >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  return run_minhash(bytes, doc_offsets, n_docs, shingle_n, K, seed, flags, sig, nullptr, 0,
                     nullptr, (hipStream_t)stream);
}

int sedd_debug_shingle_hashes(const uint8_t *bytes, const uint64_t *doc_offsets,
                              uint64_t n_docs, int32_t shingle_n, uint32_t flags, uint64_t *x,
                              uint64_t x_cap, uint64_t *shingle_offsets, void *stream) {
  if (shingle_n < 1 || shingle_n > SEDD_MAX_SHINGLE_N) return SEDD_EINVAL;
  if (flags & ~SEDD_FLAG_BYTE_SHINGLES) return SEDD_EINVAL;
  if (!shingle_offsets || (x_cap && !x)) return SEDD_EINVAL;
  if (n_docs >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  if (n_docs == 0) {
    hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(1), 0, (hipStream_t)stream, shingle_offsets);
    SEDD_LAUNCH_CHECK();
    return SEDD_OK;
  }
  if (!doc_offsets) return SEDD_EINVAL;
  return run_minhash(bytes, doc_offsets, n_docs, shingle_n, 1, 0, flags, nullptr, x, x_cap,
                     shingle_offsets, (hipStream_t)stream);
}

int sedd_debug_coeffs(uint64_t seed, int32_t K, uint64_t *a, uint64_t *b, void *stream) {
  if (K < 1 || K > SEDD_MAX_K || !a || !b) return SEDD_EINVAL;
  hipLaunchKernelGGL(k_coeffs, dim3((K + 255) / 256), dim3(256), 0, (hipStream_t)stream, seed,
                     (int)K, a, b, (CoefSplit *)nullptr, (uint64_t *)nullptr);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

int sedd_debug_minhash_from_x(const uint64_t *x, const uint64_t *shingle_offsets, uint64_t n_docs,
                              uint64_t n_shingles, int32_t K, uint64_t seed, uint32_t *sig,
                              void *stream) {
  if (K < 1 || K > SEDD_MAX_K) return SEDD_EINVAL;
  if (n_docs == 0) return SEDD_OK;
  if (!shingle_offsets || !sig || (n_shingles && !x)) return SEDD_EINVAL;
  if (n_docs >= (uint64_t(1) << 31) || n_shingles >= (uint64_t(1) << 32)) return SEDD_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const uint32_t nd = (uint32_t)n_docs;
  const uint64_t nht = n_docs + n_shingles / TS + 2;
  Carver cv;
  const uint64_t o_a = cv.take<uint64_t>(K), o_b = cv.take<uint64_t>(K);
  const uint64_t o_cs = cv.take<CoefSplit>(K);
  const uint64_t o_sbase = cv.take<uint32_t>(n_docs + 1), o_htb = cv.take<uint32_t>(n_docs + 1);
  const uint64_t o_htd = cv.take<uint32_t>(nht), o_xs = cv.take<XSplit>(n_shingles + 1);
  const uint64_t o_tmp = cv.take<uint32_t>(scan_tmp_count(n_docs + 1));
  uint8_t *A = nullptr;
  int rc = scratch_ensure(cv.off, &A);
  if (rc) return rc;
  uint64_t *coef_a = (uint64_t *)(A + o_a), *coef_b = (uint64_t *)(A + o_b);
  uint32_t *sbase = (uint32_t *)(A + o_sbase), *htb = (uint32_t *)(A + o_htb);
  uint32_t *htd = (uint32_t *)(A + o_htd), *tmp = (uint32_t *)(A + o_tmp);
  XSplit *xs = (XSplit *)(A + o_xs);
  CoefSplit *coef_s = (CoefSplit *)(A + o_cs);
  hipLaunchKernelGGL(k_coeffs, dim3((K + 255) / 256), dim3(256), 0, st, seed, (int)K, coef_a,
                     coef_b, coef_s, (uint64_t *)nullptr);
  SEDD_LAUNCH_CHECK();
  const uint64_t nsig = n_docs * (uint64_t)K;
  hipLaunchKernelGGL(k_fill_u32, dim3((uint32_t)std::min<uint64_t>((nsig + 255) / 256, 65536)),
                     dim3(256), 0, st, sig, nsig, 0xFFFFFFFFu);
  SEDD_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_from_x_prepare, dim3((nd + 1 + 255) / 256), dim3(256), 0, st,
                     shingle_offsets, nd, sbase, htb);
  SEDD_LAUNCH_CHECK();
  rc = scan_exclusive_u32(htb, htb, n_docs + 1, tmp, st);
  if (rc) return rc;
  hipLaunchKernelGGL(k_fill_tile_doc, dim3((nd + 255) / 256), dim3(256), 0, st, htb, nd, htd);
  SEDD_LAUNCH_CHECK();
  if (n_shingles) {
    hipLaunchKernelGGL(k_from_x_split, dim3((uint32_t)((n_shingles + 255) / 256)), dim3(256), 0, st,
                       x, n_shingles, xs);
    SEDD_LAUNCH_CHECK();
  }
  return launch_minhash(xs, sbase, htb, htd, nd, nht, coef_a, coef_b, coef_s, (int)K, sig, st);
}

int sedd_debug_set_chunk_bytes(uint64_t bytes) {
  g_chunk_bytes_override = bytes;
  return SEDD_OK;
}

}  // extern "C"
