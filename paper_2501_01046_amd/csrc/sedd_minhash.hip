// sedd_minhash: shingling, Eq. 1 base hash, K hash functions and per-document minimum.
// This file: the entry points, the coefficient kernels, byte shingles in both moduli, the chunk
// driver that byte shingles and the rolling-family mode share, and text in host memory.
//
// Word shingles with the affine family (the default 61-bit modulus and the paper's own prime) go
// to k_minhash_stream in sedd_minhash_stream.hip: one launch that reads the text once.  The
// kernels of the rolling-family mode are in sedd_minhash_rf.hip.
//
// Byte shingles and the rolling-family mode run per chunk of consecutive documents (all on the
// caller's stream, no host waits inside the loop):
//   1. byte tiles     each non-empty document is cut into 1 KiB tiles aligned to 16-byte
//                     addresses; a scan over per-document tile counts builds the work list.
//   2. words          (rolling family on word shingles) one wavefront per byte tile marks token
//                     starts from a 16-byte vector load per lane and counts them; after a scan a
//                     second pass writes position and length of every token.
//   3. shingle tiles  per-document shingle counts, scanned into shingle offsets and a second
//                     work list of tiles of TS shingles.
//   4. min-hash       one wavefront per shingle tile.  Phase A (lane = shingle): x(s) of Eq. 1
//                     from the tile's bytes with the reuse form of Eq. 2, into LDS.  Phase B
//                     (lane = hash function): the modular multiply-add, truncation to 32 bits
//                     and running minimum.  (Rolling family: lane = function throughout.)
#include <algorithm>
#include <vector>

#include "sedd_minhash_device.h"

namespace sedd {

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
                         uint64_t *qpow, PowSplit *ptab) {
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
      c.b = b[k];
      split[k] = c;
    }
  }
  if (qpow && k < QPOW_N) {
    const uint64_t pw = powmod(257, (uint64_t)k);
    qpow[k] = pw;
    const uint64_t P = mul257(pw);
    const uint64_t sp = ((pw << 5) & P61) | (pw >> 56);  // 32 * 257^k (a rotation, never p)
    PowSplit e;
    e.a0 = (uint32_t)P & 0x7FFFFFFFu;
    e.a0_2 = e.a0 << 1;
    e.a12 = (uint32_t)(P >> 31) << 1;
    e.pad = 0;
    e.nsp = P61 - sp;
    e.pad2 = 0;
    ptab[k] = e;
  }
}

// paper-prime coefficients a'_k = (a_k mod (p'-1)) + 1, b'_k = b_k mod p' and the token tables;
// raw (optional) receives a'_k and b'_k as 64-bit values for the stage tests
__global__ void k_coeffs_pp(uint64_t seed, int K, CoefPP *coef, PowPP *ptab, uint64_t *raw_a,
                            uint64_t *raw_b) {
  int k = blockIdx.x * blockDim.x + threadIdx.x;
  uint64_t s0 = seed % (P61 - 1) + 1;
  if (k < K) {
    const uint64_t ak = mulmod(s0, powmod(G_A, (uint64_t)k + 1));
    const uint64_t bk = mulmod(s0, powmod(G_B, (uint64_t)k + 1));
    const uint32_t a = (uint32_t)(ak % (PP - 1)) + 1, b = (uint32_t)(bk % PP);
    if (coef) {
      CoefPP c;
      c.a = a;
      c.b = b;
      c.ap = (uint32_t)((((uint64_t)a << 32) + PP - 1) / PP);  // a < p': below 2^32
      c.bp = (uint32_t)((((uint64_t)b << 32) + PP - 1) / PP);
      coef[k] = c;
    }
    if (raw_a) raw_a[k] = a;
    if (raw_b) raw_b[k] = b;
  }
  if (ptab && k < QPOW_N) {
    const uint32_t pw = powmod_pp(257u, (uint64_t)k);
    PowPP e;
    e.pw1 = mulmod_pp(pw, 257u);
    e.sp = mulmod_pp(pw, 32u);
    ptab[k] = e;
  }
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

// document owning tile t: the d with tbase[d] <= t < tbase[d+1] (documents without tiles repeat
// their neighbour's base and are skipped by the search)
__device__ __forceinline__ uint32_t tile_owner(const uint32_t *__restrict__ tbase, uint32_t nd,
                                               uint32_t t) {
  uint32_t lo = 0, hi = nd;  // invariant: tbase[lo] <= t < tbase[hi]
  while (hi - lo > 1) {
    const uint32_t mid = (lo + hi) >> 1;
    if (tbase[mid] <= t) lo = mid;
    else hi = mid;
  }
  return lo;
}

// one thread per tile (a document can own thousands of tiles)
__global__ void k_fill_btiles(const uint32_t *__restrict__ dv, const uint32_t *__restrict__ tbase,
                              uint32_t nd, uint32_t n_slots, BTile *__restrict__ tiles) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_slots || t >= tbase[nd]) return;
  const uint32_t d = tile_owner(tbase, nd, t);
  BTile bt;
  bt.vs = dv[d];
  bt.ve = dv[d + 1];
  bt.tile0 = (bt.vs & ~15u) + (t - tbase[d]) * TB;
  bt.pad = 0;
  tiles[t] = bt;
}

__global__ void k_fill_htiles(const uint32_t *__restrict__ sbase, const uint32_t *__restrict__ tbase,
                              const uint32_t *__restrict__ docw, uint32_t nd, uint32_t n,
                              uint32_t n_slots, HTile *__restrict__ tiles) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_slots || t >= tbase[nd]) return;
  const uint32_t d = tile_owner(tbase, nd, t);
  const uint32_t t0 = tbase[d], t1 = tbase[d + 1];
  const uint32_t s0 = sbase[d], S = sbase[d + 1] - s0;
  const uint32_t i0 = (t - t0) * TS;
  const uint32_t w0 = docw ? docw[d] : 0u;
  HTile ht;
  ht.doc = d;
  ht.x_off = s0 + i0;
  ht.cnt = min(TS, S - i0);
  ht.single = (t1 - t0 == 1) ? 1u : 0u;
  ht.tok0 = w0 + i0;
  ht.per = docw ? min(n, docw[d + 1] - w0) : 0u;
  ht.pad[0] = ht.pad[1] = 0;
  tiles[t] = ht;
}

// ---- tokenisation (rolling family on word shingles) -----------------------------------------

// Token starts per byte tile: one wavefront per COUNT_TILES consecutive tiles (all loads issued
// before the first is used), 16 bytes per lane, no LDS.
constexpr int COUNT_TILES = 4;
__global__ void __launch_bounds__(256)
k_count_words(const uint8_t *__restrict__ pbase, const BTile *__restrict__ tiles,
              const uint32_t *__restrict__ n_tiles, uint32_t n_slots,
              uint32_t *__restrict__ wcnt) {
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t t0 = (blockIdx.x * 4 + wave) * COUNT_TILES;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t nt = *n_tiles;
  BTile bt[COUNT_TILES];
  uint4 q[COUNT_TILES];
  uint32_t pv[COUNT_TILES];
#pragma unroll
  for (int i = 0; i < COUNT_TILES; i++) {
    bt[i].vs = bt[i].ve = bt[i].tile0 = bt[i].pad = 0;
    if (t0 + i < nt) bt[i] = tiles[t0 + i];
  }
#pragma unroll
  for (int i = 0; i < COUNT_TILES; i++) {
    q[i] = load_raw16(pbase, bt[i].tile0 + lane * 16, bt[i].vs, bt[i].ve);
    pv[i] = load_prev_byte(pbase, bt[i].tile0, bt[i].vs, bt[i].ve);
  }
#pragma unroll
  for (int i = 0; i < COUNT_TILES; i++) {
    const uint32_t t = t0 + i;
    if (t >= n_slots) break;
    const Segment sg = make_segment(q[i], bt[i].tile0 + lane * 16, bt[i].vs, bt[i].ve);
    const uint32_t starts = token_starts(lane, pv[i], sg.wm);
    const uint32_t cnt = (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_scan(__popc(starts)), 63);
    if (lane == 0) wcnt[t] = cnt;  // 0 for the slots past the tile count (they pad the scan)
  }
}

// bytes from position p0 up to the first whitespace byte or the document's end ve
__device__ __noinline__ uint32_t token_length_far(const uint8_t *__restrict__ pbase, uint32_t p0,
                                                  uint32_t ve) {
  uint32_t p = p0;
  while (p < ve && !is_ws(pbase[p])) p++;
  return p - p0;
}

// Token records of the rolling-family mode, whose functions hash the bytes themselves: position
// in the chunk frame and length of every token.  One wavefront per byte tile.
// Pass 1 (lane = 16-byte segment): the bitmap of token bytes of the tile plus LOOK bytes of
// look-ahead goes to LDS; every lane drops the positions of the tokens that start in its segment
// into LDS at their rank within the tile.
// Pass 2 (lane = token): the token's length is the run of ones in the bitmap from its position;
// consecutive lanes store consecutive records.
// (The other word-shingle modes keep no token records in memory: see k_minhash_stream.)
__global__ void __launch_bounds__(TB_LANES)
k_emit_words(const uint8_t *__restrict__ pbase, const BTile *__restrict__ tiles,
             const uint32_t *__restrict__ n_tiles, const uint32_t *__restrict__ wbase,
             TokenRecs rec) {
  __shared__ uint32_t sm_bits[TB / 32 + 4];  // token-byte bitmap: tile, look-ahead, zero pad
  __shared__ uint16_t sm_pos[MAX_TILE_TOKENS];
  const uint32_t lane = threadIdx.x;
  const uint32_t t = blockIdx.x;
  // independent loads first (the work list is allocated for the launch bound, so reading an
  // entry past the device-side count is harmless); the count decides afterwards
  const BTile bt = tiles[t];
  const uint32_t first_idx = wbase[t];
  if (t >= *n_tiles) return;
  const uint32_t vs = bt.vs, ve = bt.ve, tile0 = bt.tile0;
  const uint4 q_own = load_raw16(pbase, tile0 + lane * 16, vs, ve);
  const uint4 q_la = load_raw16(pbase, tile0 + TB, vs, ve);  // wave-uniform: scalar loads
  const uint32_t prev_byte = load_prev_byte(pbase, tile0, vs, ve);
  const Segment sg = make_segment(q_own, tile0 + lane * 16, vs, ve);
  const Segment la = make_segment(q_la, tile0 + TB, vs, ve);
  const uint32_t starts0 = token_starts(lane, prev_byte, sg.wm);

  // wave_shl:1 (lane l reads lane l + 1; the last lane gets 0)
  const uint32_t wm_up = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)sg.wm, 0x130, 0xF, 0xF, false);
  if (!(lane & 1)) sm_bits[lane >> 1] = sg.wm | (wm_up << 16);
  if (lane == 0) {
    sm_bits[TB / 32] = la.wm;
    sm_bits[TB / 32 + 1] = 0;
    sm_bits[TB / 32 + 2] = 0;
  }
  const uint32_t cnt = __popc(starts0);
  const uint32_t inc = wave_inclusive_scan(cnt);
  const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
  {
    uint32_t st = starts0, j = inc - cnt;
    while (st) {
      const uint32_t bit = __ffs(st) - 1;
      sm_pos[j++] = (uint16_t)(lane * 16 + bit);
      st &= st - 1;
    }
  }
  __syncthreads();

  // does the document end inside what the bitmap covers?
  const bool doc_ends_in_view = tile0 + TB + LOOK >= ve;
  for (uint32_t j = lane; j < tot; j += TB_LANES) {
    const uint32_t pos = sm_pos[j];
    // 64 bitmap bits from the token's first byte on
    const uint32_t dw = pos >> 5, sh = pos & 31;
    const uint32_t b0 = sm_bits[dw], b1 = sm_bits[dw + 1], b2 = sm_bits[dw + 2];
    const uint32_t w_lo = __builtin_amdgcn_alignbit(b1, b0, sh);
    const uint32_t w_hi = __builtin_amdgcn_alignbit(b2, b1, sh);
    const uint64_t zeros = ~(((uint64_t)w_hi << 32) | w_lo);
    const uint32_t run = zeros ? (uint32_t)(__ffsll((unsigned long long)zeros) - 1) : 64u;
    // the run ends at a real non-token byte (or at the document's end) inside the bitmap
    const bool seen = run <= FAST_TOKEN_MAX && (pos + run < TB + LOOK || doc_ends_in_view);
    const uint32_t len = seen ? run : token_length_far(pbase, tile0 + pos, ve);
    store_token_pos(rec, first_idx + j, tile0 + pos, len);
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

// ---- shingle hashes (Eq. 1) ----------------------------------------------------------------

// Where a tile's shingle hashes come from.
struct XSource {
  const uint8_t *pbase;   // chunk text frame (byte mode)
  const uint32_t *dv;     // document frame positions (byte mode)
  const uint32_t *sbase;  // shingle offsets per document (byte mode)
  const uint64_t *qpow;   // 257^i, i < QPOW_N
  const PowPP *ptab_pp;   // powers of 257 modulo the paper's prime, QPOW_N entries
  const uint64_t *given;  // caller-supplied hashes (debug entry), indexed like the shingle stream
  uint32_t n;             // shingle length
};
// word shingles are hashed by k_minhash_stream from its token ring (or, in the rolling-family mode,
// by k_minhash_rf_words from the bytes)
enum { X_BYTES = 1, X_GIVEN = 2 };

// x of shingle i of tile ht, 61-bit modulus: a caller-supplied value, or Horner over the window's
// bytes from the last to the first
template <int MODE>
__device__ __forceinline__ uint64_t shingle_x(const XSource &xsrc, const HTile &ht, uint32_t i) {
  static_assert(MODE == X_GIVEN || MODE == X_BYTES, "word shingles take the streaming kernel");
  if (MODE == X_GIVEN) return xsrc.given[ht.x_off + i];
  const uint32_t d = ht.doc;
  const uint32_t vs = xsrc.dv[d], len = xsrc.dv[d + 1] - vs;
  const uint32_t per = min(len, xsrc.n);
  const uint8_t *p = xsrc.pbase + vs + (ht.x_off - xsrc.sbase[d]) + i;
  uint64_t acc = 0;
  for (uint32_t j = per; j-- > 0;) acc = horner257_lazy(acc, p[j]);
  return fold61(acc);
}

// ---- the hot kernel ------------------------------------------------------------------------
//
// One wavefront per shingle tile (up to TS shingles of one document).
//
// Phase A: the 64 lanes compute the tile's Eq. 1 hashes (lane = shingle) into LDS in limb form.
// Phase B: lane l evaluates hash functions k0+l, k0+64+l, ... (F of them) over the tile; the
// shingle limbs are read from LDS at a wave-uniform address (a broadcast).  Per (shingle,
// function) the kernel needs h = ((a x + b) mod p) mod 2^32 with p = 2^61-1.
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

template <int F, int P, int MODE>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(8, 8)))
k_minhash(XSource xsrc, const HTile *__restrict__ tiles, const uint32_t *__restrict__ n_tiles,
          const uint64_t *__restrict__ coef_a, const CoefSplit *__restrict__ coef_split, int K,
          uint32_t *__restrict__ sig /* first document of the chunk */, HotConsts hc,
          unsigned long long *__restrict__ slow_tiles) {
  __shared__ XLimbs sx[TS];
  const uint32_t t = blockIdx.x;
  const HTile ht = tiles[t];  // the list is allocated for the launch bound: safe past the count
  if (t >= *n_tiles) return;
  const uint32_t d = ht.doc, cnt = ht.cnt;

  if (MODE == X_BYTES) {
    // Byte windows.  The tile's bytes are staged in LDS; lane l owns the WPL = TS / 64 windows
    // from WPL l on: it evaluates the last of them by Horner over its bytes and derives the others with the reuse
    // form of Eq. 1 (Eq. 2 read backwards, so that the step multiplies by q instead of dividing):
    //   x(i-1) = q (x(i) - c[i+per-1] q^(per-1)) + c[i-1]      (mod p).
    // The windows of row j = i mod WPL are stored from slot off_j on, consecutive lanes in
    // consecutive slots; the slots [0, cnt) then hold every window once, in an order that does
    // not matter to a minimum.
    __shared__ uint32_t sm_b[MODE == X_BYTES ? (TS + SEDD_MAX_SHINGLE_N + 8) / 4 + 1 : 1];
    const uint32_t vs = xsrc.dv[d], dlen = xsrc.dv[d + 1] - vs;
    const uint32_t per = min(dlen, xsrc.n);
    const uint32_t b0 = vs + (ht.x_off - xsrc.sbase[d]);  // frame position of the first window
    const uint32_t o = b0 & 3u;
    const uint32_t ndw = (o + cnt + per - 1 + 3) >> 2;    // aligned words that hold >= 1 byte of it
    for (uint32_t w = threadIdx.x; w < ndw; w += 64)
      sm_b[w] = *reinterpret_cast<const uint32_t *>(xsrc.pbase + (b0 - o) + 4 * w);
    __syncthreads();
    const uint8_t *tb = reinterpret_cast<const uint8_t *>(sm_b) + o;  // tb[i] = byte i of the tile
    const uint32_t l = threadIdx.x;
    constexpr uint32_t WPL = TS / 64;
    static_assert(TS % 64 == 0, "whole windows per lane");
    if (WPL * l < cnt) {
      const uint32_t m = min(WPL, cnt - WPL * l);
      const uint32_t top = WPL * l + m - 1;
      uint64_t acc = 0;
      for (uint32_t j = per; j-- > 0;) acc = horner257_lazy(acc, tb[top + j]);
      const uint64_t Q = xsrc.qpow[per - 1];  // per <= SEDD_MAX_SHINGLE_N < QPOW_N
      const uint32_t q_lo = (uint32_t)Q, q_hi = (uint32_t)(Q >> 32);
      for (uint32_t i = top;; i--) {
        const uint32_t j = i - WPL * l;
        uint32_t slot = l;  // off_j + l, off_j = sum over rows before j of ceil((cnt - row) / WPL)
        for (uint32_t row = 0; row < j; row++) slot += (cnt - row + WPL - 1) / WPL;
        sx[slot] = x_limbs(fold61(acc));
        if (i == WPL * l) break;
        // x(i-1) from x(i)
        const uint32_t c_hi = tb[i + per - 1], c_lo = tb[i - 1];
        const uint64_t lo = (uint64_t)q_lo * c_hi;
        const uint64_t hi = (uint64_t)q_hi * c_hi + (lo >> 32);
        const uint64_t tq = (((hi & 0x1FFFFFFFull) << 32) | (uint32_t)lo) + (hi >> 29);  // c_hi Q
        uint64_t dd = acc + (2 * P61 - tq);  // below 2^63
        dd = (dd & P61) + (dd >> 61);
        acc = horner257_lazy(dd, c_lo);
      }
    }
  } else {
    for (uint32_t i = threadIdx.x; i < cnt; i += 64) sx[i] = x_limbs(shingle_x<MODE>(xsrc, ht, i));
  }

  // P = 2: the two half-waves take alternate shingles and each lane evaluates F functions of
  // the 32*F this block covers (one LDS instruction then serves two shingles)
  constexpr int LW = 64 / P;
  const uint32_t grp = threadIdx.x / LW;
  const int kbase = blockIdx.y * (LW * F) + (threadIdx.x % LW);
  uint64_t b[F];
  uint32_t a0[F], a12[F], m[F];
#pragma unroll
  for (int j = 0; j < F; j++) {
    int k = kbase + LW * j;
    const int kk = k < K ? k : 0;  // lanes past K compute function 0 and store nothing
    const CoefSplit c = coef_split[kk];
    a0[j] = c.a0;
    a12[j] = c.a12;
    b[j] = c.b;
    m[j] = 0xFFFFFFFFu;
  }
  __syncthreads();

  uint32_t amb = 0;
  auto eval = [&](const XLimbs &xv) {
#pragma unroll
    for (int j = 0; j < F; j++) {
      uint64_t N = (uint64_t)a0[j] * xv.x1_4;
      N += (uint64_t)a12[j] * xv.x0_2;
      uint64_t U = (uint64_t)a12[j] * xv.x1 + b[j];
      U += (uint64_t)a0[j] * xv.x0;
      const uint64_t Sv = (uint64_t)(uint32_t)N * hc.two29 + U;
      const uint64_t W = (uint64_t)(uint32_t)(Sv >> 32) * hc.eight;  // hi: S >> 61, lo: bits 32..60
      const uint32_t h = (uint32_t)Sv + (uint32_t)(N >> 32) + (uint32_t)(W >> 32);
      amb = max(amb, (uint32_t)W);
      m[j] = min(m[j], h);
    }
  };
  const XLimbs *sxg = sx + grp;  // this half-wave's first shingle
  const uint32_t steps = cnt / P;
#pragma unroll(F >= 4 ? 2 : 4)
  for (uint32_t s = 0; s < steps; s++) eval(sxg[s * P]);
  if (P == 2 && (cnt & 1)) eval(sx[cnt - 1]);  // both halves: a repeat cannot change a minimum
  if (__any(amb >= 0xFFFFFFF0u)) {
    // rare: some evaluation sat within reach of a carry across bit 61; redo the tile exactly
    if (threadIdx.x == 0 && blockIdx.y == 0) atomicAdd(slow_tiles, 1ull);
#pragma unroll
    for (int j = 0; j < F; j++) m[j] = 0xFFFFFFFFu;
    uint64_t a[F];
#pragma unroll
    for (int j = 0; j < F; j++) a[j] = coef_a[kbase + LW * j < K ? kbase + LW * j : 0];
    for (uint32_t s = grp; s < cnt; s += P) {
      const XLimbs xv = sx[s];
      const uint64_t x = ((uint64_t)xv.x1 << 31) | xv.x0;
#pragma unroll
      for (int j = 0; j < F; j++) m[j] = min(m[j], (uint32_t)addmod(mulmod(a[j], x), b[j]));
    }
  }
  if (P == 2) {
#pragma unroll
    for (int j = 0; j < F; j++) m[j] = min(m[j], (uint32_t)__shfl_xor(m[j], 32, 64));
  }
  uint32_t *out = sig + (uint64_t)d * K;
#pragma unroll
  for (int j = 0; j < F; j++) {
    int k = kbase + LW * j;
    if (grp == 0 && k < K) {
      if (ht.single) {
        out[k] = m[j];
      } else {
        // values only ever decrease, so a (possibly stale) read that is not above m[j] settles
        // it without an atomic; a long document's tiles would otherwise queue on 4 cache lines
        const uint32_t cur = __hip_atomic_load(out + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (m[j] < cur) atomicMin(out + k, m[j]);
      }
    }
  }
}

// ---- the hot kernel of the paper-prime mode (byte shingles and caller-supplied hashes) ---------
//
// Same tiling as k_minhash: one wavefront per shingle tile, phase A fills LDS with the tile's
// x'(s) = Eq. 1 mod p', phase B evaluates h'_k(s) = (a'_k x' + b'_k) mod p' for the lane's
// functions over the tile.  (Word shingles: ArithPP in k_minhash_stream runs the same phase B.)
// Per (shingle, function):
//   q = (x ap + bp) >> 32            one 32x32+64 multiply-add; ap, bp are rounded up, so q is
//                                    the quotient of a x + b by p', or (rarely) one more
//   s = (a x + b) - q p'             low 32 bits, two 24-bit multiply-adds (a, x, q, p' < 2^24)
//   m = min(m, s)                    unsigned
// x ap + bp exceeds 2^32 (a x + b) / p' by less than x + 2, i.e. the quotient estimate by less
// than (p' + 1) / 2^32: q is one too large only if the remainder is within PP_EDGE of p'.  Then
// s = h' - p' wraps to a huge unsigned value and the minimum ignores it.  So a tile minimum
// below p' - PP_EDGE is exact (everything ignored was larger); a lane whose minimum is not
// redoes its functions over the tile with the plain reduction.  That happens with probability
// (PP_EDGE / p')^count per function: in practice only for tiles of one or two shingles, where
// the second pass costs next to nothing.  4 instructions per evaluation.

// x' of shingle i of tile ht
template <int MODE>
__device__ __forceinline__ uint32_t shingle_x_pp(const XSource &xsrc, const HTile &ht, uint32_t i) {
  static_assert(MODE == X_GIVEN || MODE == X_BYTES, "word shingles take the streaming kernel");
  if (MODE == X_GIVEN) return (uint32_t)(xsrc.given[ht.x_off + i] % PP);
  const uint32_t d = ht.doc;
  const uint32_t vs = xsrc.dv[d], len = xsrc.dv[d + 1] - vs;
  const uint32_t per = min(len, xsrc.n);
  const uint8_t *p = xsrc.pbase + vs + (ht.x_off - xsrc.sbase[d]) + i;
  uint32_t acc = 0;
  for (uint32_t j = per; j-- > 0;) acc = red_pp((uint64_t)acc * 257u + p[j]);
  return acc;
}

template <int F, int P, int MODE>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(8, 8)))
k_minhash_pp(XSource xsrc, const HTile *__restrict__ tiles, const uint32_t *__restrict__ n_tiles,
             const CoefPP *__restrict__ coef, int K,
             uint32_t *__restrict__ sig /* first document of the chunk */) {
  // half-wave g reads row g: shingle i sits at sx[i % P][i / P]; rows are padded with repeats of
  // shingle 0 (a repeat cannot change a minimum) to a common multiple of 4 entries
  constexpr uint32_t ROW = TS / P + 8;
  __shared__ __attribute__((aligned(16))) uint32_t sx[P][ROW];
  const uint32_t t = blockIdx.x;
  const HTile ht = tiles[t];  // the list is allocated for the launch bound: safe past the count
  if (t >= *n_tiles) return;
  const uint32_t d = ht.doc, cnt = ht.cnt;

  if (MODE == X_BYTES) {
    // the tile's bytes are staged in LDS; lane l owns the WPL windows from WPL l on: the last
    // of them by Horner over its bytes, the others by the reuse form of Eq. 1 (Eq. 2 read
    // backwards):  x(i-1) = q (x(i) - c[i+per-1] q^(per-1)) + c[i-1]   (mod p')
    __shared__ uint32_t sm_b[MODE == X_BYTES ? (TS + SEDD_MAX_SHINGLE_N + 8) / 4 + 1 : 1];
    const uint32_t vs = xsrc.dv[d], dlen = xsrc.dv[d + 1] - vs;
    const uint32_t per = min(dlen, xsrc.n);
    const uint32_t b0 = vs + (ht.x_off - xsrc.sbase[d]);  // frame position of the first window
    const uint32_t o = b0 & 3u;
    const uint32_t ndw = (o + cnt + per - 1 + 3) >> 2;    // aligned words that hold >= 1 byte of it
    for (uint32_t w = threadIdx.x; w < ndw; w += 64)
      sm_b[w] = *reinterpret_cast<const uint32_t *>(xsrc.pbase + (b0 - o) + 4 * w);
    __syncthreads();
    const uint8_t *tb = reinterpret_cast<const uint8_t *>(sm_b) + o;  // tb[i] = byte i of the tile
    const uint32_t l = threadIdx.x;
    constexpr uint32_t WPL = TS / 64;
    if (WPL * l < cnt) {
      const uint32_t m = min(WPL, cnt - WPL * l);
      const uint32_t top = WPL * l + m - 1;
      uint32_t acc = 0;
      for (uint32_t j = per; j-- > 0;) acc = red_pp((uint64_t)acc * 257u + tb[top + j]);
      // 257^(per-1) = pw1 of length per - 2; per = 1 needs 257^0 = 1
      const uint32_t qn = per >= 2 ? xsrc.ptab_pp[per - 2].pw1 : 1u;
      const uint32_t neg_qn = PP - qn;  // in [1, p')
      for (uint32_t i = top;; i--) {
        sx[i % P][i / P] = acc;
        if (i == WPL * l) break;
        const uint32_t c_hi = tb[i + per - 1], c_lo = tb[i - 1];
        const uint32_t dd = red_pp((uint64_t)c_hi * neg_qn + acc);  // x(i) - c_hi q^(per-1)
        acc = red_pp((uint64_t)dd * 257u + c_lo);
      }
    }
  } else {
    for (uint32_t i = threadIdx.x; i < cnt; i += 64) sx[i % P][i / P] = shingle_x_pp<MODE>(xsrc, ht, i);
  }
  __syncthreads();
  // pad every row to R entries, R = the longest row rounded up to a multiple of 4
  const uint32_t cnt0 = (cnt + P - 1) / P, R = (cnt0 + 3) & ~3u;
  if (threadIdx.x < 8 * P) {
    const uint32_t row = threadIdx.x / 8, j = threadIdx.x % 8;
    const uint32_t have = (cnt + P - 1 - row) / P;  // entries of this row
    if (have + j < R) sx[row][have + j] = sx[0][0];
  }

  constexpr int LW = 64 / P;
  const uint32_t grp = threadIdx.x / LW;
  const int kbase = blockIdx.y * (LW * F) + (threadIdx.x % LW);
  uint32_t a[F], b[F], ap[F], m[F];
  uint64_t bp[F];
#pragma unroll
  for (int j = 0; j < F; j++) {
    int k = kbase + LW * j;
    const int kk = k < K ? k : 0;  // lanes past K compute function 0 and store nothing
    const uint4 c = *reinterpret_cast<const uint4 *>(coef + kk);
    a[j] = c.x;
    b[j] = c.y;
    ap[j] = c.z;
    bp[j] = c.w;
    m[j] = 0xFFFFFFFFu;
  }
  __syncthreads();

  const int neg_p = -(int)PP;
  auto eval = [&](uint32_t x) {
#pragma unroll
    for (int j = 0; j < F; j++) {
      const uint32_t q = (uint32_t)(((uint64_t)x * ap[j] + bp[j]) >> 32);
      // the two 24-bit multiply-adds, spelled out: the compiler would otherwise emit two
      // multiplies and a three-operand addition
      uint32_t sv;
      asm("v_mad_u32_u24 %0, %2, %3, %4\n\tv_mad_i32_i24 %0, %1, %5, %0"
          : "=&v"(sv)
          : "v"(q), "v"(a[j]), "v"(x), "v"(b[j]), "s"(neg_p));
      m[j] = min(m[j], sv);
    }
  };
  const uint4 *row = reinterpret_cast<const uint4 *>(&sx[grp][0]);
  const uint32_t steps = R / 4;
#pragma unroll 2
  for (uint32_t s4 = 0; s4 < steps; s4++) {
    const uint4 xv = row[s4];
    eval(xv.x);
    eval(xv.y);
    eval(xv.z);
    eval(xv.w);
  }
  bool redo = false;
#pragma unroll
  for (int j = 0; j < F; j++) redo |= m[j] >= PP - PP_EDGE;
  if (__any(redo)) {
    // rare (see above): the plain reduction over this half-wave's row
#pragma unroll
    for (int j = 0; j < F; j++) m[j] = 0xFFFFFFFFu;
    for (uint32_t i = 0; i < R; i++) {
      const uint32_t x = sx[grp][i];
#pragma unroll
      for (int j = 0; j < F; j++) m[j] = min(m[j], red_pp((uint64_t)a[j] * x + b[j]));
    }
  }
  if (P == 2) {
#pragma unroll
    for (int j = 0; j < F; j++) m[j] = min(m[j], (uint32_t)__shfl_xor(m[j], 32, 64));
  }
  uint32_t *out = sig + (uint64_t)d * K;
#pragma unroll
  for (int j = 0; j < F; j++) {
    int k = kbase + LW * j;
    if (grp == 0 && k < K) {
      if (ht.single) {
        out[k] = m[j];
      } else {
        const uint32_t cur = __hip_atomic_load(out + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (m[j] < cur) atomicMin(out + k, m[j]);
      }
    }
  }
}

// ---- stage-level output of the shingle hashes (debug entry) ----------------------------------

template <int MODE, bool PAPER>
__global__ void __launch_bounds__(64)
k_debug_write_x(XSource xsrc, const HTile *__restrict__ tiles,
                const uint32_t *__restrict__ n_tiles, const uint64_t *__restrict__ total,
                uint64_t *__restrict__ out_x, uint64_t cap) {
  const uint32_t t = blockIdx.x;
  if (t >= *n_tiles) return;
  const HTile ht = tiles[t];
  const uint64_t base = *total + ht.x_off;
  for (uint32_t i = threadIdx.x; i < ht.cnt; i += 64) {
    uint64_t x;
    if constexpr (PAPER) x = shingle_x_pp<MODE>(xsrc, ht, i);
    else x = shingle_x<MODE>(xsrc, ht, i);
    if (base + i < cap) out_x[base + i] = x;
  }
}
__global__ void k_debug_write_offsets(const uint32_t *__restrict__ sbase, uint32_t nd,
                                      const uint64_t *__restrict__ total,
                                      uint64_t *__restrict__ out_off) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i <= nd) out_off[i] = *total + sbase[i];
}
__global__ void k_debug_add_total(uint64_t *total, const uint32_t *sbase_last) {
  *total += *sbase_last;
}

// launches the hot kernel over nht candidate tiles (tiles beyond the device-side count exit)
static int launch_minhash(int mode, const XSource &xsrc, const HTile *tiles,
                          const uint32_t *n_tiles, uint64_t nht, const uint64_t *coef_a,
                          const CoefSplit *coef_s, const CoefPP *coef_pp, int K, uint32_t *csig,
                          hipStream_t st) {
  unsigned long long *stats = nullptr;
  int rc = stats_ensure(&stats);
  if (rc) return rc;
  // functions per lane F and half-wave split P: K <= 32: (1,2), <= 64: (2,2), <= 128: (4,2),
  // larger: (4,1) with one grid row per 256 functions
  const int P = K <= 128 ? 2 : 1;
  const int F = K <= 32 ? 1 : (K <= 64 ? 2 : 4);
  const int per_block = (64 / P) * F;
  const uint32_t ky = (uint32_t)((K + per_block - 1) / per_block);
  const HotConsts hc = {1u << 29, 8u, 1u};
  dim3 grid((uint32_t)nht, ky);
  ProfScope prof(SEDD_PROF_MINHASH, st);
#define SEDD_LAUNCH_PP(FF, HW, MM)                                                         \
  hipLaunchKernelGGL((k_minhash_pp<FF, HW, MM>), grid, dim3(64), 0, st, xsrc, tiles, n_tiles, \
                     coef_pp, K, csig)
#define SEDD_LAUNCH_61(FF, HW, MM)                                                          \
  hipLaunchKernelGGL((k_minhash<FF, HW, MM>), grid, dim3(64), 0, st, xsrc, tiles, n_tiles,  \
                     coef_a, coef_s, K, csig, hc, stats + SEDD_STAT_SLOW_TILES)
#define SEDD_LAUNCH_MH_F(LAUNCH, MM)           \
  do {                                         \
    if (P == 1) LAUNCH(4, 1, MM);              \
    else if (F == 1) LAUNCH(1, 2, MM);         \
    else if (F == 2) LAUNCH(2, 2, MM);         \
    else LAUNCH(4, 2, MM);                     \
  } while (0)
  if (mode != X_BYTES && mode != X_GIVEN) return SEDD_EINVAL;  // word shingles: k_minhash_stream
  if (coef_pp) {
    if (mode == X_BYTES) SEDD_LAUNCH_MH_F(SEDD_LAUNCH_PP, X_BYTES);
    else SEDD_LAUNCH_MH_F(SEDD_LAUNCH_PP, X_GIVEN);
  } else {
    if (mode == X_BYTES) SEDD_LAUNCH_MH_F(SEDD_LAUNCH_61, X_BYTES);
    else SEDD_LAUNCH_MH_F(SEDD_LAUNCH_61, X_GIVEN);
  }
#undef SEDD_LAUNCH_MH_F
#undef SEDD_LAUNCH_61
#undef SEDD_LAUNCH_PP
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

// shingle_offsets (uint64) -> sbase (uint32, same values) and tile counts
__global__ void k_from_x_prepare(const uint64_t *__restrict__ soff, uint32_t nd,
                                 uint32_t *__restrict__ sbase, uint32_t *__restrict__ hcnt) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i > nd) return;
  sbase[i] = (uint32_t)soff[i];
  hcnt[i] = i < nd ? (uint32_t)((soff[i + 1] - soff[i] + TS - 1) / TS) : 0u;
}

// ---- chunk planning on the device ------------------------------------------------------------
//
// The host never reads the offsets array: two tiny kernels give it the first and last offset,
// a validity flag, and the chunk boundaries (document index and byte offset at every multiple of
// the chunk size in bytes and of the chunk size in documents).

struct PlanEntry {
  uint64_t doc;
  uint64_t off;
};

__global__ void k_plan_probe(const uint64_t *__restrict__ off, uint64_t n, uint64_t *__restrict__ out) {
  out[0] = off[0];
  out[1] = off[n];
}

// entries [0, n_byte): first document whose offset is >= first + k * chunk_bytes;
// entries [n_byte, n_byte + n_cnt): document (j + 1) * chunk_docs
__global__ void k_plan(const uint64_t *__restrict__ off, uint64_t n, uint64_t first,
                       uint64_t chunk_bytes, uint64_t n_byte, uint64_t chunk_docs, uint64_t n_cnt,
                       PlanEntry *__restrict__ out) {
  const uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n_byte + n_cnt) return;
  uint64_t d;
  if (k < n_byte) {
    const uint64_t target = first + k * chunk_bytes;
    uint64_t lo = 0, hi = n;  // smallest d in [0, n] with off[d] >= target (n if none)
    while (lo < hi) {
      const uint64_t mid = (lo + hi) >> 1;
      if (off[mid] >= target) hi = mid;
      else lo = mid + 1;
    }
    d = lo;
  } else {
    d = (k - n_byte + 1) * chunk_docs;
  }
  out[k].doc = d;
  out[k].off = off[d];
}

__global__ void k_validate_offsets(const uint64_t *__restrict__ off, uint64_t n, uint64_t max_doc,
                                   uint32_t *__restrict__ bad) {
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint64_t a = off[i], b = off[i + 1];
  if (b < a || b - a >= max_doc) *bad = 1u;  // every writer stores the same value
}

__global__ void k_zero_u32(uint32_t *p) { *p = 0; }

// ---- host driver ---------------------------------------------------------------------------

struct Chunk {
  uint64_t d0, d1;  // documents [d0, d1)
  uint64_t o0, o1;  // their byte range
};

static int run_minhash(const uint8_t *bytes, uint64_t n_bytes, const uint64_t *doc_offsets,
                       uint64_t n_docs, int32_t n, int32_t K, uint64_t seed, uint32_t flags,
                       uint32_t *sig, uint64_t *dbg_x, uint64_t dbg_cap, uint64_t *dbg_off,
                       hipStream_t st) {
  const bool debug = dbg_off != nullptr;
  const int byte_mode = (flags & SEDD_FLAG_BYTE_SHINGLES) ? 1 : 0;
  const bool paper = (flags & SEDD_FLAG_PAPER_PRIME) != 0;
  const bool rolling = (flags & SEDD_FLAG_ROLLING_FAMILY) != 0;
  if (!byte_mode && !rolling)
    return run_minhash_stream(bytes, n_bytes, doc_offsets, n_docs, n, K, seed, paper, sig, dbg_x,
                              dbg_cap, dbg_off, st);

  // validation and chunk planning on the device; the host sees a handful of numbers
  const uint64_t chunk_bytes =
      g_chunk_bytes_override ? std::min<uint64_t>(g_chunk_bytes_override, uint64_t(1) << 30)
                             : (byte_mode ? (uint64_t(1) << 30) : (uint64_t(256) << 20));
  const uint64_t chunk_docs = uint64_t(1) << 22;
  // chunk positions are 32-bit: a chunk is at most chunk_bytes (<= 2^30) plus one document
  const uint64_t max_doc = (uint64_t(1) << 32) - (uint64_t(1) << 30) - (uint64_t(1) << 16);
  const uint64_t plan_cap = uint64_t(1) << 20;  // boundaries per call
  int rc;
  uint64_t h_probe[2];
  std::vector<PlanEntry> bnd;
  {
    void *pin = nullptr;
    rc = pinned_ensure((plan_cap + 16) * sizeof(PlanEntry), &pin);
    if (rc) return rc;
    uint8_t *A0 = nullptr;
    rc = scratch_ensure((plan_cap + 16) * sizeof(PlanEntry) + 512, &A0);
    if (rc) return rc;
    uint64_t *d_probe = (uint64_t *)A0;
    uint32_t *d_bad = (uint32_t *)(A0 + 64);
    PlanEntry *d_plan = (PlanEntry *)(A0 + 256);
    hipLaunchKernelGGL(k_plan_probe, dim3(1), dim3(1), 0, st, doc_offsets, n_docs, d_probe);
    SEDD_LAUNCH_CHECK();
    SEDD_HIP(hipMemcpyAsync(pin, d_probe, 16, hipMemcpyDeviceToHost, st));
    SEDD_HIP(hipStreamSynchronize(st));
    h_probe[0] = ((uint64_t *)pin)[0];
    h_probe[1] = ((uint64_t *)pin)[1];
    if (h_probe[1] < h_probe[0] || h_probe[1] > n_bytes) return SEDD_EINVAL;
    if (h_probe[1] > h_probe[0] && !bytes) return SEDD_EINVAL;
    const uint64_t total = h_probe[1] - h_probe[0];
    const uint64_t n_byte = total / chunk_bytes + 1, n_cnt = (n_docs - 1) / chunk_docs;
    if (n_byte + n_cnt > plan_cap) return SEDD_EINVAL;
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(1), 0, st, d_bad);
    SEDD_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_validate_offsets, dim3((uint32_t)((n_docs + 255) / 256)), dim3(256), 0, st,
                       doc_offsets, n_docs, max_doc, d_bad);
    SEDD_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_plan, dim3((uint32_t)((n_byte + n_cnt + 255) / 256)), dim3(256), 0, st,
                       doc_offsets, n_docs, h_probe[0], chunk_bytes, n_byte, chunk_docs, n_cnt,
                       d_plan);
    SEDD_LAUNCH_CHECK();
    uint8_t *hp = (uint8_t *)pin;
    SEDD_HIP(hipMemcpyAsync(hp, d_bad, 4, hipMemcpyDeviceToHost, st));
    SEDD_HIP(hipMemcpyAsync(hp + 64, d_plan, (n_byte + n_cnt) * sizeof(PlanEntry),
                            hipMemcpyDeviceToHost, st));
    SEDD_HIP(hipStreamSynchronize(st));
    if (*(uint32_t *)hp) return SEDD_EINVAL;
    const PlanEntry *hpl = (const PlanEntry *)(hp + 64);
    bnd.assign(hpl, hpl + n_byte + n_cnt);
    bnd.push_back({n_docs, h_probe[1]});
    std::sort(bnd.begin(), bnd.end(),
              [](const PlanEntry &x, const PlanEntry &y) { return x.doc < y.doc; });
  }
  std::vector<Chunk> chunks;
  uint64_t max_cv = 0, max_nd = 0;
  {
    uint64_t d0 = 0, o0 = h_probe[0];
    for (const PlanEntry &e : bnd) {
      if (e.doc <= d0) continue;
      chunks.push_back({d0, e.doc, o0, e.off});
      max_cv = std::max(max_cv, e.off - o0 + 16);
      max_nd = std::max(max_nd, e.doc - d0);
      d0 = e.doc;
      o0 = e.off;
    }
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
  const uint64_t o_ptab = cv.take<PowSplit>(QPOW_N);
  const uint64_t o_cpp = cv.take<CoefPP>(K);
  const uint64_t o_ptpp = cv.take<PowPP>(QPOW_N);
  const uint64_t o_rfq = cv.take<uint64_t>(rolling ? K : 1);
  const uint64_t o_rfp = cv.take<uint64_t>(rolling ? (uint64_t)(RF_POW_MAX + 1) * K : 1);
  const uint64_t o_total = cv.take<uint64_t>(1);
  const uint64_t o_dv = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_btb = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_btd = cv.take<BTile>(byte_mode ? 1 : NBT);
  const uint64_t o_wbase = cv.take<uint32_t>(byte_mode ? 1 : NBT + 1);
  const uint64_t o_tv = cv.take<uint32_t>(byte_mode ? 1 : NW);
  const uint64_t o_tl = cv.take<uint8_t>(byte_mode ? 1 : NW);
  const uint64_t o_tx = cv.take<uint32_t>(byte_mode ? 1 : NW);
  const uint64_t o_docw = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_sbase = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_htb = cv.take<uint32_t>(max_nd + 1);
  const uint64_t o_htd = cv.take<HTile>(NHT);
  const uint64_t o_tmp = cv.take<uint32_t>(scan_tmp_count(std::max(NBT + 1, max_nd + 1)));
  uint8_t *A = nullptr;
  rc = scratch_ensure(cv.off, &A);
  if (rc) return rc;
  uint64_t *coef_a = (uint64_t *)(A + o_a), *coef_b = (uint64_t *)(A + o_b);
  CoefSplit *coef_s = (CoefSplit *)(A + o_cs);
  uint64_t *qpow = (uint64_t *)(A + o_qpow), *total = (uint64_t *)(A + o_total);
  PowSplit *ptab = (PowSplit *)(A + o_ptab);
  CoefPP *coef_pp = (CoefPP *)(A + o_cpp);
  PowPP *ptab_pp = (PowPP *)(A + o_ptpp);
  uint64_t *rf_q = (uint64_t *)(A + o_rfq), *rf_pw = (uint64_t *)(A + o_rfp);
  uint32_t *dv = (uint32_t *)(A + o_dv), *btb = (uint32_t *)(A + o_btb);
  BTile *btd = (BTile *)(A + o_btd);
  uint32_t *wbase = (uint32_t *)(A + o_wbase);
  TokenRecs rec;
  rec.pos = (uint32_t *)(A + o_tv);
  rec.len = (uint8_t *)(A + o_tl);
  rec.long_len = (uint32_t *)(A + o_tx);
  uint32_t *docw = (uint32_t *)(A + o_docw), *sbase = (uint32_t *)(A + o_sbase);
  uint32_t *htb = (uint32_t *)(A + o_htb);
  HTile *htd = (HTile *)(A + o_htd);
  uint32_t *tmp = (uint32_t *)(A + o_tmp);
  XSource xsrc;
  xsrc.dv = dv;
  xsrc.sbase = sbase;
  xsrc.qpow = qpow;
  xsrc.ptab_pp = ptab_pp;
  xsrc.given = nullptr;
  xsrc.n = (uint32_t)n;

  {
    int nthr = std::max(K, QPOW_N);
    if (paper)
      hipLaunchKernelGGL(k_coeffs_pp, dim3((nthr + 255) / 256), dim3(256), 0, st, seed, (int)K,
                         coef_pp, ptab_pp, (uint64_t *)nullptr, (uint64_t *)nullptr);
    else if (rolling)
      hipLaunchKernelGGL(k_coeffs_rf, dim3((nthr + 255) / 256), dim3(256), 0, st, seed, (int)K, rf_q,
                         rf_pw);
    else
      hipLaunchKernelGGL(k_coeffs, dim3((nthr + 255) / 256), dim3(256), 0, st, seed, (int)K, coef_a,
                         coef_b, coef_s, qpow, ptab);
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
    const uint64_t origin = (align + c.o0) & ~uint64_t(15);
    const uint64_t shift = align - origin;  // wraps; off[i] + shift is the aligned-frame position
    const uint8_t *pbase = bytes16 + origin;
    const uint64_t cvb = c.o1 - c.o0 + 16;
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
        hipLaunchKernelGGL(k_fill_btiles, dim3((uint32_t)((nbt + 255) / 256)), dim3(256), 0, st, dv,
                           btb, nd, (uint32_t)nbt, btd);
        SEDD_LAUNCH_CHECK();
      }
    }
    if (!byte_mode) {
      ProfScope prof(SEDD_PROF_TOKENIZE, st);
      hipLaunchKernelGGL(k_count_words,
                         dim3((uint32_t)((nbt + 1 + 4 * COUNT_TILES - 1) / (4 * COUNT_TILES))),
                         dim3(256), 0, st,
                         pbase, btd, btb + nd, (uint32_t)(nbt + 1), wbase);
      SEDD_LAUNCH_CHECK();
      rc = scan_exclusive_u32(wbase, wbase, nbt + 1, tmp, st);
      if (rc) return rc;
      hipLaunchKernelGGL(k_emit_words, dim3((uint32_t)nbt), dim3(TB_LANES), 0, st, pbase, btd,
                         btb + nd, wbase, rec);
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
      hipLaunchKernelGGL(k_fill_htiles, dim3((uint32_t)((nht + 255) / 256)), dim3(256), 0, st, sbase,
                         htb, byte_mode ? (const uint32_t *)nullptr : docw, nd, (uint32_t)n,
                         (uint32_t)nht, htd);
      SEDD_LAUNCH_CHECK();
    }
    xsrc.pbase = pbase;
    if (debug) {
#define SEDD_LAUNCH_DBG(MM, PAPER)                                                              \
  hipLaunchKernelGGL((k_debug_write_x<MM, PAPER>), dim3((uint32_t)nht), dim3(64), 0, st, xsrc, \
                     htd, htb + nd, total, dbg_x, dbg_cap)
      if (!byte_mode) return SEDD_EINVAL;  // word shingles: the debug passes of k_minhash_stream
      if (paper) SEDD_LAUNCH_DBG(X_BYTES, true);
      else SEDD_LAUNCH_DBG(X_BYTES, false);
#undef SEDD_LAUNCH_DBG
      SEDD_LAUNCH_CHECK();
      hipLaunchKernelGGL(k_debug_write_offsets, dim3(gdoc), dim3(256), 0, st, sbase, nd, total,
                         dbg_off + c.d0);
      SEDD_LAUNCH_CHECK();
      hipLaunchKernelGGL(k_debug_add_total, dim3(1), dim3(1), 0, st, total, sbase + nd);
      SEDD_LAUNCH_CHECK();
    } else if (rolling) {
      RfArgs ra;
      ra.pbase = pbase;
      ra.tok_pos = rec.pos;
      ra.tok_len = rec.len;
      ra.tok_long = rec.long_len;
      ra.dv = dv;
      ra.sbase = sbase;
      ra.qk = rf_q;
      ra.pwtab = rf_pw;
      ra.n = (uint32_t)n;
      rc = launch_minhash_rf(byte_mode, ra, htd, htb + nd, nht, (int)K, sig + c.d0 * (uint64_t)K, st);
      if (rc) return rc;
    } else {
      rc = launch_minhash(X_BYTES, xsrc, htd, htb + nd, nht, coef_a, coef_s,
                          paper ? coef_pp : (const CoefPP *)nullptr, (int)K,
                          sig + c.d0 * (uint64_t)K, st);
      if (rc) return rc;
    }
  }
  return SEDD_OK;
}

// ---- text resident in host memory -------------------------------------------------------------
//
// Two device staging buffers for the text and two for the offsets, an upload stream and four
// events, all owned by the library and kept between calls (sedd_release_scratch frees them).
struct HostFeed {
  uint8_t *text[2] = {nullptr, nullptr};
  uint64_t *offs[2] = {nullptr, nullptr};
  uint64_t text_bytes = 0, offs_count = 0;
  hipStream_t copy = nullptr;
  hipEvent_t copied[2] = {nullptr, nullptr}, done[2] = {nullptr, nullptr};
};
static HostFeed g_feed;

static int feed_ensure(uint64_t text_bytes, uint64_t offs_count) {
  HostFeed &f = g_feed;
  if (!f.copy) {
    SEDD_HIP(hipStreamCreateWithFlags(&f.copy, hipStreamNonBlocking));  // default priority
    for (int i = 0; i < 2; i++) {
      SEDD_HIP(hipEventCreateWithFlags(&f.copied[i], hipEventDisableTiming));
      SEDD_HIP(hipEventCreateWithFlags(&f.done[i], hipEventDisableTiming));
    }
  }
  if (text_bytes > f.text_bytes || offs_count > f.offs_count) {
    SEDD_HIP(hipDeviceSynchronize());  // earlier calls may still read the old buffers
    for (int i = 0; i < 2; i++) {
      if (f.text[i]) SEDD_HIP(hipFree(f.text[i]));
      if (f.offs[i]) SEDD_HIP(hipFree(f.offs[i]));
      f.text[i] = nullptr;
      f.offs[i] = nullptr;
    }
    f.text_bytes = f.offs_count = 0;
    const uint64_t tb = std::max(text_bytes, f.text_bytes) + 64, oc = std::max(offs_count, f.offs_count);
    for (int i = 0; i < 2; i++) {
      void *p = nullptr, *q = nullptr;
      hipError_t e = hipMalloc(&p, tb);
      if (e == hipSuccess) e = hipMalloc(&q, oc * sizeof(uint64_t));
      if (e != hipSuccess) {
        (void)hipGetLastError();
        if (p) (void)hipFree(p);
        set_device_error(e, "hipMalloc(upload buffers)");
        return SEDD_ENOMEM;
      }
      f.text[i] = (uint8_t *)p;
      f.offs[i] = (uint64_t *)q;
    }
    f.text_bytes = tb;
    f.offs_count = oc;
  }
  return SEDD_OK;
}

int release_host_feed() {
  HostFeed &f = g_feed;
  for (int i = 0; i < 2; i++) {
    if (f.text[i]) SEDD_HIP(hipFree(f.text[i]));
    if (f.offs[i]) SEDD_HIP(hipFree(f.offs[i]));
    f.text[i] = nullptr;
    f.offs[i] = nullptr;
  }
  f.text_bytes = f.offs_count = 0;
  return SEDD_OK;
}

}  // namespace sedd

using namespace sedd;

extern "C" {

int sedd_minhash(const uint8_t *bytes, const uint64_t *doc_offsets, uint64_t n_docs,
                 int32_t shingle_n, int32_t K, uint64_t seed, uint32_t flags, uint32_t *sig,
                 void *stream) {
  if (shingle_n < 1 || shingle_n > SEDD_MAX_SHINGLE_N || K < 1 || K > SEDD_MAX_K) return SEDD_EINVAL;
  if (flags & ~(SEDD_FLAG_BYTE_SHINGLES | SEDD_FLAG_PAPER_PRIME | SEDD_FLAG_ROLLING_FAMILY))
    return SEDD_EINVAL;
  if ((flags & SEDD_FLAG_PAPER_PRIME) && (flags & SEDD_FLAG_ROLLING_FAMILY)) return SEDD_EINVAL;
  if (n_docs == 0) return SEDD_OK;
  if (!doc_offsets || !sig || n_docs >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  if (!aligned_to(doc_offsets, 8) || !aligned_to(sig, 4)) return SEDD_EINVAL;
  return run_minhash(bytes, ~uint64_t(0), doc_offsets, n_docs, shingle_n, K, seed, flags, sig,
                     nullptr, 0, nullptr, (hipStream_t)stream);
}

int sedd_minhash_bounded(const uint8_t *bytes, uint64_t n_bytes, const uint64_t *doc_offsets,
                         uint64_t n_docs, int32_t shingle_n, int32_t K, uint64_t seed,
                         uint32_t flags, uint32_t *sig, void *stream) {
  if (shingle_n < 1 || shingle_n > SEDD_MAX_SHINGLE_N || K < 1 || K > SEDD_MAX_K) return SEDD_EINVAL;
  if (flags & ~(SEDD_FLAG_BYTE_SHINGLES | SEDD_FLAG_PAPER_PRIME | SEDD_FLAG_ROLLING_FAMILY))
    return SEDD_EINVAL;
  if ((flags & SEDD_FLAG_PAPER_PRIME) && (flags & SEDD_FLAG_ROLLING_FAMILY)) return SEDD_EINVAL;
  if (n_docs == 0) return SEDD_OK;
  if (!doc_offsets || !sig || n_docs >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  if (!aligned_to(doc_offsets, 8) || !aligned_to(sig, 4)) return SEDD_EINVAL;
  return run_minhash(bytes, n_bytes, doc_offsets, n_docs, shingle_n, K, seed, flags, sig, nullptr, 0,
                     nullptr, (hipStream_t)stream);
}

int sedd_minhash_host_chunked(const uint8_t *host_bytes, const uint64_t *host_doc_offsets,
                              uint64_t n_docs, int32_t shingle_n, int32_t K, uint64_t seed,
                              uint32_t flags, uint64_t chunk_bytes, uint32_t *sig, void *stream) {
  if (shingle_n < 1 || shingle_n > SEDD_MAX_SHINGLE_N || K < 1 || K > SEDD_MAX_K) return SEDD_EINVAL;
  if (flags & ~(SEDD_FLAG_BYTE_SHINGLES | SEDD_FLAG_PAPER_PRIME | SEDD_FLAG_ROLLING_FAMILY))
    return SEDD_EINVAL;
  if ((flags & SEDD_FLAG_PAPER_PRIME) && (flags & SEDD_FLAG_ROLLING_FAMILY)) return SEDD_EINVAL;
  if (n_docs == 0) return SEDD_OK;
  if (!host_doc_offsets || !sig || n_docs >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  if (!aligned_to(host_doc_offsets, 8) || !aligned_to(sig, 4)) return SEDD_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const uint64_t *off = host_doc_offsets;
  // the offsets are on the host: validate them here
  const uint64_t max_doc = (uint64_t(1) << 32) - (uint64_t(1) << 30) - (uint64_t(1) << 16);
  for (uint64_t d = 0; d < n_docs; d++)
    if (off[d + 1] < off[d] || off[d + 1] - off[d] >= max_doc) return SEDD_EINVAL;
  if (off[n_docs] > off[0] && !host_bytes) return SEDD_EINVAL;
  if (chunk_bytes == 0) chunk_bytes = uint64_t(2) << 30;
  const uint64_t chunk_docs = uint64_t(1) << 22;
  // chunks of whole documents: as many as fit chunk_bytes (at least one), at most chunk_docs
  std::vector<uint64_t> cuts;
  cuts.push_back(0);
  uint64_t max_text = 0, max_docs = 0;
  for (uint64_t d0 = 0; d0 < n_docs;) {
    const uint64_t *hi = std::upper_bound(off + d0 + 1, off + n_docs + 1, off[d0] + chunk_bytes);
    uint64_t d1 = (uint64_t)(hi - off) - 1;  // last index whose offset is within the budget
    d1 = std::min(std::max(d1, d0 + 1), std::min(n_docs, d0 + chunk_docs));
    max_text = std::max(max_text, off[d1] - off[d0]);
    max_docs = std::max(max_docs, d1 - d0);
    cuts.push_back(d1);
    d0 = d1;
  }
  int rc = feed_ensure(max_text, max_docs + 1);
  if (rc) return rc;
  HostFeed &f = g_feed;
  const bool streamed = !(flags & (SEDD_FLAG_BYTE_SHINGLES | SEDD_FLAG_ROLLING_FAMILY));
  const size_t n_chunks = cuts.size() - 1;
  bool used[2] = {false, false};
  auto upload = [&](size_t i) -> int {
    const uint64_t d0 = cuts[i], d1 = cuts[i + 1];
    const int s = (int)(i & 1);
    if (used[s]) SEDD_HIP(hipStreamWaitEvent(f.copy, f.done[s], 0));  // its last reader has finished
    const uint64_t nb = off[d1] - off[d0];
    if (nb) SEDD_HIP(hipMemcpyAsync(f.text[s], host_bytes + off[d0], nb, hipMemcpyHostToDevice, f.copy));
    SEDD_HIP(hipMemcpyAsync(f.offs[s], off + d0, (d1 - d0 + 1) * sizeof(uint64_t),
                            hipMemcpyHostToDevice, f.copy));
    SEDD_HIP(hipEventRecord(f.copied[s], f.copy));
    return SEDD_OK;
  };
  // the first upload must not overtake work already queued on the caller's stream that may
  // still read the staging buffers of an earlier call
  SEDD_HIP(hipEventRecord(f.done[0], st));
  SEDD_HIP(hipStreamWaitEvent(f.copy, f.done[0], 0));
  rc = upload(0);
  if (rc) return rc;
  for (size_t i = 0; i < n_chunks; i++) {
    const int s = (int)(i & 1);
    if (i + 1 < n_chunks) {
      rc = upload(i + 1);  // overlaps the hashing of chunk i
      if (rc) return rc;
    }
    const uint64_t d0 = cuts[i], d1 = cuts[i + 1];
    SEDD_HIP(hipStreamWaitEvent(st, f.copied[s], 0));
    // the staged offsets are the caller's, unshifted: the text pointer is moved back instead
    const uint8_t *base = f.text[s] - off[d0];
    const uint64_t ends[2] = {off[d0], off[d1]};
    if (streamed)
      rc = run_minhash_stream(base, off[d1], f.offs[s], d1 - d0, shingle_n, K, seed,
                              (flags & SEDD_FLAG_PAPER_PRIME) != 0, sig + d0 * (uint64_t)K, nullptr, 0,
                              nullptr, st, ends);
    else
      rc = run_minhash(base, off[d1], f.offs[s], d1 - d0, shingle_n, K, seed, flags,
                       sig + d0 * (uint64_t)K, nullptr, 0, nullptr, st);
    if (rc) return rc;
    SEDD_HIP(hipEventRecord(f.done[s], st));
    used[s] = true;
  }
  // the host buffers are free to change once the last upload has left them
  SEDD_HIP(hipEventSynchronize(f.copied[(n_chunks - 1) & 1]));
  return SEDD_OK;
}

int sedd_debug_shingle_hashes(const uint8_t *bytes, const uint64_t *doc_offsets,
                              uint64_t n_docs, int32_t shingle_n, uint32_t flags, uint64_t *x,
                              uint64_t x_cap, uint64_t *shingle_offsets, void *stream) {
  if (shingle_n < 1 || shingle_n > SEDD_MAX_SHINGLE_N) return SEDD_EINVAL;
  if (flags & ~(SEDD_FLAG_BYTE_SHINGLES | SEDD_FLAG_PAPER_PRIME)) return SEDD_EINVAL;
  if (!shingle_offsets || (x_cap && !x)) return SEDD_EINVAL;
  if (n_docs >= (uint64_t(1) << 31)) return SEDD_EINVAL;
  if (n_docs == 0) {
    hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(1), 0, (hipStream_t)stream, shingle_offsets);
    SEDD_LAUNCH_CHECK();
    return SEDD_OK;
  }
  if (!doc_offsets) return SEDD_EINVAL;
  return run_minhash(bytes, ~uint64_t(0), doc_offsets, n_docs, shingle_n, 1, 0, flags, nullptr, x,
                     x_cap, shingle_offsets, (hipStream_t)stream);
}

int sedd_debug_coeffs(uint64_t seed, int32_t K, uint64_t *a, uint64_t *b, void *stream) {
  if (K < 1 || K > SEDD_MAX_K || !a || !b) return SEDD_EINVAL;
  hipLaunchKernelGGL(k_coeffs, dim3((K + 255) / 256), dim3(256), 0, (hipStream_t)stream, seed,
                     (int)K, a, b, (CoefSplit *)nullptr, (uint64_t *)nullptr, (PowSplit *)nullptr);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

int sedd_debug_bases(uint64_t seed, int32_t K, uint64_t *q, void *stream) {
  if (K < 1 || K > SEDD_MAX_K || !q) return SEDD_EINVAL;
  hipLaunchKernelGGL(k_coeffs_rf, dim3((K + 255) / 256), dim3(256), 0, (hipStream_t)stream, seed,
                     (int)K, q, (uint64_t *)nullptr);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

int sedd_debug_coeffs_pp(uint64_t seed, int32_t K, uint64_t *a, uint64_t *b, void *stream) {
  if (K < 1 || K > SEDD_MAX_K || !a || !b) return SEDD_EINVAL;
  hipLaunchKernelGGL(k_coeffs_pp, dim3((K + 255) / 256), dim3(256), 0, (hipStream_t)stream, seed,
                     (int)K, (CoefPP *)nullptr, (PowPP *)nullptr, a, b);
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

static int minhash_from_x(const uint64_t *x, const uint64_t *shingle_offsets, uint64_t n_docs,
                          uint64_t n_shingles, int32_t K, uint64_t seed, bool paper, uint32_t *sig,
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
  const uint64_t o_cpp = cv.take<CoefPP>(K);
  const uint64_t o_sbase = cv.take<uint32_t>(n_docs + 1), o_htb = cv.take<uint32_t>(n_docs + 1);
  const uint64_t o_htd = cv.take<HTile>(nht);
  const uint64_t o_tmp = cv.take<uint32_t>(scan_tmp_count(n_docs + 1));
  uint8_t *A = nullptr;
  int rc = scratch_ensure(cv.off, &A);
  if (rc) return rc;
  uint64_t *coef_a = (uint64_t *)(A + o_a), *coef_b = (uint64_t *)(A + o_b);
  uint32_t *sbase = (uint32_t *)(A + o_sbase), *htb = (uint32_t *)(A + o_htb);
  HTile *htd = (HTile *)(A + o_htd);
  uint32_t *tmp = (uint32_t *)(A + o_tmp);
  CoefSplit *coef_s = (CoefSplit *)(A + o_cs);
  CoefPP *coef_pp = (CoefPP *)(A + o_cpp);
  if (paper)
    hipLaunchKernelGGL(k_coeffs_pp, dim3((K + 255) / 256), dim3(256), 0, st, seed, (int)K, coef_pp,
                       (PowPP *)nullptr, (uint64_t *)nullptr, (uint64_t *)nullptr);
  else
    hipLaunchKernelGGL(k_coeffs, dim3((K + 255) / 256), dim3(256), 0, st, seed, (int)K, coef_a,
                       coef_b, coef_s, (uint64_t *)nullptr, (PowSplit *)nullptr);
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
  hipLaunchKernelGGL(k_fill_htiles, dim3((uint32_t)((nht + 255) / 256)), dim3(256), 0, st, sbase,
                     htb, (const uint32_t *)nullptr, nd, 0u, (uint32_t)nht, htd);
  SEDD_LAUNCH_CHECK();
  XSource xsrc = {};
  xsrc.given = x;  // tiles index it by shingle offset
  return launch_minhash(X_GIVEN, xsrc, htd, htb + nd, nht, coef_a, coef_s,
                        paper ? coef_pp : (const CoefPP *)nullptr, (int)K, sig, st);
}

int sedd_debug_minhash_from_x(const uint64_t *x, const uint64_t *shingle_offsets, uint64_t n_docs,
                              uint64_t n_shingles, int32_t K, uint64_t seed, uint32_t *sig,
                              void *stream) {
  return minhash_from_x(x, shingle_offsets, n_docs, n_shingles, K, seed, false, sig, stream);
}

int sedd_debug_minhash_from_x_pp(const uint64_t *x, const uint64_t *shingle_offsets,
                                 uint64_t n_docs, uint64_t n_shingles, int32_t K, uint64_t seed,
                                 uint32_t *sig, void *stream) {
  return minhash_from_x(x, shingle_offsets, n_docs, n_shingles, K, seed, true, sig, stream);
}

int sedd_debug_set_chunk_bytes(uint64_t bytes) {
  g_chunk_bytes_override = bytes;
  return SEDD_OK;
}

int sedd_debug_set_piece_bytes(uint32_t bytes) {
  if (bytes % TB != 0 || bytes > (1u << 24)) return SEDD_EINVAL;
  set_piece_bytes_override(bytes);
  return SEDD_OK;
}

}  // extern "C"
