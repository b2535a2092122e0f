// sedd_minhash: shingling, Eq. 1 base hash, K hash functions and per-document minimum.
//
// Word shingles with the affine family (the default 61-bit modulus and the paper's own prime):
// k_minhash_stream, one launch that reads the text once; see the comment above that kernel.
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
#include <atomic>
#include <mutex>
#include <thread>
#include <vector>

#include "sedd_internal.h"

namespace sedd {

constexpr int TB_LANES = 64;
constexpr uint32_t TB = TB_LANES * 16;    // bytes per byte tile: one wavefront, 16 bytes per lane
constexpr uint32_t TS = 320;              // shingles per hash tile
constexpr int QPOW_N = 256;

// x(s) of Eq. 1 as the hot kernel multiplies by it: x = x1 * 2^31 + x0 with x0 < 2^31,
// x1 < 2^30, together with the pre-scaled limbs 2 x0 and 4 x1 (both fit 32 bits).
struct XLimbs {
  uint32_t x0, x1, x0_2, x1_4;
};
__device__ __forceinline__ XLimbs x_limbs(uint64_t x) {
  XLimbs r;
  r.x0 = (uint32_t)x & 0x7FFFFFFFu;
  r.x1 = (uint32_t)(x >> 31);
  r.x0_2 = r.x0 << 1;
  r.x1_4 = r.x1 << 2;
  return r;
}

// what the hot loop needs of one hash function, in one 16-byte record: a in the same limb form
// (a = a1 * 2^31 + a0) and b
struct CoefSplit {
  uint32_t a0;   // a mod 2^31
  uint32_t a12;  // 2 * (a >> 31)
  uint64_t b;
};

// Token records of the rolling-family mode, structure of arrays: pos[i] = position of token i in
// the chunk frame, len[i] = min(length, 255); a token of 255 bytes or more keeps its length in
// long_len[i] (written and read only for such tokens).
struct TokenRecs {
  uint32_t *pos;
  uint8_t *len;
  uint32_t *long_len;
};
constexpr uint32_t LONG_TOKEN = 255;  // token lengths from here on take the general shingle hash


// Per token length l < QPOW_N, what one Horner step over token records multiplies by:
// P = 257^(l+1) as a0 = P mod 2^31, a0_2 = 2 a0, a12 = 2 (P >> 31); and nsp = p - 32 * 257^l,
// which turns the hash of "token 0x20" into the hash of the bare token by one addition.
struct PowSplit {
  uint32_t a0, a0_2, a12, pad;
  uint64_t nsp, pad2;
};

// 257^e with the first QPOW_N powers from a table (a few cache lines, shared by every lane)
__device__ __forceinline__ uint64_t qpow_global(const uint64_t *__restrict__ qpow, uint32_t e) {
  return e < (uint32_t)QPOW_N ? qpow[e] : powmod(257, e);
}
// ---- paper-prime mode (SEDD_FLAG_PAPER_PRIME) ------------------------------------------------
//
// Section 3.2 quotes p' = 4,294,967 as the modulus of Eq. 1 in the paper's experiments.  p' is
// not a Mersenne prime, so a product is reduced through an estimate of its quotient.
constexpr uint32_t PP = 4294967u;
// a quotient estimate of the hash loops is off by one only for remainders this close to p' (see
// k_minhash_pp)
constexpr uint32_t PP_EDGE = 4400;  // > p' (p' + 2) / 2^32 = 4295.0

// t mod p' for t < 2^46.  With T = t >> 14 (< 2^32) and M = floor(2^46 / p'), floor(T M / 2^32)
// is the quotient or up to 2 below it; the remainder estimate then lies in [0, 3 p') (< 2^24).
__device__ __forceinline__ uint32_t red_pp(uint64_t t) {
  constexpr uint32_t M = (uint32_t)((uint64_t(1) << 46) / PP);
  const uint32_t q = __umulhi((uint32_t)(t >> 14), M);
  uint32_t r = (uint32_t)t - q * PP;
  r = min(r, r - PP);  // r - p' wraps to a huge value when r < p'
  r = min(r, r - PP);
  return r;
}
__device__ __forceinline__ uint32_t mulmod_pp(uint32_t a, uint32_t b) {
  return red_pp((uint64_t)a * b);
}
__device__ inline uint32_t powmod_pp(uint32_t g, uint64_t e) {
  uint32_t r = 1, base = g;
  while (e) {
    if (e & 1) r = mulmod_pp(r, base);
    base = mulmod_pp(base, base);
    e >>= 1;
  }
  return r;
}

// One hash function h'(x) = (a x + b) mod p' as the hot loop uses it: a, b and the 32-bit
// fixed-point reciprocals ap = ceil(a 2^32 / p'), bp = ceil(b 2^32 / p'), both rounded up.
struct CoefPP {
  uint32_t a, b, ap, bp;
};
// Per token length l < QPOW_N: pw1 = 257^(l+1) mod p', sp = 32 * 257^l mod p'.
struct PowPP {
  uint32_t pw1, sp;
};

__device__ __forceinline__ void store_token_pos(const TokenRecs &tr, uint32_t idx, uint32_t pos,
                                                uint32_t len) {
  tr.pos[idx] = pos;
  tr.len[idx] = (uint8_t)(len < LONG_TOKEN ? len : LONG_TOKEN);
  if (len >= LONG_TOKEN) tr.long_len[idx] = len;
}

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

// Work-list entries.  One load tells a block everything about its tile, so no block walks a
// chain of dependent index loads before it can touch its data.
struct BTile {      // 1 KiB byte tile of one document
  uint32_t vs, ve;  // the document's bytes [vs, ve) in the chunk frame
  uint32_t tile0;   // first byte of the tile (16-aligned)
  uint32_t pad;
};
struct HTile {       // tile of up to TS shingles of one document
  uint32_t doc;      // document index within the chunk
  uint32_t x_off;    // index of the tile's first shingle in the chunk's shingle stream
  uint32_t cnt;      // shingles in the tile
  uint32_t single;   // 1 if the document has no other tile
  uint32_t tok0;     // (word mode) index of the first token of the tile's first shingle
  uint32_t per;      // (word mode) tokens per shingle: min(n, tokens in the document)
  uint32_t pad[2];
};

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

// ---- tokenisation ------------------------------------------------------------------------

// The 16 bytes of one thread's segment and the mask of its token bytes (bit i: byte seg+i lies
// inside the document [vs, ve) and is not whitespace).  seg is 16-aligned; the load is issued
// only if the segment holds at least one byte of the document.
struct Segment {
  uint32_t w[4];
  uint32_t wm;
};
__device__ __forceinline__ uint32_t seg_byte(const Segment &sg, int i) {
  return (sg.w[i >> 2] >> (8 * (i & 3))) & 0xFFu;
}
// 4-bit mask of the bytes of w that are NOT whitespace {09..0D, 20}, by SWAR on the word
__device__ __forceinline__ uint32_t nonspace_mask4(uint32_t w) {
  const uint32_t lo7 = w & 0x7F7F7F7Fu;
  // byte == 0x20
  const uint32_t t = w ^ 0x20202020u;
  const uint32_t eq20 = ~(((t & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | t) & 0x80808080u;
  // 0x09 <= byte <= 0x0D (bytes >= 0x80 excluded by ~w)
  const uint32_t ge9 = lo7 + (0x80808080u - 0x09090909u);  // bit 7 set iff low7 >= 9
  const uint32_t le13 = ~(lo7 + (0x80808080u - 0x0E0E0E0Eu));  // bit 7 set iff low7 <= 13
  const uint32_t ws = (eq20 | (ge9 & le13 & ~w)) & 0x80808080u;
  const uint32_t ns = ~ws & 0x80808080u;
  // gather bits 7, 15, 23, 31 into bits 0..3
  return ((ns >> 7) * 0x00204081u >> 21) & 0xFu;
}
// The 16 bytes at seg (16-aligned) if the segment holds at least one byte of the document
// [vs, ve); zeros otherwise (no load is issued then).
__device__ __forceinline__ uint4 load_raw16(const uint8_t *__restrict__ pbase, uint32_t seg,
                                            uint32_t vs, uint32_t ve) {
  uint4 q = make_uint4(0, 0, 0, 0);
  if (seg < ve && seg + 16 > vs) q = *reinterpret_cast<const uint4 *>(pbase + seg);
  return q;
}
__device__ __forceinline__ Segment make_segment(const uint4 q, uint32_t seg, uint32_t vs,
                                                uint32_t ve) {
  Segment sg;
  sg.w[0] = q.x; sg.w[1] = q.y; sg.w[2] = q.z; sg.w[3] = q.w;
  const uint32_t m = nonspace_mask4(q.x) | (nonspace_mask4(q.y) << 4) |
                     (nonspace_mask4(q.z) << 8) | (nonspace_mask4(q.w) << 12);
  // bytes of the segment inside the document: [lo, hi)
  const bool inside = seg < ve && seg + 16 > vs;
  const uint32_t lo = vs > seg ? vs - seg : 0u;
  const uint32_t hi = ve - seg < 16u ? ve - seg : 16u;
  const uint32_t valid = ((1u << hi) - 1u) & ~((1u << lo) - 1u);
  sg.wm = inside ? (m & valid) : 0u;
  return sg;
}
// The byte before the tile if it belongs to the document, a space otherwise.
__device__ __forceinline__ uint32_t load_prev_byte(const uint8_t *__restrict__ pbase,
                                                   uint32_t tile0, uint32_t vs, uint32_t ve) {
  return (tile0 > vs && tile0 <= ve) ? (uint32_t)pbase[tile0 - 1] : 0x20u;
}

// Bit i of the result: byte seg+i starts a token.  Needs the token-byte bit of the byte before
// the segment: the lane below's last bit (by shuffle), or for lane 0 the byte before the tile.
// Must be called by all 64 lanes of the tile's wavefront.
__device__ __forceinline__ uint32_t token_starts(uint32_t lane, uint32_t prev_byte, uint32_t wm) {
  // wave_shr:1 (lane l reads lane l - 1; lane 0 keeps the first operand)
  uint32_t prev = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(wm >> 15), 0x138, 0xF, 0xF, false);
  if (lane == 0) prev = is_ws(prev_byte) ? 0u : 1u;
  return wm & ~((wm << 1) | prev) & 0xFFFFu;
}

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

// acc * 257 + c without full reduction: result < 2^61 + 2^10 for acc < 2^61 + 2^10
__device__ __forceinline__ uint64_t horner257_lazy(uint64_t acc, uint32_t c) {
  const uint64_t lo = (uint64_t)(uint32_t)acc * 257u + c;              // < 2^41
  const uint64_t hi = (uint64_t)(uint32_t)(acc >> 32) * 257u + (lo >> 32);  // < 2^39
  // value = hi * 2^32 + lo32; bits 61.. of it are hi >> 29, and 2^61 = 1 (mod p)
  return (((hi & 0x1FFFFFFFu) << 32) | (uint32_t)lo) + (hi >> 29);
}

// acc * 257^3 + D without full reduction, for acc < 2^61 + 2^26 and D < 2^25; the result is
// again below 2^61 + 2^26.  (257^3 fits 25 bits: one step consumes three bytes.)
constexpr uint32_t R3 = 257u * 257u * 257u;
__device__ __forceinline__ uint64_t horner3_lazy(uint64_t acc, uint32_t D) {
  const uint64_t lo = (uint64_t)(uint32_t)acc * R3 + D;                        // < 2^58
  const uint64_t hi = (uint64_t)(uint32_t)(acc >> 32) * R3 + (lo >> 32);       // < 2^55
  // value = hi * 2^32 + lo32; bits 61.. of it are hi >> 29, and 2^61 = 1 (mod p)
  return (((hi & 0x1FFFFFFFull) << 32) | (uint32_t)lo) + (hi >> 29);
}

// A token that a wavefront cannot finish from the LDS copy of its tile (64 bytes or more, or
// running past the look-ahead) is walked byte by byte in global memory.
struct WalkedToken {
  uint64_t w;  // Eq. 1 of the token, w = sum c_i 257^i
  uint32_t len;
};

// bytes from position p0 up to the first whitespace byte or the document's end ve
__device__ __noinline__ uint32_t token_length_far(const uint8_t *__restrict__ pbase, uint32_t p0,
                                                  uint32_t ve) {
  uint32_t p = p0;
  while (p < ve && !is_ws(pbase[p])) p++;
  return p - p0;
}

constexpr uint32_t LOOK = 16;
constexpr uint32_t MAX_TILE_TOKENS = TB / 2 + 2;
constexpr uint32_t FAST_TOKEN_MAX = 63;  // longest token finished from LDS
// text in LDS: tile + look-ahead + slack for the (masked) reads of lanes whose token is shorter
// than the wavefront's longest
constexpr uint32_t SM_TEXT_WORDS = (TB + LOOK + FAST_TOKEN_MAX + 9) / 4 + 2;

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

struct HotConsts {
  uint32_t two29;  // 1 << 29
  uint32_t eight;  // 8
  uint32_t one;    // 1
};

// acc <- P acc + V (mod p) for acc < 2^61 + 8, P given as (a0, a0_2, a12), V < p; the result is
// again below 2^61 + 8 (not canonical).  Same limb scheme as the hot loop, 4 multiply-adds.
__device__ __forceinline__ uint64_t horner_step_lazy(uint64_t acc, uint32_t a0, uint32_t a0_2,
                                                     uint32_t a12, uint64_t V, const HotConsts &hc) {
  const uint32_t c_lo = (uint32_t)acc, x0 = c_lo & 0x7FFFFFFFu, x0_2 = c_lo << 1;
  const uint32_t x1 = (uint32_t)(acc >> 31), x1_2 = x1 << 1;
  uint64_t N = (uint64_t)a0_2 * x1_2;
  N += (uint64_t)a12 * x0_2;
  uint64_t U = (uint64_t)a12 * x1 + V;
  U += (uint64_t)a0 * x0;
  uint64_t Z = (uint64_t)(uint32_t)N * hc.two29 + U;
  Z = (uint64_t)(uint32_t)(N >> 32) * hc.one + Z;
  return (uint64_t)(uint32_t)(Z >> 61) * hc.one + (Z & P61);
}

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

// ---- the streaming kernel (word shingles, affine family) ------------------------------------------
//
// The whole of sedd_minhash in one launch, for the default mode and the paper-prime mode (the
// template argument A holds what depends on the modulus): the text is read from HBM once,
// nothing but the signatures is written, and there is no work list.  The text (a frame that
// starts on a 16-byte boundary at or below document 0) is cut into pieces of `piece` bytes; one
// wavefront owns the tokens that START inside its piece, in document order, and with them the
// shingles that start at those tokens.  Per document that reaches into the piece it walks
// 1 KiB tiles of the document's bytes:
//   pass 1 (lane = 16 bytes)   token-byte bitmap, token starts and their ranks, as in k_emit_words;
//   rounds of 64 tokens        lane = token: Eq. 1 of the token from the LDS copy of the tile, the
//                              record (hash of "token 0x20", length) goes into a ring in LDS;
//                              lane = shingle: x(s) by Horner over its n ring records, into LDS;
//                              lane = hash function: the K multiply-adds and the running minimum
//                              over the round's shingles, exactly as in k_minhash.
// The minima stay in registers until the document ends.  A document that lies inside the piece
// is stored; one that crosses a piece boundary is merged with atomicMin by the pieces it touches
// (the signatures start out as 0xFFFFFFFF).  A piece reads on past its end, inside the document
// that crosses it, until the shingles of its own tokens are complete (n - 1 more tokens).
// The one-shingle rule for documents of fewer than n tokens belongs to the piece that owns the
// document's first token; a piece that meets the end of such a document and did not see its
// beginning looks back for an earlier token byte before it decides.

constexpr uint32_t RING = 128;  // ring of token records: the n - 1 before a round plus its 64
static_assert(RING >= 64 + SEDD_MAX_SHINGLE_N - 1 && (RING & (RING - 1)) == 0, "ring too small");

struct StreamArgs {
  const uint8_t *frame;   // 16-byte aligned address at or below the first byte of document 0
  const uint64_t *off;    // doc_offsets
  uint64_t n_docs;
  uint64_t shift;         // off[d] + shift = frame position of the first byte of document d
  uint64_t frame_end;     // frame position of the end of the last document
  uint32_t piece;         // bytes per wavefront, a multiple of TB
  uint32_t n;             // shingle length
};

// what the kernel does with a shingle hash: evaluate the K functions (production), count, or
// write it out in order (the two passes of the stage-level debug entry)
enum { SM_HASH = 0, SM_COUNT = 1, SM_WRITE = 2 };
struct StreamDebug {
  uint32_t *piece_count;  // SM_COUNT: shingles of each piece (out); SM_WRITE: their prefix sums (in)
  uint32_t *doc_piece;    // SM_COUNT: the piece that holds the first byte of a non-empty document
  uint32_t *doc_local;    // SM_COUNT: shingles that piece found before the document
  uint64_t *x;            // SM_WRITE: shingle hashes in document order
  uint64_t x_cap;         //           entries of x
  uint64_t x_base;        //           index of this call's first shingle
};

// Eq. 1 of the token that starts at p, byte by byte: up to max_len bytes or the first whitespace
__device__ __noinline__ WalkedToken walk_token_far(const uint8_t *__restrict__ p, uint64_t max_len) {
  uint64_t w = 0, pw = 1;
  uint64_t l = 0;
  for (; l < max_len; l++) {
    const uint32_t c = p[l];
    if (is_ws(c)) break;
    w = addmod(w, mulmod(pw, (uint64_t)c));
    pw = mul257(pw);
  }
  WalkedToken r;
  r.w = w;
  r.len = (uint32_t)l;
  return r;
}
// the same modulo the paper's prime (w in the low word)
__device__ __noinline__ WalkedToken walk_token_far_pp(const uint8_t *__restrict__ p, uint64_t max_len) {
  uint32_t w = 0, pw = 1;
  uint64_t l = 0;
  for (; l < max_len; l++) {
    const uint32_t c = p[l];
    if (is_ws(c)) break;
    w = red_pp((uint64_t)pw * c + w);
    pw = mulmod_pp(pw, 257u);
  }
  WalkedToken r;
  r.w = w;
  r.len = (uint32_t)l;
  return r;
}

// The digits of a token of at most 16 bytes at byte `pos` of the LDS copy of a tile: bytes 0-2,
// 3-5, 6-8, 9-11, 12-14 as c0 + 257 c1 + 257^2 c2 each, and byte 15; bytes past flen cleared.
struct TokenDigits {
  uint32_t D[5], last;
};
__device__ __forceinline__ uint32_t digit257(uint32_t d) {
  // three bytes c0 + 256 c1 + 65536 c2 -> c0 + 257 c1 + 257^2 c2
  return d + ((d >> 8) & 0xFFu) + 513u * (d >> 16);
}
__device__ __forceinline__ TokenDigits token_digits16(const uint32_t *sm_text, uint32_t pos, uint32_t flen) {
  const uint32_t wd = pos >> 2, sh = pos & 3u;
  const uint32_t t0 = sm_text[wd], t1 = sm_text[wd + 1], t2 = sm_text[wd + 2], t3 = sm_text[wd + 3],
                 t4 = sm_text[wd + 4];
  // bytes 0..7 and 8..15 of the token, those past its end cleared
  const uint32_t l_lo = min(flen, 8u), l_hi = flen - l_lo;
  const uint64_t keep_lo = l_lo ? ~0ull >> (64u - 8u * l_lo) : 0ull;
  const uint64_t keep_hi = l_hi ? ~0ull >> (64u - 8u * l_hi) : 0ull;
  const uint32_t a0 = __builtin_amdgcn_alignbyte(t1, t0, sh) & (uint32_t)keep_lo;
  const uint32_t a1 = __builtin_amdgcn_alignbyte(t2, t1, sh) & (uint32_t)(keep_lo >> 32);
  const uint32_t a2 = __builtin_amdgcn_alignbyte(t3, t2, sh) & (uint32_t)keep_hi;
  const uint32_t a3 = __builtin_amdgcn_alignbyte(t4, t3, sh) & (uint32_t)(keep_hi >> 32);
  TokenDigits r;
  r.D[0] = digit257(a0 & 0xFFFFFFu);
  r.D[1] = digit257(__builtin_amdgcn_alignbyte(a1, a0, 3u) & 0xFFFFFFu);
  r.D[2] = digit257(__builtin_amdgcn_alignbyte(a2, a1, 2u) & 0xFFFFFFu);
  r.D[3] = digit257(__builtin_amdgcn_alignbyte(a3, a2, 1u) & 0xFFFFFFu);
  r.D[4] = digit257(a3 & 0xFFFFFFu);
  r.last = a3 >> 24;
  return r;
}
// the same for at most 8 bytes: one 12-byte read, digits 0..2 (D[2] holds bytes 6-7)
__device__ __forceinline__ TokenDigits token_digits8(const uint32_t *sm_text, uint32_t pos, uint32_t flen) {
  const uint32_t wd = pos >> 2;
  const uint32_t t0 = sm_text[wd], t1 = sm_text[wd + 1], t2 = sm_text[wd + 2];
  const uint64_t keep = ~0ull >> ((64u - 8u * flen) & 63u);  // flen >= 1 where it matters
  const uint32_t a0 = __builtin_amdgcn_alignbyte(t1, t0, pos & 3u) & (uint32_t)keep;
  const uint32_t a1 = __builtin_amdgcn_alignbyte(t2, t1, pos & 3u) & (uint32_t)(keep >> 32);
  const uint32_t d2 = a1 >> 16;
  TokenDigits r;
  r.D[0] = digit257(a0 & 0xFFFFFFu);
  r.D[1] = digit257(__builtin_amdgcn_alignbyte(a1, a0, 3u) & 0xFFFFFFu);
  r.D[2] = d2 + (d2 >> 8);
  r.D[3] = r.D[4] = r.last = 0;
  return r;
}
// digit k (bytes 3k .. 3k+2) of a token of flen bytes at byte `pos`, for the general loop
__device__ __forceinline__ uint32_t token_digit_at(const uint32_t *sm_text, uint32_t pos, uint32_t flen,
                                                   uint32_t k) {
  const int rem = (int)flen - (int)(3 * k);  // bytes of the token from digit k on
  const uint32_t nbits = (uint32_t)min(max(rem, 0), 3) * 8u;
  const uint32_t msk = nbits ? (0xFFFFFFFFu >> (32u - nbits)) : 0u;
  const uint32_t o = pos + 3 * k;
  const uint32_t lo = sm_text[o >> 2], hi = sm_text[(o >> 2) + 1];
  return digit257(__builtin_amdgcn_alignbyte(hi, lo, o & 3u) & msk);
}
// number of 3-byte digits of the longest token of the round (wave-uniform)
__device__ __forceinline__ uint32_t max_digits(uint32_t flen) {
  uint32_t maxnd = (flen + 2) / 3;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) maxnd = max(maxnd, (uint32_t)__shfl_xor(maxnd, o, 64));
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)maxnd);
}

// ---- the two arithmetics of the streaming kernel -----------------------------------------------
//
// Everything that depends on the modulus: Eq. 1 of a token, the value of "token 0x20", Eq. 1 of a
// shingle from ring records, how a round's shingle hashes sit in LDS, and the hash rounds.
// Arith61 is the default (p = 2^61-1, low 32 bits kept); ArithPP is SEDD_FLAG_PAPER_PRIME.

struct StreamTables {
  const uint64_t *qpow;    // 257^i, i < QPOW_N                      (Arith61)
  const PowSplit *ptab;    // Horner multipliers per token length    (Arith61)
  const uint64_t *coef_a;  // a_k as 64-bit values, for the exact path (Arith61)
  const CoefSplit *coef_s; // a_k in limb form and b_k               (Arith61)
  const PowPP *ptab_pp;    // powers per token length                (ArithPP)
  const CoefPP *coef_pp;   // a'_k, b'_k and their reciprocals       (ArithPP)
};

struct Arith61 {
  using Value = uint64_t;  // token values in the ring
  static constexpr uint32_t SX_WORDS = 64 * 4;  // a round's shingle hashes in limb form
  template <int F>
  struct Coefs {
    uint64_t b[F];
    uint32_t a0[F], a12[F];
  };
  template <int F>
  static __device__ __forceinline__ void load(Coefs<F> &c, const StreamTables &tb, int K, int kbase, int LW) {
#pragma unroll
    for (int j = 0; j < F; j++) {
      const int k = kbase + LW * j;
      const CoefSplit s = tb.coef_s[k < K ? k : 0];  // lanes past K compute function 0, store nothing
      c.a0[j] = s.a0;
      c.a12[j] = s.a12;
      c.b[j] = s.b;
    }
  }
  // Eq. 1 of a token of flen <= FAST_TOKEN_MAX bytes in the LDS copy (flen = 0: idle lane);
  // Horner over 3-byte digits, last digit first.  Must be called by the whole wavefront.
  static __device__ __forceinline__ Value token_hash(const uint32_t *sm_text, uint32_t pos, uint32_t flen) {
    uint64_t acc;
    if (!__any(flen > 8)) {
      const TokenDigits t = token_digits8(sm_text, pos, flen);
      acc = (uint64_t)t.D[2] * R3 + t.D[1];  // exact, below 2^42
      acc = horner3_lazy(acc, t.D[0]);
    } else if (!__any(flen > 16)) {
      // at most 16 bytes (ordinary prose): one 20-byte read, five digits and a byte, no loop
      const TokenDigits t = token_digits16(sm_text, pos, flen);
      acc = (uint64_t)t.last * R3 + t.D[4];  // exact, below 2^33
      acc = horner3_lazy(acc, t.D[3]);
      acc = horner3_lazy(acc, t.D[2]);
      acc = horner3_lazy(acc, t.D[1]);
      acc = horner3_lazy(acc, t.D[0]);
    } else {
      acc = 0;
      for (uint32_t k = max_digits(flen); k-- > 0;) acc = horner3_lazy(acc, token_digit_at(sm_text, pos, flen, k));
    }
    return fold61(acc);
  }
  static __device__ __forceinline__ WalkedToken token_far(const uint8_t *p, uint64_t max_len) {
    return walk_token_far(p, max_len);
  }
  // V = w + 32 * 257^len: the token followed by the joining space
  static __device__ __forceinline__ Value with_space(Value w, uint32_t len, const StreamTables &tb) {
    if (len < (uint32_t)QPOW_N) {
      const uint64_t nsp = tb.ptab[len].nsp;  // w + 32 * 257^len = w - nsp (mod p)
      return w >= nsp ? w - nsp : w + (P61 - nsp);
    }
    const uint64_t pw = powmod(257, len);
    const uint64_t sp = ((pw << 5) & P61) | (pw >> 56);  // a shift by 5 is a rotation of the residue
    return addmod(w, sp == P61 ? 0 : sp);
  }
  // x of the shingle made of the ring records first .. first + PER - 1 (indices modulo RING); valid
  // if every token is shorter than LONG_TOKEN bytes, *long_tok says if not
  template <int PER>
  static __device__ __forceinline__ Value shingle_unrolled(const Value *ring_v, const uint32_t *ring_len,
                                                           const StreamTables &tb, uint32_t first,
                                                           const HotConsts &hc, bool *long_tok) {
    uint32_t len[PER];
    uint64_t V[PER];
#pragma unroll
    for (int m = 0; m < PER; m++) {
      len[m] = ring_len[(first + m) & (RING - 1)];
      V[m] = ring_v[(first + m) & (RING - 1)];
    }
    bool lt = false;
#pragma unroll
    for (int m = 0; m < PER; m++) {
      lt |= len[m] >= LONG_TOKEN;
      len[m] = min(len[m], LONG_TOKEN);  // keeps the table index in range; the value is redone if long
    }
    *long_tok = lt;
    uint4 e[PER];
#pragma unroll
    for (int m = 0; m < PER - 1; m++) e[m] = *reinterpret_cast<const uint4 *>(tb.ptab + len[m]);
    const uint64_t nsp = tb.ptab[len[PER - 1]].nsp;
    uint64_t acc = V[PER - 1] + nsp;  // bare last token, < 2^62
    acc = (acc & P61) + (acc >> 61);
#pragma unroll
    for (int m = PER - 2; m >= 0; m--) acc = horner_step_lazy(acc, e[m].x, e[m].y, e[m].z, V[m], hc);
    return fold61(acc);
  }
  // the same for any number of tokens and any token lengths
  static __device__ __noinline__ Value shingle_general(const Value *ring_v, const uint32_t *ring_len,
                                                       const uint64_t *__restrict__ qpow, uint32_t first,
                                                       uint32_t per) {
    const uint32_t last = first + per - 1;
    const uint64_t pw = qpow_global(qpow, ring_len[last & (RING - 1)]);
    const uint64_t sp = ((pw << 5) & P61) | (pw >> 56);  // 32 * 257^len (a rotation, never p)
    const uint64_t v_last = ring_v[last & (RING - 1)];
    uint64_t acc = v_last >= sp ? v_last - sp : v_last + P61 - sp;
    for (uint32_t m = last; m-- > first;) {
      const uint64_t Pm = qpow_global(qpow, ring_len[m & (RING - 1)] + 1);
      acc = addmod(mulmod(Pm, acc), ring_v[m & (RING - 1)]);
    }
    return acc;
  }
  static __device__ __forceinline__ Value shingle_any(const Value *ring_v, const uint32_t *ring_len,
                                                      const StreamTables &tb, uint32_t first, uint32_t per) {
    return shingle_general(ring_v, ring_len, tb.qpow, first, per);
  }
  // shingle i of the round goes to slot i (16 bytes: the limbs the hash loop multiplies by)
  template <int P>
  static __device__ __forceinline__ void put(uint32_t *sx, uint32_t i, Value x) {
    reinterpret_cast<XLimbs *>(sx)[i] = x_limbs(x);
  }
  template <int P>
  static __device__ __forceinline__ void finish(uint32_t *, uint32_t, uint32_t) {}
  template <int P>
  static __device__ __forceinline__ uint64_t get(const uint32_t *sx, uint32_t i) {
    const XLimbs xv = reinterpret_cast<const XLimbs *>(sx)[i];
    return ((uint64_t)xv.x1 << 31) | xv.x0;
  }
  // the K multiply-adds and minima over the cnt shingles of the round (see k_minhash for the
  // arithmetic); m[] receives the minima, exact
  template <int F, int P>
  static __device__ __forceinline__ void round(const uint32_t *sx_raw, uint32_t cnt, uint32_t grp,
                                               const Coefs<F> &c, const StreamTables &tb, int K, int kbase,
                                               const HotConsts &hc, unsigned long long *slow_tiles,
                                               uint32_t (&m)[F]) {
    constexpr int LW = 64 / P;
    const XLimbs *sx = reinterpret_cast<const XLimbs *>(sx_raw);
    uint32_t mr[F], amb = 0;
#pragma unroll
    for (int j = 0; j < F; j++) mr[j] = 0xFFFFFFFFu;
    auto eval = [&](const XLimbs &xv) {
#pragma unroll
      for (int j = 0; j < F; j++) {
        uint64_t N = (uint64_t)c.a0[j] * xv.x1_4;
        N += (uint64_t)c.a12[j] * xv.x0_2;
        uint64_t U = (uint64_t)c.a12[j] * xv.x1 + c.b[j];
        U += (uint64_t)c.a0[j] * xv.x0;
        const uint64_t Sv = (uint64_t)(uint32_t)N * hc.two29 + U;
        const uint64_t W = (uint64_t)(uint32_t)(Sv >> 32) * hc.eight;  // hi: S >> 61, lo: bits 32..60
        const uint32_t h = (uint32_t)Sv + (uint32_t)(N >> 32) + (uint32_t)(W >> 32);
        amb = max(amb, (uint32_t)W);
        mr[j] = min(mr[j], h);
      }
    };
    const XLimbs *sxg = sx + grp;  // this half-wave's first shingle
    const uint32_t steps = cnt / P;
#pragma unroll(F >= 4 ? 2 : 4)
    for (uint32_t s = 0; s < steps; s++) eval(sxg[s * P]);
    if (P == 2 && (cnt & 1)) eval(sx[cnt - 1]);  // both halves: a repeat cannot change a minimum
    if (__any(amb >= 0xFFFFFFF0u)) {
      // rare: some evaluation sat within reach of a carry across bit 61; redo the round exactly
      if (threadIdx.x == 0 && blockIdx.y == 0) atomicAdd(slow_tiles, 1ull);
#pragma unroll
      for (int j = 0; j < F; j++) {
        mr[j] = 0xFFFFFFFFu;
        const uint64_t a = tb.coef_a[kbase + LW * j < K ? kbase + LW * j : 0];
        for (uint32_t s = grp; s < cnt; s += P) {
          const XLimbs xv = sx[s];
          const uint64_t x = ((uint64_t)xv.x1 << 31) | xv.x0;
          mr[j] = min(mr[j], (uint32_t)addmod(mulmod(a, x), c.b[j]));
        }
      }
    }
#pragma unroll
    for (int j = 0; j < F; j++) m[j] = min(m[j], mr[j]);
  }
};

struct ArithPP {
  using Value = uint32_t;
  // half-wave g reads row g: shingle i sits at row i % P, column i / P; rows are padded with
  // repeats of shingle 0 (a repeat cannot change a minimum) to a multiple of 4 entries
  static constexpr uint32_t ROW_MAX = 64 + 8;
  static constexpr uint32_t SX_WORDS = 2 * (32 + 8) > ROW_MAX ? 2 * (32 + 8) : ROW_MAX;
  template <int F>
  struct Coefs {
    uint32_t a[F], b[F], ap[F];
    uint64_t bp[F];
  };
  template <int F>
  static __device__ __forceinline__ void load(Coefs<F> &c, const StreamTables &tb, int K, int kbase, int LW) {
#pragma unroll
    for (int j = 0; j < F; j++) {
      const int k = kbase + LW * j;
      const uint4 q = *reinterpret_cast<const uint4 *>(tb.coef_pp + (k < K ? k : 0));
      c.a[j] = q.x;
      c.b[j] = q.y;
      c.ap[j] = q.z;
      c.bp[j] = q.w;
    }
  }
  static __device__ __forceinline__ Value token_hash(const uint32_t *sm_text, uint32_t pos, uint32_t flen) {
    constexpr uint32_t R3_PP = R3 % PP;
    // acc <- acc * 257^3 + D modulo p' (the product stays below 2^45 + 2^25)
    auto absorb = [&](uint32_t acc, uint32_t D) { return red_pp((uint64_t)acc * R3_PP + D); };
    uint32_t acc;
    if (!__any(flen > 8)) {
      const TokenDigits t = token_digits8(sm_text, pos, flen);
      acc = absorb(absorb(t.D[2], t.D[1]), t.D[0]);  // D[2] < 2^17
    } else if (!__any(flen > 16)) {
      const TokenDigits t = token_digits16(sm_text, pos, flen);
      acc = absorb(absorb(absorb(absorb(absorb(t.last, t.D[4]), t.D[3]), t.D[2]), t.D[1]), t.D[0]);
    } else {
      acc = 0;
      for (uint32_t k = max_digits(flen); k-- > 0;) acc = absorb(acc, token_digit_at(sm_text, pos, flen, k));
    }
    return acc;
  }
  static __device__ __forceinline__ WalkedToken token_far(const uint8_t *p, uint64_t max_len) {
    return walk_token_far_pp(p, max_len);
  }
  static __device__ __forceinline__ Value with_space(Value w, uint32_t len, const StreamTables &tb) {
    const uint32_t sp = len < (uint32_t)QPOW_N ? tb.ptab_pp[len].sp : mulmod_pp(32u, powmod_pp(257u, len));
    const uint32_t v = w + sp;
    return min(v, v - PP);  // v - p' wraps to a huge value when v < p'
  }
  template <int PER>
  static __device__ __forceinline__ Value shingle_unrolled(const Value *ring_v, const uint32_t *ring_len,
                                                           const StreamTables &tb, uint32_t first,
                                                           const HotConsts &, bool *long_tok) {
    uint32_t len[PER], V[PER];
#pragma unroll
    for (int m = 0; m < PER; m++) {
      len[m] = ring_len[(first + m) & (RING - 1)];
      V[m] = ring_v[(first + m) & (RING - 1)];
    }
    bool lt = false;
#pragma unroll
    for (int m = 0; m < PER; m++) {
      lt |= len[m] >= LONG_TOKEN;
      len[m] = min(len[m], LONG_TOKEN);
    }
    *long_tok = lt;
    PowPP e[PER];
#pragma unroll
    for (int m = 0; m < PER; m++) e[m] = tb.ptab_pp[len[m]];
    uint32_t acc = V[PER - 1] + (PP - e[PER - 1].sp);  // the bare last token
    acc = min(acc, acc - PP);
#pragma unroll
    for (int m = PER - 2; m >= 0; m--) acc = red_pp((uint64_t)acc * e[m].pw1 + V[m]);
    return acc;
  }
  static __device__ __noinline__ Value shingle_general(const Value *ring_v, const uint32_t *ring_len,
                                                       const PowPP *__restrict__ ptab, uint32_t first,
                                                       uint32_t per) {
    const uint32_t last = first + per - 1;
    const uint32_t l_last = ring_len[last & (RING - 1)];
    const uint32_t sp = l_last < (uint32_t)QPOW_N ? ptab[l_last].sp : mulmod_pp(32u, powmod_pp(257u, l_last));
    uint32_t acc = ring_v[last & (RING - 1)] + (PP - sp);
    acc = min(acc, acc - PP);
    for (uint32_t m = last; m-- > first;) {
      const uint32_t lm = ring_len[m & (RING - 1)];
      const uint32_t pw1 = lm < (uint32_t)QPOW_N ? ptab[lm].pw1 : powmod_pp(257u, (uint64_t)lm + 1);
      acc = red_pp((uint64_t)acc * pw1 + ring_v[m & (RING - 1)]);
    }
    return acc;
  }
  static __device__ __forceinline__ Value shingle_any(const Value *ring_v, const uint32_t *ring_len,
                                                      const StreamTables &tb, uint32_t first, uint32_t per) {
    return shingle_general(ring_v, ring_len, tb.ptab_pp, first, per);
  }
  template <int P>
  static __device__ __forceinline__ void put(uint32_t *sx, uint32_t i, Value x) {
    sx[(i % P) * (64 / P + 8) + i / P] = x;
  }
  // pads every row to the longest row rounded up to a multiple of 4 (all lanes call this)
  template <int P>
  static __device__ __forceinline__ void finish(uint32_t *sx, uint32_t cnt, uint32_t lane) {
    const uint32_t cnt0 = (cnt + P - 1) / P, R = (cnt0 + 3) & ~3u;
    if (lane < 8 * P) {
      const uint32_t row = lane / 8, j = lane % 8;
      const uint32_t have = (cnt + P - 1 - row) / P;  // entries of this row
      if (have + j < R) sx[row * (64 / P + 8) + have + j] = sx[0];
    }
  }
  template <int P>
  static __device__ __forceinline__ uint64_t get(const uint32_t *sx, uint32_t i) {
    return sx[(i % P) * (64 / P + 8) + i / P];
  }
  // see k_minhash_pp for the arithmetic: quotient estimate, two 24-bit multiply-adds, and the
  // exact redo of a round whose minimum is within PP_EDGE of p'
  template <int F, int P>
  static __device__ __forceinline__ void round(const uint32_t *sx, uint32_t cnt, uint32_t grp,
                                               const Coefs<F> &c, const StreamTables &, int, int,
                                               const HotConsts &, unsigned long long *, uint32_t (&m)[F]) {
    constexpr uint32_t ROW = 64 / P + 8;
    const uint32_t cnt0 = (cnt + P - 1) / P, R = (cnt0 + 3) & ~3u;
    uint32_t mr[F];
#pragma unroll
    for (int j = 0; j < F; j++) mr[j] = 0xFFFFFFFFu;
    const int neg_p = -(int)PP;
    auto eval = [&](uint32_t x) {
#pragma unroll
      for (int j = 0; j < F; j++) {
        const uint32_t q = (uint32_t)(((uint64_t)x * c.ap[j] + c.bp[j]) >> 32);
        uint32_t sv;
        asm("v_mad_u32_u24 %0, %2, %3, %4\n\tv_mad_i32_i24 %0, %1, %5, %0"
            : "=&v"(sv)
            : "v"(q), "v"(c.a[j]), "v"(x), "v"(c.b[j]), "s"(neg_p));
        mr[j] = min(mr[j], sv);
      }
    };
    const uint4 *row = reinterpret_cast<const uint4 *>(sx + grp * ROW);
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
    for (int j = 0; j < F; j++) redo |= mr[j] >= PP - PP_EDGE;
    if (__any(redo)) {
      // rare: the plain reduction over this half-wave's row
#pragma unroll
      for (int j = 0; j < F; j++) mr[j] = 0xFFFFFFFFu;
      for (uint32_t i = 0; i < R; i++) {
        const uint32_t x = sx[grp * ROW + i];
#pragma unroll
        for (int j = 0; j < F; j++) mr[j] = min(mr[j], red_pp((uint64_t)c.a[j] * x + c.b[j]));
      }
    }
#pragma unroll
    for (int j = 0; j < F; j++) m[j] = min(m[j], mr[j]);
  }
};

template <int F, int P, int SM, typename A>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(8, 8)))
k_minhash_stream(StreamArgs sa, StreamTables tb, int K, uint32_t *__restrict__ sig, HotConsts hc,
                 unsigned long long *__restrict__ slow_tiles, StreamDebug dbg) {
  using Value = typename A::Value;
  __shared__ uint32_t sm_text[SM_TEXT_WORDS];
  __shared__ uint32_t sm_bits[TB / 32 + 4];
  __shared__ uint16_t sm_pos[MAX_TILE_TOKENS];
  __shared__ Value ring_v[RING];
  __shared__ uint32_t ring_len[RING];
  __shared__ __attribute__((aligned(16))) uint32_t sx[A::SX_WORDS];
  const uint32_t lane = threadIdx.x;
  const uint64_t P0 = (uint64_t)blockIdx.x * sa.piece;  // frame position of the piece
  const int64_t PE = (int64_t)sa.piece;                 // its end, relative to P0 like all below
  const uint8_t *pbase = sa.frame + P0;
  const uint32_t n = sa.n;

  // the lane's hash functions, as in k_minhash
  constexpr int LW = 64 / P;
  const uint32_t grp = lane / LW;
  const int kbase = blockIdx.y * (LW * F) + (lane % LW);
  typename A::template Coefs<F> coefs = {};
  uint32_t m[F];
#pragma unroll
  for (int j = 0; j < F; j++) m[j] = 0xFFFFFFFFu;
  if (SM == SM_HASH) A::template load<F>(coefs, tb, K, kbase, LW);

  // First document that reaches into the piece: the smallest d with off[d+1] + shift > P0, found
  // 64 probes at a time (the last piece ends at or before frame_end, so there is one).
  uint64_t d;
  {
    uint64_t lo = 0, hi = sa.n_docs;  // the answer lies in [lo, hi)
    while (hi - lo > 1) {
      const uint64_t span = hi - lo, step = (span + 63) / 64;
      const uint64_t last = lo + min((uint64_t)lane * step + step - 1, span - 1);
      const bool reaches = sa.off[last + 1] + sa.shift > P0;
      const uint64_t votes = __ballot(reaches);  // monotone in the lane; the last lane votes yes
      const uint32_t f = (uint32_t)__ffsll((unsigned long long)votes) - 1u;
      const uint64_t nlo = lo + (uint64_t)f * step;
      hi = min(nlo + step, hi);
      lo = nlo;
    }
    d = lo;
  }
  uint32_t emitted = 0;  // SM_COUNT / SM_WRITE: shingles this piece has produced so far
  const uint32_t out_base = SM == SM_WRITE ? dbg.piece_count[blockIdx.x] : 0u;

  for (; d < sa.n_docs; d++) {
    const int64_t vs = (int64_t)(sa.off[d] + sa.shift - P0);
    const int64_t ve = (int64_t)(sa.off[d + 1] + sa.shift - P0);
    if (vs >= PE) break;  // starts beyond the piece: the next wavefront's
    if (ve <= vs) continue;
    if (SM == SM_COUNT && vs >= 0 && lane == 0) {
      dbg.doc_piece[d] = blockIdx.x;
      dbg.doc_local[d] = emitted;
    }
    uint32_t T = 0;        // tokens of the document seen from this piece
    uint32_t n_owned = 0;  // those that start inside the piece (a prefix of the T)
    uint32_t S_next = 0;   // shingles handled so far: those starting at tokens 0 .. S_next - 1
    uint32_t nsh = 0;      // shingles evaluated for this document
    int64_t cur = vs > 0 ? (vs & ~int64_t(15)) : 0;  // tile start, 16-byte aligned
    bool done = false;

    // takes the cnt shingle hashes that lanes 0 .. cnt-1 have put into sx
    auto consume = [&](uint32_t cnt) {
      A::template finish<P>(sx, cnt, lane);
      __syncthreads();
      if (SM == SM_COUNT) {
        emitted += cnt;
      } else if (SM == SM_WRITE) {
        if (lane < cnt) {
          const uint64_t at = dbg.x_base + out_base + emitted + lane;
          if (at < dbg.x_cap) dbg.x[at] = A::template get<P>(sx, lane);
        }
        emitted += cnt;
      } else {
        A::template round<F, P>(sx, cnt, grp, coefs, tb, K, kbase, hc, slow_tiles, m);
      }
      nsh += cnt;
    };

    while (cur < ve && !done) {
      // ---- pass 1: the tile [cur, cur + TB) of the document, lane = 16 bytes ----
      const uint8_t *tp = pbase + cur;
      const uint32_t vs_t = vs > cur ? (uint32_t)(vs - cur) : 0u;  // the document inside the tile:
      const uint32_t ve_t = ve - cur > int64_t(1) << 30 ? (1u << 30) : (uint32_t)(ve - cur);  // [vs_t, ve_t)
      const uint4 q_own = load_raw16(tp, lane * 16, vs_t, ve_t);
      const uint4 q_la = load_raw16(tp, TB, vs_t, ve_t);  // wave-uniform
      const uint32_t prev_byte = cur > vs ? (uint32_t)tp[-1] : 0x20u;
      const Segment sg = make_segment(q_own, lane * 16, vs_t, ve_t);
      const Segment la = make_segment(q_la, TB, vs_t, ve_t);
      const uint32_t starts0 = token_starts(lane, prev_byte, sg.wm);
      __syncthreads();  // the previous tile's readers are done
      *reinterpret_cast<uint4 *>(&sm_text[lane * 4]) = q_own;
      const uint32_t wm_up = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)sg.wm, 0x130, 0xF, 0xF, false);
      if (!(lane & 1)) sm_bits[lane >> 1] = sg.wm | (wm_up << 16);
      if (lane == 0) {
        *reinterpret_cast<uint4 *>(&sm_text[TB / 4]) = q_la;
        sm_bits[TB / 32] = la.wm;
        sm_bits[TB / 32 + 1] = 0;
        sm_bits[TB / 32 + 2] = 0;
      }
      const uint32_t scnt = __popc(starts0);
      const uint32_t inc = wave_inclusive_scan(scnt);
      const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
      {
        uint32_t stb = starts0, j = inc - scnt;
        while (stb) {
          const uint32_t bit = __ffs(stb) - 1;
          sm_pos[j++] = (uint16_t)(lane * 16 + bit);
          stb &= stb - 1;
        }
      }
      __syncthreads();
      const bool doc_ends_in_view = TB + LOOK >= ve_t;

      // ---- rounds of 64 tokens ----
      for (uint32_t base = 0; base < tot; base += TB_LANES) {
        const uint32_t j = base + lane;
        const bool active = j < tot;
        const uint32_t pos = active ? sm_pos[j] : 0u;
        // 64 bitmap bits from the token's first byte on: its length is the run of ones
        const uint32_t dw = pos >> 5, sh = pos & 31;
        const uint32_t b0 = sm_bits[dw], b1 = sm_bits[dw + 1], b2 = sm_bits[dw + 2];
        const uint32_t w_lo = __builtin_amdgcn_alignbit(b1, b0, sh);
        const uint32_t w_hi = __builtin_amdgcn_alignbit(b2, b1, sh);
        const uint64_t zeros = ~(((uint64_t)w_hi << 32) | w_lo);
        const uint32_t run = zeros ? (uint32_t)(__ffsll((unsigned long long)zeros) - 1) : 64u;
        // the run ends at a real non-token byte (or at the document's end) inside the LDS copy
        const bool fast =
            active && run <= FAST_TOKEN_MAX && (pos + run < TB + LOOK || doc_ends_in_view);
        const uint32_t flen = fast ? run : 0u;
        Value w = A::token_hash(sm_text, pos, flen);
        uint32_t len = flen;
        if (active && !fast) {
          const WalkedToken wt = A::token_far(tp + pos, (uint64_t)(ve - cur - (int64_t)pos));
          w = (Value)wt.w;
          len = wt.len;
        }
        if (active) {
          const uint32_t ri = (T + lane) & (RING - 1);
          ring_v[ri] = A::with_space(w, len, tb);
          ring_len[ri] = len;
        }
        const uint32_t in_round = min((uint32_t)TB_LANES, tot - base);
        n_owned += (uint32_t)__popcll(__ballot(active && cur + (int64_t)pos < PE));
        T += in_round;
        __syncthreads();  // the ring is written
        // shingles whose last token has arrived and whose first token is this piece's
        const uint32_t S_hi = T >= n ? T - n + 1 : 0u;
        const uint32_t S_lim = min(S_hi, n_owned);
        if (S_lim > S_next) {
          const uint32_t cnt = S_lim - S_next;  // at most 64
          if (lane < cnt) {
            const uint32_t first = S_next + lane;
            bool long_tok = false;
            Value x;
            if (n == 5) x = A::template shingle_unrolled<5>(ring_v, ring_len, tb, first, hc, &long_tok);
            else if (n == 3) x = A::template shingle_unrolled<3>(ring_v, ring_len, tb, first, hc, &long_tok);
            else if (n == 4) x = A::template shingle_unrolled<4>(ring_v, ring_len, tb, first, hc, &long_tok);
            else if (n == 2) x = A::template shingle_unrolled<2>(ring_v, ring_len, tb, first, hc, &long_tok);
            else if (n == 1) x = A::template shingle_unrolled<1>(ring_v, ring_len, tb, first, hc, &long_tok);
            else {
              long_tok = true;
              x = 0;
            }
            if (long_tok) x = A::shingle_any(ring_v, ring_len, tb, first, n);
            A::template put<P>(sx, lane, x);
          }
          __syncthreads();
          consume(cnt);
          S_next = S_lim;
        }
      }
      cur += TB;
      // past the end of the piece every owned token is known: stop once their shingles are done
      if (cur >= PE && S_next >= n_owned) done = true;
    }

    // A document of 1 .. n-1 tokens is one shingle of all of them, owned with its first token.
    // Here: the end of the document was reached without a full shingle, and a token of this piece
    // came first in what the piece saw.  It is the document's first token unless the document
    // began before the piece and holds a token byte there.
    if (!done && S_next == 0 && T >= 1 && T < n && n_owned >= 1) {
      bool earlier = false;
      if (vs < 0) {
        for (int64_t q = -1; q >= vs && !earlier; q -= 64) {
          const int64_t pq = q - (int64_t)lane;
          const bool tok_byte = pq >= vs && !is_ws(pbase[pq]);
          earlier = __any(tok_byte);
        }
      }
      if (!earlier) {
        if (lane == 0) A::template put<P>(sx, 0u, A::shingle_any(ring_v, ring_len, tb, 0u, T));
        __syncthreads();
        consume(1u);
      }
    }

    if (SM == SM_HASH && nsh) {
      if (P == 2) {
#pragma unroll
        for (int j = 0; j < F; j++) m[j] = min(m[j], (uint32_t)__shfl_xor(m[j], 32, 64));
      }
      uint32_t *out = sig + d * (uint64_t)K;
      const bool whole = vs >= 0 && ve <= PE;  // no other piece sees this document
#pragma unroll
      for (int j = 0; j < F; j++) {
        const int k = kbase + LW * j;
        if (grp == 0 && k < K) {
          if (whole) {
            out[k] = m[j];
          } else {
            // values only ever decrease: a (possibly stale) read that is not above m[j] settles it
            const uint32_t c = __hip_atomic_load(out + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (m[j] < c) atomicMin(out + k, m[j]);
          }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < F; j++) m[j] = 0xFFFFFFFFu;
    if (ve >= PE) break;  // the document runs to the end of the piece or beyond: nothing after it is ours
  }
  if (SM == SM_COUNT && lane == 0) dbg.piece_count[blockIdx.x] = emitted;
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

// ---- rolling-family mode (SEDD_FLAG_ROLLING_FAMILY) --------------------------------------------
//
// The other reading of "H hash functions" next to Eq. 1: function k is Eq. 1 itself to a base q_k
// of its own, h_k(s) = (sum_i s_i q_k^(i-1) mod p) mod 2^32, q_k = 257 + (a_k mod (p - 257)).
// Nothing is shared between the functions any more: every (shingle, function) pair has to see
// the shingle's characters.  Lane = function (F per lane); the characters are wave-uniform.
//
// Word shingles: a shingle of tokens t_0 .. t_{n-1} joined by single spaces is
//   x = S_0 + P_0 (S_1 + P_1 (... + P_{n-2} T_{n-1})),  T_j = Eq. 1 of token j to the base q_k,
//   S_j = T_j + 32 q_k^len_j (the token and its space),  P_j = q_k^(len_j + 1).
// A lane walks the tile's tokens once: it hashes the new last token from its bytes (len
// multiply-adds), combines it with the n - 1 pairs (S, P) it keeps of the tokens before it
// (n - 1 multiply-adds), and shifts that window by one token.  The powers q_k^e, e <= RF_POW_MAX,
// come from a table laid out [e][k]; longer tokens take a per-lane power.  About len + n
// modular multiply-adds per (shingle, function) against one in the affine family.
// Shingles of more than RF_RING + 1 tokens are hashed from their bytes, token by token.
//
// Byte shingles: Eq. 2, the reuse form, read backwards per function:
//   x(i-1) = q_k (x(i) - c[i+n-1] q_k^(n-1)) + c[i-1]    (two multiply-adds per window).

constexpr int RF_POW_MAX = 64;  // table rows: q_k^0 .. q_k^RF_POW_MAX
constexpr int RF_RING = 4;      // tokens kept per lane: shingles of up to 5 tokens

// q_k and the table of its powers
__global__ void k_coeffs_rf(uint64_t seed, int K, uint64_t *__restrict__ qk,
                            uint64_t *__restrict__ pwtab) {
  int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= K) return;
  const uint64_t s0 = seed % (P61 - 1) + 1;
  const uint64_t ak = mulmod(s0, powmod(G_A, (uint64_t)k + 1));
  const uint64_t q = 257 + ak % (P61 - 257);
  qk[k] = q;
  if (pwtab) {
    uint64_t pw = 1;
    for (int e = 0; e <= RF_POW_MAX; e++) {
      pwtab[(size_t)e * K + k] = pw;
      pw = mulmod(pw, q);
    }
  }
}

struct MulSplit {
  uint32_t a0, a0_2, a12;
};
__device__ __forceinline__ MulSplit mul_split(uint64_t P) {
  MulSplit r;
  r.a0 = (uint32_t)P & 0x7FFFFFFFu;
  r.a0_2 = r.a0 << 1;
  r.a12 = (uint32_t)(P >> 31) << 1;
  return r;
}
// 32 v for v < p: a shift by 5 is a rotation of the 61-bit residue
__device__ __forceinline__ uint64_t mul32_mod(uint64_t v) {
  return ((v << 5) & P61) | (v >> 56);
}

struct RfArgs {
  const uint8_t *pbase;     // chunk text frame
  const uint32_t *tok_pos;  // token positions in the frame (word mode)
  const uint8_t *tok_len;   // min(len, LONG_TOKEN)
  const uint32_t *tok_long; // lengths of the tokens of LONG_TOKEN bytes or more
  const uint32_t *dv;       // document frame positions (byte mode)
  const uint32_t *sbase;    // shingle offsets per document (byte mode)
  const uint64_t *qk;       // bases
  const uint64_t *pwtab;    // [RF_POW_MAX + 1][K] powers
  uint32_t n;               // shingle length
};

template <int F>
struct RfLane {
  uint64_t q[F];   // the lane's bases
  MulSplit qs[F];
  int k[F];        // function index; >= K for a lane with nothing to store
  int col[F];      // its column of the power table (a lane past K reads column 0)
};

// q_k^e for the lane's functions (e is wave-uniform)
template <int F>
__device__ __forceinline__ void rf_powers(const RfArgs &ra, const RfLane<F> &ln, int K, uint32_t e,
                                          uint64_t (&out)[F]) {
#pragma unroll
  for (int j = 0; j < F; j++)
    out[j] = e <= (uint32_t)RF_POW_MAX ? ra.pwtab[(size_t)e * K + ln.col[j]] : powmod(ln.q[j], e);
}

// T = Eq. 1 of the bytes [pos, pos + len) to the lane's bases (Horner from the last byte), added
// on top of acc * q^len: acc <- acc q^len + T.  acc may be lazily reduced (< 2^61 + 8).
template <int F>
__device__ __forceinline__ void rf_absorb_bytes(const RfArgs &ra, const RfLane<F> &ln, uint32_t pos,
                                                uint32_t len, const HotConsts &hc,
                                                uint64_t (&acc)[F]) {
  // the bytes come in as aligned words (the frame starts on a 16-byte boundary and a word that
  // holds one byte of the text lies inside the text's allocation), last word first
  uint32_t i = pos + len;
  while (i > pos) {
    const uint32_t wb = (i - 1) & ~3u;
    const uint32_t w = *reinterpret_cast<const uint32_t *>(ra.pbase + wb);
    const uint32_t lo = max(wb, pos);
    for (uint32_t b = i; b-- > lo;) {
      const uint32_t c = (w >> (8u * (b - wb))) & 0xFFu;
#pragma unroll
      for (int j = 0; j < F; j++)
        acc[j] = horner_step_lazy(acc[j], ln.qs[j].a0, ln.qs[j].a0_2, ln.qs[j].a12, c, hc);
    }
    i = lo;
  }
}

template <int F>
__device__ __forceinline__ void rf_store(const HTile &ht, const RfLane<F> &ln, int K,
                                         uint32_t *__restrict__ sig, const uint32_t (&m)[F]) {
  uint32_t *out = sig + (uint64_t)ht.doc * K;
#pragma unroll
  for (int j = 0; j < F; j++) {
    const int k = ln.k[j];
    if (k < K) {
      if (ht.single) {
        out[k] = m[j];
      } else {
        const uint32_t cur = __hip_atomic_load(out + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (m[j] < cur) atomicMin(out + k, m[j]);
      }
    }
  }
}

template <int F>
__device__ __forceinline__ void rf_lane_init(const RfArgs &ra, int K, RfLane<F> &ln) {
#pragma unroll
  for (int j = 0; j < F; j++) {
    const int k = blockIdx.y * (64 * F) + 64 * j + threadIdx.x;
    ln.k[j] = k;
    ln.col[j] = k < K ? k : 0;  // lanes past K compute function 0 and store nothing
    ln.q[j] = ra.qk[ln.col[j]];
    ln.qs[j] = mul_split(ln.q[j]);
  }
}

template <int F>
__global__ void __launch_bounds__(64)
k_minhash_rf_words(RfArgs ra, const HTile *__restrict__ tiles, const uint32_t *__restrict__ n_tiles,
                   int K, uint32_t *__restrict__ sig, HotConsts hc) {
  const uint32_t t = blockIdx.x;
  const HTile ht = tiles[t];  // the list is allocated for the launch bound: safe past the count
  if (t >= *n_tiles) return;
  RfLane<F> ln;
  rf_lane_init<F>(ra, K, ln);

  const uint32_t per = ht.per, cnt = ht.cnt;
  uint32_t m[F];
#pragma unroll
  for (int j = 0; j < F; j++) m[j] = 0xFFFFFFFFu;

  auto tok_len = [&](uint32_t i) {
    uint32_t l = ra.tok_len[i];
    if (l == LONG_TOKEN) l = ra.tok_long[i];
    return l;
  };

  if (per > (uint32_t)RF_RING + 1) {
    // long shingles: every shingle from its bytes, last token first
    for (uint32_t i = 0; i < cnt; i++) {
      uint64_t x[F];
#pragma unroll
      for (int j = 0; j < F; j++) x[j] = 0;
      for (uint32_t tkn = ht.tok0 + i + per; tkn-- > ht.tok0 + i;) {
        if (tkn != ht.tok0 + i + per - 1) {
#pragma unroll
          for (int j = 0; j < F; j++)  // the space after this token
            x[j] = horner_step_lazy(x[j], ln.qs[j].a0, ln.qs[j].a0_2, ln.qs[j].a12, 32u, hc);
        }
        rf_absorb_bytes<F>(ra, ln, ra.tok_pos[tkn], tok_len(tkn), hc, x);
      }
#pragma unroll
      for (int j = 0; j < F; j++) m[j] = min(m[j], (uint32_t)fold61(x[j]));
    }
    rf_store<F>(ht, ln, K, sig, m);
    return;
  }

  // the window of the per - 1 tokens before the newest one: S (token and its space) and P
  uint64_t S[RF_RING][F], Pw[RF_RING][F];
#pragma unroll
  for (int r = 0; r < RF_RING; r++)
#pragma unroll
    for (int j = 0; j < F; j++) S[r][j] = Pw[r][j] = 0;

  // token -> T (bare), and its (S, P) pair
  auto hash_token = [&](uint32_t tkn, uint64_t (&T)[F], uint64_t (&Sn)[F], uint64_t (&Pn)[F]) {
    const uint32_t len = tok_len(tkn);
#pragma unroll
    for (int j = 0; j < F; j++) T[j] = 0;
    rf_absorb_bytes<F>(ra, ln, ra.tok_pos[tkn], len, hc, T);
    uint64_t ql[F];
    rf_powers<F>(ra, ln, K, len, ql);
    rf_powers<F>(ra, ln, K, len + 1, Pn);
#pragma unroll
    for (int j = 0; j < F; j++) {
      const uint64_t sp = mul32_mod(ql[j]);       // < 2^61
      const uint64_t v = T[j] + sp;                // < 2^62 + 8
      Sn[j] = (v & P61) + (v >> 61);               // < 2^61 + 2
    }
  };

  // warm-up: the first per - 1 tokens fill the window
  for (uint32_t w = 0; w + 1 < per; w++) {
    uint64_t T[F], Sn[F], Pn[F];
    hash_token(ht.tok0 + w, T, Sn, Pn);
#pragma unroll
    for (int r = 0; r < RF_RING; r++) {
      if ((uint32_t)r == w) {
#pragma unroll
        for (int j = 0; j < F; j++) {
          S[r][j] = Sn[j];
          Pw[r][j] = Pn[j];
        }
      }
    }
  }
  for (uint32_t i = 0; i < cnt; i++) {
    uint64_t T[F], Sn[F], Pn[F];
    hash_token(ht.tok0 + i + per - 1, T, Sn, Pn);
    uint64_t x[F];
#pragma unroll
    for (int j = 0; j < F; j++) x[j] = T[j];
#pragma unroll
    for (int r = RF_RING - 1; r >= 0; r--) {
      if ((uint32_t)r + 1 < per) {  // wave-uniform
#pragma unroll
        for (int j = 0; j < F; j++) {
          const MulSplit ps = mul_split(Pw[r][j]);
          x[j] = horner_step_lazy(x[j], ps.a0, ps.a0_2, ps.a12, S[r][j], hc);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < F; j++) m[j] = min(m[j], (uint32_t)fold61(x[j]));
    // shift the window: slot r <- slot r + 1, the newest token enters slot per - 2
#pragma unroll
    for (int r = 0; r < RF_RING; r++) {
#pragma unroll
      for (int j = 0; j < F; j++) {
        if ((uint32_t)r + 2 == per) {
          S[r][j] = Sn[j];
          Pw[r][j] = Pn[j];
        } else if (r + 1 < RF_RING) {
          S[r][j] = S[r + 1][j];
          Pw[r][j] = Pw[r + 1][j];
        }
      }
    }
  }
  rf_store<F>(ht, ln, K, sig, m);
}

template <int F>
__global__ void __launch_bounds__(64)
k_minhash_rf_bytes(RfArgs ra, const HTile *__restrict__ tiles, const uint32_t *__restrict__ n_tiles,
                   int K, uint32_t *__restrict__ sig, HotConsts hc) {
  __shared__ uint32_t sm_b[(TS + SEDD_MAX_SHINGLE_N + 8) / 4 + 1];
  const uint32_t t = blockIdx.x;
  const HTile ht = tiles[t];
  if (t >= *n_tiles) return;
  RfLane<F> ln;
  rf_lane_init<F>(ra, K, ln);
  const uint32_t d = ht.doc, cnt = ht.cnt;
  const uint32_t vs = ra.dv[d], dlen = ra.dv[d + 1] - vs;
  const uint32_t per = min(dlen, ra.n);
  const uint32_t b0 = vs + (ht.x_off - ra.sbase[d]);  // frame position of the first window
  const uint32_t o = b0 & 3u;
  const uint32_t ndw = (o + cnt + per - 1 + 3) >> 2;
  for (uint32_t w = threadIdx.x; w < ndw; w += 64)
    sm_b[w] = *reinterpret_cast<const uint32_t *>(ra.pbase + (b0 - o) + 4 * w);
  __syncthreads();
  const uint8_t *tb = reinterpret_cast<const uint8_t *>(sm_b) + o;  // tb[i] = byte i of the tile

  uint64_t x[F], nqn[F];
  uint32_t m[F];
#pragma unroll
  for (int j = 0; j < F; j++) {
    x[j] = 0;
    nqn[j] = P61 - powmod(ln.q[j], per - 1);  // -q^(per-1), in [1, p - 1]
  }
  // the last window by Horner, then backwards
  for (uint32_t jb = per; jb-- > 0;) {
    const uint32_t c = tb[cnt - 1 + jb];
#pragma unroll
    for (int j = 0; j < F; j++)
      x[j] = horner_step_lazy(x[j], ln.qs[j].a0, ln.qs[j].a0_2, ln.qs[j].a12, c, hc);
  }
#pragma unroll
  for (int j = 0; j < F; j++) m[j] = (uint32_t)fold61(x[j]);
  for (uint32_t i = cnt - 1; i > 0; i--) {
    const uint32_t c_hi = tb[i + per - 1], c_lo = tb[i - 1];
#pragma unroll
    for (int j = 0; j < F; j++) {
      // x(i) - c_hi q^(per-1): c_hi (p - q^(per-1)) < 2^69 is folded in two halves
      const uint64_t lo = (uint64_t)(uint32_t)nqn[j] * c_hi;
      const uint64_t hi = (uint64_t)(uint32_t)(nqn[j] >> 32) * c_hi + (lo >> 32);  // < 2^37
      const uint64_t tq = (((hi & 0x1FFFFFFFull) << 32) | (uint32_t)lo) + (hi >> 29);
      uint64_t dd = x[j] + tq;  // < 2^62 + 2^9
      dd = (dd & P61) + (dd >> 61);
      x[j] = horner_step_lazy(dd, ln.qs[j].a0, ln.qs[j].a0_2, ln.qs[j].a12, c_lo, hc);
      m[j] = min(m[j], (uint32_t)fold61(x[j]));
    }
  }
  rf_store<F>(ht, ln, K, sig, m);
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

// the same for the rolling-family kernels: lane = function, F = 2 functions per lane above K = 64
static int launch_minhash_rf(int byte_mode, const RfArgs &ra, const HTile *tiles,
                             const uint32_t *n_tiles, uint64_t nht, int K, uint32_t *csig,
                             hipStream_t st) {
  const int F = K > 64 ? 2 : 1;
  const HotConsts hc = {1u << 29, 8u, 1u};
  dim3 grid((uint32_t)nht, (uint32_t)((K + 64 * F - 1) / (64 * F)));
  ProfScope prof(SEDD_PROF_MINHASH, st);
#define SEDD_LAUNCH_RF(KERNEL, FF) \
  hipLaunchKernelGGL((KERNEL<FF>), grid, dim3(64), 0, st, ra, tiles, n_tiles, K, csig, hc)
  if (byte_mode) {
    if (F == 2) SEDD_LAUNCH_RF(k_minhash_rf_bytes, 2);
    else SEDD_LAUNCH_RF(k_minhash_rf_bytes, 1);
  } else {
    if (F == 2) SEDD_LAUNCH_RF(k_minhash_rf_words, 2);
    else SEDD_LAUNCH_RF(k_minhash_rf_words, 1);
  }
#undef SEDD_LAUNCH_RF
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

// ---- host driver of the streaming kernel ---------------------------------------------------------

static uint32_t g_piece_bytes_override = 0;

// first and last offset and the validity flag in one 32-byte record
__global__ void k_stream_probe(const uint64_t *__restrict__ off, uint64_t n, uint64_t *__restrict__ out) {
  out[0] = off[0];
  out[1] = off[n];
}

// debug entry: shingle offsets per document from the counting pass.  A non-empty document's
// count was recorded by the piece that holds its first byte; an empty document takes the offset
// of the next non-empty one (or the total).
__global__ void k_stream_soff(const uint64_t *__restrict__ off, uint64_t n_docs,
                              const uint32_t *__restrict__ piece_base,
                              const uint32_t *__restrict__ doc_piece,
                              const uint32_t *__restrict__ doc_local, uint32_t n_pieces,
                              uint64_t *__restrict__ soff) {
  const uint64_t d = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (d > n_docs) return;
  uint64_t e = d;
  while (e < n_docs && off[e + 1] == off[e]) e++;
  soff[d] = e < n_docs ? (uint64_t)piece_base[doc_piece[e]] + doc_local[e]
                       : (uint64_t)piece_base[n_pieces];
}

// ---- state of the streaming path that calls on different streams and threads may share --------
//
// Coefficient sets: the K coefficients of a seed (64-bit values and limb form, or the paper-prime
// form) with the tables 257^i and the per-length Horner multipliers behind them, written once by
// k_coeffs / k_coeffs_pp and only read afterwards.  A set is created on the stream of the call that first asks for it; a call on
// another stream waits for the creating kernel through an event until that event has been seen
// complete.  A call holds its set (TablesLease) from the look-up until its kernels are enqueued;
// when the cache is full, the sets that no call holds are freed after a device synchronisation,
// so no kernel, enqueued or about to be, can still read them.  Probe slots: a small ring of pinned host records that the offset probe and the
// validation kernel write directly, one per call in flight.
struct TableSet {
  int K;
  uint64_t seed;
  bool paper;
  uint8_t *dev;
  hipEvent_t ready;
  bool settled;
  int users;  // calls between look-up and the launch of their last kernel
};
constexpr size_t MAX_TABLE_SETS = 16;
constexpr uint32_t PROBE_SLOTS = 64;
struct ProbeSlot {
  uint64_t off0, offn;
  uint32_t bad, pad[3];
};
static std::mutex g_stream_mutex;
static std::vector<TableSet> g_table_sets;
static ProbeSlot *g_probe_ring = nullptr;
static std::atomic<uint32_t> g_probe_next{0};
static std::atomic<bool> g_probe_busy[PROBE_SLOTS];  // a call holds its record until it has read it

static void tables_release(const uint8_t *dev) {
  std::lock_guard<std::mutex> lock(g_stream_mutex);
  for (TableSet &t : g_table_sets)
    if (t.dev == dev && t.users > 0) {
      t.users--;
      return;
    }
}
struct TablesLease {
  const uint8_t *dev = nullptr;
  ~TablesLease() {
    if (dev) tables_release(dev);
  }
};

static int tables_acquire(int K, uint64_t seed, bool paper, hipStream_t st, StreamTables *out,
                          TablesLease *lease) {
  std::lock_guard<std::mutex> lock(g_stream_mutex);
  Carver cv;
  uint64_t o_a = 0, o_b = 0, o_cs = 0, o_qpow = 0, o_ptab = 0, o_cpp = 0, o_ptpp = 0;
  if (paper) {
    o_cpp = cv.take<CoefPP>(K);
    o_ptpp = cv.take<PowPP>(QPOW_N);
  } else {
    o_a = cv.take<uint64_t>(K);
    o_b = cv.take<uint64_t>(K);
    o_cs = cv.take<CoefSplit>(K);
    o_qpow = cv.take<uint64_t>(QPOW_N);
    o_ptab = cv.take<PowSplit>(QPOW_N);
  }
  *out = StreamTables{};
  auto bind = [&](uint8_t *A) {
    if (paper) {
      out->coef_pp = (const CoefPP *)(A + o_cpp);
      out->ptab_pp = (const PowPP *)(A + o_ptpp);
    } else {
      out->coef_a = (const uint64_t *)(A + o_a);
      out->coef_s = (const CoefSplit *)(A + o_cs);
      out->qpow = (const uint64_t *)(A + o_qpow);
      out->ptab = (const PowSplit *)(A + o_ptab);
    }
  };
  for (TableSet &t : g_table_sets) {
    if (t.K != K || t.seed != seed || t.paper != paper) continue;
    if (!t.settled) {
      if (hipEventQuery(t.ready) == hipSuccess) t.settled = true;
      else SEDD_HIP(hipStreamWaitEvent(st, t.ready, 0));
      (void)hipGetLastError();  // hipEventQuery reports "not ready" as an error value
    }
    bind(t.dev);
    t.users++;
    lease->dev = t.dev;
    return SEDD_OK;
  }
  if (g_table_sets.size() >= MAX_TABLE_SETS) {
    // rare: more distinct (K, seed, modulus) triples than slots.  Sets that a call still holds
    // stay; the others go once nothing enqueued can still read them.
    SEDD_HIP(hipDeviceSynchronize());
    std::vector<TableSet> kept;
    for (TableSet &t : g_table_sets) {
      if (t.users > 0) {
        kept.push_back(t);
        continue;
      }
      (void)hipFree(t.dev);
      (void)hipEventDestroy(t.ready);
    }
    g_table_sets.swap(kept);
  }
  TableSet t;
  t.K = K;
  t.seed = seed;
  t.paper = paper;
  t.settled = false;
  t.users = 1;
  void *p = nullptr;
  if (hipMalloc(&p, cv.off) != hipSuccess) {
    (void)hipGetLastError();
    return SEDD_ENOMEM;
  }
  t.dev = (uint8_t *)p;
  bind(t.dev);
  if (paper)
    hipLaunchKernelGGL(k_coeffs_pp, dim3((std::max(K, QPOW_N) + 255) / 256), dim3(256), 0, st, seed, K,
                       (CoefPP *)(t.dev + o_cpp), (PowPP *)(t.dev + o_ptpp), (uint64_t *)nullptr,
                       (uint64_t *)nullptr);
  else
    hipLaunchKernelGGL(k_coeffs, dim3((std::max(K, QPOW_N) + 255) / 256), dim3(256), 0, st, seed, K,
                       (uint64_t *)(t.dev + o_a), (uint64_t *)(t.dev + o_b),
                       (CoefSplit *)(t.dev + o_cs), (uint64_t *)(t.dev + o_qpow),
                       (PowSplit *)(t.dev + o_ptab));
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipEventCreateWithFlags(&t.ready, hipEventDisableTiming);
  if (e != hipSuccess) {
    // an asynchronous error may stem from the launch above: let it finish before the free
    (void)hipStreamSynchronize(st);
    (void)hipFree(t.dev);
    return set_device_error(e, "coefficient set");
  }
  SEDD_HIP(hipEventRecord(t.ready, st));
  g_table_sets.push_back(t);
  lease->dev = t.dev;
  return SEDD_OK;
}

static int probe_slot_acquire(ProbeSlot **slot) {
  {
    std::lock_guard<std::mutex> lock(g_stream_mutex);
    if (!g_probe_ring) {
      void *p = nullptr;
      if (hipHostMalloc(&p, PROBE_SLOTS * sizeof(ProbeSlot), hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        return SEDD_ENOMEM;
      }
      g_probe_ring = (ProbeSlot *)p;
    }
  }
  // a record nobody holds; with more calls in flight than records, wait for one to come back
  for (;;) {
    for (uint32_t tries = 0; tries < PROBE_SLOTS; tries++) {
      const uint32_t i = g_probe_next.fetch_add(1) % PROBE_SLOTS;
      if (!g_probe_busy[i].exchange(true)) {
        *slot = g_probe_ring + i;
        return SEDD_OK;
      }
    }
    std::this_thread::yield();
  }
}
static void probe_slot_release(ProbeSlot *slot) {
  if (slot) g_probe_busy[slot - g_probe_ring].store(false);
}
struct ProbeLease {
  ProbeSlot *slot = nullptr;
  hipStream_t st = nullptr;
  bool pending = false;  // a kernel that writes the record may still be enqueued
  ~ProbeLease() {
    if (pending) (void)hipStreamSynchronize(st);  // an error path: nobody else gets the record before
    probe_slot_release(slot);
  }
};

// frees the coefficient sets and the probe ring (the device must be idle)
int release_stream_state() {
  std::lock_guard<std::mutex> lock(g_stream_mutex);
  for (TableSet &t : g_table_sets) {
    (void)hipFree(t.dev);
    (void)hipEventDestroy(t.ready);
  }
  g_table_sets.clear();
  if (g_probe_ring) (void)hipHostFree(g_probe_ring);
  g_probe_ring = nullptr;
  return SEDD_OK;
}

// Word shingles with the affine family (61-bit modulus, or the paper's prime with `paper`):
// validation, coefficients, the signature fill and one launch of k_minhash_stream.  One host wait,
// for the first and last offset and the validity flag.  With dbg_off the two debug passes run
// instead.
// host_ends: {doc_offsets[0], doc_offsets[n_docs]} when the caller has the offsets on the host and
// has validated them there (then nothing waits on the device); nullptr otherwise.
static int run_minhash_stream(const uint8_t *bytes, uint64_t n_bytes, const uint64_t *doc_offsets,
                              uint64_t n_docs, int32_t n, int32_t K, uint64_t seed, bool paper,
                              uint32_t *sig, uint64_t *dbg_x, uint64_t dbg_cap, uint64_t *dbg_off,
                              hipStream_t st, const uint64_t *host_ends = nullptr) {
  const bool debug = dbg_off != nullptr;
  const uint64_t max_doc = (uint64_t(1) << 32) - (uint64_t(1) << 30) - (uint64_t(1) << 16);
  int rc;
  uint64_t off0, offn;
  if (host_ends) {
    off0 = host_ends[0];
    offn = host_ends[1];
  } else {
    // the probe and the validation kernel write straight into a pinned host record
    ProbeLease held;  // given back when this block has read the record
    rc = probe_slot_acquire(&held.slot);
    if (rc) return rc;
    ProbeSlot *slot = held.slot;
    held.st = st;
    slot->off0 = slot->offn = 0;
    slot->bad = 0;
    held.pending = true;
    hipLaunchKernelGGL(k_stream_probe, dim3(1), dim3(1), 0, st, doc_offsets, n_docs, &slot->off0);
    SEDD_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_validate_offsets, dim3((uint32_t)((n_docs + 255) / 256)), dim3(256), 0, st,
                       doc_offsets, n_docs, max_doc, &slot->bad);
    SEDD_LAUNCH_CHECK();
    SEDD_HIP(hipStreamSynchronize(st));
    held.pending = false;
    off0 = slot->off0;
    offn = slot->offn;
    if (slot->bad) return SEDD_EINVAL;
  }
  if (offn < off0 || offn > n_bytes) return SEDD_EINVAL;
  if (offn > off0 && !bytes) return SEDD_EINVAL;

  // the frame: 16-byte aligned, at or below the first byte of document 0
  const uintptr_t first_byte = (uintptr_t)bytes + off0;
  const uint64_t lead = first_byte & 15;
  StreamArgs sa;
  sa.frame = (const uint8_t *)(first_byte - lead);
  sa.off = doc_offsets;
  sa.n_docs = n_docs;
  sa.shift = lead - off0;  // wraps; off[d] + shift is the frame position
  sa.frame_end = lead + (offn - off0);
  sa.n = (uint32_t)n;
  // piece size: enough pieces to fill the chip several times over, few enough that the work per
  // piece outweighs its start-up (document search, coefficient loads, the tokens read past its end)
  uint32_t piece = g_piece_bytes_override;
  if (!piece) {
    piece = (uint32_t)std::min<uint64_t>(8192, (sa.frame_end / 32768) & ~uint64_t(TB - 1));
    if (piece < TB) piece = TB;
  }
  sa.piece = piece;
  const uint64_t n_pieces = offn > off0 ? (sa.frame_end + piece - 1) / piece : 0;
  if (n_pieces >= (uint64_t(1) << 31)) return SEDD_EINVAL;

  StreamTables tb;
  TablesLease lease;  // released when this call has enqueued its kernels
  rc = tables_acquire((int)K, seed, paper, st, &tb, &lease);
  if (rc) return rc;
  // the two debug passes keep their counters in the arena (they are not meant to run concurrently)
  Carver cv;
  uint64_t o_pc = 0, o_dp = 0, o_dl = 0, o_tmp = 0;
  uint8_t *A = nullptr;
  if (debug) {
    o_pc = cv.take<uint32_t>(n_pieces + 1);
    o_dp = cv.take<uint32_t>(n_docs);
    o_dl = cv.take<uint32_t>(n_docs);
    o_tmp = cv.take<uint32_t>(scan_tmp_count(n_pieces + 1));
    rc = scratch_ensure(cv.off, &A);
    if (rc) return rc;
  }
  const HotConsts hc = {1u << 29, 8u, 1u};
  StreamDebug dbg = {};

  if (debug) {
    if (n_pieces >= (uint64_t(1) << 31) || sa.frame_end >= (uint64_t(1) << 32)) return SEDD_EINVAL;
    uint32_t *pc = (uint32_t *)(A + o_pc);
    dbg.piece_count = pc;
    dbg.doc_piece = (uint32_t *)(A + o_dp);
    dbg.doc_local = (uint32_t *)(A + o_dl);
    dbg.x = dbg_x;
    dbg.x_cap = dbg_cap;
    dbg.x_base = 0;
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, pc + n_pieces, (uint64_t)1, 0u);
    SEDD_LAUNCH_CHECK();
#define SEDD_LAUNCH_STREAM_DBG(SM)                                                                \
  do {                                                                                           \
    if (paper)                                                                                   \
      hipLaunchKernelGGL((k_minhash_stream<1, 1, SM, ArithPP>), dim3((uint32_t)n_pieces), dim3(64), \
                         0, st, sa, tb, 1, (uint32_t *)nullptr, hc, (unsigned long long *)nullptr, dbg); \
    else                                                                                         \
      hipLaunchKernelGGL((k_minhash_stream<1, 1, SM, Arith61>), dim3((uint32_t)n_pieces), dim3(64), \
                         0, st, sa, tb, 1, (uint32_t *)nullptr, hc, (unsigned long long *)nullptr, dbg); \
  } while (0)
    if (n_pieces) {
      SEDD_LAUNCH_STREAM_DBG(SM_COUNT);
      SEDD_LAUNCH_CHECK();
    }
    rc = scan_exclusive_u32(pc, pc, n_pieces + 1, (uint32_t *)(A + o_tmp), st);
    if (rc) return rc;
    hipLaunchKernelGGL(k_stream_soff, dim3((uint32_t)((n_docs + 1 + 255) / 256)), dim3(256), 0, st,
                       doc_offsets, n_docs, pc, dbg.doc_piece, dbg.doc_local, (uint32_t)n_pieces,
                       dbg_off);
    SEDD_LAUNCH_CHECK();
    if (dbg_cap && n_pieces) {
      SEDD_LAUNCH_STREAM_DBG(SM_WRITE);
      SEDD_LAUNCH_CHECK();
    }
#undef SEDD_LAUNCH_STREAM_DBG
    return SEDD_OK;
  }

  unsigned long long *stats = nullptr;
  rc = stats_ensure(&stats);
  if (rc) return rc;
  {
    const uint64_t nsig = n_docs * (uint64_t)K;
    const uint32_t grid = (uint32_t)std::min<uint64_t>((nsig + 255) / 256, 65536);
    hipLaunchKernelGGL(k_fill_u32, dim3(grid), dim3(256), 0, st, sig, nsig, 0xFFFFFFFFu);
    SEDD_LAUNCH_CHECK();
  }
  if (!n_pieces) return SEDD_OK;
  // functions per lane F and half-wave split P as in launch_minhash
  const int P = K <= 128 ? 2 : 1;
  const int F = K <= 32 ? 1 : (K <= 64 ? 2 : 4);
  const int per_block = (64 / P) * F;
  dim3 grid((uint32_t)n_pieces, (uint32_t)((K + per_block - 1) / per_block));
  ProfScope prof(SEDD_PROF_MINHASH, st);
#define SEDD_LAUNCH_STREAM(FF, HW)                                                               \
  do {                                                                                           \
    if (paper)                                                                                   \
      hipLaunchKernelGGL((k_minhash_stream<FF, HW, SM_HASH, ArithPP>), grid, dim3(64), 0, st, sa, tb, \
                         (int)K, sig, hc, stats + SEDD_STAT_SLOW_TILES, dbg);                    \
    else                                                                                         \
      hipLaunchKernelGGL((k_minhash_stream<FF, HW, SM_HASH, Arith61>), grid, dim3(64), 0, st, sa, tb, \
                         (int)K, sig, hc, stats + SEDD_STAT_SLOW_TILES, dbg);                    \
  } while (0)
  if (P == 1) SEDD_LAUNCH_STREAM(4, 1);
  else if (F == 1) SEDD_LAUNCH_STREAM(1, 2);
  else if (F == 2) SEDD_LAUNCH_STREAM(2, 2);
  else SEDD_LAUNCH_STREAM(4, 2);
#undef SEDD_LAUNCH_STREAM
  SEDD_LAUNCH_CHECK();
  return SEDD_OK;
}

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
                             : (byte_mode ? (uint64_t(128) << 20) : (uint64_t(256) << 20));
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
      if (hipMalloc(&p, tb) != hipSuccess || hipMalloc(&q, oc * sizeof(uint64_t)) != hipSuccess) {
        (void)hipGetLastError();
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
  g_piece_bytes_override = bytes;
  return SEDD_OK;
}

}  // extern "C"
