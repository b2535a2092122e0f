// Device-side definitions shared by the translation units of sedd_minhash: the limb forms of
// Eq. 1 values and coefficients, the arithmetic modulo the paper's prime, the tokenisation
// helpers, the lazily reduced Horner steps, the work-list records, and the declarations of what
// one unit launches or calls from another.
//   sedd_minhash.hip         entry points, coefficients, byte shingles (shingle tiles), text in
//                            host memory
//   sedd_minhash_stream.hip  word shingles with the affine family: the streaming kernel
//   sedd_minhash_rf.hip      the rolling-family mode
#ifndef SEDD_MINHASH_DEVICE_H
#define SEDD_MINHASH_DEVICE_H

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

// ---- tokenisation helpers ------------------------------------------------------------------

// The 16 bytes of one thread's segment and the mask of its token bytes (bit i: byte seg+i lies
// inside the document [vs, ve) and is not whitespace).  seg is 16-aligned; the load is issued
// only if the segment holds at least one byte of the document.
struct Segment {
  uint32_t w[4];
  uint32_t wm;
};
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

constexpr uint32_t LOOK = 16;
constexpr uint32_t MAX_TILE_TOKENS = TB / 2 + 2;
constexpr uint32_t FAST_TOKEN_MAX = 63;  // longest token finished from LDS
// text in LDS: tile + look-ahead + slack for the (masked) reads of lanes whose token is shorter
// than the wavefront's longest
constexpr uint32_t SM_TEXT_WORDS = (TB + LOOK + FAST_TOKEN_MAX + 9) / 4 + 2;

// The multipliers 2^29, 8 and 1 of the hash loops are passed as kernel arguments so that they
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

// ---- kernels and host routines that more than one translation unit uses -----------------------

// defined in sedd_minhash.hip
__global__ void k_fill_u32(uint32_t *p, uint64_t n, uint32_t v);
__global__ void k_coeffs(uint64_t seed, int K, uint64_t *a, uint64_t *b, CoefSplit *split,
                         uint64_t *qpow, PowSplit *ptab);
__global__ void k_coeffs_pp(uint64_t seed, int K, CoefPP *coef, PowPP *ptab, uint64_t *raw_a,
                            uint64_t *raw_b);
__global__ void k_validate_offsets(const uint64_t *__restrict__ off, uint64_t n, uint64_t max_doc,
                                   uint32_t *__restrict__ bad);

// sedd_minhash_stream.hip.  Word shingles with the affine family (61-bit modulus, or the paper's
// prime with `paper`): validation, coefficients, the signature fill and one launch of
// k_minhash_stream.  With dbg_off the two debug passes run instead.  host_ends:
// {doc_offsets[0], doc_offsets[n_docs]} when the caller has the offsets on the host and has
// validated them there (then nothing waits on the device); nullptr otherwise.
int run_minhash_stream(const uint8_t *bytes, uint64_t n_bytes, const uint64_t *doc_offsets,
                       uint64_t n_docs, int32_t n, int32_t K, uint64_t seed, bool paper,
                       uint32_t *sig, uint64_t *dbg_x, uint64_t dbg_cap, uint64_t *dbg_off,
                       hipStream_t st, const uint64_t *host_ends = nullptr);
void set_piece_bytes_override(uint32_t bytes);  // 0: the built-in choice

// sedd_minhash_rf.hip
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
constexpr int RF_POW_MAX = 64;  // table rows: q_k^0 .. q_k^RF_POW_MAX
__global__ void k_coeffs_rf(uint64_t seed, int K, uint64_t *__restrict__ qk,
                            uint64_t *__restrict__ pwtab);
int launch_minhash_rf(int byte_mode, const RfArgs &ra, const HTile *tiles, const uint32_t *n_tiles,
                      uint64_t nht, int K, uint32_t *csig, hipStream_t st);

}  // namespace sedd

#endif
