// sedd_minhash on word shingles with the affine family (the default 61-bit modulus and the
// paper's own prime): k_minhash_stream, one launch from raw text to signatures, and its host side
// (coefficient sets, offset probe, piece size, the two debug passes).
#include <algorithm>
#include <atomic>
#include <mutex>
#include <thread>
#include <vector>

#include "sedd_minhash_device.h"

namespace sedd {

// ---- the streaming kernel (word shingles, affine family) ------------------------------------------
//
// The whole of sedd_minhash in one launch, for the default mode and the paper-prime mode (the
// template argument A holds what depends on the modulus): the text is read from HBM once,
// nothing but the signatures is written, and there is no work list.  The text (a frame that
// starts on a 16-byte boundary at or below document 0) is cut into pieces of `piece` bytes; one
// wavefront owns the tokens that START inside its piece, in document order, and with them the
// shingles that start at those tokens.  Per document that reaches into the piece it walks
// 1 KiB tiles of the document's bytes:
//   pass 1 (lane = 16 bytes)   token-byte bitmap into LDS, token starts ranked with a wave prefix sum;
//   rounds of 64 tokens        lane = token: Eq. 1 of the token from the LDS copy of the tile, the
//                              record (hash of "token 0x20", length) goes into a ring in LDS;
//                              lane = shingle: x(s) by Horner over its n ring records, into LDS;
//                              lane = hash function: the K multiply-adds and the running minimum
//                              over the round's shingles, the loop of k_minhash (sedd_minhash.hip).
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
  // the K multiply-adds and minima over the cnt shingles of the round (the arithmetic is
  // described above k_minhash in sedd_minhash.hip); m[] receives the minima, exact
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
  // see k_minhash_pp (sedd_minhash.hip) for the arithmetic: quotient estimate, two 24-bit multiply-adds, and the
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

  // the lane's hash functions: F per lane, LW lanes per grid row
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

// ---- host driver of the streaming kernel ---------------------------------------------------------

static uint32_t g_piece_bytes_override = 0;
void set_piece_bytes_override(uint32_t bytes) { g_piece_bytes_override = bytes; }

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
  hipError_t e = hipMalloc(&p, cv.off);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    set_device_error(e, "hipMalloc(coefficient tables)");
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
  e = hipGetLastError();
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
      const hipError_t e = hipHostMalloc(&p, PROBE_SLOTS * sizeof(ProbeSlot), hipHostMallocDefault);
      if (e != hipSuccess) {
        (void)hipGetLastError();
        set_device_error(e, "hipHostMalloc(offset probe records)");
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
int run_minhash_stream(const uint8_t *bytes, uint64_t n_bytes, const uint64_t *doc_offsets,
                       uint64_t n_docs, int32_t n, int32_t K, uint64_t seed, bool paper,
                       uint32_t *sig, uint64_t *dbg_x, uint64_t dbg_cap, uint64_t *dbg_off,
                       hipStream_t st, const uint64_t *host_ends) {
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
  // functions per lane F and half-wave split P: K <= 32: (1,2), <= 64: (2,2), <= 128: (4,2),
  // larger: (4,1) with one grid row per 256 functions
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

}  // namespace sedd
