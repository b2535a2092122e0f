// sedd_minhash with SEDD_FLAG_ROLLING_FAMILY: the kernels of the mode whose K functions are Eq. 1
// to K bases.  Tiles, token records and work lists come from the chunk driver in sedd_minhash.hip.
#include "sedd_minhash_device.h"

namespace sedd {

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

// launches the kernel over nht candidate tiles (tiles beyond the device-side count exit):
// lane = function, F = 2 functions per lane above K = 64
int launch_minhash_rf(int byte_mode, const RfArgs &ra, const HTile *tiles, const uint32_t *n_tiles,
                      uint64_t nht, int K, uint32_t *csig, hipStream_t st) {
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

}  // namespace sedd
