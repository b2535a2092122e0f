/*
 * CPU oracle for MinHash-LSH deduplication: signatures, band keys, clusters.
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT.  Plain, slow, single-threaded C that
 * writes the definitions out directly.  Only the test-suite, the smoke check
 * and the benchmark's CPU-baseline leg may call it.  It shares no code with
 * the HIP library and includes none of its headers.
 *
 * What it follows (SEDD paper):
 *   - Section 2.2 "MinHash generation": shingle every document, apply H hash
 *     functions to every shingle, keep the minimum per function.
 *   - Section 3.2 Eq. 1: the shingle hash h(s) = (sum_i c_i q^(i-1)) mod p
 *     with c_i the characters of the shingle.  It is evaluated here directly
 *     from Eq. 1 for every shingle; the reuse of Eq. 2 is an optimisation
 *     that yields the same integer and is deliberately not used.
 *   - Section 2.3 / Appendix A.2: split the signature into b bands of r
 *     values, hash each band; documents sharing a band hash in the same band
 *     are linked.
 *   - Section 2.2 "Constructing a union graph" and "Generating the final
 *     list": connected components; the representative is the lowest index.
 *
 * Readings fixed where the paper leaves a choice (all integer, all exact):
 *   p = 2^61 - 1, q = 257, characters are raw byte values 0..255.
 *   H hash functions: h_k(s) = ((a_k * x(s) + b_k) mod p) mod 2^32, where
 *   x(s) is Eq. 1's value; a_k = s0 * Ga^(k+1) mod p, b_k = s0 * Gb^(k+1)
 *   mod p, s0 = (seed mod (p-1)) + 1.
 *   Word shingles: tokens are maximal runs of bytes outside
 *   {09,0A,0B,0C,0D,20}; a shingle is n consecutive tokens joined by one 20.
 *   A document with 1..n-1 tokens has one shingle made of all of them; with
 *   none it has no shingle and its signature is all 0xFFFFFFFF.
 *   Byte shingles: every window of n bytes; a document of 1..n-1 bytes has
 *   one shingle (the whole document).
 *   Band key: Eq. 1's polynomial over the band's r values with base Q, mod p.
 *   Paper-prime mode (flags bit 1): Section 3.2 names p' = 4,294,967 as the
 *   modulus of its experiments.  With that bit set, Eq. 1 is taken mod p'
 *   and the H functions are h'_k(s) = (a'_k * x'(s) + b'_k) mod p' with
 *   a'_k = (a_k mod (p'-1)) + 1 and b'_k = b_k mod p' (a_k, b_k as above);
 *   the value is below 2^23 and is stored as it is.
 *   Rolling-family mode (flags bit 2): the other way to read "H hash
 *   functions" next to Eq. 1: every function is Eq. 1 itself with a base of
 *   its own, h_k(s) = (sum_i s_i * q_k^(i-1) mod p) mod 2^32 with
 *   q_k = 257 + (a_k mod (p - 257)), a base above the alphabet size as
 *   Section 3.2 asks; p = 2^61 - 1.  b_k is not used.  Not combinable with
 *   the paper-prime bit.
 *
 * Parity with the paper authors' released code is unpinned: the paper prints
 * no hash value, signature or bucket id for any input.  The functions here
 * are pinned by the CPU test-suite against closed forms, big-integer
 * arithmetic, brute-force Jaccard / connected components and the LSH
 * collision-probability curve.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define SEDD_REF_OK 0
#define SEDD_REF_EINVAL (-1)
#define SEDD_REF_ENOMEM (-2)

typedef unsigned __int128 u128;

static const uint64_t P61 = 2305843009213693951ULL;  /* 2^61 - 1 */
static const uint64_t Q_CHAR = 257ULL;                /* Eq. 1 base, > 255 */
static const uint64_t Q_BAND = 1687994237021934823ULL;
static const uint64_t G_A = 1425089352415399810ULL;
static const uint64_t G_B = 955111447119501601ULL;

/* x mod (2^61-1) for x < 2^125, using 2^61 = 1 (mod p) */
static uint64_t mod_p(u128 x) {
  u128 y = (x & P61) + (x >> 61);          /* < 2^61 + 2^64 */
  uint64_t z = (uint64_t)(y & P61) + (uint64_t)(y >> 61);
  while (z >= P61) z -= P61;
  return z;
}

static uint64_t mulmod(uint64_t a, uint64_t b) { return mod_p((u128)a * b); }
static uint64_t addmod(uint64_t a, uint64_t b) { return mod_p((u128)a + b); }

/* exported for the arithmetic pins */
uint64_t sedd_ref_mulmod(uint64_t a, uint64_t b) { return mulmod(a, b); }
uint64_t sedd_ref_addmod(uint64_t a, uint64_t b) { return addmod(a, b); }

uint64_t sedd_ref_powmod(uint64_t g, uint64_t e) {
  uint64_t r = 1;
  for (uint64_t i = 0; i < e; i++) r = mulmod(r, g);  /* plain repeated product */
  return r;
}

/* Eq. 1: x(s) = sum_{i=1..len} s_i * q^(i-1) mod p, first character at q^0 */
uint64_t sedd_ref_base_hash(const uint8_t *s, uint64_t len) {
  uint64_t x = 0, pw = 1;
  for (uint64_t i = 0; i < len; i++) {
    x = addmod(x, mulmod((uint64_t)s[i], pw));
    pw = mulmod(pw, Q_CHAR);
  }
  return x;
}

/* ---- paper-prime mode: the modulus Section 3.2 quotes for the paper's experiments ---- */

static const uint64_t P_PAPER = 4294967ULL;

/* Eq. 1 with p' in place of p */
uint64_t sedd_ref_base_hash_pp(const uint8_t *s, uint64_t len) {
  uint64_t x = 0, pw = 1;
  for (uint64_t i = 0; i < len; i++) {
    x = (x + (uint64_t)s[i] * pw) % P_PAPER;    /* < 2^8 * 2^23 + 2^23: no overflow */
    pw = (pw * Q_CHAR) % P_PAPER;
  }
  return x;
}

/* Eq. 1 with an arbitrary base q < p */
uint64_t sedd_ref_base_hash_q(const uint8_t *s, uint64_t len, uint64_t q) {
  uint64_t x = 0, pw = 1;
  for (uint64_t i = 0; i < len; i++) {
    x = addmod(x, mulmod((uint64_t)s[i], pw));
    pw = mulmod(pw, q);
  }
  return x;
}

/* coefficients of the K hash functions */
int sedd_ref_coeffs(uint64_t seed, int32_t K, uint64_t *a, uint64_t *b) {
  if (K < 1 || !a || !b) return SEDD_REF_EINVAL;
  uint64_t s0 = seed % (P61 - 1) + 1;
  uint64_t ga = 1, gb = 1;
  for (int32_t k = 0; k < K; k++) {
    ga = mulmod(ga, G_A);   /* Ga^(k+1) */
    gb = mulmod(gb, G_B);
    a[k] = mulmod(s0, ga);
    b[k] = mulmod(s0, gb);
  }
  return SEDD_REF_OK;
}

/* paper-prime coefficients: a'_k in [1, p'-1], b'_k in [0, p'-1] */
int sedd_ref_coeffs_pp(uint64_t seed, int32_t K, uint64_t *a, uint64_t *b) {
  int rc = sedd_ref_coeffs(seed, K, a, b);
  if (rc) return rc;
  for (int32_t k = 0; k < K; k++) {
    a[k] = a[k] % (P_PAPER - 1) + 1;
    b[k] = b[k] % P_PAPER;
  }
  return SEDD_REF_OK;
}

/* bases of the rolling-family mode: q_k in [257, p-1] */
int sedd_ref_bases(uint64_t seed, int32_t K, uint64_t *q) {
  if (K < 1 || !q) return SEDD_REF_EINVAL;
  uint64_t *b = (uint64_t *)malloc((size_t)K * 8);
  if (!b) return SEDD_REF_ENOMEM;
  sedd_ref_coeffs(seed, K, q, b);
  for (int32_t k = 0; k < K; k++) q[k] = 257 + q[k] % (P61 - 257);
  free(b);
  return SEDD_REF_OK;
}

/* the shingle hash of the mode: q is the base where flags bit 2 is set, else ignored */
static uint64_t shingle_hash(const uint8_t *s, uint64_t len, uint32_t flags, uint64_t q) {
  if (flags & 4u) return sedd_ref_base_hash_q(s, len, q);
  return (flags & 2u) ? sedd_ref_base_hash_pp(s, len) : sedd_ref_base_hash(s, len);
}

static int is_space(uint8_t c) { return c == 0x20 || (c >= 0x09 && c <= 0x0D); }

/*
 * Base hashes of the shingles of one document, in document order.
 * Returns the number of shingles; writes at most cap of them to out
 * (out may be NULL to count only).
 */
static uint64_t doc_shingles_q(const uint8_t *t, uint64_t len, int32_t n, uint32_t flags,
                               uint64_t q, uint64_t *out, uint64_t cap) {
  uint64_t count = 0;
  if (n < 1) return 0;
  if (flags & 1u) {                                   /* byte n-grams */
    if (len == 0) return 0;
    if (len < (uint64_t)n) { if (out && cap) out[0] = shingle_hash(t, len, flags, q); return 1; }
    for (uint64_t i = 0; i + n <= len; i++) {
      if (out && count < cap) out[count] = shingle_hash(t + i, (uint64_t)n, flags, q);
      count++;
    }
    return count;
  }
  /* word n-grams: token list first */
  uint64_t n_tok = 0, i = 0;
  while (i < len) {
    while (i < len && is_space(t[i])) i++;
    if (i == len) break;
    while (i < len && !is_space(t[i])) i++;
    n_tok++;
  }
  if (n_tok == 0) return 0;
  uint64_t *ts = (uint64_t *)malloc(n_tok * 8), *tl = (uint64_t *)malloc(n_tok * 8);
  uint64_t k = 0; i = 0;
  while (i < len) {
    while (i < len && is_space(t[i])) i++;
    if (i == len) break;
    uint64_t s = i;
    while (i < len && !is_space(t[i])) i++;
    ts[k] = s; tl[k] = i - s; k++;
  }
  uint64_t per = n_tok < (uint64_t)n ? n_tok : (uint64_t)n;   /* tokens per shingle */
  uint64_t n_sh = n_tok - per + 1;
  uint8_t *buf = NULL; uint64_t bcap = 0;
  for (uint64_t s = 0; s < n_sh; s++) {
    uint64_t need = per - 1;
    for (uint64_t j = 0; j < per; j++) need += tl[s + j];
    if (need > bcap) { bcap = need * 2; buf = (uint8_t *)realloc(buf, bcap); }
    uint64_t w = 0;
    for (uint64_t j = 0; j < per; j++) {
      if (j) buf[w++] = 0x20;
      memcpy(buf + w, t + ts[s + j], tl[s + j]); w += tl[s + j];
    }
    if (out && count < cap) out[count] = shingle_hash(buf, w, flags, q);
    count++;
  }
  free(buf); free(ts); free(tl);
  return count;
}

uint64_t sedd_ref_doc_shingles(const uint8_t *t, uint64_t len, int32_t n, uint32_t flags,
                               uint64_t *out, uint64_t cap) {
  return doc_shingles_q(t, len, n, flags & 3u, 0, out, cap);
}

/* the same with Eq. 1 taken to the base q (rolling-family mode) */
uint64_t sedd_ref_doc_shingles_q(const uint8_t *t, uint64_t len, int32_t n, uint32_t flags,
                                 uint64_t q, uint64_t *out, uint64_t cap) {
  return doc_shingles_q(t, len, n, (flags & 1u) | 4u, q, out, cap);
}

/*
 * Signature of a document given the base hashes of its shingles (a multiset;
 * order and repetition do not matter).  sig holds K values.
 */
int sedd_ref_minhash_shingles(const uint64_t *x, uint64_t n_sh, int32_t K, uint64_t seed,
                              uint32_t *sig) {
  if (K < 1 || !sig || (n_sh && !x)) return SEDD_REF_EINVAL;
  uint64_t *a = (uint64_t *)malloc((size_t)K * 8), *b = (uint64_t *)malloc((size_t)K * 8);
  if (!a || !b) { free(a); free(b); return SEDD_REF_ENOMEM; }
  sedd_ref_coeffs(seed, K, a, b);
  for (int32_t k = 0; k < K; k++) {
    uint32_t m = 0xFFFFFFFFu;
    for (uint64_t s = 0; s < n_sh; s++) {
      uint64_t h = addmod(mulmod(a[k], x[s]), b[k]);
      uint32_t h32 = (uint32_t)(h & 0xFFFFFFFFu);
      if (h32 < m) m = h32;
    }
    sig[k] = m;
  }
  free(a); free(b);
  return SEDD_REF_OK;
}

/* the same with the paper-prime functions h'_k */
int sedd_ref_minhash_shingles_pp(const uint64_t *x, uint64_t n_sh, int32_t K, uint64_t seed,
                                 uint32_t *sig) {
  if (K < 1 || !sig || (n_sh && !x)) return SEDD_REF_EINVAL;
  uint64_t *a = (uint64_t *)malloc((size_t)K * 8), *b = (uint64_t *)malloc((size_t)K * 8);
  if (!a || !b) { free(a); free(b); return SEDD_REF_ENOMEM; }
  sedd_ref_coeffs_pp(seed, K, a, b);
  for (int32_t k = 0; k < K; k++) {
    uint32_t m = 0xFFFFFFFFu;
    for (uint64_t s = 0; s < n_sh; s++) {
      uint64_t h = (a[k] * (x[s] % P_PAPER) + b[k]) % P_PAPER;   /* < 2^46: no overflow */
      if ((uint32_t)h < m) m = (uint32_t)h;
    }
    sig[k] = m;
  }
  free(a); free(b);
  return SEDD_REF_OK;
}

/* sig[d*K + k] = min over the shingles s of document d of h_k(s) */
int sedd_ref_minhash(const uint8_t *bytes, const uint64_t *doc_offsets, uint64_t n_docs,
                     int32_t shingle_n, int32_t K, uint64_t seed, uint32_t flags,
                     uint32_t *sig) {
  if (shingle_n < 1 || K < 1 || (flags & ~7u) || (flags & 6u) == 6u) return SEDD_REF_EINVAL;
  if (n_docs == 0) return SEDD_REF_OK;
  if (!doc_offsets || !sig) return SEDD_REF_EINVAL;
  for (uint64_t d = 0; d < n_docs; d++)
    if (doc_offsets[d + 1] < doc_offsets[d]) return SEDD_REF_EINVAL;
  if (doc_offsets[n_docs] > doc_offsets[0] && !bytes) return SEDD_REF_EINVAL;
  uint64_t *x = NULL, xcap = 0;
  uint64_t *qk = NULL;
  if (flags & 4u) {
    qk = (uint64_t *)malloc((size_t)K * 8);
    if (!qk) return SEDD_REF_ENOMEM;
    sedd_ref_bases(seed, K, qk);
  }
  for (uint64_t d = 0; d < n_docs; d++) {
    const uint8_t *t = bytes + doc_offsets[d];
    uint64_t len = doc_offsets[d + 1] - doc_offsets[d];
    uint64_t n_sh = doc_shingles_q(t, len, shingle_n, flags, 257, NULL, 0);
    if (n_sh > xcap) { xcap = n_sh * 2; free(x); x = (uint64_t *)malloc(xcap * 8); if (!x) { free(qk); return SEDD_REF_ENOMEM; } }
    if (flags & 4u) {
      /* every function hashes the shingles itself, with its own base */
      for (int32_t k = 0; k < K; k++) {
        doc_shingles_q(t, len, shingle_n, flags, qk[k], x, n_sh);
        uint32_t m = 0xFFFFFFFFu;
        for (uint64_t s = 0; s < n_sh; s++) {
          uint32_t h32 = (uint32_t)(x[s] & 0xFFFFFFFFu);
          if (h32 < m) m = h32;
        }
        sig[d * (uint64_t)K + k] = m;
      }
      continue;
    }
    sedd_ref_doc_shingles(t, len, shingle_n, flags, x, n_sh);
    int rc = (flags & 2u) ? sedd_ref_minhash_shingles_pp(x, n_sh, K, seed, sig + d * (uint64_t)K)
                          : sedd_ref_minhash_shingles(x, n_sh, K, seed, sig + d * (uint64_t)K);
    if (rc) { free(x); return rc; }
  }
  free(x);
  free(qk);
  return SEDD_REF_OK;
}

/* key[d*b + j] = sum_{i<r} sig[d*K + j*r + i] * Q^i mod p */
int sedd_ref_lsh_keys(const uint32_t *sig, uint64_t n_docs, int32_t K, int32_t b, int32_t r,
                      uint64_t *keys) {
  if (K < 1 || b < 1 || r < 1 || (int64_t)b * r > K) return SEDD_REF_EINVAL;
  if (n_docs == 0) return SEDD_REF_OK;
  if (!sig || !keys) return SEDD_REF_EINVAL;
  for (uint64_t d = 0; d < n_docs; d++)
    for (int32_t j = 0; j < b; j++) {
      uint64_t key = 0, pw = 1;
      for (int32_t i = 0; i < r; i++) {
        key = addmod(key, mulmod((uint64_t)sig[d * (uint64_t)K + (uint64_t)j * r + i], pw));
        pw = mulmod(pw, Q_BAND);
      }
      keys[d * (uint64_t)b + j] = key;
    }
  return SEDD_REF_OK;
}

/* ---- clusters: connected components of "shares a band key in the same band" ---- */

typedef struct { uint64_t key; uint64_t doc; } kd_t;
static int kd_cmp(const void *pa, const void *pb) {
  const kd_t *a = (const kd_t *)pa, *b = (const kd_t *)pb;
  if (a->key != b->key) return a->key < b->key ? -1 : 1;
  if (a->doc != b->doc) return a->doc < b->doc ? -1 : 1;
  return 0;
}
static uint64_t uf_find(uint64_t *parent, uint64_t v) {
  uint64_t root = v;
  while (parent[root] != root) root = parent[root];
  while (parent[v] != root) { uint64_t nx = parent[v]; parent[v] = root; v = nx; }
  return root;
}

int sedd_ref_cluster(const uint64_t *keys, uint64_t n_docs, int32_t b, int64_t *cluster_id) {
  if (b < 1) return SEDD_REF_EINVAL;
  if (n_docs == 0) return SEDD_REF_OK;
  if (!keys || !cluster_id) return SEDD_REF_EINVAL;
  uint64_t *parent = (uint64_t *)malloc(n_docs * 8);
  kd_t *col = (kd_t *)malloc(n_docs * sizeof(kd_t));
  uint64_t *lowest = (uint64_t *)malloc(n_docs * 8);
  if (!parent || !col || !lowest) { free(parent); free(col); free(lowest); return SEDD_REF_ENOMEM; }
  for (uint64_t d = 0; d < n_docs; d++) parent[d] = d;
  for (int32_t j = 0; j < b; j++) {
    for (uint64_t d = 0; d < n_docs; d++) { col[d].key = keys[d * (uint64_t)b + j]; col[d].doc = d; }
    qsort(col, n_docs, sizeof(kd_t), kd_cmp);
    for (uint64_t i = 1; i < n_docs; i++)
      if (col[i].key == col[i - 1].key) {
        uint64_t ra = uf_find(parent, col[i - 1].doc), rb = uf_find(parent, col[i].doc);
        if (ra != rb) parent[rb] = ra;
      }
  }
  for (uint64_t d = 0; d < n_docs; d++) lowest[d] = UINT64_MAX;
  for (uint64_t d = 0; d < n_docs; d++) {
    uint64_t rt = uf_find(parent, d);
    if (d < lowest[rt]) lowest[rt] = d;
  }
  for (uint64_t d = 0; d < n_docs; d++) cluster_id[d] = (int64_t)lowest[uf_find(parent, d)];
  free(parent); free(col); free(lowest);
  return SEDD_REF_OK;
}

/*
 * Verified clusters (Section 2.3 last step; Section 3.3, the count-match matrix M_ij).
 * A bucket is the set of documents with the same key in the same band.  Inside every bucket all
 * pairs i < j are compared (the paper's exhaustive O(D^2) comparison, Section 3.1): the pair is
 * a duplicate iff the number of positions k < K with sig[i][k] == sig[j][k] is at least
 * min_match (min_match = the smallest integer >= theta * K; the caller takes that ceiling once,
 * so no floating point is involved here).  Duplicate pairs are the edges of the union graph;
 * cluster_id[d] = lowest index of d's connected component.
 */
int sedd_ref_cluster_verified(const uint64_t *keys, const uint32_t *sig, uint64_t n_docs,
                              int32_t K, int32_t b, int32_t min_match, int64_t *cluster_id) {
  if (b < 1 || K < 1 || min_match < 0) return SEDD_REF_EINVAL;
  if (n_docs == 0) return SEDD_REF_OK;
  if (!keys || !sig || !cluster_id) return SEDD_REF_EINVAL;
  uint64_t *parent = (uint64_t *)malloc(n_docs * 8);
  kd_t *col = (kd_t *)malloc(n_docs * sizeof(kd_t));
  uint64_t *lowest = (uint64_t *)malloc(n_docs * 8);
  if (!parent || !col || !lowest) { free(parent); free(col); free(lowest); return SEDD_REF_ENOMEM; }
  for (uint64_t d = 0; d < n_docs; d++) parent[d] = d;
  for (int32_t j = 0; j < b; j++) {
    for (uint64_t d = 0; d < n_docs; d++) { col[d].key = keys[d * (uint64_t)b + j]; col[d].doc = d; }
    qsort(col, n_docs, sizeof(kd_t), kd_cmp);
    uint64_t s = 0;
    while (s < n_docs) {                               /* bucket = run [s, e) of one key */
      uint64_t e = s + 1;
      while (e < n_docs && col[e].key == col[s].key) e++;
      for (uint64_t x = s; x < e; x++)
        for (uint64_t y = x + 1; y < e; y++) {         /* upper triangle of M */
          const uint32_t *sx = sig + col[x].doc * (uint64_t)K, *sy = sig + col[y].doc * (uint64_t)K;
          int32_t same = 0;
          for (int32_t k = 0; k < K; k++) same += sx[k] == sy[k];
          if (same >= min_match) {
            uint64_t ra = uf_find(parent, col[x].doc), rb = uf_find(parent, col[y].doc);
            if (ra != rb) parent[rb] = ra;
          }
        }
      s = e;
    }
  }
  for (uint64_t d = 0; d < n_docs; d++) lowest[d] = UINT64_MAX;
  for (uint64_t d = 0; d < n_docs; d++) {
    uint64_t rt = uf_find(parent, d);
    if (d < lowest[rt]) lowest[rt] = d;
  }
  for (uint64_t d = 0; d < n_docs; d++) cluster_id[d] = (int64_t)lowest[uf_find(parent, d)];
  free(parent); free(col); free(lowest);
  return SEDD_REF_OK;
}

/*
 * Dense bucket ids (Section 3.2, last paragraph): the r values of a band are summed and the
 * bucket is the remainder of the sum modulo the number of buckets,
 *   key[d*b + j] = (sum_{i<r} sig[d*K + j*r + i]) mod n_buckets.
 * The sum is the exact integer (it stays below r * 2^32).  The paper sets the number of buckets
 * to 4 sqrt(N); the caller passes it.  Buckets are deliberately coarse: they only propose
 * candidate pairs, which sedd_ref_cluster_verified then tests on the full signatures.
 */
int sedd_ref_lsh_dense_keys(const uint32_t *sig, uint64_t n_docs, int32_t K, int32_t b, int32_t r,
                            uint64_t n_buckets, uint64_t *keys) {
  if (K < 1 || b < 1 || r < 1 || (int64_t)b * r > K || n_buckets < 1) return SEDD_REF_EINVAL;
  if (n_docs == 0) return SEDD_REF_OK;
  if (!sig || !keys) return SEDD_REF_EINVAL;
  for (uint64_t d = 0; d < n_docs; d++)
    for (int32_t j = 0; j < b; j++) {
      u128 sum = 0;
      for (int32_t i = 0; i < r; i++) sum += sig[d * (uint64_t)K + (uint64_t)j * r + i];
      keys[d * (uint64_t)b + j] = (uint64_t)(sum % n_buckets);
    }
  return SEDD_REF_OK;
}
