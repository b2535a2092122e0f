/*
 * Seeded synthetic web-text corpus generator (host only, plain C + OpenMP).
 *
 * This file produces INPUTS: concatenated document bytes plus document
 * offsets.  It contains none of the deduplication method's arithmetic (no
 * shingling, no hashing of shingles, no signatures).  Both the CPU oracle's
 * tests and the GPU path's tests feed on what it writes.
 *
 * Every document is a pure function of (seed, doc id): all random numbers
 * come from a counter-based generator keyed by (seed, doc, stream), so any
 * document range can be produced independently, by any number of threads,
 * with identical bytes.
 *
 * Shape of the text (stands in for the web-text corpora the paper measures
 * on, Section 4.1):
 *   - vocabulary of `vocab` distinct lowercase words, 2..8 letters each,
 *     optionally a percentage of them spelled with 2-byte UTF-8 letters;
 *   - word rank drawn Zipf(s): P(rank i) ~ i^-s;
 *   - words per fresh document: lognormal(median, sigma) clipped to
 *     [len_lo, len_hi]; a fraction `long_frac` of documents instead draws a
 *     log-uniform length in [long_lo, long_hi];
 *   - a fraction `near_frac` of documents are near-duplicates of a uniformly
 *     chosen earlier document: each source word is, with probability = the
 *     document's edit rate (uniform in [edit_lo, edit_hi]), replaced,
 *     preceded by an inserted word, or deleted (one third each); the source
 *     may itself be a duplicate (chains), up to `max_chain` links;
 *   - a fraction `exact_frac` are byte-identical copies of an earlier one;
 *   - words are joined by a single 0x20 unless `ws_variety` is set, in which
 *     case separators vary (runs of spaces, tabs, newlines) and documents
 *     may start or end with whitespace.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  uint64_t seed;
  uint64_t n_docs;
  uint32_t vocab;       /* number of distinct words */
  uint32_t utf8_pct;    /* percent of vocabulary words using 2-byte letters */
  double zipf_s;
  double len_median, len_sigma;
  uint32_t len_lo, len_hi;
  double long_frac;
  uint32_t long_lo, long_hi;
  double near_frac, exact_frac;
  double edit_lo, edit_hi;
  uint32_t max_chain;
  uint32_t ws_variety;  /* 0: single spaces; 1: mixed whitespace */
} corpus_params;

typedef struct {
  corpus_params p;
  uint8_t *word_bytes;   /* concatenated vocabulary spellings */
  uint32_t *word_off;    /* vocab+1 offsets into word_bytes */
  double *cdf;           /* vocab cumulative probabilities */
  uint32_t *guide;       /* guide table for inverse-CDF lookup */
  uint32_t n_guide;
} corpus_t;

enum { STREAM_KIND = 1, STREAM_LEN = 2, STREAM_WORDS = 3, STREAM_EDIT = 4,
       STREAM_NEW = 5, STREAM_WS = 6, STREAM_VOCAB = 7 };

static inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30; z *= 0xbf58476d1ce4e5b9ULL;
  z ^= z >> 27; z *= 0x94d049bb133111ebULL;
  z ^= z >> 31; return z;
}
static inline uint64_t make_key(uint64_t seed, uint64_t doc, uint64_t stream) {
  return mix64(mix64(seed * 0x9e3779b97f4a7c15ULL + stream) ^
               (doc * 0xd1342543de82ef95ULL + 0x2545f4914f6cdd1dULL));
}
static inline uint64_t rnd(uint64_t key, uint64_t ctr) {
  return mix64(key + 0x9e3779b97f4a7c15ULL * (ctr + 1));
}
static inline double u01(uint64_t r) { return (double)(r >> 11) * (1.0 / 9007199254740992.0); }

/* ---- vocabulary ------------------------------------------------------- */

static int spell(const corpus_params *p, uint32_t w, uint32_t attempt, uint8_t *out) {
  uint64_t key = make_key(p->seed, w, STREAM_VOCAB);
  uint64_t r0 = rnd(key, 64ULL * attempt);
  int letters = 2 + (int)(r0 % 7);
  int wide = ((r0 >> 8) % 100) < p->utf8_pct;
  int n = 0;
  for (int i = 0; i < letters; i++) {
    uint32_t c = (uint32_t)(rnd(key, 64ULL * attempt + 1 + i) % 26);
    if (wide) { out[n++] = 0xC3; out[n++] = (uint8_t)(0xA0 + c); }
    else out[n++] = (uint8_t)('a' + c);
  }
  return n;
}

static uint64_t bytes_hash(const uint8_t *s, int n) {
  uint64_t h = 1469598103934665603ULL;
  for (int i = 0; i < n; i++) { h ^= s[i]; h *= 1099511628211ULL; }
  return mix64(h);
}

corpus_t *corpus_create(const corpus_params *p) {
  if (!p || p->vocab == 0) return NULL;
  corpus_t *c = (corpus_t *)calloc(1, sizeof(*c));
  c->p = *p;
  uint32_t V = p->vocab;
  c->word_bytes = (uint8_t *)malloc((size_t)V * 16);
  c->word_off = (uint32_t *)malloc(((size_t)V + 1) * 4);
  /* distinct spellings: open-addressing set over spellings already taken */
  uint32_t cap = 1; while (cap < 4 * V) cap <<= 1;
  int32_t *slot = (int32_t *)malloc((size_t)cap * 4);
  for (uint32_t i = 0; i < cap; i++) slot[i] = -1;
  uint32_t off = 0;
  for (uint32_t w = 0; w < V; w++) {
    uint8_t buf[16]; int n = 0;
    for (uint32_t attempt = 0;; attempt++) {
      n = spell(p, w, attempt, buf);
      uint32_t h = (uint32_t)bytes_hash(buf, n) & (cap - 1);
      int dup = 0;
      while (slot[h] >= 0) {
        uint32_t o = c->word_off[slot[h]], l = c->word_off[slot[h] + 1] - o;
        if ((int)l == n && memcmp(c->word_bytes + o, buf, n) == 0) { dup = 1; break; }
        h = (h + 1) & (cap - 1);
      }
      if (!dup) { slot[h] = (int32_t)w; break; }
    }
    c->word_off[w] = off;
    memcpy(c->word_bytes + off, buf, n);
    off += n;
    c->word_off[w + 1] = off;
  }
  free(slot);
  /* Zipf CDF + guide table */
  c->cdf = (double *)malloc((size_t)V * 8);
  double tot = 0;
  for (uint32_t i = 0; i < V; i++) { tot += pow((double)(i + 1), -p->zipf_s); c->cdf[i] = tot; }
  for (uint32_t i = 0; i < V; i++) c->cdf[i] /= tot;
  c->cdf[V - 1] = 1.0;
  c->n_guide = 1u << 16;
  c->guide = (uint32_t *)malloc((size_t)c->n_guide * 4);
  uint32_t r = 0;
  for (uint32_t g = 0; g < c->n_guide; g++) {
    double u = (double)g / c->n_guide;
    while (r < V - 1 && c->cdf[r] <= u) r++;
    c->guide[g] = r;
  }
  return c;
}

void corpus_destroy(corpus_t *c) {
  if (!c) return;
  free(c->word_bytes); free(c->word_off); free(c->cdf); free(c->guide); free(c);
}

static inline uint32_t zipf_draw(const corpus_t *c, uint64_t r) {
  double u = u01(r);
  uint32_t i = c->guide[(uint32_t)(u * c->n_guide)];
  while (c->cdf[i] <= u && i < c->p.vocab - 1) i++;
  return i;
}

/* ---- per-document plan -------------------------------------------------- */

/* raw (chain-unaware) kind: 0 fresh, 1 near-duplicate, 2 exact copy */
static int raw_kind(const corpus_t *c, uint64_t doc, uint64_t *src, double *rate) {
  if (doc == 0) return 0;
  uint64_t key = make_key(c->p.seed, doc, STREAM_KIND);
  double u = u01(rnd(key, 0));
  int kind = u < c->p.exact_frac ? 2 : (u < c->p.exact_frac + c->p.near_frac ? 1 : 0);
  if (kind) {
    *src = rnd(key, 1) % doc;
    *rate = c->p.edit_lo + (c->p.edit_hi - c->p.edit_lo) * u01(rnd(key, 2));
  }
  return kind;
}

typedef struct { uint64_t doc; int kind; double rate; } link_t;

/*
 * Resolve doc's ancestry: chain[0] is the document that is generated fresh,
 * chain[n-1] is `doc`.  A document whose chain would have more than
 * max_chain links is generated fresh instead (so is every use of it as a
 * source), which keeps "content is a pure function of the id" true.
 */
static int resolve_chain(const corpus_t *c, uint64_t doc, link_t **out) {
  int cap = 16, n = 0;
  link_t *up = (link_t *)malloc(sizeof(link_t) * cap);
  uint64_t d = doc;
  for (;;) {
    uint64_t src = 0; double rate = 0;
    int k = raw_kind(c, d, &src, &rate);
    if (n == cap) { cap *= 2; up = (link_t *)realloc(up, sizeof(link_t) * cap); }
    up[n].doc = d; up[n].kind = k; up[n].rate = rate; n++;
    if (!k) break;
    d = src;
  }
  /* up[n-1] is the raw-fresh root; walk down assigning depths */
  int start = n - 1; int depth = 0;
  for (int i = n - 2; i >= 0; i--) {
    depth++;
    if ((uint32_t)depth > c->p.max_chain) { up[i].kind = 0; depth = 0; start = i; }
  }
  int m = start + 1;
  link_t *ch = (link_t *)malloc(sizeof(link_t) * m);
  for (int i = 0; i < m; i++) ch[i] = up[start - i];
  free(up);
  *out = ch;
  return m;
}

typedef struct { uint32_t *v; size_t n, cap; } idvec;
static inline void idv_push(idvec *a, uint32_t x) {
  if (a->n == a->cap) { a->cap = a->cap ? a->cap * 2 : 1024; a->v = (uint32_t *)realloc(a->v, a->cap * 4); }
  a->v[a->n++] = x;
}

static uint64_t fresh_len(const corpus_t *c, uint64_t doc) {
  const corpus_params *p = &c->p;
  uint64_t key = make_key(p->seed, doc, STREAM_LEN);
  if (p->long_frac > 0 && u01(rnd(key, 0)) < p->long_frac) {
    double lo = log((double)p->long_lo), hi = log((double)p->long_hi);
    return (uint64_t)llround(exp(lo + (hi - lo) * u01(rnd(key, 1))));
  }
  double u1 = u01(rnd(key, 2)), u2 = u01(rnd(key, 3));
  if (u1 < 1e-300) u1 = 1e-300;
  double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2);
  double w = exp(log(p->len_median) + p->len_sigma * z);
  double r = floor(w + 0.5);
  if (r < p->len_lo) r = p->len_lo;
  if (r > p->len_hi) r = p->len_hi;
  return (uint64_t)r;
}

/* word ids of `doc` into out (out->n reset) ; tmp is scratch */
static void doc_word_ids(const corpus_t *c, uint64_t doc, idvec *out, idvec *tmp) {
  link_t *ch; int m = resolve_chain(c, doc, &ch);
  out->n = 0;
  uint64_t root = ch[0].doc;
  uint64_t L = fresh_len(c, root);
  uint64_t wkey = make_key(c->p.seed, root, STREAM_WORDS);
  for (uint64_t t = 0; t < L; t++) idv_push(out, zipf_draw(c, rnd(wkey, t)));
  for (int i = 1; i < m; i++) {
    if (ch[i].kind == 2) continue;               /* exact copy: same words */
    uint64_t ekey = make_key(c->p.seed, ch[i].doc, STREAM_EDIT);
    uint64_t nkey = make_key(c->p.seed, ch[i].doc, STREAM_NEW);
    tmp->n = 0;
    uint64_t fresh = 0;
    for (size_t t = 0; t < out->n; t++) {
      uint64_t r = rnd(ekey, t);
      if (u01(r) < ch[i].rate) {
        uint32_t op = (uint32_t)((r & 0x7ff) % 3);
        if (op == 0) idv_push(tmp, zipf_draw(c, rnd(nkey, fresh++)));
        else if (op == 1) { idv_push(tmp, zipf_draw(c, rnd(nkey, fresh++))); idv_push(tmp, out->v[t]); }
        /* op == 2: delete */
      } else idv_push(tmp, out->v[t]);
    }
    idvec sw = *out; *out = *tmp; *tmp = sw;
  }
  free(ch);
}

/* whitespace separator before word t (t==0: leading) and trailing */
static inline int sep_bytes(const corpus_t *c, uint64_t wskey, uint64_t t, int first, uint8_t *buf) {
  if (!c->p.ws_variety) { if (first) return 0; buf[0] = 0x20; return 1; }
  uint64_t r = rnd(wskey, t);
  uint32_t sel = (uint32_t)(r % 16);
  static const uint8_t ws[6] = {0x20, 0x09, 0x0A, 0x0D, 0x0B, 0x0C};
  if (first) { if (sel != 0) return 0; buf[0] = ws[(r >> 8) % 6]; return 1; }
  if (sel < 12) { buf[0] = 0x20; return 1; }
  int n = 1 + (int)((r >> 16) % 3);
  for (int i = 0; i < n; i++) buf[i] = ws[(r >> (24 + 8 * i)) % 6];
  return n;
}

typedef struct { uint8_t *v; size_t n, cap; } bytevec;
static inline void bv_reserve(bytevec *a, size_t extra) {
  if (a->n + extra > a->cap) {
    size_t nc = a->cap ? a->cap * 2 : (1u << 20);
    while (nc < a->n + extra) nc *= 2;
    a->v = (uint8_t *)realloc(a->v, nc); a->cap = nc;
  }
}

static void render_doc(const corpus_t *c, uint64_t doc, idvec *ids, idvec *tmp, bytevec *out) {
  /* exact copies must be byte-identical: render as the nearest non-copy ancestor */
  uint64_t render_as = doc;
  for (;;) {
    link_t *ch; int m = resolve_chain(c, render_as, &ch);
    int k = ch[m - 1].kind; uint64_t parent = m >= 2 ? ch[m - 2].doc : 0;
    free(ch);
    if (k == 2) render_as = parent; else break;
  }
  doc_word_ids(c, render_as, ids, tmp);
  uint64_t wskey = make_key(c->p.seed, render_as, STREAM_WS);
  uint8_t sb[4];
  for (size_t t = 0; t < ids->n; t++) {
    int ns = sep_bytes(c, wskey, t, t == 0, sb);
    uint32_t o = c->word_off[ids->v[t]], l = c->word_off[ids->v[t] + 1] - o;
    bv_reserve(out, ns + l + 4);
    memcpy(out->v + out->n, sb, ns); out->n += ns;
    memcpy(out->v + out->n, c->word_bytes + o, l); out->n += l;
  }
  if (c->p.ws_variety && ids->n && (rnd(wskey, ~0ULL) % 16) == 0) { bv_reserve(out, 1); out->v[out->n++] = 0x0A; }
}

/* ---- public entry points ------------------------------------------------ */

typedef struct { bytevec bytes; uint64_t d0, d1; } shard_t;

/*
 * Generate documents [d0, d1).  offsets must hold d1-d0+1 entries and
 * receives offsets relative to the first generated byte.  Returns a malloc'd
 * buffer with the concatenated bytes (release with corpus_free_bytes), and
 * its size in *total.
 */
uint8_t *corpus_generate(const corpus_t *c, uint64_t d0, uint64_t d1, uint64_t *offsets,
                         uint64_t *total, int threads) {
  uint64_t n = d1 > d0 ? d1 - d0 : 0;
  if (threads < 1) threads = 1;
  uint64_t n_sh = (uint64_t)threads * 16;
  if (n_sh > n) n_sh = n ? n : 1;
  shard_t *sh = (shard_t *)calloc(n_sh, sizeof(shard_t));
  uint64_t *sizes = (uint64_t *)malloc((n + 1) * 8);
  for (uint64_t s = 0; s < n_sh; s++) { sh[s].d0 = d0 + n * s / n_sh; sh[s].d1 = d0 + n * (s + 1) / n_sh; }
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
  for (int64_t s = 0; s < (int64_t)n_sh; s++) {
    idvec ids = {0, 0, 0}, tmp = {0, 0, 0};
    for (uint64_t d = sh[s].d0; d < sh[s].d1; d++) {
      size_t before = sh[s].bytes.n;
      render_doc(c, d, &ids, &tmp, &sh[s].bytes);
      sizes[d - d0] = sh[s].bytes.n - before;
    }
    free(ids.v); free(tmp.v);
  }
  uint64_t acc = 0;
  for (uint64_t i = 0; i < n; i++) { offsets[i] = acc; acc += sizes[i]; }
  offsets[n] = acc;
  *total = acc;
  uint8_t *out = (uint8_t *)malloc(acc ? acc : 1);
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
  for (int64_t s = 0; s < (int64_t)n_sh; s++) {
    if (sh[s].d1 > sh[s].d0) memcpy(out + offsets[sh[s].d0 - d0], sh[s].bytes.v, sh[s].bytes.n);
    free(sh[s].bytes.v);
  }
  free(sh); free(sizes);
  return out;
}

void corpus_free_bytes(uint8_t *p) { free(p); }

/* kind (after chain capping), source document and edit rate of `doc` */
int corpus_doc_meta(const corpus_t *c, uint64_t doc, uint64_t *src, double *rate) {
  link_t *ch; int m = resolve_chain(c, doc, &ch);
  int k = ch[m - 1].kind;
  *src = m >= 2 ? ch[m - 2].doc : doc;
  *rate = ch[m - 1].rate;
  free(ch);
  return k;
}

/* word ids of one document; returns the count, writes at most cap ids */
uint64_t corpus_doc_words(const corpus_t *c, uint64_t doc, uint32_t *out, uint64_t cap) {
  idvec ids = {0, 0, 0}, tmp = {0, 0, 0};
  doc_word_ids(c, doc, &ids, &tmp);
  uint64_t n = ids.n;
  for (uint64_t i = 0; i < n && i < cap; i++) out[i] = ids.v[i];
  free(ids.v); free(tmp.v);
  return n;
}

/* spelling of vocabulary word w; returns its length in bytes (<= 16) */
int corpus_word(const corpus_t *c, uint32_t w, uint8_t *out) {
  if (w >= c->p.vocab) return -1;
  uint32_t o = c->word_off[w], l = c->word_off[w + 1] - o;
  memcpy(out, c->word_bytes + o, l);
  return (int)l;
}
