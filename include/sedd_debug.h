/*
 * Stage-level entry points of libsedd, for parity tests of the intermediate results.
 * Same conventions as sedd.h: device pointers owned by the caller, a hipStream_t as void*,
 * SEDD_OK or a negative code.  They run the same kernels the three public calls run.
 */
#ifndef SEDD_DEBUG_H
#define SEDD_DEBUG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Base hashes x(s) of every shingle (Section 3.2, Eq. 1), in document order (modulo 2^61-1, or
 * modulo 4,294,967 with SEDD_FLAG_PAPER_PRIME; SEDD_FLAG_ROLLING_FAMILY has no function-independent
 * shingle hash and is rejected).
 *   shingle_offsets  device, uint64[n_docs+1]: document d owns x[shingle_offsets[d] ..
 *                    shingle_offsets[d+1]).
 *   x                device, uint64[x_cap]; entries beyond x_cap are not written (the
 *                    offsets are still complete, so a first call may size the second).
 */
int sedd_debug_shingle_hashes(const uint8_t *bytes, const uint64_t *doc_offsets,
                              uint64_t n_docs, int32_t shingle_n, uint32_t flags, uint64_t *x,
                              uint64_t x_cap, uint64_t *shingle_offsets, void *stream);

/* Coefficients a_k, b_k of the K hash functions: device uint64[K] each. */
int sedd_debug_coeffs(uint64_t seed, int32_t K, uint64_t *a, uint64_t *b, void *stream);

/* The same for SEDD_FLAG_PAPER_PRIME: a'_k and b'_k (both below 4,294,967) as uint64. */
int sedd_debug_coeffs_pp(uint64_t seed, int32_t K, uint64_t *a, uint64_t *b, void *stream);

/* Bases q_k of SEDD_FLAG_ROLLING_FAMILY: device uint64[K]. */
int sedd_debug_bases(uint64_t seed, int32_t K, uint64_t *q, void *stream);

/* Exclusive prefix sum of n uint32 values (device), out may alias in. */
int sedd_debug_scan_u32(const uint32_t *in, uint32_t *out, uint64_t n, void *stream);

/*
 * The sort inside sedd_cluster: for every band j the (key, doc) records sorted by key,
 * stable in doc.  keys_sorted uint64[b*n_docs] and docs_sorted uint32[b*n_docs] are
 * band-major (band j occupies [j*n_docs, (j+1)*n_docs)).
 */
int sedd_debug_sort_bands(const uint64_t *keys, uint64_t n_docs, int32_t b,
                          uint64_t *keys_sorted, uint32_t *docs_sorted, void *stream);

/*
 * The K-hash / minimum kernel alone, on caller-supplied shingle hashes: document d owns
 * x[shingle_offsets[d] .. shingle_offsets[d+1]) (values < 2^61-1, any order, repeats allowed).
 * n_shingles = the length of x; shingle_offsets[n_docs] <= n_shingles < 2^32.  sig as in
 * sedd_minhash.
 */
int sedd_debug_minhash_from_x(const uint64_t *x, const uint64_t *shingle_offsets, uint64_t n_docs,
                              uint64_t n_shingles, int32_t K, uint64_t seed, uint32_t *sig,
                              void *stream);

/* The same with the functions of SEDD_FLAG_PAPER_PRIME; x is taken modulo 4,294,967. */
int sedd_debug_minhash_from_x_pp(const uint64_t *x, const uint64_t *shingle_offsets,
                                 uint64_t n_docs, uint64_t n_shingles, int32_t K, uint64_t seed,
                                 uint32_t *sig, void *stream);

/*
 * Device-side counters since the library was loaded, copied to the HOST array out[SEDD_STAT_N]
 * (waits for the device to go idle first).
 */
#define SEDD_STAT_SLOW_TILES 0 /* shingle tiles the min-hash kernel recomputed on its exact path */
#define SEDD_STAT_N 16
int sedd_debug_stats(uint64_t *out);

/*
 * Per-stage timing with HIP events on the stream the kernels are launched on.  While enabled,
 * every call records an event pair around each stage; sedd_profile_read waits for them, adds
 * the elapsed milliseconds and the number of timed spans per stage into the HOST arrays
 * ms[SEDD_PROF_N], spans[SEDD_PROF_N], and forgets them.
 */
#define SEDD_PROF_MINHASH 0  /* Eq. 1 per shingle + K hash functions + minimum (the dominant kernel) */
#define SEDD_PROF_TOKENIZE 1 /* token marking, counting and token records */
#define SEDD_PROF_WORKLIST 2 /* tile lists and scans */
#define SEDD_PROF_LSH_KEYS 3
#define SEDD_PROF_SORT 4
#define SEDD_PROF_UNION 5
#define SEDD_PROF_VERIFY 6   /* pairwise signature comparison inside buckets + union-find */
#define SEDD_PROF_N 8
int sedd_profile_enable(int on);
int sedd_profile_read(double *ms, uint64_t *spans);
const char *sedd_profile_label(int label);

/*
 * Whether the most recent sedd_cluster / sedd_cluster_verified call had to sort its records by
 * the whole key (1) or grouped them by the low key bits alone (0), copied to the HOST word *out
 * (waits for the device to go idle first).  Band keys from sedd_lsh_keys never need the whole key.
 */
int sedd_debug_last_regroup(uint32_t *out);

/*
 * Upper bound on the text bytes processed per internal chunk of sedd_minhash (0 restores
 * the default).  Results never depend on it; tests use small values to cross chunk edges.
 */
int sedd_debug_set_chunk_bytes(uint64_t bytes);

/*
 * Makes every request for more than `bytes` of library-owned scratch fail with SEDD_ENOMEM, as a
 * full device would (0 lifts the cap).  For tests of that return path: the failing call writes
 * nothing and enqueues nothing, and the next call after the cap is lifted succeeds.
 */
int sedd_debug_set_scratch_cap(uint64_t bytes);

/*
 * Bytes of text per wavefront of the streaming min-hash kernel (word shingles, 61-bit modulus):
 * a multiple of 1024, at most 2^24; 0 restores the default.  Results never depend on it; tests
 * use it to move the places where documents are split between wavefronts.
 */
int sedd_debug_set_piece_bytes(uint32_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* SEDD_DEBUG_H */
