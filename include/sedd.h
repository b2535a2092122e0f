/*
 * libsedd: MinHash-LSH near-duplicate detection on one MI355X (gfx950).
 *
 * The three calls follow the pipeline of the SEDD paper (Sections 2.2, 2.3):
 *   documents -> signature matrix -> per-band bucket keys -> union graph ->
 *   lowest-index representative of each connected component.
 *
 * Conventions shared by every call
 *   - Every pointer is a DEVICE pointer to memory the caller owns.  The
 *     library never frees or keeps a caller pointer.  Outputs are written only
 *     by the work the call enqueues.  Arrays must be aligned to their element
 *     size (uint32: 4, uint64 / int64: 8; `bytes` may start anywhere); a
 *     misaligned pointer is SEDD_EINVAL.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue their kernels on it and return; results are ready when the
 *     stream has drained.  sedd_minhash first validates `doc_offsets` with two
 *     small kernels and waits once for the first and last offset and the verdict
 *     (twice with byte shingles or the rolling-family mode, which also plan
 *     bounded-size chunks); everything after that is enqueued without host waits.
 *   - Return value: SEDD_OK (0) or a negative error code.  On an error no output
 *     is written.  Bad scalars, null or misaligned pointers are found before any
 *     device work; offsets that decrease, exceed a document's size limit or (in
 *     sedd_minhash_bounded) point past the text are found by two small validation
 *     kernels, which read doc_offsets only, before anything reads the text.
 *     `n_docs == 0` is a successful no-op that touches nothing.
 *   - Device scratch (chunk work lists, sort buffers, the union-find forest)
 *     lives in a grow-only allocation owned by the library, shared by the
 *     calls that use it: those must not overlap in time, neither on different
 *     streams nor from different threads.  sedd_release_scratch() frees it.
 *     Calls that do NOT use it may run concurrently from several threads on
 *     several streams: sedd_minhash / sedd_minhash_bounded on word shingles
 *     without SEDD_FLAG_ROLLING_FAMILY (the default mode and the paper-prime
 *     mode; their coefficient tables are cached per (K, seed, modulus) and
 *     read-only), sedd_lsh_keys, sedd_lsh_dense_keys, and sedd_cluster_ws /
 *     sedd_cluster_verified_ws with a workspace per call.
 *   - All arithmetic is exact unsigned integer arithmetic; results do not
 *     depend on launch shape, chunking or timing.
 */
#ifndef SEDD_H
#define SEDD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SEDD_OK 0
#define SEDD_EINVAL (-1)  /* bad argument (null pointer, K<1, b*r>K, offsets decreasing, ...) */
#define SEDD_ENOMEM (-2)  /* device or pinned-host allocation failed; sedd_last_device_error() names it */
#define SEDD_EDEVICE (-3) /* a HIP call failed; sedd_last_device_error() names it */
#define SEDD_ELIMIT (-4)  /* the input exceeds a fixed limit of the entry point (sedd_cluster_static) */

/* flags of sedd_minhash */
#define SEDD_FLAG_BYTE_SHINGLES 1u /* shingles are byte n-grams instead of word n-grams */
#define SEDD_FLAG_PAPER_PRIME 2u   /* Eq. 1 and the K functions modulo 4,294,967 (see below) */
#define SEDD_FLAG_ROLLING_FAMILY 4u /* function k is Eq. 1 itself to a base q_k (see below) */

/* largest K / shingle_n / b the kernels accept */
#define SEDD_MAX_K 4096
#define SEDD_MAX_SHINGLE_N 64
#define SEDD_MAX_BANDS 4096

/*
 * MinHash signature generation (Section 2.2 "MinHash generation"; shingle hash of
 * Section 3.2, Eq. 1).
 *
 * For every document d = bytes[doc_offsets[d] .. doc_offsets[d+1]):
 *   1. shingles.  Word mode (default): tokens are the maximal runs of bytes outside
 *      {0x09,0x0A,0x0B,0x0C,0x0D,0x20}; shingle i is tokens i..i+shingle_n-1 joined by a
 *      single 0x20.  A document with 1..shingle_n-1 tokens has one shingle (all its
 *      tokens); with none it has no shingle.  Byte mode (SEDD_FLAG_BYTE_SHINGLES): every
 *      window of shingle_n bytes; a document of 1..shingle_n-1 bytes has one shingle.
 *   2. x(s) = (sum_i s_i * 257^(i-1)) mod (2^61-1) over the bytes s_i of the shingle
 *      (Eq. 1 with q = 257, p = 2^61-1).
 *   3. h_k(s) = ((a_k * x(s) + b_k) mod p) mod 2^32 for k = 0..K-1, with
 *      a_k = s0 * Ga^(k+1) mod p, b_k = s0 * Gb^(k+1) mod p, s0 = (seed mod (p-1)) + 1,
 *      Ga = 1425089352415399810, Gb = 955111447119501601.
 *   4. sig[d*K + k] = min over the document's shingles of h_k(s); 0xFFFFFFFF if none.
 *
 * SEDD_FLAG_PAPER_PRIME: Section 3.2 quotes p' = 4,294,967 as the modulus of the paper's
 * experiments (small enough that h * q stays a 32-bit integer).  With this flag steps 2 and 3
 * use it: x'(s) = (sum_i s_i * 257^(i-1)) mod p' and h'_k(s) = (a'_k * x'(s) + b'_k) mod p' with
 * a'_k = (a_k mod (p'-1)) + 1, b'_k = b_k mod p'; the values are below 2^23 and are stored as
 * they are.  A 22-bit range is exhausted by documents with millions of shingles (every
 * minimum tends to 0): the mode is meant for comparison with the paper's setting.
 *
 * SEDD_FLAG_ROLLING_FAMILY: the other way to obtain K functions from Section 3.2: function k is
 * Eq. 1 with a base of its own, h_k(s) = ((sum_i s_i * q_k^(i-1)) mod p) mod 2^32 with
 * q_k = 257 + (a_k mod (p - 257)) and p = 2^61-1; b_k is not used.  Every function then has to
 * hash every shingle from its characters (about 10 times the work of step 3 on 5-word
 * shingles), and shingles that differ only in their first character keep their order under
 * every function.  Provided for comparison; not combinable with SEDD_FLAG_PAPER_PRIME.
 *
 * bytes        device, uint8; read in [doc_offsets[0], doc_offsets[n_docs]).
 * doc_offsets  device, uint64[n_docs+1], non-decreasing byte offsets into `bytes`.
 * shingle_n    1..SEDD_MAX_SHINGLE_N.   K  1..SEDD_MAX_K.
 * sig          device, uint32[n_docs*K], document-major; fully overwritten.
 * A single document must be smaller than 2^32 - 2^30 - 2^16 bytes; n_docs < 2^31.
 */
int sedd_minhash(const uint8_t *bytes, const uint64_t *doc_offsets, uint64_t n_docs,
                 int32_t shingle_n, int32_t K, uint64_t seed, uint32_t flags, uint32_t *sig,
                 void *stream);

/*
 * sedd_minhash with the size of the text stated: the same call, but doc_offsets[n_docs] > n_bytes
 * (offsets that point past the caller's buffer) is SEDD_EINVAL, found before any kernel reads
 * the text.  Bindings that know the buffer's size should call this one.
 */
int sedd_minhash_bounded(const uint8_t *bytes, uint64_t n_bytes, const uint64_t *doc_offsets,
                         uint64_t n_docs, int32_t shingle_n, int32_t K, uint64_t seed,
                         uint32_t flags, uint32_t *sig, void *stream);

/*
 * sedd_minhash for text that lives in HOST memory (Section 3.4: the paper hides the transfer of
 * the text behind the hashing with double buffering).  host_bytes and host_doc_offsets are HOST
 * pointers; sig is a DEVICE pointer as everywhere else.  The documents are cut into chunks of
 * whole documents of at most chunk_bytes of text (0: 2 GiB; a longer document is a chunk of its
 * own; at most 2^22 documents per chunk).  Chunk i+1 is uploaded on a stream of the library's own
 * into one of two device staging buffers while chunk i is hashed on `stream`; the signatures are
 * those of one sedd_minhash call on the whole text.
 * Host memory should be pinned (hipHostMalloc): uploads from pageable memory are correct but do
 * not overlap.  The offsets are validated on the host, so word shingles of the default and the
 * paper-prime mode enqueue everything without waiting on the device; the call returns when the last upload has left the
 * host buffers (they may then be changed or freed) and `sig` is complete when `stream` drains.
 * The staging buffers (2 x the largest chunk) are kept for later calls; sedd_release_scratch
 * frees them.  Like the scratch arena they are shared: calls must not overlap in time.
 */
int sedd_minhash_host_chunked(const uint8_t *host_bytes, const uint64_t *host_doc_offsets,
                              uint64_t n_docs, int32_t shingle_n, int32_t K, uint64_t seed,
                              uint32_t flags, uint64_t chunk_bytes, uint32_t *sig, void *stream);

/*
 * LSH band keys (Section 2.3: the signature is cut into b bands of r rows and each band
 * is hashed to a bucket).  key[d*b + j] = (sum_{i<r} sig[d*K + j*r + i] * Q^i) mod p with
 * Q = 1687994237021934823: Eq. 1's polynomial over the band's values.  Equal bands give
 * equal keys; unequal bands collide with probability about 2^-61.  Requires b*r <= K; the
 * first b*r columns of sig are used.
 *
 * sig   device, uint32[n_docs*K].   keys  device, uint64[n_docs*b], document-major.
 */
int sedd_lsh_keys(const uint32_t *sig, uint64_t n_docs, int32_t K, int32_t b, int32_t r,
                  uint64_t *keys, void *stream);

/*
 * Dense bucket ids (Section 3.2, last paragraph: the r values of a band are summed and the
 * remainder modulo the number of buckets is the bucket).  key[d*b + j] =
 * (sum_{i<r} sig[d*K + j*r + i]) mod n_buckets, the sum being the exact integer.  The paper sets
 * n_buckets = 4 sqrt(n_docs).  These buckets are coarse on purpose: they only propose candidate
 * pairs and are meant to be followed by sedd_cluster_verified, not by sedd_cluster.
 *
 * sig, keys as in sedd_lsh_keys; 1 <= n_buckets < 2^61.
 */
int sedd_lsh_dense_keys(const uint32_t *sig, uint64_t n_docs, int32_t K, int32_t b, int32_t r,
                        uint64_t n_buckets, uint64_t *keys, void *stream);

/*
 * Bucket grouping into duplicate clusters (Section 2.2 "Constructing a union graph" and
 * "Generating the final list of duplicates"; Appendix A.2: per-band graphs are merged).
 * Documents u, v are linked when keys[u*b + j] == keys[v*b + j] for some band j (same j on
 * both sides).  cluster_id[d] = the smallest document index in d's connected component.
 *
 * keys        device, uint64[n_docs*b], document-major, values < 2^61.
 * cluster_id  device, int64[n_docs].       n_docs < 2^31, n_docs*b < 2^32.
 * Cost: the (key, document) records of every band are radix-sorted by the low 16..32 key bits
 * (2^bits >= n_docs: 2 to 4 passes over 12 bytes per record), then every record looks back
 * over at most 64 records of its band for its key.  That suffices whenever those bits spread
 * the keys (band keys of sedd_lsh_keys do).  If some record does not find its key or the end of
 * its group within 64 records, the remaining passes up to bit 61 run as well (8 in all) and every
 * record is linked to its predecessor in the full order.  Either way the work is linear in
 * n_docs*b, nothing waits on the host, and the result is the same.
 */
int sedd_cluster(const uint64_t *keys, uint64_t n_docs, int32_t b, int64_t *cluster_id,
                 void *stream);

/*
 * sedd_cluster for callers that cannot allocate device memory while they call: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * result, same kernels as sedd_cluster; the sort buffers, the digit histograms and the
 * union-find forest live in a fixed array of SEDD_STATIC_SCRATCH_MIB MiB that is part of the
 * library's code object (each GPU the library runs on holds its copy until the process ends).
 * The call makes no hipMalloc / hipFree, creates no event, and never touches the grow-only
 * arena of the other calls.  Apart from one symbol look-up on its first call on a device it
 * only launches kernels on `stream`; stage timing (sedd_profile_enable) skips it.
 *
 * Limit: the call needs 24 bytes per (document, band) record, 4 bytes per document, 1 KiB per
 * band per 4096 documents and about 70 KiB besides; n_docs * b <= 1,048,576 with b <= 64 always
 * fits (for example 65,536 documents x 16 bands).  A larger input returns SEDD_ELIMIT and
 * enqueues nothing.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (on two
 * streams, or from two threads) race; calls on one stream, or otherwise ordered, do not.
 * Nothing in the array has to survive between calls; every call clears what it reads.
 */
#define SEDD_STATIC_SCRATCH_MIB 32
int sedd_cluster_static(const uint64_t *keys, uint64_t n_docs, int32_t b, int64_t *cluster_id,
                        void *stream);

/*
 * Verified duplicate clusters (Section 2.3, last step; Section 3.3: inside every bucket all
 * document pairs are compared on their full signatures).  Documents u, v are linked when they
 * share a key in some band AND the number of positions k < K with sig[u*K + k] == sig[v*K + k]
 * is at least min_match; cluster_id[d] = the smallest document index in d's connected component
 * of that graph.  min_match is the smallest integer >= theta * K for the paper's similarity
 * threshold theta (theta = 0.8, K = 128: 103); the caller takes that ceiling, so the test is on
 * integers.  min_match = 0 gives the clusters of sedd_cluster.
 *
 * keys, cluster_id as in sedd_cluster; sig device, uint32[n_docs*K], all K columns are compared.
 * Cost: in a bucket of at most 64 documents every document is compared with the bucket's first
 * document, and only those that fail with the rest of the bucket.  A larger bucket is compared
 * all pairs, 64 x 64 documents at a time, first against its leading 64 documents; blocks of pairs
 * whose documents are all joined to the bucket's first document by then are skipped.  There the
 * match count of a pair is first bounded from one-bit sketches of the two signatures (entries
 * whose lowest bits differ are unequal) and the signatures are compared entry by entry only if
 * the bound reaches min_match.  All of this yields the components of the exhaustive comparison.
 * Scratch: beside the sort buffers, n_docs * ceil(K / 32) * 4 bytes for the sketches.
 * The records are first sorted by the low key bits only (2^bits >= 256 n_docs); every comparison
 * also compares the whole keys, so a group that holds a few records of another bucket costs a few
 * comparisons more.  When more than n_docs * b / 1024 records sit in groups of more than 64 that
 * hold different keys, the call sorts by the whole key before it compares anything: keys that
 * agree in their low bits never merge buckets into all-pairs blocks of unbounded size.
 */
int sedd_cluster_verified(const uint64_t *keys, const uint32_t *sig, uint64_t n_docs, int32_t K,
                          int32_t b, int32_t min_match, int64_t *cluster_id, void *stream);

/*
 * The count that the threshold test of Section 3.3, Eq. 3 ("similarity >= theta * H") needs, for
 * theta = theta_num / theta_den: the smallest integer m with m * theta_den >= theta_num * K.
 * Integer arithmetic only (0.8 * 125 is exactly 100, 0.8 * 128 gives 103).  Host-side, touches no
 * device.  Returns SEDD_EINVAL for theta_den == 0, K < 0 or a result above 2^31 - 1.
 */
int32_t sedd_min_match(uint64_t theta_num, uint64_t theta_den, int32_t K);

/*
 * The number of dense buckets the paper pairs with sedd_lsh_dense_keys: k * sqrt(n_docs), k = 4 in
 * Section 3.2 (the appendix on the effect of k varies it), taken as floor(sqrt(k^2 * n_docs)) and
 * at least 1.  Integer arithmetic only, host-side.
 */
uint64_t sedd_dense_bucket_count(uint64_t n_docs, uint32_t k);

/*
 * Caller-provided workspace (Section 3.3's per-bucket buffers and the union graph of Section 2.2
 * are scratch here: nothing in them outlives a call).  sedd_cluster_ws and
 * sedd_cluster_verified_ws are sedd_cluster and sedd_cluster_verified with every scratch buffer
 * carved out of `workspace` (device memory, any alignment) instead of the library's arena: they
 * allocate nothing, and calls with different workspaces may overlap on different streams.
 * sedd_cluster_workspace_bytes gives the size to pass: K = 0 for sedd_cluster_ws, the signature
 * length for sedd_cluster_verified_ws; it returns 0 for arguments the calls would reject.
 * A workspace that is too small is SEDD_ELIMIT, a null one SEDD_EINVAL; nothing is enqueued then.
 */
uint64_t sedd_cluster_workspace_bytes(uint64_t n_docs, int32_t b, int32_t K);
int sedd_cluster_ws(const uint64_t *keys, uint64_t n_docs, int32_t b, int64_t *cluster_id,
                    void *workspace, uint64_t workspace_bytes, void *stream);
int sedd_cluster_verified_ws(const uint64_t *keys, const uint32_t *sig, uint64_t n_docs, int32_t K,
                             int32_t b, int32_t min_match, int64_t *cluster_id, void *workspace,
                             uint64_t workspace_bytes, void *stream);

/* Text for an error code (static storage). */
const char *sedd_strerror(int code);
/* Text of the HIP error behind the last SEDD_EDEVICE or SEDD_ENOMEM of this thread (static storage). */
const char *sedd_last_device_error(void);
/* Library version, major*10000 + minor*100 + patch. */
int sedd_version(void);
/* Free the library-owned device and pinned-host scratch (blocks until the device is idle). */
int sedd_release_scratch(void);
/* Bytes of device scratch currently held. */
uint64_t sedd_scratch_bytes(void);

#ifdef __cplusplus
}
#endif
#endif /* SEDD_H */
