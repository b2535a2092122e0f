"""ctypes binding of the CPU oracle (``sedd_oracle.c``).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg import this package.  It takes and returns
host numpy arrays and never touches the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sedd_oracle.c")
_LIB = os.path.join(_HERE, "libsedd_oracle.so")

P61 = (1 << 61) - 1
P_PAPER = 4294967           # the modulus Section 3.2 quotes for the paper's experiments
FLAG_BYTE_SHINGLES = 1
FLAG_PAPER_PRIME = 2
FLAG_ROLLING_FAMILY = 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = C.CDLL(_LIB)
        u64, i32, u32, vp = C.c_uint64, C.c_int32, C.c_uint32, C.c_void_p
        lib.sedd_ref_mulmod.restype = u64
        lib.sedd_ref_mulmod.argtypes = [u64, u64]
        lib.sedd_ref_addmod.restype = u64
        lib.sedd_ref_addmod.argtypes = [u64, u64]
        lib.sedd_ref_powmod.restype = u64
        lib.sedd_ref_powmod.argtypes = [u64, u64]
        lib.sedd_ref_base_hash.restype = u64
        lib.sedd_ref_base_hash.argtypes = [vp, u64]
        lib.sedd_ref_base_hash_pp.restype = u64
        lib.sedd_ref_base_hash_pp.argtypes = [vp, u64]
        lib.sedd_ref_coeffs_pp.restype = C.c_int
        lib.sedd_ref_coeffs_pp.argtypes = [u64, i32, vp, vp]
        lib.sedd_ref_minhash_shingles_pp.restype = C.c_int
        lib.sedd_ref_minhash_shingles_pp.argtypes = [vp, u64, i32, u64, vp]
        lib.sedd_ref_base_hash_q.restype = u64
        lib.sedd_ref_base_hash_q.argtypes = [vp, u64, u64]
        lib.sedd_ref_bases.restype = C.c_int
        lib.sedd_ref_bases.argtypes = [u64, i32, vp]
        lib.sedd_ref_doc_shingles_q.restype = u64
        lib.sedd_ref_doc_shingles_q.argtypes = [vp, u64, i32, u32, u64, vp, u64]
        lib.sedd_ref_coeffs.restype = C.c_int
        lib.sedd_ref_coeffs.argtypes = [u64, i32, vp, vp]
        lib.sedd_ref_doc_shingles.restype = u64
        lib.sedd_ref_doc_shingles.argtypes = [vp, u64, i32, u32, vp, u64]
        lib.sedd_ref_minhash_shingles.restype = C.c_int
        lib.sedd_ref_minhash_shingles.argtypes = [vp, u64, i32, u64, vp]
        lib.sedd_ref_minhash.restype = C.c_int
        lib.sedd_ref_minhash.argtypes = [vp, vp, u64, i32, i32, u64, u32, vp]
        lib.sedd_ref_lsh_keys.restype = C.c_int
        lib.sedd_ref_lsh_keys.argtypes = [vp, u64, i32, i32, i32, vp]
        lib.sedd_ref_cluster.restype = C.c_int
        lib.sedd_ref_cluster.argtypes = [vp, u64, i32, vp]
        lib.sedd_ref_lsh_dense_keys.restype = C.c_int
        lib.sedd_ref_lsh_dense_keys.argtypes = [vp, u64, i32, i32, i32, u64, vp]
        lib.sedd_ref_cluster_verified.restype = C.c_int
        lib.sedd_ref_cluster_verified.argtypes = [vp, vp, u64, i32, i32, i32, vp]
        _lib = lib
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle returned {code}")
        self.code = code


def _ptr(a):
    return a.ctypes.data if a is not None and a.size else None


def _as_bytes(data) -> np.ndarray:
    if isinstance(data, (bytes, bytearray)):
        return np.frombuffer(bytes(data), dtype=np.uint8)
    return np.ascontiguousarray(data, dtype=np.uint8)


def mulmod(a: int, b: int) -> int:
    return _load().sedd_ref_mulmod(a, b)


def addmod(a: int, b: int) -> int:
    return _load().sedd_ref_addmod(a, b)


def powmod(g: int, e: int) -> int:
    return _load().sedd_ref_powmod(g, e)


def base_hash(s) -> int:
    s = _as_bytes(s)
    return _load().sedd_ref_base_hash(_ptr(s), s.size)


def base_hash_pp(s) -> int:
    """Eq. 1 modulo the paper's own prime."""
    s = _as_bytes(s)
    return _load().sedd_ref_base_hash_pp(_ptr(s), s.size)


def base_hash_q(s, q: int) -> int:
    """Eq. 1 to the base q, modulo 2^61 - 1."""
    s = _as_bytes(s)
    return _load().sedd_ref_base_hash_q(_ptr(s), s.size, q)


def bases(seed: int, K: int) -> np.ndarray:
    """Bases q_k of the rolling-family mode."""
    q = np.zeros(K, dtype=np.uint64)
    rc = _load().sedd_ref_bases(seed, K, q.ctypes.data)
    if rc:
        raise OracleError(rc)
    return q


def doc_shingles_q(text, n: int, q: int, byte_mode: bool = False) -> np.ndarray:
    """Eq. 1 to the base q of the shingles of one document, in order."""
    t = _as_bytes(text)
    lib = _load()
    flags = FLAG_BYTE_SHINGLES if byte_mode else 0
    cnt = lib.sedd_ref_doc_shingles_q(_ptr(t), t.size, n, flags, q, None, 0)
    out = np.zeros(cnt, dtype=np.uint64)
    if cnt:
        lib.sedd_ref_doc_shingles_q(_ptr(t), t.size, n, flags, q, out.ctypes.data, cnt)
    return out


def coeffs(seed: int, K: int, paper_prime: bool = False):
    a = np.zeros(K, dtype=np.uint64)
    b = np.zeros(K, dtype=np.uint64)
    fn = _load().sedd_ref_coeffs_pp if paper_prime else _load().sedd_ref_coeffs
    rc = fn(seed, K, a.ctypes.data, b.ctypes.data)
    if rc:
        raise OracleError(rc)
    return a, b


def doc_shingles(text, n: int, byte_mode: bool = False, paper_prime: bool = False) -> np.ndarray:
    """Base hashes (Eq. 1) of the shingles of one document, in order."""
    t = _as_bytes(text)
    lib = _load()
    flags = (FLAG_BYTE_SHINGLES if byte_mode else 0) | (FLAG_PAPER_PRIME if paper_prime else 0)
    cnt = lib.sedd_ref_doc_shingles(_ptr(t), t.size, n, flags, None, 0)
    out = np.zeros(cnt, dtype=np.uint64)
    if cnt:
        lib.sedd_ref_doc_shingles(_ptr(t), t.size, n, flags, out.ctypes.data, cnt)
    return out


def minhash_shingles(x, K: int, seed: int = 0, paper_prime: bool = False) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.uint64)
    sig = np.zeros(K, dtype=np.uint32)
    fn = _load().sedd_ref_minhash_shingles_pp if paper_prime else _load().sedd_ref_minhash_shingles
    rc = fn(_ptr(x), x.size, K, seed, sig.ctypes.data)
    if rc:
        raise OracleError(rc)
    return sig


def minhash(data, doc_offsets, shingle_n: int, K: int, seed: int = 0, flags: int = 0) -> np.ndarray:
    data = _as_bytes(data)
    off = np.ascontiguousarray(doc_offsets, dtype=np.uint64)
    n_docs = max(0, off.size - 1)
    sig = np.zeros((n_docs, max(K, 0)), dtype=np.uint32)
    rc = _load().sedd_ref_minhash(_ptr(data), _ptr(off), n_docs, shingle_n, K, seed, flags,
                                  _ptr(sig))
    if rc:
        raise OracleError(rc)
    return sig


def lsh_keys(sig, b: int, r: int) -> np.ndarray:
    sig = np.ascontiguousarray(sig, dtype=np.uint32)
    n_docs, K = sig.shape
    keys = np.zeros((n_docs, max(b, 0)), dtype=np.uint64)
    rc = _load().sedd_ref_lsh_keys(_ptr(sig), n_docs, K, b, r, _ptr(keys))
    if rc:
        raise OracleError(rc)
    return keys


def cluster(keys) -> np.ndarray:
    keys = np.ascontiguousarray(keys, dtype=np.uint64)
    n_docs, b = keys.shape
    cid = np.zeros(n_docs, dtype=np.int64)
    rc = _load().sedd_ref_cluster(_ptr(keys), n_docs, b, _ptr(cid))
    if rc:
        raise OracleError(rc)
    return cid


def dense_bucket_count(n_docs: int, k: int = 4) -> int:
    """The paper's number of buckets, k * sqrt(N) with k = 4 (Section 3.2), as the integer
    floor(sqrt(k^2 N)), at least 1."""
    import math
    return max(1, math.isqrt(k * k * int(n_docs)))


def lsh_dense_keys(sig, b: int, r: int, n_buckets: int) -> np.ndarray:
    """Dense bucket ids: sum of the band's values modulo the number of buckets (Section 3.2)."""
    sig = np.ascontiguousarray(sig, dtype=np.uint32)
    n_docs, K = sig.shape
    keys = np.zeros((n_docs, max(b, 0)), dtype=np.uint64)
    rc = _load().sedd_ref_lsh_dense_keys(_ptr(sig), n_docs, K, b, r, int(n_buckets), _ptr(keys))
    if rc:
        raise OracleError(rc)
    return keys


def min_match_for(theta: float, K: int) -> int:
    """Smallest integer m with m >= theta * K (the threshold test of Section 3.3 on integers).
    theta is taken as the decimal fraction it prints as, so 0.8 * 125 is exactly 100."""
    from fractions import Fraction
    t = Fraction(str(theta)) * K
    return int(-((-t.numerator) // t.denominator))


def cluster_verified(keys, sig, min_match: int) -> np.ndarray:
    """Clusters from duplicate pairs verified on the full signatures (Section 3.3)."""
    keys = np.ascontiguousarray(keys, dtype=np.uint64)
    sig = np.ascontiguousarray(sig, dtype=np.uint32)
    n_docs, b = keys.shape
    K = sig.shape[1]
    assert sig.shape[0] == n_docs
    cid = np.zeros(n_docs, dtype=np.int64)
    rc = _load().sedd_ref_cluster_verified(_ptr(keys), _ptr(sig), n_docs, K, b, int(min_match),
                                           _ptr(cid))
    if rc:
        raise OracleError(rc)
    return cid


def minhash_sharded(data, doc_offsets, shingle_n: int, K: int, seed: int = 0, flags: int = 0,
                    procs: int = 1) -> np.ndarray:
    """The single-threaded oracle run by `procs` worker threads over disjoint document ranges.

    Each worker calls the same C routine (``sedd_ref_minhash``, which holds no shared state and
    runs without the interpreter lock) on a contiguous range of documents: its text slice and its
    offsets rebased to that slice.  A document's signature depends on nothing but its own bytes,
    so the result equals ``minhash`` on the whole corpus (pinned in tests/test_oracle_minhash.py).
    Threads rather than forked processes: the callers may hold a GPU context, which must not be
    forked.
    """
    data = _as_bytes(data)
    off = np.ascontiguousarray(doc_offsets, dtype=np.uint64)
    n_docs = max(0, off.size - 1)
    if procs <= 1 or n_docs < 2 * procs:
        return minhash(data, off, shingle_n, K, seed, flags)
    from concurrent.futures import ThreadPoolExecutor
    _load()
    n_sh = procs * 8
    cuts = [n_docs * i // n_sh for i in range(n_sh + 1)]
    jobs = [(cuts[i], cuts[i + 1]) for i in range(n_sh) if cuts[i + 1] > cuts[i]]
    sig = np.zeros((n_docs, K), dtype=np.uint32)

    def work(rng):
        d0, d1 = rng
        base = int(off[d0])
        sub = data[base:int(off[d1])]
        sig[d0:d1] = minhash(sub, off[d0:d1 + 1] - np.uint64(base), shingle_n, K, seed, flags)

    with ThreadPoolExecutor(max_workers=procs) as pool:
        list(pool.map(work, jobs))
    return sig
