"""MI355X-native MinHash-LSH deduplication hot path (SEDD paper, Sections 2.2-3.2).

Thin binding over the C-ABI library ``libsedd.so`` (hand-written HIP for gfx950).  The
functions here only marshal arguments: torch supplies device memory and the current HIP
stream, every step of the path runs in the library's kernels.  There is no CPU fallback:
if the library has not been built, or there is no GPU, the calls raise.

    sig  = sedd_minhash(text_u8, doc_offsets_u64, shingle_n=5, K=128)   # uint32 [n_docs, K]
    keys = sedd_lsh_keys(sig, b=16, r=8)                                  # uint64 [n_docs, b]
    cid  = sedd_cluster(keys)                                             # int64  [n_docs]
    cid  = sedd_cluster_verified(keys, sig, min_match_for(0.8, 128))      # Section 3.3 clusters
"""
from __future__ import annotations

import ctypes as C
import os

__all__ = [
    "SeddError", "lib", "lib_path", "sedd_minhash", "sedd_minhash_host_chunked", "sedd_lsh_keys", "sedd_cluster",
    "sedd_cluster_verified", "sedd_cluster_static", "sedd_cluster_ws",
    "sedd_cluster_workspace_bytes", "min_match_for", "sedd_lsh_dense_keys", "dense_bucket_count",
    "sedd_release_scratch", "sedd_scratch_bytes", "sedd_version", "debug_shingle_hashes",
    "debug_coeffs", "debug_scan_u32", "debug_sort_bands", "debug_set_chunk_bytes",
    "debug_minhash_from_x", "debug_stats", "profile_enable", "profile_read",
    "debug_shingle_hashes_offsets",
    "FLAG_BYTE_SHINGLES", "FLAG_PAPER_PRIME", "FLAG_ROLLING_FAMILY", "debug_bases",
]

FLAG_BYTE_SHINGLES = 1
FLAG_PAPER_PRIME = 2      # Eq. 1 and the K functions modulo 4,294,967 (Section 3.2)
FLAG_ROLLING_FAMILY = 4   # function k is Eq. 1 itself to a base q_k of its own
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsedd.so")
_lib = None


class SeddError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        msg = f"{where} failed with code {code}"
        if detail:
            msg += f": {detail}"
        super().__init__(msg)


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2501_01046_amd.build` "
                "(there is no fallback path)")
        # torch first: it brings its own HIP runtime, and the library must bind to that one.  Loaded
        # before torch, the library pulls in the system's runtime instead, torch then finds a runtime
        # that is not the one it was built with, and allocations fail.
        import torch  # noqa: F401
        L = C.CDLL(_LIB_PATH)
        u64, i32, u32, vp = C.c_uint64, C.c_int32, C.c_uint32, C.c_void_p
        L.sedd_minhash.restype = C.c_int
        L.sedd_minhash.argtypes = [vp, vp, u64, i32, i32, u64, u32, vp, vp]
        L.sedd_minhash_bounded.restype = C.c_int
        L.sedd_minhash_bounded.argtypes = [vp, u64, vp, u64, i32, i32, u64, u32, vp, vp]
        L.sedd_debug_set_piece_bytes.restype = C.c_int
        L.sedd_debug_set_piece_bytes.argtypes = [u32]
        L.sedd_minhash_host_chunked.restype = C.c_int
        L.sedd_minhash_host_chunked.argtypes = [vp, vp, u64, i32, i32, u64, u32, u64, vp, vp]
        L.sedd_lsh_keys.restype = C.c_int
        L.sedd_lsh_keys.argtypes = [vp, u64, i32, i32, i32, vp, vp]
        L.sedd_cluster.restype = C.c_int
        L.sedd_cluster.argtypes = [vp, u64, i32, vp, vp]
        L.sedd_cluster_static.restype = C.c_int
        L.sedd_cluster_static.argtypes = [vp, u64, i32, vp, vp]
        L.sedd_cluster_workspace_bytes.restype = u64
        L.sedd_cluster_workspace_bytes.argtypes = [u64, i32, i32]
        L.sedd_cluster_ws.restype = C.c_int
        L.sedd_cluster_ws.argtypes = [vp, u64, i32, vp, vp, u64, vp]
        L.sedd_cluster_verified_ws.restype = C.c_int
        L.sedd_cluster_verified_ws.argtypes = [vp, vp, u64, i32, i32, i32, vp, vp, u64, vp]
        L.sedd_debug_set_scratch_cap.restype = C.c_int
        L.sedd_debug_set_scratch_cap.argtypes = [u64]
        L.sedd_lsh_dense_keys.restype = C.c_int
        L.sedd_lsh_dense_keys.argtypes = [vp, u64, i32, i32, i32, u64, vp, vp]
        L.sedd_cluster_verified.restype = C.c_int
        L.sedd_cluster_verified.argtypes = [vp, vp, u64, i32, i32, i32, vp, vp]
        L.sedd_min_match.restype = i32
        L.sedd_min_match.argtypes = [u64, u64, i32]
        L.sedd_dense_bucket_count.restype = u64
        L.sedd_dense_bucket_count.argtypes = [u64, u32]
        L.sedd_strerror.restype = C.c_char_p
        L.sedd_strerror.argtypes = [C.c_int]
        L.sedd_last_device_error.restype = C.c_char_p
        L.sedd_version.restype = C.c_int
        L.sedd_release_scratch.restype = C.c_int
        L.sedd_scratch_bytes.restype = u64
        L.sedd_debug_shingle_hashes.restype = C.c_int
        L.sedd_debug_shingle_hashes.argtypes = [vp, vp, u64, i32, u32, vp, u64, vp, vp]
        L.sedd_debug_coeffs.restype = C.c_int
        L.sedd_debug_coeffs.argtypes = [u64, i32, vp, vp, vp]
        L.sedd_debug_scan_u32.restype = C.c_int
        L.sedd_debug_scan_u32.argtypes = [vp, vp, u64, vp]
        L.sedd_debug_sort_bands.restype = C.c_int
        L.sedd_debug_sort_bands.argtypes = [vp, u64, i32, vp, vp, vp]
        L.sedd_debug_minhash_from_x.restype = C.c_int
        L.sedd_debug_minhash_from_x.argtypes = [vp, vp, u64, u64, i32, u64, vp, vp]
        L.sedd_debug_minhash_from_x_pp.restype = C.c_int
        L.sedd_debug_minhash_from_x_pp.argtypes = [vp, vp, u64, u64, i32, u64, vp, vp]
        L.sedd_debug_bases.restype = C.c_int
        L.sedd_debug_bases.argtypes = [u64, i32, vp, vp]
        L.sedd_debug_coeffs_pp.restype = C.c_int
        L.sedd_debug_coeffs_pp.argtypes = [u64, i32, vp, vp, vp]
        L.sedd_debug_stats.restype = C.c_int
        L.sedd_debug_stats.argtypes = [vp]
        L.sedd_profile_enable.restype = C.c_int
        L.sedd_profile_enable.argtypes = [C.c_int]
        L.sedd_profile_read.restype = C.c_int
        L.sedd_profile_read.argtypes = [vp, vp]
        L.sedd_profile_label.restype = C.c_char_p
        L.sedd_profile_label.argtypes = [C.c_int]
        L.sedd_debug_last_regroup.restype = C.c_int
        L.sedd_debug_last_regroup.argtypes = [vp]
        L.sedd_debug_set_chunk_bytes.restype = C.c_int
        L.sedd_debug_set_chunk_bytes.argtypes = [u64]
        _lib = L
    return _lib


def _check(rc: int, where: str):
    if rc != 0:
        L = lib()
        detail = L.sedd_strerror(rc).decode()
        if rc in (-2, -3):
            last = L.sedd_last_device_error().decode()
            if last:
                detail += " / " + last
        raise SeddError(rc, where, detail)


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: the sedd_* calls run only on a HIP device")
    return torch


def _dev(t, dtype, name):
    torch = _torch()
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _ptr(t):
    return t.data_ptr() if t.numel() else None


def _stream(stream):
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def sedd_minhash(text, doc_offsets, shingle_n: int, K: int, seed: int = 0, flags: int = 0,
                 out=None, stream=None):
    """uint32 [n_docs, K] signatures of the documents text[doc_offsets[d]:doc_offsets[d+1]]."""
    torch = _torch()
    text = _dev(text, torch.uint8, "text")
    doc_offsets = _dev(doc_offsets, torch.uint64, "doc_offsets")
    n_docs = max(0, doc_offsets.numel() - 1)
    if out is None:
        out = torch.empty((n_docs, max(int(K), 0)), dtype=torch.uint32, device=text.device)
    else:
        out = _dev(out, torch.uint32, "out")
        if out.numel() != n_docs * K:
            raise ValueError("out has the wrong size")
    # the bounded entry point: offsets that point past `text` are rejected, not followed
    _check(lib().sedd_minhash_bounded(_ptr(text), text.numel(), _ptr(doc_offsets), n_docs, shingle_n,
                                      K, seed, flags, _ptr(out), _stream(stream)), "sedd_minhash")
    return out


def sedd_minhash_host_chunked(text, doc_offsets, shingle_n: int, K: int, seed: int = 0,
                              flags: int = 0, chunk_bytes: int = 0, out=None, stream=None):
    """sedd_minhash for text in host memory: `text` (uint8) and `doc_offsets` (uint64 or int64,
    n_docs + 1 entries) are CPU tensors, ideally pinned; the library uploads chunks of at most
    chunk_bytes behind the hashing of the previous chunk.  Returns device signatures."""
    torch = _torch()
    for t, name in ((text, "text"), (doc_offsets, "doc_offsets")):
        if not isinstance(t, torch.Tensor) or t.is_cuda or not t.is_contiguous():
            raise TypeError(f"{name} must be a contiguous CPU tensor")
    if text.dtype != torch.uint8 or doc_offsets.dtype not in (torch.uint64, torch.int64):
        raise TypeError("text must be uint8 and doc_offsets uint64 (or int64)")
    n_docs = max(0, doc_offsets.numel() - 1)
    if out is None:
        out = torch.empty((n_docs, max(int(K), 0)), dtype=torch.uint32, device="cuda")
    else:
        out = _dev(out, torch.uint32, "out")
        if out.numel() != n_docs * K:
            raise ValueError("out has the wrong size")
    _check(lib().sedd_minhash_host_chunked(_ptr(text), _ptr(doc_offsets), n_docs, shingle_n, K, seed,
                                           flags, int(chunk_bytes), _ptr(out), _stream(stream)),
           "sedd_minhash_host_chunked")
    return out


def sedd_lsh_keys(sig, b: int, r: int, out=None, stream=None):
    """uint64 [n_docs, b] band keys of uint32 [n_docs, K] signatures."""
    torch = _torch()
    sig = _dev(sig, torch.uint32, "sig")
    n_docs, K = sig.shape
    if out is None:
        out = torch.empty((n_docs, max(int(b), 0)), dtype=torch.uint64, device=sig.device)
    else:
        out = _dev(out, torch.uint64, "out")
        if out.numel() != n_docs * b:
            raise ValueError("out has the wrong size")
    _check(lib().sedd_lsh_keys(_ptr(sig), n_docs, K, b, r, _ptr(out), _stream(stream)),
           "sedd_lsh_keys")
    return out


def sedd_cluster(keys, out=None, stream=None):
    """int64 [n_docs] smallest document index of each document's connected component."""
    torch = _torch()
    keys = _dev(keys, torch.uint64, "keys")
    n_docs, b = keys.shape
    if out is None:
        out = torch.empty((n_docs,), dtype=torch.int64, device=keys.device)
    else:
        out = _dev(out, torch.int64, "out")
        if out.numel() != n_docs:
            raise ValueError("out has the wrong size")
    _check(lib().sedd_cluster(_ptr(keys), n_docs, b, _ptr(out), _stream(stream)), "sedd_cluster")
    return out


def sedd_cluster_static(keys, out, stream=None):
    """sedd_cluster through the entry point that allocates nothing: `out` (int64 [n_docs]) is
    required, scratch is the library's fixed array; raises SeddError(-4) beyond its limit."""
    torch = _torch()
    keys = _dev(keys, torch.uint64, "keys")
    out = _dev(out, torch.int64, "out")
    n_docs, b = keys.shape
    if out.numel() != n_docs:
        raise ValueError("out has the wrong size")
    _check(lib().sedd_cluster_static(_ptr(keys), n_docs, b, _ptr(out), _stream(stream)),
           "sedd_cluster_static")
    return out


def sedd_cluster_workspace_bytes(n_docs: int, b: int, K: int = 0) -> int:
    """Bytes of workspace sedd_cluster (K = 0) or sedd_cluster_verified (K = signature length)
    needs when the caller provides it."""
    return int(lib().sedd_cluster_workspace_bytes(int(n_docs), int(b), int(K)))


def sedd_cluster_ws(keys, workspace, out=None, sig=None, min_match=None, stream=None):
    """sedd_cluster (or, with sig and min_match, sedd_cluster_verified) on a caller-provided
    workspace: a uint8 device tensor of at least sedd_cluster_workspace_bytes(...) bytes."""
    torch = _torch()
    keys = _dev(keys, torch.uint64, "keys")
    workspace = _dev(workspace, torch.uint8, "workspace")
    n_docs, b = keys.shape
    if out is None:
        out = torch.empty((n_docs,), dtype=torch.int64, device=keys.device)
    else:
        out = _dev(out, torch.int64, "out")
        if out.numel() != n_docs:
            raise ValueError("out has the wrong size")
    if sig is None:
        _check(lib().sedd_cluster_ws(_ptr(keys), n_docs, b, _ptr(out), _ptr(workspace),
                                     workspace.numel(), _stream(stream)), "sedd_cluster_ws")
    else:
        sig = _dev(sig, torch.uint32, "sig")
        if sig.shape[0] != n_docs:
            raise ValueError("sig and keys describe different numbers of documents")
        _check(lib().sedd_cluster_verified_ws(_ptr(keys), _ptr(sig), n_docs, sig.shape[1], b,
                                              int(min_match), _ptr(out), _ptr(workspace),
                                              workspace.numel(), _stream(stream)),
               "sedd_cluster_verified_ws")
    return out


def debug_set_scratch_cap(n: int):
    _check(lib().sedd_debug_set_scratch_cap(n), "sedd_debug_set_scratch_cap")


def dense_bucket_count(n_docs: int, k: int = 4) -> int:
    """Number of dense buckets the paper uses, k * sqrt(N) with k = 4: floor(sqrt(k^2 N)), >= 1."""
    return int(lib().sedd_dense_bucket_count(int(n_docs), int(k)))


def sedd_lsh_dense_keys(sig, b: int, r: int, n_buckets: int, out=None, stream=None):
    """uint64 [n_docs, b] dense bucket ids: band sum modulo n_buckets (Section 3.2)."""
    torch = _torch()
    sig = _dev(sig, torch.uint32, "sig")
    n_docs, K = sig.shape
    if out is None:
        out = torch.empty((n_docs, max(b, 0)), dtype=torch.uint64, device=sig.device)
    else:
        out = _dev(out, torch.uint64, "out")
        if out.numel() != n_docs * b:
            raise ValueError("out has the wrong size")
    _check(lib().sedd_lsh_dense_keys(_ptr(sig), n_docs, K, b, r, int(n_buckets), _ptr(out),
                                     _stream(stream)), "sedd_lsh_dense_keys")
    return out


def min_match_for(theta: float, K: int) -> int:
    """Smallest integer m with m >= theta * K: the count the threshold test of Section 3.3 needs.
    theta is read as the decimal fraction it prints as (0.8 * 125 is exactly 100)."""
    from decimal import Decimal
    num, den = Decimal(str(theta)).as_integer_ratio()
    m = lib().sedd_min_match(num, den, int(K))
    if m < 0:
        raise SeddError(m, "sedd_min_match", "theta must be a non-negative fraction, K >= 0")
    return int(m)


def sedd_cluster_verified(keys, sig, min_match: int, out=None, stream=None):
    """int64 [n_docs] clusters of document pairs that share a band key and agree on at least
    min_match signature entries (min_match = min_match_for(theta, K))."""
    torch = _torch()
    keys = _dev(keys, torch.uint64, "keys")
    sig = _dev(sig, torch.uint32, "sig")
    n_docs, b = keys.shape
    if sig.shape[0] != n_docs:
        raise ValueError("sig and keys describe different numbers of documents")
    K = sig.shape[1]
    if out is None:
        out = torch.empty((n_docs,), dtype=torch.int64, device=keys.device)
    else:
        out = _dev(out, torch.int64, "out")
        if out.numel() != n_docs:
            raise ValueError("out has the wrong size")
    _check(lib().sedd_cluster_verified(_ptr(keys), _ptr(sig), n_docs, K, b, int(min_match),
                                       _ptr(out), _stream(stream)), "sedd_cluster_verified")
    return out


def sedd_release_scratch():
    _check(lib().sedd_release_scratch(), "sedd_release_scratch")


def sedd_scratch_bytes() -> int:
    return lib().sedd_scratch_bytes()


def sedd_version() -> int:
    return lib().sedd_version()


# ---- stage-level entry points (parity tests of intermediate results) -----------------------

def debug_shingle_hashes(text, doc_offsets, shingle_n: int, flags: int = 0, stream=None):
    """(x uint64[n_shingles], shingle_offsets uint64[n_docs+1]) of Eq. 1 base hashes."""
    torch = _torch()
    text = _dev(text, torch.uint8, "text")
    doc_offsets = _dev(doc_offsets, torch.uint64, "doc_offsets")
    n_docs = max(0, doc_offsets.numel() - 1)
    soff = torch.zeros(n_docs + 1, dtype=torch.uint64, device=text.device)
    L = lib()
    _check(L.sedd_debug_shingle_hashes(_ptr(text), _ptr(doc_offsets), n_docs, shingle_n, flags,
                                       None, 0, _ptr(soff), _stream(stream)),
           "sedd_debug_shingle_hashes")
    total = int(soff[-1].item())
    x = torch.zeros(total, dtype=torch.uint64, device=text.device)
    _check(L.sedd_debug_shingle_hashes(_ptr(text), _ptr(doc_offsets), n_docs, shingle_n, flags,
                                       _ptr(x), total, _ptr(soff), _stream(stream)),
           "sedd_debug_shingle_hashes")
    return x, soff


def debug_shingle_hashes_offsets(text, doc_offsets, shingle_n: int, flags: int = 0, stream=None):
    """(None, shingle_offsets as a host numpy array): the counting half of debug_shingle_hashes."""
    torch = _torch()
    text = _dev(text, torch.uint8, "text")
    doc_offsets = _dev(doc_offsets, torch.uint64, "doc_offsets")
    n_docs = max(0, doc_offsets.numel() - 1)
    soff = torch.zeros(n_docs + 1, dtype=torch.uint64, device=text.device)
    _check(lib().sedd_debug_shingle_hashes(_ptr(text), _ptr(doc_offsets), n_docs, shingle_n, flags,
                                           None, 0, _ptr(soff), _stream(stream)),
           "sedd_debug_shingle_hashes")
    return None, soff.cpu().numpy()


def debug_coeffs(seed: int, K: int, stream=None, paper_prime: bool = False):
    torch = _torch()
    a = torch.zeros(max(K, 0), dtype=torch.uint64, device="cuda")
    b = torch.zeros(max(K, 0), dtype=torch.uint64, device="cuda")
    fn = lib().sedd_debug_coeffs_pp if paper_prime else lib().sedd_debug_coeffs
    _check(fn(seed, K, _ptr(a), _ptr(b), _stream(stream)), "sedd_debug_coeffs")
    return a, b


def debug_bases(seed: int, K: int, stream=None):
    torch = _torch()
    q = torch.zeros(max(K, 0), dtype=torch.uint64, device="cuda")
    _check(lib().sedd_debug_bases(seed, K, _ptr(q), _stream(stream)), "sedd_debug_bases")
    return q


def debug_scan_u32(values, stream=None):
    torch = _torch()
    values = _dev(values, torch.uint32, "values")
    out = torch.empty_like(values)
    _check(lib().sedd_debug_scan_u32(_ptr(values), _ptr(out), values.numel(), _stream(stream)),
           "sedd_debug_scan_u32")
    return out


def debug_sort_bands(keys, stream=None):
    torch = _torch()
    keys = _dev(keys, torch.uint64, "keys")
    n_docs, b = keys.shape
    ks = torch.empty((b, n_docs), dtype=torch.uint64, device=keys.device)
    ds = torch.empty((b, n_docs), dtype=torch.uint32, device=keys.device)
    _check(lib().sedd_debug_sort_bands(_ptr(keys), n_docs, b, _ptr(ks), _ptr(ds), _stream(stream)),
           "sedd_debug_sort_bands")
    return ks, ds


def debug_set_chunk_bytes(n: int):
    _check(lib().sedd_debug_set_chunk_bytes(n), "sedd_debug_set_chunk_bytes")


def debug_set_piece_bytes(n: int):
    _check(lib().sedd_debug_set_piece_bytes(n), "sedd_debug_set_piece_bytes")


def debug_minhash_from_x(x, shingle_offsets, K: int, seed: int = 0, stream=None, out=None,
                         paper_prime: bool = False):
    """Signatures from caller-supplied shingle hashes (the K-hash / minimum kernel alone)."""
    torch = _torch()
    x = _dev(x, torch.uint64, "x")
    shingle_offsets = _dev(shingle_offsets, torch.uint64, "shingle_offsets")
    n_docs = max(0, shingle_offsets.numel() - 1)
    if out is None:
        sig = torch.empty((n_docs, max(K, 0)), dtype=torch.uint32, device=x.device)
    else:
        sig = _dev(out, torch.uint32, "out")
        if sig.numel() != n_docs * K:
            raise ValueError("out has the wrong size")
    fn = lib().sedd_debug_minhash_from_x_pp if paper_prime else lib().sedd_debug_minhash_from_x
    _check(fn(_ptr(x), _ptr(shingle_offsets), n_docs, x.numel(), K, seed, _ptr(sig),
              _stream(stream)), "sedd_debug_minhash_from_x")
    return sig


STAT_SLOW_TILES = 0
_STAT_N = 16
_PROF_N = 8


def debug_stats():
    """Device-side counters since the library was loaded (list of ints; waits for the device)."""
    buf = (C.c_uint64 * _STAT_N)()
    _check(lib().sedd_debug_stats(buf), "sedd_debug_stats")
    return list(buf)


def debug_last_regroup() -> int:
    """1 if the last clustering call fell back to sorting by the whole key (waits for the device)."""
    out = C.c_uint32(0)
    _check(lib().sedd_debug_last_regroup(C.byref(out)), "sedd_debug_last_regroup")
    return int(out.value)


def profile_enable(on: bool):
    _check(lib().sedd_profile_enable(1 if on else 0), "sedd_profile_enable")


def profile_read():
    """{stage: (milliseconds, timed spans)} accumulated since the last read (waits for them)."""
    ms = (C.c_double * _PROF_N)()
    spans = (C.c_uint64 * _PROF_N)()
    L = lib()
    _check(L.sedd_profile_read(ms, spans), "sedd_profile_read")
    out = {}
    for i in range(_PROF_N):
        name = L.sedd_profile_label(i).decode()
        if name:
            out[name] = (ms[i], int(spans[i]))
    return out
