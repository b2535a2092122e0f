"""Seeded synthetic corpora (inputs only).

Thin ctypes binding over ``corpus_gen.c``.  Nothing here shingles, hashes or
clusters: this module only manufactures document bytes and offsets, for the
CPU oracle's tests and for the GPU path alike.

The named recipes follow the five benchmark workloads (web-text shaped
corpora standing in for the RealNews / C4 / RedPajama text the paper measures
on, Section 4.1).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, replace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "corpus_gen.c")
_LIB = os.path.join(_HERE, "libsedd_corpus.so")


def build(force: bool = False) -> str:
    """Compile the generator with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Params(C.Structure):
    _fields_ = [
        ("seed", C.c_uint64), ("n_docs", C.c_uint64),
        ("vocab", C.c_uint32), ("utf8_pct", C.c_uint32),
        ("zipf_s", C.c_double),
        ("len_median", C.c_double), ("len_sigma", C.c_double),
        ("len_lo", C.c_uint32), ("len_hi", C.c_uint32),
        ("long_frac", C.c_double),
        ("long_lo", C.c_uint32), ("long_hi", C.c_uint32),
        ("near_frac", C.c_double), ("exact_frac", C.c_double),
        ("edit_lo", C.c_double), ("edit_hi", C.c_double),
        ("max_chain", C.c_uint32), ("ws_variety", C.c_uint32),
    ]


@dataclass(frozen=True)
class Recipe:
    """Corpus recipe plus the method parameters the workload is run with."""
    name: str
    seed: int
    n_docs: int
    vocab: int = 50_000
    utf8_pct: int = 0
    zipf_s: float = 1.1
    len_median: float = 300.0
    len_sigma: float = 0.8
    len_lo: int = 20
    len_hi: int = 5000
    long_frac: float = 0.0
    long_lo: int = 200_000
    long_hi: int = 2_000_000
    near_frac: float = 0.10
    exact_frac: float = 0.0
    edit_lo: float = 0.05
    edit_hi: float = 0.05
    max_chain: int = 8
    ws_variety: int = 0
    # method parameters of the workload (not used by the generator)
    shingle_n: int = 5
    byte_mode: bool = False
    K: int = 128
    b: int = 16
    r: int = 8

    def scaled(self, n_docs: int, **kw) -> "Recipe":
        return replace(self, n_docs=n_docs, **kw)


def config(i: int) -> Recipe:
    """The five workloads, numbered 1..5 (corpus seed = number - 1)."""
    if i == 1:
        return Recipe("cfg1_tiny_5k", seed=0, n_docs=5_000)
    if i == 2:
        return Recipe("cfg2_medium_1M", seed=1, n_docs=1_000_000, near_frac=0.15,
                      edit_lo=0.01, edit_hi=0.20)
    if i == 3:
        return Recipe("cfg3_web_10M", seed=2, n_docs=10_000_000, len_median=500.0,
                      len_sigma=1.2, len_lo=10, len_hi=100_000, near_frac=0.20,
                      exact_frac=0.03, edit_lo=0.01, edit_hi=0.20, K=256, b=32, r=8)
    if i == 4:
        return Recipe("cfg4_longdoc_200k", seed=3, n_docs=200_000, len_median=200.0,
                      long_frac=0.01, near_frac=0.10, edit_lo=0.03, edit_hi=0.03,
                      utf8_pct=5, shingle_n=13, byte_mode=True)
    if i == 5:
        return Recipe("cfg5_sweep_2M", seed=4, n_docs=2_000_000, near_frac=0.15,
                      edit_lo=0.01, edit_hi=0.20)
    raise ValueError("config number must be 1..5")


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = C.CDLL(_LIB)
        lib.corpus_create.restype = C.c_void_p
        lib.corpus_create.argtypes = [C.POINTER(_Params)]
        lib.corpus_destroy.argtypes = [C.c_void_p]
        lib.corpus_generate.restype = C.c_void_p
        lib.corpus_generate.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p,
                                        C.POINTER(C.c_uint64), C.c_int]
        lib.corpus_free_bytes.argtypes = [C.c_void_p]
        lib.corpus_doc_meta.restype = C.c_int
        lib.corpus_doc_meta.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64),
                                        C.POINTER(C.c_double)]
        lib.corpus_doc_words.restype = C.c_uint64
        lib.corpus_doc_words.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64]
        lib.corpus_word.restype = C.c_int
        lib.corpus_word.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p]
        _lib = lib
    return _lib


class Corpus:
    """A generator bound to one recipe; documents are pure functions of (seed, id)."""

    def __init__(self, recipe: Recipe):
        self.recipe = recipe
        lib = _load()
        p = _Params(
            seed=recipe.seed, n_docs=recipe.n_docs, vocab=recipe.vocab, utf8_pct=recipe.utf8_pct,
            zipf_s=recipe.zipf_s, len_median=recipe.len_median, len_sigma=recipe.len_sigma,
            len_lo=recipe.len_lo, len_hi=recipe.len_hi, long_frac=recipe.long_frac,
            long_lo=recipe.long_lo, long_hi=recipe.long_hi, near_frac=recipe.near_frac,
            exact_frac=recipe.exact_frac, edit_lo=recipe.edit_lo, edit_hi=recipe.edit_hi,
            max_chain=recipe.max_chain, ws_variety=recipe.ws_variety)
        self._h = lib.corpus_create(C.byref(p))
        if not self._h:
            raise RuntimeError("corpus_create failed")

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.corpus_destroy(self._h)
            self._h = None

    def generate(self, d0: int = 0, d1: int | None = None, threads: int | None = None):
        """Documents [d0, d1) -> (bytes uint8[total], offsets uint64[d1-d0+1])."""
        if d1 is None:
            d1 = self.recipe.n_docs
        if threads is None:
            threads = min(16, os.cpu_count() or 1)
        n = max(0, d1 - d0)
        offsets = np.zeros(n + 1, dtype=np.uint64)
        total = C.c_uint64(0)
        ptr = _lib.corpus_generate(self._h, d0, d1, offsets.ctypes.data, C.byref(total), threads)
        out = np.empty(total.value, dtype=np.uint8)
        if total.value:
            C.memmove(out.ctypes.data, ptr, total.value)
        _lib.corpus_free_bytes(ptr)
        return out, offsets

    def meta(self, doc: int):
        """(kind, source doc, edit rate); kind 0 fresh, 1 near-duplicate, 2 exact copy."""
        src = C.c_uint64(0)
        rate = C.c_double(0.0)
        k = _lib.corpus_doc_meta(self._h, doc, C.byref(src), C.byref(rate))
        return k, src.value, rate.value

    def word_ids(self, doc: int) -> np.ndarray:
        n = _lib.corpus_doc_words(self._h, doc, None, 0)
        out = np.empty(n, dtype=np.uint32)
        _lib.corpus_doc_words(self._h, doc, out.ctypes.data, n)
        return out

    def word(self, w: int) -> bytes:
        buf = (C.c_uint8 * 16)()
        n = _lib.corpus_word(self._h, w, buf)
        return bytes(buf[:n])


def generate(recipe: Recipe, d0: int = 0, d1: int | None = None, threads: int | None = None):
    """Convenience: bytes and offsets of documents [d0, d1) of a recipe."""
    return Corpus(recipe).generate(d0, d1, threads)
