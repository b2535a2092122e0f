"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports every
symbol the headers declare, and rejects bad arguments before touching the device."""
import ctypes as C
import glob
import os
import re

import pytest

import paper_2501_01046_amd as sedd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = []
    for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        src = open(h).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names += re.findall(r"\b(sedd_\w+)\s*\(", src)
    return sorted(set(names))


def test_headers_declare_the_three_calls():
    names = _declared_symbols()
    for must in ("sedd_minhash", "sedd_lsh_keys", "sedd_cluster", "sedd_strerror"):
        assert must in names


def test_library_exports_every_declared_symbol():
    L = sedd.lib()
    for name in _declared_symbols():
        assert hasattr(L, name), name


def test_version_and_error_strings():
    L = sedd.lib()
    assert L.sedd_version() >= 100
    for code in (0, -1, -2, -3, -99):
        assert L.sedd_strerror(code)
    assert b"invalid" in L.sedd_strerror(-1)


u64 = C.c_uint64
FAKE = C.c_void_p(0x1000)     # never dereferenced: these calls must fail validation first


@pytest.mark.parametrize("n,K,flags", [(0, 8, 0), (65, 8, 0), (5, 0, 0), (5, 4097, 0), (5, 8, 8), (5, 8, 6), (5, 8, 0x80000000), (-1, 8, 0)])
def test_minhash_rejects_bad_scalars(n, K, flags):
    L = sedd.lib()
    assert L.sedd_minhash(FAKE, FAKE, u64(4), n, K, u64(0), flags, FAKE, None) == -1


def test_minhash_rejects_null_pointers_and_accepts_zero_docs():
    L = sedd.lib()
    assert L.sedd_minhash(FAKE, None, u64(4), 5, 8, u64(0), 0, FAKE, None) == -1
    assert L.sedd_minhash(FAKE, FAKE, u64(4), 5, 8, u64(0), 0, None, None) == -1
    assert L.sedd_minhash(FAKE, FAKE, u64(1 << 31), 5, 8, u64(0), 0, FAKE, None) == -1
    assert L.sedd_minhash(None, None, u64(0), 5, 8, u64(0), 0, None, None) == 0


@pytest.mark.parametrize("K,b,r", [(128, 0, 8), (128, 16, 0), (128, 17, 8), (0, 1, 1), (64, 65, 1)])
def test_lsh_keys_rejects_bad_shapes(K, b, r):
    L = sedd.lib()
    assert L.sedd_lsh_keys(FAKE, u64(4), K, b, r, FAKE, None) == -1


def test_lsh_keys_and_cluster_null_and_empty():
    L = sedd.lib()
    assert L.sedd_lsh_keys(None, u64(4), 128, 16, 8, FAKE, None) == -1
    assert L.sedd_lsh_keys(FAKE, u64(4), 128, 16, 8, None, None) == -1
    assert L.sedd_lsh_keys(None, u64(0), 128, 16, 8, None, None) == 0
    assert L.sedd_cluster(None, u64(4), 16, FAKE, None) == -1
    assert L.sedd_cluster(FAKE, u64(4), 16, None, None) == -1
    assert L.sedd_cluster(FAKE, u64(4), 0, FAKE, None) == -1
    assert L.sedd_cluster(FAKE, u64(1 << 31), 1, FAKE, None) == -1
    assert L.sedd_cluster(FAKE, u64(1 << 30), 16, FAKE, None) == -1      # n_docs*b >= 2^32
    assert L.sedd_cluster(None, u64(0), 16, None, None) == 0


def test_binding_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        sedd.sedd_minhash(torch.zeros(4, dtype=torch.uint8), torch.zeros(2, dtype=torch.uint64), 5, 8)


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2501_01046_amd")
    for path in glob.glob(os.path.join(pkg, "**", "*"), recursive=True):
        if path.endswith((".py", ".hip", ".h", ".c")):
            text = open(path, errors="replace").read()
            assert "import oracle" not in text and "from oracle" not in text, path
            assert "sedd_oracle" not in text and "sedd_ref_" not in text, path


def test_verified_and_dense_calls_reject_bad_arguments_before_the_device():
    L = sedd.lib()
    L.sedd_cluster_verified.argtypes = [C.c_void_p, C.c_void_p, u64, C.c_int32, C.c_int32, C.c_int32,
                                        C.c_void_p, C.c_void_p]
    L.sedd_lsh_dense_keys.argtypes = [C.c_void_p, u64, C.c_int32, C.c_int32, C.c_int32, u64,
                                      C.c_void_p, C.c_void_p]
    assert L.sedd_cluster_verified(FAKE, FAKE, u64(4), 0, 16, 1, FAKE, None) == -1        # K < 1
    assert L.sedd_cluster_verified(FAKE, FAKE, u64(4), 128, 16, -1, FAKE, None) == -1     # min_match < 0
    assert L.sedd_cluster_verified(FAKE, None, u64(4), 128, 16, 103, FAKE, None) == -1    # no signatures
    assert L.sedd_cluster_verified(None, FAKE, u64(4), 128, 16, 103, FAKE, None) == -1
    assert L.sedd_cluster_verified(FAKE, FAKE, u64(4), 128, 0, 103, FAKE, None) == -1
    assert L.sedd_cluster_verified(None, None, u64(0), 128, 16, 103, None, None) == 0
    assert L.sedd_lsh_dense_keys(FAKE, u64(4), 128, 16, 8, u64(0), FAKE, None) == -1       # no buckets
    assert L.sedd_lsh_dense_keys(FAKE, u64(4), 128, 17, 8, u64(10), FAKE, None) == -1      # b*r > K
    assert L.sedd_lsh_dense_keys(FAKE, u64(4), 128, 16, 8, u64(1 << 61), FAKE, None) == -1
    assert L.sedd_lsh_dense_keys(None, u64(0), 128, 16, 8, u64(10), None, None) == 0


def test_misaligned_arrays_are_rejected_before_the_device():
    L = sedd.lib()
    L.sedd_cluster_verified.argtypes = [C.c_void_p, C.c_void_p, u64, C.c_int32, C.c_int32, C.c_int32,
                                        C.c_void_p, C.c_void_p]
    L.sedd_lsh_dense_keys.argtypes = [C.c_void_p, u64, C.c_int32, C.c_int32, C.c_int32, u64,
                                      C.c_void_p, C.c_void_p]
    odd4, odd8 = C.c_void_p(0x1002), C.c_void_p(0x1004)       # not multiples of 4 / of 8
    assert L.sedd_minhash(FAKE, odd8, u64(4), 5, 8, u64(0), 0, FAKE, None) == -1      # doc_offsets
    assert L.sedd_minhash(FAKE, FAKE, u64(4), 5, 8, u64(0), 0, odd4, None) == -1      # sig
    assert L.sedd_lsh_keys(odd4, u64(4), 128, 16, 8, FAKE, None) == -1
    assert L.sedd_lsh_keys(FAKE, u64(4), 128, 16, 8, odd8, None) == -1
    assert L.sedd_lsh_dense_keys(FAKE, u64(4), 128, 16, 8, u64(10), odd8, None) == -1
    assert L.sedd_cluster(odd8, u64(4), 16, FAKE, None) == -1
    assert L.sedd_cluster(FAKE, u64(4), 16, odd8, None) == -1
    assert L.sedd_cluster_verified(FAKE, odd4, u64(4), 128, 16, 103, FAKE, None) == -1
    assert L.sedd_cluster_verified(odd8, FAKE, u64(4), 128, 16, 103, FAKE, None) == -1


def test_threshold_and_bucket_count_helpers():
    assert sedd.min_match_for(0.8, 128) == 103 and sedd.min_match_for(0.8, 125) == 100
    assert sedd.min_match_for(0.7, 10) == 7 and sedd.min_match_for(0.0, 5) == 0
    assert sedd.dense_bucket_count(1_000_000) == 4000 and sedd.dense_bucket_count(0) == 1
    assert sedd.dense_bucket_count(40_000) == 800 and sedd.dense_bucket_count(10, k=1) == 3


def test_threshold_and_bucket_count_through_the_c_abi():
    """sedd_min_match (Section 3.3, Eq. 3) and sedd_dense_bucket_count (Section 3.2) called
    directly: integer arithmetic, hand values, big-integer cross-check, error returns."""
    import math
    import random
    L = sedd.lib()
    mm, nb = L.sedd_min_match, L.sedd_dense_bucket_count
    assert mm(u64(8), u64(10), 128) == 103          # 102.4 -> 103
    assert mm(u64(8), u64(10), 125) == 100          # exactly 100 stays 100
    assert mm(u64(4), u64(5), 125) == 100           # the same theta, other fraction
    assert mm(u64(1), u64(2), 3) == 2 and mm(u64(1), u64(1), 64) == 64 and mm(u64(0), u64(7), 64) == 0
    assert mm(u64(3), u64(2), 10) == 15             # theta > 1: above K, links nothing
    assert mm(u64(8), u64(0), 128) == -1 and mm(u64(8), u64(10), -1) == -1
    assert mm(u64((1 << 64) - 1), u64(1), 4096) == -1            # result beyond int32
    rng = random.Random(5)
    for _ in range(300):
        num, den, K = rng.randrange(0, 1 << 40), rng.randrange(1, 1 << 40), rng.randrange(0, 4097)
        want = -((-num * K) // den)
        assert mm(u64(num), u64(den), K) == (want if want < (1 << 31) else -1)
    assert nb(u64(1_000_000), 4) == 4000 and nb(u64(40_000), 4) == 800 and nb(u64(0), 4) == 1
    assert nb(u64(10), 1) == 3 and nb(u64(32_800_000), 2) == 11454 and nb(u64(5), 0) == 1
    for _ in range(300):
        n, k = rng.randrange(0, 1 << 63), rng.randrange(0, 1 << 32)
        assert nb(u64(n), k) == max(1, math.isqrt(k * k * n))


def test_scratch_cap_turns_into_enomem_before_the_device():
    """SEDD_ENOMEM return path, forced from the host: with a cap on the library's scratch, a call
    whose buffers exceed it fails before it touches the device; lifting the cap restores it."""
    L = sedd.lib()
    L.sedd_debug_set_scratch_cap.argtypes = [u64]
    assert L.sedd_debug_set_scratch_cap(u64(1)) == 0
    try:
        assert L.sedd_cluster(FAKE, u64(4), 16, FAKE, None) == -2
        assert b"allocation" in L.sedd_strerror(-2)
        assert b"cap" in L.sedd_last_device_error()
    finally:
        assert L.sedd_debug_set_scratch_cap(u64(0)) == 0


def test_workspace_size_and_argument_checks():
    L = sedd.lib()
    wb = L.sedd_cluster_workspace_bytes
    wb.restype, wb.argtypes = u64, [u64, C.c_int32, C.c_int32]
    plain, ver = wb(u64(100_000), 16, 0), wb(u64(100_000), 16, 128)
    # 24 bytes per (document, band) record dominate; the verified call adds sketches and group lists
    assert 24 * 1_600_000 < plain < 26 * 1_600_000
    assert ver > plain + 100_000 * 4 * 4
    assert wb(u64(0), 16, 0) > 0
    assert wb(u64(100), 0, 0) == 0 and wb(u64(100), 16, -1) == 0 and wb(u64(1 << 31), 1, 0) == 0
    assert wb(u64(65_536), 16, 0) <= (32 << 20) + 256       # what the static entry point promises
    L.sedd_cluster_ws.argtypes = [C.c_void_p, u64, C.c_int32, C.c_void_p, C.c_void_p, u64, C.c_void_p]
    L.sedd_cluster_verified_ws.argtypes = [C.c_void_p, C.c_void_p, u64, C.c_int32, C.c_int32, C.c_int32,
                                           C.c_void_p, C.c_void_p, u64, C.c_void_p]
    assert L.sedd_cluster_ws(FAKE, u64(4), 16, FAKE, None, u64(1 << 20), None) == -1       # no workspace
    assert L.sedd_cluster_ws(FAKE, u64(4), 16, FAKE, FAKE, u64(100), None) == -4           # too small
    assert L.sedd_cluster_ws(FAKE, u64(4), 0, FAKE, FAKE, u64(1 << 20), None) == -1
    assert L.sedd_cluster_ws(None, u64(0), 16, None, None, u64(0), None) == 0
    assert L.sedd_cluster_verified_ws(FAKE, FAKE, u64(4), 128, 16, 103, FAKE, FAKE, u64(100), None) == -4
    assert L.sedd_cluster_verified_ws(FAKE, None, u64(4), 128, 16, 103, FAKE, FAKE, u64(1 << 20), None) == -1


def test_loading_the_library_first_still_leaves_one_hip_runtime_in_the_process():
    """torch ships a HIP runtime of its own.  A process that loaded libsedd.so before torch held two
    runtimes (the system's for the library, torch's for the tensors) and the library's first
    allocation failed on the GPU.  The binding therefore imports torch before it loads the library:
    in a fresh interpreter that only asks for the library, every libamdhip64 mapped afterwards is
    one and the same file."""
    import subprocess
    import sys
    code = (
        "import paper_2501_01046_amd as s\n"
        "s.lib()\n"
        "import sys, os\n"
        "assert 'torch' in sys.modules\n"
        "paths = {os.path.realpath(l.split()[-1]) for l in open('/proc/self/maps')\n"
        "         if 'libamdhip64' in l}\n"
        "print(sorted(paths))\n"
        "assert len(paths) == 1, paths\n"
    )
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True,
                       timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
