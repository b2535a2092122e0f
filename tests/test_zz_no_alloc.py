"""The entry point that allocates nothing (sedd_cluster_static) against sedd_cluster.

Called through the C ABI with ctypes on raw device pointers: two calls in a row on the same
GPU, the second with a smaller input (the fixed scratch array keeps the first call's contents),
then inputs at and beyond the limit.  Cluster ids are integers with one correct value, so the
bar is exact equality with sedd_cluster's output, which the other GPU tests hold to the oracle.
"""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

u64 = C.c_uint64


def _keys(seed, n, b, span):
    rng = np.random.default_rng(seed)
    k = rng.integers(0, span, size=(n, b), dtype=np.uint64)
    if n > 3:
        k[n // 2:, 0] = k[: n - n // 2, 0]            # guaranteed duplicates in band 0
    return torch.from_numpy(k).cuda()


def _both(L, keys):
    """(static result, sedd_cluster result) as host arrays, via raw pointers."""
    n, b = keys.shape
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    a = torch.full((n,), -7, dtype=torch.int64, device="cuda")
    w = torch.full((n,), -9, dtype=torch.int64, device="cuda")
    rc = L.sedd_cluster_static(C.c_void_p(keys.data_ptr()), u64(n), b, C.c_void_p(a.data_ptr()), stream)
    assert rc == 0, rc
    rc = L.sedd_cluster(C.c_void_p(keys.data_ptr()), u64(n), b, C.c_void_p(w.data_ptr()), stream)
    assert rc == 0, rc
    torch.cuda.synchronize()
    return a.cpu().numpy(), w.cpu().numpy()


def test_static_entry_point_equals_sedd_cluster_on_two_calls_in_a_row():
    import paper_2501_01046_amd as sedd
    L = sedd.lib()
    L.sedd_cluster_static.argtypes = [C.c_void_p, u64, C.c_int32, C.c_void_p, C.c_void_p]
    L.sedd_cluster.argtypes = [C.c_void_p, u64, C.c_int32, C.c_void_p, C.c_void_p]
    print("static: 60000 x 16, then 3000 x 5", flush=True)
    big = _keys(1, 60_000, 16, 80_000)
    got, want = _both(L, big)
    assert np.array_equal(got, want)
    assert (want != np.arange(want.size)).sum() > 1000       # the case is not trivial
    small = _keys(2, 3_000, 5, 700)
    got, want = _both(L, small)
    assert np.array_equal(got, want)
    # a third call: keys that agree in their low bits (the whole-key sort inside the same scratch)
    print("static: keys d << 32", flush=True)
    d = torch.arange(50_000, dtype=torch.int64, device="cuda")
    odd = torch.stack([(d // 3) << 32, (d % 1000) << 35], dim=1).contiguous().view(torch.uint64)
    got, want = _both(L, odd)
    assert np.array_equal(got, want)
    assert sedd.debug_last_regroup() == 1
    # and the first input again: nothing of the calls in between may leak into the result
    got2, _ = _both(L, big)
    assert np.array_equal(got2, _both(L, big)[1])


def test_static_entry_point_limit_and_arguments():
    import paper_2501_01046_amd as sedd
    L = sedd.lib()
    L.sedd_cluster_static.argtypes = [C.c_void_p, u64, C.c_int32, C.c_void_p, C.c_void_p]
    L.sedd_cluster.argtypes = [C.c_void_p, u64, C.c_int32, C.c_void_p, C.c_void_p]
    print("static: at the documented limit (65536 x 16)", flush=True)
    edge = _keys(3, 65_536, 16, 1 << 61)
    got, want = _both(L, edge)
    assert np.array_equal(got, want)
    print("static: beyond the limit", flush=True)
    n, b = 200_000, 16
    keys = _keys(4, n, b, 1 << 61)
    out = torch.full((n,), -7, dtype=torch.int64, device="cuda")
    before = sedd.sedd_scratch_bytes()
    rc = L.sedd_cluster_static(C.c_void_p(keys.data_ptr()), u64(n), b, C.c_void_p(out.data_ptr()), None)
    assert rc == -4 and b"limit" in L.sedd_strerror(rc)
    torch.cuda.synchronize()
    assert bool((out == -7).all())                            # nothing was enqueued
    assert sedd.sedd_scratch_bytes() == before                # the arena was not touched
    assert L.sedd_cluster_static(None, u64(0), 16, None, None) == 0
    assert L.sedd_cluster_static(None, u64(4), 16, C.c_void_p(out.data_ptr()), None) == -1
    # the binding's wrapper raises the same code
    with pytest.raises(sedd.SeddError) as e:
        sedd.sedd_cluster_static(keys, out)
    assert e.value.code == -4


def test_static_entry_point_under_graph_capture():
    """The callers the entry point is for: sedd_lsh_keys + sedd_cluster_static captured into one
    HIP graph and replayed on new inputs written into the same buffers, with eager work and
    synchronisation between the replays; every replay against sedd_cluster run eagerly."""
    import paper_2501_01046_amd as sedd
    sedd.lib()
    n, K, b, r = 40_000, 64, 8, 8
    rng = np.random.default_rng(21)

    def signatures(seed):
        g = np.random.default_rng(seed)
        proto = g.integers(0, 1 << 32, size=(n // 3, K), dtype=np.uint64).astype(np.uint32)
        return torch.from_numpy(proto[g.integers(0, n // 3, size=n)].copy()).cuda()
    sig = signatures(0)
    keys = torch.empty((n, b), dtype=torch.uint64, device="cuda")
    cid = torch.empty((n,), dtype=torch.int64, device="cuda")
    # first call outside the capture: the one symbol look-up per device happens here
    sedd.sedd_lsh_keys(sig, b, r, out=keys)
    sedd.sedd_cluster_static(keys, cid)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sedd.sedd_lsh_keys(sig, b, r, out=keys)
        sedd.sedd_cluster_static(keys, cid)
    for seed in (1, 2, 3, 4):
        print("static: graph replay", seed, flush=True)
        sig.copy_(signatures(seed))
        graph.replay()
        torch.cuda.synchronize()
        got = cid.cpu().numpy().copy()
        want = sedd.sedd_cluster(sedd.sedd_lsh_keys(sig, b, r)).cpu().numpy()     # eager, arena scratch
        assert np.array_equal(got, want), seed
        assert (want != np.arange(n)).sum() > n // 2
