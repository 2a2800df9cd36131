"""GPU checks of the library's device primitives against NumPy: exclusive scan, stable radix
sort (bit-exact), and the MFMA tile routine (the lane layout of the matrix instruction)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_1705_07860_amd import binding as ob
    c = ob.Context(arena_bytes=256 << 20)
    yield c
    c.close()


@pytest.mark.parametrize("n", [0, 1, 255, 1024, 1025, 4095, 4096, 4097, 5000, 300001])
def test_scan(ctx, n):
    rng = np.random.default_rng(n)
    a = rng.integers(0, 1000, size=n).astype(np.uint32)
    out, tot = ctx.test_scan(a)
    ref = np.concatenate([[0], np.cumsum(a.astype(np.uint64))[:-1]]).astype(np.uint32) if n else a
    assert np.array_equal(out, ref)
    assert tot == int(a.sum())


@pytest.mark.parametrize("n,lo,bits", [(1, 0, 8), (2, 0, 1), (64, 0, 8), (1000, 0, 18), (1023, 5, 26), (1025, 32, 10),
                                       (4097, 0, 5), (4097, 0, 26), (8192, 0, 24), (8192, 7, 17), (8193, 0, 9),
                                       (240000, 0, 18), (240000, 32, 18), (196608, 0, 12), (196609, 3, 12), (80000, 0, 17),
                                       (262144, 0, 9), (262145, 0, 16), (700001, 4, 12)])
def test_radix_sort_is_stable_and_exact(ctx, n, lo, bits):
    rng = np.random.default_rng(n + lo)
    keys = rng.integers(0, 1 << 62, size=n, dtype=np.uint64)
    keys[::3] = keys[0]                      # many duplicates to exercise stability
    vals = np.arange(n, dtype=np.uint32)
    ko, vo = ctx.test_sort(keys, vals, lo, bits)
    field = (keys >> np.uint64(lo)) & np.uint64((1 << bits) - 1)
    order = np.argsort(field, kind="stable")
    assert np.array_equal(vo, vals[order])
    assert np.array_equal(ko, keys[order])


def test_two_field_sort_matches_lexicographic_order(ctx):
    # sort by the low field, then by the field at bit 32: the schedule's (depth, representative) key
    rng = np.random.default_rng(7)
    n = 50000
    lo = rng.integers(0, 1 << 16, size=n, dtype=np.uint64)
    hi = rng.integers(0, 600, size=n, dtype=np.uint64)
    keys = (hi << np.uint64(32)) | lo
    vals = np.arange(n, dtype=np.uint32)
    k1, v1 = ctx.test_sort(keys, vals, 0, 16)
    k2, v2 = ctx.test_sort(k1, v1, 32, 16)
    order = np.lexsort((vals, lo, hi))
    assert np.array_equal(v2, vals[order])


@pytest.mark.parametrize("M,N,K", [(32, 32, 8), (64, 1024, 256), (1, 5, 256), (33, 50, 512), (70, 35, 7),
                                   (3, 3, 1), (128, 96, 36)])
def test_mfma_tile_gemm(ctx, M, N, K):
    rng = np.random.default_rng(M * 1000 + N + K)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((N, K)).astype(np.float32)
    C = ctx.test_gemm(A, B)
    ref = A.astype(np.float64) @ B.astype(np.float64).T
    err = np.max(np.abs(C - ref)) / max(np.max(np.abs(ref)), 1e-30)
    assert err < 1e-5, err
