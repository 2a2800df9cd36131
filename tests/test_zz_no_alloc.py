"""The entry point for callers that cannot allocate (ob_sort_pairs_noalloc), called through the C
ABI on device arrays and checked against the existing sort entry point (ob_test_sort) and against
NumPy's stable sort: bit-exact, two calls in a row, the second with a smaller input, so that
whatever the first call left in the library's built-in scratch array must not matter."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _case(rng, n, lo_bit, n_bits):
    keys = rng.integers(0, 1 << 62, size=n, dtype=np.uint64)
    keys[rng.integers(0, n, size=n // 3)] = keys[0]            # many equal keys: stability matters
    vals = rng.permutation(n).astype(np.uint32)
    return keys, vals, lo_bit, n_bits


def _noalloc(torch, ob, keys, vals, lo_bit, n_bits):
    kd = torch.from_numpy(keys.view(np.int64).copy()).cuda()
    vd = torch.from_numpy(vals.view(np.int32).copy()).cuda()
    s = torch.cuda.current_stream()
    ob.sort_pairs_noalloc(s.cuda_stream, keys.shape[0], kd.data_ptr(), vd.data_ptr(), lo_bit, n_bits)
    s.synchronize()
    return kd.cpu().numpy().view(np.uint64), vd.cpu().numpy().view(np.uint32)


def test_sort_without_allocation_matches_the_sort_entry_point():
    import torch
    from paper_1705_07860_amd import binding as ob
    rng = np.random.default_rng(20171107)
    c = ob.Context(arena_bytes=64 << 20)
    # 200 003 pairs: 196 blocks of 1024 and a ragged tail, three 8-bit passes (odd: the result is copied
    # back from the second buffers); then 5 001 pairs on two passes through the one-workgroup path;
    # then sizes around the block and the path boundaries
    for n, lo_bit, n_bits in [(200003, 0, 20), (5001, 16, 13), (8193, 32, 9), (1, 0, 8), (1025, 3, 64 - 3)]:
        keys, vals, lo, nb = _case(rng, n, lo_bit, n_bits)
        got_k, got_v = _noalloc(torch, ob, keys, vals, lo, nb)
        ref_k, ref_v = c.test_sort(keys, vals, lo, nb)          # the existing entry point (arena scratch)
        assert np.array_equal(got_k, ref_k) and np.array_equal(got_v, ref_v), (n, lo, nb)
        digit = (keys >> np.uint64(lo)) & np.uint64((1 << nb) - 1 if nb < 64 else 0xffffffffffffffff)
        order = np.argsort(digit, kind="stable")
        assert np.array_equal(got_k, keys[order]) and np.array_equal(got_v, vals[order]), (n, lo, nb)
    c.close()


def test_sort_without_allocation_rejects_what_does_not_fit():
    import torch
    from paper_1705_07860_amd import binding as ob
    kd = torch.zeros(8, dtype=torch.int64, device="cuda")
    vd = torch.zeros(8, dtype=torch.int32, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    with pytest.raises(ob.ObError) as e:
        ob.sort_pairs_noalloc(s, ob.OB_NOALLOC_MAX_PAIRS + 1, kd.data_ptr(), vd.data_ptr(), 0, 8)
    assert e.value.code == -3 and "at most" in str(e.value)
    with pytest.raises(ob.ObError) as e:
        ob.sort_pairs_noalloc(s, 8, kd.data_ptr(), vd.data_ptr(), 60, 8)
    assert e.value.code == -8
    with pytest.raises(ob.ObError) as e:
        ob.sort_pairs_noalloc(s, 8, 0, vd.data_ptr(), 0, 8)
    assert e.value.code == -8
    ob.sort_pairs_noalloc(s, 0, 0, 0, 0, 8)                      # nothing to do is not an error
    # the largest size that fits
    n = ob.OB_NOALLOC_MAX_PAIRS
    rng = np.random.default_rng(3)
    keys = rng.integers(0, 1 << 40, size=n, dtype=np.uint64)
    vals = np.arange(n, dtype=np.uint32)
    got_k, got_v = _noalloc(torch, ob, keys, vals, 0, 40)
    order = np.argsort(keys, kind="stable")
    assert np.array_equal(got_k, keys[order]) and np.array_equal(got_v, vals[order])
