"""Host-side frequency reordering (VQ-LLM Sec. V-B): the weight must not change, the hot entries must lead.

The check of "the weight does not change" goes through the CPU oracle's dequantization, which shares no code
with the library.
"""
import ctypes

import numpy as np
import pytest

import oracle
import paper_2503_02236_amd as vq
from paper_2503_02236_amd import workloads as wl
from paper_2503_02236_amd.binding import vq_weight_t


@pytest.mark.parametrize("N,K,v,bits,R,E,zipf", [
    (64, 256, 8, 16, 1, 65536, 1.0),     # big codebook, skewed
    (64, 256, 8, 16, 1, 4096, None),     # uniform
    (48, 128, 4, 8, 2, 256, 1.2),        # two residual codebooks, each reordered on its own
    (16, 64, 8, 8, 4, 200, 0.8),         # E not a power of two
])
def test_reorder_keeps_the_weight_and_sorts_by_use(N, K, v, bits, R, E, zipf):
    w = wl.shuffle_entries(wl.make_weight(N, K, v, bits, R, E, 0.02, seed=400 + N + R, zipf_s=zipf), seed=5)
    r = vq.vq_reorder_by_frequency(w)
    before = oracle.dequant(w.codes, w.codebooks)
    after = oracle.dequant(r.codes, r.codebooks)
    assert before.tobytes() == after.tobytes()                       # bit-identical fp32 tiles
    for k in range(R):
        counts = np.bincount(r.codes[..., k].ravel().astype(np.int64), minlength=E)
        assert (np.diff(counts) <= 0).all()                          # most used first
        # same multiset of entries, as bit patterns
        assert sorted(map(bytes, w.codebooks[k].view(np.uint16))) == sorted(map(bytes, r.codebooks[k].view(np.uint16)))
        # hot_entries: the shortest prefix that serves half of the codes (maximum over the codebooks)
        assert 2 * counts[:r.hot_entries].sum() >= counts.sum()
    per_cb = []
    for k in range(R):
        counts = np.bincount(r.codes[..., k].ravel().astype(np.int64), minlength=E)
        per_cb.append(int(np.searchsorted(2 * np.cumsum(counts), counts.sum()) + 1))
    assert r.hot_entries == max(per_cb)
    again = vq.vq_reorder_by_frequency(r)                            # already sorted: a fixed point
    assert np.array_equal(again.codes, r.codes) and again.codebooks.tobytes() == r.codebooks.tobytes()


def test_reorder_packed_12bit_codes():
    """VQ<8,12,2> (Tbl. III): the packed 12-bit string is unpacked, reordered and packed again."""
    w = wl.shuffle_entries(wl.make_weight(24, 256, 8, 12, 2, 4096, 0.01, seed=812, zipf_s=1.0), seed=9)
    shape = (w.N, w.K // w.v, 2)
    r = vq.vq_reorder_by_frequency(w)
    assert r.codes.dtype == np.uint8 and r.codes.size == w.codes.size          # same packed size, no over-read
    before = oracle.dequant(oracle.Packed12(w.codes, shape), w.codebooks)
    after = oracle.dequant(oracle.Packed12(r.codes, shape), r.codebooks)
    assert before.tobytes() == after.tobytes()
    un = oracle.unpack12(r.codes, int(np.prod(shape))).reshape(shape)
    for k in range(2):
        counts = np.bincount(un[..., k].ravel().astype(np.int64), minlength=4096)
        assert (np.diff(counts) <= 0).all()
        assert 2 * counts[:r.hot_entries].sum() >= counts.sum()
    # a code beyond n_entries in the packed string is rejected (n_entries below 2^12)
    lib = vq.lib()
    codes = np.ascontiguousarray(w.codes)
    cb = np.ascontiguousarray(w.codebooks[:, :1000])
    d = vq_weight_t(w.N, w.K, 8, 12, 2, 1000, codes.ctypes.data, cb.ctypes.data, None, None)
    out_c, out_cb = np.empty_like(codes), np.empty_like(cb)
    assert lib.vq_reorder_by_frequency(ctypes.byref(d), out_c.ctypes.data, out_cb.ctypes.data, None) == -2


def test_reorder_argument_validation():
    lib = vq.lib()
    w = wl.make_weight(8, 64, 8, 8, 1, 16, 0.02, seed=1)
    codes = np.ascontiguousarray(w.codes)
    cb = np.ascontiguousarray(w.codebooks)
    out_c, out_cb = np.empty_like(codes), np.empty_like(cb)
    d = vq_weight_t(8, 64, 8, 8, 1, 16, codes.ctypes.data, cb.ctypes.data, None, None)
    f = lib.vq_reorder_by_frequency
    assert f(None, out_c.ctypes.data, out_cb.ctypes.data, None) == -1
    assert f(ctypes.byref(d), None, out_cb.ctypes.data, None) == -1
    assert f(ctypes.byref(d), out_c.ctypes.data, cb.ctypes.data, None) == -2      # codebooks cannot be reordered in place
    assert f(ctypes.byref(d), codes.ctypes.data, out_cb.ctypes.data, None) == 0    # codes can
    bad = codes.copy()
    bad[0, 0, 0] = 16                                                        # code >= n_entries
    d2 = vq_weight_t(8, 64, 8, 8, 1, 16, bad.ctypes.data, cb.ctypes.data, None, None)
    assert f(ctypes.byref(d2), out_c.ctypes.data, out_cb.ctypes.data, None) == -2
    d3 = vq_weight_t(8, 60, 8, 8, 1, 16, codes.ctypes.data, cb.ctypes.data, None, None)
    assert f(ctypes.byref(d3), out_c.ctypes.data, out_cb.ctypes.data, None) == -2  # K % v
