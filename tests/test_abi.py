"""Host-side checks of the C ABI (no GPU): the library loads, exports every declared symbol,
and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2503_02236_amd as vq
from paper_2503_02236_amd.binding import SYMBOLS, vq_kv_t, vq_weight_t

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "vq_mi355x.h")

VQ_ERR_NULL, VQ_ERR_SHAPE, VQ_ERR_UNSUPPORTED, VQ_ERR_ALIGN, VQ_ERR_WORKSPACE = -1, -2, -3, -4, -5
P = 0x10000  # a 16-byte aligned fake device address; never dereferenced on the error paths


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vq_[a-z_]+)\s*\(", text)))


def test_header_declares_and_library_exports_the_same_symbols():
    names = declared_functions()
    assert {"vq_gemv", "vq_gemm", "vq_attn_decode", "vq_dequant", "vq_kv_dequant"} <= set(names)
    lib = vq.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(SYMBOLS) == names       # the binding wraps exactly what the header declares


def test_status_strings():
    assert vq.status_str(0) == "VQ_OK"
    for s in range(-6, 0):
        assert vq.status_str(s).startswith("VQ_ERR_")
    assert "unknown" in vq.status_str(-99)
    assert vq.lib().vq_version() >= 100


def weight(**kw):
    d = dict(N=64, K=64, v=8, code_bits=8, n_codebooks=1, n_entries=256, codes=P, codebooks=P, scale=None,
             gemv_pack=None)
    d.update(kw)
    return vq_weight_t(**d)


def kvdesc(**kw):
    d = dict(B=1, H=1, D=128, T=16, v=4, n_entries=256, cb_groups=1, k_codes=P, v_codes=P, k_codebooks=P,
             v_codebooks=P, seq_lens=None)
    d.update(kw)
    return vq_kv_t(**d)


def gemv(w, x=P, bs=1, y=P, ws=None, ws_bytes=0):
    return vq.lib().vq_gemv(ctypes.byref(w), x, bs, y, ws, ws_bytes, None)


def gemm(w, x=P, M=1, y=P):
    return vq.lib().vq_gemm(ctypes.byref(w), x, M, y, None, 0, None)


@pytest.mark.parametrize("w,want", [
    (weight(codes=None), VQ_ERR_NULL),
    (weight(codebooks=None), VQ_ERR_NULL),
    (weight(v=3), VQ_ERR_UNSUPPORTED),
    (weight(v=16), VQ_ERR_UNSUPPORTED),
    (weight(code_bits=10), VQ_ERR_UNSUPPORTED),
    (weight(n_codebooks=0), VQ_ERR_UNSUPPORTED),
    (weight(n_codebooks=5), VQ_ERR_UNSUPPORTED),
    (weight(n_entries=257), VQ_ERR_UNSUPPORTED),
    (weight(n_entries=0), VQ_ERR_UNSUPPORTED),
    (weight(K=60), VQ_ERR_SHAPE),
    (weight(N=-1), VQ_ERR_SHAPE),
    (weight(codes=P + 8), VQ_ERR_ALIGN),
    (weight(codebooks=P + 2), VQ_ERR_ALIGN),
    (weight(scale=P + 4), VQ_ERR_ALIGN),
])
def test_weight_descriptor_validation(w, want):
    assert gemv(w) == want
    assert gemm(w) == want
    assert vq.lib().vq_dequant(ctypes.byref(w), P, 1, None) == want
    assert vq.lib().vq_gemv_workspace(ctypes.byref(w), 1) == 0


def test_gemv_gemm_argument_validation():
    w = weight()
    assert vq.lib().vq_gemv(None, P, 1, P, None, 0, None) == VQ_ERR_NULL
    assert gemv(w, x=None) == VQ_ERR_NULL
    assert gemv(w, y=None) == VQ_ERR_NULL
    assert gemv(w, bs=0) == VQ_ERR_SHAPE
    assert gemv(w, bs=17) == VQ_ERR_SHAPE
    assert gemv(w, x=P + 2) == VQ_ERR_ALIGN
    assert gemv(w, y=P + 6) == VQ_ERR_ALIGN
    assert gemm(w, M=0) == VQ_ERR_SHAPE
    assert gemm(w, x=None) == VQ_ERR_NULL
    assert gemm(w, y=P + 2) == VQ_ERR_ALIGN
    assert vq.lib().vq_dequant(ctypes.byref(w), None, 1, None) == VQ_ERR_NULL
    # N == 0 is a valid empty problem: success without a launch
    assert gemv(weight(N=0)) == 0
    assert gemm(weight(N=0)) == 0


@pytest.mark.parametrize("kv,want", [
    (kvdesc(k_codes=None), VQ_ERR_NULL),
    (kvdesc(v_codebooks=None), VQ_ERR_NULL),
    (kvdesc(v=3), VQ_ERR_UNSUPPORTED),
    (kvdesc(n_entries=512), VQ_ERR_UNSUPPORTED),
    (kvdesc(D=126), VQ_ERR_SHAPE),
    (kvdesc(cb_groups=3), VQ_ERR_SHAPE),
    (kvdesc(cb_groups=0), VQ_ERR_SHAPE),
    (kvdesc(T=-1), VQ_ERR_SHAPE),
    (kvdesc(k_codes=P + 1), VQ_ERR_ALIGN),
    (kvdesc(seq_lens=P + 2), VQ_ERR_ALIGN),
])
def test_kv_descriptor_validation(kv, want):
    lib = vq.lib()
    assert lib.vq_attn_decode(ctypes.byref(kv), P, 0.1, P, None, 0, None) == want
    assert lib.vq_kv_dequant(ctypes.byref(kv), 0, P, None) == want
    assert lib.vq_attn_decode_workspace(ctypes.byref(kv)) == 0


def test_attention_argument_validation():
    lib = vq.lib()
    kv = kvdesc()
    assert lib.vq_attn_decode(ctypes.byref(kv), None, 0.1, P, None, 0, None) == VQ_ERR_NULL
    assert lib.vq_attn_decode(ctypes.byref(kv), P, 0.1, P + 8, None, 0, None) == VQ_ERR_ALIGN
    assert lib.vq_kv_dequant(ctypes.byref(kv), 2, P, None) == VQ_ERR_SHAPE
    big = kvdesc(T=100000, B=2, H=2)
    need = lib.vq_attn_decode_workspace(ctypes.byref(big))
    assert need > 0                                    # long caches are split and need partials
    assert lib.vq_attn_decode(ctypes.byref(big), P, 0.1, P, None, 0, None) == VQ_ERR_WORKSPACE
    assert lib.vq_attn_decode(ctypes.byref(big), P, 0.1, P, P, need - 1, None) == VQ_ERR_WORKSPACE
    assert lib.vq_attn_decode(ctypes.byref(kvdesc(B=0)), P, 0.1, P, None, 0, None) == 0


def test_attention_channel_parallel_argument_validation():
    lib = vq.lib()
    f, wsq = lib.vq_attn_decode_channel_parallel, lib.vq_attn_decode_channel_parallel_workspace
    cq = kvdesc(cb_groups=32)                            # D = 128, v = 4: 4 channel groups of 8 codebooks
    need = wsq(ctypes.byref(cq))
    assert need == cq.B * cq.H * (128 // 32 + 1) * cq.T * 4
    assert f(ctypes.byref(cq), None, 0.1, P, P, need, None) == VQ_ERR_NULL
    assert f(ctypes.byref(cq), P, 0.1, P + 8, P, need, None) == VQ_ERR_ALIGN
    assert f(ctypes.byref(cq), P, 0.1, P, None, 0, None) == VQ_ERR_WORKSPACE
    assert f(ctypes.byref(cq), P, 0.1, P, P, need - 1, None) == VQ_ERR_WORKSPACE
    assert f(ctypes.byref(cq), P, 0.1, P, P + 4, need, None) == VQ_ERR_ALIGN
    one = kvdesc()                                       # one codebook per head: does not divide over 4 channel groups
    assert wsq(ctypes.byref(one)) == 0
    assert f(ctypes.byref(one), P, 0.1, P, P, 1 << 30, None) == VQ_ERR_UNSUPPORTED
    assert f(ctypes.byref(kvdesc(cb_groups=32, B=0)), P, 0.1, P, None, 0, None) == 0


def test_kv_quantize_argument_validation():
    lib = vq.lib()
    kv = kvdesc()
    f = lib.vq_kv_quantize
    assert f(ctypes.byref(kv), None, P, 1, 0, None) == VQ_ERR_NULL
    assert f(ctypes.byref(kv), P, P + 2, 1, 0, None) == VQ_ERR_ALIGN
    assert f(ctypes.byref(kv), P, P, -1, 0, None) == VQ_ERR_SHAPE
    assert f(ctypes.byref(kv), P, P, 1, -1, None) == VQ_ERR_SHAPE
    assert f(ctypes.byref(kv), P, P, 2, kv.T - 1, None) == VQ_ERR_SHAPE     # runs past the end of the cache
    assert f(ctypes.byref(kv), P, P, 0, 0, None) == 0                       # nothing to do
    assert f(ctypes.byref(kvdesc(v=3)), P, P, 1, 0, None) == VQ_ERR_UNSUPPORTED


def test_packed_gemv_validation():
    import numpy as np
    from paper_2503_02236_amd import workloads as wl
    from paper_2503_02236_amd.binding import vq_gemv_pack_t
    lib = vq.lib()
    w = wl.make_weight(128, 512, 8, 16, 1, 65536, 0.02, seed=9)
    buf, pack = vq.vq_gemv_prepack(w)
    d = weight(N=128, K=512, code_bits=16, n_entries=65536, codes=None)
    assert gemv(d) == VQ_ERR_NULL                                  # neither codes nor a pack
    pack.data = P                                                  # pretend it was uploaded
    d.gemv_pack = ctypes.pointer(pack)
    need = lib.vq_gemv_workspace(ctypes.byref(d), 1)
    assert need == pack.S * 128 * 4 + 4096      # S x N partial sums in blocks of 64 rows, plus one 4 KiB fetch unit
    assert gemv(d) == VQ_ERR_WORKSPACE
    assert gemv(d, ws=P, ws_bytes=need - 1) == VQ_ERR_WORKSPACE
    assert gemv(d, bs=2) == VQ_ERR_NULL                            # bs > 1 needs the canonical codes
    other = weight(N=256, K=512, code_bits=16, n_entries=65536, codes=None)
    other.gemv_pack = ctypes.pointer(pack)
    assert gemv(other, ws=P, ws_bytes=1 << 30) == VQ_ERR_SHAPE     # pack built for another shape
    pack.data = P + 4
    assert gemv(d, ws=P, ws_bytes=need) == VQ_ERR_ALIGN
    # the packer itself
    out = np.empty(buf.size + 16, dtype=np.uint8)
    hd = vq_weight_t(128, 512, 8, 16, 1, 65536, w.codes.ctypes.data, None, None, None)
    pk = vq_gemv_pack_t()
    assert lib.vq_gemv_prepack(ctypes.byref(hd), None, buf.size, ctypes.byref(pk)) == VQ_ERR_NULL
    aligned = out.ctypes.data + (-out.ctypes.data) % 16
    assert lib.vq_gemv_prepack(ctypes.byref(hd), aligned, buf.size - 1, ctypes.byref(pk)) == VQ_ERR_WORKSPACE
    assert lib.vq_gemv_prepack(ctypes.byref(hd), aligned + 1, buf.size, ctypes.byref(pk)) == VQ_ERR_ALIGN
    hd.v = 4
    assert lib.vq_gemv_prepack(ctypes.byref(hd), aligned, buf.size, ctypes.byref(pk)) == VQ_ERR_UNSUPPORTED
    assert lib.vq_gemv_prepack_bytes(ctypes.byref(hd)) == 0


def test_per_tile_codebook_descriptor_validation():
    assert gemv(weight(K=256, cb_tile_n=32, cb_tile_k=0)) == VQ_ERR_SHAPE    # both or neither
    assert gemv(weight(K=256, cb_tile_n=24, cb_tile_k=64)) == VQ_ERR_SHAPE   # rows per tile: multiple of 16
    assert gemv(weight(K=256, cb_tile_n=32, cb_tile_k=32)) == VQ_ERR_SHAPE   # columns per tile: multiple of 64
    assert gemv(weight(K=320, cb_tile_n=32, cb_tile_k=128)) == VQ_ERR_SHAPE  # K not a whole number of tiles
    assert gemv(weight(K=64 * 600, cb_tile_n=32, cb_tile_k=64)) == VQ_ERR_UNSUPPORTED  # 600 sets of 4 KiB > LDS


def test_packed_12_bit_descriptor_validation():
    ok = dict(code_bits=12, n_entries=4096, n_codebooks=2, K=256)          # 32 positions x 2 = 64 codes per row
    assert gemv(weight(**ok), x=None) == VQ_ERR_NULL                        # descriptor accepted, x missing
    assert gemv(weight(**dict(ok, n_entries=4097))) == VQ_ERR_UNSUPPORTED   # more entries than 12 bits address
    assert gemv(weight(**dict(ok, K=40))) == VQ_ERR_SHAPE                   # 5 x 2 = 10 codes: not whole 12-byte words
    assert gemv(weight(**dict(ok, n_codebooks=4))) == VQ_ERR_UNSUPPORTED    # 256 KiB of codebooks do not fit LDS
    assert gemv(weight(**dict(ok, n_codebooks=3, K=512))) == VQ_ERR_UNSUPPORTED
    assert gemv(weight(**dict(ok, cb_tile_n=32, cb_tile_k=64))) == VQ_ERR_UNSUPPORTED
    assert gemv(weight(code_bits=10)) == VQ_ERR_UNSUPPORTED


def test_gemv_batch_validation():
    lib = vq.lib()
    WP = ctypes.POINTER(vq_weight_t)
    d = weight()
    def batch(ws_list, xs, ys, count=None, ws=None, ws_bytes=0):
        n = len(ws_list)
        wa = (WP * n)(*[ctypes.pointer(w) if w is not None else WP() for w in ws_list])
        xa = (ctypes.c_void_p * n)(*xs)
        ya = (ctypes.c_void_p * n)(*ys)
        return lib.vq_gemv_batch(wa, xa, ya, n if count is None else count, ws, ws_bytes, None)
    assert lib.vq_gemv_batch(None, None, None, 1, None, 0, None) == VQ_ERR_NULL
    assert batch([d], [P], [P], count=0) == VQ_ERR_SHAPE
    assert batch([d] * 5, [P] * 5, [P] * 5) == VQ_ERR_SHAPE             # more than VQ_GEMV_BATCH_MAX
    assert batch([d, None], [P, P], [P, P]) == VQ_ERR_NULL
    assert batch([d, d], [P, None], [P, P]) == VQ_ERR_NULL
    assert batch([d, d], [P, P], [P, P + 2]) == VQ_ERR_ALIGN
    assert batch([d, weight(K=100)], [P, P], [P, P]) == VQ_ERR_SHAPE    # every member is validated
    wa = (WP * 2)(ctypes.pointer(d), ctypes.pointer(d))
    assert lib.vq_gemv_batch_workspace(wa, 2) == 0                      # canonical codes, LDS codebook: no scratch
    assert lib.vq_gemv_batch_workspace(wa, 9) == 0
    assert batch([weight(N=0)], [P], [P]) == 0                          # nothing to do, nothing launched


def test_gemv_sequence_validation():
    """Host-side checks of vq_gemv_sequence: every call and member is validated before anything is launched."""
    import numpy as np
    from paper_2503_02236_amd import workloads as wl
    from paper_2503_02236_amd.binding import vq_gemv_call_t
    lib = vq.lib()
    WP = ctypes.POINTER(vq_weight_t)
    w = wl.make_weight(128, 512, 8, 16, 1, 65536, 0.02, seed=5)
    buf, pack = vq.vq_gemv_prepack(w)
    pack.data = P                                            # a (fake) aligned device address: nothing is launched here
    packed = vq_weight_t(w.N, w.K, 8, 16, 1, 65536, None, P, None, ctypes.pointer(pack))
    canonical = weight()

    def call(ws_list, xs, ys, count=None):
        n = len(ws_list)
        c = vq_gemv_call_t()
        c._keep = ((WP * n)(*[ctypes.pointer(x) if x is not None else WP() for x in ws_list]),
                   (ctypes.c_void_p * n)(*xs), (ctypes.c_void_p * n)(*ys))
        c.w, c.x, c.y = (ctypes.cast(c._keep[0], ctypes.POINTER(WP)), ctypes.cast(c._keep[1], ctypes.POINTER(ctypes.c_void_p)),
                         ctypes.cast(c._keep[2], ctypes.POINTER(ctypes.c_void_p)))
        c.count = n if count is None else count
        return c

    def seq(calls, ws=P, ws_bytes=1 << 30):
        arr = (vq_gemv_call_t * len(calls))(*calls)
        return lib.vq_gemv_sequence(arr, len(calls), ws, ws_bytes, None), lib.vq_gemv_sequence_workspace(arr, len(calls))

    good = call([packed, packed], [P, P], [P, P])
    assert lib.vq_gemv_sequence(None, 1, P, 1 << 30, None) == VQ_ERR_NULL
    arr = (vq_gemv_call_t * 1)(good)
    assert lib.vq_gemv_sequence(arr, 0, P, 1 << 30, None) == VQ_ERR_SHAPE
    need = lib.vq_gemv_sequence_workspace(arr, 1)
    assert need == 2 * (2 * (32 * 128 * 4 + 4096))            # two halves, each the two problems' 32 x 128 partial sums (+ 4 KiB each)
    assert seq([good], ws=None)[0] == VQ_ERR_WORKSPACE
    assert seq([good], ws_bytes=need - 1)[0] == VQ_ERR_WORKSPACE
    assert seq([good], ws=P + 4)[0] == VQ_ERR_ALIGN
    assert seq([good, call([canonical], [P], [P])]) == (VQ_ERR_UNSUPPORTED, 0)     # a member without re-tiled codes
    assert seq([call([packed], [P], [P], count=0)]) == (VQ_ERR_SHAPE, 0)
    assert seq([call([packed] * 5, [P] * 5, [P] * 5)]) == (VQ_ERR_SHAPE, 0)
    assert seq([good, call([packed, None], [P, P], [P, P])]) == (VQ_ERR_NULL, 0)
    assert seq([call([packed], [None], [P])]) == (VQ_ERR_NULL, 0)
    assert seq([call([packed], [P], [P + 2])]) == (VQ_ERR_ALIGN, 0)
    # several streams: the struct is validated before any event or stream is touched
    from paper_2503_02236_amd.binding import vq_side_streams_t
    side = vq_side_streams_t()
    f = lib.vq_gemv_sequence_streams
    assert lib.vq_gemv_sequence_streams_workspace(arr, 1, 1) == need
    assert lib.vq_gemv_sequence_streams_workspace(arr, 1, 0) == 0 and lib.vq_gemv_sequence_streams_workspace(arr, 1, 9) == 0
    two = (vq_gemv_call_t * 2)(good, good)
    assert lib.vq_gemv_sequence_streams_workspace(two, 2, 2) == 2 * need          # one run per stream, two halves each
    assert lib.vq_gemv_sequence_streams_workspace(two, 2, 4) == 2 * need          # runs without calls need nothing
    side.n = 8
    assert f(arr, 1, P, 1 << 30, None, ctypes.byref(side)) == VQ_ERR_SHAPE
    side.n = -1
    assert f(arr, 1, P, 1 << 30, None, ctypes.byref(side)) == VQ_ERR_SHAPE
    side.n = 1
    assert f(arr, 1, P, 1 << 30, None, ctypes.byref(side)) == VQ_ERR_NULL           # no start event
    side.start = P
    assert f(arr, 1, P, 1 << 30, None, ctypes.byref(side)) == VQ_ERR_NULL           # no side stream / done event
    side.n = 0
    assert f(arr, 1, None, 0, None, ctypes.byref(side)) == VQ_ERR_WORKSPACE         # n = 0: the one-stream call


def test_gemv_pipeline_validation():
    """Host-side checks of vq_gemv_pipeline_*: everything is validated before any GPU call; no handle on failure."""
    from paper_2503_02236_amd import workloads as wl
    from paper_2503_02236_amd.binding import vq_gemv_call_t
    lib = vq.lib()
    WP = ctypes.POINTER(vq_weight_t)
    w = wl.make_weight(128, 512, 8, 16, 1, 65536, 0.02, seed=5)
    buf, pack = vq.vq_gemv_prepack(w)
    pack.data = P                                            # a (fake) aligned device address: nothing is launched here
    packed = vq_weight_t(w.N, w.K, 8, 16, 1, 65536, None, P, None, ctypes.pointer(pack))
    canonical = weight()

    def call(ws_list, xs, ys):
        n = len(ws_list)
        c = vq_gemv_call_t()
        c._keep = ((WP * n)(*[ctypes.pointer(x) for x in ws_list]), (ctypes.c_void_p * n)(*xs), (ctypes.c_void_p * n)(*ys))
        c.w, c.x, c.y = (ctypes.cast(c._keep[0], ctypes.POINTER(WP)), ctypes.cast(c._keep[1], ctypes.POINTER(ctypes.c_void_p)),
                         ctypes.cast(c._keep[2], ctypes.POINTER(ctypes.c_void_p)))
        c.count = n
        return c

    def create(calls, ws=P, ws_bytes=1 << 30):                # (P is 256-byte aligned)
        arr = (vq_gemv_call_t * len(calls))(*calls)
        h = ctypes.c_void_p(1)
        st = lib.vq_gemv_pipeline_create(arr, len(calls), ws, ws_bytes, None, ctypes.byref(h))
        assert h.value is None                               # every failure leaves a null handle
        return st, lib.vq_gemv_pipeline_workspace(arr, len(calls))

    assert P % 256 == 0
    good = call([packed, packed], [P, P], [P, P])
    arr = (vq_gemv_call_t * 1)(good)
    need = lib.vq_gemv_pipeline_workspace(arr, 1)
    # status words (256 B), a table of 2 problems (rounded to 256 B), 32 x 1 partial sums for each of 128 rows, twice
    assert need > 256 + 2 * 32 * 128 * 4 and need % 256 == 0
    h = ctypes.c_void_p()
    assert lib.vq_gemv_pipeline_create(arr, 1, P, 1 << 30, None, None) == VQ_ERR_NULL
    assert lib.vq_gemv_pipeline_create(None, 1, P, 1 << 30, None, ctypes.byref(h)) == VQ_ERR_NULL
    assert lib.vq_gemv_pipeline_create(arr, 0, P, 1 << 30, None, ctypes.byref(h)) == VQ_ERR_SHAPE
    assert create([good], ws=None) == (VQ_ERR_WORKSPACE, need)
    assert create([good], ws_bytes=need - 1) == (VQ_ERR_WORKSPACE, need)
    assert create([good], ws=P + 16) == (VQ_ERR_ALIGN, need) # 16-byte aligned is not enough here
    assert create([good, call([canonical], [P], [P])]) == (VQ_ERR_UNSUPPORTED, 0)
    assert create([call([packed], [None], [P])]) == (VQ_ERR_NULL, 0)
    assert create([call([packed], [P], [P + 2])]) == (VQ_ERR_ALIGN, 0)
    assert lib.vq_gemv_pipeline_run(None, None) == VQ_ERR_NULL
    st = ctypes.c_int(7)
    assert lib.vq_gemv_pipeline_status(None, None, ctypes.byref(st)) == VQ_ERR_NULL
    lib.vq_gemv_pipeline_destroy(None)                       # allowed


def test_gemv_pipeline_small_codebook_list_validation():
    """vq_gemv_pipeline_* with canonical uint8 weights of small codebooks (the second kind of list): the workspace is
    the problem table alone; lists that mix kinds or codebook counts are refused before any GPU call."""
    from paper_2503_02236_amd import workloads as wl
    from paper_2503_02236_amd.binding import vq_gemv_call_t
    lib = vq.lib()
    WP = ctypes.POINTER(vq_weight_t)

    def call(ws_list, xs, ys):
        n = len(ws_list)
        c = vq_gemv_call_t()
        c._keep = ((WP * n)(*[ctypes.pointer(x) for x in ws_list]), (ctypes.c_void_p * n)(*xs), (ctypes.c_void_p * n)(*ys))
        c.w, c.x, c.y = (ctypes.cast(c._keep[0], ctypes.POINTER(WP)), ctypes.cast(c._keep[1], ctypes.POINTER(ctypes.c_void_p)),
                         ctypes.cast(c._keep[2], ctypes.POINTER(ctypes.c_void_p)))
        c.count = n
        return c

    def create(calls, ws=P, ws_bytes=1 << 20):
        arr = (vq_gemv_call_t * len(calls))(*calls)
        h = ctypes.c_void_p(1)
        st = lib.vq_gemv_pipeline_create(arr, len(calls), ws, ws_bytes, None, ctypes.byref(h))
        assert h.value is None
        return st, lib.vq_gemv_pipeline_workspace(arr, len(calls))

    two = weight(N=4096, K=4096, n_codebooks=2)
    one = weight(N=300, K=1024, n_codebooks=1, n_entries=64)
    odd_k = weight(N=300, K=1000, n_codebooks=2)              # K not a multiple of 64: not this kind (and not re-tiled)
    wide = weight(N=300, K=16384, n_codebooks=2)              # x does not fit next to the codebook copies
    w16 = wl.make_weight(128, 512, 8, 16, 1, 65536, 0.02, seed=5)
    buf, pack = vq.vq_gemv_prepack(w16)
    pack.data = P
    packed = vq_weight_t(w16.N, w16.K, 8, 16, 1, 65536, None, P, None, ctypes.pointer(pack))
    good = [call([two, two, two], [P, P, P], [P, P, P]), call([two], [P], [P])]
    need = 256                                                # four table entries of 56 bytes, rounded up to 256
    assert create(good, ws=None) == (VQ_ERR_WORKSPACE, need)
    assert create(good, ws_bytes=need - 1) == (VQ_ERR_WORKSPACE, need)
    assert create(good, ws=P + 16) == (VQ_ERR_ALIGN, need)
    assert create([call([two], [P + 2], [P])]) == (VQ_ERR_ALIGN, 0)
    assert create([call([two], [None], [P])]) == (VQ_ERR_NULL, 0)
    assert create([call([two, one], [P, P], [P, P])]) == (VQ_ERR_UNSUPPORTED, 0)     # one and two codebooks in a list
    assert create([call([two], [P], [P]), call([packed], [P], [P])]) == (VQ_ERR_UNSUPPORTED, 0)   # the two kinds mixed
    assert create([call([two, odd_k], [P, P], [P, P])]) == (VQ_ERR_UNSUPPORTED, 0)
    assert create([call([wide], [P], [P])]) == (VQ_ERR_UNSUPPORTED, 0)
    assert create([call([one], [P], [P])], ws=None) == (VQ_ERR_WORKSPACE, 256)       # a single-codebook list is fine


def test_probe_argument_validation():
    lib = vq.lib()
    assert lib.vq_probe_copy(None, P, 16, None) == VQ_ERR_NULL
    assert lib.vq_probe_copy(P, P, 15, None) == VQ_ERR_SHAPE
    assert lib.vq_probe_read(P + 4, 16, P, None) == VQ_ERR_ALIGN
    assert lib.vq_probe_copy(P, P, 0, None) == 0
    assert lib.vq_probe_mfma(1, 1, 0, None, None) == VQ_ERR_NULL
    assert lib.vq_probe_mfma(-1, 1, 0, P, None) == VQ_ERR_SHAPE
    assert lib.vq_probe_mfma(0, 1, 1, P, None) == 0


def test_binding_refuses_host_tensors():
    import torch
    from paper_2503_02236_amd import workloads as wl
    w, x = wl.config1_tiny()
    wd = vq.VQWeightDev(w.N, w.K, w.v, w.code_bits, torch.from_numpy(w.codes), torch.from_numpy(w.codebooks), None)
    with pytest.raises(ValueError):
        vq.vq_gemv(wd, torch.from_numpy(x))
