"""Pins for the CPU oracle (no GPU): what the paper's definitions and plain mathematics fix.

The paper prints no numeric example, so the pins are closed forms, special cases
that reduce to an index sum or to a dense library matmul, invariants (linearity,
entry permutation, token-range splitting) and a hand-worked VQ<4,2,2> instance.
Each pin is aimed at one kind of mistake: a dropped residual, a wrong codebook or
group index, a transposed operand, a missing scale, a wrong softmax normaliser.
"""
import json
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- fp16 conversion

def test_half_to_float_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.half_to_float(bits)
    want = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))  # signed zeros too


# ---------------------------------------------------------------- hand-worked VQ<4,2,2>

def _golden():
    with open(os.path.join(GOLDEN, "vq_4_2_2_handworked.json")) as f:
        g = json.load(f)
    codes = np.array(g["codes"], dtype=np.uint8)
    cb = np.array(g["codebooks"], dtype=np.float16)
    x = np.array(g["x"], dtype=np.float16)
    return g, codes, cb, x


def test_dequant_handworked_vq_4_2_2():
    g, codes, cb, _ = _golden()
    W = oracle.dequant(codes, cb)
    assert W.dtype == np.float32
    assert np.array_equal(W, np.array(g["W"], dtype=np.float32))


def test_gemm_handworked_vq_4_2_2():
    g, codes, cb, x = _golden()
    y = oracle.gemm(codes, cb, None, x)
    assert np.array_equal(y, np.array(g["y_unscaled"], dtype=np.float64))
    ys = oracle.gemm(codes, cb, np.array(g["scale"], dtype=np.float16), x)
    assert np.array_equal(ys, np.array(g["y_scaled"], dtype=np.float64))
    # uint16 storage of the same codes gives the same result
    assert np.array_equal(oracle.gemm(codes.astype(np.uint16), cb, None, x), y)


# ---------------------------------------------------------------- one-hot codebook = index sum

@pytest.mark.parametrize("v,code_dtype", [(8, np.uint8), (4, np.uint16)])
def test_one_hot_codebook_is_index_sum(v, code_dtype):
    r = rng(11)
    N, K, M = 37, 24 * v, 3           # N != K and M > 1: a transposed operand cannot pass
    J = K // v
    E = v + 1                         # e_0 .. e_{v-1}, then the zero vector
    cb = np.zeros((1, E, v), dtype=np.float16)
    cb[0, :v] = np.eye(v, dtype=np.float16)
    codes = r.integers(0, E, size=(N, J, 1)).astype(code_dtype)
    x = r.normal(size=(M, K)).astype(np.float16)
    y = oracle.gemm(codes, cb, None, x)
    want = np.zeros((M, N))
    xd = x.astype(np.float64)
    for m in range(M):
        for n in range(N):
            s = 0.0
            for j in range(J):
                c = int(codes[n, j, 0])
                if c < v:
                    s += xd[m, j * v + c]
            want[m, n] = s
    assert np.array_equal(y, want)    # same addends, same order -> identical


# ---------------------------------------------------------------- palette codebooks = dense matmul

def test_palette_codebooks_equal_dense_fp64_matmul():
    r = rng(12)
    v, N, K, M = 4, 48, 64, 5
    J = K // v
    palette = r.normal(0, 0.02, size=256).astype(np.float16)
    cb = np.zeros((v, 256, v), dtype=np.float16)      # codebook r holds palette[e] * e_r
    for i in range(v):
        cb[i, :, i] = palette
    codes = r.integers(0, 256, size=(N, J, v), dtype=np.uint8)
    W = palette[codes].reshape(N, K).astype(np.float64)   # dense weight, no dequant code involved
    x = r.normal(size=(M, K)).astype(np.float16)
    scale = r.uniform(0.5, 1.5, size=N).astype(np.float16)
    y = oracle.gemm(codes, cb, scale, x)
    want = (x.astype(np.float64) @ W.T) * scale.astype(np.float64)[None, :]
    assert y.shape == (M, N)
    np.testing.assert_allclose(y, want, rtol=0, atol=1e-13 * np.abs(want).max() * K)
    assert np.array_equal(oracle.dequant(codes, cb).astype(np.float64), W)


# ---------------------------------------------------------------- linearity, scale, rows, permutation

def _dyadic_weight(r, N, K, v, R, E, code_dtype):
    # entries are multiples of 2^-6 in [-2, 2): any sum of R <= 4 of them is exact in fp32
    cb = (r.integers(-128, 128, size=(R, E, v)) / 64.0).astype(np.float16)
    codes = r.integers(0, E, size=(N, K // v, R)).astype(code_dtype)
    return codes, cb


def test_linear_in_residual_codebooks_and_scale():
    r = rng(13)
    N, K, v, M = 29, 96, 8, 2
    codes, cb = _dyadic_weight(r, N, K, v, 2, 256, np.uint8)
    x = (r.integers(-64, 64, size=(M, K)) / 16.0).astype(np.float16)
    both = oracle.gemm(codes, cb, None, x)
    only0 = oracle.gemm(codes[:, :, :1].copy(), cb[:1].copy(), None, x)
    only1 = oracle.gemm(codes[:, :, 1:].copy(), cb[1:].copy(), None, x)
    assert np.array_equal(both, only0 + only1)        # dyadic inputs: every sum is exact
    assert np.abs(only1).max() > 0                    # the second residual is not silently dropped
    scale = np.array([0.5, 2.0, 1.5] * 10, dtype=np.float16)[:N]
    scaled = oracle.gemm(codes, cb, scale, x)
    assert np.array_equal(scaled, both * scale.astype(np.float64)[None, :])


def test_three_residuals_sum_left_to_right_in_fp32():
    # 1 + 2^-24 + 2^-24 in fp32: (1 + 2^-24) rounds to 1, then again 1; right-to-left would give 1 + 2^-23.
    cb = np.zeros((3, 2, 4), dtype=np.float16)
    cb[0, 1] = 1.0
    cb[1, 1] = 2.0 ** -24
    cb[2, 1] = 2.0 ** -24
    codes = np.ones((1, 1, 3), dtype=np.uint8)
    W = oracle.dequant(codes, cb)
    assert np.array_equal(W, np.ones((1, 4), dtype=np.float32))


def test_gemm_rows_equal_separate_gemvs_and_row_subsets():
    r = rng(14)
    N, K, v, M = 40, 64, 8, 6
    codes = r.integers(0, 512, size=(N, K // v, 1)).astype(np.uint16)
    cb = r.normal(0, 0.02, size=(1, 512, v)).astype(np.float16)
    scale = r.uniform(0.5, 1.5, size=N).astype(np.float16)
    x = r.normal(size=(M, K)).astype(np.float16)
    Y = oracle.gemm(codes, cb, scale, x)
    for m in range(M):
        assert np.array_equal(Y[m:m + 1], oracle.gemv(codes, cb, scale, x[m:m + 1]))
    rows = [39, 0, 7, 7, 21]
    assert np.array_equal(oracle.gemm(codes, cb, scale, x, rows=rows), Y[:, rows])


def test_entry_permutation_with_reindexed_codes_is_invariant():
    # Sec. V-B: entries may be reordered offline if the codes are re-indexed.
    r = rng(15)
    N, K, v, E = 16, 64, 8, 256
    codes = r.integers(0, E, size=(N, K // v, 2), dtype=np.uint8)
    cb = r.normal(0, 0.01, size=(2, E, v)).astype(np.float16)
    W = oracle.dequant(codes, cb)
    perm = np.stack([r.permutation(E), r.permutation(E)])        # new index -> old index
    inv = np.empty_like(perm)
    for i in range(2):
        inv[i, perm[i]] = np.arange(E)
    cb2 = np.stack([cb[i][perm[i]] for i in range(2)])
    codes2 = np.stack([inv[i][codes[:, :, i]] for i in range(2)], axis=-1).astype(np.uint8)
    assert np.array_equal(oracle.dequant(codes2, cb2).view(np.uint32), W.view(np.uint32))


def test_dequant_r1_keeps_fp16_bits_including_subnormals_and_negative_zero():
    cb = np.array([[[6e-8, -6e-8, 0.0, -0.0], [3.0e-5, -6.1e-5, 65504.0, -65504.0]]], dtype=np.float16)
    codes = np.array([[[0], [1]], [[1], [0]]], dtype=np.uint8)
    W = oracle.dequant(codes, cb)
    back = W.astype(np.float16).view(np.uint16)
    want = np.concatenate([cb[0, 0], cb[0, 1], cb[0, 1], cb[0, 0]]).view(np.uint16).reshape(2, 8)
    assert np.array_equal(back, want)
    assert np.array_equal(W.view(np.uint32), cb[0][codes[:, :, 0]].reshape(2, 8).astype(np.float32).view(np.uint32))


def test_dequant_matches_numpy_gather_on_random_data():
    r = rng(16)
    N, K, v, E = 33, 72, 8, 1000
    codes = r.integers(0, E, size=(N, K // v, 2)).astype(np.uint16)
    cb = r.normal(0, 0.02, size=(2, E, v)).astype(np.float16)
    want = (cb[0][codes[:, :, 0]].astype(np.float32) + cb[1][codes[:, :, 1]].astype(np.float32)).reshape(N, K)
    assert np.array_equal(oracle.dequant(codes, cb).view(np.uint32), want.view(np.uint32))


def test_fp16_output_rounding_sits_well_inside_the_tolerance():
    r = rng(17)
    N, K, v = 256, 512, 8
    codes = r.integers(0, 256, size=(N, K // v, 1), dtype=np.uint8)
    cb = r.normal(0, 0.02, size=(1, 256, v)).astype(np.float16)
    x = r.normal(size=(1, K)).astype(np.float16)
    y = oracle.gemv(codes, cb, None, x)
    y16 = y.astype(np.float16).astype(np.float64)
    rel = np.linalg.norm(y16 - y) / np.linalg.norm(y)
    assert 5e-5 < rel < 6e-4          # about 2^-11/sqrt(3); the parity bar is 2e-3


# ---------------------------------------------------------------- KV cache dequant

def test_kv_dequant_handworked_group_mapping():
    # B=1, H=2, T=2, D=8, v=2 -> 4 sub-vectors per token; G=2 -> sub-vectors 0,1 use codebook 0; 2,3 use codebook 1
    cb = np.zeros((2, 2, 3, 2), dtype=np.float16)
    for h in range(2):
        for g in range(2):
            for e in range(3):
                cb[h, g, e] = [100 * h + 10 * g + e, -(100 * h + 10 * g + e)]
    codes = np.array([[[[0, 1, 2, 0], [2, 2, 1, 1]],
                       [[1, 0, 0, 2], [0, 0, 0, 0]]]], dtype=np.uint8)
    out = oracle.kv_dequant(codes, cb)
    want = np.array([[[[0, -0, 1, -1, 12, -12, 10, -10], [2, -2, 2, -2, 11, -11, 11, -11]],
                      [[101, -101, 100, -100, 110, -110, 112, -112], [100, -100, 100, -100, 110, -110, 110, -110]]]],
                    dtype=np.float32)
    assert np.array_equal(out, want)


def test_kv_dequant_g1_equals_replicated_group_codebooks():
    r = rng(18)
    B, H, T, D, v, E = 2, 3, 5, 16, 4, 256
    codes = r.integers(0, E, size=(B, H, T, D // v), dtype=np.uint8)
    cb1 = r.normal(size=(H, 1, E, v)).astype(np.float16)
    cbG = np.repeat(cb1, D // v, axis=1)
    assert np.array_equal(oracle.kv_dequant(codes, cb1), oracle.kv_dequant(codes, cbG))


# ---------------------------------------------------------------- attention

def _kv(seed, B=2, H=3, T=19, D=16, v=4, E=256, G=1):
    r = rng(seed)
    P = D // v
    return dict(
        k_codes=r.integers(0, E, size=(B, H, T, P), dtype=np.uint8),
        v_codes=r.integers(0, E, size=(B, H, T, P), dtype=np.uint8),
        k_codebooks=r.normal(size=(H, G, E, v)).astype(np.float16),
        v_codebooks=r.normal(size=(H, G, E, v)).astype(np.float16),
        q=r.normal(size=(B, H, D)).astype(np.float16),
    )


def test_attention_single_token_returns_its_value_vector():
    kv = _kv(21, T=1)
    out = oracle.attn_decode(**kv, sm_scale=0.25)
    Vd = oracle.kv_dequant(kv["v_codes"], kv["v_codebooks"])
    assert np.array_equal(out, Vd[:, :, 0, :].astype(np.float64))


def test_attention_zero_query_returns_mean_value():
    kv = _kv(22)
    kv["q"] = np.zeros_like(kv["q"])
    out = oracle.attn_decode(**kv, sm_scale=0.25)
    Vd = oracle.kv_dequant(kv["v_codes"], kv["v_codebooks"]).astype(np.float64)
    np.testing.assert_allclose(out, Vd.mean(axis=2), rtol=0, atol=1e-14)


def test_attention_dominant_key_selects_its_value():
    kv = _kv(23, B=1, H=1, T=9, D=8, v=4, E=4)
    # K codebook: entry 3 is large and aligned with q; the others are zero
    kv["k_codebooks"] = np.zeros((1, 1, 4, 4), dtype=np.float16)
    kv["k_codebooks"][0, 0, 3] = 8.0
    kv["q"] = np.full((1, 1, 8), 4.0, dtype=np.float16)
    kv["k_codes"] = np.zeros((1, 1, 9, 2), dtype=np.uint8)
    kv["k_codes"][0, 0, 5] = 3                               # token 5: score 1.0 * 8*4*8 = 256, others 0
    out = oracle.attn_decode(**kv, sm_scale=1.0)
    Vd = oracle.kv_dequant(kv["v_codes"], kv["v_codebooks"]).astype(np.float64)
    np.testing.assert_allclose(out[0, 0], Vd[0, 0, 5], rtol=0, atol=1e-30 + 9 * np.exp(-256.0) * 10)


@pytest.mark.parametrize("G", [1, 4])
def test_attention_equals_dense_fp64_softmax_attention(G):
    kv = _kv(24, G=G)
    sm = 1.0 / np.sqrt(16.0)
    out = oracle.attn_decode(**kv, sm_scale=sm)
    Kd = oracle.kv_dequant(kv["k_codes"], kv["k_codebooks"]).astype(np.float64)
    Vd = oracle.kv_dequant(kv["v_codes"], kv["v_codebooks"]).astype(np.float64)
    q = kv["q"].astype(np.float64)
    s = np.einsum("bhd,bhtd->bht", q, Kd) * sm
    p = np.exp(s - s.max(axis=-1, keepdims=True))
    p /= p.sum(axis=-1, keepdims=True)
    want = np.einsum("bht,bhtd->bhd", p, Vd)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-13)
    # sm_scale is applied to the scores, not the output: doubling it must change the result
    assert np.abs(oracle.attn_decode(**kv, sm_scale=2 * sm) - out).max() > 1e-3


def test_attention_token_range_split_merges_by_log_sum_exp():
    kv = _kv(25, T=23)
    sm = 0.3
    full = oracle.attn_decode(**kv, sm_scale=sm)
    o1, m1, l1 = oracle.attn_decode(**kv, sm_scale=sm, t_range=(0, 9), return_stats=True)
    o2, m2, l2 = oracle.attn_decode(**kv, sm_scale=sm, t_range=(9, 23), return_stats=True)
    m = np.maximum(m1, m2)
    w1, w2 = l1 * np.exp(m1 - m), l2 * np.exp(m2 - m)
    merged = (o1 * w1[..., None] + o2 * w2[..., None]) / (w1 + w2)[..., None]
    np.testing.assert_allclose(merged, full, rtol=0, atol=1e-13)


def test_attention_seq_lens_equal_truncated_cache():
    kv = _kv(26, B=3, T=12)
    lens = np.array([12, 5, 1], dtype=np.int32)
    out = oracle.attn_decode(**kv, sm_scale=0.25, seq_lens=lens)
    for b in range(3):
        cut = {k: (a[b:b + 1, :, :lens[b]] if k.endswith("codes") else a) for k, a in kv.items()}
        cut["q"] = kv["q"][b:b + 1]
        assert np.array_equal(out[b:b + 1], oracle.attn_decode(**cut, sm_scale=0.25))


def test_attention_g1_equals_replicated_group_codebooks():
    kv = _kv(27)
    out1 = oracle.attn_decode(**kv, sm_scale=0.25)
    kvG = dict(kv)
    kvG["k_codebooks"] = np.repeat(kv["k_codebooks"], 4, axis=1)
    kvG["v_codebooks"] = np.repeat(kv["v_codebooks"], 4, axis=1)
    assert np.array_equal(out1, oracle.attn_decode(**kvG, sm_scale=0.25))


# ---------------------------------------------------------------- per-tile codebooks (Sec. III-B, Tbl. III)

def test_per_tile_codebooks_equal_per_tensor_results_assembled_tile_by_tile():
    # Each (tile_n, tile_k) tile of W has its own codebooks.  Tile by tile this is the per-tensor case (pinned
    # above) on the tile's codes, so the tiled dequantization must equal the blocks stitched together, and the
    # product must equal a dense fp64 matmul of that stitched matrix.
    rng = np.random.default_rng(77)
    N, K, v, R, E, tn, tk = 20, 48, 4, 2, 16, 8, 16          # ragged last row tile (20 = 8 + 8 + 4)
    TN, TK = -(-N // tn), K // tk
    cbs = rng.integers(-8, 9, size=(TN, TK, R, E, v)).astype(np.float16)
    codes = rng.integers(0, E, size=(N, K // v, R)).astype(np.uint8)
    W = oracle.dequant(codes, cbs, cb_tile=(tn, tk))
    want = np.empty((N, K), dtype=np.float32)
    for a in range(TN):
        for b in range(TK):
            rows = slice(a * tn, min(N, (a + 1) * tn))
            cols = slice(b * tk // v, (b + 1) * tk // v)
            want[rows, b * tk:(b + 1) * tk] = oracle.dequant(np.ascontiguousarray(codes[rows, cols]), cbs[a, b])
    assert W.tobytes() == want.tobytes()
    x = rng.integers(-4, 5, size=(3, K)).astype(np.float16)
    scale = rng.uniform(0.5, 1.5, size=N).astype(np.float16)
    Y = oracle.gemm(codes, cbs, scale, x, cb_tile=(tn, tk))
    dense = (x.astype(np.float64) @ want.astype(np.float64).T) * scale.astype(np.float64)[None, :]
    np.testing.assert_allclose(Y, dense, rtol=1e-14, atol=0)


def test_per_tile_codebooks_with_identical_tiles_reduce_to_one_codebook():
    rng = np.random.default_rng(78)
    N, K, v, R, E = 32, 64, 8, 1, 32
    cb = rng.normal(0, 0.02, size=(R, E, v)).astype(np.float16)
    codes = rng.integers(0, E, size=(N, K // v, R)).astype(np.uint8)
    tiled = np.broadcast_to(cb, (2, 4, R, E, v)).copy()
    assert oracle.dequant(codes, tiled, cb_tile=(16, 16)).tobytes() == oracle.dequant(codes, cb).tobytes()
    # and a tile that differs changes exactly its block
    tiled[1, 2] += np.float16(1.0)
    d = oracle.dequant(codes, tiled, cb_tile=(16, 16)) - oracle.dequant(codes, cb)
    mask = np.zeros((N, K), dtype=bool)
    mask[16:32, 32:48] = True
    assert (d[~mask] == 0).all() and (d[mask] != 0).all()


# ---------------------------------------------------------------- 12-bit code strings (reading; Sec. VII-B)

def _pack12_numpy(codes):
    """Independent packer: build the bit string with Python integers, bit by bit."""
    codes = [int(c) for c in np.asarray(codes).ravel()]
    big = 0
    for i, c in enumerate(codes):
        big |= c << (12 * i)
    return np.frombuffer(big.to_bytes(len(codes) * 3 // 2, "little"), dtype=np.uint8).copy()


def test_unpack12_hand_worked_bytes():
    import json, os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "packed12_handworked.json")))
    got = oracle.unpack12(np.array(g["bytes"], dtype=np.uint8), len(g["codes"]))
    assert got.tolist() == g["codes"]
    assert _pack12_numpy(g["codes"]).tolist() == g["bytes"]


def test_packed12_weight_equals_the_same_codes_stored_as_uint16():
    rng = np.random.default_rng(91)
    N, K, v, R, E = 12, 64, 8, 2, 4096
    codes = rng.integers(0, E, size=(N, K // v, R)).astype(np.uint16)
    codes[0, 0, 0], codes[0, 0, 1], codes[-1, -1, -1] = 4095, 0, 4095      # extremes at both ends of the string
    cb = rng.normal(0, 0.02, size=(R, E, v)).astype(np.float16)
    packed = oracle.Packed12(_pack12_numpy(codes), codes.shape)
    assert oracle.unpack12(packed.data, codes.size).tolist() == codes.ravel().tolist()
    assert oracle.dequant(packed, cb).tobytes() == oracle.dequant(codes, cb).tobytes()
    x = rng.normal(0, 1, size=(3, K)).astype(np.float16)
    scale = rng.uniform(0.5, 1.5, size=N).astype(np.float16)
    assert np.array_equal(oracle.gemm(packed, cb, scale, x), oracle.gemm(codes, cb, scale, x))


# ---------------------------------------------------------------- KV quantization: closest entry (Sec. II-A)

def test_kv_quantize_recovers_entries_and_matches_exact_integer_brute_force():
    rng = np.random.default_rng(101)
    B, H, n, D, v, E, G = 2, 3, 5, 16, 4, 32, 2
    # integer-valued entries and vectors: every distance is an exact small integer, so any correct
    # implementation in any precision agrees, and a brute force in Python integers is the reference
    cb = rng.integers(-6, 7, size=(H, G, E, v)).astype(np.float16)
    x = rng.integers(-6, 7, size=(B, H, n, D)).astype(np.float16)
    got = oracle.kv_quantize(x, cb)
    P = D // v
    for b in range(B):
        for h in range(H):
            for t in range(n):
                for p in range(P):
                    g = p * G // P
                    xv = [int(a) for a in x[b, h, t, p * v:(p + 1) * v]]
                    d = [sum((a - int(c)) ** 2 for a, c in zip(xv, cb[h, g, e])) for e in range(E)]
                    assert got[b, h, t, p] == d.index(min(d))           # ties: the smallest index
    # a vector that IS an entry gets that entry's index (first of equal entries), and dequantizing the
    # codes gives the vector back
    codes = rng.integers(0, E, size=(B, H, n, P)).astype(np.uint8)
    xd = oracle.kv_dequant(codes, cb).astype(np.float16)
    back = oracle.kv_quantize(xd, cb)
    assert np.array_equal(oracle.kv_dequant(back, cb), xd.astype(np.float32))


def test_kv_quantize_agrees_with_float64_argmin_when_the_gap_is_clear():
    rng = np.random.default_rng(102)
    B, H, n, D, v, E, G = 1, 2, 40, 32, 4, 256, 8
    cb = rng.normal(0, 1, size=(H, G, E, v)).astype(np.float16)
    x = rng.normal(0, 1, size=(B, H, n, D)).astype(np.float16)
    got = oracle.kv_quantize(x, cb)
    P = D // v
    checked = 0
    for h in range(H):
        for t in range(n):
            for p in range(P):
                g = p * G // P
                d = ((cb[h, g].astype(np.float64) - x[0, h, t, p * v:(p + 1) * v].astype(np.float64)) ** 2).sum(axis=1)
                order = np.argsort(d)
                if d[order[1]] - d[order[0]] > 1e-4 * d[order[1]]:       # fp32 rounding cannot flip these
                    assert got[0, h, t, p] == order[0]
                    checked += 1
    assert checked > 0.9 * H * n * P
