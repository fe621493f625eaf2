"""Seeded synthetic inputs for the VQ hot path (shared by the oracle tests and the GPU path).

This module holds NO arithmetic of the method: it only draws codes, codebooks,
scales, activations and queries with the shapes and distributions of the five
benchmark configurations, from numpy's PCG64 generator.

Seed convention: ``20250302 + 1000 * config + layer_index``.

The paper (VQ-LLM, arXiv 2503.02236, Sec. VII-A) evaluates on Llama-7B / 65B
layers quantized by QuiP#, AQLM, GPTVQ and CQ; those weights are not available,
so uniformly drawn codes over randomly drawn codebooks of the same shapes stand
in for them.  ``zipf_codes`` additionally gives a skewed code distribution of the
kind Sec. V-A (Fig. 7) reports, with entry 0 the most frequent, as after the
frequency reordering of Sec. V-B.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

BASE_SEED = 20250302

#: Llama-7B linear layer shapes (N out, K in): attention projections, MLP up/gate, MLP down.
LLAMA7B_SHAPES = ((4096, 4096), (11008, 4096), (4096, 11008))
#: One decoder block: q, k, v, o projections, gate, up, down.
LLAMA7B_BLOCK = (0, 0, 0, 0, 1, 1, 2)


def seed_for(config: int, layer: int = 0) -> int:
    return BASE_SEED + 1000 * config + layer


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


@dataclass
class VQWeight:
    """Host copy of one VQ-compressed weight matrix, canonical layout."""
    N: int
    K: int
    v: int
    code_bits: int
    codes: np.ndarray          # uint8/uint16 [N][K/v][R]; code_bits = 12: packed uint8 [N][K/v*R*3/2] (pack12)
    codebooks: np.ndarray      # float16 [R][E][v]
    scale: Optional[np.ndarray]  # float16 [N] or None
    hot_entries: int = 0       # set by the frequency reordering tool: leading entries that serve half of the codes
    cb_tile: Optional[tuple] = None  # (tile_n, tile_k): codebooks are [ceil(N/tile_n)][K/tile_k][R][E][v]

    @property
    def R(self) -> int:
        return int(self.codebooks.shape[-3])

    @property
    def E(self) -> int:
        return int(self.codebooks.shape[-2])

    def effective_bytes(self, bs: int = 1) -> int:
        """Algorithmic bytes of one product: codes + codebook once + x + scale + y."""
        b = self.codes.nbytes + self.codebooks.nbytes + bs * self.K * 2 + bs * self.N * 2
        if self.scale is not None:
            b += self.scale.nbytes
        return int(b)


def make_weight(N: int, K: int, v: int, code_bits: int, R: int, E: int, sigma: float, seed: int,
                with_scale: bool = True, zipf_s: Optional[float] = None,
                cb_tile: Optional[tuple] = None) -> VQWeight:
    """Uniform (or Zipf-skewed) codes, N(0, sigma) codebooks, U(0.5, 1.5) per-channel scale.

    ``cb_tile=(tile_n, tile_k)`` draws one set of codebooks per tile of W (per-tile codebook scope)."""
    if K % v:
        raise ValueError("K must be a multiple of v")
    if E > (1 << code_bits):
        raise ValueError("E exceeds the code range")
    if code_bits == 12 and ((K // v) * R) % 8:
        raise ValueError("12-bit rows must hold a multiple of 8 codes")
    rng = _rng(seed)
    dt = np.uint8 if code_bits == 8 else np.uint16
    shape = (N, K // v, R)
    if zipf_s is None:
        codes = rng.integers(0, E, size=shape, dtype=dt)
    else:
        codes = zipf_codes(rng, E, shape, zipf_s).astype(dt)
    cb_shape = (R, E, v) if cb_tile is None else (-(-N // cb_tile[0]), K // cb_tile[1], R, E, v)
    codebooks = rng.normal(0.0, sigma, size=cb_shape).astype(np.float16)
    scale = rng.uniform(0.5, 1.5, size=(N,)).astype(np.float16) if with_scale else None
    if code_bits == 12:
        codes = pack12(codes)
    return VQWeight(N, K, v, code_bits, codes, codebooks, scale, cb_tile=cb_tile)


def pack12(codes: np.ndarray) -> np.ndarray:
    """Logical codes [N][J][R] (< 4096) -> packed uint8 [N][J*R*3/2]: a little-endian bit string per row, code i in
    bits [12 i, 12 i + 12) (two codes in three bytes).  Storage format only; nothing is computed here."""
    N = codes.shape[0]
    c = codes.reshape(N, -1, 2).astype(np.uint32)
    out = np.empty((N, c.shape[1], 3), dtype=np.uint8)
    out[..., 0] = c[..., 0] & 0xFF
    out[..., 1] = (c[..., 0] >> 8) | ((c[..., 1] & 0xF) << 4)
    out[..., 2] = c[..., 1] >> 4
    return out.reshape(N, -1)


def aqlm3_like_layer(shape_idx: int, layer: int = 0) -> VQWeight:
    """The paper's VQ<8,12,2> row (Tbl. III): two additive 4096-entry codebooks of 8-vectors, packed 12-bit codes
    (3 bits per weight), Llama-7B shapes."""
    N, K = LLAMA7B_SHAPES[shape_idx]
    return make_weight(N, K, 8, 12, 2, 4096, 0.01, seed_for(8, layer * 3 + shape_idx))


def zipf_codes(rng: np.random.Generator, E: int, shape, s: float = 1.0) -> np.ndarray:
    """Codes with P(e) proportional to 1/(e+1)^s: index 0 is the hottest entry."""
    p = 1.0 / np.power(np.arange(1, E + 1, dtype=np.float64), s)
    cdf = np.cumsum(p / p.sum())
    u = rng.random(size=shape)
    return np.minimum(np.searchsorted(cdf, u), E - 1)


def shuffle_entries(w: "VQWeight", seed: int) -> "VQWeight":
    """The same weight with every codebook's entries in a random order (codes rewritten to follow).

    ``zipf_codes`` makes index 0 the hottest entry; a quantizer's codebook has no such order, so skewed
    workloads are shuffled before anything that is supposed to find the hot entries sees them.
    """
    rng = _rng(seed ^ 0x5AFE)
    codes = np.empty_like(w.codes)
    cbs = np.empty_like(w.codebooks)
    for r in range(w.R):
        perm = rng.permutation(w.E)              # new position -> old entry
        inv = np.empty(w.E, dtype=np.int64)
        inv[perm] = np.arange(w.E)
        cbs[r] = w.codebooks[r][perm]
        codes[..., r] = inv[w.codes[..., r]].astype(w.codes.dtype)
    return VQWeight(w.N, w.K, w.v, w.code_bits, codes, cbs, w.scale)


def make_activations(M: int, K: int, seed: int) -> np.ndarray:
    """fp16 activations ~ N(0, 1), [M][K]."""
    return _rng(seed ^ 0x5EED).normal(0.0, 1.0, size=(M, K)).astype(np.float16)


@dataclass
class VQKVCache:
    """Host copy of a VQ-compressed KV cache of one layer."""
    B: int
    H: int
    D: int
    T: int
    v: int
    k_codes: np.ndarray        # uint8 [B][H][T][D/v]
    v_codes: np.ndarray        # uint8 [B][H][T][D/v]
    k_codebooks: np.ndarray    # float16 [H][G][E][v]
    v_codebooks: np.ndarray    # float16 [H][G][E][v]
    q: np.ndarray              # float16 [B][H][D]
    seq_lens: Optional[np.ndarray]  # int32 [B] or None

    @property
    def G(self) -> int:
        return int(self.k_codebooks.shape[1])

    @property
    def E(self) -> int:
        return int(self.k_codebooks.shape[2])

    def effective_bytes(self) -> int:
        return int(self.k_codes.nbytes + self.v_codes.nbytes + self.k_codebooks.nbytes
                   + self.v_codebooks.nbytes + 2 * self.q.nbytes)


def make_kv(B: int, H: int, D: int, T: int, v: int, E: int, G: int, seed: int,
            ragged: bool = False) -> VQKVCache:
    """uint8 codes uniform, N(0,1) codebooks per (head, group, K|V), N(0,1) fp16 queries."""
    rng = _rng(seed)
    P = D // v
    k_codes = rng.integers(0, E, size=(B, H, T, P), dtype=np.uint8)
    v_codes = rng.integers(0, E, size=(B, H, T, P), dtype=np.uint8)
    k_cb = rng.normal(0.0, 1.0, size=(H, G, E, v)).astype(np.float16)
    v_cb = rng.normal(0.0, 1.0, size=(H, G, E, v)).astype(np.float16)
    q = rng.normal(0.0, 1.0, size=(B, H, D)).astype(np.float16)
    seq_lens = None
    if ragged:
        seq_lens = rng.integers(1, T + 1, size=(B,)).astype(np.int32)
        seq_lens[0] = T
    return VQKVCache(B, H, D, T, v, k_codes, v_codes, k_cb, v_cb, q, seq_lens)


# --- the five benchmark configurations -------------------------------------------------------

def config1_tiny() -> tuple:
    """Tiny VQ-GEMV: M=1, K=256, N=256, v=8, one 256x8 codebook N(0,0.02), uint8 codes, no scale."""
    w = make_weight(256, 256, 8, 8, 1, 256, 0.02, seed_for(1), with_scale=False)
    return w, make_activations(1, 256, seed_for(1))


def config2_layer(shape_idx: int, layer: int = 0, zipf_s: Optional[float] = None) -> VQWeight:
    """Llama-7B decode layer, one 2^16 x 8 codebook N(0,0.02), uint16 codes, fp16 scale."""
    N, K = LLAMA7B_SHAPES[shape_idx]
    return make_weight(N, K, 8, 16, 1, 65536, 0.02, seed_for(2, layer * 3 + shape_idx), zipf_s=zipf_s)


def gptvq_like_layer(shape_idx: int, layer: int = 0) -> VQWeight:
    """Per-tile codebook scope as in the paper's GPTVQ-2 row (Tbl. III): VQ<4,8,1>, one 256-entry codebook per
    (256, 256) tile of the weight, Llama-7B shapes."""
    N, K = LLAMA7B_SHAPES[shape_idx]
    return make_weight(N, K, 4, 8, 1, 256, 0.02, seed_for(7, layer * 3 + shape_idx), cb_tile=(256, 256))


def config3_layer(shape_idx: int, layer: int = 0) -> VQWeight:
    """Additive 2 x (256 x 8) codebooks N(0,0.01), uint8 code pairs, fp16 scale."""
    N, K = LLAMA7B_SHAPES[shape_idx]
    return make_weight(N, K, 8, 8, 2, 256, 0.01, seed_for(3, layer * 3 + shape_idx))


def config4_layer(N: int, v: int) -> VQWeight:
    """Prefill weight: K=4096, 2^16 x v codebook N(0,0.02) (v=8: 2 bit/weight, v=4: 4 bit), no scale."""
    return make_weight(N, 4096, v, 16, 1, 65536, 0.02, seed_for(4, (N // 4096) * 2 + (v == 4)),
                       with_scale=False)


def config5_kv(B: int = 16, H: int = 32, D: int = 128, T: int = 4096, G: int = 1,
               ragged: bool = False, v: int = 4) -> VQKVCache:
    """VQ KV cache decode attention: v=4, 256-entry codebooks ~N(0,1) per (head, K|V).
    v=2 with G=64 is the paper's CQ-4 row of Tbl. III (one codebook per 2-channel sub-space, 4 bits per value)."""
    return make_kv(B, H, D, T, v, 256, G, seed_for(5, G + (100 if v != 4 else 0)), ragged=ragged)
