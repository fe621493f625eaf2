"""CPU oracle for VQ matrix products and VQ-cache decode attention.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The GPU library never imports
it and shares no code with it.

The arithmetic lives in ``vq_oracle.c`` (plain C, fp64 accumulation, written
from Sec. II-A / II-B of the VQ-LLM paper, arXiv 2503.02236).  This module only
marshals numpy arrays into that C code through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vq_oracle.c")
_LIB = os.path.join(_HERE, "libvq_oracle.so")


def build(force: bool = False) -> str:
    """Compile vq_oracle.c with gcc (OpenMP over output rows / (batch, head))."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c_int, c_void, c_dbl = ctypes.c_int, ctypes.c_void_p, ctypes.c_double
        lib.vq_oracle_half_to_float.restype = ctypes.c_float
        lib.vq_oracle_half_to_float.argtypes = [ctypes.c_uint16]
        lib.vq_oracle_half_to_float_array.restype = None
        lib.vq_oracle_half_to_float_array.argtypes = [c_void, c_void, ctypes.c_size_t]
        lib.vq_oracle_threads.restype = c_int
        lib.vq_oracle_set_threads.restype = None
        lib.vq_oracle_set_threads.argtypes = [c_int]
        lib.vq_oracle_dequant.restype = None
        lib.vq_oracle_dequant.argtypes = [c_int] * 8 + [c_void] * 3
        lib.vq_oracle_unpack12.restype = None
        lib.vq_oracle_unpack12.argtypes = [c_void, ctypes.c_size_t, c_void]
        lib.vq_oracle_gemm.restype = None
        lib.vq_oracle_gemm.argtypes = [c_int] * 8 + [c_void] * 4 + [c_int, c_void, c_int, c_void]
        lib.vq_oracle_kv_quantize.restype = None
        lib.vq_oracle_kv_quantize.argtypes = [c_int] * 7 + [c_void] * 3
        lib.vq_oracle_kv_dequant.restype = None
        lib.vq_oracle_kv_dequant.argtypes = [c_int] * 7 + [c_void] * 3
        lib.vq_oracle_attn_decode.restype = None
        lib.vq_oracle_attn_decode.argtypes = ([c_int] * 7 + [c_void] * 6 + [c_dbl, c_int, c_int]
                                              + [c_void] * 3)
        _lib = lib
    return _lib


def set_threads(n: int) -> None:
    """Thread count of the following calls (for timing the oracle on one core); results do not depend on it."""
    _load().vq_oracle_set_threads(int(n))


def threads() -> int:
    """Number of OpenMP threads the C oracle will use."""
    return int(_load().vq_oracle_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f16_bits(a: np.ndarray, name: str) -> np.ndarray:
    if a.dtype != np.float16:
        raise TypeError(f"{name} must be float16, got {a.dtype}")
    return np.ascontiguousarray(a).view(np.uint16)


def half_to_float(bits: np.ndarray) -> np.ndarray:
    """fp16 bit patterns (uint16) -> fp32 values through the oracle's own converter."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float32)
    _load().vq_oracle_half_to_float_array(_ptr(bits), _ptr(out), bits.size)
    return out


def unpack12(packed: np.ndarray, n_codes: int) -> np.ndarray:
    """The first n_codes 12-bit codes of a packed byte string (through the C reader, for tests)."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8).ravel()
    if packed.size * 2 < n_codes * 3:
        raise ValueError("packed buffer too short")
    out = np.empty(n_codes, dtype=np.uint32)
    _load().vq_oracle_unpack12(_ptr(packed), n_codes, _ptr(out))
    return out


class Packed12:
    """12-bit codes: ``data`` is the packed uint8 string of the logical array [N][K/v][R] (row-major)."""

    def __init__(self, data: np.ndarray, shape):
        self.data = np.ascontiguousarray(data, dtype=np.uint8).ravel()
        self.shape = tuple(int(x) for x in shape)
        n = self.shape[0] * self.shape[1] * self.shape[2]
        if n % 2 or self.data.size != n * 3 // 2:
            raise ValueError("packed size does not match the logical shape")
        self.dtype = np.dtype(np.uint8)
        self.size = n

    def max(self):
        return int(unpack12(self.data, self.size).max()) if self.size else 0


def _code_bits(codes) -> int:
    return 12 if isinstance(codes, Packed12) else codes.dtype.itemsize * 8


def _code_buf(codes):
    return codes.data if isinstance(codes, Packed12) else np.ascontiguousarray(codes)


def _check_weight(codes, codebooks, scale, N, K, v, cb_tile):
    if not isinstance(codes, Packed12) and codes.dtype not in (np.uint8, np.uint16):
        raise TypeError("codes must be uint8, uint16 or Packed12")
    if cb_tile is None:
        if codebooks.ndim != 3:
            raise ValueError("codebooks must be [R][E][v]")
        tn = tk = 0
    else:
        tn, tk = int(cb_tile[0]), int(cb_tile[1])
        if tn <= 0 or tk <= 0 or K % tk != 0 or tk % v != 0:
            raise ValueError("codebook tile must be positive, divide K and hold whole sub-vectors")
        if codebooks.ndim != 5 or codebooks.shape[:2] != (-(-N // tn), K // tk):
            raise ValueError("per-tile codebooks must be [ceil(N/tile_n)][K/tile_k][R][E][v]")
    R, E, vv = codebooks.shape[-3:]
    if vv != v or K % v != 0:
        raise ValueError("vector length mismatch")
    if codes.shape != (N, K // v, R):
        raise ValueError(f"codes shape {codes.shape} != {(N, K // v, R)}")
    if codes.size and int(codes.max()) >= E:
        raise ValueError("code out of range")
    if scale is not None and scale.shape != (N,):
        raise ValueError("scale shape")
    return R, E, tn, tk


def dequant(codes: np.ndarray, codebooks: np.ndarray, cb_tile=None) -> np.ndarray:
    """codes [N][K/v][R] + codebooks fp16 [R][E][v] -> dense fp32 W[N][K] (Sec. II-A).

    ``cb_tile=(tile_n, tile_k)``: one set of codebooks per tile of W, codebooks
    [ceil(N/tile_n)][K/tile_k][R][E][v] (Sec. III-B, Tbl. III).
    """
    N, J, _ = codes.shape
    v = codebooks.shape[-1]
    K = J * v
    R, E, tn, tk = _check_weight(codes, codebooks, None, N, K, v, cb_tile)
    bits, codes = _code_bits(codes), _code_buf(codes)
    cb = _f16_bits(codebooks, "codebooks")
    W = np.empty((N, K), dtype=np.float32)
    _load().vq_oracle_dequant(N, K, v, bits, R, E, tn, tk, _ptr(codes), _ptr(cb), _ptr(W))
    return W


def gemm(codes: np.ndarray, codebooks: np.ndarray, scale: Optional[np.ndarray], x: np.ndarray,
         rows: Optional[Sequence[int]] = None, cb_tile=None) -> np.ndarray:
    """Y[m][n] = scale[n] * sum_k W[n][k] x[m][k] in fp64; x fp16 [M][K].

    ``rows`` restricts the evaluation to those output channels (sampled parity at
    full size); the result is then [M][len(rows)].  ``cb_tile``: see :func:`dequant`.
    """
    N, J, _ = codes.shape
    v = codebooks.shape[-1]
    K = J * v
    R, E, tn, tk = _check_weight(codes, codebooks, scale, N, K, v, cb_tile)
    if x.ndim != 2 or x.shape[1] != K:
        raise ValueError("x must be [M][K]")
    M = x.shape[0]
    bits, codes = _code_bits(codes), _code_buf(codes)
    cb = _f16_bits(codebooks, "codebooks")
    sc = None if scale is None else _f16_bits(scale, "scale")
    xb = _f16_bits(x, "x")
    rows_a = None
    NR = N
    if rows is not None:
        rows_a = np.ascontiguousarray(rows, dtype=np.int32)
        if rows_a.size and (rows_a.min() < 0 or rows_a.max() >= N):
            raise ValueError("rows out of range")
        NR = int(rows_a.size)
    Y = np.empty((M, NR), dtype=np.float64)
    _load().vq_oracle_gemm(N, K, v, bits, R, E, tn, tk, _ptr(codes), _ptr(cb), _ptr(sc),
                           _ptr(xb), M, _ptr(rows_a), NR, _ptr(Y))
    return Y


def gemv(codes, codebooks, scale, x, rows=None, cb_tile=None) -> np.ndarray:
    """Decode-phase product: same definition as :func:`gemm` with M = batch (1..16)."""
    return gemm(codes, codebooks, scale, x, rows, cb_tile)


def _check_kv(codes, codebooks, B, H, T, D):
    if codes.dtype != np.uint8:
        raise TypeError("KV codes must be uint8")
    Hc, G, E, v = codebooks.shape
    if Hc != H or D % v != 0 or codes.shape != (B, H, T, D // v):
        raise ValueError("KV shape mismatch")
    P = D // v
    if G < 1 or P % G != 0:
        raise ValueError("cb_groups must divide D/v")
    if codes.size and int(codes.max()) >= E:
        raise ValueError("code out of range")
    return G, E, v


def kv_dequant(codes: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """uint8 codes [B][H][T][D/v] + fp16 codebooks [H][G][E][v] -> fp32 [B][H][T][D]."""
    B, H, T, P = codes.shape
    v = codebooks.shape[3]
    D = P * v
    G, E, v = _check_kv(codes, codebooks, B, H, T, D)
    codes = np.ascontiguousarray(codes)
    cb = _f16_bits(codebooks, "codebooks")
    out = np.empty((B, H, T, D), dtype=np.float32)
    _load().vq_oracle_kv_dequant(B, H, D, T, v, E, G, _ptr(codes), _ptr(cb), _ptr(out))
    return out


def kv_quantize(x: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """fp16 vectors [B][H][n][D] + fp16 codebooks [H][G][E][v] -> uint8 codes [B][H][n][D/v]: index of the
    closest entry per sub-vector (fp32 squared distance, fixed order, ties to the smallest index)."""
    B, H, n, D = x.shape
    Hc, G, E, v = codebooks.shape
    if Hc != H or D % v != 0 or (D // v) % G != 0 or E > 256:
        raise ValueError("shape mismatch")
    xb = _f16_bits(x, "x")
    cb = _f16_bits(codebooks, "codebooks")
    out = np.empty((B, H, n, D // v), dtype=np.uint8)
    _load().vq_oracle_kv_quantize(B, H, D, n, v, E, G, _ptr(xb), _ptr(cb), _ptr(out))
    return out


def attn_decode(k_codes, v_codes, k_codebooks, v_codebooks, q, sm_scale: float,
                seq_lens: Optional[np.ndarray] = None, t_range=None, return_stats: bool = False):
    """softmax(q K^T * sm_scale) V per (batch, head) over the dequantized cache, fp64.

    q fp16 [B][H][D] -> out fp64 [B][H][D]; with ``return_stats`` also the max score
    m[B][H] and the normaliser l[B][H] of the token range ``t_range`` = (t0, t1).
    """
    B, H, T, P = k_codes.shape
    v = k_codebooks.shape[3]
    D = P * v
    G, E, v = _check_kv(k_codes, k_codebooks, B, H, T, D)
    G2, E2, v2 = _check_kv(v_codes, v_codebooks, B, H, T, D)
    if (G2, E2, v2) != (G, E, v):
        raise ValueError("K and V codebook shapes differ")
    if q.shape != (B, H, D):
        raise ValueError("q must be [B][H][D]")
    kc, vc = np.ascontiguousarray(k_codes), np.ascontiguousarray(v_codes)
    kcb, vcb = _f16_bits(k_codebooks, "k_codebooks"), _f16_bits(v_codebooks, "v_codebooks")
    qb = _f16_bits(q, "q")
    sl = None
    if seq_lens is not None:
        sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
        if sl.shape != (B,) or sl.min() < 0 or sl.max() > T:
            raise ValueError("seq_lens")
    t0, t1 = (0, T) if t_range is None else t_range
    out = np.empty((B, H, D), dtype=np.float64)
    m = np.empty((B, H), dtype=np.float64)
    l = np.empty((B, H), dtype=np.float64)
    _load().vq_oracle_attn_decode(B, H, D, T, v, E, G, _ptr(kc), _ptr(vc), _ptr(kcb), _ptr(vcb),
                                  _ptr(sl), _ptr(qb), float(sm_scale), int(t0), int(t1),
                                  _ptr(out), _ptr(m), _ptr(l))
    return (out, m, l) if return_stats else out
