"""Thin ctypes binding over libvqmi.so (argument marshalling only).

Every function here has the name and semantics of the C entry point it wraps
(``include/vq_mi355x.h``); torch is used for device memory and the current HIP
stream, nothing else.  There is no fallback: if the library has not been built
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libvqmi.so")


class VQError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_str(status)} ({status})")


class vq_gemv_pack_t(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("bytes", ctypes.c_uint64), ("S", ctypes.c_uint32), ("RB", ctypes.c_uint32),
                ("rows_per_block", ctypes.c_uint32), ("entry_bits", ctypes.c_uint32),
                ("parts", ctypes.c_uint32), ("part_cols", ctypes.c_uint32), ("wg_pitch", ctypes.c_uint32),
                ("task_off", ctypes.c_uint64), ("steps_off", ctypes.c_uint64), ("atom_off", ctypes.c_uint64),
                ("group_steps", ctypes.c_uint16 * 128)]


class vq_weight_t(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int), ("K", ctypes.c_int), ("v", ctypes.c_int), ("code_bits", ctypes.c_int),
                ("n_codebooks", ctypes.c_int), ("n_entries", ctypes.c_int),
                ("codes", ctypes.c_void_p), ("codebooks", ctypes.c_void_p), ("scale", ctypes.c_void_p),
                ("gemv_pack", ctypes.POINTER(vq_gemv_pack_t)), ("hot_entries", ctypes.c_int),
                ("cb_tile_n", ctypes.c_int), ("cb_tile_k", ctypes.c_int)]


class vq_kv_t(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int), ("H", ctypes.c_int), ("D", ctypes.c_int), ("T", ctypes.c_int),
                ("v", ctypes.c_int), ("n_entries", ctypes.c_int), ("cb_groups", ctypes.c_int),
                ("k_codes", ctypes.c_void_p), ("v_codes", ctypes.c_void_p),
                ("k_codebooks", ctypes.c_void_p), ("v_codebooks", ctypes.c_void_p),
                ("seq_lens", ctypes.c_void_p)]


class vq_gemv_call_t(ctypes.Structure):
    _fields_ = [("w", ctypes.POINTER(ctypes.POINTER(vq_weight_t))), ("x", ctypes.POINTER(ctypes.c_void_p)),
                ("y", ctypes.POINTER(ctypes.c_void_p)), ("count", ctypes.c_int)]


class vq_side_streams_t(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int), ("stream", ctypes.c_void_p * 7), ("done", ctypes.c_void_p * 7),
                ("start", ctypes.c_void_p)]


_lib = None

#: name -> (restype, argtypes); must list every symbol the header declares
SYMBOLS = {
    "vq_gemv": (ctypes.c_int, [ctypes.POINTER(vq_weight_t), ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                               ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "vq_gemv_workspace": (ctypes.c_size_t, [ctypes.POINTER(vq_weight_t), ctypes.c_int]),
    "vq_init": (ctypes.c_int, []),
    "vq_gemv_noalloc_max_workspace": (ctypes.c_size_t, []),
    "vq_gemv_noalloc": (ctypes.c_int, [ctypes.POINTER(vq_weight_t), ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                       ctypes.c_void_p]),
    "vq_reorder_by_frequency": (ctypes.c_int, [ctypes.POINTER(vq_weight_t), ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.POINTER(ctypes.c_int)]),
    "vq_gemv_batch": (ctypes.c_int, [ctypes.POINTER(ctypes.POINTER(vq_weight_t)), ctypes.POINTER(ctypes.c_void_p),
                                     ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p,
                                     ctypes.c_size_t, ctypes.c_void_p]),
    "vq_gemv_batch_workspace": (ctypes.c_size_t, [ctypes.POINTER(ctypes.POINTER(vq_weight_t)), ctypes.c_int]),
    "vq_gemv_sequence": (ctypes.c_int, [ctypes.POINTER(vq_gemv_call_t), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                        ctypes.c_void_p]),
    "vq_gemv_sequence_workspace": (ctypes.c_size_t, [ctypes.POINTER(vq_gemv_call_t), ctypes.c_int]),
    "vq_gemv_sequence_streams": (ctypes.c_int, [ctypes.POINTER(vq_gemv_call_t), ctypes.c_int, ctypes.c_void_p,
                                                ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(vq_side_streams_t)]),
    "vq_gemv_sequence_streams_workspace": (ctypes.c_size_t, [ctypes.POINTER(vq_gemv_call_t), ctypes.c_int, ctypes.c_int]),
    "vq_gemv_pipeline_workspace": (ctypes.c_size_t, [ctypes.POINTER(vq_gemv_call_t), ctypes.c_int]),
    "vq_gemv_pipeline_create": (ctypes.c_int, [ctypes.POINTER(vq_gemv_call_t), ctypes.c_int, ctypes.c_void_p,
                                                ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]),
    "vq_gemv_pipeline_run": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p]),
    "vq_gemv_pipeline_status": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)]),
    "vq_gemv_pipeline_destroy": (None, [ctypes.c_void_p]),
    "vq_gemv_prepack_bytes": (ctypes.c_size_t, [ctypes.POINTER(vq_weight_t)]),
    "vq_gemv_prepack": (ctypes.c_int, [ctypes.POINTER(vq_weight_t), ctypes.c_void_p, ctypes.c_size_t,
                                       ctypes.POINTER(vq_gemv_pack_t)]),
    "vq_gemm": (ctypes.c_int, [ctypes.POINTER(vq_weight_t), ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                               ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "vq_gemm_workspace": (ctypes.c_size_t, [ctypes.POINTER(vq_weight_t), ctypes.c_int]),
    "vq_attn_decode": (ctypes.c_int, [ctypes.POINTER(vq_kv_t), ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "vq_attn_decode_workspace": (ctypes.c_size_t, [ctypes.POINTER(vq_kv_t)]),
    "vq_attn_decode_channel_parallel": (ctypes.c_int, [ctypes.POINTER(vq_kv_t), ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p,
                                                       ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "vq_attn_decode_channel_parallel_workspace": (ctypes.c_size_t, [ctypes.POINTER(vq_kv_t)]),
    "vq_dequant": (ctypes.c_int, [ctypes.POINTER(vq_weight_t), ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]),
    "vq_kv_dequant": (ctypes.c_int, [ctypes.POINTER(vq_kv_t), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]),
    "vq_kv_quantize": (ctypes.c_int, [ctypes.POINTER(vq_kv_t), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_void_p]),
    "vq_probe_copy": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "vq_probe_read": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]),
    "vq_probe_mfma": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]),
    "vq_status_str": (ctypes.c_char_p, [ctypes.c_int]),
    "vq_version": (ctypes.c_int, []),
}


def lib() -> ctypes.CDLL:
    """Load libvqmi.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_02236_amd.build` "
                               "(or __graft_entry__.build()); there is no CPU or PyTorch fallback")
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def status_str(status: int) -> str:
    return lib().vq_status_str(int(status)).decode()


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _dev(t: Optional[torch.Tensor], name: str, dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return int(t.data_ptr())


@dataclass
class VQWeightDev:
    """Device-resident VQ weight: codes [N][K/v][R] (uint8/uint16), codebooks fp16 [R][E][v], scale fp16 [N]."""
    N: int
    K: int
    v: int
    code_bits: int
    codes: Optional[torch.Tensor]
    codebooks: torch.Tensor
    scale: Optional[torch.Tensor]
    pack_data: Optional[torch.Tensor] = None     # device copy of the vq_gemv_prepack buffer
    pack: Optional[vq_gemv_pack_t] = None        # its descriptor (data already points at pack_data)
    hot_entries: int = 0                         # from vq_reorder_by_frequency (0: entries in no particular order)
    cb_tile: Optional[tuple] = None              # (tile_n, tile_k): codebooks [N/tile_n][K/tile_k][R][E][v]

    def desc(self, use_pack: bool = True) -> vq_weight_t:
        R, E, v = self.codebooks.shape[-3:]
        tn, tk = self.cb_tile if self.cb_tile else (0, 0)
        code_dt = torch.uint16 if self.code_bits == 16 else torch.uint8   # 12-bit codes: packed bytes
        d = vq_weight_t(self.N, self.K, self.v, self.code_bits, R, E,
                        _dev(self.codes, "codes", code_dt), _dev(self.codebooks, "codebooks", torch.float16),
                        _dev(self.scale, "scale", torch.float16), None, int(self.hot_entries), int(tn), int(tk))
        if use_pack and self.pack is not None:
            d.gemv_pack = ctypes.pointer(self.pack)
        return d


@dataclass
class VQKVDev:
    """Device-resident VQ KV cache of one layer (uint8 codes [B][H][T][D/v], fp16 codebooks [H][G][E][v])."""
    B: int
    H: int
    D: int
    T: int
    v: int
    k_codes: torch.Tensor
    v_codes: torch.Tensor
    k_codebooks: torch.Tensor
    v_codebooks: torch.Tensor
    seq_lens: Optional[torch.Tensor] = None

    def desc(self) -> vq_kv_t:
        _, G, E, _ = self.k_codebooks.shape
        return vq_kv_t(self.B, self.H, self.D, self.T, self.v, E, G,
                       _dev(self.k_codes, "k_codes", torch.uint8), _dev(self.v_codes, "v_codes", torch.uint8),
                       _dev(self.k_codebooks, "k_codebooks", torch.float16),
                       _dev(self.v_codebooks, "v_codebooks", torch.float16),
                       _dev(self.seq_lens, "seq_lens", torch.int32))


def vq_gemv_prepack(w):
    """Offline re-tiling of a host ``workloads.VQWeight`` for the bs = 1 gemv (host only, no GPU).

    Returns (packed uint8 numpy buffer, vq_gemv_pack_t whose ``data`` points at that buffer), or
    (None, None) if the configuration has no packed form.
    """
    import numpy as np
    codes = np.ascontiguousarray(w.codes)
    d = vq_weight_t(w.N, w.K, w.v, w.code_bits, int(w.codebooks.shape[0]), int(w.codebooks.shape[1]),
                    codes.ctypes.data, None, None, None)
    n = int(lib().vq_gemv_prepack_bytes(ctypes.byref(d)))
    if n == 0:
        return None, None
    buf = np.empty(n + 16, dtype=np.uint8)
    off = (-buf.ctypes.data) % 16
    out = buf[off:off + n]
    pack = vq_gemv_pack_t()
    _check(lib().vq_gemv_prepack(ctypes.byref(d), out.ctypes.data, n, ctypes.byref(pack)), "vq_gemv_prepack")
    return out, pack


def vq_reorder_by_frequency(w):
    """Offline frequency reordering of a host ``workloads.VQWeight`` (host only, no GPU).

    Returns a new VQWeight with the same dequantized values whose codebook entries are sorted by
    descending use; its ``hot_entries`` is the number of leading entries that serve half of the codes.
    """
    import numpy as np
    from .workloads import VQWeight
    codes = np.ascontiguousarray(w.codes)
    cb = np.ascontiguousarray(w.codebooks)
    d = vq_weight_t(w.N, w.K, w.v, w.code_bits, int(cb.shape[0]), int(cb.shape[1]),
                    codes.ctypes.data, cb.ctypes.data, None, None)
    codes_out = np.empty_like(codes)
    cb_out = np.empty_like(cb)
    hot = ctypes.c_int(0)
    _check(lib().vq_reorder_by_frequency(ctypes.byref(d), codes_out.ctypes.data, cb_out.ctypes.data,
                                         ctypes.byref(hot)), "vq_reorder_by_frequency")
    return VQWeight(w.N, w.K, w.v, w.code_bits, codes_out, cb_out, w.scale, hot_entries=int(hot.value))


def weight_to_device(w, device="cuda:0", prepack: bool = False, keep_codes: bool = True) -> VQWeightDev:
    """Upload a host ``workloads.VQWeight`` (numpy) to the GPU; ``prepack`` adds the re-tiled gemv codes."""
    import numpy as np
    codes = None
    if keep_codes or not prepack:
        codes = torch.from_numpy(w.codes.view(np.uint16 if w.code_bits == 16 else np.uint8)).to(device)
    cb = torch.from_numpy(w.codebooks).to(device)
    sc = None if w.scale is None else torch.from_numpy(w.scale).to(device)
    wd = VQWeightDev(w.N, w.K, w.v, w.code_bits, codes, cb, sc, hot_entries=int(getattr(w, "hot_entries", 0)),
                     cb_tile=getattr(w, "cb_tile", None))
    if prepack:
        buf, pack = vq_gemv_prepack(w)
        if buf is None:
            raise ValueError("this VQ configuration has no packed gemv form")
        wd.pack_data = torch.from_numpy(buf).to(device)
        pack.data = int(wd.pack_data.data_ptr())
        wd.pack = pack
    return wd


def new_workspace(nbytes: int, device="cuda:0") -> torch.Tensor:
    """Device scratch of at least ``nbytes`` bytes (contents need no initialisation)."""
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def kv_to_device(kv, device="cuda:0") -> VQKVDev:
    """Upload a host ``workloads.VQKVCache`` (numpy) to the GPU."""
    t = lambda a: None if a is None else torch.from_numpy(a).to(device)
    return VQKVDev(kv.B, kv.H, kv.D, kv.T, kv.v, t(kv.k_codes), t(kv.v_codes), t(kv.k_codebooks),
                   t(kv.v_codebooks), t(kv.seq_lens))


def _check(status: int, where: str):
    if status != 0:
        raise VQError(status, where)


def _workspace(nbytes: int, device, ws: Optional[torch.Tensor]):
    if ws is not None:
        return ws, _dev(ws, "ws"), ws.numel() * ws.element_size()
    if nbytes == 0:
        return None, None, 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return ws, int(ws.data_ptr()), nbytes


def vq_gemv_workspace(w: VQWeightDev, bs: int) -> int:
    d = w.desc()
    return int(lib().vq_gemv_workspace(ctypes.byref(d), bs))


def vq_gemv(w: VQWeightDev, x: torch.Tensor, y: Optional[torch.Tensor] = None,
            ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """y[bs][N] = scale * (x[bs][K] @ dequant(W)^T) on the current stream."""
    bs = x.shape[0]
    if y is None:
        y = torch.empty((bs, w.N), dtype=torch.float16, device=x.device)
    d = w.desc()
    ws_t, ws_p, ws_n = _workspace(int(lib().vq_gemv_workspace(ctypes.byref(d), bs)), x.device, ws)
    _check(lib().vq_gemv(ctypes.byref(d), _dev(x, "x", torch.float16), bs, _dev(y, "y", torch.float16),
                         ws_p, ws_n, _stream()), "vq_gemv")
    return y


def vq_gemv_noalloc(w: VQWeightDev, x: torch.Tensor, y: torch.Tensor) -> torch.Tensor:
    """``vq_gemv`` with the library's built-in scratch: the caller passes inputs and the output, nothing is allocated."""
    d = w.desc()
    _check(lib().vq_gemv_noalloc(ctypes.byref(d), _dev(x, "x", torch.float16), x.shape[0],
                                 _dev(y, "y", torch.float16), _stream()), "vq_gemv_noalloc")
    return y


class GemvBatch:
    """Marshalled arguments of one ``vq_gemv_batch`` call (host pointer arrays built once)."""

    def __init__(self, ws_list, xs, ys):
        n = len(ws_list)
        self.keep = (list(ws_list), list(xs), list(ys))
        self.descs = [w.desc() for w in ws_list]
        self.w_arr = (ctypes.POINTER(vq_weight_t) * n)(*[ctypes.pointer(d) for d in self.descs])
        self.x_arr = (ctypes.c_void_p * n)(*[_dev(x, "x", torch.float16) for x in xs])
        self.y_arr = (ctypes.c_void_p * n)(*[_dev(y, "y", torch.float16) for y in ys])
        self.count = n

    def workspace(self) -> int:
        return int(lib().vq_gemv_batch_workspace(self.w_arr, self.count))

    def run(self, ws_ptr, ws_bytes) -> int:
        return lib().vq_gemv_batch(self.w_arr, self.x_arr, self.y_arr, self.count, ws_ptr, ws_bytes, _stream())


def vq_gemv_batch(ws_list, xs, ys=None, ws: Optional[torch.Tensor] = None):
    """Independent bs = 1 problems y_i = scale_i * (W_i x_i) in one call; returns the list of y_i."""
    if ys is None:
        ys = [torch.empty((1, w.N), dtype=torch.float16, device=x.device) for w, x in zip(ws_list, xs)]
    call = GemvBatch(ws_list, xs, ys)
    ws_t, ws_p, ws_n = _workspace(call.workspace(), xs[0].device, ws)
    _check(call.run(ws_p, ws_n), "vq_gemv_batch")
    return ys


class GemvSequence:
    """Marshalled arguments of one ``vq_gemv_sequence`` call: a list of calls, each a list of (weight, x, y)."""

    def __init__(self, calls):
        self.batches = [GemvBatch([t[0] for t in c], [t[1] for t in c], [t[2] for t in c]) for c in calls]
        self.arr = (vq_gemv_call_t * len(self.batches))()
        for i, b in enumerate(self.batches):
            self.arr[i].w = ctypes.cast(b.w_arr, ctypes.POINTER(ctypes.POINTER(vq_weight_t)))
            self.arr[i].x = ctypes.cast(b.x_arr, ctypes.POINTER(ctypes.c_void_p))
            self.arr[i].y = ctypes.cast(b.y_arr, ctypes.POINTER(ctypes.c_void_p))
            self.arr[i].count = b.count
        self.n = len(self.batches)

    def workspace(self) -> int:
        return int(lib().vq_gemv_sequence_workspace(self.arr, self.n))

    def run(self, ws_ptr, ws_bytes) -> int:
        return lib().vq_gemv_sequence(self.arr, self.n, ws_ptr, ws_bytes, _stream())

    def workspace_streams(self, n_streams: int) -> int:
        return int(lib().vq_gemv_sequence_streams_workspace(self.arr, self.n, n_streams))

    def run_streams(self, ws_ptr, ws_bytes, side: "SideStreams") -> int:
        return lib().vq_gemv_sequence_streams(self.arr, self.n, ws_ptr, ws_bytes, _stream(), ctypes.byref(side.c))


class GemvPipeline:
    """``vq_gemv_pipeline_*``: all products of a sequence in one persistent launch.  ``calls`` as for GemvSequence;
    the workspace tensor (256-byte aligned, allocated here unless given) and the handle live as long as this object."""

    def __init__(self, calls, ws: Optional[torch.Tensor] = None):
        self.seq = GemvSequence(calls)
        need = int(lib().vq_gemv_pipeline_workspace(self.seq.arr, self.seq.n))
        self.handle = ctypes.c_void_p()
        if need == 0:   # invalid calls: let create name the error
            _check(lib().vq_gemv_pipeline_create(self.seq.arr, self.seq.n, None, 0, _stream(), ctypes.byref(self.handle)),
                   "vq_gemv_pipeline_create")
        device = calls[0][0][1].device
        self.ws = ws if ws is not None else torch.empty(need + 256, dtype=torch.uint8, device=device)
        base = self.ws.data_ptr()
        self.ws_ptr = (base + 255) & ~255
        self.ws_bytes = self.ws.numel() - (self.ws_ptr - base)
        _check(lib().vq_gemv_pipeline_create(self.seq.arr, self.seq.n, self.ws_ptr, self.ws_bytes, _stream(),
                                             ctypes.byref(self.handle)), "vq_gemv_pipeline_create")

    def run(self) -> int:
        return lib().vq_gemv_pipeline_run(self.handle, _stream())

    def status(self) -> int:
        v = ctypes.c_int(-1)
        _check(lib().vq_gemv_pipeline_status(self.handle, _stream(), ctypes.byref(v)), "vq_gemv_pipeline_status")
        return int(v.value)

    def close(self):
        if self.handle:
            lib().vq_gemv_pipeline_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class SideStreams:
    """Side streams and events for ``vq_gemv_sequence_streams``: torch streams (default priority) and torch events
    (no timing), kept alive here; the C struct holds their raw handles."""

    def __init__(self, n: int, device="cuda:0"):
        self.streams = [torch.cuda.Stream(device=device) for _ in range(n)]
        self.events = [torch.cuda.Event(enable_timing=False) for _ in range(n + 1)]
        for e in self.events:      # torch creates the HIP event on first use
            e.record(torch.cuda.current_stream(device))
        torch.cuda.synchronize(device)
        self.c = vq_side_streams_t()
        self.c.n = n
        for i, st in enumerate(self.streams):
            self.c.stream[i] = int(st.cuda_stream)
            self.c.done[i] = int(self.events[i].cuda_event)
        self.c.start = int(self.events[n].cuda_event)


def vq_gemv_sequence(calls, ws: Optional[torch.Tensor] = None):
    """Independent batches of bs = 1 products, one launch each plus one reduction launch at the end.

    ``calls``: list of lists of (VQWeightDev, x, y).  Returns the marshalled sequence (its y tensors are filled)."""
    seq = GemvSequence(calls)
    ws_t, ws_p, ws_n = _workspace(seq.workspace(), calls[0][0][1].device, ws)
    _check(seq.run(ws_p, ws_n), "vq_gemv_sequence")
    return seq


def vq_gemm_workspace(w: VQWeightDev, M: int) -> int:
    d = w.desc()
    return int(lib().vq_gemm_workspace(ctypes.byref(d), M))


def vq_gemm(w: VQWeightDev, X: torch.Tensor, Y: Optional[torch.Tensor] = None,
            ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y[M][N] = scale * (X[M][K] @ dequant(W)^T) on the current stream (matrix cores)."""
    M = X.shape[0]
    if Y is None:
        Y = torch.empty((M, w.N), dtype=torch.float16, device=X.device)
    d = w.desc()
    ws_t, ws_p, ws_n = _workspace(int(lib().vq_gemm_workspace(ctypes.byref(d), M)), X.device, ws)
    _check(lib().vq_gemm(ctypes.byref(d), _dev(X, "X", torch.float16), M, _dev(Y, "Y", torch.float16),
                         ws_p, ws_n, _stream()), "vq_gemm")
    return Y


def vq_attn_decode_workspace(kv: VQKVDev) -> int:
    d = kv.desc()
    return int(lib().vq_attn_decode_workspace(ctypes.byref(d)))


def vq_attn_decode(kv: VQKVDev, q: torch.Tensor, sm_scale: float, out: Optional[torch.Tensor] = None,
                   ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out[B][H][D] = softmax(sm_scale * q K^T) V over the VQ cache, on the current stream."""
    if out is None:
        out = torch.empty_like(q)
    d = kv.desc()
    ws_t, ws_p, ws_n = _workspace(int(lib().vq_attn_decode_workspace(ctypes.byref(d))), q.device, ws)
    _check(lib().vq_attn_decode(ctypes.byref(d), _dev(q, "q", torch.float16), float(sm_scale),
                                _dev(out, "out", torch.float16), ws_p, ws_n, _stream()), "vq_attn_decode")
    return out


def vq_attn_decode_channel_parallel(kv: VQKVDev, q: torch.Tensor, sm_scale: float, out: Optional[torch.Tensor] = None,
                                    ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The same product by the channel-parallel dataflow (caches with one codebook per channel sub-space)."""
    if out is None:
        out = torch.empty_like(q)
    d = kv.desc()
    ws_t, ws_p, ws_n = _workspace(int(lib().vq_attn_decode_channel_parallel_workspace(ctypes.byref(d))), q.device, ws)
    _check(lib().vq_attn_decode_channel_parallel(ctypes.byref(d), _dev(q, "q", torch.float16), float(sm_scale),
                                                 _dev(out, "out", torch.float16), ws_p, ws_n, _stream()),
           "vq_attn_decode_channel_parallel")
    return out


def vq_dequant(w: VQWeightDev, out_fp32: bool = True) -> torch.Tensor:
    """Dense W[N][K] (fp32 sum of residual entries, or its fp16 rounding): test hook."""
    W = torch.empty((w.N, w.K), dtype=torch.float32 if out_fp32 else torch.float16, device=w.codes.device)
    d = w.desc()
    _check(lib().vq_dequant(ctypes.byref(d), _dev(W, "W"), 1 if out_fp32 else 0, _stream()), "vq_dequant")
    return W


def vq_kv_quantize(kv: VQKVDev, k_new: torch.Tensor, v_new: torch.Tensor, pos: int) -> None:
    """Quantize new tokens (fp16 [B][H][n][D] each) and store their codes at positions [pos, pos + n)."""
    n = k_new.shape[2]
    d = kv.desc()
    _check(lib().vq_kv_quantize(ctypes.byref(d), _dev(k_new, "k_new", torch.float16),
                                _dev(v_new, "v_new", torch.float16), int(n), int(pos), _stream()), "vq_kv_quantize")


def vq_kv_dequant(kv: VQKVDev, which: int) -> torch.Tensor:
    """Dense fp16 K (which=0) or V (which=1) [B][H][T][D]: test hook."""
    out = torch.empty((kv.B, kv.H, kv.T, kv.D), dtype=torch.float16, device=kv.k_codes.device)
    d = kv.desc()
    _check(lib().vq_kv_dequant(ctypes.byref(d), which, _dev(out, "out"), _stream()), "vq_kv_dequant")
    return out


def vq_probe_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    n = src.numel() * src.element_size()
    _check(lib().vq_probe_copy(_dev(dst, "dst"), _dev(src, "src"), n, _stream()), "vq_probe_copy")


def vq_probe_mfma(workgroups: int, iters: int, sink: torch.Tensor, random_operands: int = 0) -> None:
    """fp16 MFMA loop without global memory traffic: workgroups x 4 waves x iters x 8 MFMAs.

    random_operands: 0 smooth register operands, 1 random register operands, 2 fresh random operands from LDS."""
    _check(lib().vq_probe_mfma(int(workgroups), int(iters), int(random_operands), _dev(sink, "sink"), _stream()),
           "vq_probe_mfma")


def vq_probe_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    n = src.numel() * src.element_size()
    _check(lib().vq_probe_read(_dev(src, "src"), n, _dev(sink, "sink"), _stream()), "vq_probe_read")
