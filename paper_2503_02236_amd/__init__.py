"""MI355X-native fused vector-quantization kernels (VQ-gemv, VQ-gemm, VQ-attn decode).

The product is ``libvqmi.so`` (hand-written gfx950 HIP kernels behind a C ABI declared in
``include/vq_mi355x.h``); this package is its thin Python binding plus the seeded synthetic
workload generators.  Import is cheap: the library is loaded on first use and its absence is
an error, never a fallback.
"""
from . import workloads  # noqa: F401
from .binding import (  # noqa: F401
    LIB_PATH, VQError, VQKVDev, VQWeightDev, kv_to_device, lib, status_str, vq_attn_decode, vq_attn_decode_channel_parallel,
    vq_attn_decode_workspace, vq_dequant, vq_gemm, vq_gemm_workspace, vq_gemv, vq_gemv_prepack,
    vq_gemv_workspace, new_workspace, vq_gemv_batch, GemvBatch, vq_gemv_sequence, GemvSequence, GemvPipeline, SideStreams, vq_reorder_by_frequency,
    vq_kv_dequant, vq_kv_quantize, vq_gemv_noalloc, vq_probe_copy, vq_probe_read, vq_probe_mfma, weight_to_device,
)
