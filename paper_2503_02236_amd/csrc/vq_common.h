// Internal helpers shared by the gfx950 kernels of libvqmi (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "vq_mi355x.h"

namespace vq {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// 16-byte value that can be viewed as codes, packed halves or dwords.
union alignas(16) V16 {
    uint4 u;
    uint32_t w[4];
    uint16_t h[8];
    uint8_t b[16];
    half2_t h2[4];
    half8_t h8;
};

union alignas(8) V8 {
    uint2 u;
    uint32_t w[2];
    uint16_t h[4];
    half2_t h2[2];
    half4_t h4;
};

__device__ __forceinline__ V16 ld16(const void *p) {
    V16 r;
    r.u = *reinterpret_cast<const uint4 *>(p);
    return r;
}
__device__ __forceinline__ V8 ld8(const void *p) {
    V8 r;
    r.u = *reinterpret_cast<const uint2 *>(p);
    return r;
}

// a.x*b.x + a.y*b.y + c with fp32 accumulation (v_dot2_f32_f16).
__device__ __forceinline__ float dot2(half2_t a, half2_t b, float c) {
    return __builtin_amdgcn_fdot2(a, b, c, false);
}

// Sum over the 64 lanes of a wavefront; every lane gets the total.
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
    return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x = fmaxf(x, __shfl_xor(x, m, 64));
    return x;
}

// Tag type for packed 12-bit codes (VQ-LLM Sec. VII-B: VQ<8,12,2> has an unaligned 12-bit storage format).
// Reading of the layout: one little-endian bit string, code i in bits [12 i, 12 i + 12), i.e. two codes in
// three bytes, in the canonical order [N][K/v][R].
struct Code12 {};

// Code number idx of a canonical code array.
template <typename CodeT>
__device__ __forceinline__ unsigned read_code(const void *codes, size_t idx) {
    return reinterpret_cast<const CodeT *>(codes)[idx];
}
template <>
__device__ __forceinline__ unsigned read_code<Code12>(const void *codes, size_t idx) {
    const uint8_t *b = reinterpret_cast<const uint8_t *>(codes) + (idx >> 1) * 3;
    return (idx & 1) ? ((unsigned)b[1] >> 4) | ((unsigned)b[2] << 4) : (unsigned)b[0] | (((unsigned)b[1] & 0xFu) << 8);
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Host-side validation shared by the entry points (no HIP calls).
int check_weight(const vq_weight_t *w, bool need_codes);
int check_pack(const vq_weight_t *w);
bool gemv_uses_pack(const vq_weight_t *w, int bs);
size_t gemv_packed_workspace(const vq_weight_t *w);
int launch_gemv_packed(const vq_weight_t *w, const void *x, void *y, void *ws, hipStream_t s);
size_t gemv_packed_batch_workspace(const vq_weight_t *const *w, int count);
int launch_gemv_packed_batch(const vq_weight_t *const *w, const void *const *x, void *const *y, int count, void *ws,
                             hipStream_t s);
size_t gemv_packed_sequence_workspace(const vq_gemv_call_t *calls, int n_calls);
int launch_gemv_packed_sequence(const vq_gemv_call_t *calls, int n_calls, void *ws, hipStream_t s);
// The pipelined launch (one persistent kernel for all problems of a sequence).
struct GemvPipeline;
size_t gemv_pipeline_workspace(const vq_gemv_call_t *calls, int n_calls);
bool gemv_pipeline_supports(const vq_weight_t *w);
int gemv_pipeline_create(const vq_gemv_call_t *calls, int n_calls, void *ws, hipStream_t s, GemvPipeline **out);
void gemv_pipeline_destroy(GemvPipeline *h);
int launch_gemv_pipeline(const GemvPipeline *h, hipStream_t s);
int gemv_pipeline_status(const GemvPipeline *h, hipStream_t s, int *status);
int check_kv(const vq_kv_t *kv);

// Kernel launchers (defined next to their kernels).
int launch_dequant(const vq_weight_t *w, void *W, int out_fp32, hipStream_t s);
int launch_kv_dequant(const vq_kv_t *kv, int which, void *out, hipStream_t s);
int launch_gemv(const vq_weight_t *w, const void *x, int bs, void *y, void *ws, hipStream_t s);
size_t gemv_workspace(const vq_weight_t *w, int bs);
int launch_gemv_rows(const vq_weight_t *w, const void *x, int bs, void *y, hipStream_t s);
bool gemv_mfma_supported(const vq_weight_t *w);
int launch_gemv_mfma(const vq_weight_t *w, const void *x, int bs, void *y, hipStream_t s);
int launch_gemv_generic(const vq_weight_t *w, const void *x, int bs, void *y, hipStream_t s);
int launch_gemm(const vq_weight_t *w, const void *X, int M, void *Y, void *ws, hipStream_t s);
size_t gemm_workspace(const vq_weight_t *w, int M);
int launch_gemm_dense(const half_t *A, const half_t *B, const half_t *scale, half_t *C, int M, int N, int K,
                      hipStream_t s);
bool gemv_mfma_batch_supported(const vq_weight_t *const *w, int count);
int launch_gemv_mfma_batch(const vq_weight_t *const *w, const void *const *x, void *const *y, int count, hipStream_t s);
// bs = 1 with 16 LDS copies of every entry of a small codebook: a list of problems in one launch (gemv_replica.hip)
struct GemvReplicaList;
bool gemv_replica_supported(const vq_weight_t *w);
size_t gemv_replica_list_workspace(int n);
int gemv_replica_list_create(const vq_gemv_call_t *calls, int n_calls, void *ws, hipStream_t s, GemvReplicaList **out);
void gemv_replica_list_destroy(GemvReplicaList *h);
int launch_gemv_replica_list(const GemvReplicaList *h, hipStream_t s);
int launch_attn_decode(const vq_kv_t *kv, const void *q, float sm_scale, void *out, void *ws, hipStream_t s);
// channel-parallel variant for caches with one codebook per channel sub-space (attn_channel.hip)
bool attn_channel_supported(const vq_kv_t *kv);
size_t attn_channel_workspace(const vq_kv_t *kv);
int launch_attn_channel(const vq_kv_t *kv, const void *q, float sm_scale, void *out, void *ws, hipStream_t s);
size_t attn_decode_workspace(const vq_kv_t *kv);
int launch_kv_quantize(const vq_kv_t *kv, const void *k_new, const void *v_new, int n_new, int pos, hipStream_t s);
int launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t s);
int launch_probe_read(const void *src, size_t bytes, void *sink, hipStream_t s);
int launch_probe_mfma(int workgroups, int iters, int random_operands, void *sink, hipStream_t s);

inline int launch_status() { return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_LAUNCH; }

// Per-kernel launch set-up that HIP keeps per device: the dynamic LDS limit above 64 KiB, and -- for kernels
// that form absolute LDS addresses, which is only right when their dynamic LDS starts at address 0 -- the
// check that the kernel has no static LDS.  What has been done is remembered per device in atomics (calls may
// come from several host threads; doing either step twice is harmless), one object per kernel.
constexpr int kMaxDevices = 64;
struct KernelSetup {
    std::atomic<size_t> lds_granted[kMaxDevices];
    std::atomic<int> static_lds[kMaxDevices];   // 0: not looked at yet, 1: none, 2: the kernel has static LDS
};
// Returns VQ_OK, or VQ_ERR_LAUNCH when the runtime refuses or (need_lds_base_0) the kernel has static LDS.
inline int kernel_setup(const void *kernel, size_t lds, bool need_lds_base_0, KernelSetup &ks) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VQ_ERR_LAUNCH;
    if (need_lds_base_0) {
        int st = ks.static_lds[dev].load(std::memory_order_relaxed);
        if (st == 0) {
            hipFuncAttributes fa;
            if (hipFuncGetAttributes(&fa, kernel) != hipSuccess) return VQ_ERR_LAUNCH;
            st = fa.sharedSizeBytes == 0 ? 1 : 2;
            ks.static_lds[dev].store(st, std::memory_order_relaxed);
        }
        if (st != 1) return VQ_ERR_LAUNCH;
    }
    if (lds > 64 * 1024 && lds > ks.lds_granted[dev].load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return VQ_ERR_LAUNCH;
        ks.lds_granted[dev].store(lds, std::memory_order_relaxed);
    }
    return VQ_OK;
}

}  // namespace vq
