// Test-hook kernels: the dequantized operand itself (VQ-LLM Sec. II-A, dequantization:
// look up one entry per residual codebook, add them element-wise, concatenate sub-vectors),
// plus two streaming probes used to calibrate bandwidth measurements.
#include "vq_common.h"

namespace vq {

// One thread per sub-vector: W[n][j*V .. j*V+V) = sum_r C_r[code[n][j][r]] (fp32, r ascending).
template <typename CodeT, int V, bool OUT32>
__global__ __launch_bounds__(256) void dequant_kernel(const void *__restrict__ codes,
                                                      const half_t *__restrict__ cb_all, void *__restrict__ out,
                                                      long n_vec, int R, int E, int J, int tile_n, int tile_j,
                                                      int tiles_k) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long stride = (long)gridDim.x * blockDim.x;
    for (; i < n_vec; i += stride) {
        float acc[V];
        half_t first[V];
        // per-tile codebooks (Sec. III-B, Tbl. III): the set of the tile that holds sub-vector (n, j)
        const half_t *cb = cb_all;
        if (tile_n > 0) cb += ((size_t)((i / J) / tile_n) * tiles_k + (size_t)((i % J) / tile_j)) * ((size_t)R * E * V);
        for (int r = 0; r < R; ++r) {
            unsigned c = read_code<CodeT>(codes, (size_t)i * R + r);
            const half_t *e = cb + ((size_t)r * E + c) * V;
#pragma unroll
            for (int k = 0; k < V; ++k) {
                half_t h = e[k];
                if (r == 0) {
                    first[k] = h;
                    acc[k] = (float)h;
                } else {
                    acc[k] += (float)h;
                }
            }
        }
        if (OUT32) {
            float *o = reinterpret_cast<float *>(out) + i * V;
#pragma unroll
            for (int k = 0; k < V; ++k) o[k] = acc[k];
        } else {
            half_t *o = reinterpret_cast<half_t *>(out) + i * V;
#pragma unroll
            for (int k = 0; k < V; ++k) o[k] = (R == 1) ? first[k] : (half_t)acc[k];  // RNE
        }
    }
}

int launch_dequant(const vq_weight_t *w, void *W, int out_fp32, hipStream_t s) {
    long n_vec = (long)w->N * (w->K / w->v);
    int blocks = (int)((n_vec + 255) / 256 < 65536 ? (n_vec + 255) / 256 : 65536);
    const int J = w->K / w->v, tile_n = w->cb_tile_n, tile_j = tile_n > 0 ? w->cb_tile_k / w->v : 1,
              tiles_k = tile_n > 0 ? w->K / w->cb_tile_k : 1;
#define VQ_DQ(CT, V)                                                                                            \
    do {                                                                                                        \
        if (out_fp32)                                                                                           \
            dequant_kernel<CT, V, true><<<blocks, 256, 0, s>>>(w->codes, (const half_t *)w->codebooks, W, \
                                                               n_vec, w->n_codebooks, w->n_entries, J, tile_n, tile_j, tiles_k); \
        else                                                                                                    \
            dequant_kernel<CT, V, false><<<blocks, 256, 0, s>>>(w->codes, (const half_t *)w->codebooks, W, \
                                                                n_vec, w->n_codebooks, w->n_entries, J, tile_n, tile_j, tiles_k); \
    } while (0)
    if (w->code_bits == 8) {
        if (w->v == 8) VQ_DQ(uint8_t, 8); else VQ_DQ(uint8_t, 4);
    } else if (w->code_bits == 12) {
        if (w->v == 8) VQ_DQ(Code12, 8); else VQ_DQ(Code12, 4);
    } else {
        if (w->v == 8) VQ_DQ(uint16_t, 8); else VQ_DQ(uint16_t, 4);
    }
#undef VQ_DQ
    return launch_status();
}

// One thread per (b, h, t, p): copies entry k/v_codebooks[h][g(p)][code] verbatim.
__global__ __launch_bounds__(256) void kv_dequant_kernel(const uint8_t *__restrict__ codes,
                                                         const uint16_t *__restrict__ cb,
                                                         uint16_t *__restrict__ out, long n_vec, int H, int T,
                                                         int P, int v, int E, int G) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long stride = (long)gridDim.x * blockDim.x;
    for (; i < n_vec; i += stride) {
        int p = (int)(i % P);
        long bht = i / P;
        int h = (int)((bht / T) % H);
        int g = (int)(((long)p * G) / P);
        const uint16_t *e = cb + (((size_t)h * G + g) * E + codes[i]) * v;
        for (int k = 0; k < v; ++k) out[i * v + k] = e[k];
    }
}

int launch_kv_dequant(const vq_kv_t *kv, int which, void *out, hipStream_t s) {
    int P = kv->D / kv->v;
    long n_vec = (long)kv->B * kv->H * kv->T * P;
    int blocks = (int)((n_vec + 255) / 256 < 65536 ? (n_vec + 255) / 256 : 65536);
    kv_dequant_kernel<<<blocks, 256, 0, s>>>((const uint8_t *)(which ? kv->v_codes : kv->k_codes),
                                             (const uint16_t *)(which ? kv->v_codebooks : kv->k_codebooks),
                                             (uint16_t *)out, n_vec, kv->H, kv->T, P, kv->v, kv->n_entries,
                                             kv->cb_groups);
    return launch_status();
}

// ---- measurement probes: 128-bit streaming copy / read-reduce -------------------------------

__global__ __launch_bounds__(256) void probe_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src,
                                                         size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}

// A contiguous chunk per workgroup, eight independent non-temporal 16-byte loads in flight per thread: the
// fastest plain read of a large buffer found on this chip (grid-stride order and ordinary loads are 10 - 15 %
// slower).
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4 *__restrict__ src, size_t n16,
                                                         uint4 *__restrict__ sink) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    constexpr int U = 8;
    const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t begin = (size_t)blockIdx.x * per_wg, end = begin + per_wg < n16 ? begin + per_wg : n16;
    const u32x4_t *p = reinterpret_cast<const u32x4_t *>(src);
    u32x4_t a = {0, 0, 0, 0};
    size_t i = begin + threadIdx.x;
    for (; i + (U - 1) * 256 < end; i += U * 256) {
        u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
        for (int u = 0; u < U; ++u) a ^= v[u];
    }
    for (; i < end; i += 256) a ^= __builtin_nontemporal_load(p + i);
    // fold the block into one value so the loads cannot be removed
    __shared__ uint4 red[256];
    red[threadIdx.x] = make_uint4(a.x, a.y, a.z, a.w);
    __syncthreads();
    if (threadIdx.x == 0) {
        uint4 t = make_uint4(0, 0, 0, 0);
        for (int k = 0; k < 256; ++k) { t.x ^= red[k].x; t.y ^= red[k].y; t.z ^= red[k].z; t.w ^= red[k].w; }
        sink[blockIdx.x] = t;
    }
}

// Register-resident matrix-core loop: 8 independent 32x32x16 fp16 MFMA accumulator chains per wavefront,
// no memory traffic.  What the fp16 matrix cores sustain on this chip, for the second roofline fraction.
// RANDOM: four operand pairs of pseudo-random halves in [-1, 1) per lane, taken in turn, as in a gemm on
// real data; the smooth operands of the other form (one pair, values that barely differ between lanes)
// toggle far fewer bits, and the chip clocks higher on them.
template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float *sink) {
    float16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    constexpr int P = RANDOM ? 4 : 1;
    half8_t a[P], b[P];
    uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (RANDOM) {
                h = h * 1664525u + 1013904223u;
                a[p][i] = (half_t)(((int)(h >> 16) - 32768) * (1.f / 32768.f));
                h = h * 1664525u + 1013904223u;
                b[p][i] = (half_t)(((int)(h >> 16) - 32768) * (1.f / 32768.f));
            } else {
                a[p][i] = (half_t)(threadIdx.x * 0.001f);
                b[p][i] = (half_t)(i * 0.01f);
            }
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i % P], b[(i / 2) % P], acc[i], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += acc[i][0];
    if (t == 12345.f) sink[0] = t;  // keeps the loop alive; practically never stores
}

// The same eight MFMAs per iteration, but fed the way a gemm feeds them: six fresh operands (four of one
// matrix, two of the other) read from LDS for every iteration, random halves in [-1, 1).  32 KiB of LDS per
// workgroup, so four workgroups (16 wavefronts) share a CU and cover each other's LDS latency.  No global
// memory traffic.  This is what the matrix cores sustain on operands that change with every instruction.
__global__ __launch_bounds__(256) void probe_mfma_lds_kernel(int iters, float *sink) {
    __shared__ __align__(16) half_t pool[16384];
    uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 977u;
    for (int i = threadIdx.x; i < 16384; i += 256) {
        h = h * 1664525u + 1013904223u;
        pool[i] = (half_t)(((int)(h >> 16) - 32768) * (1.f / 32768.f));
    }
    __syncthreads();
    float16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    const unsigned char *base = reinterpret_cast<const unsigned char *>(pool) + (threadIdx.x & 63) * 16;
    unsigned off = (threadIdx.x >> 6) * 6144u;
    for (int it = 0; it < iters; ++it) {
        half8_t op[6];
#pragma unroll
        for (int q = 0; q < 6; ++q)  // a wave-wide read of 1 KiB of consecutive bytes: no bank conflicts
            op[q] = *reinterpret_cast<const half8_t *>(base + ((off + q * 1024u) & 0x7C00u));
        off += 6144u;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(op[4 + (i & 1)], op[i >> 1], acc[i], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += acc[i][0];
    if (t == 12345.f) sink[0] = t;  // keeps the loop alive; practically never stores
}

int launch_probe_mfma(int workgroups, int iters, int random_operands, void *sink, hipStream_t s) {
    if (random_operands == 2)
        probe_mfma_lds_kernel<<<workgroups, 256, 0, s>>>(iters, (float *)sink);
    else if (random_operands)
        probe_mfma_kernel<true><<<workgroups, 256, 0, s>>>(iters, (float *)sink);
    else
        probe_mfma_kernel<false><<<workgroups, 256, 0, s>>>(iters, (float *)sink);
    return launch_status();
}

int launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t s) {
    size_t n16 = bytes / 16;
    int blocks = (int)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
    probe_copy_kernel<<<blocks, 256, 0, s>>>((uint4 *)dst, (const uint4 *)src, n16);
    return launch_status();
}

int launch_probe_read(const void *src, size_t bytes, void *sink, hipStream_t s) {
    size_t n16 = bytes / 16;
    int blocks = (int)((n16 + 2047) / 2048 < 512 ? (n16 + 2047) / 2048 : 512);   // (the sink holds one value per block)
    if (blocks < 1) blocks = 1;
    probe_read_kernel<<<blocks, 256, 0, s>>>((const uint4 *)src, n16, (uint4 *)sink);
    return launch_status();
}

}  // namespace vq
