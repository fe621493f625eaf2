// VQ-gemv for gfx950: y[m][n] = scale[n] * sum_k W[n][k] x[m][k] with W held as VQ codes.
// Operation: VQ-LLM (arXiv 2503.02236) Sec. III-C "VQ-gemv", dequantization of Sec. II-A
// fused into the product (Alg. 2: load codebook, access entries, compute, reduce).
//
// Mapping (wave64): a wavefront owns a contiguous K-range of 64 "chunks" (one 128-bit code
// load per lane) and walks over rows; the activation fragment of its K-range stays in
// registers for all rows.  Each lane dequantizes whole sub-vectors, so the dequantized
// layout is already the layout the dot product wants: no cross-lane exchange before the
// reduction (the register-level fusion of Sec. VI-B needs zero shuffles here).  The
// reduction axis K is split over the wavefronts of a workgroup and reduced through LDS in
// a fixed order (the "global reduction" of Sec. VI-A kept inside one workgroup).
#include "vq_common.h"

namespace vq {

struct GemvArgs {
    const void *codes;
    const half_t *cb;
    const half_t *scale;
    const half_t *x;
    half_t *y;
    int N, K, E;
    int bs;      // tokens in this pass (<= BS)
    int CH;      // 16-byte code chunks per row
    int KR;      // wavefronts along K (each covers 64 chunks)
    int RW;      // wavefronts along rows
    int n_rg;    // row groups of RW * U rows
};

// rows in flight per wavefront: fewer when several tokens share the register file
constexpr int gemv_rows_in_flight(int bs) { return bs >= 4 ? 2 : 4; }

template <typename CodeT, int V, int R, bool LDSCB, int BS>
__global__ __launch_bounds__(256) void gemv_rows_kernel(GemvArgs a) {
    constexpr int CBY = sizeof(CodeT);
    constexpr int VPC = 16 / (CBY * R);  // sub-vectors per 16-byte chunk
    constexpr int KPC = VPC * V;         // input features per chunk
    constexpr int U = gemv_rows_in_flight(BS);
    static_assert(16 % (CBY * R) == 0, "chunk must hold whole code tuples");

    extern __shared__ __align__(16) unsigned char smem[];
    half_t *cb_lds = reinterpret_cast<half_t *>(smem);
    float *part = reinterpret_cast<float *>(smem + (LDSCB ? (size_t)R * a.E * V * sizeof(half_t) : 0));

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int kr = wave % a.KR, rw = wave / a.KR;
    const int c = kr * 64 + lane;
    const bool active = c < a.CH;
    const int rows_wg = a.RW * U;

    if (LDSCB) {  // whole codebook(s) into LDS, 128-bit copies
        const int n16 = R * a.E * V / 8;
        for (int i = threadIdx.x; i < n16; i += blockDim.x)
            reinterpret_cast<uint4 *>(cb_lds)[i] = reinterpret_cast<const uint4 *>(a.cb)[i];
    }

    // activation fragment of this lane's chunk, all tokens of the pass
    half2_t xf[BS][KPC / 2];
#pragma unroll
    for (int t = 0; t < BS; ++t) {
#pragma unroll
        for (int i = 0; i < KPC / 8; ++i) {
            V16 xv;
            xv.u = make_uint4(0, 0, 0, 0);
            if (active && t < a.bs) xv = ld16(a.x + (size_t)t * a.K + (size_t)c * KPC + i * 8);
#pragma unroll
            for (int p = 0; p < 4; ++p) xf[t][i * 4 + p] = xv.h2[p];
        }
    }
    if (LDSCB) __syncthreads();

    const half_t *cbase = LDSCB ? cb_lds : a.cb;

    for (int rg = blockIdx.x; rg < a.n_rg; rg += gridDim.x) {
        const int row0 = rg * rows_wg + rw * U;
        if (R > 1) {
            // keep the packed fp16 activations opaque per iteration, so their fp32 conversions are
            // not hoisted out of the row loop (that would double the live registers)
#pragma unroll
            for (int t = 0; t < BS; ++t)
#pragma unroll
                for (int i = 0; i < KPC / 2; ++i) asm volatile("" : "+v"(xf[t][i]));
        }
        float acc[U][BS];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < BS; ++t) acc[u][t] = 0.f;

        if (active) {
            V16 cd[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int row = row0 + u;
                row = row < a.N ? row : a.N - 1;  // clamp: rows past the end are computed and dropped
                cd[u] = ld16(reinterpret_cast<const unsigned char *>(a.codes) + ((size_t)row * a.CH + c) * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int i = 0; i < VPC; ++i) {
                    if (R == 1) {
                        unsigned code = (CBY == 1) ? cd[u].b[i] : cd[u].h[i];
                        half2_t e[V / 2];
                        if (V == 8) {
                            V16 ev = ld16(cbase + (size_t)code * 8);
#pragma unroll
                            for (int p = 0; p < 4; ++p) e[p] = ev.h2[p];
                        } else {
                            V8 ev = ld8(cbase + (size_t)code * 4);
#pragma unroll
                            for (int p = 0; p < V / 2; ++p) e[p] = ev.h2[p];
                        }
#pragma unroll
                        for (int t = 0; t < BS; ++t)
#pragma unroll
                            for (int p = 0; p < V / 2; ++p) acc[u][t] = dot2(e[p], xf[t][i * (V / 2) + p], acc[u][t]);
                    } else {
                        float wv[V];
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            unsigned code = (CBY == 1) ? cd[u].b[i * R + r] : cd[u].h[i * R + r];
                            const half_t *ep = cbase + ((size_t)r * a.E + code) * V;
                            half_t eh[V];
                            if (V == 8) {
                                V16 ev = ld16(ep);
#pragma unroll
                                for (int k = 0; k < 8; ++k) eh[k] = ev.h8[k];
                            } else {
                                V8 ev = ld8(ep);
#pragma unroll
                                for (int k = 0; k < 4; ++k) eh[k] = ev.h4[k];
                            }
#pragma unroll
                            for (int k = 0; k < V; ++k) wv[k] = (r == 0) ? (float)eh[k] : wv[k] + (float)eh[k];
                        }
#pragma unroll
                        for (int t = 0; t < BS; ++t)
#pragma unroll
                            for (int k = 0; k < V; ++k)
                                acc[u][t] += wv[k] * (float)xf[t][(i * V + k) / 2][(i * V + k) & 1];
                    }
                }
            }
        }

        // wavefront reduction, then fixed-order reduction over the K-range wavefronts
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < BS; ++t) acc[u][t] = wave_sum(acc[u][t]);

        if (a.KR == 1) {
            if (lane == 0) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    int row = row0 + u;
                    if (row < a.N) {
                        float s = a.scale ? (float)a.scale[row] : 1.f;
#pragma unroll
                        for (int t = 0; t < BS; ++t)
                            if (t < a.bs) a.y[(size_t)t * a.N + row] = (half_t)(acc[u][t] * s);
                    }
                }
            }
        } else {
            __syncthreads();  // previous round's readers are done
            if (lane == 0) {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int t = 0; t < BS; ++t) part[((kr * a.RW + rw) * U + u) * BS + t] = acc[u][t];
            }
            __syncthreads();
            int idx = threadIdx.x;
            if (idx < rows_wg * BS) {
                int t = idx % BS, ru = idx / BS;  // ru = rw * U + u
                int row = rg * rows_wg + ru;
                float s = 0.f;
                for (int k2 = 0; k2 < a.KR; ++k2) s += part[(k2 * rows_wg + ru) * BS + t];
                if (row < a.N && t < a.bs) {
                    float sc = a.scale ? (float)a.scale[row] : 1.f;
                    a.y[(size_t)t * a.N + row] = (half_t)(s * sc);
                }
            }
        }
    }
}

// Any shape with K % v == 0: one wavefront per row, lanes stride over sub-vectors.
template <typename CodeT, int V>
__global__ __launch_bounds__(256) void gemv_generic_kernel(const CodeT *__restrict__ codes,
                                                           const half_t *__restrict__ cb,
                                                           const half_t *__restrict__ scale,
                                                           const half_t *__restrict__ x, half_t *__restrict__ y,
                                                           int N, int K, int E, int R, int bs) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    if (row >= N) return;
    const int J = K / V;
    float acc[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) acc[t] = 0.f;
    for (int j = lane; j < J; j += 64) {
        float wv[V];
        for (int r = 0; r < R; ++r) {
            unsigned code = codes[((size_t)row * J + j) * R + r];
            const half_t *ep = cb + ((size_t)r * E + code) * V;
#pragma unroll
            for (int k = 0; k < V; ++k) wv[k] = (r == 0) ? (float)ep[k] : wv[k] + (float)ep[k];
        }
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            if (t < bs) {
                const half_t *xp = x + (size_t)t * K + (size_t)j * V;
#pragma unroll
                for (int k = 0; k < V; ++k) acc[t] += wv[k] * (float)xp[k];
            }
        }
    }
    float s = scale ? (float)scale[row] : 1.f;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        if (t < bs) {
            float v = wave_sum(acc[t]);
            if (lane == 0) y[(size_t)t * N + row] = (half_t)(v * s);
        }
    }
}

__global__ void fill_zero_kernel(half_t *p, long n) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (half_t)0.f;
}

size_t gemv_workspace(const vq_weight_t *w, int bs) { return gemv_uses_pack(w, bs) ? gemv_packed_workspace(w) : 0; }

namespace {

template <typename CodeT, int V, int R, bool LDSCB, int BS>
int run_rows(const vq_weight_t *w, const half_t *x, int bs, half_t *y, hipStream_t s) {
    constexpr int KPC = (16 / ((int)sizeof(CodeT) * R)) * V;
    GemvArgs a;
    a.codes = w->codes;
    a.cb = (const half_t *)w->codebooks;
    a.scale = (const half_t *)w->scale;
    a.N = w->N;
    a.K = w->K;
    a.E = w->n_entries;
    a.CH = w->K / KPC;
    a.KR = (a.CH + 63) / 64;
    a.RW = 4 / a.KR;
    const int rows_wg = a.RW * gemv_rows_in_flight(BS);
    a.n_rg = (w->N + rows_wg - 1) / rows_wg;
    size_t lds = (LDSCB ? (size_t)R * a.E * V * sizeof(half_t) : 0) + (size_t)a.KR * rows_wg * BS * sizeof(float);
    int grid = a.n_rg < 512 ? a.n_rg : 512;  // persistent workgroups amortize the x / codebook staging
    for (int t0 = 0; t0 < bs; t0 += BS) {
        a.x = x + (size_t)t0 * w->K;
        a.y = y + (size_t)t0 * w->N;
        a.bs = bs - t0 < BS ? bs - t0 : BS;
        gemv_rows_kernel<CodeT, V, R, LDSCB, BS><<<grid, 64 * a.KR * a.RW, lds, s>>>(a);
    }
    return launch_status();
}

template <typename CodeT, int V, int R, bool LDSCB>
int run_rows_bs(const vq_weight_t *w, const half_t *x, int bs, half_t *y, hipStream_t s) {
    constexpr int KPC = (16 / ((int)sizeof(CodeT) * R)) * V;
    constexpr int BSMAX = KPC >= 128 ? 2 : 4;  // keeps the activation fragment within 128 registers
    if (bs == 1) return run_rows<CodeT, V, R, LDSCB, 1>(w, x, bs, y, s);
    if (bs == 2 || BSMAX == 2) return run_rows<CodeT, V, R, LDSCB, 2>(w, x, bs, y, s);
    return run_rows<CodeT, V, R, LDSCB, BSMAX>(w, x, bs, y, s);
}

template <typename CodeT, int V, int R>
int run_rows_cb(const vq_weight_t *w, const half_t *x, int bs, half_t *y, hipStream_t s) {
    size_t cb_bytes = (size_t)R * w->n_entries * V * sizeof(half_t);
    if (cb_bytes <= 64 * 1024 && (R * w->n_entries * V) % 8 == 0) return run_rows_bs<CodeT, V, R, true>(w, x, bs, y, s);
    return run_rows_bs<CodeT, V, R, false>(w, x, bs, y, s);
}

}  // namespace

template <typename CodeT, int V>
static int run_generic(const vq_weight_t *w, const half_t *x, int bs, half_t *y, hipStream_t s) {
    gemv_generic_kernel<CodeT, V><<<(w->N + 3) / 4, 256, 0, s>>>((const CodeT *)w->codes, (const half_t *)w->codebooks,
                                                                (const half_t *)w->scale, x, y, w->N, w->K,
                                                                w->n_entries, w->n_codebooks, bs);
    return launch_status();
}

int launch_gemv_generic(const vq_weight_t *w, const void *x, int bs, void *y, hipStream_t s) {
    const half_t *xp = (const half_t *)x;
    half_t *yp = (half_t *)y;
    if (w->code_bits == 8) return w->v == 8 ? run_generic<uint8_t, 8>(w, xp, bs, yp, s) : run_generic<uint8_t, 4>(w, xp, bs, yp, s);
    return w->v == 8 ? run_generic<uint16_t, 8>(w, xp, bs, yp, s) : run_generic<uint16_t, 4>(w, xp, bs, yp, s);
}

namespace {

template <typename CodeT, int V>
int dispatch(const vq_weight_t *w, const half_t *x, int bs, half_t *y, hipStream_t s) {
    const int R = w->n_codebooks;
    const int cby = (int)sizeof(CodeT);
    bool fast = (R == 1 || R == 2) && (16 % (cby * R) == 0);
    if (fast) {
        int KPC = (16 / (cby * R)) * V;
        int CH = w->K / KPC;
        fast = (w->K % KPC == 0) && CH >= 1 && CH <= 256;
    }
    if (!fast) return run_generic<CodeT, V>(w, x, bs, y, s);
    if (R == 1) return run_rows_cb<CodeT, V, 1>(w, x, bs, y, s);
    return run_rows_cb<CodeT, V, 2>(w, x, bs, y, s);
}

}  // namespace

int launch_gemv(const vq_weight_t *w, const void *x, int bs, void *y, void *ws, hipStream_t s) {
    if (gemv_uses_pack(w, bs) && w->K > 0) return launch_gemv_packed(w, x, y, ws, s);
    return launch_gemv_rows(w, x, bs, y, s);
}

// From the canonical code layout (any batch size 1..16).
int launch_gemv_rows(const vq_weight_t *w, const void *x, int bs, void *y, hipStream_t s) {
    const half_t *xp = (const half_t *)x;
    half_t *yp = (half_t *)y;
    if (w->K == 0) {  // empty reduction: y = 0 (a fill kernel, so the call can be graph-captured)
        long n = (long)bs * w->N;
        fill_zero_kernel<<<(int)((n + 255) / 256), 256, 0, s>>>(yp, n);
        return launch_status();
    }
    if (gemv_mfma_supported(w)) return launch_gemv_mfma(w, x, bs, y, s);  // codebooks in LDS, matrix cores
    if (w->cb_tile_n > 0 || w->code_bits == 12) return VQ_ERR_UNSUPPORTED;  // those formats exist on that path only
    if (w->code_bits == 8) return w->v == 8 ? dispatch<uint8_t, 8>(w, xp, bs, yp, s) : dispatch<uint8_t, 4>(w, xp, bs, yp, s);
    return w->v == 8 ? dispatch<uint16_t, 8>(w, xp, bs, yp, s) : dispatch<uint16_t, 4>(w, xp, bs, yp, s);
}

}  // namespace vq
