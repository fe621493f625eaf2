// VQ-gemm for gfx950: Y[m][n] = scale[n] * sum_k W[n][k] X[m][k], W held as VQ codes,
// contraction on the fp16 matrix cores (v_mfma_f32_32x32x16_f16), fp32 accumulation.
// Operation: VQ-LLM (arXiv 2503.02236) Sec. III-C "VQ-gemm"; dequantization of Sec. II-A
// fused in front of the matrix instruction (Alg. 2).
//
// Layout fusion (Sec. VI-B asks how dequantized data reaches the layout the matrix
// instruction wants).  On gfx950 the B operand of the 32x32x16 fp16 MFMA is, per lane,
// 8 fp16 values consecutive along k for one column n.  With sub-vectors along K, a v = 8
// codebook entry IS one lane's B operand (v = 4: two entries), so each lane gathers its
// operand straight from the codebook into registers: no shuffle and no LDS round trip for
// the weights.  The four wavefronts of a workgroup are laid out 1 x 4 along N so that no two
// of them need the same weight columns, i.e. no entry is gathered twice inside a workgroup.
// X tiles go through LDS (all four wavefronts read the same rows).
//
// k-assignment inside a 64-wide K block q (free, as long as A and B agree): MFMA step s
// (0..3), lane half h (lane / 32) covers sub-vector j = 8q + 4h + s, so a lane uses 4
// consecutive codes (v = 8) per block and loads them with one 64-bit load.
#include "vq_common.h"

namespace vq {

constexpr int kGemmBK = 64;                    // K per main-loop iteration
constexpr int kGemmLdsRow = kGemmBK * 2 + 16;  // bytes per X row in LDS; +16 keeps 128-bit reads conflict-free

struct GemmArgs {
    const void *codes;
    const half_t *cb;
    const half_t *scale;
    const half_t *X;
    half_t *Y;
    int M, N, K, E;
    int tiles_m, tiles_n;
};

// MT x NT MFMA tiles (32 x 32) per wavefront; workgroup tile = (32*MT) x (4*32*NT).
template <int V, int R, int MT, int NT>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs a) {
    constexpr int BM = 32 * MT;
    constexpr int WN = 32 * NT;      // columns per wavefront
    constexpr int BN = 4 * WN;
    constexpr int CPV = 8 / V;       // codes per lane operand (1 or 2)
    constexpr int A_PASSES = BM / 32;  // 256 threads x 16 B cover 32 rows of 128 B

    extern __shared__ __align__(16) unsigned char smem[];  // 2 x BM x kGemmLdsRow

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int ln = lane & 31, lh = lane >> 5;

    // tile order: consecutive workgroups share the weight columns (tile_n) and walk over M
    const int tile_n = blockIdx.x / a.tiles_m, tile_m = blockIdx.x % a.tiles_m;
    const int m0 = tile_m * BM, n0 = tile_n * BN + wave * WN;
    const int J = a.K / V;  // codes per weight row (per residual)

    float16_t acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // global -> register staging of the X tile: thread covers row (tid/8 + 32*p), 16-byte segment tid%8
    const int a_row = tid >> 3, a_seg = tid & 7;
    uint4 areg[A_PASSES];
    auto load_a = [&](int kt) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            int m = m0 + a_row + 32 * p;
            if (m < a.M)
                areg[p] = *reinterpret_cast<const uint4 *>(a.X + (size_t)m * a.K + (size_t)kt * kGemmBK + a_seg * 8);
            else
                areg[p] = make_uint4(0, 0, 0, 0);
        }
    };
    auto store_a = [&](int buf) {
        unsigned char *base = smem + (size_t)buf * BM * kGemmLdsRow;
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p)
            *reinterpret_cast<uint4 *>(base + (size_t)(a_row + 32 * p) * kGemmLdsRow + a_seg * 16) = areg[p];
    };

    // this lane's weight rows (clamped; columns past N are computed and dropped)
    int nrow[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        int n = n0 + j * 32 + ln;
        nrow[j] = n < a.N ? n : a.N - 1;
    }

    const int KT = a.K / kGemmBK;
    load_a(0);
    store_a(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_a(kt + 1);

        // codes of this K block: 4 (v=8) or 8 (v=4) consecutive codes per residual
        // index of first code: (kt*64)/V + 4*h*CPV
        half8_t bfrag[4][NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            if (R == 1) {
                const uint16_t *cp = reinterpret_cast<const uint16_t *>(a.codes);
                unsigned cd[4 * CPV];
                if (CPV == 1) {
                    V8 c8 = ld8(cp + (size_t)nrow[j] * J + (size_t)kt * 8 + 4 * lh);
#pragma unroll
                    for (int s = 0; s < 4; ++s) cd[s] = c8.h[s];
                } else {
                    V16 c16 = ld16(cp + (size_t)nrow[j] * J + (size_t)kt * 16 + 8 * lh);
#pragma unroll
                    for (int s = 0; s < 8; ++s) cd[s] = c16.h[s];
                }
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    if (CPV == 1) {
                        bfrag[s][j] = ld16(a.cb + (size_t)cd[s] * 8).h8;
                    } else {
                        V8 e0 = ld8(a.cb + (size_t)cd[2 * s] * 4), e1 = ld8(a.cb + (size_t)cd[2 * s + 1] * 4);
                        V16 e;
                        e.w[0] = e0.w[0]; e.w[1] = e0.w[1]; e.w[2] = e1.w[0]; e.w[3] = e1.w[1];
                        bfrag[s][j] = e.h8;
                    }
                }
            }
        }

        const unsigned char *abase = smem + (size_t)buf * BM * kGemmLdsRow;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                half8_t af = *reinterpret_cast<const half8_t *>(abase + (size_t)(i * 32 + ln) * kGemmLdsRow +
                                                                (4 * lh + s) * 16);
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bfrag[s][j], acc[i][j], 0, 0, 0);
            }
        }

        if (kt + 1 < KT) store_a(buf ^ 1);
        __syncthreads();
    }

    // epilogue: acc register r of lane (ln, lh) is row 8*(r/4) + 4*lh + r%4, column ln of its 32x32 tile
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        int n = n0 + j * 32 + ln;
        if (n >= a.N) continue;
        float sc = a.scale ? (float)a.scale[n] : 1.f;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int m = m0 + i * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (m < a.M) a.Y[(size_t)m * a.N + n] = (half_t)(acc[i][j][r] * sc);
            }
        }
    }
}

// Large M: dequantize once into the workspace (fp16 [N][K]) and run the dense matrix-core kernel.
// Small M: one M tile would not reuse the dequantized weights, so the fused kernel gathers them directly.
static bool gemm_two_stage(const vq_weight_t *w, int M) { return M > 256 && w->K > 0 && w->K % 64 == 0; }

size_t gemm_workspace(const vq_weight_t *w, int M) {
    return gemm_two_stage(w, M) ? (size_t)w->N * w->K * sizeof(half_t) : 0;
}

namespace {

template <int V, int MT, int NT>
int run_mfma(const vq_weight_t *w, const half_t *X, int M, half_t *Y, hipStream_t s) {
    constexpr int BM = 32 * MT, BN = 128 * NT;
    GemmArgs a;
    a.codes = w->codes;
    a.cb = (const half_t *)w->codebooks;
    a.scale = (const half_t *)w->scale;
    a.X = X;
    a.Y = Y;
    a.M = M;
    a.N = w->N;
    a.K = w->K;
    a.E = w->n_entries;
    a.tiles_m = (M + BM - 1) / BM;
    a.tiles_n = (w->N + BN - 1) / BN;
    size_t lds = 2 * (size_t)BM * kGemmLdsRow;
    static KernelSetup setup;
    if (int st = kernel_setup(reinterpret_cast<const void *>(&gemm_mfma_kernel<V, 1, MT, NT>), lds, false, setup)) return st;
    gemm_mfma_kernel<V, 1, MT, NT><<<a.tiles_m * a.tiles_n, 256, lds, s>>>(a);
    return launch_status();
}

}  // namespace

int launch_gemm(const vq_weight_t *w, const void *X, int M, void *Y, void *ws, hipStream_t s) {
    const half_t *Xp = (const half_t *)X;
    half_t *Yp = (half_t *)Y;
    if (gemm_two_stage(w, M)) {
        int st = launch_dequant(w, ws, /*out_fp32=*/0, s);
        if (st != VQ_OK) return st;
        return launch_gemm_dense(Xp, (const half_t *)ws, (const half_t *)w->scale, Yp, M, w->N, w->K, s);
    }
    // matrix-core path: uint16 codes, one codebook, K a multiple of the 64-wide block
    bool fast = w->cb_tile_n == 0 && w->code_bits == 16 && w->n_codebooks == 1 && w->K % kGemmBK == 0 && w->K > 0 && M >= 32 &&
                ((size_t)w->K / w->v * 2) % 16 == 0;
    if (fast) {
        if (w->v == 8) return run_mfma<8, 8, 2>(w, Xp, M, Yp, s);
        return run_mfma<4, 8, 2>(w, Xp, M, Yp, s);
    }
    // any other configuration: 16 tokens at a time through the generic row kernel
    for (int m = 0; m < M; m += 16) {
        int bs = M - m < 16 ? M - m : 16;
        int st = launch_gemv_rows(w, Xp + (size_t)m * w->K, bs, Yp + (size_t)m * w->N, s);
        if (st != VQ_OK) return st;
    }
    return VQ_OK;
}

}  // namespace vq
