// Second stage of the prefill VQ-gemm when M is large: Y = X * Wd^T with Wd the fp16
// dequantized weight (written once per call into the workspace by the dequantization
// kernel), on v_mfma_f32_32x32x16_f16 with fp32 accumulation.
//
// Why two stages (VQ-LLM, arXiv 2503.02236, Sec. VII-B notes that dequantization hurts the
// compute-bound GeMM most): with a 2^16-entry codebook every dequantized 16-byte operand is a
// random gather from L2, and MI355X sustains only ~0.44 such gathers per clock per CU.  A
// fused 256-row tile needs one gather per lane per 8 MFMAs (1 per clock per CU), so fusing
// caps the matrix cores at ~44 %; every extra M tile repeats the gathers.  Dequantizing once
// (N*K/v gathers in total, ~8 us for 4096 x 4096) and streaming the fp16 tile through LDS
// keeps the main loop free of gathers.  The fp16 tile this kernel consumes is exactly the
// bit-exact tile of vq_dequant.
//
// Tile: BM x BN = 256 x 128 per workgroup (256 tiles for M = 2048, N = 4096: one per CU),
// four wavefronts 2 x 2, each 128 x 64 = 4 x 2 MFMA tiles.  K in blocks of 64, both operands
// K-contiguous, so a lane's MFMA operand (8 consecutive k) is one 128-bit LDS read.
// LDS rows are padded by 16 bytes: 128-bit reads of 8 consecutive rows then hit 8 distinct
// bank groups.  Double-buffered LDS, next block prefetched into registers during the MFMAs.
#include "vq_common.h"

namespace vq {

constexpr int kDenseBK = 64;
constexpr int kDenseRow = kDenseBK * 2 + 16;  // bytes per tile row in LDS

struct DenseArgs {
    const half_t *A;      // [M][K]
    const half_t *B;      // [N][K] dequantized weight
    const half_t *scale;  // [N] or null
    half_t *C;            // [M][N]
    int M, N, K;
    int tiles_m, tiles_n;
};

template <int MT, int NT>
__global__ __launch_bounds__(256) void gemm_dense_kernel(DenseArgs a) {
    constexpr int BM = 64 * MT, BN = 64 * NT;
    constexpr int AP = BM / 32, BP = BN / 32;  // 16-byte loads per thread per K block
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int kStage = (BM + BN) * kDenseRow;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int ln = lane & 31, lh = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    // workgroups are dealt round-robin to the 8 compute dies: give each die a contiguous run of
    // tiles (column-major: same weight columns, walking over M) so that its L2 sees each weight
    // block once per few tiles
    const int n_tiles = a.tiles_m * a.tiles_n;
    const int per_die = (n_tiles + 7) / 8;
    const int t = (blockIdx.x & 7) * per_die + (blockIdx.x >> 3);
    if (t >= n_tiles) return;
    const int tile_n = t / a.tiles_m, tile_m = t % a.tiles_m;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    float16_t acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int s_row = tid >> 3, s_seg = tid & 7;
    uint4 areg[AP], breg[BP];
    auto load_tiles = [&](int kt) {
#pragma unroll
        for (int p = 0; p < AP; ++p) {
            int m = m0 + s_row + 32 * p;
            areg[p] = m < a.M ? *reinterpret_cast<const uint4 *>(a.A + (size_t)m * a.K + (size_t)kt * kDenseBK + s_seg * 8)
                              : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int p = 0; p < BP; ++p) {
            int n = n0 + s_row + 32 * p;
            breg[p] = n < a.N ? *reinterpret_cast<const uint4 *>(a.B + (size_t)n * a.K + (size_t)kt * kDenseBK + s_seg * 8)
                              : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_tiles = [&](int buf) {
        unsigned char *ab = smem + (size_t)buf * kStage;
        unsigned char *bb = ab + BM * kDenseRow;
#pragma unroll
        for (int p = 0; p < AP; ++p)
            *reinterpret_cast<uint4 *>(ab + (size_t)(s_row + 32 * p) * kDenseRow + s_seg * 16) = areg[p];
#pragma unroll
        for (int p = 0; p < BP; ++p)
            *reinterpret_cast<uint4 *>(bb + (size_t)(s_row + 32 * p) * kDenseRow + s_seg * 16) = breg[p];
    };

    // All tiles walk K in the same order: workgroups of a die then ask for the same operand blocks at
    // about the same time and share them in its L2 (starting each tile at its own K block was slower).
    const int KT = a.K / kDenseBK;
    auto kblock = [&](int i) { return i; };
    load_tiles(kblock(0));
    store_tiles(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_tiles(kblock(kt + 1));
        const unsigned char *ab = smem + (size_t)buf * kStage + (size_t)(wm * 32 * MT + ln) * kDenseRow + lh * 16;
        const unsigned char *bb = smem + (size_t)buf * kStage + BM * kDenseRow + (size_t)(wn * 32 * NT + ln) * kDenseRow + lh * 16;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            half8_t af[MT], bf[NT];
#pragma unroll
            for (int i = 0; i < MT; ++i) af[i] = *reinterpret_cast<const half8_t *>(ab + (size_t)i * 32 * kDenseRow + s * 32);
#pragma unroll
            for (int j = 0; j < NT; ++j) bf[j] = *reinterpret_cast<const half8_t *>(bb + (size_t)j * 32 * kDenseRow + s * 32);
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // epilogue: accumulator register r of lane (ln, lh) is row 8*(r/4) + 4*lh + r%4, column ln
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int n = n0 + wn * 32 * NT + j * 32 + ln;
        if (n >= a.N) continue;
        const float sc = a.scale ? (float)a.scale[n] : 1.f;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 32 * MT + i * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (m < a.M) a.C[(size_t)m * a.N + n] = (half_t)(acc[i][j][r] * sc);
            }
        }
    }
}

int launch_gemm_dense(const half_t *A, const half_t *B, const half_t *scale, half_t *C, int M, int N, int K,
                      hipStream_t s) {
    constexpr int MT = 4, NT = 2;
    constexpr int BM = 64 * MT, BN = 64 * NT;
    DenseArgs a;
    a.A = A;
    a.B = B;
    a.scale = scale;
    a.C = C;
    a.M = M;
    a.N = N;
    a.K = K;
    a.tiles_m = (M + BM - 1) / BM;
    a.tiles_n = (N + BN - 1) / BN;
    const size_t lds = 2 * (size_t)(BM + BN) * kDenseRow;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_dense_kernel<MT, NT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const int n_tiles = a.tiles_m * a.tiles_n;
    const int grid = ((n_tiles + 7) / 8) * 8;
    gemm_dense_kernel<MT, NT><<<grid, 256, lds, s>>>(a);
    return launch_status();
}

}  // namespace vq
