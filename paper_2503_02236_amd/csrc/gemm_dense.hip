// Second stage of the prefill VQ-gemm when M is large: Y = X * Wd^T with Wd the fp16
// dequantized weight (written once per call into the workspace by the dequantization
// kernel), on v_mfma_f32_32x32x16_f16 with fp32 accumulation.
//
// Why two stages (VQ-LLM, arXiv 2503.02236, Sec. VII-B notes that dequantization hurts the
// compute-bound GeMM most): with a 2^16-entry codebook every dequantized 16-byte operand is a
// random gather from L2, and MI355X sustains only ~0.44 such gathers per clock per CU.  A
// fused 256-row tile needs one gather per lane per 8 MFMAs (1 per clock per CU), so fusing
// caps the matrix cores at ~44 %; every extra M tile repeats the gathers.  Dequantizing once
// (N*K/v gathers in total) and streaming the fp16 tile through LDS keeps the main loop free
// of gathers.  The fp16 tile this kernel consumes is exactly the bit-exact tile of vq_dequant.
//
// Tile: BM x BN = 256 x 128 per workgroup (256 tiles for M = 2048, N = 4096: one per CU),
// four wavefronts 2 x 2, each 128 x 64 = 4 x 2 MFMA tiles.  K in blocks of 64; both operands
// are K-contiguous, so a lane's MFMA operand (8 consecutive k) is one 128-bit LDS read.
//
// Data movement: global -> LDS directly (global_load_lds_dwordx4, no registers), three LDS
// stages, so the loads of K block kt+2 are in flight while block kt is multiplied.  The direct
// load writes lane l's 16 bytes at (base + 16 l), so a wavefront fills 8 tile rows of 128
// bytes; bank conflicts of the operand reads are avoided by a XOR swizzle of the 16-byte
// segment index with the row (each lane fetches the segment that belongs in its slot).
// Operand reads of MFMA step s+1 are issued before the MFMAs of step s.
//
// Measured limits of this design on MI355X (M = 2048, N = K = 4096): the MFMA + LDS-read loop alone runs
// in ~44 us, the loads alone in ~55 us, together 78 us (35 % of the fp16 peak).  The loads are the floor:
// a 256 x 128 tile moves 48 KiB per K block into LDS, and the L2 -> LDS path of one CU sustains only
// ~27 bytes per clock here, whether the operands come from memory or sit in L2 (pointing every tile at the
// same 3 MiB gives the same time; touching lines in L2 ahead of time makes it slower).  A larger tile would
// halve the traffic per flop but leaves half of the 256 CUs without a tile at this problem size.
#include "vq_common.h"

namespace vq {

constexpr int kDenseBK = 64;      // K per stage
constexpr int kDenseStages = 3;   // LDS ring
constexpr int kDenseRowB = 128;   // bytes per tile row in LDS (64 halves, unpadded)

struct DenseArgs {
    const half_t *A;      // [M][K]
    const half_t *B;      // [N][K] dequantized weight
    const half_t *scale;  // [N] or null
    half_t *C;            // [M][N]
    int M, N, K;
    int tiles_m, tiles_n;
};

// 16-byte segment swizzle: any 8 consecutive rows, and the rows of equal parity among any aligned
// 16, get distinct values
__device__ __forceinline__ int dense_swz(int row) { return (row ^ (row >> 3)) & 7; }

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void global_void_t;

template <int MT, int NT>
__global__ __launch_bounds__(256) void gemm_dense_kernel(DenseArgs a) {
    constexpr int BM = 64 * MT, BN = 64 * NT;
    constexpr int kStage = (BM + BN) * kDenseRowB;
    constexpr int A_LOADS = BM / 32;  // wave-wide 1 KiB loads per wavefront per stage (8 rows each)
    constexpr int B_LOADS = BN / 32;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int ln = lane & 31, lh = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    // workgroups are dealt round-robin to the 8 compute dies: give each die a contiguous run of
    // tiles (column-major: same weight columns, walking over M); all tiles walk K in the same order,
    // so the workgroups of a die ask for the same operand blocks at about the same time and share
    // them in its L2 (starting each tile at its own K block was measured slower)
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

    // global source of this lane for each of its wave-wide loads: tile row = chunk row + lane / 8,
    // logical segment = slot ^ swizzle(row).  Rows past the end are clamped (never stored).
    const half_t *asrc[A_LOADS];
    const half_t *bsrc[B_LOADS];
#pragma unroll
    for (int p = 0; p < A_LOADS; ++p) {
        const int r = wave * (BM / 4) + p * 8 + (lane >> 3);
        const int seg = (lane & 7) ^ dense_swz(r);
        const int m = min(m0 + r, a.M - 1);
        asrc[p] = a.A + (size_t)m * a.K + seg * 8;
    }
#pragma unroll
    for (int p = 0; p < B_LOADS; ++p) {
        const int r = wave * (BN / 4) + p * 8 + (lane >> 3);
        const int seg = (lane & 7) ^ dense_swz(r);
        const int n = min(n0 + r, a.N - 1);
        bsrc[p] = a.B + (size_t)n * a.K + seg * 8;
    }
    auto issue_stage = [&](int kt, int buf) {
        unsigned char *ab = smem + (size_t)buf * kStage + (size_t)wave * (BM / 4) * kDenseRowB;
        unsigned char *bb = smem + (size_t)buf * kStage + BM * kDenseRowB + (size_t)wave * (BN / 4) * kDenseRowB;
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p)
            __builtin_amdgcn_global_load_lds((global_void_t *)(asrc[p] + (size_t)kt * kDenseBK),
                                             (lds_void_t *)(ab + p * 1024), 16, 0, 0);
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p)
            __builtin_amdgcn_global_load_lds((global_void_t *)(bsrc[p] + (size_t)kt * kDenseBK),
                                             (lds_void_t *)(bb + p * 1024), 16, 0, 0);
    };

    // operand rows of this lane inside a stage; 32 rows further down the swizzle has bit 2 flipped
    const int a_row = wm * 32 * MT + ln, b_row = wn * 32 * NT + ln;
    const int a_swz = dense_swz(a_row), b_swz = dense_swz(b_row);

    const int KT = a.K / kDenseBK;
    issue_stage(0, 0);
    if (KT > 1) issue_stage(1, 1);

    int buf = 0;
    for (int kt = 0; kt < KT; ++kt) {
        // stage kt has landed (the newer stage may still be in flight); after the barrier every
        // wavefront is also done with stage kt-1, whose buffer the next loads overwrite
        if (kt + 1 < KT)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(A_LOADS + B_LOADS) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (kt + 2 < KT) issue_stage(kt + 2, buf >= 1 ? buf - 1 : kDenseStages - 1);

        const unsigned char *ab = smem + (size_t)buf * kStage + (size_t)a_row * kDenseRowB;
        const unsigned char *bb = smem + (size_t)buf * kStage + BM * kDenseRowB + (size_t)b_row * kDenseRowB;
        half8_t af[2][MT], bf[2][NT];
        auto read_frags = [&](int s, int slot) {
            const int ao = (((2 * s + lh) ^ a_swz) << 4), bo = (((2 * s + lh) ^ b_swz) << 4);
#pragma unroll
            for (int i = 0; i < MT; ++i)
                af[slot][i] = *reinterpret_cast<const half8_t *>(ab + i * 32 * kDenseRowB + (ao ^ ((i & 1) << 6)));
#pragma unroll
            for (int j = 0; j < NT; ++j)
                bf[slot][j] = *reinterpret_cast<const half8_t *>(bb + j * 32 * kDenseRowB + (bo ^ ((j & 1) << 6)));
        };
        read_frags(0, 0);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s < 3) read_frags(s + 1, (s + 1) & 1);
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[s & 1][i], bf[s & 1][j], acc[i][j], 0, 0, 0);
        }
        // instruction order for the block above (the compiler would otherwise sink every LDS read to
        // just before its first use): the reads of step 0, then per step one LDS read of the next
        // step's operands between consecutive MFMAs of the current one
        __builtin_amdgcn_sched_group_barrier(0x100, MT + NT, 0);
#pragma unroll
        for (int s = 0; s < 3; ++s) {
#pragma unroll
            for (int q = 0; q < MT + NT; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, MT * NT - (MT + NT), 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MT * NT, 0);
        buf = buf + 1 == kDenseStages ? 0 : buf + 1;
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
    const size_t lds = (size_t)kDenseStages * (BM + BN) * kDenseRowB;
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
