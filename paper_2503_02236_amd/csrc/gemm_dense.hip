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
// stages, so the loads of K blocks kt+1 and kt+2 are in flight while block kt is multiplied.  The direct
// load writes lane l's 16 bytes at (base + 16 l), so a wavefront fills 8 tile rows of 128
// bytes; bank conflicts of the operand reads are avoided by a XOR swizzle of the 16-byte
// segment index with the row (each lane fetches the segment that belongs in its slot).
// Operand reads of MFMA step s+1 are issued between the MFMAs of step s, and so are the loads, one after
// every second MFMA.
//
// Measured on MI355X (M = 2048, N = K = 4096, parts of the main loop timed alone): MFMAs alone 41 us on
// all-zero operands and 55 us on random ones (the chip clocks lower the more operand bits toggle: a
// register-resident MFMA loop sustains 2.05 PFLOP/s on smooth and 1.64 on random operands), with the LDS
// reads the same; the loads alone 33 us; everything together 60 us on random data, 67 us with the
// epilogue.  What mattered on the way there: (1) __syncthreads() waits for every outstanding load, so the
// ring was never more than one stage deep -- a bare s_barrier after a counted wait; (2) twelve loads
// issued as a burst hold up the wavefront's MFMAs behind them (76 us -> 63 us when spread out);
// (3) LDS destinations (M0) from a scalar wavefront index (63 -> 59 us); (4) 16-byte stores of whole lines
// in the epilogue instead of 2-byte stores.  Pointing every tile at the same 3 MiB (all loads hit L2)
// changes nothing: the loop is bound by the matrix cores at the clock the data allows.
#include "vq_common.h"

#include <type_traits>

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
    constexpr int N_LOADS = A_LOADS + B_LOADS;
    static_assert(N_LOADS == 2 * (MT + NT) && MT * NT >= MT + NT, "the main loop issues one load after every second operand read");
    extern __shared__ __align__(16) unsigned char smem[];

    // the wavefront index as a scalar: LDS destinations of the direct loads (M0) then need no vector instructions
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
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
    // load p of a stage: p < A_LOADS is a chunk of the X tile, the rest chunks of the weight tile
    auto issue_load = [&](int kt, int buf, int p) {
        unsigned char *ab = smem + (size_t)buf * kStage + (size_t)wave * (BM / 4) * kDenseRowB;
        unsigned char *bb = smem + (size_t)buf * kStage + BM * kDenseRowB + (size_t)wave * (BN / 4) * kDenseRowB;
        if (p < A_LOADS)
            __builtin_amdgcn_global_load_lds((global_void_t *)(asrc[p] + (size_t)kt * kDenseBK),
                                             (lds_void_t *)(ab + p * 1024), 16, 0, 0);
        else
            __builtin_amdgcn_global_load_lds((global_void_t *)(bsrc[p - A_LOADS] + (size_t)kt * kDenseBK),
                                             (lds_void_t *)(bb + (p - A_LOADS) * 1024), 16, 0, 0);
    };
    auto issue_stage = [&](int kt, int buf) {
#pragma unroll
        for (int p = 0; p < N_LOADS; ++p) issue_load(kt, buf, p);
    };

    // operand rows of this lane inside a stage; 32 rows further down the swizzle has bit 2 flipped
    const int a_row = wm * 32 * MT + ln, b_row = wn * 32 * NT + ln;
    const int a_swz = dense_swz(a_row), b_swz = dense_swz(b_row);

    const int KT = a.K / kDenseBK;
    issue_stage(0, 0);
    if (KT > 1) issue_stage(1, 1);

    // One K block.  MORE: stage kt + 2 exists and is requested while block kt is multiplied.  The loads are
    // spread over the whole block, one after every second MFMA: issued as a burst they hold up the
    // wavefront's MFMAs behind them.
    // The source order of the memory operations below is the intended issue order (direct-to-LDS loads
    // and LDS reads are not reordered against each other by the compiler); the group barriers place the
    // MFMAs between them.
    int buf = 0;
    half8_t af[2][MT], bf[2][NT];
    auto k_block = [&](int kt, auto more_tag) {
        constexpr bool MORE = decltype(more_tag)::value;
        // stage kt has landed (the newer stage may still be in flight); after the barrier every wavefront
        // is also done with stage kt-1, whose buffer the next loads overwrite.  A bare s_barrier:
        // __syncthreads() carries a fence that waits for every outstanding load, the newer stage included.
        if (kt + 1 < KT)
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N_LOADS) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const int lbuf = buf >= 1 ? buf - 1 : kDenseStages - 1;

        const unsigned char *ab = smem + (size_t)buf * kStage + (size_t)a_row * kDenseRowB;
        const unsigned char *bb = smem + (size_t)buf * kStage + BM * kDenseRowB + (size_t)b_row * kDenseRowB;
        // operand q of MFMA step s: q < MT is a row block of X, the rest column blocks of the weight
        auto read_operand = [&](int s, int slot, int q) {
            const int ao = (((2 * s + lh) ^ a_swz) << 4), bo = (((2 * s + lh) ^ b_swz) << 4);
            if (q < MT)
                af[slot][q] = *reinterpret_cast<const half8_t *>(ab + q * 32 * kDenseRowB + (ao ^ ((q & 1) << 6)));
            else
                bf[slot][q - MT] = *reinterpret_cast<const half8_t *>(bb + (q - MT) * 32 * kDenseRowB +
                                                                      (bo ^ (((q - MT) & 1) << 6)));
        };
#pragma unroll
        for (int q = 0; q < MT + NT; ++q) read_operand(0, 0, q);
        __builtin_amdgcn_sched_group_barrier(0x100, MT + NT, 0);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int q = 0; q < MT + NT; ++q) {
                if (s < 3) read_operand(s + 1, (s + 1) & 1, q);
                if (MORE && (q & 1)) issue_load(kt + 2, lbuf, s * (N_LOADS / 4) + q / 2);
            }
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[s & 1][j], af[s & 1][i], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int q = 0; q < MT + NT; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (s < 3) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (MORE && (q & 1)) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, MT * NT - (MT + NT), 0);
        }
        buf = buf + 1 == kDenseStages ? 0 : buf + 1;
    };
    int kt = 0;
    for (; kt + 2 < KT; ++kt) k_block(kt, std::true_type{});
    for (; kt < KT; ++kt) k_block(kt, std::false_type{});

    // Epilogue.  The weight tile is the MFMA's first operand, so an accumulator holds Y^T: lane (ln, lh),
    // register r is output row m = ln, column n = 8 (r / 4) + 4 lh + r % 4 of its 32 x 32 block -- four
    // consecutive columns per lane.  Scaled and rounded, they go through a private LDS region of the
    // wavefront (rows of 32 NT halves + 16 bytes of padding: conflict-free 8-byte writes and 16-byte reads)
    // and leave as 16 bytes per lane, whole 128-byte lines per row.  (Two-byte stores straight from the
    // accumulators, half a line per row and instruction, cost 20 us of an 80 us kernel.)
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");  // every wavefront is done with the ring
    const int wave_m0 = m0 + wm * 32 * MT, wave_n0 = n0 + wn * 32 * NT;
    if ((a.N & 7) == 0) {
        constexpr int kOutRowB = 32 * NT * 2 + 16;
        constexpr int kSegs = 4 * NT, kRowsPerStore = 64 / kSegs;  // 16-byte segments per row; rows per wave-wide store
        static_assert(4 * 32 * MT * kOutRowB <= kDenseStages * kStage, "output staging must fit the ring's LDS");
        unsigned char *out = smem + (size_t)wave * (32 * MT) * kOutRowB;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int nl = j * 32 + 8 * g + 4 * lh;
                float sc[4] = {1.f, 1.f, 1.f, 1.f};
                if (a.scale && wave_n0 + nl < a.N) {  // N is a multiple of 8 here: the four columns are in range together
                    const half4_t h = *reinterpret_cast<const half4_t *>(a.scale + wave_n0 + nl);
#pragma unroll
                    for (int t = 0; t < 4; ++t) sc[t] = (float)h[t];
                }
#pragma unroll
                for (int i = 0; i < MT; ++i) {
                    half4_t o;
#pragma unroll
                    for (int t = 0; t < 4; ++t) o[t] = (half_t)(acc[i][j][4 * g + t] * sc[t]);
                    *reinterpret_cast<half4_t *>(out + (i * 32 + ln) * kOutRowB + nl * 2) = o;
                }
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // same wavefront wrote what it now reads
#pragma unroll
        for (int t = 0; t < 32 * MT / kRowsPerStore; ++t) {
            const int row = t * kRowsPerStore + lane / kSegs, seg = lane % kSegs;
            const uint4 v = *reinterpret_cast<const uint4 *>(out + row * kOutRowB + seg * 16);
            const int m = wave_m0 + row, n = wave_n0 + seg * 8;
            if (m < a.M && n < a.N) *reinterpret_cast<uint4 *>(a.C + (size_t)m * a.N + n) = v;
        }
    } else {
        // rows of Y are not 16-byte aligned: element stores
#pragma unroll
        for (int j = 0; j < NT; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = wave_n0 + j * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (n >= a.N) continue;
                const float sc = a.scale ? (float)a.scale[n] : 1.f;
#pragma unroll
                for (int i = 0; i < MT; ++i) {
                    const int m = wave_m0 + i * 32 + ln;
                    if (m < a.M) a.C[(size_t)m * a.N + n] = (half_t)(acc[i][j][r] * sc);
                }
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
    static KernelSetup setup;
    if (int st = kernel_setup(reinterpret_cast<const void *>(&gemm_dense_kernel<MT, NT>), lds, false, setup)) return st;
    const int n_tiles = a.tiles_m * a.tiles_n;
    const int grid = ((n_tiles + 7) / 8) * 8;
    gemm_dense_kernel<MT, NT><<<grid, 256, lds, s>>>(a);
    return launch_status();
}

}  // namespace vq
