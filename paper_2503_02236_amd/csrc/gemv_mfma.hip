// VQ-gemv for small batches (bs = 1..16) when the codebooks fit LDS, on the matrix cores of gfx950.
// Operation: VQ-LLM (arXiv 2503.02236) Sec. III-C "VQ-gemv", batch sizes of Sec. VII (1..16);
// residual codebooks summed as in Sec. II-A.
//
// Why matrix cores for a gemv: with a lane-per-code mapping on the vector ALU, every (row, token)
// pair needs its own reduction over the 64 lanes, so the cost grows with bs (16 wave reductions per
// row at bs = 16).  v_mfma_f32_16x16x32_f16 does that reduction itself: A = 16 weight rows x 32 k,
// B = 32 k x 16 tokens, C = 16 x 16 fp32.  A lane's A operand is 8 consecutive k of one row, i.e.
// exactly one dequantized v = 8 sub-vector (two for v = 4): gathered from the LDS codebook straight
// into the operand registers (layout fusion, Sec. VI-B: no shuffle, no LDS round trip).  Batches
// below 16 leave token columns zero; the gathers, not the MFMAs, bound the kernel.
//
// Mapping: one workgroup per 16 weight rows (256 workgroups at N = 4096).  Lane (r = lane % 16,
// g = lane / 16) loads 16 (or 8) bytes of codes of row r: CPL consecutive sub-vector positions.  One
// "iteration" of a wavefront therefore covers 4 * CPL positions of all 16 rows, with CPL / (8/v)
// MFMAs; x operands for those positions come straight from global memory (L2-resident).
// Iterations are dealt round-robin to the wavefronts (K = 4096, uint8 pairs: 16 iterations, one
// per wavefront at N = 4096); the per-wavefront 16 x 16 partial tiles are added in wavefront order through LDS.
// RT = 2: a workgroup takes 32 rows, two tiles of 16 that share every x operand.  Each workgroup reads all
// of x once -- bs * K * 2 bytes from L2 --, which at bs = 16 is what the kernel waits for (N = 11008,
// K = 4096: 688 workgroups x 128 KiB = 88 MB through the L2s at ~11 TB/s, 8 of the 18 us); with two tiles per
// workgroup it is half of that.  Used where enough workgroups remain to fill the chip.
#include <algorithm>

#include "vq_common.h"

namespace vq {

typedef float float4v_t __attribute__((ext_vector_type(4)));

struct GemvMfmaArgs {
    const void *codes;
    const half_t *cb, *scale, *x;
    half_t *y;
    int N, K, J, E, bs, nit;
    int n_hot;  // entries of each codebook held in LDS (all of them unless HOT)
    // per-tile codebooks (Sec. III-B, Tbl. III): sets per row of tiles, sub-vector positions per tile, rows per tile
    int tiles_k, tile_j, tile_n;
};

// One code load per lane and iteration: 16 bytes, or 8 for single uint8 codes (16 positions would need
// 16 x operands in registers); packed 12-bit codes come in 12-byte words of 8 codes.
template <typename CodeT, int R>
struct GemvMfmaShape {
    static constexpr int BITS = (int)sizeof(CodeT) * 8;
    static constexpr int LB = R * (int)sizeof(CodeT) == 1 ? 8 : 16;
    static constexpr int CPL = LB / (R * (int)sizeof(CodeT));
};
template <int R>
struct GemvMfmaShape<Code12, R> {
    static constexpr int BITS = 12;
    static constexpr int LB = 12;
    static constexpr int CPL = 8 / R;
};

// Code number q of the lane's code word (static q).
template <typename CodeT>
__device__ __forceinline__ unsigned word_code(const V16 &cd, int q) {
    return sizeof(CodeT) == 1 ? cd.b[q] : cd.h[q];
}
template <>
__device__ __forceinline__ unsigned word_code<Code12>(const V16 &cd, int q) {
    const int bit = 12 * q, wi = bit >> 5, sh = bit & 31;
    unsigned v = cd.w[wi] >> sh;
    if (sh > 20) v |= cd.w[wi + 1] << (32 - sh);  // straddles two dwords (q = 2, 5)
    return v & 0xFFFu;
}

// HOT: the codebook does not fit LDS.  Its first n_hot entries are cached there and the rest is gathered
// from global memory (L2): the shared-memory level of the hierarchical codebook cache of Sec. V-B.  It
// pays off when the entries have been reordered by frequency (vq_reorder_by_frequency), so that most
// codes are small; with uniformly used entries nearly every lookup takes the L2 path.
template <typename CodeT, int V, int R, bool HOT, int RT>
__device__ __forceinline__ void gemv_mfma_body(const GemvMfmaArgs &a, const int bx) {
    constexpr int LB = GemvMfmaShape<CodeT, R>::LB;     // bytes of codes per lane and iteration
    constexpr int CPL = GemvMfmaShape<CodeT, R>::CPL;   // sub-vector positions per code load
    constexpr int CPO = 8 / V;                          // codes per MFMA operand (8 consecutive k)
    constexpr int MPI = CPL / CPO;                      // MFMAs per iteration
    constexpr int BITS = GemvMfmaShape<CodeT, R>::BITS;
    static_assert(CPL * R * BITS == LB * 8 && MPI >= 1, "unsupported code width");
    extern __shared__ __align__(16) unsigned char smem[];
    half_t *cbl = reinterpret_cast<half_t *>(smem);                      // [R][E][V]
    const int set_halves = R * a.n_hot * V;          // one set of codebooks
    const int cb_bytes = set_halves * 2 * a.tiles_k;  // every set of this workgroup's row of tiles
    float4v_t *red = reinterpret_cast<float4v_t *>(smem + ((cb_bytes + 15) & ~15));  // [waves][64]

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, nwaves = blockDim.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int n0 = bx * 16 * RT;
    // codes and x of this wavefront's first iteration are requested before the codebook is staged
    const unsigned char *crow[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int n = min(n0 + 16 * t + r, a.N - 1);  // rows past the end are computed and dropped
        crow[t] = reinterpret_cast<const unsigned char *>(a.codes) + (size_t)n * a.J * R * BITS / 8;
    }
    // Codes and x operands of iteration `it` (< nit) of this wavefront; returns whether this lane's part
    // counts.  The loads carry no condition: a lane past the end of the row, or of a token past the batch,
    // reads a position / token that exists and its x operand is zeroed where it is used (a zero B operand
    // cancels whatever A holds).  With a branch around the loads their results meet the zeros of the
    // other path in a register copy right behind them, and a copy waits for the data: the code load was
    // waited for (a trip to HBM) before the x loads were even issued.
    auto lane_pos = [&](int it, bool &ok) {
        const int jb = (it * 4 + g) * CPL;  // first position of this lane; J % CPL == 0
        ok = jb < a.J;
        return ok ? jb : a.J - CPL;
    };
    auto load_codes = [&](int it, int t, V16 &cd) {
        bool ok;
        const unsigned char *cp = crow[t] + (size_t)lane_pos(it, ok) * R * BITS / 8;
        if (LB == 16) {
            cd = ld16(cp);
        } else if (LB == 12) {  // 4-byte aligned: a row is a whole number of 12-byte words
            const uint32_t *c3 = reinterpret_cast<const uint32_t *>(cp);
            cd.w[0] = c3[0];
            cd.w[1] = c3[1];
            cd.w[2] = c3[2];
            cd.w[3] = 0;
        } else {
            V8 c8 = ld8(cp);
            cd.w[0] = c8.w[0];
            cd.w[1] = c8.w[1];
            cd.w[2] = cd.w[3] = 0;
        }
    };
    auto load_x = [&](int it, half8_t (&xb)[MPI]) {
        bool ok;
        const half_t *xr = a.x + (size_t)min(r, a.bs - 1) * a.K + (size_t)lane_pos(it, ok) * V;
#pragma unroll
        for (int m = 0; m < MPI; ++m) xb[m] = ld16(xr + m * 8).h8;
        return ok && r < a.bs;
    };
    V16 cd[RT];
    half8_t xb[MPI];
    // (every wavefront loads: one without an iteration repeats the last one and never uses it)
#pragma unroll
    for (int t = 0; t < RT; ++t) load_codes(min(wave, a.nit - 1), t, cd[t]);
    bool use_x = load_x(min(wave, a.nit - 1), xb);
    // per-channel scales of the four output rows this lane writes at the very end (rows n0 + 4 g + i): asked
    // for now, with everything else, as raw halves and without a branch (without scales: any readable halves,
    // ignored later).  Loaded where they are used they are four dependent round trips to L2 at the tail of a
    // kernel that lasts a few microseconds; converted or selected here they would be waited for here.
    // (of the tile whose sums this wavefront adds up at the end: tile wave % RT)
    half_t sc4[4];
    {
        const half_t *sp = a.scale ? a.scale : a.x;
#pragma unroll
        for (int i = 0; i < 4; ++i) sc4[i] = sp[a.scale ? min(n0 + 16 * (wave % RT) + 4 * g + i, a.N - 1) : 0];
    }

    // all codebooks (with per-tile codebooks: the sets of the tiles this workgroup's 16 rows cross), or (HOT,
    // one codebook) its first n_hot entries
    const half_t *cb_src = a.cb + (a.tile_n > 0 ? (size_t)(n0 / a.tile_n) * a.tiles_k * set_halves : 0);
    for (int i = tid; i < cb_bytes / 16; i += blockDim.x)
        reinterpret_cast<uint4 *>(cbl)[i] = reinterpret_cast<const uint4 *>(cb_src)[i];
    __syncthreads();

    float4v_t acc[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) acc[t] = float4v_t{0.f, 0.f, 0.f, 0.f};
    for (int it = wave; it < a.nit; it += nwaves) {
        // the next iteration's codes (a trip to HBM) are requested now, its x operands (L2) when this
        // iteration's have been used: they land while the next iteration's entries are looked up
        const bool more = it + nwaves < a.nit;
        V16 cd_next[RT];
        if (more) {
#pragma unroll
            for (int t = 0; t < RT; ++t) load_codes(it + nwaves, t, cd_next[t]);
        }
        // codebook set of this lane's positions (a load never straddles two tiles)
        // (lanes past the end of the row are clamped to the last set; their x operand is zero)
        const half_t *cbt = cbl + (size_t)min(((it * 4 + g) * CPL) / a.tile_j, a.tiles_k - 1) * set_halves;
        // MC MFMA operands at a time: all their entry lookups are issued before the first is used (taken one
        // operand at a time, every operand waits out its own LDS round trip)
        constexpr int kEntryRegs = CPO * R * (V == 8 ? 4 : 2);   // registers of one operand's entries
        constexpr int MC = (MPI % 4 == 0 && 4 * kEntryRegs <= 32) ? 4 : (MPI % 2 == 0 && 2 * kEntryRegs <= 32) ? 2 : 1;
#pragma unroll
        for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int m0 = 0; m0 < MPI; m0 += MC) {
            V16 ev[MC][CPO][R];
#pragma unroll
            for (int mi = 0; mi < MC; ++mi)
#pragma unroll
                for (int h = 0; h < CPO; ++h) {
                    const int c = (m0 + mi) * CPO + h;  // code position inside the 16-byte word
#pragma unroll
                    for (int rr = 0; rr < R; ++rr) {
                        const unsigned code = word_code<CodeT>(cd[t], c * R + rr);
                        // the entry: from the LDS copy, or (cold entry of a partly cached codebook) from L2.  The two
                        // loads are kept apart by their address spaces, so neither becomes a generic-pointer load
                        V16 e;
                        e.u = make_uint4(0, 0, 0, 0);
                        typedef unsigned raw4_t __attribute__((ext_vector_type(4)));
                        typedef unsigned raw2_t __attribute__((ext_vector_type(2)));
                        const half_t *le = cbt + ((size_t)rr * a.n_hot + code) * V;
                        const half_t *ge = a.cb + ((size_t)rr * a.E + code) * V;
                        if (!HOT || code < (unsigned)a.n_hot) {
                            if (V == 8) {
                                const raw4_t t = *(const __attribute__((address_space(3))) raw4_t *)le;
                                e.w[0] = t.x; e.w[1] = t.y; e.w[2] = t.z; e.w[3] = t.w;
                            } else {
                                const raw2_t t = *(const __attribute__((address_space(3))) raw2_t *)le;
                                e.w[0] = t.x; e.w[1] = t.y;
                            }
                        } else {
                            if (V == 8) {
                                const raw4_t t = *(const __attribute__((address_space(1))) raw4_t *)ge;
                                e.w[0] = t.x; e.w[1] = t.y; e.w[2] = t.z; e.w[3] = t.w;
                            } else {
                                const raw2_t t = *(const __attribute__((address_space(1))) raw2_t *)ge;
                                e.w[0] = t.x; e.w[1] = t.y;
                            }
                        }
                        ev[mi][h][rr] = e;
                    }
                }
            if (!HOT) __builtin_amdgcn_sched_group_barrier(0x100, MC * CPO * R, 0);  // the LDS reads first
#pragma unroll
            for (int mi = 0; mi < MC; ++mi) {
                V16 op;
                if constexpr (R <= 2) {
                    // One or two entries: a single fp16 addition rounds the exact sum once, which is the fp32
                    // sum of Sec. II-A rounded to fp16 whenever that fp32 sum is exact -- always, unless the two
                    // exponents lie more than 13 apart; then the two roundings of fp32-then-fp16 can differ from
                    // this single one by one fp16 ulp on a tie.
#pragma unroll
                    for (int h = 0; h < CPO; ++h)
#pragma unroll
                        for (int rr = 0; rr < R; ++rr) {
                            const V16 &e = ev[mi][h][rr];
                            if (V == 8) {
                                if (rr == 0) {
                                    op = e;
                                } else {
#pragma unroll
                                    for (int q = 0; q < 4; ++q) op.h2[q] += e.h2[q];
                                }
                            } else {
                                if (rr == 0) {
                                    op.h2[2 * h] = e.h2[0];
                                    op.h2[2 * h + 1] = e.h2[1];
                                } else {
                                    op.h2[2 * h] += e.h2[0];
                                    op.h2[2 * h + 1] += e.h2[1];
                                }
                            }
                        }
                } else {
                    // Three or more residual entries: fp32 sum, r ascending, rounded to fp16 once -- the
                    // dequantized tile of Sec. II-A bit for bit (repeated fp16 additions would round R - 1 times).
                    float f[8];
#pragma unroll
                    for (int h = 0; h < CPO; ++h)
#pragma unroll
                        for (int rr = 0; rr < R; ++rr) {
                            const V16 &e = ev[mi][h][rr];
#pragma unroll
                            for (int i = 0; i < V; ++i) {
                                const float t = (float)e.h8[i];
                                f[h * V + i] = rr == 0 ? t : f[h * V + i] + t;
                            }
                        }
#pragma unroll
                    for (int i = 0; i < 8; ++i) op.h8[i] = (half_t)f[i];
                }
                half8_t xop = xb[m0 + mi];
                if (!use_x) xop = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(op.h8, xop, acc[t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int t = 0; t < RT; ++t) cd[t] = cd_next[t];
        if (more) use_x = load_x(it + nwaves, xb);
    }

    // partial tiles -> LDS [tile][wavefront][lane], each tile summed in wavefront order by one wavefront
    // (tile t by wavefront t; a workgroup with fewer wavefronts than tiles: wavefront 0 takes them in turn).
    // C layout: lane holds token (lane % 16), rows 4 (lane / 16) + 0..3.
#pragma unroll
    for (int t = 0; t < RT; ++t) red[(t * nwaves + wave) * 64 + lane] = acc[t];
    __syncthreads();
    for (int t = wave; t < RT; t += nwaves) {
        float4v_t sum = red[(t * nwaves) * 64 + lane];
        for (int w = 1; w < nwaves; ++w) {
            const float4v_t p = red[(t * nwaves + w) * 64 + lane];
            sum += p;
        }
        if (r < a.bs) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int nn = n0 + 16 * t + 4 * g + i;
                // (the scales were prefetched for tile wave % RT: any other tile, only with fewer wavefronts than
                // tiles, reads its own)
                const float sc = !a.scale ? 1.f : (t == wave % RT ? (float)sc4[i] : (float)a.scale[min(nn, a.N - 1)]);
                if (nn < a.N) a.y[(size_t)r * a.N + nn] = (half_t)(sum[i] * sc);
            }
        }
    }
}

template <typename CodeT, int V, int R, bool HOT, int RT>
__global__ __launch_bounds__(RT == 1 ? 1024 : 512) void gemv_mfma_kernel(GemvMfmaArgs a) {  // (two tiles: twice the operands in flight, up to 8 wavefronts)
    gemv_mfma_body<CodeT, V, R, HOT, RT>(a, blockIdx.x);
}

// Several independent problems of one kind in one launch (blockIdx.y picks the problem): the fixed costs of a
// launch -- ramp-up, first touches, drain; about as long as the useful part of a bs = 1 product of this size --
// are paid once, and workgroups of different problems share the compute units.
constexpr int kGemvMfmaBatch = 4;
struct GemvMfmaBatch {
    GemvMfmaArgs a[kGemvMfmaBatch];
    int n_wg[kGemvMfmaBatch];
};
template <typename CodeT, int V, int R>
__global__ __launch_bounds__(1024) void gemv_mfma_batch_kernel(GemvMfmaBatch b) {
    if ((int)blockIdx.x >= b.n_wg[blockIdx.y]) return;
    gemv_mfma_body<CodeT, V, R, false, 1>(b.a[blockIdx.y], blockIdx.x);
}

namespace {

constexpr size_t kGemvMfmaLdsCodebook = 128 * 1024;  // whole codebooks up to this size live in LDS
constexpr int kGemvMfmaHotEntries8 = 4096;           // v = 8 entries of a larger codebook cached in LDS (64 KiB)

template <typename CodeT, int V, int R, bool HOT, int RT>
int run(const vq_weight_t *w, const half_t *x, int bs, half_t *y, hipStream_t s) {
    constexpr int CPL = GemvMfmaShape<CodeT, R>::CPL;
    GemvMfmaArgs a;
    a.codes = w->codes;
    a.cb = (const half_t *)w->codebooks;
    a.scale = (const half_t *)w->scale;
    a.x = x;
    a.y = y;
    a.N = w->N;
    a.K = w->K;
    a.J = w->K / V;
    a.E = w->n_entries;
    a.bs = bs;
    a.nit = (a.J + 4 * CPL - 1) / (4 * CPL);
    // wavefronts per workgroup: the chip holds 16 per CU (4096 in all); with more than 256 workgroups
    // fewer, longer-running wavefronts keep every workgroup resident at once (measured on N = 11008:
    // 4 wavefronts 11.5 us, 8: 13.3, 16: 16.5 at bs = 1)
    const int n_wg = (a.N + 16 * RT - 1) / (16 * RT);
    int waves = 16;
    while (waves > 4 && n_wg * waves > 4096) waves >>= 1;
    // codebooks of more than half the LDS: one workgroup per CU anyway, so give it all 16 wavefronts
    if ((size_t)R * a.E * V * 2 > 72 * 1024 && w->hot_entries == 0) waves = 16;
    if (RT > 1 && waves > 8) waves = 8;  // (that build is compiled for 512 threads)
    if (waves > a.nit) waves = a.nit;
    if (waves < 1) waves = 1;
    a.tile_n = w->cb_tile_n;
    a.tiles_k = w->cb_tile_n > 0 ? w->K / w->cb_tile_k : 1;
    a.tile_j = w->cb_tile_n > 0 ? w->cb_tile_k / V : (1 << 30);
    // hot prefix: 64 KiB of entries with one workgroup per CU, 32 KiB when several share a CU
    a.n_hot = a.E;
    if (HOT) {
        const int cap = (n_wg <= 256 ? 64 * 1024 : 32 * 1024) / (V * 2);
        a.n_hot = a.E < cap ? a.E : cap;
    }
    const size_t cb_bytes = (size_t)R * a.n_hot * V * 2 * a.tiles_k;
    const size_t lds = ((cb_bytes + 15) & ~(size_t)15) + (size_t)RT * waves * 64 * sizeof(float4v_t);
    static KernelSetup setup;
    if (int st = kernel_setup(reinterpret_cast<const void *>(&gemv_mfma_kernel<CodeT, V, R, HOT, RT>), lds, false, setup)) return st;
    gemv_mfma_kernel<CodeT, V, R, HOT, RT><<<n_wg, waves * 64, lds, s>>>(a);
    return launch_status();
}

template <typename CodeT, int V>
int by_r(const vq_weight_t *w, const half_t *x, int bs, half_t *y, hipStream_t s) {
    const bool hot = w->cb_tile_n == 0 && (size_t)w->n_codebooks * w->n_entries * w->v * 2 > kGemvMfmaLdsCodebook;
    if (hot) return run<CodeT, V, 1, true, 1>(w, x, bs, y, s);  // only single codebooks are cached partly
    // two row tiles per workgroup halve the x traffic of a batch, where 32-row workgroups still fill the chip
    // (per-tile codebooks: the 32 rows must lie in one row of tiles)
    // (N = 11008, K = 4096, two codebooks: bs = 16 18.3 -> 17.1 us, one codebook per tile 19.0 -> 15.9, 12-bit codes
    // 26.3 -> 22.9; at bs = 4 the x traffic is small and 344 workgroups spread worse over 256 CUs than 688: 11.1 -> 14.0)
    const bool two = bs >= 8 && (w->N + 31) / 32 >= 256 && (w->cb_tile_n == 0 || w->cb_tile_n % 32 == 0);
    switch (w->n_codebooks) {
        case 1: return two ? run<CodeT, V, 1, false, 2>(w, x, bs, y, s) : run<CodeT, V, 1, false, 1>(w, x, bs, y, s);
        case 2: return two ? run<CodeT, V, 2, false, 2>(w, x, bs, y, s) : run<CodeT, V, 2, false, 1>(w, x, bs, y, s);
        default: return two ? run<CodeT, V, 4, false, 2>(w, x, bs, y, s) : run<CodeT, V, 4, false, 1>(w, x, bs, y, s);
    }
}

// One problem of a batched launch: the arguments of the plain one-tile build (whole codebooks in LDS).
template <typename CodeT, int V, int R>
GemvMfmaArgs batch_args(const vq_weight_t *w, const half_t *x, half_t *y) {
    constexpr int CPL = GemvMfmaShape<CodeT, R>::CPL;
    GemvMfmaArgs a;
    a.codes = w->codes;
    a.cb = (const half_t *)w->codebooks;
    a.scale = (const half_t *)w->scale;
    a.x = x;
    a.y = y;
    a.N = w->N;
    a.K = w->K;
    a.J = w->K / V;
    a.E = w->n_entries;
    a.bs = 1;
    a.nit = (a.J + 4 * CPL - 1) / (4 * CPL);
    a.tile_n = w->cb_tile_n;
    a.tiles_k = w->cb_tile_n > 0 ? w->K / w->cb_tile_k : 1;
    a.tile_j = w->cb_tile_n > 0 ? w->cb_tile_k / V : (1 << 30);
    a.n_hot = a.E;
    return a;
}

template <typename CodeT, int V, int R>
int run_batch(const vq_weight_t *const *w, const void *const *x, void *const *y, int count, hipStream_t s) {
    GemvMfmaBatch b;
    int grid = 0, total = 0, min_nit = 1 << 30;
    size_t cb_bytes = 0;
    for (int i = 0; i < kGemvMfmaBatch; ++i) {
        const int k = i < count ? i : 0;   // unused slots repeat problem 0 (never launched: grid.y = count)
        b.a[i] = batch_args<CodeT, V, R>(w[k], (const half_t *)x[k], (half_t *)y[k]);
        b.n_wg[i] = (w[k]->N + 15) / 16;
        if (i < count) {
            grid = std::max(grid, b.n_wg[i]);
            total += b.n_wg[i];
            min_nit = std::min(min_nit, b.a[i].nit);
            cb_bytes = std::max(cb_bytes, (size_t)R * b.a[i].n_hot * V * 2 * b.a[i].tiles_k);
        }
    }
    // wavefronts per workgroup as for one problem with all the workgroups of the batch
    int waves = 16;
    while (waves > 4 && total * waves > 4096) waves >>= 1;
    if (waves > min_nit) waves = min_nit;
    if (waves < 1) waves = 1;
    const size_t lds = ((cb_bytes + 15) & ~(size_t)15) + (size_t)waves * 64 * sizeof(float4v_t);
    static KernelSetup setup;
    if (int st = kernel_setup(reinterpret_cast<const void *>(&gemv_mfma_batch_kernel<CodeT, V, R>), lds, false, setup)) return st;
    gemv_mfma_batch_kernel<CodeT, V, R><<<dim3(grid, count), waves * 64, lds, s>>>(b);
    return launch_status();
}

}  // namespace

// Whether `count` bs = 1 problems can share one launch of the matrix-core gemv: all of one kind (code width, v,
// number of codebooks), whole codebooks in LDS, none empty.
bool gemv_mfma_batch_supported(const vq_weight_t *const *w, int count) {
    if (count < 2 || count > kGemvMfmaBatch) return false;
    for (int i = 0; i < count; ++i) {
        if (!w[i] || w[i]->N <= 0 || w[i]->K <= 0 || !gemv_mfma_supported(w[i])) return false;
        if (w[i]->code_bits != w[0]->code_bits || w[i]->v != w[0]->v || w[i]->n_codebooks != w[0]->n_codebooks) return false;
        if (w[i]->cb_tile_n == 0 && (size_t)w[i]->n_codebooks * w[i]->n_entries * w[i]->v * 2 > kGemvMfmaLdsCodebook) return false;
        if (w[i]->n_codebooks != 1 && w[i]->n_codebooks != 2 && w[i]->n_codebooks != 4) return false;
    }
    return true;
}

int launch_gemv_mfma_batch(const vq_weight_t *const *w, const void *const *x, void *const *y, int count, hipStream_t s) {
#define VQ_MB(CodeT, V)                                                                   \
    switch (w[0]->n_codebooks) {                                                          \
        case 1: return run_batch<CodeT, V, 1>(w, x, y, count, s);                         \
        case 2: return run_batch<CodeT, V, 2>(w, x, y, count, s);                         \
        default: return run_batch<CodeT, V, 4>(w, x, y, count, s);                        \
    }
    if (w[0]->code_bits == 8) {
        if (w[0]->v == 8) { VQ_MB(uint8_t, 8) } else { VQ_MB(uint8_t, 4) }
    } else if (w[0]->code_bits == 12) {
        if (w[0]->v == 8) { VQ_MB(Code12, 8) } else { VQ_MB(Code12, 4) }
    } else {
        if (w[0]->v == 8) { VQ_MB(uint16_t, 8) } else { VQ_MB(uint16_t, 4) }
    }
#undef VQ_MB
}

// Codebooks must fit LDS next to the reduction buffer (a single larger codebook is cached partly), and a
// row of codes must be a whole number of code words made of whole sub-vector positions.
bool gemv_mfma_supported(const vq_weight_t *w) {
    const int R = w->n_codebooks, sz = w->code_bits / 8;
    if (w->v != 8 && w->v != 4) return false;
    if (R != 1 && R != 2 && R != 4) return false;
    if (w->code_bits != 12 && R * sz > 8) return false;
    const int cpl = w->code_bits == 12 ? 8 / R : (R * sz == 1 ? 8 : 16) / (R * sz), cpo = 8 / w->v;
    if (cpl < cpo) return false;
    if (w->K <= 0 || (w->K / w->v) % cpl != 0) return false;
    if (w->cb_tile_n > 0) {
        // per-tile codebooks: the sets of one row of tiles live in LDS together (size checked with the descriptor)
    } else if ((size_t)R * w->n_entries * w->v * 2 > kGemvMfmaLdsCodebook) {
        // a single large codebook is cached partly, if the caller says that its front is hot enough
        if (R != 1 || w->hot_entries <= 0 || w->hot_entries > kGemvMfmaHotEntries8 * 8 / w->v) return false;
    }
    if ((R * w->n_entries * w->v * 2) % 16 != 0) return false;
    return true;
}

int launch_gemv_mfma(const vq_weight_t *w, const void *x, int bs, void *y, hipStream_t s) {
    const half_t *xp = (const half_t *)x;
    half_t *yp = (half_t *)y;
    if (w->code_bits == 8) return w->v == 8 ? by_r<uint8_t, 8>(w, xp, bs, yp, s) : by_r<uint8_t, 4>(w, xp, bs, yp, s);
    if (w->code_bits == 12) return w->v == 8 ? by_r<Code12, 8>(w, xp, bs, yp, s) : by_r<Code12, 4>(w, xp, bs, yp, s);
    return w->v == 8 ? by_r<uint16_t, 8>(w, xp, bs, yp, s) : by_r<uint16_t, 4>(w, xp, bs, yp, s);
}

}  // namespace vq
