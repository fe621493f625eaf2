// VQ-attn (decode) for gfx950: out[b][h] = softmax_t(sm_scale * q . K[t]) . V[t] over a KV
// cache stored as uint8 VQ codes.  Formula: VQ-LLM (arXiv 2503.02236) Sec. II-B; setup
// VQ<4,8,1>, 32 heads x 128 channels: Sec. III-A; token-parallel split with a merge of the
// local softmax statistics: Sec. III-B (flash-decoding dataflow of Fig. 5).
//
// Mapping (wave64): one lane owns one token at a time.  It dequantizes the token's whole
// K vector sub-vector by sub-vector and dots it with q (row-wise: no exchange needed,
// Sec. III-B Fig. 6), and later dequantizes the token's V vector and adds p_t * V[t] into
// its PRIVATE 128-float accumulator.  The column-wise accumulation over tokens that forces a
// shared-memory round trip in the paper's baseline is thereby deferred to one butterfly
// reduction over the 64 lanes at the very end, so dequantized values never travel through
// LDS.  Codebooks live in LDS (2 KB each for one codebook per head and side).
//
// A workgroup streams over its token range in tiles of 32 codes per lane and side (1 token
// for v = 4).  The codes of the next two tiles are in flight while a tile is processed (register
// double buffers), so the HBM stream and the LDS gathers overlap.  Softmax is kept online
// per wavefront: a wave-uniform running maximum; the accumulators are rescaled only when a
// tile raises it (rare after the first tiles).
#include "vq_common.h"

namespace vq {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kAttnMinTokens = 512;   // do not split token ranges below this
constexpr int kAttnTargetWgs = 512;   // two workgroups per compute unit

// tokens per lane per tile: 32 code bytes per lane and side (one token of 64 for v = 2)
template <int V>
struct AttnTile {
    static constexpr int NI = V == 2 ? 1 : 32 / (128 / V);
    static constexpr int TOKENS = 256 * NI;  // per workgroup and tile
};

struct AttnArgs {
    const uint8_t *k_codes, *v_codes;
    const half_t *k_cb, *v_cb;
    const int *seq_lens;
    const half_t *q;
    half_t *out;
    float *ws;      // [B*H][S][D + 2] partials when S > 1
    int B, H, T, E, G, S;
    int tc;         // tokens per workgroup (token-range split), a multiple of the tile
    int pg_shift;   // log2 of sub-vectors per codebook group
    float scale2;   // sm_scale * log2(e)
};

// Butterfly sum of acc[0..N) over the 64 lanes; afterwards lane l holds the totals of
// elements 2l and 2l+1 in acc[0], acc[1].  In every step a lane keeps one half of its values and
// adds the partner lane's copy of that half.  The two big steps (partner 32 and 16 lanes away)
// use the gfx950 lane-swap instructions: one swap puts "mine" and "the partner's" of the kept
// half side by side; the small steps go through ds_bpermute.
template <int N>
__device__ __forceinline__ void lanes_reduce_scatter(float (&acc)[N], int lane) {
    static_assert(N == 128, "written for 128 accumulators");
#pragma unroll
    for (int i = 0; i < 64; ++i) {  // upper 32 lanes of lo <-> lower 32 lanes of hi
        auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i]), __float_as_uint(acc[i + 64]), false, false);
        acc[i] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) {  // odd rows of 16 of lo <-> even rows of hi
        auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(acc[i]), __float_as_uint(acc[i + 32]), false, false);
        acc[i] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
#pragma unroll
    for (int step = 2; step < 6; ++step) {
        const int m = 32 >> step;       // lane mask
        const int half = 64 >> step;    // elements kept
        const bool upper = (lane & m) != 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (i < half) {
                float lo = acc[i], hi = acc[i + half];
                float send = upper ? lo : hi;
                float keep = upper ? hi : lo;
                acc[i] = keep + __shfl_xor(send, m, 64);
            }
        }
    }
}

// Maximum over the wavefront as a wave-uniform value, on the vector ALU only (lane permutes inside
// rows of 16, then one read per row), so it does not queue behind the LDS gathers.
template <int CTRL>
__device__ __forceinline__ float dpp_max_step(float x) {
    int y = __builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, 0xF, 0xF, false);
    return fmaxf(x, __int_as_float(y));
}
__device__ __forceinline__ float wave_max_uniform(float x) {
    x = dpp_max_step<0xB1>(x);   // quad_perm [1,0,3,2]
    x = dpp_max_step<0x4E>(x);   // quad_perm [2,3,0,1]
    x = dpp_max_step<0x141>(x);  // row_half_mirror
    x = dpp_max_step<0x140>(x);  // row_mirror: every lane now holds the maximum of its row of 16
    const int xi = __float_as_int(x);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(xi, 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(xi, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(xi, 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(xi, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// One codebook entry as it is held in registers, and its load from an LDS byte address.
template <int V> struct AttnEntry;
template <> struct AttnEntry<8> {
    typedef V16 type;
    static __device__ __forceinline__ type load(unsigned addr) {
        typedef unsigned raw_t __attribute__((ext_vector_type(4)));
        const raw_t r = *reinterpret_cast<const __attribute__((address_space(3))) raw_t *>((uintptr_t)addr);
        type e;
        e.w[0] = r.x; e.w[1] = r.y; e.w[2] = r.z; e.w[3] = r.w;
        return e;
    }
};
template <> struct AttnEntry<4> {
    typedef V8 type;
    static __device__ __forceinline__ type load(unsigned addr) {
        typedef unsigned raw_t __attribute__((ext_vector_type(2)));
        const raw_t r = *reinterpret_cast<const __attribute__((address_space(3))) raw_t *>((uintptr_t)addr);
        type e;
        e.w[0] = r.x; e.w[1] = r.y;
        return e;
    }
};
template <> struct AttnEntry<2> {
    typedef half2_t type;
    static __device__ __forceinline__ type load(unsigned addr) {
        return *reinterpret_cast<const __attribute__((address_space(3))) half2_t *>((uintptr_t)addr);
    }
};

// (byte B of w) << sh in one instruction (the compiler emits an extract and a shift-add)
template <int B>
__device__ __forceinline__ unsigned byte_shl(unsigned w, unsigned sh) {
    unsigned r;
    if (B == 0)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0"
            : "=v"(r) : "v"(sh), "v"(w));
    else if (B == 1)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1"
            : "=v"(r) : "v"(sh), "v"(w));
    else if (B == 2)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2"
            : "=v"(r) : "v"(sh), "v"(w));
    else
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3"
            : "=v"(r) : "v"(sh), "v"(w));
    return r;
}

// ONE: a single codebook per head and side (cb_groups == 1, at most 4 KiB each): the K codebook
// sits at LDS offset 0 and the V codebook at 4096, so an entry's address is (code * v * 2) plus a
// constant that folds into the offset field of the LDS instruction.
//
// Inside a tile the 64 lookups of a side go in small groups: the LDS gathers of group g+1 are
// issued before the arithmetic of group g, so that gathers (limited by LDS bank conflicts) and
// vector arithmetic overlap inside one wavefront; only two wavefronts per SIMD fit the 128
// private accumulators.
template <int V, bool ONE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_decode_kernel(AttnArgs a) {
    constexpr int D = 128;
    constexpr int P = D / V;          // codes (bytes) per token and side
    constexpr int NI = AttnTile<V>::NI;
    constexpr int TILE = AttnTile<V>::TOKENS;
    constexpr int GS = V == 8 ? 4 : 8;  // lookups per group (at most 16 registers of entries per group)
    constexpr int NG = NI * P / GS;   // groups per tile and side
    constexpr int NC = NI * P / 16;   // 16-byte code words per lane, tile and side
    constexpr unsigned SH = V == 8 ? 4 : V == 4 ? 3 : 2;  // log2 of the entry size in bytes
    typedef typename AttnEntry<V>::type entry_t;
    extern __shared__ __align__(16) unsigned char smem[];
    // Entry addresses are formed as plain LDS byte offsets (shifted code + constant), which is only
    // right if the dynamic LDS block starts at LDS address 0: true for a kernel without static LDS.
    // The base is a link-time constant, so this check is decided once per build.
    if ((unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem != 0u) return;
    const int cb_bytes = a.G * a.E * V * 2;        // per side
    const int v_off = ONE ? 4096 : cb_bytes;       // LDS offset of the V codebook
    float *xw = reinterpret_cast<float *>(smem + 2 * (size_t)v_off);  // [4][D] + [4] + [4]
    float *xw_m = xw + 4 * D, *xw_l = xw_m + 4;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bh = blockIdx.x, split = blockIdx.y;
    const int b = bh / a.H, h = bh % a.H;
    const int len = a.seq_lens ? min(max(a.seq_lens[b], 0), a.T) : a.T;
    const int start = split * a.tc;
    const int end = min(len, start + a.tc);  // this workgroup attends tokens [start, end)

    // query: uniform over the workgroup and never written by this kernel; read through the constant
    // address space so that it is fetched with scalar loads and lives in scalar registers
    half2_t qf[D / 2];
    {
        typedef const __attribute__((address_space(4))) half2_t const_half2_t;
        const_half2_t *qp = (const_half2_t *)(uintptr_t)(a.q + (size_t)bh * D);
#pragma unroll
        for (int i = 0; i < D / 2; ++i) qf[i] = qp[i];
    }

    if (start >= end) {  // nothing to attend in this token range (uniform over the workgroup)
        if (tid < D) {
            if (a.S == 1) {
                a.out[(size_t)bh * D + tid] = (half_t)0.f;
            } else {
                float *wp = a.ws + ((size_t)bh * a.S + split) * (D + 2);
                wp[tid] = 0.f;
                if (tid == 0) {
                    wp[D] = -INFINITY;
                    wp[D + 1] = 0.f;
                }
            }
        }
        return;
    }

    const int ntiles = (end - start + TILE - 1) / TILE;
    const size_t row0 = (size_t)bh * a.T;
    const int t_lane = start + wave * 64 + lane;  // token of (tile it, sub-token i): + it*TILE + i*256

    // codes of one tile and side -> registers; tokens past the end re-read the last valid token
    auto load_codes = [&](const uint8_t *codes, int it, V16 (&buf)[NC]) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int t = min(t_lane + it * TILE + i * 256, end - 1);
            const uint8_t *cp = codes + (row0 + t) * P;
#pragma unroll
            for (int c = 0; c < P / 16; ++c) buf[i * (P / 16) + c] = ld16(cp + c * 16);
        }
    };

    // 1. codebooks of this head (both sides): global loads first, they are the first to be needed
    const int n16 = cb_bytes / 16;
    const uint4 *ks = reinterpret_cast<const uint4 *>(a.k_cb + (size_t)h * (cb_bytes / 2));
    const uint4 *vs = reinterpret_cast<const uint4 *>(a.v_cb + (size_t)h * (cb_bytes / 2));
    uint4 kst = make_uint4(0, 0, 0, 0), vst = kst;
    if (tid < n16) {
        kst = ks[tid];
        vst = vs[tid];
    }
    // 2. codes of the first two tiles
    V16 kA[NC], vA[NC], kB[NC], vB[NC];
    load_codes(a.k_codes, 0, kA);
    load_codes(a.v_codes, 0, vA);
    load_codes(a.k_codes, 1, kB);
    load_codes(a.v_codes, 1, vB);
    if (tid < n16) {
        reinterpret_cast<uint4 *>(smem)[tid] = kst;
        reinterpret_cast<uint4 *>(smem + v_off)[tid] = vst;
    }
    for (int i = tid + 256; i < n16; i += 256) {  // codebooks larger than 4 KiB per side
        reinterpret_cast<uint4 *>(smem)[i] = ks[i];
        reinterpret_cast<uint4 *>(smem + v_off)[i] = vs[i];
    }
    __syncthreads();

    const unsigned sh = SH;
    // gathers of group g (lookups GS g .. GS g + GS - 1 of the tile; lookup u = sub-token u / P, sub-vector u % P)
    auto gather = [&](const V16 (&codes)[NC], int g, int base, entry_t (&e)[GS]) {
#pragma unroll
        for (int j = 0; j < GS; ++j) {
            const int u = g * GS + j, p = u % P;
            const unsigned w = codes[u / 16].w[(u % 16) / 4];
            unsigned off = (u % 4) == 0 ? byte_shl<0>(w, sh)
                           : (u % 4) == 1 ? byte_shl<1>(w, sh)
                           : (u % 4) == 2 ? byte_shl<2>(w, sh) : byte_shl<3>(w, sh);
            if (!ONE) off += ((unsigned)(p >> a.pg_shift) * a.E) << SH;
            e[j] = AttnEntry<V>::load((unsigned)base + off);
        }
    };

    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;
    float lsum = 0.f;          // per lane
    float m_run = -INFINITY;   // wave-uniform running maximum of the scores (log2 domain)

    // Gathered entries of the group being used and of the one in flight.  The lookups of a tile form
    // one sequence of 2 NG groups (K side, then V side) that continues into the next tile, so the LDS
    // queue never drains at the boundaries between the two sides or between tiles.
    static_assert(NG % 2 == 0, "the double buffer must be back at slot 0 after each side");
    entry_t e[2][GS];
    gather(kA, 0, 0, e[0]);

    // kn: K codes of the following tile (the other register buffer)
    auto tile_step = [&](int it, V16 (&kc)[NC], V16 (&vc)[NC], const V16 (&kn)[NC]) {
        // ---- scores of the lane's NI tokens (two partial sums each to shorten the dependent chain).
        // Masked tokens get -inf through an additive bias: a select on the finished score would make
        // the compiler branch around the arithmetic and pull every gather of the tile in front of it.
        float sc[NI], bias[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) bias[i] = (t_lane + it * TILE + i * 256 < end) ? 0.f : -INFINITY;
        {
            float d0 = 0.f, d1 = 0.f;
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                if (g + 1 < NG)
                    gather(kc, g + 1, 0, e[(g + 1) & 1]);
                else
                    gather(vc, 0, v_off, e[0]);
                __builtin_amdgcn_sched_barrier(0);  // keep the gathers of g+1 ahead of the arithmetic of g
#pragma unroll
                for (int j = 0; j < GS; ++j) {
                    const int p = (g * GS + j) % P;
                    const entry_t &ev = e[g & 1][j];
                    if constexpr (V == 8) {
                        d0 = dot2(ev.h2[0], qf[p * 4 + 0], d0);
                        d1 = dot2(ev.h2[1], qf[p * 4 + 1], d1);
                        d0 = dot2(ev.h2[2], qf[p * 4 + 2], d0);
                        d1 = dot2(ev.h2[3], qf[p * 4 + 3], d1);
                    } else if constexpr (V == 4) {
                        d0 = dot2(ev.h2[0], qf[p * 2], d0);
                        d1 = dot2(ev.h2[1], qf[p * 2 + 1], d1);
                    } else {
                        if (j & 1)
                            d1 = dot2(ev, qf[p], d1);
                        else
                            d0 = dot2(ev, qf[p], d0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if ((g + 1) * GS % P == 0) {  // last group of a sub-token
                    const int i = (g * GS) / P;
                    sc[i] = __builtin_fmaf(d0 + d1, a.scale2, bias[i]);
                    d0 = d1 = 0.f;
                }
            }
        }
        load_codes(a.k_codes, it + 2, kc);  // the K codes of this tile are used up

        // ---- online softmax: raise the wave's running maximum if needed (uniform branch)
        float tmax = sc[0];
#pragma unroll
        for (int i = 1; i < NI; ++i) tmax = fmaxf(tmax, sc[i]);
        tmax = wave_max_uniform(tmax);
        if (tmax > m_run) {
            const float f = __builtin_amdgcn_exp2f(m_run - tmax);  // 0 while nothing was accumulated
#pragma unroll
            for (int d = 0; d < D; ++d) acc[d] *= f;
            lsum *= f;
            m_run = tmax;
        }

        // ---- acc += p_t * V[t]
        {
            float p_t = 0.f;
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                if (g + 1 < NG)
                    gather(vc, g + 1, v_off, e[(g + 1) & 1]);
                else
                    gather(kn, 0, 0, e[0]);  // first K group of the next tile
                __builtin_amdgcn_sched_barrier(0);
                if ((g * GS) % P == 0) {  // first group of a sub-token
                    const float s = sc[(g * GS) / P];
                    p_t = s == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s - m_run);
                    lsum += p_t;
                }
#pragma unroll
                for (int j = 0; j < GS; ++j) {
                    const int p = (g * GS + j) % P;
                    const entry_t &ev = e[g & 1][j];
                    if constexpr (V == 8) {
#pragma unroll
                        for (int k = 0; k < 8; ++k) acc[p * 8 + k] += p_t * (float)ev.h8[k];
                    } else if constexpr (V == 4) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) acc[p * 4 + k] += p_t * (float)ev.h4[k];
                    } else {
                        acc[p * 2] += p_t * (float)ev[0];
                        acc[p * 2 + 1] += p_t * (float)ev[1];
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        load_codes(a.v_codes, it + 2, vc);
    };

    for (int it = 0; it < ntiles; it += 2) {
        tile_step(it, kA, vA, kB);
        if (it + 1 < ntiles) tile_step(it + 1, kB, vB, kA);
    }

    // ---- reduce over lanes, then over the four wavefronts (fixed order) ---------------------
    lanes_reduce_scatter<D>(acc, lane);
    lsum = wave_sum(lsum);
    xw[wave * D + 2 * lane] = acc[0];
    xw[wave * D + 2 * lane + 1] = acc[1];
    if (lane == 0) {
        xw_m[wave] = m_run;
        xw_l[wave] = lsum;
    }
    __syncthreads();
    if (tid < D) {
        float M = fmaxf(fmaxf(xw_m[0], xw_m[1]), fmaxf(xw_m[2], xw_m[3]));
        float L = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            float wgt = (xw_m[w] == -INFINITY) ? 0.f : exp2f(xw_m[w] - M);
            L += xw_l[w] * wgt;
            o += xw[w * D + tid] * wgt;
        }
        if (a.S == 1) {
            a.out[(size_t)bh * D + tid] = (half_t)(L > 0.f ? o / L : 0.f);
        } else {
            float *wp = a.ws + ((size_t)bh * a.S + split) * (D + 2);
            wp[tid] = o;
            if (tid == 0) {
                wp[D] = M;
                wp[D + 1] = L;
            }
        }
    }
}

// Merge of the token-range partials by log-sum-exp (base 2), one workgroup per (b, h).
__global__ __launch_bounds__(128) void attn_merge_kernel(const float *__restrict__ ws, half_t *__restrict__ out,
                                                         int S) {
    constexpr int D = 128;
    const int bh = blockIdx.x, d = threadIdx.x;
    const float *wp = ws + (size_t)bh * S * (D + 2);
    float M = -INFINITY;
    for (int s = 0; s < S; ++s) M = fmaxf(M, wp[s * (D + 2) + D]);
    float L = 0.f, o = 0.f;
    for (int s = 0; s < S; ++s) {
        float ms = wp[s * (D + 2) + D];
        float wgt = (ms == -INFINITY) ? 0.f : exp2f(ms - M);
        L += wp[s * (D + 2) + D + 1] * wgt;
        o += wp[s * (D + 2) + d] * wgt;
    }
    out[(size_t)bh * D + d] = (half_t)(L > 0.f ? o / L : 0.f);
}

// Token-range split: enough workgroups to fill the chip (two per compute unit) when batch x heads
// alone does not, ranges of at least kAttnMinTokens tokens, rounded to whole tiles.
static void attn_split(const vq_kv_t *kv, int *S, int *tc) {
    const int tile = kv->v == 8 ? AttnTile<8>::TOKENS : kv->v == 4 ? AttnTile<4>::TOKENS : AttnTile<2>::TOKENS;
    const long long bh = (long long)kv->B * kv->H;
    long long want = bh > 0 ? (kAttnTargetWgs + bh - 1) / bh : 1;
    long long most = (kv->T + kAttnMinTokens - 1) / kAttnMinTokens;
    long long s = want < most ? want : most;
    if (s < 1) s = 1;
    long long per = (kv->T + s - 1) / s;
    per = (per + tile - 1) / tile * tile;
    if (per < tile) per = tile;
    *tc = (int)per;
    *S = (int)((kv->T + per - 1) / per);
    if (*S < 1) *S = 1;
}

size_t attn_decode_workspace(const vq_kv_t *kv) {
    int S, tc;
    attn_split(kv, &S, &tc);
    if (S == 1) return 0;
    return (size_t)kv->B * kv->H * S * (kv->D + 2) * sizeof(float);
}

template <int V, bool ONE>
static int run_attn(const AttnArgs &a, hipStream_t s) {
    const size_t side = ONE ? 4096 : (size_t)a.G * a.E * V * sizeof(half_t);  // matches the kernel's layout
    size_t lds = 2 * side + (4 * 128 + 8) * sizeof(float);
    static size_t attr_lds = 0;
    if (lds > 64 * 1024 && lds > attr_lds) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_decode_kernel<V, ONE>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_lds = lds;
    }
    attn_decode_kernel<V, ONE><<<dim3(a.B * a.H, a.S), 256, lds, s>>>(a);
    if (a.S > 1) attn_merge_kernel<<<a.B * a.H, 128, 0, s>>>(a.ws, a.out, a.S);
    return launch_status();
}

int launch_attn_decode(const vq_kv_t *kv, const void *q, float sm_scale, void *out, void *ws, hipStream_t s) {
    if (kv->D != 128) return VQ_ERR_UNSUPPORTED;
    if ((kv->cb_groups * kv->n_entries * kv->v) % 8 != 0) return VQ_ERR_UNSUPPORTED;  // 128-bit codebook staging
    AttnArgs a;
    a.k_codes = (const uint8_t *)kv->k_codes;
    a.v_codes = (const uint8_t *)kv->v_codes;
    a.k_cb = (const half_t *)kv->k_codebooks;
    a.v_cb = (const half_t *)kv->v_codebooks;
    a.seq_lens = kv->seq_lens;
    a.q = (const half_t *)q;
    a.out = (half_t *)out;
    a.ws = (float *)ws;
    a.B = kv->B;
    a.H = kv->H;
    a.T = kv->T;
    a.E = kv->n_entries;
    a.G = kv->cb_groups;
    attn_split(kv, &a.S, &a.tc);
    a.scale2 = sm_scale * kLog2e;
    {
        int pg = (kv->D / kv->v) / kv->cb_groups, sh = 0;
        while ((1 << sh) < pg) ++sh;
        if ((1 << sh) != pg) return VQ_ERR_UNSUPPORTED;
        a.pg_shift = sh;
    }
    const bool one = kv->cb_groups == 1;
    if (kv->v == 8) return one ? run_attn<8, true>(a, s) : run_attn<8, false>(a, s);
    if (kv->v == 4) return one ? run_attn<4, true>(a, s) : run_attn<4, false>(a, s);
    return one ? run_attn<2, true>(a, s) : run_attn<2, false>(a, s);
}

}  // namespace vq
