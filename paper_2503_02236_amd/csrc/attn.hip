// VQ-attn (decode) for gfx950: out[b][h] = softmax_t(sm_scale * q . K[t]) . V[t] over a KV
// cache stored as uint8 VQ codes.  Formula: VQ-LLM (arXiv 2503.02236) Sec. II-B; setup
// VQ<4,8,1>, 32 heads x 128 channels: Sec. III-A; token-parallel split with a merge of the
// local softmax statistics: Sec. III-B (flash-decoding dataflow of Fig. 5).
//
// Mapping (wave64): four lanes share a token.  Lane (tok = lane % 16, g = lane / 16) owns channels
// [32 g, 32 g + 32) of token tok of the current 16-token step.
//   K side: the scores come from the matrix cores.  v_mfma_f32_16x16x32_f16 takes, per lane, 8
//   consecutive k of one column as its B operand: with k = channel and column = token that is
//   8 / v dequantized sub-vectors of the lane's token, gathered from the LDS codebook straight into the
//   operand registers (layout fusion, Sec. VI-B: no shuffle, no LDS round trip).  The A operand is q,
//   the same in all 16 rows, so every accumulator row holds the score and each of a token's four
//   lanes reads its token's score from its own registers.  Four MFMAs cover the 128 channels.
//   V side: the lane dequantizes its 32 channels of the token's V vector and adds p_t * V[t] into 32
//   PRIVATE fp32 accumulators.  The column-wise accumulation over tokens that forces a shared-memory
//   round trip in the paper's baseline (Sec. III-B, Fig. 6) is deferred to one butterfly over the 16
//   token lanes at the very end, so dequantized values never travel through LDS.
// Only ~130 registers per lane are needed, so 16 wavefronts per CU hide the gather latency.
// Codebooks live in LDS (2 KB each for one codebook per head and side).
//
// A workgroup streams over its token range in tiles of 16 code bytes per lane and side (32 tokens
// per wavefront for v = 4).  The codes of the
// next two tiles are in flight while a tile is processed (register double buffers), so the HBM stream
// and the LDS gathers overlap.  Softmax is kept online per wavefront: a wave-uniform running
// maximum; the accumulators are rescaled only when a tile raises it (rare after the first tiles).
#include "vq_common.h"

namespace vq {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kAttnMinTokens = 512;   // do not split token ranges below this
constexpr int kAttnTargetWgs = 512;   // two workgroups per compute unit

constexpr int kAttnWaves = 8;   // wavefronts per workgroup
// 16-token steps per wavefront and tile: 16 bytes of codes per lane, tile and side
constexpr int attn_steps(int v) { return v / 2; }
constexpr int attn_tile(int v) { return kAttnWaves * 16 * attn_steps(v); }  // tokens per workgroup and tile

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

// Butterfly sum of acc[0..32) over the 16 lanes of a row (lanes that share lane / 16); afterwards
// lane l holds the totals of elements 2 (l % 16) and 2 (l % 16) + 1 in acc[0], acc[1].  In every step
// a lane keeps one half of its values and adds the partner lane's copy of that half.
__device__ __forceinline__ void row_reduce_scatter(float (&acc)[32], int lane) {
#pragma unroll
    for (int step = 0; step < 4; ++step) {
        const int m = 8 >> step;        // lane mask
        const int half = 16 >> step;    // elements kept
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

// Load of one codebook entry (v halves) from an LDS byte address into bytes [at, at + 2 v) of a
// 64-byte register block.
template <int V>
__device__ __forceinline__ void lds_entry_into(V16 (&blk)[4], int at, unsigned addr) {
    if constexpr (V == 8) {
        typedef unsigned raw_t __attribute__((ext_vector_type(4)));
        const raw_t r = *reinterpret_cast<const __attribute__((address_space(3))) raw_t *>((uintptr_t)addr);
        blk[at / 16].w[0] = r.x; blk[at / 16].w[1] = r.y; blk[at / 16].w[2] = r.z; blk[at / 16].w[3] = r.w;
    } else if constexpr (V == 4) {
        typedef unsigned raw_t __attribute__((ext_vector_type(2)));
        const raw_t r = *reinterpret_cast<const __attribute__((address_space(3))) raw_t *>((uintptr_t)addr);
        blk[at / 16].w[(at % 16) / 4] = r.x; blk[at / 16].w[(at % 16) / 4 + 1] = r.y;
    } else {
        blk[at / 16].w[(at % 16) / 4] = *reinterpret_cast<const __attribute__((address_space(3))) unsigned *>((uintptr_t)addr);
    }
}

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
// The lookups of a tile form one sequence of groups (per 16-token step: the lane's 32 K channels, later
// its 32 V channels); the LDS gathers of group n+1 are written before the arithmetic of group n, and the
// sequence continues across the K/V boundary and into the next tile, so the LDS queue never drains.
//
// SEQ: sequences per workgroup (1 or 2).  With 2, wavefronts 0-7 and 8-15 attend two batch entries of
// the SAME head and share its codebooks in LDS: the layout with one codebook per sub-space needs 128 KiB
// for them, so only one workgroup fits a CU, and this keeps 16 wavefronts on it and stages the
// codebooks once per pair.
//
// REP (v = 4, one codebook per head and side): every entry is stored 32 times, copy c of entry e at byte
// e * 256 + c * 8, and lane l reads copy l % 32.  LDS serves the 8-byte reads of 32 consecutive lanes in one pass
// if they fall into 32 different 8-byte columns (address / 8 mod 32) and needs one more pass per further address
// in a column: the 32 lanes of a pass now sit in 32 different columns whatever their codes are, where random
// entries of one shared copy take 2.4 passes (the paper's takeaway on shared-memory bank conflicts, Sec. III-B).
// 64 KiB per side; one workgroup of two sequences (SEQ = 2) per compute unit.  An address is one byte
// permute: (code << 8) | lane constant, the V side's constant carrying its base of 64 KiB.
constexpr int kAttnRepCopies = 32;
constexpr int kAttnRepSide = 65536;   // bytes per side: 256 entries x 32 copies x 8 bytes
constexpr int kAttnRepMinWgs = 192;   // fewer workgroups than this: two small workgroups per CU (shared copy) fill the chip better

template <int V, bool ONE, int SEQ, bool REP = false>
__global__ __launch_bounds__(kAttnWaves * 64 * SEQ) __attribute__((amdgpu_waves_per_eu(4, 4))) void attn_decode_kernel(AttnArgs a) {
    static_assert(!REP || (V == 4 && ONE), "replicated codebooks: one codebook of 8-byte entries per side");
    constexpr int D = 128;
    constexpr int P = D / V;          // codes (bytes) per token and side
    constexpr int CB = 32 / V;        // codes (bytes) per lane, step and side: the lane's 32 channels
    constexpr int CW = (CB + 3) / 4;  // dwords holding them
    constexpr int NS = attn_steps(V);
    constexpr int TILE = attn_tile(V);
    constexpr unsigned SH = V == 8 ? 4 : V == 4 ? 3 : 2;  // log2 of the entry size in bytes
    extern __shared__ __align__(16) unsigned char smem[];
    // Entry addresses are formed as plain LDS byte offsets (shifted code + constant), which is only
    // right if the dynamic LDS block starts at LDS address 0: true for a kernel without static LDS.
    // The launcher checks that (kernel_setup) and returns an error instead of launching otherwise.
    const int cb_bytes = a.G * a.E * V * 2;        // per side
    const int v_off = REP ? kAttnRepSide : ONE ? 4096 : cb_bytes;       // LDS offset of the V codebook
    const int tid = threadIdx.x, lane = tid & 63;
    const int seq = (tid >> 6) / kAttnWaves, wave = (tid >> 6) % kAttnWaves;  // sequence of the workgroup, wavefront in it
    const int tok = lane & 15, g = lane >> 4;
    const int h = blockIdx.x % a.H, split = blockIdx.y;
    const int b = (blockIdx.x / a.H) * SEQ + seq;
    const bool valid = b < a.B;                      // an odd batch leaves the last pair half empty
    const int bh = (valid ? b : 0) * a.H + h;
    float *xw = reinterpret_cast<float *>(smem + 2 * (size_t)v_off) + seq * (kAttnWaves * (D + 2));  // [waves][D] + [waves] + [waves]
    float *xw_m = xw + kAttnWaves * D, *xw_l = xw_m + kAttnWaves;
    const int len = !valid ? 0 : a.seq_lens ? min(max(a.seq_lens[b], 0), a.T) : a.T;
    const int start = split * a.tc;
    const int end = min(len, start + a.tc);  // this sequence attends tokens [start, end) here
    // nothing to attend in this token range: the wavefronts still take part in the barriers and
    // deliver an empty partial result (uniform over the wavefronts of a sequence)
    const bool active = start < end;

    const int ntiles = active ? (end - start + TILE - 1) / TILE : 0;
    const size_t row0 = (size_t)bh * a.T;
    // token of (tile it, step s) for this lane: t_lane + it * TILE + s * 16
    const int t_lane = start + wave * (16 * NS) + tok;

    // codes of one tile and side -> registers (the lane's CB bytes of each of its NS tokens); tokens
    // past the end re-read the last valid token (their scores are masked)
    auto load_codes = [&](const uint8_t *codes, int it, uint32_t (&buf)[NS][CW]) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int t = min(t_lane + it * TILE + s * 16, end - 1);
            const uint8_t *cp = codes + (row0 + t) * P + g * CB;
            if constexpr (CB == 4) {
                buf[s][0] = *reinterpret_cast<const uint32_t *>(cp);
            } else if constexpr (CB == 8) {
                V8 c = ld8(cp);
                buf[s][0] = c.w[0]; buf[s][1] = c.w[1];
            } else {
                V16 c = ld16(cp);
#pragma unroll
                for (int i = 0; i < 4; ++i) buf[s][i] = c.w[i];
            }
        }
    };

    // 1. codebooks of this head (both sides): global loads first, they are the first to be needed
    const int n16 = cb_bytes / 16;
    const uint4 *ks = reinterpret_cast<const uint4 *>(a.k_cb + (size_t)h * (cb_bytes / 2));
    const uint4 *vs = reinterpret_cast<const uint4 *>(a.v_cb + (size_t)h * (cb_bytes / 2));
    uint4 kst = make_uint4(0, 0, 0, 0), vst = kst;
    if (!REP && tid < n16) {
        kst = ks[tid];
        vst = vs[tid];
    }
    // 2. codes of the first two tiles, and q as the A operands of the four MFMAs: channels
    //    32 g + 8 i .. + 7 (the same for every row of the operand)
    uint32_t kA[NS][CW] = {}, vA[NS][CW] = {}, kB[NS][CW] = {}, vB[NS][CW] = {};
    half8_t qop[4] = {};
    if (active) {
        load_codes(a.k_codes, 0, kA);
        load_codes(a.v_codes, 0, vA);
        load_codes(a.k_codes, 1, kB);
        load_codes(a.v_codes, 1, vB);
#pragma unroll
        for (int i = 0; i < 4; ++i) qop[i] = ld16(a.q + (size_t)bh * D + 32 * g + 8 * i).h8;
    }
    if constexpr (REP) {
        // 32 copies of every entry: consecutive lanes write consecutive 8-byte units (copy c = unit % 32 of entry
        // unit / 32); the 32 lanes of a copy set read one global address
        const uint2 *k8 = reinterpret_cast<const uint2 *>(ks), *v8 = reinterpret_cast<const uint2 *>(vs);
        for (int u = tid; u < a.E * kAttnRepCopies; u += (int)blockDim.x) {
            reinterpret_cast<uint2 *>(smem)[u] = k8[u >> 5];
            reinterpret_cast<uint2 *>(smem + kAttnRepSide)[u] = v8[u >> 5];
        }
    } else {
        if (tid < n16) {
            reinterpret_cast<uint4 *>(smem)[tid] = kst;
            reinterpret_cast<uint4 *>(smem + v_off)[tid] = vst;
        }
        for (int i = tid + (int)blockDim.x; i < n16; i += (int)blockDim.x) {  // larger codebooks
            reinterpret_cast<uint4 *>(smem)[i] = ks[i];
            reinterpret_cast<uint4 *>(smem + v_off)[i] = vs[i];
        }
    }
    __syncthreads();

    const unsigned sh = SH;
    // gathers of one group: the CB entries of step s, into a 64-byte register block in channel order
    // REP: lane constants of the two sides, byte 0 = 8 (lane % 32), byte 2 = the side's base / 65536
    const unsigned rep_k = (unsigned)(lane & 31) * 8u, rep_v = rep_k + (unsigned)kAttnRepSide;
    auto gather = [&](const uint32_t (&codes)[NS][CW], int s, int base, V16 (&blk)[4]) {
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            const unsigned w = codes[s][c / 4];
            if constexpr (REP) {
                // address bytes: [lane constant b0][code][lane constant b2][0]
                const unsigned sel = 0x0c020000u | ((4u + (unsigned)(c % 4)) << 8);
                lds_entry_into<V>(blk, c * V * 2, __builtin_amdgcn_perm(w, base ? rep_v : rep_k, sel));
                continue;
            }
            unsigned off = (c % 4) == 0 ? byte_shl<0>(w, sh)
                           : (c % 4) == 1 ? byte_shl<1>(w, sh)
                           : (c % 4) == 2 ? byte_shl<2>(w, sh) : byte_shl<3>(w, sh);
            if (!ONE) off += ((unsigned)((g * CB + c) >> a.pg_shift) * a.E) << SH;
            lds_entry_into<V>(blk, c * V * 2, (unsigned)base + off);
        }
    };

    float acc[32];  // channels 32 g .. 32 g + 31 of sum_t p_t V[t]
#pragma unroll
    for (int d = 0; d < 32; ++d) acc[d] = 0.f;
    float lsum = 0.f;          // per lane (every token is counted by its four lanes)
    float m_run = -INFINITY;   // wave-uniform running maximum of the scores (log2 domain)

    V16 eb[2][4];  // entries of the group being used and of the one in flight
    gather(kA, 0, 0, eb[0]);  // (codes are zero when there is nothing to attend: entry 0, unused)

    // kn: K codes of the following tile (the other register buffer)
    auto tile_step = [&](int it, uint32_t (&kc)[NS][CW], uint32_t (&vc)[NS][CW], const uint32_t (&kn)[NS][CW]) {
        // ---- scores.  Masked tokens get -inf through an additive bias (a select on the finished score
        // would make the compiler branch around the arithmetic and move the gathers).
        float sc[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (s + 1 < NS)
                gather(kc, s + 1, 0, eb[(s + 1) & 1]);
            else
                gather(vc, 0, v_off, eb[NS & 1]);
            float4_t c4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 4; ++i) c4 = __builtin_amdgcn_mfma_f32_16x16x32_f16(qop[i], eb[s & 1][i].h8, c4, 0, 0, 0);
            const float bias = (t_lane + it * TILE + s * 16 < end) ? 0.f : -INFINITY;
            sc[s] = __builtin_fmaf(c4[0], a.scale2, bias);
        }
        load_codes(a.k_codes, it + 2, kc);  // the K codes of this tile are used up

        // ---- online softmax: raise the wave's running maximum if needed (uniform branch)
        float tmax = sc[0];
#pragma unroll
        for (int s = 1; s < NS; ++s) tmax = fmaxf(tmax, sc[s]);
        tmax = wave_max_uniform(tmax);
        if (tmax > m_run) {
            const float f = __builtin_amdgcn_exp2f(m_run - tmax);  // 0 while nothing was accumulated
#pragma unroll
            for (int d = 0; d < 32; ++d) acc[d] *= f;
            lsum *= f;
            m_run = tmax;
        }

        // ---- acc += p_t * V[t] on the lane's 32 channels
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (s + 1 < NS)
                gather(vc, s + 1, v_off, eb[(NS + s + 1) & 1]);
            else
                gather(kn, 0, 0, eb[0]);  // first K group of the next tile (2 NS is even)
            const float p_t = sc[s] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sc[s] - m_run);
            lsum += p_t;
            const V16 (&ev)[4] = eb[(NS + s) & 1];
#pragma unroll
            for (int d = 0; d < 32; ++d) acc[d] += p_t * (float)ev[d / 8].h8[d % 8];
        }
        load_codes(a.v_codes, it + 2, vc);
    };

    for (int it = 0; it < ntiles; it += 2) {
        tile_step(it, kA, vA, kB);
        if (it + 1 < ntiles) tile_step(it + 1, kB, vB, kA);
    }

    // ---- reduce over the 16 token lanes, then over the wavefronts (fixed order) -------------
    row_reduce_scatter(acc, lane);
    lsum = wave_sum(lsum) * 0.25f;  // four lanes per token
    xw[wave * D + 32 * g + 2 * tok] = acc[0];
    xw[wave * D + 32 * g + 2 * tok + 1] = acc[1];
    if (lane == 0) {
        xw_m[wave] = m_run;
        xw_l[wave] = lsum;
    }
    __syncthreads();
    if (valid && tid - seq * (kAttnWaves * 64) < D) {
        const int d = tid - seq * (kAttnWaves * 64);
        float M = xw_m[0];
#pragma unroll
        for (int w = 1; w < kAttnWaves; ++w) M = fmaxf(M, xw_m[w]);
        float L = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) {
            float wgt = (xw_m[w] == -INFINITY) ? 0.f : exp2f(xw_m[w] - M);
            L += xw_l[w] * wgt;
            o += xw[w * D + d] * wgt;
        }
        if (a.S == 1) {
            a.out[(size_t)bh * D + d] = (half_t)(L > 0.f ? o / L : 0.f);
        } else {
            float *wp = a.ws + ((size_t)bh * a.S + split) * (D + 2);
            wp[d] = o;
            if (d == 0) {
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
    const int tile = attn_tile(kv->v);
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

template <int V, bool ONE, int SEQ, bool REP = false>
static int run_attn_seq(const AttnArgs &a, hipStream_t s) {
    const size_t side = REP ? (size_t)kAttnRepSide : ONE ? 4096 : (size_t)a.G * a.E * V * sizeof(half_t);  // matches the kernel's layout
    size_t lds = 2 * side + (size_t)SEQ * kAttnWaves * (128 + 2) * sizeof(float);
    // the kernel forms absolute LDS addresses: refused here, with an error, if it ever had static LDS
    static KernelSetup setup;
    if (int st = kernel_setup(reinterpret_cast<const void *>(&attn_decode_kernel<V, ONE, SEQ, REP>), lds, true, setup)) return st;
    const int groups = (a.B + SEQ - 1) / SEQ;
    attn_decode_kernel<V, ONE, SEQ, REP><<<dim3(groups * a.H, a.S), kAttnWaves * 64 * SEQ, lds, s>>>(a);
    if (a.S > 1) attn_merge_kernel<<<a.B * a.H, 128, 0, s>>>(a.ws, a.out, a.S);
    return launch_status();
}

template <int V, bool ONE>
static int run_attn(const AttnArgs &a, hipStream_t s) {
    // two sequences of a head per workgroup when the codebooks are so large that only one workgroup fits a CU
    const size_t side = ONE ? 4096 : (size_t)a.G * a.E * V * sizeof(half_t);
    if (!ONE && a.B >= 2 && 2 * (2 * side + 4200) > 160 * 1024) return run_attn_seq<V, false, 2>(a, s);
    if constexpr (ONE && V == 4) {
        // replicated codebooks (no bank conflicts) where pairs of sequences give every compute unit a workgroup:
        // 128 KiB of LDS per workgroup, so exactly one fits
        const long long wgs = (long long)((a.B + 1) / 2) * a.H * a.S;
        if (a.B >= 2 && a.E * kAttnRepCopies * 8 <= kAttnRepSide && wgs >= kAttnRepMinWgs) return run_attn_seq<4, true, 2, true>(a, s);
    }
    return run_attn_seq<V, ONE, 1>(a, s);
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
