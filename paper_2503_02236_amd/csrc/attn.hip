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
// Scores of a wavefront's tokens are kept in registers: pass 1 computes them and their
// maximum, pass 2 the exponentials and the V accumulation, so nothing is ever rescaled.
#include "vq_common.h"

namespace vq {

constexpr int kAttnNI = 8;                   // tokens per lane per workgroup
constexpr int kAttnTC = 256 * kAttnNI;       // tokens per workgroup (token-range split)
constexpr float kLog2e = 1.4426950408889634f;

struct AttnArgs {
    const uint8_t *k_codes, *v_codes;
    const half_t *k_cb, *v_cb;
    const int *seq_lens;
    const half_t *q;
    half_t *out;
    float *ws;      // [B*H][S][D + 2] partials when S > 1
    int B, H, T, E, G, S;
    int pg_shift;   // log2 of sub-vectors per codebook group
    float scale2;   // sm_scale * log2(e)
};

// Butterfly sum of acc[0..N) over the 64 lanes; afterwards lane l holds the totals of
// elements 2l and 2l+1 in acc[0], acc[1].
template <int N>
__device__ __forceinline__ void lanes_reduce_scatter(float (&acc)[N], int lane) {
    static_assert(N == 128, "written for 128 accumulators");
#pragma unroll
    for (int step = 0; step < 6; ++step) {
        const int m = 32 >> step;       // lane mask
        const int half = 64 >> step;    // elements kept
        const bool upper = (lane & m) != 0;
#pragma unroll
        for (int i = 0; i < 64; ++i) {
            if (i < half) {
                float lo = acc[i], hi = acc[i + half];
                float send = upper ? lo : hi;
                float keep = upper ? hi : lo;
                acc[i] = keep + __shfl_xor(send, m, 64);
            }
        }
    }
}

template <int V>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnArgs a) {
    constexpr int D = 128;
    constexpr int P = D / V;          // codes (bytes) per token and side
    constexpr int NI = kAttnNI;
    extern __shared__ __align__(16) unsigned char smem[];
    const int cb_halves = a.G * a.E * V;  // per side
    half_t *kcb = reinterpret_cast<half_t *>(smem);
    half_t *vcb = kcb + cb_halves;
    float *xw = reinterpret_cast<float *>(smem + (size_t)2 * cb_halves * sizeof(half_t));  // [4][D] + [4] + [4]
    float *xw_m = xw + 4 * D, *xw_l = xw_m + 4;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bh = blockIdx.x, split = blockIdx.y;
    const int b = bh / a.H, h = bh % a.H;
    const int len = a.seq_lens ? min(max(a.seq_lens[b], 0), a.T) : a.T;

    // stage this head's codebooks (both sides) into LDS
    {
        const uint4 *ks = reinterpret_cast<const uint4 *>(a.k_cb + (size_t)h * cb_halves);
        const uint4 *vs = reinterpret_cast<const uint4 *>(a.v_cb + (size_t)h * cb_halves);
        const int n16 = cb_halves / 8;
        for (int i = tid; i < n16; i += 256) {
            reinterpret_cast<uint4 *>(kcb)[i] = ks[i];
            reinterpret_cast<uint4 *>(vcb)[i] = vs[i];
        }
    }
    // query (uniform over the workgroup)
    half2_t qf[D / 2];
    {
        const half2_t *qp = reinterpret_cast<const half2_t *>(a.q + (size_t)bh * D);
#pragma unroll
        for (int i = 0; i < D / 2; ++i) qf[i] = qp[i];
    }
    __syncthreads();

    const size_t row0 = (size_t)bh * a.T;
    const int t_base = split * kAttnTC + wave * 64 + lane;

    // ---- pass 1: scores -----------------------------------------------------------------
    float sc[NI];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int t = t_base + i * 256;
        float s = -INFINITY;
        if (t < len) {
            const uint8_t *cp = a.k_codes + (row0 + t) * P;
            float d = 0.f;
#pragma unroll
            for (int c16 = 0; c16 < P / 16; ++c16) {
                V16 cd = ld16(cp + c16 * 16);
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int p = c16 * 16 + j;
                    const half_t *e = kcb + ((size_t)(p >> a.pg_shift) * a.E + cd.b[j]) * V;
                    if (V == 8) {
                        V16 ev = ld16(e);
#pragma unroll
                        for (int k = 0; k < 4; ++k) d = dot2(ev.h2[k], qf[p * 4 + k], d);
                    } else if (V == 4) {
                        V8 ev = ld8(e);
                        d = dot2(ev.h2[0], qf[p * 2], d);
                        d = dot2(ev.h2[1], qf[p * 2 + 1], d);
                    } else {
                        half2_t ev = *reinterpret_cast<const half2_t *>(e);
                        d = dot2(ev, qf[p], d);
                    }
                }
            }
            s = d * a.scale2;
        }
        sc[i] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);

    // ---- pass 2: p_t = 2^(s_t - max), acc += p_t * V[t] ------------------------------------
    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;
    float lsum = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int t = t_base + i * 256;
        if (t < len) {
            const float p_t = exp2f(sc[i] - mx);
            lsum += p_t;
            const uint8_t *cp = a.v_codes + (row0 + t) * P;
#pragma unroll
            for (int c16 = 0; c16 < P / 16; ++c16) {
                V16 cd = ld16(cp + c16 * 16);
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int p = c16 * 16 + j;
                    const half_t *e = vcb + ((size_t)(p >> a.pg_shift) * a.E + cd.b[j]) * V;
                    if (V == 8) {
                        V16 ev = ld16(e);
#pragma unroll
                        for (int k = 0; k < 8; ++k) acc[p * 8 + k] += p_t * (float)ev.h8[k];
                    } else if (V == 4) {
                        V8 ev = ld8(e);
#pragma unroll
                        for (int k = 0; k < 4; ++k) acc[p * 4 + k] += p_t * (float)ev.h4[k];
                    } else {
                        half2_t ev = *reinterpret_cast<const half2_t *>(e);
                        acc[p * 2] += p_t * (float)ev[0];
                        acc[p * 2 + 1] += p_t * (float)ev[1];
                    }
                }
            }
        }
    }

    // ---- reduce over lanes, then over the four wavefronts (fixed order) ---------------------
    lanes_reduce_scatter<D>(acc, lane);
    lsum = wave_sum(lsum);
    xw[wave * D + 2 * lane] = acc[0];
    xw[wave * D + 2 * lane + 1] = acc[1];
    if (lane == 0) {
        xw_m[wave] = mx;
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

static int attn_splits(const vq_kv_t *kv) {
    int S = (kv->T + kAttnTC - 1) / kAttnTC;
    return S < 1 ? 1 : S;
}

size_t attn_decode_workspace(const vq_kv_t *kv) {
    int S = attn_splits(kv);
    if (S == 1) return 0;
    return (size_t)kv->B * kv->H * S * (kv->D + 2) * sizeof(float);
}

template <int V>
static int run_attn(const AttnArgs &a, hipStream_t s) {
    size_t lds = (size_t)2 * a.G * a.E * V * sizeof(half_t) + (4 * 128 + 8) * sizeof(float);
    static size_t attr_lds = 0;
    if (lds > 64 * 1024 && lds > attr_lds) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_decode_kernel<V>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_lds = lds;
    }
    attn_decode_kernel<V><<<dim3(a.B * a.H, a.S), 256, lds, s>>>(a);
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
    a.S = attn_splits(kv);
    a.scale2 = sm_scale * kLog2e;
    {
        int pg = (kv->D / kv->v) / kv->cb_groups, sh = 0;
        while ((1 << sh) < pg) ++sh;
        if ((1 << sh) != pg) return VQ_ERR_UNSUPPORTED;
        a.pg_shift = sh;
    }
    if (kv->v == 8) return run_attn<8>(a, s);
    if (kv->v == 4) return run_attn<4>(a, s);
    return run_attn<2>(a, s);
}

}  // namespace vq
