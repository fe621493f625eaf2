// Decode attention over a VQ KV cache, CHANNEL-PARALLEL (codebook-centric) variant for caches with one codebook per
// channel sub-space (coupled quantization: VQ-LLM, arXiv 2503.02236, Sec. III-B and Tbl. IV; dataflow of Sec. VI-A).
//
// The token-parallel kernel (attn.hip) gives every workgroup all channels of its tokens, so a workgroup needs all G
// codebooks of a head and side in LDS (64 KiB per side for G = 32) and switches codebook with every sub-vector.
// Here the channel axis is cut instead: workgroup (b, h, c) owns the 32 channels [32 c, 32 c + 32) of a head and
// stages only the G / C codebooks of those channels (C = D / 32 channel groups).  The price is the paper's
// "global accumulation": a token's score q . K[t] is a sum over all channels, so every channel group writes its
// partial inner products to global memory, a second kernel adds them (fixed order), takes the softmax over the
// tokens and writes the probabilities, and a third kernel -- channel-parallel again, V's channels are independent
// of each other -- accumulates p_t V[t] for its 32 channels.  Three launches and (C + 1) T floats per (b, h) of
// extra traffic; the code bytes are read in 32 / v-byte pieces of each token's row.
//
// Everything is order-fixed: repeated calls give identical bits.
#include "vq_common.h"

namespace vq {

constexpr int kCpChannels = 32;   // channels per workgroup
constexpr int kCpThreads = 256;

struct AttnCpArgs {
    const uint8_t *k_codes, *v_codes;   // [B][H][T][D/v]
    const half_t *k_cb, *v_cb;          // [H][G][E][v]
    const half_t *q;                    // [B][H][D]
    half_t *out;                        // [B][H][D]
    const int *seq_lens;
    float *scores;                      // [B*H][C][T] partial inner products
    float *prob;                        // [B*H][T]
    int B, H, D, T, E, G, C;
    float sm_scale;
};

__device__ __forceinline__ int cp_len(const AttnCpArgs &a, int b) {
    return a.seq_lens ? min(max(a.seq_lens[b], 0), a.T) : a.T;
}

// Stages the G / C codebooks of channel group c of one side into LDS (fp16, as stored).
template <int V>
__device__ __forceinline__ void cp_stage(const half_t *cb, int h, int c, const AttnCpArgs &a, half_t *lds) {
    const int per = a.G / a.C;                                  // codebooks of this channel group
    const size_t halves = (size_t)per * a.E * V;
    const half_t *src = cb + ((size_t)h * a.G + (size_t)c * per) * a.E * V;
    for (size_t i = threadIdx.x; i < halves / 8; i += kCpThreads)
        reinterpret_cast<uint4 *>(lds)[i] = reinterpret_cast<const uint4 *>(src)[i];
    __syncthreads();
}

// The PC = 32 / V codes of token t that belong to channel group c.
template <int V>
__device__ __forceinline__ void cp_codes(const uint8_t *codes, size_t bh, int t, int c, const AttnCpArgs &a, uint8_t (&out)[kCpChannels / V]) {
    constexpr int PC = kCpChannels / V;
    const uint8_t *p = codes + (bh * a.T + t) * (size_t)(a.D / V) + (size_t)c * PC;
    if constexpr (PC == 16) {
        const V16 w = ld16(p);
#pragma unroll
        for (int i = 0; i < 16; ++i) out[i] = w.b[i];
    } else if constexpr (PC == 8) {
        const V8 w = ld8(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = (uint8_t)(w.w[i / 4] >> (8 * (i % 4)));
    } else {
        const uint32_t w = *reinterpret_cast<const uint32_t *>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = (uint8_t)(w >> (8 * i));
    }
}

// Entry `code` of the codebook that sub-vector j (0 .. PC - 1) of this channel group uses.
template <int V>
__device__ __forceinline__ const half_t *cp_entry(const half_t *lds, int j, int code, const AttnCpArgs &a) {
    constexpr int PC = kCpChannels / V;
    const int per = a.G / a.C;               // codebooks of the group; sub-vector j uses codebook j * per / PC
    return lds + ((size_t)(j * per / PC) * a.E + code) * V;
}

// (1) partial inner products of channel group c: scores[bh][c][t] = sum over the group's 32 channels of q K[t]
template <int V>
__global__ __launch_bounds__(kCpThreads) void attn_cp_scores_kernel(AttnCpArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    half_t *lds = reinterpret_cast<half_t *>(smem);
    constexpr int PC = kCpChannels / V;
    const int bh = blockIdx.x, c = blockIdx.y, h = bh % a.H, b = bh / a.H;
    const int len = cp_len(a, b);
    const int t = blockIdx.z * kCpThreads + threadIdx.x;
    if ((int)blockIdx.z * kCpThreads >= len) return;             // (whole workgroup: nothing of this range is valid)
    cp_stage<V>(a.k_cb, h, c, a, lds);
    float qf[kCpChannels];
    const half_t *qp = a.q + (size_t)bh * a.D + c * kCpChannels;
#pragma unroll
    for (int i = 0; i < kCpChannels; ++i) qf[i] = (float)qp[i];
    if (t >= len) return;
    uint8_t code[PC];
    cp_codes<V>(a.k_codes, (size_t)bh, t, c, a, code);
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < PC; ++j) {
        const half_t *e = cp_entry<V>(lds, j, code[j], a);
#pragma unroll
        for (int i = 0; i < V; ++i) s += qf[j * V + i] * (float)e[i];
    }
    a.scores[((size_t)bh * a.C + c) * a.T + t] = s;
}

// (2) global accumulation and softmax over the tokens of one (b, h): prob[t] = exp(s_t - m) / l
__global__ __launch_bounds__(kCpThreads) void attn_cp_softmax_kernel(AttnCpArgs a) {
    __shared__ float red[kCpThreads / 64];
    const int bh = blockIdx.x, b = bh / a.H;
    const int len = cp_len(a, b);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    auto block_reduce = [&](float v, bool is_max) {
        for (int m = 32; m >= 1; m >>= 1) {
            const float o = __shfl_xor(v, m, 64);
            v = is_max ? fmaxf(v, o) : v + o;
        }
        __syncthreads();                      // (red is reused)
        if (lane == 0) red[wave] = v;
        __syncthreads();
        float r = red[0];
        for (int w = 1; w < kCpThreads / 64; ++w) r = is_max ? fmaxf(r, red[w]) : r + red[w];
        return r;
    };
    float *prob = a.prob + (size_t)bh * a.T;
    // pass 1: the summed, scaled scores (kept in prob) and their maximum
    float mx = -INFINITY;
    for (int t = threadIdx.x; t < len; t += kCpThreads) {
        float s = 0.f;
        for (int c = 0; c < a.C; ++c) s += a.scores[((size_t)bh * a.C + c) * a.T + t];   // channel groups in ascending order
        s *= a.sm_scale;
        prob[t] = s;
        mx = fmaxf(mx, s);
    }
    mx = block_reduce(mx, true);
    // pass 2: exponentials and their sum (each thread re-reads what it wrote itself)
    float sum = 0.f;
    for (int t = threadIdx.x; t < len; t += kCpThreads) {
        const float e = __expf(prob[t] - mx);
        prob[t] = e;
        sum += e;
    }
    sum = block_reduce(sum, false);
    const float inv = sum > 0.f ? 1.f / sum : 0.f;
    for (int t = threadIdx.x; t < len; t += kCpThreads) prob[t] *= inv;
}

// (3) the 32 output channels of channel group c: out[c*32 + i] = sum_t prob[t] V[t][c*32 + i]
template <int V>
__global__ __launch_bounds__(kCpThreads) void attn_cp_values_kernel(AttnCpArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    half_t *lds = reinterpret_cast<half_t *>(smem);
    __shared__ float part[kCpThreads / 64][kCpChannels];
    constexpr int PC = kCpChannels / V;
    const int bh = blockIdx.x, c = blockIdx.y, h = bh % a.H, b = bh / a.H;
    const int len = cp_len(a, b);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    cp_stage<V>(a.v_cb, h, c, a, lds);
    float acc[kCpChannels];
#pragma unroll
    for (int i = 0; i < kCpChannels; ++i) acc[i] = 0.f;
    const float *prob = a.prob + (size_t)bh * a.T;
    for (int t = threadIdx.x; t < len; t += kCpThreads) {       // each lane its tokens in ascending order
        const float p = prob[t];
        uint8_t code[PC];
        cp_codes<V>(a.v_codes, (size_t)bh, t, c, a, code);
#pragma unroll
        for (int j = 0; j < PC; ++j) {
            const half_t *e = cp_entry<V>(lds, j, code[j], a);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[j * V + i] += p * (float)e[i];
        }
    }
    // lanes of a wavefront (butterfly), then the wavefronts in ascending order
#pragma unroll
    for (int i = 0; i < kCpChannels; ++i) {
        float v = acc[i];
        for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
        if (lane == 0) part[wave][i] = v;
    }
    __syncthreads();
    if (threadIdx.x < kCpChannels) {
        float v = part[0][threadIdx.x];
        for (int w = 1; w < kCpThreads / 64; ++w) v += part[w][threadIdx.x];
        a.out[(size_t)bh * a.D + c * kCpChannels + threadIdx.x] = (half_t)v;
    }
}

// Which caches the variant takes: D a multiple of 32, as many codebook groups as divide evenly over the D / 32 channel
// groups, a channel group's codebooks within 60 KiB, codes readable in aligned pieces.
bool attn_channel_supported(const vq_kv_t *kv) {
    if (kv->v != 2 && kv->v != 4 && kv->v != 8) return false;
    if (kv->D <= 0 || kv->D % kCpChannels != 0) return false;
    const int C = kv->D / kCpChannels;
    if (kv->cb_groups % C != 0) return false;
    const size_t cb_bytes = (size_t)(kv->cb_groups / C) * kv->n_entries * kv->v * sizeof(half_t);
    return cb_bytes <= 60 * 1024 && cb_bytes % 16 == 0;   // (beside 512 bytes of static LDS, within the default 64 KiB)
}

size_t attn_channel_workspace(const vq_kv_t *kv) {
    const size_t C = (size_t)kv->D / kCpChannels;
    return (size_t)kv->B * kv->H * (C + 1) * kv->T * sizeof(float);
}

int launch_attn_channel(const vq_kv_t *kv, const void *q, float sm_scale, void *out, void *ws, hipStream_t s) {
    AttnCpArgs a;
    a.k_codes = (const uint8_t *)kv->k_codes;
    a.v_codes = (const uint8_t *)kv->v_codes;
    a.k_cb = (const half_t *)kv->k_codebooks;
    a.v_cb = (const half_t *)kv->v_codebooks;
    a.q = (const half_t *)q;
    a.out = (half_t *)out;
    a.seq_lens = kv->seq_lens;
    a.B = kv->B; a.H = kv->H; a.D = kv->D; a.T = kv->T; a.E = kv->n_entries; a.G = kv->cb_groups;
    a.C = kv->D / kCpChannels;
    a.sm_scale = sm_scale;
    a.scores = (float *)ws;
    a.prob = a.scores + (size_t)kv->B * kv->H * a.C * kv->T;
    const size_t lds = (size_t)(a.G / a.C) * a.E * kv->v * sizeof(half_t);
    const int bh = kv->B * kv->H, ranges = (kv->T + kCpThreads - 1) / kCpThreads;
    // (an empty cache: no scores; the last kernel alone writes the zeros)
#define VQ_CP(V)                                                                                   \
    do {                                                                                           \
        if (ranges > 0) {                                                                          \
            attn_cp_scores_kernel<V><<<dim3(bh, a.C, ranges), kCpThreads, lds, s>>>(a);            \
            if (int st = launch_status()) return st;                                               \
            attn_cp_softmax_kernel<<<bh, kCpThreads, 0, s>>>(a);                                   \
            if (int st = launch_status()) return st;                                               \
        }                                                                                          \
        attn_cp_values_kernel<V><<<dim3(bh, a.C), kCpThreads, lds, s>>>(a);                        \
    } while (0)
    if (kv->v == 8)
        VQ_CP(8);
    else if (kv->v == 4)
        VQ_CP(4);
    else
        VQ_CP(2);
#undef VQ_CP
    return launch_status();
}

}  // namespace vq
