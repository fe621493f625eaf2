// On-the-fly KV quantization for gfx950: the codes of new tokens' K and V vectors.
// VQ-LLM (arXiv 2503.02236) Sec. II-A (assignment step: a sub-vector is replaced by the index of its
// closest codebook entry) and Sec. VII "Quantization Overhead" (it runs for the new token in every decode
// step and for all prompt tokens in prefill).
//
// A floating-point comparison decides an integer, so order and precision are part of the definition
// (the paper gives none; this is the reading the CPU reference follows too): squared Euclidean distance
// in fp32, elements in ascending order, every subtraction, multiplication and addition rounded on its own
// (floating-point contraction is switched off for the kernel); strict "<" while walking the entries in
// ascending order, so ties go to the smallest index.
//
// One workgroup per (batch, head, chunk of new tokens): the head's codebooks of one side (G * E entries) are
// staged in LDS (converted to fp32 once when that fits), then L lanes share a (token, sub-vector) item: each
// walks every L-th entry and the L partial winners are merged by (distance, index).  L = 1 for
// prefill-sized calls; a decode step (one token) has only D / v items per head, so 8 lanes split the entries.
#include <type_traits>

#include "vq_common.h"

namespace vq {

constexpr int kQuantTokens = 64;  // new tokens per workgroup (L = 1)

struct KvQuantArgs {
    const half_t *x[2];    // K, V: [B][H][n_new][D]
    const half_t *cb[2];   // [H][G][E][v]
    uint8_t *codes[2];     // [B][H][T][D/v]
    int H, T, D, v, E, G, n_new, pos;
    int L, tokens_per_wg;  // lanes per item (power of two <= 64, divides E), tokens per workgroup
    int both;              // the codebooks of both sides fit LDS together: staged at once, one barrier
    int par;               // 512 threads, the two sides handled side by side by 256 threads each (needs both)
};

template <int V, bool F32>
__global__ __launch_bounds__(512) void kv_quantize_kernel(KvQuantArgs a) {
#pragma clang fp contract(off)  // the distance must not be computed with fused multiply-adds
    extern __shared__ __align__(16) unsigned char smem[];
    typedef typename std::conditional<F32, float, half_t>::type cb_t;
    cb_t *cbl = reinterpret_cast<cb_t *>(smem);
    const int P = a.D / V;
    const int bh = blockIdx.x, h = bh % a.H;
    const int t0 = blockIdx.y * a.tokens_per_wg;
    const int nt = min(a.tokens_per_wg, a.n_new - t0);
    const int cb_halves = a.G * a.E * V;
    const int nthreads = a.par ? 512 : 256;
    const int tx = threadIdx.x % 256;             // thread within its side
    const int side0 = a.par ? (int)threadIdx.x / 256 : 0, side1 = a.par ? side0 + 1 : 2;
    const int L = a.L, sub = tx % L, per_lane = a.E / L;
    // the lane's part of item `local` of this workgroup: which (token, sub-vector), and its elements
    struct Item { bool live; int t, p; };
    auto item_of = [&](int r) {
        const int item = (r * 256 + tx) / L;
        Item it;
        it.live = item < nt * P;
        it.t = t0 + (it.live ? item / P : 0);
        it.p = it.live ? item % P : 0;
        return it;
    };
    auto load_x = [&](int side, const Item &it, float (&xv)[V]) {
        const half_t *xp = a.x[side] + (((size_t)bh * a.n_new + it.t) * a.D) + it.p * V;
        if constexpr (V == 8) {
            const V16 x8 = ld16(xp);
#pragma unroll
            for (int i = 0; i < 8; ++i) xv[i] = (float)x8.h8[i];
        } else if constexpr (V == 4) {
            const V8 x4 = ld8(xp);
#pragma unroll
            for (int i = 0; i < 4; ++i) xv[i] = (float)x4.h4[i];
        } else {
            const half2_t x2 = *reinterpret_cast<const half2_t *>(xp);
            xv[0] = (float)x2[0];
            xv[1] = (float)x2[1];
        }
    };
    // the first item's elements are asked for before the codebooks (they come from further away)
    float x_first[V];
    load_x(side0, item_of(0), x_first);
    auto stage = [&](int side, cb_t *dst) {
        const half_t *src = a.cb[side] + (size_t)h * cb_halves;
        if (F32) {
            for (int i = threadIdx.x; i < cb_halves / 8; i += nthreads) {
                const V16 e8 = ld16(src + i * 8);
#pragma unroll
                for (int k = 0; k < 8; ++k) dst[i * 8 + k] = (cb_t)e8.h8[k];
            }
        } else {
            for (int i = threadIdx.x; i < cb_halves / 8; i += nthreads)
                reinterpret_cast<uint4 *>(dst)[i] = reinterpret_cast<const uint4 *>(src)[i];
        }
    };
    if (a.both) {
        stage(0, cbl);
        stage(1, cbl + cb_halves);
        __syncthreads();
    }
    for (int side = side0; side < side1; ++side) {
        const cb_t *cbs = cbl + (a.both ? side * cb_halves : 0);
        if (!a.both) {
            __syncthreads();  // the previous side's lookups are done before its codebooks are overwritten
            stage(side, cbl);
            __syncthreads();
        }
        // all lanes of a wavefront run the same number of rounds (the merge below uses lane shuffles)
        const int n_items = nt * P, rounds = (n_items * L + 255) / 256;
        for (int r = 0; r < rounds; ++r) {
            const Item it = item_of(r);
            const bool live = it.live;
            const int t = it.t, p = it.p;
            float xv[V];
            if (side == side0 && r == 0) {
#pragma unroll
                for (int i = 0; i < V; ++i) xv[i] = x_first[i];
            } else {
                load_x(side, it, xv);
            }
            const cb_t *grp = cbs + (size_t)(p * a.G / P) * a.E * V;
            // the L lanes of an item take the entries in turn (lane `sub`: sub, sub + L, ...), so that at every
            // step they read L neighbouring entries: with a block of consecutive entries per lane the L
            // addresses of a step are 16 * E / L bytes apart, all in the same LDS banks -- an 8-way conflict
            // that made the walk of a decode step 7 us long.  Each lane still meets its entries in ascending
            // order, so its strict "<" keeps the smallest index among equals.
            int best = sub;
            float best_d = INFINITY;
#pragma unroll 4
            for (int k = 0; k < per_lane; ++k) {
                const int e = sub + k * L;
                float d = 0.f;
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    const float diff = xv[i] - (float)grp[e * V + i];
                    const float sq = diff * diff;
                    d = i == 0 ? sq : d + sq;  // (0 + sq is sq: the same value as the reference's first addition)
                }
                if (d < best_d) {  // strict: the first of equal distances stays
                    best = e;
                    best_d = d;
                }
            }
            // merge the L lanes of the item: smaller distance, then smaller index
            for (int m = 1; m < L; m <<= 1) {
                const float od = __shfl_xor(best_d, m, 64);
                const int oe = __shfl_xor(best, m, 64);
                if (od < best_d || (od == best_d && oe < best)) {
                    best_d = od;
                    best = oe;
                }
            }
            if (live && sub == 0) a.codes[side][((size_t)bh * a.T + a.pos + t) * P + p] = (uint8_t)best;
        }
    }
}

int launch_kv_quantize(const vq_kv_t *kv, const void *k_new, const void *v_new, int n_new, int pos, hipStream_t s) {
    KvQuantArgs a;
    a.x[0] = (const half_t *)k_new;
    a.x[1] = (const half_t *)v_new;
    a.cb[0] = (const half_t *)kv->k_codebooks;
    a.cb[1] = (const half_t *)kv->v_codebooks;
    a.codes[0] = (uint8_t *)const_cast<void *>(kv->k_codes);
    a.codes[1] = (uint8_t *)const_cast<void *>(kv->v_codes);
    a.H = kv->H;
    a.T = kv->T;
    a.D = kv->D;
    a.v = kv->v;
    a.E = kv->n_entries;
    a.G = kv->cb_groups;
    a.n_new = n_new;
    a.pos = pos;
    const size_t cb_elems = (size_t)kv->cb_groups * kv->n_entries * kv->v;
    if (cb_elems * sizeof(half_t) > 64 * 1024 || (cb_elems * sizeof(half_t)) % 16 != 0) return VQ_ERR_UNSUPPORTED;
    const bool f32 = cb_elems * sizeof(float) <= 64 * 1024;  // converted once per workgroup instead of per use
    const size_t one = cb_elems * (f32 ? sizeof(float) : sizeof(half_t));
    a.both = 2 * one <= 64 * 1024;
    const size_t lds = a.both ? 2 * one : one;
    a.tokens_per_wg = n_new < kQuantTokens ? n_new : kQuantTokens;
    // lanes per item: fill the 256 threads when a workgroup has few items (decode), 1 otherwise
    const int items = a.tokens_per_wg * (kv->D / kv->v);
    int L = 1;
    while (L < 64 && items * (L * 2) <= 256 && kv->n_entries % (L * 2) == 0) L *= 2;
    a.L = L;
    // a decode-sized call (one round of items per side) runs the two sides side by side
    a.par = a.both && items * L <= 256;
    const int threads = a.par ? 512 : 256;
    const dim3 grid(kv->B * kv->H, (n_new + a.tokens_per_wg - 1) / a.tokens_per_wg);
#define VQ_KVQ(V)                                                         \
    do {                                                                  \
        if (f32)                                                          \
            kv_quantize_kernel<V, true><<<grid, threads, lds, s>>>(a);    \
        else                                                              \
            kv_quantize_kernel<V, false><<<grid, threads, lds, s>>>(a);   \
    } while (0)
    if (kv->v == 8)
        VQ_KVQ(8);
    else if (kv->v == 4)
        VQ_KVQ(4);
    else
        VQ_KVQ(2);
#undef VQ_KVQ
    return launch_status();
}

}  // namespace vq
