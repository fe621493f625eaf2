// Offline frequency reordering of codebook entries (host code, no GPU).
// VQ-LLM (arXiv 2503.02236) Sec. V-B: entries are used very unevenly; sorting them by how often the
// codes point at them and rewriting the codes accordingly puts the hot entries in front, where a
// kernel's on-chip cache (the first entries of the codebook) finds them.  The weight is unchanged:
// entry order is arbitrary as long as the codes follow.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <numeric>
#include <vector>

#include "vq_common.h"

using namespace vq;

namespace {

template <typename CodeT>
int reorder(const vq_weight_t *w, void *codes_out, void *codebooks_out) {
    const int R = w->n_codebooks, E = w->n_entries, v = w->v;
    const size_t n_codes = (size_t)w->N * (w->K / v);  // per codebook
    const CodeT *codes = (const CodeT *)w->codes;
    CodeT *out = (CodeT *)codes_out;
    const uint16_t *cb = (const uint16_t *)w->codebooks;  // fp16 bits, moved verbatim
    uint16_t *cb_out = (uint16_t *)codebooks_out;
    std::vector<uint64_t> count(E);
    std::vector<uint32_t> order(E), rank(E);
    int hot = 0;
    for (int r = 0; r < R; ++r) {
        std::fill(count.begin(), count.end(), 0);
        for (size_t i = 0; i < n_codes; ++i) ++count[codes[i * R + r]];
        std::iota(order.begin(), order.end(), 0u);
        // most used first; equal counts keep their original order, so the result is unique
        std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) { return count[x] > count[y]; });
        for (int pos = 0; pos < E; ++pos) {
            rank[order[pos]] = (uint32_t)pos;
            std::memcpy(cb_out + ((size_t)r * E + pos) * v, cb + ((size_t)r * E + order[pos]) * v, (size_t)v * 2);
        }
        for (size_t i = 0; i < n_codes; ++i) out[i * R + r] = (CodeT)rank[codes[i * R + r]];
        // leading entries that serve half of this codebook's codes
        uint64_t served = 0;
        int n = 0;
        while (n < E && 2 * served < n_codes) served += count[order[n++]];
        hot = n > hot ? n : hot;
    }
    return hot;
}

}  // namespace

extern "C" int vq_reorder_by_frequency(const vq_weight_t *w_host, void *codes_out_host, void *codebooks_out_host,
                                       int *hot_entries_out) {
    if (!w_host || !codes_out_host || !codebooks_out_host) return VQ_ERR_NULL;
    int st = check_weight(w_host, true);
    if (st == VQ_ERR_ALIGN) st = VQ_OK;  // host buffers need no 16-byte alignment
    if (st != VQ_OK) return st;
    if (w_host->cb_tile_n != 0) return VQ_ERR_UNSUPPORTED;  // per-tensor codebooks only
    if (codebooks_out_host == w_host->codebooks) return VQ_ERR_SHAPE;  // entries move: not in place
    if (w_host->N == 0 || w_host->K == 0) {
        std::memcpy(codebooks_out_host, w_host->codebooks, (size_t)w_host->n_codebooks * w_host->n_entries * w_host->v * 2);
        if (hot_entries_out) *hot_entries_out = 0;
        return VQ_OK;
    }
    // codes >= n_entries would index past the histogram: reject instead of assuming the precondition
    int hot = 0;
    const size_t total = (size_t)w_host->N * (w_host->K / w_host->v) * w_host->n_codebooks;
    if (w_host->code_bits == 8) {
        const uint8_t *c = (const uint8_t *)w_host->codes;
        for (size_t i = 0; i < total; ++i)
            if (c[i] >= w_host->n_entries) return VQ_ERR_SHAPE;
        hot = reorder<uint8_t>(w_host, codes_out_host, codebooks_out_host);
    } else {
        const uint16_t *c = (const uint16_t *)w_host->codes;
        for (size_t i = 0; i < total; ++i)
            if (c[i] >= w_host->n_entries) return VQ_ERR_SHAPE;
        hot = reorder<uint16_t>(w_host, codes_out_host, codebooks_out_host);
    }
    if (hot_entries_out) *hot_entries_out = hot;
    return VQ_OK;
}
