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

// Code i of a canonical code array on the host: uint8, uint16, or the packed 12-bit string (little-endian
// bit string, code i in bits [12 i, 12 i + 12)).
unsigned host_code(const void *codes, int bits, size_t i) {
    if (bits == 8) return ((const uint8_t *)codes)[i];
    if (bits == 16) return ((const uint16_t *)codes)[i];
    const uint8_t *b = (const uint8_t *)codes + (i >> 1) * 3;
    return (i & 1) ? ((unsigned)b[1] >> 4) | ((unsigned)b[2] << 4) : (unsigned)b[0] | (((unsigned)b[1] & 0xFu) << 8);
}
void host_code_store(void *codes, int bits, size_t i, unsigned c) {
    if (bits == 8) {
        ((uint8_t *)codes)[i] = (uint8_t)c;
    } else if (bits == 16) {
        ((uint16_t *)codes)[i] = (uint16_t)c;
    } else {
        uint8_t *b = (uint8_t *)codes + (i >> 1) * 3;
        if (i & 1) {
            b[1] = (uint8_t)((b[1] & 0x0Fu) | ((c & 0xFu) << 4));
            b[2] = (uint8_t)(c >> 4);
        } else {
            b[0] = (uint8_t)c;
            b[1] = (uint8_t)((b[1] & 0xF0u) | ((c >> 8) & 0xFu));
        }
    }
}

// `codes` holds the unpacked codes [n_codes][R]; rewritten in place.  Returns the hot-entry count.
int reorder(const vq_weight_t *w, std::vector<uint16_t> &codes, void *codebooks_out) {
    const int R = w->n_codebooks, E = w->n_entries, v = w->v;
    const size_t n_codes = (size_t)w->N * (w->K / v);  // per codebook
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
        for (size_t i = 0; i < n_codes; ++i) codes[i * R + r] = (uint16_t)rank[codes[i * R + r]];
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
    // every storage width is unpacked into one working array (the packed 12-bit string of VQ<8,12,2> included:
    // two codes in three bytes, N * K/v * R * 3/2 bytes in all)
    const int bits = w_host->code_bits;
    const size_t total = (size_t)w_host->N * (w_host->K / w_host->v) * w_host->n_codebooks;
    std::vector<uint16_t> codes(total);
    for (size_t i = 0; i < total; ++i) {
        const unsigned c = host_code(w_host->codes, bits, i);
        // codes >= n_entries would index past the histogram: reject instead of assuming the precondition
        if (c >= (unsigned)w_host->n_entries) return VQ_ERR_SHAPE;
        codes[i] = (uint16_t)c;
    }
    const int hot = reorder(w_host, codes, codebooks_out_host);
    for (size_t i = 0; i < total; ++i) host_code_store(codes_out_host, bits, i, codes[i]);
    if (hot_entries_out) *hot_entries_out = hot;
    return VQ_OK;
}
