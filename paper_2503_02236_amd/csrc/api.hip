// C ABI of libvqmi: host-side argument validation and dispatch to the gfx950 kernels.
// Operand format and operations: VQ-LLM (arXiv 2503.02236) Sec. II-A, II-B, III-C.
#include <new>

#include "vq_common.h"

namespace vq {

int check_weight(const vq_weight_t *w, bool need_codes) {
    if (!w) return VQ_ERR_NULL;
    if ((need_codes && !w->codes) || !w->codebooks) return VQ_ERR_NULL;
    if (w->N < 0 || w->K < 0) return VQ_ERR_SHAPE;
    if (w->v != 4 && w->v != 8) return VQ_ERR_UNSUPPORTED;
    if (w->code_bits != 8 && w->code_bits != 12 && w->code_bits != 16) return VQ_ERR_UNSUPPORTED;
    if (w->n_codebooks < 1 || w->n_codebooks > 4) return VQ_ERR_UNSUPPORTED;
    if (w->n_entries < 1 || w->n_entries > (1 << w->code_bits)) return VQ_ERR_UNSUPPORTED;
    if (w->K % w->v != 0) return VQ_ERR_SHAPE;
    if (w->code_bits == 12) {
        // a row of the packed string must be whole 12-byte words (8 codes); per-tensor codebooks only
        if (((long)(w->K / w->v) * w->n_codebooks) % 8 != 0) return VQ_ERR_SHAPE;
        if (w->cb_tile_n != 0 || w->cb_tile_k != 0 || w->gemv_pack || w->n_codebooks == 3) return VQ_ERR_UNSUPPORTED;
        // the kernels for this format keep all codebooks in LDS
        if ((size_t)w->n_codebooks * w->n_entries * w->v * 2 > 128 * 1024) return VQ_ERR_UNSUPPORTED;
    }
    if (w->cb_tile_n != 0 || w->cb_tile_k != 0) {  // per-tile codebooks
        if (w->cb_tile_n <= 0 || w->cb_tile_k <= 0) return VQ_ERR_SHAPE;
        if (w->cb_tile_n % 16 != 0 || w->cb_tile_k % 64 != 0 || w->K % w->cb_tile_k != 0) return VQ_ERR_SHAPE;
        if ((size_t)(w->K / w->cb_tile_k) * w->n_codebooks * w->n_entries * w->v * 2 > 128 * 1024)
            return VQ_ERR_UNSUPPORTED;
        if (w->gemv_pack || w->n_codebooks == 3) return VQ_ERR_UNSUPPORTED;
    }
    if ((w->codes && !aligned16(w->codes)) || !aligned16(w->codebooks)) return VQ_ERR_ALIGN;
    if (w->scale && !aligned16(w->scale)) return VQ_ERR_ALIGN;
    return VQ_OK;
}

int check_kv(const vq_kv_t *kv) {
    if (!kv) return VQ_ERR_NULL;
    if (!kv->k_codes || !kv->v_codes || !kv->k_codebooks || !kv->v_codebooks) return VQ_ERR_NULL;
    if (kv->B < 0 || kv->H < 0 || kv->T < 0 || kv->D <= 0) return VQ_ERR_SHAPE;
    if (kv->v != 2 && kv->v != 4 && kv->v != 8) return VQ_ERR_UNSUPPORTED;
    if (kv->n_entries < 1 || kv->n_entries > 256) return VQ_ERR_UNSUPPORTED;
    if (kv->D % kv->v != 0) return VQ_ERR_SHAPE;
    int P = kv->D / kv->v;
    if (kv->cb_groups < 1 || P % kv->cb_groups != 0) return VQ_ERR_SHAPE;
    if (kv->D > 256 || kv->D % 8 != 0) return VQ_ERR_UNSUPPORTED;
    if (!aligned16(kv->k_codes) || !aligned16(kv->v_codes) || !aligned16(kv->k_codebooks) ||
        !aligned16(kv->v_codebooks))
        return VQ_ERR_ALIGN;
    if (kv->seq_lens && (reinterpret_cast<uintptr_t>(kv->seq_lens) & 3u)) return VQ_ERR_ALIGN;
    return VQ_OK;
}

}  // namespace vq

using namespace vq;

extern "C" {

int vq_version(void) { return 100; }

const char *vq_status_str(int status) {
    switch (status) {
        case VQ_OK: return "VQ_OK";
        case VQ_ERR_NULL: return "VQ_ERR_NULL: required pointer is NULL";
        case VQ_ERR_SHAPE: return "VQ_ERR_SHAPE: inconsistent or out-of-range sizes";
        case VQ_ERR_UNSUPPORTED: return "VQ_ERR_UNSUPPORTED: VQ configuration not supported";
        case VQ_ERR_ALIGN: return "VQ_ERR_ALIGN: data pointer not 16-byte aligned";
        case VQ_ERR_WORKSPACE: return "VQ_ERR_WORKSPACE: workspace missing or too small";
        case VQ_ERR_LAUNCH: return "VQ_ERR_LAUNCH: HIP launch failed";
        default: return "unknown vq_status";
    }
}

size_t vq_gemv_workspace(const vq_weight_t *w, int bs) {
    if (!w || bs < 1 || bs > 16) return 0;
    const bool packed = gemv_uses_pack(w, bs);
    if (check_weight(w, !packed) != VQ_OK) return 0;
    if (packed && check_pack(w) != VQ_OK) return 0;
    return gemv_workspace(w, bs);
}

int vq_gemv(const vq_weight_t *w, const void *x, int bs, void *y, void *ws, size_t ws_bytes, void *stream) {
    if (!w) return VQ_ERR_NULL;
    if (bs < 1 || bs > 16) return VQ_ERR_SHAPE;
    const bool packed = gemv_uses_pack(w, bs);
    int st = check_weight(w, !packed);
    if (st != VQ_OK) return st;
    if (packed && (st = check_pack(w)) != VQ_OK) return st;
    if (!x || !y) return VQ_ERR_NULL;
    if (!aligned16(x) || !aligned16(y)) return VQ_ERR_ALIGN;
    size_t need = gemv_workspace(w, bs);
    if (need && (!ws || ws_bytes < need)) return VQ_ERR_WORKSPACE;
    if (ws && !aligned16(ws)) return VQ_ERR_ALIGN;
    if (w->N == 0) return VQ_OK;
    return launch_gemv(w, x, bs, y, ws, static_cast<hipStream_t>(stream));
}

// ---- vq_gemv for callers that cannot allocate: scratch inside the library ------------------------------
namespace {

// Scratch of vq_gemv_noalloc: the partial sums that the re-tiled bs = 1 gemv exchanges between its two kernels.
// One copy per GPU, at an address of its own on each, held until the process ends.  In host code the
// array's name is only a stand-in for the symbol: the address that kernels, copies and fills may use comes
// from hipGetSymbolAddress, once per device, and is kept in scratch_ptr.
constexpr size_t kGemvScratchBytes = 2u << 20;
static __device__ __align__(256) unsigned char scratch[kGemvScratchBytes];
std::atomic<void *> scratch_ptr[kMaxDevices];

int scratch_address(void **out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VQ_ERR_LAUNCH;
    void *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return VQ_ERR_LAUNCH;
        }
        scratch_ptr[dev].store(p, std::memory_order_release);   // (two threads racing here store the same address)
    }
    *out = p;
    return VQ_OK;
}

}  // namespace

int vq_init(void) {
    void *p;
    return scratch_address(&p);
}

size_t vq_gemv_noalloc_max_workspace(void) { return kGemvScratchBytes; }

int vq_gemv_noalloc(const vq_weight_t *w, const void *x, int bs, void *y, void *stream) {
    if (!w) return VQ_ERR_NULL;
    if (bs < 1 || bs > 16) return VQ_ERR_SHAPE;
    const bool packed = gemv_uses_pack(w, bs);
    int st = check_weight(w, !packed);
    if (st != VQ_OK) return st;
    if (packed && (st = check_pack(w)) != VQ_OK) return st;
    const size_t need = gemv_workspace(w, bs);
    if (need > kGemvScratchBytes) return VQ_ERR_WORKSPACE;   // beyond the built-in scratch: use vq_gemv with a workspace
    void *ws = nullptr;
    if (need && (st = scratch_address(&ws)) != VQ_OK) return st;
    // Nothing in the scratch has to start at zero: every partial sum that the second kernel reads is written
    // by the first kernel of the same call.
    return vq_gemv(w, x, bs, y, ws, need ? kGemvScratchBytes : 0, stream);
}

// Every problem of the batch can run from re-tiled codes in one launch.
static bool batch_all_packed(const vq_weight_t *const *w, int count) {
    for (int i = 0; i < count; ++i)
        if (!w[i] || !gemv_uses_pack(w[i], 1) || w[i]->K <= 0 || w[i]->N <= 0) return false;
    return true;
}

static size_t batch_slot(const vq_weight_t *w) { return (gemv_workspace(w, 1) + 255) & ~(size_t)255; }

size_t vq_gemv_batch_workspace(const vq_weight_t *const *w, int count) {
    if (!w || count < 1 || count > VQ_GEMV_BATCH_MAX) return 0;
    size_t total = 0;
    for (int i = 0; i < count; ++i) {
        if (!w[i]) return 0;
        const bool packed = gemv_uses_pack(w[i], 1);
        if (check_weight(w[i], !packed) != VQ_OK || (packed && check_pack(w[i]) != VQ_OK)) return 0;
        total += batch_slot(w[i]);
    }
    return total;
}

int vq_gemv_batch(const vq_weight_t *const *w, const void *const *x, void *const *y, int count, void *ws,
                  size_t ws_bytes, void *stream) {
    if (!w || !x || !y) return VQ_ERR_NULL;
    if (count < 1 || count > VQ_GEMV_BATCH_MAX) return VQ_ERR_SHAPE;
    size_t need = 0;
    for (int i = 0; i < count; ++i) {
        if (!w[i]) return VQ_ERR_NULL;
        const bool packed = gemv_uses_pack(w[i], 1);
        int st = check_weight(w[i], !packed);
        if (st != VQ_OK) return st;
        if (packed && (st = check_pack(w[i])) != VQ_OK) return st;
        if (!x[i] || !y[i]) return VQ_ERR_NULL;
        if (!aligned16(x[i]) || !aligned16(y[i])) return VQ_ERR_ALIGN;
        need += batch_slot(w[i]);
    }
    if (need && (!ws || ws_bytes < need)) return VQ_ERR_WORKSPACE;
    if (ws && !aligned16(ws)) return VQ_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (batch_all_packed(w, count)) return launch_gemv_packed_batch(w, x, y, count, ws, s);
    // canonical codes with whole codebooks in LDS, all of one kind: one launch of the matrix-core gemv
    bool none_packed = true;
    for (int i = 0; i < count; ++i) none_packed = none_packed && !gemv_uses_pack(w[i], 1);
    if (none_packed && gemv_mfma_batch_supported(w, count)) return launch_gemv_mfma_batch(w, x, y, count, s);
    // any other mix: one launch per problem, each with its own slot of the workspace
    size_t off = 0;
    for (int i = 0; i < count; ++i) {
        if (w[i]->N > 0) {
            int st = launch_gemv(w[i], x[i], 1, y[i], (unsigned char *)ws + off, s);
            if (st != VQ_OK) return st;
        }
        off += batch_slot(w[i]);
    }
    return VQ_OK;
}

// Validation of one call of a sequence: every problem must run from re-tiled codes.
static int check_sequence_call(const vq_gemv_call_t *c) {
    if (!c->w || !c->x || !c->y) return VQ_ERR_NULL;
    if (c->count < 1 || c->count > VQ_GEMV_BATCH_MAX) return VQ_ERR_SHAPE;
    for (int i = 0; i < c->count; ++i) {
        const vq_weight_t *w = c->w[i];
        if (!w) return VQ_ERR_NULL;
        if (!w->gemv_pack) return VQ_ERR_UNSUPPORTED;
        if (!gemv_uses_pack(w, 1) || w->K <= 0 || w->N <= 0) return VQ_ERR_UNSUPPORTED;
        int st = check_weight(w, false);
        if (st != VQ_OK) return st;
        if ((st = check_pack(w)) != VQ_OK) return st;
        if (!c->x[i] || !c->y[i]) return VQ_ERR_NULL;
        if (!aligned16(c->x[i]) || !aligned16(c->y[i])) return VQ_ERR_ALIGN;
    }
    return VQ_OK;
}

size_t vq_gemv_sequence_workspace(const vq_gemv_call_t *calls, int n_calls) {
    if (!calls || n_calls < 1) return 0;
    for (int c = 0; c < n_calls; ++c)
        if (check_sequence_call(&calls[c]) != VQ_OK) return 0;
    return gemv_packed_sequence_workspace(calls, n_calls);
}

int vq_gemv_sequence(const vq_gemv_call_t *calls, int n_calls, void *ws, size_t ws_bytes, void *stream) {
    if (!calls) return VQ_ERR_NULL;
    if (n_calls < 1) return VQ_ERR_SHAPE;
    for (int c = 0; c < n_calls; ++c)
        if (int st = check_sequence_call(&calls[c])) return st;
    const size_t need = gemv_packed_sequence_workspace(calls, n_calls);
    if (!ws || ws_bytes < need) return VQ_ERR_WORKSPACE;
    if (!aligned16(ws)) return VQ_ERR_ALIGN;
    return launch_gemv_packed_sequence(calls, n_calls, ws, static_cast<hipStream_t>(stream));
}

// A pipeline is one of two kinds, after its weights: re-tiled codes of a large codebook (the persistent two-image
// kernel), or canonical uint8 codes with small codebooks (the kernel that holds 16 LDS copies of every entry).
struct vq_gemv_pipeline {
    GemvPipeline *impl;
    GemvReplicaList *rep;
};

// 1 if every problem can run on the small-codebook kernel, 0 if none can (or some weight is re-tiled), < 0 on a
// mix or an invalid argument.
static int replica_calls(const vq_gemv_call_t *calls, int n_calls) {
    if (!calls) return VQ_ERR_NULL;
    if (n_calls < 1) return VQ_ERR_SHAPE;
    int yes = 0, no = 0, R = 0;
    for (int c = 0; c < n_calls; ++c) {
        if (!calls[c].w || !calls[c].x || !calls[c].y) return VQ_ERR_NULL;
        if (calls[c].count < 1 || calls[c].count > VQ_GEMV_BATCH_MAX) return VQ_ERR_SHAPE;
        for (int i = 0; i < calls[c].count; ++i) {
            const vq_weight_t *w = calls[c].w[i];
            if (!w) return VQ_ERR_NULL;
            if (w->gemv_pack || check_weight(w, true) != VQ_OK || !gemv_replica_supported(w)) { ++no; continue; }
            if (R && w->n_codebooks != R) return VQ_ERR_UNSUPPORTED;
            R = w->n_codebooks;
            if (!calls[c].x[i] || !calls[c].y[i]) return VQ_ERR_NULL;
            if (!aligned16(calls[c].x[i]) || !aligned16(calls[c].y[i])) return VQ_ERR_ALIGN;
            ++yes;
        }
    }
    if (yes && no) return VQ_ERR_UNSUPPORTED;
    return yes ? 1 : 0;
}
static int count_problems(const vq_gemv_call_t *calls, int n_calls) {
    int n = 0;
    for (int c = 0; c < n_calls; ++c) n += calls[c].count;
    return n;
}

static int check_pipeline_calls(const vq_gemv_call_t *calls, int n_calls) {
    if (!calls) return VQ_ERR_NULL;
    if (n_calls < 1) return VQ_ERR_SHAPE;
    for (int c = 0; c < n_calls; ++c) {
        if (int st = check_sequence_call(&calls[c])) return st;
        for (int i = 0; i < calls[c].count; ++i)
            if (!gemv_pipeline_supports(calls[c].w[i])) return VQ_ERR_UNSUPPORTED;
    }
    return VQ_OK;
}

size_t vq_gemv_pipeline_workspace(const vq_gemv_call_t *calls, int n_calls) {
    const int rep = replica_calls(calls, n_calls);
    if (rep == 1) return gemv_replica_list_workspace(count_problems(calls, n_calls));
    if (rep < 0 || check_pipeline_calls(calls, n_calls) != VQ_OK) return 0;
    return gemv_pipeline_workspace(calls, n_calls);
}

int vq_gemv_pipeline_create(const vq_gemv_call_t *calls, int n_calls, void *ws, size_t ws_bytes, void *stream,
                            vq_gemv_pipeline_t **out) {
    if (!out) return VQ_ERR_NULL;
    *out = nullptr;
    const int rep = replica_calls(calls, n_calls);
    if (rep < 0) return rep;
    if (rep == 0)
        if (int st = check_pipeline_calls(calls, n_calls)) return st;
    const size_t need = rep ? gemv_replica_list_workspace(count_problems(calls, n_calls)) : gemv_pipeline_workspace(calls, n_calls);
    if (!ws || ws_bytes < need) return VQ_ERR_WORKSPACE;
    if (((uintptr_t)ws & 255) != 0) return VQ_ERR_ALIGN;
    vq_gemv_pipeline *h = new (std::nothrow) vq_gemv_pipeline;
    if (!h) return VQ_ERR_LAUNCH;
    h->impl = nullptr;
    h->rep = nullptr;
    const int st = rep ? gemv_replica_list_create(calls, n_calls, ws, static_cast<hipStream_t>(stream), &h->rep)
                       : gemv_pipeline_create(calls, n_calls, ws, static_cast<hipStream_t>(stream), &h->impl);
    if (st != VQ_OK) {
        delete h;
        return st;
    }
    *out = h;
    return VQ_OK;
}

int vq_gemv_pipeline_run(const vq_gemv_pipeline_t *p, void *stream) {
    if (!p || (!p->impl && !p->rep)) return VQ_ERR_NULL;
    if (p->rep) return launch_gemv_replica_list(p->rep, static_cast<hipStream_t>(stream));
    return launch_gemv_pipeline(p->impl, static_cast<hipStream_t>(stream));
}

int vq_gemv_pipeline_status(const vq_gemv_pipeline_t *p, void *stream, int *status) {
    if (!p || (!p->impl && !p->rep) || !status) return VQ_ERR_NULL;
    if (p->rep) {   // (that kernel has no waits it could give up)
        *status = 0;
        return hipStreamSynchronize(static_cast<hipStream_t>(stream)) == hipSuccess ? VQ_OK : VQ_ERR_LAUNCH;
    }
    return gemv_pipeline_status(p->impl, static_cast<hipStream_t>(stream), status);
}

void vq_gemv_pipeline_destroy(vq_gemv_pipeline_t *p) {
    if (!p) return;
    if (p->impl) gemv_pipeline_destroy(p->impl);
    if (p->rep) gemv_replica_list_destroy(p->rep);
    delete p;
}

// Run r of n_runs contiguous runs of the calls: [first, first + count).
static void sequence_run(int n_calls, int n_runs, int r, int *first, int *count) {
    const int per = (n_calls + n_runs - 1) / n_runs;
    *first = r * per < n_calls ? r * per : n_calls;
    *count = n_calls - *first < per ? n_calls - *first : per;
}

size_t vq_gemv_sequence_streams_workspace(const vq_gemv_call_t *calls, int n_calls, int n_streams) {
    if (!calls || n_calls < 1 || n_streams < 1 || n_streams > VQ_SEQUENCE_MAX_SIDE_STREAMS + 1) return 0;
    for (int c = 0; c < n_calls; ++c)
        if (check_sequence_call(&calls[c]) != VQ_OK) return 0;
    size_t total = 0;
    for (int r = 0; r < n_streams; ++r) {
        int first, count;
        sequence_run(n_calls, n_streams, r, &first, &count);
        if (count > 0) total += gemv_packed_sequence_workspace(calls + first, count);
    }
    return total;
}

int vq_gemv_sequence_streams(const vq_gemv_call_t *calls, int n_calls, void *ws, size_t ws_bytes, void *stream,
                             const vq_side_streams_t *side) {
    if (!side || side->n == 0) return vq_gemv_sequence(calls, n_calls, ws, ws_bytes, stream);
    if (!calls) return VQ_ERR_NULL;
    if (n_calls < 1 || side->n < 0 || side->n > VQ_SEQUENCE_MAX_SIDE_STREAMS) return VQ_ERR_SHAPE;
    if (!side->start) return VQ_ERR_NULL;
    for (int i = 0; i < side->n; ++i)
        if (!side->stream[i] || !side->done[i]) return VQ_ERR_NULL;
    for (int c = 0; c < n_calls; ++c)
        if (int st = check_sequence_call(&calls[c])) return st;
    const int n_runs = side->n + 1;
    const size_t need = vq_gemv_sequence_streams_workspace(calls, n_calls, n_runs);
    if (!ws || ws_bytes < need) return VQ_ERR_WORKSPACE;
    if (!aligned16(ws)) return VQ_ERR_ALIGN;
    hipStream_t main_stream = static_cast<hipStream_t>(stream);
    if (hipEventRecord(static_cast<hipEvent_t>(side->start), main_stream) != hipSuccess) return VQ_ERR_LAUNCH;
    size_t off = 0;
    int status = VQ_OK;
    for (int r = 0; r < n_runs; ++r) {
        int first, count;
        sequence_run(n_calls, n_runs, r, &first, &count);
        hipStream_t s = r == 0 ? main_stream : static_cast<hipStream_t>(side->stream[r - 1]);
        if (r > 0 && hipStreamWaitEvent(s, static_cast<hipEvent_t>(side->start), 0) != hipSuccess) status = VQ_ERR_LAUNCH;
        if (count > 0 && status == VQ_OK) {
            status = launch_gemv_packed_sequence(calls + first, count, (unsigned char *)ws + off, s);
            off += gemv_packed_sequence_workspace(calls + first, count);
        }
        // the join is made even after a failure, so that a capture in progress is left in a consistent state
        if (r > 0) {
            if (hipEventRecord(static_cast<hipEvent_t>(side->done[r - 1]), s) != hipSuccess) status = VQ_ERR_LAUNCH;
            if (hipStreamWaitEvent(main_stream, static_cast<hipEvent_t>(side->done[r - 1]), 0) != hipSuccess) status = VQ_ERR_LAUNCH;
        }
    }
    return status;
}

size_t vq_gemm_workspace(const vq_weight_t *w, int M) {
    if (check_weight(w, true) != VQ_OK || M < 1) return 0;
    return gemm_workspace(w, M);
}

int vq_gemm(const vq_weight_t *w, const void *X, int M, void *Y, void *ws, size_t ws_bytes, void *stream) {
    int st = check_weight(w, true);
    if (st != VQ_OK) return st;
    if (!X || !Y) return VQ_ERR_NULL;
    if (M < 1) return VQ_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(Y)) return VQ_ERR_ALIGN;
    size_t need = gemm_workspace(w, M);
    if (need && (!ws || ws_bytes < need)) return VQ_ERR_WORKSPACE;
    if (ws && !aligned16(ws)) return VQ_ERR_ALIGN;
    if (w->N == 0) return VQ_OK;
    return launch_gemm(w, X, M, Y, ws, static_cast<hipStream_t>(stream));
}

size_t vq_attn_decode_workspace(const vq_kv_t *kv) {
    if (check_kv(kv) != VQ_OK) return 0;
    return attn_decode_workspace(kv);
}

int vq_attn_decode(const vq_kv_t *kv, const void *q, float sm_scale, void *out, void *ws, size_t ws_bytes,
                   void *stream) {
    int st = check_kv(kv);
    if (st != VQ_OK) return st;
    if (!q || !out) return VQ_ERR_NULL;
    if (!aligned16(q) || !aligned16(out)) return VQ_ERR_ALIGN;
    size_t need = attn_decode_workspace(kv);
    if (need && (!ws || ws_bytes < need)) return VQ_ERR_WORKSPACE;
    if (ws && !aligned16(ws)) return VQ_ERR_ALIGN;
    if (kv->B == 0 || kv->H == 0) return VQ_OK;
    return launch_attn_decode(kv, q, sm_scale, out, ws, static_cast<hipStream_t>(stream));
}

size_t vq_attn_decode_channel_parallel_workspace(const vq_kv_t *kv) {
    if (check_kv(kv) != VQ_OK || !attn_channel_supported(kv)) return 0;
    return attn_channel_workspace(kv);
}

int vq_attn_decode_channel_parallel(const vq_kv_t *kv, const void *q, float sm_scale, void *out, void *ws, size_t ws_bytes,
                                    void *stream) {
    int st = check_kv(kv);
    if (st != VQ_OK) return st;
    if (!attn_channel_supported(kv)) return VQ_ERR_UNSUPPORTED;
    if (!q || !out) return VQ_ERR_NULL;
    if (!aligned16(q) || !aligned16(out)) return VQ_ERR_ALIGN;
    if (kv->B == 0 || kv->H == 0) return VQ_OK;
    const size_t need = attn_channel_workspace(kv);
    if (need && (!ws || ws_bytes < need)) return VQ_ERR_WORKSPACE;
    if (ws && !aligned16(ws)) return VQ_ERR_ALIGN;
    return launch_attn_channel(kv, q, sm_scale, out, ws, static_cast<hipStream_t>(stream));
}

int vq_kv_quantize(const vq_kv_t *kv, const void *k_new, const void *v_new, int n_new, int pos, void *stream) {
    int st = check_kv(kv);
    if (st != VQ_OK) return st;
    if (!k_new || !v_new) return VQ_ERR_NULL;
    if (n_new < 0 || pos < 0 || (long)pos + n_new > kv->T) return VQ_ERR_SHAPE;
    if (!aligned16(k_new) || !aligned16(v_new)) return VQ_ERR_ALIGN;
    if (n_new == 0 || kv->B == 0 || kv->H == 0) return VQ_OK;
    return launch_kv_quantize(kv, k_new, v_new, n_new, pos, static_cast<hipStream_t>(stream));
}

int vq_dequant(const vq_weight_t *w, void *W, int out_fp32, void *stream) {
    int st = check_weight(w, true);
    if (st != VQ_OK) return st;
    if (!W) return VQ_ERR_NULL;
    if (!aligned16(W)) return VQ_ERR_ALIGN;
    if (w->N == 0 || w->K == 0) return VQ_OK;
    return launch_dequant(w, W, out_fp32, static_cast<hipStream_t>(stream));
}

int vq_kv_dequant(const vq_kv_t *kv, int which, void *out, void *stream) {
    int st = check_kv(kv);
    if (st != VQ_OK) return st;
    if (!out) return VQ_ERR_NULL;
    if (which != 0 && which != 1) return VQ_ERR_SHAPE;
    if (!aligned16(out)) return VQ_ERR_ALIGN;
    if (kv->B == 0 || kv->H == 0 || kv->T == 0) return VQ_OK;
    return launch_kv_dequant(kv, which, out, static_cast<hipStream_t>(stream));
}

int vq_probe_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src) return VQ_ERR_NULL;
    if (bytes % 16 != 0) return VQ_ERR_SHAPE;
    if (!aligned16(dst) || !aligned16(src)) return VQ_ERR_ALIGN;
    if (bytes == 0) return VQ_OK;
    return launch_probe_copy(dst, src, bytes, static_cast<hipStream_t>(stream));
}

int vq_probe_read(const void *src, size_t bytes, void *sink, void *stream) {
    if (!sink || !src) return VQ_ERR_NULL;
    if (bytes % 16 != 0) return VQ_ERR_SHAPE;
    if (!aligned16(sink) || !aligned16(src)) return VQ_ERR_ALIGN;
    if (bytes == 0) return VQ_OK;
    return launch_probe_read(src, bytes, sink, static_cast<hipStream_t>(stream));
}

int vq_probe_mfma(int workgroups, int iters, int random_operands, void *sink, void *stream) {
    if (!sink) return VQ_ERR_NULL;
    if (workgroups < 0 || iters < 0 || workgroups > (1 << 20) || iters > (1 << 24)) return VQ_ERR_SHAPE;
    if (!aligned16(sink)) return VQ_ERR_ALIGN;
    if (workgroups == 0) return VQ_OK;
    return launch_probe_mfma(workgroups, iters, random_operands, sink, static_cast<hipStream_t>(stream));
}

}  // extern "C"
