/*
 * vq_mi355x.h -- C ABI of libvqmi: matrix products on AMD MI355X (gfx950) whose
 * weight or KV-cache operand is stored as vector-quantization (VQ) codes, with
 * the codebook lookup fused into the contraction.
 *
 * Method: VQ-LLM (arXiv 2503.02236).  The operand format is the paper's
 * VQ<vector size, log2 #entries, residuals> (Sec. II-A, Tbl. I): a tensor is
 * cut into sub-vectors of `v` elements, each replaced by `R` indices ("codes"),
 * one per residual codebook; the value is the element-wise sum of the R looked-up
 * entries (Sec. II-A, dequantization).  The three operations are the kernels the
 * paper names VQ-gemv, VQ-gemm and VQ-attn (Sec. III-C, Sec. VI-C Alg. 2).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; descriptor
 *     structs are HOST memory, read during the call only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     are asynchronous on that stream; the library never synchronizes, never
 *     allocates and never frees device memory.  Scratch comes in through `ws`.
 *   - Return value: VQ_OK (0) or a negative vq_status.  Arguments are validated
 *     on the host before anything is launched; a failed call launches nothing.
 *   - Data pointers must be 16-byte aligned (VQ_ERR_ALIGN otherwise).
 *   - Codes >= n_entries are a precondition violation and are not checked on
 *     the device (with n_entries = 2^code_bits every code is valid).
 *   - Arithmetic: fp16 inputs, fp32 accumulation, fp16 round-to-nearest-even
 *     outputs; reductions are order-deterministic (no floating-point atomics),
 *     so repeated calls give bit-identical results.
 */
#ifndef VQ_MI355X_H
#define VQ_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum vq_status {
    VQ_OK = 0,
    VQ_ERR_NULL = -1,        /* a required pointer is NULL */
    VQ_ERR_SHAPE = -2,       /* K % v, bs / M range, D % v, cb_groups, negative sizes */
    VQ_ERR_UNSUPPORTED = -3, /* v / code_bits / n_entries / n_codebooks combination */
    VQ_ERR_ALIGN = -4,       /* a data pointer is not 16-byte aligned */
    VQ_ERR_WORKSPACE = -5,   /* ws is NULL or smaller than the *_workspace() query */
    VQ_ERR_LAUNCH = -6       /* the HIP runtime refused a launch (hipGetLastError) */
} vq_status;

/*
 * Kernel-private re-tiling of the codes of one weight matrix for the bs = 1 VQ-gemv
 * (weights are quantized offline, Sec. II-C; the paper itself rewrites indices offline when
 * it reorders codebook entries, Sec. V-B).  Produced on the HOST by vq_gemv_prepack(); the
 * caller uploads `data` to the device and hands this struct back unchanged.
 *
 * Idea (codebook-centric dataflow, Sec. VI-A, taken to the entry level): the codebook is cut
 * into S slices of 2^entry_bits entries that fit LDS, rows into RB blocks; workgroup (slice, block) sees
 * only the codes that point into its slice.  A row's K/8 sub-vector positions are cut into `parts` parts of
 * part_cols positions; a lane task = (row, part) walks the codes of that row and part.  A code is stored as
 * a 21-bit "atom": the entry's index inside the slice (entry_bits bits, low) and the position inside the
 * part (21 - entry_bits bits); both are 16-byte units of the workgroup's LDS image
 * [slice][part 0 of x, 16 zero units][part 1 of x, 16 zero units]...; padding atoms name a zero unit as x_j.
 * Three atoms fill a 64-bit step word; tasks of similar length are grouped 64 at a time (one lane each);
 * the order of a task's atoms is chosen offline so that the lanes' LDS reads collide as little as possible.
 * Partial sums of the S slices are added in a fixed order by a second kernel (Sec. VI-A "global reduction").
 * Group g of every workgroup starts at block  wg * wg_pitch + sum_{g' < g} group_steps[g']  (512-byte
 * blocks), so the kernel derives every address from this struct alone; how many of those blocks a
 * workgroup's group really uses comes from a small table inside `data`.  That needs codes that spread evenly
 * over the codebook (as quantizers produce them): vq_gemv_prepack declines (VQ_ERR_UNSUPPORTED,
 * vq_gemv_prepack_bytes = 0) when the common shape would cost more than a quarter more blocks and more than
 * 1 MiB, or a workgroup has more than VQ_PACK_MAX_GROUPS groups; vq_gemv then runs from the canonical codes.
 * Entries that codes point at must be finite (a padding atom adds 0 times an entry that some code of the same
 * 64 tasks uses; entries that no code points at are never read).  Layout of `data`: see the format description
 * in the source of vq_gemv_prepack.
 */
#define VQ_PACK_MAX_GROUPS 128
typedef struct vq_gemv_pack_t {
    const void *data;         /* DEVICE pointer when passed to vq_gemv (HOST buffer while packing) */
    uint64_t bytes;           /* size of data */
    uint32_t S, RB;           /* codebook slices, row blocks; S * RB workgroups */
    uint32_t rows_per_block;
    uint32_t entry_bits;      /* slices of 2^entry_bits entries */
    uint32_t parts, part_cols; /* parts of a row, sub-vector positions per part */
    uint32_t wg_pitch;        /* 512-byte atom blocks per workgroup (the sum of group_steps) */
    uint64_t task_off, steps_off, atom_off; /* byte offsets of the three tables in data */
    uint16_t group_steps[VQ_PACK_MAX_GROUPS]; /* blocks reserved for group g of every workgroup; 0 past the last group */
} vq_gemv_pack_t;

/*
 * A VQ-compressed weight matrix W[N][K] of a linear layer y = W x
 * (N output features, K input features).  Sub-vectors lie along K, the
 * reduction axis, so row n holds K/v sub-vectors.
 *   W[n][j*v + i] = sum_{r < n_codebooks} codebooks[r][codes[n][j][r]][i]
 * summed in fp32, r ascending (Sec. II-A; "Residual" of Tbl. I = n_codebooks).  vq_dequant returns exactly
 * this sum (or its fp16 rounding).  The kernels that feed the matrix cores consume the fp16 rounding of it:
 * for three or four codebooks the fp32 sum rounded once; for two codebooks one fp16 addition of the two
 * entries (the exact sum rounded once), which is the same value whenever the fp32 sum is exact, i.e. always
 * unless the two entries' exponents lie more than 13 apart (then it can differ by one fp16 ulp on a tie).
 * With per-tile codebooks (cb_tile_n, cb_tile_k > 0) `codebooks` above is the set of the tile that holds
 * (n, j*v).  Re-tiled gemv codes (gemv_pack), hot_entries and the fused small-M matrix-core path of vq_gemm
 * apply to per-tensor codebooks only.
 */
typedef struct vq_weight_t {
    int N, K;              /* output / input features; K % v == 0 */
    int v;                 /* vector size: 4 or 8 */
    int code_bits;         /* storage width of one code: 8 (uint8), 16 (uint16, little endian), or 12: the packed
                              string of VQ<8,12,2> (Sec. VII-B "unaligned 12-bit storage"; layout is this
                              library's reading): codes in the same [N][K/v][R] order form a little-endian bit
                              string, code i in bits [12 i, 12 i + 12) -- two codes in three bytes; a row must
                              hold a multiple of 8 codes; per-tensor codebooks, 1, 2 or 4 of them, together at most
                              128 KiB (R * E * v * 2 bytes); no gemv_pack */
    int n_codebooks;       /* R >= 1 additive (residual) codebooks, R <= 4 */
    int n_entries;         /* E entries per codebook, 1 <= E <= 2^code_bits */
    const void *codes;     /* device, [N][K/v][R], r fastest (12-bit: N * K/v * R * 3/2 bytes) */
    const void *codebooks; /* device, fp16 [R][E][v] */
    const void *scale;     /* device, fp16 [N] per output channel, or NULL (= 1) */
    const vq_gemv_pack_t *gemv_pack; /* host pointer, optional: re-tiled codes for vq_gemv with bs = 1 */
    int hot_entries;       /* 0, or (after vq_reorder_by_frequency) how many leading entries serve half of
                              the codes: lets vq_gemv keep the hot front of a large codebook in LDS */
    int cb_tile_n, cb_tile_k; /* codebook scope (Sec. III-B, Tbl. III).  0, 0: one set of codebooks for the tensor.
                              Otherwise one set per (cb_tile_n x cb_tile_k) tile of W (e.g. 256 x 256):
                              codebooks are fp16 [ceil(N/cb_tile_n)][K/cb_tile_k][R][E][v] and element (n, k)
                              uses set (n / cb_tile_n, k / cb_tile_k).  cb_tile_n % 16 == 0, cb_tile_k % 64 == 0,
                              K % cb_tile_k == 0; n_codebooks 1, 2 or 4; all sets of one row of tiles must fit LDS together
                              ((K / cb_tile_k) * R * E * v * 2 <= 128 KiB) */
} vq_weight_t;

/*
 * VQ-gemv (decode phase, Sec. III-C / Sec. VII "GeMV", batch sizes 1..16):
 *   y[m][n] = scale[n] * sum_k W[n][k] * x[m][k],   m < bs
 * x: device fp16 [bs][K]; y: device fp16 [bs][N]; 1 <= bs <= 16.
 * ws: device scratch of at least vq_gemv_workspace(w, bs) bytes (may be NULL
 * when that is 0).  Errors: NULL / SHAPE / UNSUPPORTED / ALIGN / WORKSPACE / LAUNCH.
 */
int vq_gemv(const vq_weight_t *w, const void *x, int bs, void *y,
            void *ws, size_t ws_bytes, void *stream);
size_t vq_gemv_workspace(const vq_weight_t *w, int bs);

/*
 * vq_gemv for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same operation, arguments, results (bit for bit) and
 * errors as vq_gemv, but the scratch that the re-tiled bs = 1 path needs (S x N fp32 partial sums) lies
 * inside the library: a fixed array of vq_gemv_noalloc_max_workspace() bytes (2 MiB) in every GPU's memory,
 * held until the process ends.  The call allocates nothing and frees nothing.
 *   - A problem whose vq_gemv_workspace() exceeds that size is refused with VQ_ERR_WORKSPACE (use vq_gemv).
 *   - All calls on one GPU share that GPU's array: calls that may overlap in time (different streams, or
 *     graph branches without an edge between them) race on it and must not be issued; calls on one stream
 *     are safe.  Nothing in the array has to be cleared between calls.
 *   - The array's address is looked up once per GPU, on the first call there or in vq_init(); call vq_init()
 *     (no arguments; VQ_OK or VQ_ERR_LAUNCH) once on each GPU before capturing a graph that holds this call.
 */
int vq_init(void);
size_t vq_gemv_noalloc_max_workspace(void);
int vq_gemv_noalloc(const vq_weight_t *w, const void *x, int bs, void *y, void *stream);

/*
 * Offline re-tiling for vq_gemv (see vq_gemv_pack_t).  HOST function: w->codes is read from
 * HOST memory here (codebooks / scale are not touched); no GPU is needed.
 *   vq_gemv_prepack_bytes: size of the packed buffer for this matrix, 0 if the configuration
 *     has no packed form (supported: v = 8, uint16 codes, one codebook, E a power of two
 *     >= 4096, K <= 64512, codes that spread evenly over the codebook: see vq_gemv_pack_t).
 *   vq_gemv_prepack: writes the packed buffer into out_host (>= that size, 16-byte aligned)
 *     and fills *pack (pack->data = out_host; replace it by the device copy's address before
 *     passing the struct to vq_gemv).  Errors: NULL / UNSUPPORTED / SHAPE (a code >= n_entries) / WORKSPACE
 *     (buffer too small).
 * With w->gemv_pack set and bs == 1, vq_gemv runs from the packed codes (w->codes may then be
 * NULL) and needs the workspace vq_gemv_workspace() reports (S x N fp32 partial sums; calls that
 * share one workspace must not overlap).
 */
size_t vq_gemv_prepack_bytes(const vq_weight_t *w_host);
int vq_gemv_prepack(const vq_weight_t *w_host, void *out_host, size_t out_bytes, vq_gemv_pack_t *pack);

/*
 * Offline frequency reordering of the codebook entries of one weight (Sec. V-B: entries are used very
 * unevenly; the hot ones belong at the front, where a kernel's on-chip cache of the first entries finds
 * them).  HOST function, no GPU: w_host->codes and w_host->codebooks are HOST memory.  For every
 * codebook r the entries are sorted by descending number of codes that point at them (ties keep their
 * order) and the codes are rewritten to follow, so the dequantized weight is bit-identical.
 *   codes_out_host:     same type and shape as w_host->codes (may be the same buffer)
 *   codebooks_out_host: fp16 [R][E][v] (must NOT be w_host->codebooks)
 *   hot_entries_out:    optional; the smallest n such that the first n entries of every codebook serve
 *                       at least half of its codes (the paper sets its cache boundaries from the same
 *                       offline histogram).  Put it into vq_weight_t.hot_entries of the reordered weight:
 *                       when a single codebook is too large for LDS and hot_entries fits the on-chip
 *                       cache (4096 entries of v = 8), vq_gemv on canonical codes keeps the front of the
 *                       codebook in LDS and gathers only the rest from L2.  Results never depend on it.
 * Errors: NULL / SHAPE (a code >= n_entries, or output aliasing the input codebooks) / UNSUPPORTED.
 */
int vq_reorder_by_frequency(const vq_weight_t *w_host, void *codes_out_host, void *codebooks_out_host,
                            int *hot_entries_out);

/*
 * Several independent bs = 1 VQ-gemv problems y_i = W_i x_i in one call (count <= VQ_GEMV_BATCH_MAX):
 * the projections of a decoder block that do not depend on each other (query/key/value; gate/up).
 * When every W_i carries re-tiled codes (gemv_pack) the whole batch is ONE launch of the codebook-centric
 * kernel (Sec. VI-A) plus one launch of its global reduction, so the fixed latencies of a launch are paid
 * once, and the results are bit-identical to separate vq_gemv calls.  A batch of canonical-code weights of one
 * kind (same code width, v and number of codebooks) whose codebooks fit LDS is one launch of the matrix-core
 * gemv; it may split K over another number of wavefronts than a single call does, so its results equal those of
 * vq_gemv up to the order of the fp32 additions (and are the same from call to call).  Any other mix is run as
 * `count` vq_gemv calls.
 * w, x, y: HOST arrays of `count` pointers (x_i: device fp16 [K_i], y_i: device fp16 [N_i]; the x_i may
 * be the same buffer).  ws: vq_gemv_batch_workspace(w, count) bytes.
 * Errors: as vq_gemv; VQ_ERR_SHAPE for count outside 1..VQ_GEMV_BATCH_MAX.
 */
#define VQ_GEMV_BATCH_MAX 4
int vq_gemv_batch(const vq_weight_t *const *w, const void *const *x, void *const *y, int count,
                  void *ws, size_t ws_bytes, void *stream);
size_t vq_gemv_batch_workspace(const vq_weight_t *const *w, int count);

/*
 * A sequence of bs = 1 VQ-gemv calls on one stream, call c being a batch of calls[c].count independent problems
 * (as vq_gemv_batch takes them).  Same results, bit for bit, as the vq_gemv_batch calls made one after the other.
 * What it saves: the explicit global reduction of the codebook-centric kernel (Sec. VI-A: its cost grows with
 * split x output) needs a kernel boundary behind every launch; here the boundary is the next call's launch,
 * whose workgroups take the previous call's rows along and add their partial sums in their prologue and
 * epilogue, so a sequence of n calls is n + 1 kernel launches instead of 2 n.
 * Consequence: the outputs of call c are complete only when the work of the whole sequence is; the inputs of a
 * call must therefore not depend on outputs of earlier calls OF THE SAME SEQUENCE (products that depend on each
 * other through kernels in between belong to different sequences, or to vq_gemv / vq_gemv_batch).
 * Every weight must carry re-tiled codes (gemv_pack); VQ_ERR_UNSUPPORTED otherwise.  calls, and the arrays they
 * point at, are HOST memory.  ws: vq_gemv_sequence_workspace(calls, n_calls) bytes (twice the largest call's
 * partial sums).  Errors: as vq_gemv_batch; VQ_ERR_SHAPE for n_calls < 1.
 */
typedef struct vq_gemv_call_t {
    const vq_weight_t *const *w;   /* count weights */
    const void *const *x;          /* count device pointers, fp16 [K_i] */
    void *const *y;                /* count device pointers, fp16 [N_i] */
    int count;                     /* 1 .. VQ_GEMV_BATCH_MAX */
} vq_gemv_call_t;
int vq_gemv_sequence(const vq_gemv_call_t *calls, int n_calls, void *ws, size_t ws_bytes, void *stream);
size_t vq_gemv_sequence_workspace(const vq_gemv_call_t *calls, int n_calls);

/*
 * The same sequence spread over several HIP streams of the caller, so that launches of different calls overlap
 * on the GPU (the calls of a sequence are independent of each other by contract; on one stream every launch
 * waits for the previous one to drain, and a bs = 1 product is too short to hide its own start-up).
 * The calls are cut into side->n + 1 contiguous runs; run 0 goes to `stream`, run i to side->stream[i - 1], each
 * run being a vq_gemv_sequence of its own.  Ordering towards the caller is that of a call on `stream` alone:
 * the side streams first wait for side->start (recorded on `stream` at entry), and `stream` finally waits for
 * side->done[i] of every side stream, so work queued on `stream` afterwards sees every output.
 * side: HOST struct; streams (default priority) and events (hipEventDisableTiming is enough) are created and
 * owned by the caller and must not be in use by anything else during the call; NULL or n = 0 gives
 * vq_gemv_sequence.  The call may be captured into a HIP graph from `stream` (the side streams join the capture
 * through the events).  ws: vq_gemv_sequence_streams_workspace(calls, n_calls, side->n + 1) bytes.
 * Errors: as vq_gemv_sequence; VQ_ERR_SHAPE for side->n outside 0..VQ_SEQUENCE_MAX_SIDE_STREAMS; VQ_ERR_NULL for a
 * missing stream or event; VQ_ERR_LAUNCH if the runtime refuses an event operation.
 */
#define VQ_SEQUENCE_MAX_SIDE_STREAMS 7
typedef struct vq_side_streams_t {
    int n;                                        /* side streams in use */
    void *stream[VQ_SEQUENCE_MAX_SIDE_STREAMS];   /* hipStream_t */
    void *done[VQ_SEQUENCE_MAX_SIDE_STREAMS];     /* hipEvent_t, one per side stream */
    void *start;                                  /* hipEvent_t */
} vq_side_streams_t;
int vq_gemv_sequence_streams(const vq_gemv_call_t *calls, int n_calls, void *ws, size_t ws_bytes, void *stream,
                             const vq_side_streams_t *side);
size_t vq_gemv_sequence_streams_workspace(const vq_gemv_call_t *calls, int n_calls, int n_streams);

/*
 * The same sequence as ONE persistent launch (plus one reduction launch): 256 workgroups, one per compute unit,
 * each of which walks through a list of problems with two LDS images -- its producer wavefronts stage the
 * codebook slice and x of problem k + 1 while its consumer wavefronts gather problem k, and the consumers'
 * requests for re-tiled codes run two pieces of work ahead, across problem boundaries.  Separate launches
 * (vq_gemv_sequence) run staging, gathers and stores of a product in lockstep on all units, so that memory, LDS
 * and arithmetic take turns idling; at Llama-7B sizes each of these phases is 1 - 4 us long.  When every problem
 * has row blocks enough, a workgroup takes 2 or 4 row blocks of its slice per image and the launch splits into 2
 * or 4 lanes of workgroups that work on different problems at the same time.  (The dataflow inside a problem is
 * that of Sec. VI-A: codebook slice in shared memory, split-x partial sums, explicit global reduction.)
 * Contract as vq_gemv_sequence (independent calls, outputs complete when the whole run is); every output has the
 * bits vq_gemv gives (the same additions in the same order).
 *   vq_gemv_pipeline_create: validates the calls, writes the problem table into ws (a synchronous copy on
 *     `stream`; calls and their arrays need not outlive the call) and returns a HOST handle.  x, y, weights and
 *     ws are bound at creation: a pipeline is re-created when any of these pointers changes.
 *     ws: device, 256-byte aligned (VQ_ERR_ALIGN), vq_gemv_pipeline_workspace(calls, n_calls) bytes, owned by the
 *     caller and in use by the pipeline until it is destroyed.
 *     VQ_ERR_UNSUPPORTED: a weight without re-tiled codes, or one that does not fit the persistent launch
 *     (more than 256 row-block x slice workgroups, an LDS image above 64 KiB - 64 B, x in more than about three parts,
 *     or more sums per image than its LDS buffer holds).
 *   vq_gemv_pipeline_run: two kernel launches on `stream`; no allocation, no synchronisation; capturable.  Runs of
 *     one pipeline must not overlap (they share ws).  VQ_ERR_LAUNCH when called with another GPU current.
 *   vq_gemv_pipeline_status: copies the device status word to *status (synchronises `stream`): 0, or 1 if a
 *     wavefront of some run gave up one of its bounded waits inside the kernel (the outputs of that run are then
 *     invalid; this takes a workgroup whose own wavefronts stop making progress for tens of milliseconds).
 *   vq_gemv_pipeline_destroy: frees the handle (not ws); NULL is allowed.
 *
 * Second kind of list: weights with SMALL codebooks in the canonical layout (no re-tiled codes; uint8 codes, v = 8,
 * one or two additive codebooks of <= 256 entries, K a multiple of 64 in [512, 12288]; Sec. II-A residual
 * quantization, Sec. III-C VQ-gemv).  All problems of the list must be of this kind and have the same number of
 * codebooks (a mix: VQ_ERR_UNSUPPORTED).  One launch: a workgroup per compute unit holds 16 copies of every entry
 * of the current problem's codebooks in LDS, one per bank column, so that the random entry reads of a wavefront never
 * collide; groups of workgroups work on different problems at the same time and re-stage between problems while
 * the next problem's codes are already in flight.  No partial sums, no second launch: ws holds only the problem
 * table.  Outputs are within the gemv tolerance of the definition but not bit-identical to vq_gemv's (another
 * summation order); repeated runs give identical bits.  vq_gemv_pipeline_status reports 0 (this kernel has no waits
 * it could give up).
 */
typedef struct vq_gemv_pipeline vq_gemv_pipeline_t;
size_t vq_gemv_pipeline_workspace(const vq_gemv_call_t *calls, int n_calls);
int vq_gemv_pipeline_create(const vq_gemv_call_t *calls, int n_calls, void *ws, size_t ws_bytes, void *stream,
                            vq_gemv_pipeline_t **out);
int vq_gemv_pipeline_run(const vq_gemv_pipeline_t *p, void *stream);
int vq_gemv_pipeline_status(const vq_gemv_pipeline_t *p, void *stream, int *status);
void vq_gemv_pipeline_destroy(vq_gemv_pipeline_t *p);

/*
 * VQ-gemm (prefill phase, Sec. III-C / Sec. VII "GeMM"): Y = X W^T with the
 * dequantized tile fed to the fp16 matrix cores, fp32 accumulation.
 *   Y[m][n] = scale[n] * sum_k W[n][k] * X[m][k],   m < M
 * X: device fp16 [M][K]; Y: device fp16 [M][N]; M >= 1.
 * ws: vq_gemm_workspace(w, M) bytes.  For M > 256 that is N*K*2: the weight is dequantized once per
 * call into ws (fp16, the same bits vq_dequant returns) and multiplied by a dense matrix-core kernel;
 * for smaller M the dequantization is fused into the matrix-core loop and no workspace is needed.
 */
int vq_gemm(const vq_weight_t *w, const void *X, int M, void *Y,
            void *ws, size_t ws_bytes, void *stream);
size_t vq_gemm_workspace(const vq_weight_t *w, int M);

/*
 * A VQ-compressed KV cache of one layer (Sec. III-A setup: VQ<4,8,1> as in CQ-2,
 * 32 heads x 128 channels).  Every token's K (and V) vector of D channels is cut
 * into D/v sub-vectors, each stored as one uint8 code.
 *   K[b][h][t][p*v + i] = k_codebooks[h][g(p)][k_codes[b][h][t][p]][i],
 *   g(p) = p * cb_groups / (D/v)
 * cb_groups = 1: one codebook per (head, K|V); cb_groups = D/v: one codebook per
 * sub-space, the coupled-quantization layout whose codebook switches along the
 * channel axis (Sec. III-B, Tbl. IV) -- any divisor of D/v is accepted.
 */
typedef struct vq_kv_t {
    int B, H, D, T;          /* batch, heads, head dim, cache length (row stride of the code arrays) */
    int v;                   /* sub-vector length: 2, 4 or 8; D % v == 0 */
    int n_entries;           /* E <= 256 */
    int cb_groups;           /* G codebooks per (head, side); divides D/v */
    const void *k_codes;     /* device, uint8 [B][H][T][D/v] */
    const void *v_codes;     /* device, uint8 [B][H][T][D/v] */
    const void *k_codebooks; /* device, fp16 [H][G][E][v] */
    const void *v_codebooks; /* device, fp16 [H][G][E][v] */
    const int *seq_lens;     /* device, int32 [B], valid tokens per sequence (0..T), or NULL = T */
} vq_kv_t;

/*
 * VQ-attn (decode attention over the VQ cache; Sec. II-B formula, one query per
 * sequence and head, all cached tokens attended, no mask):
 *   out[b][h] = softmax_t( sm_scale * q[b][h] . K[b][h][t] ) . V[b][h][t]
 * q, out: device fp16 [B][H][D].  sm_scale is usually 1/sqrt(D).
 * A sequence with seq_lens[b] == 0 yields zeros.
 * ws: at least vq_attn_decode_workspace(kv) bytes (partial softmax statistics
 * and accumulators of the token-range split, merged by log-sum-exp).
 */
int vq_attn_decode(const vq_kv_t *kv, const void *q, float sm_scale, void *out,
                   void *ws, size_t ws_bytes, void *stream);

/*
 * The same product by the CHANNEL-PARALLEL, codebook-centric dataflow of Sec. VI-A for caches with one codebook
 * per channel sub-space (coupled quantization, Sec. III-B / Tbl. IV): a workgroup owns 32 channels of a head and
 * stages only their codebooks; the partial inner products of the D / 32 channel groups are accumulated through
 * global memory (three launches: partial scores, sum + softmax over the tokens, values).  vq_attn_decode keeps
 * all codebooks of a head in LDS and switches between them instead (token-parallel); this entry point exists so
 * that the two sides of the paper's trade-off can be measured against each other.  Same arguments and results
 * (within the tolerance of the fp32 reductions, whose order differs); repeated calls are bit-identical.
 * Needs D % 32 == 0, cb_groups a multiple of D / 32 and at most 60 KiB of codebooks per channel group
 * (VQ_ERR_UNSUPPORTED otherwise).  ws: vq_attn_decode_channel_parallel_workspace(kv) bytes
 * (B H (D / 32 + 1) T floats), 16-byte aligned; the query returns 0 for an unsupported cache.
 */
int vq_attn_decode_channel_parallel(const vq_kv_t *kv, const void *q, float sm_scale, void *out,
                                    void *ws, size_t ws_bytes, void *stream);
size_t vq_attn_decode_channel_parallel_workspace(const vq_kv_t *kv);
size_t vq_attn_decode_workspace(const vq_kv_t *kv);

/*
 * On-the-fly KV quantization (Sec. II-A, assignment step: a sub-vector is replaced by the index of its
 * closest codebook entry; Sec. VII "Quantization Overhead": run for the new token of every decode step
 * and for all prompt tokens in prefill).  Quantizes n_new tokens per sequence and WRITES their codes
 * into kv->k_codes / kv->v_codes at positions [pos, pos + n_new) of every (b, h) row (the const in the
 * descriptor notwithstanding); kv->seq_lens is not read or changed.
 *   k_new, v_new: device fp16 [B][H][n_new][D];  0 <= pos, pos + n_new <= T (VQ_ERR_SHAPE otherwise).
 * Definition of "closest" (the paper gives none): squared Euclidean distance in fp32, elements in
 * ascending order, each operation rounded separately; ties go to the smallest index.  Codebooks of one
 * side of a head (cb_groups * n_entries * v * 2 bytes) must fit 64 KiB (VQ_ERR_UNSUPPORTED otherwise).
 */
int vq_kv_quantize(const vq_kv_t *kv, const void *k_new, const void *v_new, int n_new, int pos, void *stream);

/*
 * Test hooks: the dequantized operand itself (Sec. II-A), for bit-exact checks.
 * vq_dequant: W[N][K], fp32 (out_fp32 = 1: the fp32 sum of the residual entries)
 *             or fp16 (out_fp32 = 0: that sum rounded to nearest even).
 * vq_kv_dequant: which = 0 -> K, 1 -> V; out fp16 [B][H][T][D] (entries verbatim).
 */
int vq_dequant(const vq_weight_t *w, void *W, int out_fp32, void *stream);
int vq_kv_dequant(const vq_kv_t *kv, int which, void *out, void *stream);

/*
 * Measurement helpers (not part of the method): a plain streaming copy and a
 * streaming read-reduce of `bytes` bytes (multiple of 16) with 128-bit accesses,
 * used to calibrate HBM counters and the achievable-bandwidth ceiling.
 * vq_probe_read writes one 16-byte checksum per workgroup into sink (>= 64 KiB).
 */
int vq_probe_copy(void *dst, const void *src, size_t bytes, void *stream);
int vq_probe_read(const void *src, size_t bytes, void *sink, void *stream);
/*
 * vq_probe_mfma: `workgroups` x 4 wavefronts, each running `iters` x 8 back-to-back register-resident
 * v_mfma_f32_32x32x16_f16 (32768 flops each) with no memory traffic: the matrix-core rate this chip
 * sustains, as the second reference beside the vendor peak.  random_operands = 0: one smooth operand
 * pair (few bits toggle); != 0: four pairs of pseudo-random halves in [-1, 1) per lane taken in turn, as
 * a gemm on real data presents them (the chip clocks lower on these); 2: six fresh random operands per
 * iteration read from LDS (32 KiB per workgroup), the way a gemm's main loop is fed.  sink: >= 16 device bytes
 * (practically never written).
 */
int vq_probe_mfma(int workgroups, int iters, int random_operands, void *sink, void *stream);

/* Human-readable name of a status code (static storage). */
const char *vq_status_str(int status);

/* Library version, as 10000*major + 100*minor + patch. */
int vq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VQ_MI355X_H */
