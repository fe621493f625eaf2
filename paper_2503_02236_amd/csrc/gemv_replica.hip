// VQ-gemv at batch size 1 for MANY weights whose codebooks are small (uint8 codes, v = 8, one or two additive
// codebooks of <= 256 entries), all in one launch: the form vq_gemv_pipeline takes for such weights.  Every codebook
// entry is held SIXTEEN times in LDS, once per 16-byte bank column, so that the random entry reads of a wavefront
// never collide.
// Operation: VQ-LLM (arXiv 2503.02236) Sec. III-C "VQ-gemv" at bs = 1; residual codebooks summed as in Sec. II-A;
// the bank conflicts of random codebook reads are the paper's Sec. III-B observation ("#entries >> #banks"), the
// per-lane operand layout its Sec. VI-B layout fusion.
//
// LDS.  A wavefront's 16-byte reads are served in four passes of 16 lanes -- lanes {0-3, 12-15, 20-27},
// {4-11, 16-19, 28-31} and the same + 32 -- and every further distinct address in the same 16-byte column
// (address / 16 mod 16) costs a pass more: 12 clocks per wave-wide read at random addresses, 4.8 without collisions.
// The lanes of a pass all differ in lane % 16, so copy c of entry e at byte e * 256 + c * 16, read by the lanes with
// lane % 16 = c, is collision free whatever the codes are: 2 x 64 KiB of the CU's 160 KiB for two codebooks.  The
// address is one v_perm_b32: the code byte dropped into byte 1 of a per-lane constant.
//
// Mapping.  One persistent workgroup of 16 wavefronts per compute unit.  The workgroups form up to 32 groups; group g
// takes problems g, g + groups, ... of the list, and each of its workgroups a contiguous range of rows of every
// such problem (the more rows per workgroup, the less the re-staging of codebooks between problems weighs).  A row's
// codes are cut into chunks of 512 positions: lane l of a wavefront loads the 8 (x R) code bytes of positions
// [8 l, 8 l + 8) of the chunk with one coalesced load and keeps x for those positions in 32 registers (from the LDS
// copy of x, re-read only when the wavefront moves to another chunk index).  The (row, chunk) items of a workgroup
// are dealt to its wavefronts in chunk-major runs, so a wavefront changes chunk index at most twice per problem.
// The dot product of an entry with x_j runs on the matrix cores: v_mfma_f32_4x4x4_16b_f16 multiplies sixteen
// independent pairs of 4 x 4 matrices, row i of the first and column i of the second operand of a pair held by the
// same lane, so diagonal element i of a product is that lane's own 4-term dot product, in accumulator register
// lane % 4 (the other three registers collect cross terms and are never read).  An item's 64 lane sums are added by
// DPP steps; chunk sums meet in LDS and thread t of the workgroup finishes rows t and t + 1024 of its range:
// y = fp16(scale * sum), chunks in ascending order.  Every order is fixed: repeated runs give the same bits.
//
// Between two problems the workgroup re-stages: each thread holds one entry of the next problem (and up to 32 bytes
// of its x, and the scales of its rows), requested a whole problem earlier, and writes the 16 copies -- lane l starts
// at copy l % 16, so the writes of a pass fall into 16 different columns too.  The codes of a wavefront's next three
// items are also in flight, across problem boundaries (a ring of three slots, each refilled as soon as its item has
// been worked on); the workgroup barriers wait for LDS traffic
// only, so these requests stay in flight across them.
//
// What bounds it: instruction issue.  An item (512 positions of a row, 1024 gathers with two codebooks) is about 130
// issue slots per wavefront -- 16 address permutes, 16 LDS reads, 32 matrix instructions of two slots each (the same
// 64 slots as v_dot2 would take), ~30 for the sums and the bookkeeping -- against 77 clocks of LDS time.
#include <algorithm>
#include <new>
#include <vector>

#include "vq_common.h"

namespace vq {

constexpr int kRepThreads = 1024;  // 16 wavefronts, four per SIMD, 128 registers each (12 wavefronts: 4 % slower, 8: 11 %)
constexpr int kRepHalves = 2;      // an item's gathers are issued in this many blocks, each in front of its own arithmetic
constexpr int kRepWaves = kRepThreads / kWave;
constexpr int kRepCopies = 16;
constexpr int kRepCbStride = 256 * kRepCopies * 16;     // 64 KiB: LDS bytes of one codebook
constexpr int kRepX = 2 * kRepCbStride;                 // x of the current problem (zeros past its end)
constexpr int kRepMaxK = 12288;                         // 24 KiB of x in LDS
constexpr int kRepXPer = (kRepMaxK / 8 + kRepThreads - 1) / kRepThreads;   // 16-byte units of x per thread
constexpr int kRepPart = kRepX + kRepMaxK * 2;          // chunk sums [chunk][row of the workgroup], fp32
constexpr int kRepPartFloats = 2048;                     // chunks x rows of one problem per workgroup
constexpr int kRepLds = kRepPart + kRepPartFloats * 4;
static_assert(kRepLds <= 160 * 1024, "one workgroup per CU, all of its LDS");
constexpr int kRepMaxGroups = 32;                       // groups of workgroups that work on different problems
constexpr int kRepRound = 3;                            // items (16-byte code loads) a wavefront has in flight per round

struct RepProblem {
    const uint8_t *codes;   // [N][K/8][R]
    const half_t *cb;       // [R][E][8]
    const half_t *scale;    // [N] or null
    const half_t *x;        // [K]
    half_t *y;              // [N]
    int N, K, E;
    int rows_per_wg;        // workgroup b owns rows [b * rows_per_wg, ...): ceil(N / workgroups of the launch)
};
static_assert(sizeof(RepProblem) == 56, "table layout");

typedef const __attribute__((address_space(1))) unsigned char rbyte_t;

__device__ __forceinline__ V16 rep_lds16(uint32_t addr) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t v = *(const __attribute__((address_space(3))) u32x4_t *)(uintptr_t)addr;
    V16 r;
    r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
    return r;
}
__device__ __forceinline__ void rep_lds16_store(uint32_t addr, const uint4 &v) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    *(__attribute__((address_space(3))) u32x4_t *)(uintptr_t)addr = u32x4_t{v.x, v.y, v.z, v.w};
}
// 16-byte unit number i of a global array
__device__ __forceinline__ uint4 rep_global16(const void *base, int i) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t v = ((const __attribute__((address_space(1))) u32x4_t *)base)[i];
    return uint4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ half4_t rep_half4(uint32_t lo, uint32_t hi) {
    V8 t;
    t.w[0] = lo; t.w[1] = hi;
    return t.h4;
}

// Workgroup barrier for LDS traffic only.  __syncthreads() also waits for every global load in flight -- here the
// requests for the next problem and the next round of codes, which are meant to stay in flight across it.
__device__ __forceinline__ void rep_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int CTRL, int ROWS>
__device__ __forceinline__ float rep_dpp_add(float x) {
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROWS, 0xF, false);
    return x + __int_as_float(y);
}
// Sum over the wavefront, in lane 63, on the vector ALU only.
__device__ __forceinline__ float rep_wave_sum_to_63(float x) {
    x = rep_dpp_add<0x111, 0xF>(x);   // row_shr:1
    x = rep_dpp_add<0x112, 0xF>(x);   // row_shr:2
    x = rep_dpp_add<0x114, 0xF>(x);   // row_shr:4
    x = rep_dpp_add<0x118, 0xF>(x);   // row_shr:8 -- lane 15 of every row of 16 holds the row's sum
    x = rep_dpp_add<0x142, 0xA>(x);   // row_bcast:15 into rows 1 and 3
    x = rep_dpp_add<0x143, 0xC>(x);   // row_bcast:31 into rows 2 and 3
    return x;
}

// What a workgroup and one of its wavefronts have to do for a problem.
struct RepShare {
    int row0, rows;      // the workgroup's rows
    int nch;             // chunks per row
    int lane_chunks;     // K / 64: 8-position pieces per row
    int first, end;      // the wavefront's run of items (item u: chunk u / rows, row u % rows)
};
__device__ __forceinline__ RepShare rep_share(const RepProblem &p, int wave, int wb) {
    RepShare s;
    // (no division on the device: the split of the rows comes with the problem)
    s.row0 = min(wb * p.rows_per_wg, p.N);
    s.rows = min(p.N - s.row0, p.rows_per_wg);
    s.lane_chunks = p.K >> 6;
    s.nch = (s.lane_chunks + 63) >> 6;
    const int total = s.rows * s.nch, per = (total + kRepWaves - 1) / kRepWaves;
    s.first = min(wave * per, total);
    s.end = min(s.first + per, total);
    return s;
}

// Where a wavefront stands in its run of items of one problem (all wave-uniform).
struct RepRun {
    int u, end;       // next item, end of the run
    int c, row;       // chunk index and row (inside the workgroup's share) of item u
    int rows;         // rows of the workgroup's share
};
__device__ __forceinline__ RepRun rep_run(const RepShare &s) {
    RepRun r;
    r.u = s.first; r.end = s.end; r.rows = s.rows;
    r.c = (s.first >= s.rows ? 1 : 0) + (s.first >= 2 * s.rows ? 1 : 0);
    r.row = s.first - r.c * s.rows;
    return r;
}
__device__ __forceinline__ void rep_step(RepRun &r) {
    ++r.u;
    ++r.row;
    if (r.row == r.rows) { r.row = 0; ++r.c; }
}

template <int R>
struct RepCodes {
    uint32_t w[2 * R];
};
// The lane's 8 R code bytes of an item.  A lane past the end of the row (last chunk of a ragged row) re-reads the
// row's first bytes: an unconditional load of valid memory; what it computes from them is dropped.
template <int R>
__device__ __forceinline__ RepCodes<R> rep_load(const uint8_t *codes, uint32_t row_bytes, int row0, int lane_chunks, const RepRun &r,
                                                int lane) {
    const int lc = r.c * 64 + lane;
    // (a uniform row address plus a 32-bit lane offset: the load takes them as they are, no address arithmetic per lane)
    rbyte_t *rowp = (rbyte_t *)codes + (size_t)(row0 + r.row) * row_bytes;
    rbyte_t *src = rowp + (uint32_t)(lc < lane_chunks ? lc : 0) * (8u * R);
    RepCodes<R> q;
    if constexpr (R == 2) {
        typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
        const u32x4_t v = *(const __attribute__((address_space(1))) u32x4_t *)src;
        q.w[0] = v.x; q.w[1] = v.y; q.w[2] = v.z; q.w[3] = v.w;
    } else {
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        const u32x2_t v = *(const __attribute__((address_space(1))) u32x2_t *)src;
        q.w[0] = v.x; q.w[1] = v.y;
    }
    return q;
}

// One item: 8 positions of one row.  Returns the lane's sum over its 8 positions.
template <int R>
__device__ __forceinline__ float rep_item_sum(const RepCodes<R> &q, const V16 (&xr)[8], uint32_t k0, uint32_t k1, int lane) {
    // The gathers of an item go out in kRepHalves blocks, each block issued whole before anything waits: as asm,
    // because the compiler, left to order them, takes one entry at a time through one set of registers and waits out
    // a full LDS round trip for each.  (One block of 16 needs 64 registers for the entries; two of 8 leave room for more
    // wavefronts per SIMD, which hide the second block's round trip.)  The wait is for everything (scalar loads count in the same counter and return out of order, so no partial count
    // is safe here) and names every destination, so nothing that reads one can move in front of it.
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    constexpr int G = 8 * R / kRepHalves;   // gathers per block
    // two accumulators in turn, one for each half of an entry (four, so that no matrix instruction waits for the one
    // before it, cost more in the additions at the end than the waits do: 2 % slower)
    float4_t a[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int h = 0; h < kRepHalves; ++h) {
        u32x4_t ev[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int i = h * G + g;
            // byte 0: copy column (lane constant), byte 1: the code, byte 2: codebook (lane constant), byte 3: 0
            const uint32_t sel = 0x0C060004u | ((uint32_t)(i & 3) << 8);
            const uint32_t addr = __builtin_amdgcn_perm((R == 2 && (i & 1)) ? k1 : k0, q.w[i >> 2], sel);
            asm volatile("ds_read_b128 %0, %1" : "=v"(ev[g]) : "v"(addr));
        }
        if constexpr (G == 16) {
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(ev[0]), "+v"(ev[1]), "+v"(ev[2]), "+v"(ev[3]), "+v"(ev[4]), "+v"(ev[5]), "+v"(ev[6]), "+v"(ev[7]),
                           "+v"(ev[8]), "+v"(ev[9]), "+v"(ev[10]), "+v"(ev[11]), "+v"(ev[12]), "+v"(ev[13]), "+v"(ev[14]), "+v"(ev[15]));
        } else if constexpr (G == 8) {
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(ev[0]), "+v"(ev[1]), "+v"(ev[2]), "+v"(ev[3]), "+v"(ev[4]), "+v"(ev[5]), "+v"(ev[6]), "+v"(ev[7]));
        } else {
            static_assert(G == 4, "gathers per block");
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(ev[0]), "+v"(ev[1]), "+v"(ev[2]), "+v"(ev[3]));
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int pos = (h * G + g) / R;
            const half4_t xl = rep_half4(xr[pos].w[0], xr[pos].w[1]), xh = rep_half4(xr[pos].w[2], xr[pos].w[3]);
            a[0] = __builtin_amdgcn_mfma_f32_4x4x4f16(rep_half4(ev[g].x, ev[g].y), xl, a[0], 0, 0, 0);
            a[1] = __builtin_amdgcn_mfma_f32_4x4x4f16(rep_half4(ev[g].z, ev[g].w), xh, a[1], 0, 0, 0);
        }
    }
    float4_t s = a[0] + a[1];
    asm volatile("" : "+v"(s));   // (all four sums, then two selects: no branches)
    const float s01 = (lane & 1) ? s.y : s.x, s23 = (lane & 1) ? s.w : s.z;
    return (lane & 2) ? s23 : s01;
}

template <int R, class Table>
__device__ __forceinline__ void gemv_replica_body(const Table &table, const int n, const int groups) {
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // (in a scalar register: what follows from it is uniform)
    const uint32_t k0 = (uint32_t)(lane & 15) << 4, k1 = k0 | (uint32_t)kRepCbStride;
    // The workgroups form `groups` independent groups (workgroup b: group b % groups, so a group lies on few dies);
    // group g takes problems g, g + groups, ... and splits the rows of each over its workgroups.
    const int grp = (int)blockIdx.x % groups, wb = (int)blockIdx.x / groups;
    if (grp >= n) return;

    // what this thread stages of a problem: one codebook entry and up to three 16-byte pieces of x
    struct Staged {
        uint4 ent;
        uint4 x[kRepXPer];
        float sc[2];   // scales of the rows that this thread finishes: tid and tid + 1024 of the workgroup's share
    };
    auto request = [&](const RepProblem &p) {
        Staged st;
        {
            const RepShare sh = rep_share(p, wave, wb);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int r = tid + j * kRepThreads;
                st.sc[j] = 1.f;
                if (p.scale) st.sc[j] = (float)((const __attribute__((address_space(1))) half_t *)p.scale)[sh.row0 + (r < sh.rows ? r : 0)];
            }
        }
        const uint4 z = {0u, 0u, 0u, 0u};
        const int n_ent = R * p.E;
        st.ent = rep_global16(p.cb, tid < n_ent ? tid : 0);
        const int xunits = p.K >> 3;   // 16-byte units of x
#pragma unroll
        for (int j = 0; j < kRepXPer; ++j) {
            const int ux = j * kRepThreads + tid;
            st.x[j] = rep_global16(p.x, ux < xunits ? ux : 0);
            if (ux >= xunits) st.x[j] = z;
        }
        return st;
    };
    auto stage = [&](const RepProblem &p, const Staged &st) {
        const int n_ent = R * p.E;
        if (tid < n_ent) {
            const int r = tid >= p.E ? 1 : 0, en = tid - r * p.E;   // (R <= 2)
            const uint32_t base = (uint32_t)r * kRepCbStride + (uint32_t)en * (kRepCopies * 16);
#pragma unroll
            for (int cpy = 0; cpy < kRepCopies; ++cpy) rep_lds16_store(base + (((uint32_t)(cpy + lane) & 15u) << 4), st.ent);
        }
#pragma unroll
        for (int j = 0; j < kRepXPer; ++j)
            if (j * kRepThreads + tid < kRepMaxK / 8) rep_lds16_store(kRepX + (uint32_t)(j * kRepThreads + tid) * 16u, st.x[j]);
    };

    // The codes of a wavefront's items are requested one round (kRepRound items) ahead: slot t of the ring holds item t
    // of the current round until it has been worked on and is then refilled with item t of the next round -- of the
    // same problem, or of the next problem in which the wavefront has items (every problem starts a round of its own:
    // the slots past the end of a run hold its last item once more and are never used).  `ahead` runs over the
    // problems one round in front of the work.
    int ahead_k = grp - groups;
    bool ahead_none = false;
    RepRun ahead = {0, 0, 0, 0, 0};
    const uint8_t *ahead_codes = nullptr;
    uint32_t ahead_row_bytes = 0;
    int ahead_row0 = 0, ahead_lane_chunks = 0;
    RepCodes<R> qn[kRepRound];
    auto request_slot = [&](int t) {
        if (t == 0) {
            if (ahead.u > ahead.end) ahead.u = ahead.end;
            while (!ahead_none && ahead.u >= ahead.end) {   // on to the next problem in which the wavefront has items
                ahead_k += groups;
                if (ahead_k >= n) { ahead_none = true; break; }
                const RepProblem p = table[ahead_k];
                const RepShare s = rep_share(p, wave, wb);
                ahead = rep_run(s);
                ahead_codes = p.codes;
                ahead_row_bytes = (uint32_t)(p.K >> 3) * R;
                ahead_row0 = s.row0;
                ahead_lane_chunks = s.lane_chunks;
            }
        }
        if (ahead_none) return;
        qn[t] = rep_load<R>(ahead_codes, ahead_row_bytes, ahead_row0, ahead_lane_chunks, ahead, lane);
        if (ahead.u + 1 < ahead.end || t == kRepRound - 1) rep_step(ahead);
    };

    // Row `tid` of the workgroup's share of a problem: y = fp16(scale * sum of the chunk sums, ascending).
    auto finish_rows = [&](const RepProblem &pp, const float (&sc)[2]) {
        const RepShare ps = rep_share(pp, wave, wb);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int r = tid + j * kRepThreads;
            if (r < ps.rows) {
                float sum = 0.f;
                for (int c = 0; c < ps.nch; ++c)
                    sum += *(const __attribute__((address_space(3))) float *)(uintptr_t)(kRepPart + (uint32_t)(c * ps.rows + r) * 4u);
                ((__attribute__((address_space(1))) half_t *)pp.y)[ps.row0 + r] = (half_t)(sum * sc[j]);
            }
        }
    };
    Staged st = request(table[grp]);
    float sc_done[2] = {1.f, 1.f};
#pragma unroll
    for (int t = 0; t < kRepRound; ++t) request_slot(t);
    int k_last = grp;
    for (int k = grp; k < n; k += groups) {
        k_last = k;
        const RepProblem p = table[k];
        const RepShare s = rep_share(p, wave, wb);
        if (k > grp) {
            rep_barrier();   // the chunk sums of problem k - 1 are complete, its codebooks no longer read
            finish_rows(table[k - groups], sc_done);
        }
        stage(p, st);
        sc_done[0] = st.sc[0]; sc_done[1] = st.sc[1];
        rep_barrier();
        if (k + groups < n) st = request(table[k + groups]);

        RepRun run = rep_run(s);
        int cur_c = -1;
        bool active = true;
        V16 xr[8];
        while (run.u < run.end) {
#pragma unroll
            for (int t = 0; t < kRepRound; ++t) {
                const RepCodes<R> q = qn[t];
                request_slot(t);
                if (run.u < run.end) {
                    if (run.c != cur_c) {   // (uniform) the wavefront moves to another chunk index: its x from LDS
                        cur_c = run.c;
                        const int lc = run.c * 64 + lane;
                        active = lc < s.lane_chunks;
#pragma unroll
                        for (int i = 0; i < 8; ++i) xr[i] = rep_lds16(kRepX + (uint32_t)(lc * 8 + i) * 16u);
                    }
                    // (a lane past the end of the row has computed with codes that are not its own: dropped here)
                    const float item = rep_item_sum<R>(q, xr, k0, k1, lane);
                    const float total = rep_wave_sum_to_63(active ? item : 0.f);
                    if (lane == 63)
                        *(__attribute__((address_space(3))) float *)(uintptr_t)(kRepPart + (uint32_t)(run.c * run.rows + run.row) * 4u) = total;
                    rep_step(run);
                }
            }
        }
    }
    rep_barrier();
    finish_rows(table[k_last], sc_done);
}

// The problem list lies in device memory and is read with scalar loads.
struct RepTable {
    const __attribute__((address_space(4))) unsigned char *t;
    __device__ __forceinline__ RepProblem operator[](int k) const {
        const __attribute__((address_space(4))) uint64_t *q = (const __attribute__((address_space(4))) uint64_t *)(t + (size_t)k * sizeof(RepProblem));
        const __attribute__((address_space(4))) int *qi = (const __attribute__((address_space(4))) int *)(q + 5);
        RepProblem r;
        r.codes = (const uint8_t *)q[0];
        r.cb = (const half_t *)q[1];
        r.scale = (const half_t *)q[2];
        r.x = (const half_t *)q[3];
        r.y = (half_t *)q[4];
        r.N = qi[0]; r.K = qi[1]; r.E = qi[2]; r.rows_per_wg = qi[3];
        return r;
    }
};

template <int R>
__global__ __launch_bounds__(kRepThreads) void gemv_replica_table_kernel(const RepProblem *table, int n, int groups) {
    const RepTable t{(const __attribute__((address_space(4))) unsigned char *)(uintptr_t)table};
    gemv_replica_body<R>(t, n, groups);
}

namespace {
KernelSetup g_rep_setup[2];
}  // namespace

bool gemv_replica_supported(const vq_weight_t *w) {
    if (w->code_bits != 8 || w->v != 8 || w->cb_tile_n > 0) return false;
    if (w->n_codebooks != 1 && w->n_codebooks != 2) return false;
    if (w->n_entries < 1 || w->n_entries > 256) return false;
    if (w->K < 512 || w->K > kRepMaxK || w->K % 64 != 0) return false;
    if (w->N < 1) return false;
    return true;
}

// A list of problems for one launch: the table in device memory and the launch shape.
struct GemvReplicaList {
    int device, n, R, grid, groups;
    const RepProblem *table;   // device
};

size_t gemv_replica_list_workspace(int n) { return (((size_t)n * sizeof(RepProblem)) + 255) & ~(size_t)255; }

int gemv_replica_list_create(const vq_gemv_call_t *calls, int n_calls, void *ws, hipStream_t s, GemvReplicaList **out) {
    int n = 0, max_n = 0;
    for (int c = 0; c < n_calls; ++c) n += calls[c].count;
    GemvReplicaList *h = new (std::nothrow) GemvReplicaList;
    if (!h) return VQ_ERR_LAUNCH;
    int cus = 0;
    if (hipGetDevice(&h->device) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device) != hipSuccess || cus < 1) {
        delete h;
        return VQ_ERR_LAUNCH;
    }
    for (int c = 0; c < n_calls; ++c)
        for (int i = 0; i < calls[c].count; ++i) max_n = std::max(max_n, calls[c].w[i]->N);
    // One workgroup per compute unit.  The problems are dealt to up to 32 groups of workgroups (a power of two that
    // divides the workgroups): the more rows of a problem a workgroup gets, the less its re-staging weighs.
    h->n = n;
    h->R = calls[0].w[0]->n_codebooks;
    h->grid = cus;
    h->groups = 1;
    auto fits = [&](int groups) {   // every problem's share of a workgroup within the sums buffer and two rows per thread
        const int per = h->grid / groups;
        for (int c = 0; c < n_calls; ++c)
            for (int i = 0; i < calls[c].count; ++i) {
                const vq_weight_t *w = calls[c].w[i];
                const int rows = (w->N + per - 1) / per, nch = (w->K / 64 + 63) / 64;
                if (rows > 2 * kRepThreads || rows * nch > kRepPartFloats) return false;
            }
        return true;
    };
    while (h->groups < kRepMaxGroups && h->groups * 2 <= n && h->grid % (h->groups * 2) == 0 && fits(h->groups * 2)) h->groups *= 2;
    if (!fits(h->groups)) { delete h; return VQ_ERR_UNSUPPORTED; }
    const int per_problem = h->grid / h->groups;
    std::vector<RepProblem> table((size_t)n);
    int k = 0;
    for (int c = 0; c < n_calls; ++c)
        for (int i = 0; i < calls[c].count; ++i, ++k) {
            const vq_weight_t *w = calls[c].w[i];
            RepProblem &p = table[(size_t)k];
            p.codes = (const uint8_t *)w->codes;
            p.cb = (const half_t *)w->codebooks;
            p.scale = (const half_t *)w->scale;
            p.x = (const half_t *)calls[c].x[i];
            p.y = (half_t *)calls[c].y[i];
            p.N = w->N; p.K = w->K; p.E = w->n_entries;
            p.rows_per_wg = (w->N + per_problem - 1) / per_problem;
        }
    if (hipMemcpyAsync(ws, table.data(), (size_t)n * sizeof(RepProblem), hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
        (void)hipGetLastError();
        delete h;
        return VQ_ERR_LAUNCH;
    }
    h->table = (const RepProblem *)ws;
    *out = h;
    return VQ_OK;
}

void gemv_replica_list_destroy(GemvReplicaList *h) { delete h; }

int launch_gemv_replica_list(const GemvReplicaList *h, hipStream_t s) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != h->device) return VQ_ERR_LAUNCH;
    const void *fn = h->R == 2 ? (const void *)gemv_replica_table_kernel<2> : (const void *)gemv_replica_table_kernel<1>;
    const int st = kernel_setup(fn, kRepLds, true, g_rep_setup[h->R - 1]);
    if (st != VQ_OK) return st;
    if (h->R == 2) gemv_replica_table_kernel<2><<<h->grid, kRepThreads, kRepLds, s>>>(h->table, h->n, h->groups);
    else gemv_replica_table_kernel<1><<<h->grid, kRepThreads, kRepLds, s>>>(h->table, h->n, h->groups);
    return launch_status();
}

}  // namespace vq
