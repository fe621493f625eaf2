// bs = 1 VQ-gemv from re-tiled ("packed") codes: codebook slices in LDS, LDS gathers scheduled offline.
//
// Why: with a 2^16 x 8 fp16 codebook (1 MiB) the entries cannot live in LDS, and random 16-byte gathers
// from L2 run at ~0.44 per clock per CU on MI355X (each one moves a 128-byte line), an order of magnitude
// below what the HBM code stream could feed.  LDS serves them at 5 (random addresses) to 13 (no bank
// conflicts) per clock per CU.  So the product is partitioned along the codebook itself -- the
// codebook-centric dataflow of VQ-LLM (arXiv 2503.02236) Sec. VI-A pushed from "one codebook per block" to
// "one codebook slice per block":
//   workgroup (s, rb) holds slice s (2^EB entries) and the activation vector in LDS and processes, for the
//   rows of block rb, exactly the codes that point into slice s.
// Those codes are found offline (Sec. II-C: weights are quantized offline; Sec. V-B already rewrites indices
// offline) by vq_gemv_prepack.
//
// Lane tasks.  A row's sub-vector positions are cut into P parts of Jp positions (P = 1 unless the row is
// longer than an atom's position field).  A task = (row, part): the codes of that row and part that point
// into the slice.  One lane owns one task: it gathers entry and x_j of each of its codes from LDS and
// accumulates privately, so there is no cross-lane reduction.  The tasks of a workgroup are sorted by length
// and grouped 64 at a time (one wavefront per group), so the lanes of a wavefront run nearly the same trip
// count; a group takes as many steps as its longest task needs.
//
// Atoms.  A code is stored as a 21-bit atom: EB bits entry index inside the slice (low bits), then
// XB = 21 - EB bits position inside the part.  Three atoms make a 64-bit step word (atom k in bits
// [21 k, 21 k + 21), bit 63 zero); a step of a group is a block of 64 step words, lane l's at byte 8 l.
// LDS image of a workgroup, in 16-byte units: [slice: 2^EB][part 0: Jp units of x, 16 zero units][part 1: ...],
// so an entry's address is (index << 4) and x_j's is the lane's part base + (position << 4).  A task that is
// shorter than its group is filled up with padding atoms, which name one of the 16 zero units of the part as
// x_j (and an entry that some code of the same group uses) and add entry * 0: no validity test in the loop.
// (Entries that no code points at are never read; entries in use must be finite.)
//
// Order of a task's atoms = order of the additions to its sum; it is fixed offline, so results are
// bit-reproducible -- and it is free.  LDS serves the 16-byte reads of a wavefront in four passes of 16 lanes
// (measured on MI355X, two lanes at a time against a background of one shared address: lanes 0-3, 12-15 and
// 20-27 go together, lanes 4-11, 16-19 and 28-31, and the same two sets in the upper half of the wavefront) and
// needs one more pass for every further distinct address that falls into the same 16-byte column
// (address / 16 mod 16) inside such a set: random addresses take ~2.6 passes each.  The packer therefore orders
// the atoms of every such set of 16 lanes so that, position by position, their entry addresses and their x
// addresses hit different columns wherever the lists allow it (greedy, the lanes with the least room first;
// padding atoms go where nothing fits and pick a free zero unit).
//
// The S partial sums of a row are added in slice order by a second small kernel (Sec. VI-A "explicit global
// reduction"), which keeps the result independent of timing.
//
// Packed buffer (little endian; offsets from the start of the buffer, each 256-byte aligned):
//   task table   [S*RB][G][64] uint16   slot of lane l of group g: part * rows_per_block + row inside the block;
//                                       0xFFFF = idle lane.  G = ceil(rows_per_block * P / 64)
//   step table   [S*RB][G] uint32       steps of group g of this workgroup
//   atoms        blocks of 512 bytes; group g of workgroup wg starts at block
//                wg * wg_pitch + sum_{g' < g} group_steps[g'], where group_steps[g] (in the descriptor) is the
//                maximum over all workgroups: every address follows from launch arguments alone, and only the
//                trip counts come from the step table (one scalar load, issued first, needed after the slice
//                has landed).  Blocks between a group's own steps and group_steps[g] hold padding atoms and are
//                read only by a few blocks of prefetch; 16 more padding blocks follow the last workgroup's.
// Codes too uneven for a common address shape (skewed code distributions: more than a quarter more blocks than
// needed and more than 1 MiB of them) are declined: the canonical-code kernels serve them.
#include <algorithm>
#include <cstring>
#include <thread>
#include <type_traits>
#include <cstddef>
#include <new>
#include <vector>

#include "vq_common.h"

namespace vq {

constexpr int kAtomBits = 21;
constexpr int kStepAtoms = 3;
constexpr int kZeroUnits = 16;        // zero units behind every part of x: one per 16-byte column
constexpr int kStepBytes = 512;       // 64 lanes x 8 bytes
// atom blocks behind the last workgroup's: the kernels read up to this many blocks past the end of a group
// without looking (a clamp per load costs more instructions than the load)
constexpr int kPackTailBlocks = 16;
constexpr int kPackMaxParts = 8;
constexpr size_t kPackMaxLds = 144 * 1024;
#ifndef VQ_PACK_TARGET_WGS
#define VQ_PACK_TARGET_WGS 256
#endif
constexpr uint32_t kPackTargetWgs = VQ_PACK_TARGET_WGS;

struct PackPlan {
    uint32_t EB, XB, slice_entries, S, RB, rows_per_block, P, Jp, tasks, G;
    size_t lds;   // bytes of the workgroup's LDS image + accumulator buffer
};

static size_t pack_lds_bytes(uint32_t slice_entries, uint32_t P, uint32_t Jp, uint32_t tasks) {
    return ((size_t)slice_entries + (size_t)P * (Jp + kZeroUnits)) * 16 + (size_t)tasks * sizeof(float);
}

// S * RB = 256 workgroups, one per compute unit, when the matrix has rows enough.
static bool pack_plan(const vq_weight_t *w, PackPlan *out) {
    if (w->v != 8 || w->code_bits != 16 || w->n_codebooks != 1) return false;
    const int E = w->n_entries;
    if (E < 4096 || (E & (E - 1)) != 0) return false;
    if (w->K <= 0 || w->N <= 0) return false;
    PackPlan p;
    p.EB = 11;
    p.XB = kAtomBits - p.EB;
    p.slice_entries = 1u << p.EB;
    const uint32_t J = (uint32_t)w->K / 8, cap = (1u << p.XB) - kZeroUnits;
    p.P = (J + cap - 1) / cap;
    if (p.P > (uint32_t)kPackMaxParts) return false;
    p.Jp = (J + p.P - 1) / p.P;
    p.S = (uint32_t)E / p.slice_entries;
    uint32_t rb = kPackTargetWgs / p.S;
    const uint32_t max_rb = ((uint32_t)w->N + 63) / 64;   // at least one full 64-row group per block
    if (rb > max_rb) rb = max_rb;
    if (rb < 1) rb = 1;
    p.RB = rb;
    p.rows_per_block = ((uint32_t)w->N + rb - 1) / rb;
    p.tasks = p.rows_per_block * p.P;
    p.G = (p.tasks + 63) / 64;
    if (p.G > VQ_PACK_MAX_GROUPS || p.tasks >= 0xFFFFu) return false;
    p.lds = pack_lds_bytes(p.slice_entries, p.P, p.Jp, p.tasks);
    if (p.lds > kPackMaxLds) return false;
    *out = p;
    return true;
}

static bool pack_supported(const vq_weight_t *w) {
    PackPlan p;
    return pack_plan(w, &p);
}

static inline uint64_t align256(uint64_t x) { return (x + 255) & ~(uint64_t)255; }

namespace {

// The four sets of 16 lanes whose 16-byte LDS reads are served in one pass each (see the head of this file).
const uint8_t kLdsPassLanes[4][16] = {
    {0, 1, 2, 3, 12, 13, 14, 15, 20, 21, 22, 23, 24, 25, 26, 27},
    {4, 5, 6, 7, 8, 9, 10, 11, 16, 17, 18, 19, 28, 29, 30, 31},
    {32, 33, 34, 35, 44, 45, 46, 47, 52, 53, 54, 55, 56, 57, 58, 59},
    {36, 37, 38, 39, 40, 41, 42, 43, 48, 49, 50, 51, 60, 61, 62, 63}};

struct HostAtom {
    uint16_t e, x;   // entry index inside the slice, position inside the part
};

// Order of the atoms of 16 lanes that LDS serves in one pass, over `npos` positions.  lists[l] holds lane l's atoms
// (at most npos of them; consumed); col0[l] is the 16-byte column of position 0 of lane l's part, so position
// x of that lane lies in column (x + col0[l]) % 16 and its zero units (positions Jp .. Jp + 15) cover every
// column.  out[l * npos + pos] receives the 21-bit atoms, padding included.  Greedy, position by position: the
// lanes with the least room to wait choose first; a lane takes an atom whose entry column and x column are
// both still free at this position; if none is, it looks for one lane that chose before it and can move to
// another of its atoms to make room; failing that it waits (takes a padding atom) if it has room, and otherwise
// takes the atom that adds the fewest passes.  Deterministic.
void order_quad(std::vector<HostAtom> (&lists)[16], const uint32_t (&col0)[16], const int (&pad_entry)[16], uint32_t npos,
                uint32_t EB, uint32_t Jp, uint32_t *out) {
    uint32_t rem[16];
    for (int l = 0; l < 16; ++l) rem[l] = (uint32_t)lists[l].size();
    auto ecol = [&](int l, int i) { return (int)(lists[l][i].e & 15u); };
    auto xcol = [&](int l, int i) { return (int)((lists[l][i].x + col0[l]) & 15u); };
    for (uint32_t pos = 0; pos < npos; ++pos) {
        uint8_t ue[16] = {0}, ux[16] = {0};
        int8_t owner_e[16], owner_x[16];   // the lane that holds a column alone (-1: free or shared)
        for (int c = 0; c < 16; ++c) owner_e[c] = owner_x[c] = -1;
        int chosen[16];                     // index of the atom a lane takes at this position, -1: padding
        for (int l = 0; l < 16; ++l) chosen[l] = -1;
        const uint32_t left = npos - pos;
        int order[16];
        for (int l = 0; l < 16; ++l) order[l] = l;
        std::stable_sort(order, order + 16, [&](int a, int b) { return (left - rem[a]) < (left - rem[b]); });
        auto take = [&](int l, int i) {
            chosen[l] = i;
            const int ce = ecol(l, i), cx = xcol(l, i);
            owner_e[ce] = ue[ce] == 0 ? (int8_t)l : (int8_t)-1;
            owner_x[cx] = ux[cx] == 0 ? (int8_t)l : (int8_t)-1;
            ++ue[ce];
            ++ux[cx];
        };
        auto drop = [&](int l) {   // only for a lane that holds both of its columns alone
            const int ce = ecol(l, chosen[l]), cx = xcol(l, chosen[l]);
            ue[ce] = ux[cx] = 0;
            owner_e[ce] = owner_x[cx] = -1;
            chosen[l] = -1;
        };
        for (int oi = 0; oi < 16; ++oi) {
            const int l = order[oi];
            if (rem[l] == 0) continue;
            const uint32_t slack = left - rem[l];
            int best = -1, best_score = 1 << 30;
            for (uint32_t i = 0; i < rem[l]; ++i) {
                const int sc = ue[ecol(l, (int)i)] + ux[xcol(l, (int)i)];
                if (sc < best_score) {
                    best_score = sc;
                    best = (int)i;
                    if (sc == 0) break;
                }
            }
            if (best_score == 0) {
                take(l, best);
                continue;
            }
            // no atom of this lane fits as things stand: see whether ONE lane that chose earlier can move to
            // another of its atoms and make room (its columns are its own, so moving it frees them)
            bool done = false;
            for (uint32_t i = 0; i < rem[l] && !done; ++i) {
                const int ce = ecol(l, (int)i), cx = xcol(l, (int)i);
                if (ue[ce] > 1 || ux[cx] > 1) continue;
                const int be = ue[ce] ? owner_e[ce] : -1, bx = ux[cx] ? owner_x[cx] : -1;
                if ((ue[ce] && be < 0) || (ux[cx] && bx < 0)) continue;
                if (be >= 0 && bx >= 0 && be != bx) continue;        // two different lanes in the way
                const int b = be >= 0 ? be : bx;
                const int bce = ecol(b, chosen[b]), bcx = xcol(b, chosen[b]);
                if (owner_e[bce] != b || owner_x[bcx] != b) continue;  // (b shares a column already: leave it)
                const int old = chosen[b];
                drop(b);
                for (uint32_t k = 0; k < rem[b]; ++k) {
                    if ((int)k == old) continue;
                    const int kce = ecol(b, (int)k), kcx = xcol(b, (int)k);
                    if (ue[kce] || ux[kcx] || kce == ce || kcx == cx) continue;
                    take(b, (int)k);
                    take(l, (int)i);
                    done = true;
                    break;
                }
                if (!done) take(b, old);
            }
            if (done) continue;
            if (slack > 0) continue;   // wait: a padding atom goes here
            // must go now: the atom that raises the passes of this position least
            int me = 0, mx = 0;
            for (int c = 0; c < 16; ++c) {
                me = std::max<int>(me, ue[c]);
                mx = std::max<int>(mx, ux[c]);
            }
            best = 0;
            best_score = 1 << 30;
            for (uint32_t i = 0; i < rem[l]; ++i) {
                const int ce = ecol(l, (int)i), cx = xcol(l, (int)i);
                const int sc = 16 * (std::max(me, ue[ce] + 1) + std::max(mx, ux[cx] + 1)) + ue[ce] + ux[cx];
                if (sc < best_score) {
                    best_score = sc;
                    best = (int)i;
                }
            }
            take(l, best);
        }
        // write the position out and remove the atoms taken (highest list index first is not needed: one per lane)
        for (int l = 0; l < 16; ++l) {
            if (chosen[l] < 0) continue;
            const HostAtom a = lists[l][chosen[l]];
            lists[l][chosen[l]] = lists[l][rem[l] - 1];
            --rem[l];
            out[l * npos + pos] = (uint32_t)a.e | ((uint32_t)a.x << EB);
        }
        // padding atoms: the least used zero unit, and the least used entry column among those that have an
        // entry which a code of this group really uses (pad_entry[c], -1 if none: a padding atom never reads an
        // entry that no code points at)
        for (int l = 0; l < 16; ++l) {
            if (chosen[l] >= 0) continue;
            int ce = -1, cx = 0;
            for (int c = 0; c < 16; ++c) {
                if (pad_entry[c] >= 0 && (ce < 0 || ue[c] < ue[ce])) ce = c;
                if (ux[c] < ux[cx]) cx = c;
            }
            ++ue[ce];
            ++ux[cx];
            const uint32_t zx = Jp + ((uint32_t)cx + 32u - ((Jp + col0[l]) & 15u)) % 16u;   // the zero unit in column cx
            out[l * npos + pos] = (uint32_t)pad_entry[ce] | (zx << EB);
        }
    }
}

unsigned pack_threads() {
    unsigned n = std::thread::hardware_concurrency();
    if (n < 1) n = 1;
    return n > 16 ? 16 : n;
}

template <class F>
void parallel_for(uint32_t n, F f) {
    const unsigned nt = std::min<unsigned>(pack_threads(), n);
    if (nt <= 1) {
        for (uint32_t i = 0; i < n; ++i) f(i);
        return;
    }
    std::vector<std::thread> th;
    for (unsigned t = 0; t < nt; ++t)
        th.emplace_back([=]() {
            for (uint32_t i = t; i < n; i += nt) f(i);
        });
    for (auto &t : th) t.join();
}

}  // namespace

// One function builds everything; `out` == nullptr only measures.  Returns 0 when the matrix has no packed
// form; *bad_code is set when that is because a code >= n_entries was found.
static uint64_t pack_build(const vq_weight_t *w, unsigned char *out, vq_gemv_pack_t *pack, bool *bad_code) {
    PackPlan p;
    if (bad_code) *bad_code = false;
    if (!pack_plan(w, &p)) return 0;
    const uint32_t J = (uint32_t)w->K / 8, N = (uint32_t)w->N;
    const uint16_t *codes = reinterpret_cast<const uint16_t *>(w->codes);
    const uint32_t nwg = p.S * p.RB, ng = p.G;
    if ((uint32_t)w->n_entries < 65536u) {   // (with 2^16 entries every uint16 code is valid)
        std::vector<int> bad(p.RB, 0);
        parallel_for(p.RB, [&](uint32_t rb) {
            const uint32_t r0 = rb * p.rows_per_block, r1 = std::min<uint64_t>(N, (uint64_t)r0 + p.rows_per_block);
            for (uint32_t n = r0; n < r1; ++n)
                for (uint32_t j = 0; j < J; ++j)
                    if (codes[(size_t)n * J + j] >= (uint32_t)w->n_entries) bad[rb] = 1;
        });
        for (int b : bad)
            if (b) {
                if (bad_code) *bad_code = true;
                return 0;
            }
    }

    // pass 1: lengths of all tasks; per workgroup the tasks sorted by length (descending, ties by slot)
    std::vector<uint32_t> cnt((size_t)nwg * p.tasks, 0);
    parallel_for(p.RB, [&](uint32_t rb) {
        const uint32_t r0 = rb * p.rows_per_block, r1 = std::min<uint64_t>(N, (uint64_t)r0 + p.rows_per_block);
        for (uint32_t n = r0; n < r1; ++n) {
            const uint16_t *row = codes + (size_t)n * J;
            for (uint32_t j = 0; j < J; ++j) {
                const uint32_t s = row[j] >> p.EB, part = j / p.Jp;
                ++cnt[((size_t)s * p.RB + rb) * p.tasks + part * p.rows_per_block + (n - r0)];
            }
        }
    });
    std::vector<uint16_t> slots((size_t)nwg * ng * 64, 0xFFFF);
    std::vector<uint32_t> steps((size_t)nwg * ng, 0);
    parallel_for(nwg, [&](uint32_t wg) {
        const uint32_t rb = wg % p.RB;
        uint32_t rows_here = 0;
        if ((uint64_t)rb * p.rows_per_block < N) rows_here = std::min<uint32_t>(p.rows_per_block, N - rb * p.rows_per_block);
        const uint32_t *c = &cnt[(size_t)wg * p.tasks];
        std::vector<uint32_t> order;
        order.reserve(p.tasks);
        for (uint32_t part = 0; part < p.P; ++part)
            for (uint32_t r = 0; r < rows_here; ++r) order.push_back(part * p.rows_per_block + r);
        std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return c[a] > c[b]; });
        for (uint32_t g = 0; g < ng; ++g) {
            const size_t first = (size_t)g * 64;
            // a group's first task is its longest
            steps[(size_t)wg * ng + g] = first < order.size() ? (c[order[first]] + kStepAtoms - 1) / kStepAtoms : 0;
            for (uint32_t l = 0; l < 64; ++l)
                if (first + l < order.size()) slots[((size_t)wg * ng + g) * 64 + l] = (uint16_t)order[first + l];
        }
    });
    // the common address shape of all workgroups (at least one block each: wavefronts without work read it)
    std::vector<uint32_t> max_steps(ng, 0), prefix(ng, 0);
    uint64_t needed_blocks = 0;
    for (uint32_t wg = 0; wg < nwg; ++wg)
        for (uint32_t g = 0; g < ng; ++g) {
            max_steps[g] = std::max(max_steps[g], steps[(size_t)wg * ng + g]);
            needed_blocks += steps[(size_t)wg * ng + g];
        }
    if (max_steps[0] == 0) max_steps[0] = 1;
    uint64_t pitch = 0;
    for (uint32_t g = 0; g < ng; ++g) {
        prefix[g] = (uint32_t)pitch;
        pitch += max_steps[g];
    }
    if (pitch > 65535) return 0;
    // too uneven: more than a quarter more blocks than needed -- unless that is less than 1 MiB (small or
    // ragged matrices, where a group of a few tasks is as long as its longest task in the unluckiest workgroup)
    const uint64_t padded = pitch * nwg;
    if (padded > needed_blocks + needed_blocks / 4 + nwg && (padded - needed_blocks) * kStepBytes > (1u << 20)) return 0;

    const uint64_t task_off = 0;
    const uint64_t steps_off = align256(task_off + slots.size() * 2);
    const uint64_t atom_off = align256(steps_off + steps.size() * 4);
    const uint64_t total = atom_off + (padded + kPackTailBlocks) * kStepBytes;
    if (pack) {
        std::memset(pack, 0, sizeof(*pack));
        pack->data = out;
        pack->bytes = total;
        pack->S = p.S;
        pack->RB = p.RB;
        pack->rows_per_block = p.rows_per_block;
        pack->entry_bits = p.EB;
        pack->parts = p.P;
        pack->part_cols = p.Jp;
        pack->wg_pitch = (uint32_t)pitch;
        pack->task_off = task_off;
        pack->steps_off = steps_off;
        pack->atom_off = atom_off;
        for (uint32_t g = 0; g < VQ_PACK_MAX_GROUPS; ++g) pack->group_steps[g] = g < ng ? (uint16_t)max_steps[g] : (uint16_t)0;
    }
    if (!out) return total;

    std::memset(out, 0, (size_t)atom_off);
    std::memcpy(out + task_off, slots.data(), slots.size() * 2);
    std::memcpy(out + steps_off, steps.data(), steps.size() * 4);
    uint64_t *words = reinterpret_cast<uint64_t *>(out + atom_off);   // out is 16-byte aligned, atom_off 256
    // padding everywhere first (blocks that no group uses: read by prefetches at most, never consumed)
    {
        const uint64_t pad = (uint64_t)p.Jp << p.EB;
        const uint64_t pw = pad | (pad << kAtomBits) | (pad << (2 * kAtomBits));
        const uint64_t n_words = (padded + kPackTailBlocks) * 64;
        parallel_for(64, [&](uint32_t t) {
            const uint64_t a = n_words * t / 64, b = n_words * (t + 1) / 64;
            for (uint64_t i = a; i < b; ++i) words[i] = pw;
        });
    }
    // pass 2: per row block the atoms of every (slice, task), then per workgroup and 16 lanes their order
    parallel_for(p.RB, [&](uint32_t rb) {
        const uint32_t r0 = rb * p.rows_per_block, r1 = std::min<uint64_t>(N, (uint64_t)r0 + p.rows_per_block);
        std::vector<std::vector<HostAtom>> lists((size_t)p.S * p.tasks);
        for (uint32_t s = 0; s < p.S; ++s)
            for (uint32_t t = 0; t < p.tasks; ++t)
                lists[(size_t)s * p.tasks + t].reserve(cnt[((size_t)s * p.RB + rb) * p.tasks + t]);
        for (uint32_t n = r0; n < r1; ++n) {
            const uint16_t *row = codes + (size_t)n * J;
            for (uint32_t j = 0; j < J; ++j) {
                const uint32_t s = row[j] >> p.EB, part = j / p.Jp;
                lists[(size_t)s * p.tasks + part * p.rows_per_block + (n - r0)].push_back(
                    HostAtom{(uint16_t)(row[j] & (p.slice_entries - 1)), (uint16_t)(j - part * p.Jp)});
            }
        }
        std::vector<uint32_t> ordered;
        for (uint32_t s = 0; s < p.S; ++s) {
            const uint32_t wg = s * p.RB + rb;
            for (uint32_t g = 0; g < ng; ++g) {
                const uint32_t st = steps[(size_t)wg * ng + g], npos = st * kStepAtoms;
                if (st == 0) continue;
                const uint64_t first_block = (uint64_t)wg * pitch + prefix[g];
                ordered.assign((size_t)16 * npos, 0);
                // one really used entry per 16-byte column, for the padding atoms (the group's first task has an
                // atom, or the group would have no steps)
                int pad_entry[16];
                for (int c = 0; c < 16; ++c) pad_entry[c] = -1;
                for (uint32_t l = 0; l < 64; ++l) {
                    const uint16_t slot = slots[((size_t)wg * ng + g) * 64 + l];
                    if (slot == 0xFFFF) continue;
                    for (const HostAtom &a : lists[(size_t)s * p.tasks + slot])
                        if (pad_entry[a.e & 15u] < 0) pad_entry[a.e & 15u] = a.e;
                }
                for (uint32_t q = 0; q < 4; ++q) {
                    std::vector<HostAtom> quad[16];
                    uint32_t col0[16];
                    for (uint32_t l = 0; l < 16; ++l) {
                        const uint16_t slot = slots[((size_t)wg * ng + g) * 64 + kLdsPassLanes[q][l]];
                        const uint32_t part = slot == 0xFFFF ? 0 : slot / p.rows_per_block;
                        if (slot != 0xFFFF) quad[l].swap(lists[(size_t)s * p.tasks + slot]);
                        // unit of position 0 of the part: slice_entries + part * (Jp + 16); slices are multiples of 16 units
                        col0[l] = (part * (p.Jp + kZeroUnits)) & 15u;
                    }
                    order_quad(quad, col0, pad_entry, npos, p.EB, p.Jp, ordered.data());
                    for (uint32_t l = 0; l < 16; ++l) {
                        const uint32_t lane = kLdsPassLanes[q][l];
                        for (uint32_t t = 0; t < st; ++t) {
                            const uint64_t a0 = ordered[l * npos + 3 * t], a1 = ordered[l * npos + 3 * t + 1],
                                           a2 = ordered[l * npos + 3 * t + 2];
                            words[(first_block + t) * 64 + lane] = a0 | (a1 << kAtomBits) | (a2 << (2 * kAtomBits));
                        }
                    }
                }
            }
        }
    });
    return total;
}

// ---------------------------------------------------------------------------------- kernel

// What the main kernel needs of the launch arguments before its first vector load leaves ...
struct PackedCore {
    const unsigned char *data;
    const half_t *cb, *x;
    float *partial;       // [S][N]
    int N, J, S, RB, rows_per_block;
    int EB;               // entry bits of an atom; slices of 2^EB entries
    int P, Jp;            // parts of a row, positions per part
    int n_groups;         // groups (of 64 tasks) per workgroup
    int nwaves;           // wavefronts per workgroup of the launch (saves a load of the hidden launch arguments)
    unsigned wg_pitch;    // group g of workgroup wg: atom blocks from wg * wg_pitch + prefix[g] on
    unsigned long long task_off, steps_off, atom_off;
};
// ... and the rest: one 32-bit word per group, prefix << 16 | common steps, so that a scalar load can fetch it
struct PackedArgs : PackedCore {
    const half_t *scale;
    half_t *y;
    uint32_t group[VQ_PACK_MAX_GROUPS];
};

// Keeps a launch argument in scalar registers from here on.  Left to itself the compiler fetches each
// argument where it is first used (and again later rather than keep it): seven dependent round trips of
// 35 - 400 ns each at the head of the gemv kernel, before the first vector load leaves.
template <class T>
__device__ __forceinline__ void pin_scalar(T &v) {
    asm volatile("" : "+s"(v));
}

constexpr int kPackMaxSlices = 32;  // 2^16 entries / 2048 per slice
// Steps in flight per wavefront (8 bytes per lane each), and how many of them are requested before the barrier.
// More requested ahead does not arrive sooner: what is requested ahead of another wavefront's slice transfer
// delays that transfer and with it the barrier.
constexpr int kPackAhead = 2;

// 16 bytes at an absolute LDS address.  The kernels below have no static LDS, so the dynamic region (the
// image the atoms index) starts at address 0 and a unit number is an address after one shift; going through
// a pointer into the region would cost one more add per gather for a base the compiler cannot see is 0.
// (A test compiles this file and checks that these kernels have no static LDS; the launcher checks it too.)
__device__ __forceinline__ V16 lds_unit(uint32_t byte_address) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t v = *(const __attribute__((address_space(3))) u32x4_t *)(uintptr_t)byte_address;
    V16 r;
    r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
    return r;
}

__device__ __forceinline__ float atom_fma(const V16 &e, const V16 &xv, float acc) {
    acc = dot2(e.h2[0], xv.h2[0], acc);
    acc = dot2(e.h2[1], xv.h2[1], acc);
    acc = dot2(e.h2[2], xv.h2[2], acc);
    return dot2(e.h2[3], xv.h2[3], acc);
}

struct Acc3 {
    float a[3];
};
// What turns an atom into its two LDS addresses: (atom & emask) << 4 and ((atom >> EB) & xmask) << 4 + xbase.
struct AtomDecode {
    uint32_t emask4;   // ((1 << EB) - 1) << 4
    uint32_t eb, xb;   // field widths
    uint32_t xbase;    // byte address of position 0 of this lane's part
    uint32_t ebase;    // byte address of the slice (a multiple of the slice size: OR-ed in); 0 in the one-image kernels
};

// NST steps at once (one or two): the 6 NST gathers (entry and x_j of every atom) are issued before the
// first dot product -- taken one atom at a time, as the compiler orders them when left alone, every atom
// waits out a full LDS round trip.  Atom k of a step always adds into accumulator k, so two steps taken
// together give the same sums as taken one after the other.
template <int NST>
__device__ __forceinline__ void steps_dot(const uint32_t (&lo)[NST], const uint32_t (&hi)[NST], const AtomDecode &d, Acc3 &acc) {
    uint32_t at[3 * NST];
#pragma unroll
    for (int s = 0; s < NST; ++s) {
        at[3 * s] = lo[s];
        at[3 * s + 1] = __builtin_amdgcn_alignbit(hi[s], lo[s], kAtomBits);
        at[3 * s + 2] = hi[s] >> (2 * kAtomBits - 32);
    }
    V16 e[3 * NST], xv[3 * NST];
#pragma unroll
    for (int i = 0; i < 3 * NST; ++i) {
        e[i] = lds_unit(((at[i] << 4) & d.emask4) | d.ebase);
        xv[i] = lds_unit((__builtin_amdgcn_ubfe(at[i], d.eb, d.xb) << 4) + d.xbase);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 6 * NST, 0);   // these LDS reads first,
    __builtin_amdgcn_sched_group_barrier(0x002, 12 * NST, 0);  // then the arithmetic on them
#pragma unroll
    for (int i = 0; i < 3 * NST; ++i) acc.a[i % 3] = atom_fma(e[i], xv[i], acc.a[i % 3]);
}

// (pointers that went through pin_scalar, or came out of a table, have to be told that they are global)
typedef const __attribute__((address_space(1))) unsigned char gbyte_t;
typedef const __attribute__((address_space(1))) uint16_t gu16_t;
typedef const __attribute__((address_space(1))) uint32_t gu32_t;
typedef const __attribute__((address_space(4))) uint32_t cu32_t;   // read with scalar loads

// Step st of the group whose first block this lane sees at `base`.  No look at the group's length: a
// branch around a load keeps the compiler from counting which loads are in flight (it then waits for
// all of them before every use), and a clamp costs more instructions than the load.  Blocks past the
// end of a group belong to the next one, or to the tail of the buffer, and are never used.
__device__ __forceinline__ void load_step(uint32_t (&dst)[2], gbyte_t *base, uint32_t st) {
    gu32_t *p = (gu32_t *)(base + (size_t)st * kStepBytes);
    dst[0] = p[0]; dst[1] = p[1];
}

// The sum of one task (lane) over the n_steps steps of its group.  The ring q holds the group's first PF
// steps (requested, not necessarily landed); slot k is refilled with step st + PF as soon as step st has been
// taken out of it -- except in the group's last round: what would be requested there lies past the end of the
// group.  Steps are taken two at a time when PAIR.
template <int PF, bool PAIR>
__device__ __forceinline__ float unit_sum(uint32_t (&q)[PF][2], gbyte_t *gbase, const uint32_t n_steps, const AtomDecode &dec) {
    static_assert(!PAIR || PF % 2 == 0, "steps are taken two at a time");
    static_assert(2 * PF - 2 <= kPackTailBlocks, "reads run up to 2 PF - 2 blocks past the end of a group");
    Acc3 acc = {{0.f, 0.f, 0.f}};
    auto ring_round = [&](uint32_t base, auto refill_tag) {
        if constexpr (PAIR) {
#pragma unroll
            for (int k = 0; k < PF; k += 2) {
                const uint32_t lo[2] = {q[k][0], q[k + 1][0]}, hi[2] = {q[k][1], q[k + 1][1]};
                if constexpr (decltype(refill_tag)::value) {
                    load_step(q[k], gbase, base + k + PF);
                    load_step(q[k + 1], gbase, base + k + 1 + PF);
                }
                if (base + k + 1 < n_steps) {
                    steps_dot<2>(lo, hi, dec, acc);
                } else if (base + k < n_steps) {
                    const uint32_t lo1[1] = {lo[0]}, hi1[1] = {hi[0]};
                    steps_dot<1>(lo1, hi1, dec, acc);
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < PF; ++k) {
                const uint32_t lo1[1] = {q[k][0]}, hi1[1] = {q[k][1]};
                if constexpr (decltype(refill_tag)::value) load_step(q[k], gbase, base + k + PF);
                if (base + k < n_steps) steps_dot<1>(lo1, hi1, dec, acc);
            }
        }
    };
    // (the first round outside the loop: at a loop head the ring would be copied, and a copy needs
    // all of its data)
    uint32_t base = 0;
    if (n_steps > (uint32_t)PF) {
        ring_round(0, std::true_type{});
        for (base = PF; base + PF < n_steps; base += PF) ring_round(base, std::true_type{});
    }
    if (n_steps > 0) ring_round(base, std::false_type{});
    return (acc.a[0] + acc.a[1]) + acc.a[2];
}

// Direct global -> LDS transfers (no registers).  M0 is written and used inside one asm statement only; it is a
// reserved register that the compiler neither allocates nor accepts in a clobber list, and nothing else in
// these kernels uses it.
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
// 64 lanes x 16 bytes -> dst_wave_base + 16 lane
__device__ __forceinline__ void dma_1k(const uint4 *src_lane, unsigned char *dst_wave_base) {
    const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_byte_t *)dst_wave_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(m0), "v"(src_lane) : "memory");
}
// a contiguous 4 KiB: four such transfers 1 KiB apart in both address spaces, one M0 write
__device__ __forceinline__ void dma_4k(const uint4 *src_lane, unsigned char *dst_wave_base) {
    const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_byte_t *)dst_wave_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, off\n\t"
                 "global_load_lds_dwordx4 %1, off offset:1024\n\t"
                 "global_load_lds_dwordx4 %1, off offset:2048\n\t"
                 "global_load_lds_dwordx4 %1, off offset:3072" ::"s"(m0), "v"(src_lane) : "memory");
}

// Workgroup number -> (codebook slice, row block).  Workgroups are dealt round-robin to the 8 compute dies, each
// with its own L2.  All row blocks of one codebook slice run on the same die, so a slice is fetched from memory
// by one L2 only (otherwise every die pulls the whole 1 MiB codebook: 8 MiB per launch).
__device__ __forceinline__ void slice_and_block(int bid, int S, int RB, int &s, int &rb) {
    if (S % 8 == 0) {  // S is a power of two: shifts instead of a division
        const int die = bid & 7, local = bid >> 3, per_die = S >> 3, sh = __builtin_ctz(per_die);
        s = die * per_die + (local & (per_die - 1));
        rb = local >> sh;
    } else {
        s = bid / RB;
        rb = bid % RB;
    }
}

// The LDS image of one workgroup: codebook slice s, then the parts of x with kZeroUnits zero units (what padding
// atoms point at) behind each.  Wavefronts wave = 0 .. nwaves - 1 share the transfers: 4 KiB chunks dealt in turn.
__device__ __forceinline__ void stage_image(const half_t *cb, const half_t *x, int s, uint32_t slice_entries, int P, int Jp,
                                            int J, unsigned char *img, int wave, int nwaves, int lane) {
    const uint32_t slice_bytes = slice_entries * 16u;
    const uint32_t part_pitch = ((uint32_t)Jp + kZeroUnits) * 16u;
    unsigned char *xl = img + slice_bytes;
    const uint4 *src = reinterpret_cast<const uint4 *>(cb) + (size_t)s * slice_entries;
    const uint4 *xs = reinterpret_cast<const uint4 *>(x);
    const int slice_chunks = (int)(slice_bytes >> 12);          // slices are multiples of 256 entries
    for (int c = wave; c < slice_chunks; c += nwaves) dma_4k(src + c * 256 + lane, img + c * 4096);
    int turn = slice_chunks;   // whose turn the next chunk is
    for (int p = 0; p < P; ++p) {
        const int len = min(Jp, J - p * Jp);   // positions of this part
        const uint4 *xp = xs + p * Jp;
        unsigned char *dst = xl + (size_t)p * part_pitch;
        const int full = len >> 8;             // whole 4 KiB chunks
        for (int c = 0; c < full; ++c, ++turn)
            if (turn % nwaves == wave) dma_4k(xp + c * 256 + lane, dst + c * 4096);
        if ((len & 255) && turn % nwaves == wave)    // the rest of the part: up to three transfers, the last one partly masked
            for (int t = full * 4; t * 64 < len; ++t)
                if (t * 64 + lane < len) dma_1k(xp + t * 64 + lane, dst + t * 1024);
        turn += (len & 255) ? 1 : 0;
    }
    for (int i = wave * 64 + lane; i < P * 64; i += nwaves * 64)
        reinterpret_cast<uint32_t *>(xl + (size_t)(i >> 6) * part_pitch + (size_t)Jp * 16)[i & 63] = 0u;
}

// ---- the global reduction of the PREVIOUS launch, done in the prologue and epilogue of this one -------------
// A launch leaves S partial sums per row; adding them needs every workgroup of that launch to have finished,
// i.e. a kernel boundary.  When several products follow each other on a stream (vq_gemv_sequence), the next
// launch is that boundary: each of its workgroups takes a share of the pending rows, requests their partial
// sums straight into LDS at its very start (no registers; the requests travel with the slice transfers) and
// adds them up in slice order after its own work, so the reduction costs no launch of its own.  The last
// launch of a sequence is followed by the plain reduction kernel.  The pending rows are handed out in blocks
// of 64 (one wavefront each), at most kFinChunks per workgroup.
constexpr int kPackMaxBatch = 4;
constexpr int kFinChunks = 2;        // a workgroup takes at most this many blocks of 64 pending rows
constexpr int kFinChunkBytes = 8192; // LDS per block: 32 slices x 64 rows x 4 bytes
// Layout of the partial sums of one problem: blocks of 64 rows, [block][slice][row % 64] -- the S x 64 sums of
// a block are contiguous, so the next launch fetches them with a few wide transfers.  (The workspace is 4 KiB
// longer than the sums: a block is fetched in units of 4 KiB, whatever S is.)
__host__ __device__ __forceinline__ size_t partial_index(int S, int s, int n) {
    return ((size_t)(n >> 6) * S + s) * 64 + (n & 63);
}
// The epilogue y = fp16(scale * sum): the fp32 product is rounded to fp32 first and to fp16 (nearest even)
// second, in every kernel that finishes a row.  The empty asm statement keeps the compiler from merging the
// multiplication into a mixed-precision instruction that rounds only once in one kernel and not in another:
// the reduction folded into a following launch must give the bits of the reduction kernel.
__device__ __forceinline__ half_t scaled_output(float sum, float sc) {
    float prod = sum * sc;
    asm volatile("" : "+v"(prod));
    return (half_t)prod;
}
struct FinalizeArgs {
    const float *partial;   // blocked, see partial_index
    const half_t *scale;    // [N] or null
    half_t *y;              // [N]
    int N, S;
};
struct PendingArgs {
    FinalizeArgs a[kPackMaxBatch];
    int first_block[kPackMaxBatch];   // where problem i starts in the list of blocks (INT_MAX past the last problem)
    int count;            // pending problems (0: nothing to do)
    int blocks_total;     // sum of their ceil(N / 64): the blocks form one list, problem after problem
    int blocks_per_wg;    // ceil(blocks_total / workgroups of this launch) <= kFinChunks
};
// What a kernel needs of PendingArgs before its first load leaves (fetched with the other launch arguments).
struct PendingHead {
    int first_block[kPackMaxBatch];
    int count, blocks_total, blocks_per_wg;
};
struct FinBlock {        // what a reducing wavefront keeps between the two halves
    FinalizeArgs a;      // the problem of its block (wave-uniform)
    int row;             // this lane's row (may lie past the problem's last row)
};

// Requests the partial sums of block `bid` of the concatenated list: S x 64 floats, contiguous, into fin (LDS).
// Returns where this lane finds its scale (some readable address if the problem has none): the caller loads it
// outside of any condition -- a value loaded under a condition would be waited for on the spot, in front of
// this wavefront's own atom requests.
__device__ __forceinline__ const uint16_t *fin_issue(const PendingArgs &pd, const PendingHead &ph, int bid, unsigned char *fin,
                                                     int lane, FinBlock &f) {
    int q = 0;
#pragma unroll
    for (int i = 1; i < kPackMaxBatch; ++i) q += bid >= ph.first_block[i] ? 1 : 0;
    int base = ph.first_block[0];
#pragma unroll
    for (int i = 1; i < kPackMaxBatch; ++i) base = q == i ? ph.first_block[i] : base;
    f.a = pd.a[q];   // (q is wave-uniform: one scalar load of the 32-byte struct)
    pin_scalar(f.a.partial); pin_scalar(f.a.scale); pin_scalar(f.a.y); pin_scalar(f.a.N); pin_scalar(f.a.S);
    const int blk = bid - base;
    f.row = blk * 64 + lane;
    const uint4 *src = reinterpret_cast<const uint4 *>(f.a.partial + (size_t)blk * f.a.S * 64) + lane;
    dma_4k(src, fin);                                    // slices 0 .. 15
    if (f.a.S > 16) dma_4k(src + 256, fin + 4096);       // slices 16 .. 31
    return f.a.scale ? reinterpret_cast<const uint16_t *>(f.a.scale) + min(f.row, f.a.N - 1)
                     : reinterpret_cast<const uint16_t *>(f.a.partial);
}

// y[n] = scale[n] * sum_s partial[s][n], slices ascending: the same additions as the reduction kernel.
__device__ __forceinline__ void fin_complete(const FinBlock &f, uint32_t scale_bits, const float *fin, int lane) {
    const FinalizeArgs &a = f.a;
    float v[kPackMaxSlices];
#pragma unroll
    for (int k = 0; k < kPackMaxSlices; ++k) v[k] = fin[k * 64 + lane];   // (all 32 rows of the LDS block exist)
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < kPackMaxSlices; ++k) sum += k < a.S ? v[k] : 0.f;
    union { uint16_t u; half_t h; } sb;
    sb.u = (uint16_t)scale_bits;
    const float sc = a.scale ? (float)sb.h : 1.f;
    if (f.row < a.N) ((__attribute__((address_space(1))) half_t *)a.y)[f.row] = scaled_output(sum, sc);
}

// All global loads of a workgroup are issued before anything waits: at these sizes a launch is a chain of
// memory latencies (slice -> atoms -> partials) as much as a bandwidth problem.
// PF: steps in the ring (taken two at a time when PAIR); AHEAD of them requested before the barrier.
// wg_linear / n_wg: this workgroup's number among all workgroups of the launch (for its share of the pending rows).
template <int PF, bool PAIR, int AHEAD = kPackAhead>
__device__ __forceinline__ void gemv_packed_body(const PackedArgs &ka, const int bid, const PendingArgs &pd, const int wg_linear) {
    extern __shared__ __align__(16) unsigned char smem[];
    static_assert(AHEAD <= PF, "the ring holds what is requested ahead");
    // all launch arguments in one round of scalar loads
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: group lookups, block numbers and
                                                                         // addresses derived from it stay scalar
    PackedCore a = ka;
    pin_scalar(a.data); pin_scalar(a.cb); pin_scalar(a.x); pin_scalar(a.partial);
    pin_scalar(a.N); pin_scalar(a.J); pin_scalar(a.S); pin_scalar(a.RB); pin_scalar(a.rows_per_block);
    pin_scalar(a.EB); pin_scalar(a.P); pin_scalar(a.Jp); pin_scalar(a.n_groups); pin_scalar(a.nwaves);
    pin_scalar(a.wg_pitch); pin_scalar(a.task_off); pin_scalar(a.steps_off); pin_scalar(a.atom_off);
    PendingHead ph;
#pragma unroll
    for (int i = 0; i < kPackMaxBatch; ++i) {
        ph.first_block[i] = pd.first_block[i];
        pin_scalar(ph.first_block[i]);
    }
    ph.count = pd.count; ph.blocks_total = pd.blocks_total; ph.blocks_per_wg = pd.blocks_per_wg;
    pin_scalar(ph.count); pin_scalar(ph.blocks_total); pin_scalar(ph.blocks_per_wg);
    const int my_group = min(wave, a.n_groups - 1);   // a wavefront without a group repeats the last one's loads
    uint32_t group_word = ka.group[my_group];
    pin_scalar(group_word);
    // the LDS image the atoms index: [slice][parts of x, 16 zero units behind each]; then one float per task
    const uint32_t slice_entries = 1u << a.EB, slice_bytes = slice_entries * 16u;
    const uint32_t part_pitch = ((uint32_t)a.Jp + kZeroUnits) * 16u;   // bytes
    unsigned char *xl = smem + slice_bytes;
    float *accbuf = reinterpret_cast<float *>(xl + (size_t)a.P * part_pitch);
    unsigned char *fin = reinterpret_cast<unsigned char *>(accbuf + (size_t)a.rows_per_block * a.P);   // [kFinChunks][32][64] floats, only with pending rows

    const int tid = threadIdx.x, lane = tid & 63, nwaves = a.nwaves;
    int s, rb;
    slice_and_block(bid, a.S, a.RB, s, rb);
    const int wg = s * a.RB + rb;  // index into the packed tables
    gbyte_t *gdata = (gbyte_t *)a.data;
    gu16_t *tasks = (gu16_t *)(gdata + a.task_off) + (size_t)wg * a.n_groups * 64;
    cu32_t *own_steps = (cu32_t *)(a.data + a.steps_off) + (size_t)wg * a.n_groups;
    gu32_t *own_steps_v = (gu32_t *)(gdata + a.steps_off) + (size_t)wg * a.n_groups;
    // atom block b of this lane: a scalar base (block numbers are wave-uniform) plus a 32-bit lane offset
    gbyte_t *atoms = gdata + a.atom_off + (size_t)wg * a.wg_pitch * kStepBytes;
    const uint32_t lane_off = (uint32_t)lane * 8u;

    // (1) codebook slice and x go straight from global memory into LDS (no registers): wave-wide 1 KiB
    //     transfers, lane l's 16 bytes land at base + 16 l.  Written as asm statements: with the builtin the
    //     compiler knows that LDS is being written behind its back and makes the first LDS read wait for every
    //     outstanding load, the atoms included, which puts the whole memory phase of a launch in front of its
    //     whole gather phase.  The transfers complete in issue order with the other loads, and the counted
    //     wait below is what orders them against the gathers.
    //     The LDS base of a transfer comes from M0, and writing M0 while transfers are in flight stalls the
    //     wavefront (measured: four transfers with four M0 writes take 260 - 300 ns to issue, against 50 ns with
    //     one).  The instruction's immediate offset moves the global address and the LDS address alike, so a
    //     contiguous 4 KiB goes out as one M0 write and four transfers.
    stage_image(a.cb, a.x, s, slice_entries, a.P, a.Jp, a.J, smem, wave, nwaves, lane);
    // (2) this wavefront's first group: where its atoms lie follows from the launch arguments alone, so
    //     the task slots and the atoms are requested right behind the slice.  Loads complete in the order
    //     they were issued, so the wait below counts the loads of this step as still in flight and lets
    //     the gathers start as soon as the slice and x are in, while the atoms stream in behind them.
    //     The empty statement keeps the compiler from moving a load above the staging transfers.
    asm volatile("" ::: "memory");
    auto group_base = [&](uint32_t word) { return atoms + (size_t)(word >> 16) * kStepBytes + lane_off; };
    // Every wavefront issues the same AHEAD + 1 loads, so the count in the wait holds for all of them.
    const bool has_group = wave < a.n_groups;
    // this workgroup's trip count for the group: needed only behind the barrier.  A vector load (of one address),
    // older than the loads the wait counts: a scalar load here would be waited for by the next use of any
    // other scalar load's result, i.e. long before the barrier.
    uint32_t steps_idx = (uint32_t)my_group;
    asm volatile("" : "+v"(steps_idx));
    const uint32_t my_steps_v = own_steps_v[steps_idx];
    uint32_t slot = tasks[(size_t)my_group * 64 + lane];
    uint32_t q[PF][2];  // the ring: the step words of the next PF steps
    gbyte_t *gbase = group_base(group_word);
#pragma unroll
    for (int st = 0; st < AHEAD; ++st) load_step(q[st], gbase, st);
    // (2b) the pending rows of the previous launch: the last wavefronts (the shortest groups) take a block of 64
    //      each.  Requested behind everything this workgroup's barrier depends on, and not waited for there: the
    //      sums are needed at the very end only (the wavefront's own first look at its atoms does wait for them,
    //      which its short group can afford).
    FinBlock fl;
    const int fin_chunk = nwaves - 1 - wave;
    const int fin_bid = wg_linear * ph.blocks_per_wg + fin_chunk;
    const bool fin_mine = ph.count > 0 && fin_chunk < ph.blocks_per_wg && fin_bid < ph.blocks_total;   // wave-uniform
    const uint16_t *scale_at = reinterpret_cast<const uint16_t *>(a.data);   // (any readable address)
    if (fin_mine) scale_at = fin_issue(pd, ph, fin_bid, fin + (size_t)fin_chunk * kFinChunkBytes, lane, fl);
    const uint32_t fin_scale_bits = *(const __attribute__((address_space(1))) uint16_t *)scale_at;   // every wavefront: no condition
    // AHEAD atom loads and the task slots were issued behind the staging transfers, and behind those the scale
    // and (fin_mine) the four or eight transfers of the pending block: when at most that many loads are pending,
    // the staging transfers have landed.  (A test compiles this file and counts those loads in each build.)
    // (lgkmcnt: the stores of the zero units)
    if (!fin_mine)
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(AHEAD + 2) : "memory");
    else if (fl.a.S <= 16)
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(AHEAD + 2 + 4) : "memory");
    else
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(AHEAD + 2 + 8) : "memory");
    // (3) the slice and x of this wavefront have landed (direct-to-LDS transfers count as vector memory
    //     loads); after the barrier those of all wavefronts are visible.  A bare s_barrier: __syncthreads()
    //     would wait for the atoms as well.
    asm volatile("s_barrier" ::: "memory");
#pragma unroll
    for (int st = AHEAD; st < PF; ++st) load_step(q[st], gbase, st);  // the rest of the ring
    const uint32_t my_steps = __builtin_amdgcn_readfirstlane(my_steps_v);

    AtomDecode dec;
    dec.emask4 = (slice_entries - 1u) << 4;
    dec.eb = (uint32_t)a.EB;
    dec.xb = (uint32_t)(kAtomBits - a.EB);
    dec.ebase = 0u;
    // (4) gathers and dot products: lane = task; results go to LDS by slot.  The ring already holds the
    //     group's first PF steps.
    auto run_group = [&](const uint32_t n_steps, const uint32_t slot, gbyte_t *gbase) {
        // position 0 of the lane's part: its part is how many multiples of rows_per_block fit under the slot
        uint32_t part = 0;
        for (int p = 1; p < a.P; ++p) part += (slot != 0xFFFFu && slot >= (uint32_t)(p * a.rows_per_block)) ? 1u : 0u;
        dec.xbase = slice_bytes + part * part_pitch;
        const float sum = unit_sum<PF, PAIR>(q, gbase, n_steps, dec);
        if (slot != 0xFFFFu) accbuf[slot] = sum;
    };
    if (has_group) run_group(my_steps, slot, gbase);
    for (int g = wave + nwaves; g < a.n_groups; g += nwaves) {  // only when a block has more groups than wavefronts
        const uint32_t steps2 = own_steps[g];
        const uint32_t slot2 = tasks[(size_t)g * 64 + lane];
        gbyte_t *gbase2 = group_base(ka.group[g]);
#pragma unroll
        for (int k = 0; k < PF; ++k) load_step(q[k], gbase2, k);
        run_group(steps2, slot2, gbase2);
    }
    __syncthreads();

    // (5) this slice's partial sums, in natural row order (coalesced): the parts of a row added in part order.
    // A second, tiny kernel adds the S partials of every row in slice order -- the "explicit global reduction"
    // of Sec. VI-A.  It is a kernel of its own because device-wide synchronisation inside one kernel costs
    // more here.  Measured with the "last workgroup of a row block reduces" pattern at the 4096 x 4096 shape
    // (one thread per workgroup takes a ticket): a relaxed device-scope ticket returns after 1.8 us (median),
    // an acquire-release one (L2 write-back and invalidate) after 3.8 us, and the last workgroup then needs
    // 4 us to read the 64 KiB of partials through its emptied L2 -- 9.5 us from the first partial store to
    // the end, against ~3.5 us for the second launch.
    for (int r = tid; r < a.rows_per_block; r += nwaves * 64) {
        const int n = rb * a.rows_per_block + r;
        if (n < a.N) {
            float sum = accbuf[r];
            for (int p = 1; p < a.P; ++p) sum += accbuf[p * a.rows_per_block + r];
            ((__attribute__((address_space(1))) float *)a.partial)[partial_index(a.S, s, n)] = sum;
        }
    }
    // (6) the pending rows: their partial sums landed in LDS before the barrier of (3)
    if (fin_mine) fin_complete(fl, fin_scale_bits, reinterpret_cast<const float *>(fin + (size_t)fin_chunk * kFinChunkBytes), lane);
}

// A workgroup of a batched launch that has no part of its own problem (the problem needs fewer workgroups
// than the largest of the batch) still takes its share of the pending rows.
__device__ __forceinline__ void pending_only(const PendingArgs &pd, const int wg_linear, const int nwaves) {
    extern __shared__ __align__(16) unsigned char smem[];
    if (pd.count == 0) return;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int fin_chunk = nwaves - 1 - wave;
    const int fin_bid = wg_linear * pd.blocks_per_wg + fin_chunk;
    if (fin_chunk >= pd.blocks_per_wg || fin_bid >= pd.blocks_total) return;
    PendingHead ph;
#pragma unroll
    for (int i = 0; i < kPackMaxBatch; ++i) ph.first_block[i] = pd.first_block[i];
    ph.count = pd.count; ph.blocks_total = pd.blocks_total; ph.blocks_per_wg = pd.blocks_per_wg;
    unsigned char *fin = smem + (size_t)fin_chunk * kFinChunkBytes;
    FinBlock fl;
    const uint16_t *scale_at = fin_issue(pd, ph, fin_bid, fin, lane, fl);
    const uint32_t scale_bits = *(const __attribute__((address_space(1))) uint16_t *)scale_at;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // (the transfers of this wavefront; nobody else reads them)
    fin_complete(fl, scale_bits, reinterpret_cast<const float *>(fin), lane);
}

// One problem: 8 to 16 wavefronts, one per group of the block (more groups than that: several each).
__global__ __launch_bounds__(1024) void gemv_packed_kernel(PackedArgs a, PendingArgs pd) {
    gemv_packed_body<6, true>(a, blockIdx.x, pd, blockIdx.x);
}

// Several independent problems in one launch (blockIdx.y picks the problem): the fixed latencies of a
// launch (ramp-up, first touches of tables and atoms, drain) are paid once for all of them, and
// workgroups of different problems share a CU.
struct PackedBatch {
    PackedArgs a[kPackMaxBatch];
};
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(6))) void gemv_packed_batch_kernel(PackedBatch b, PendingArgs pd) {
    const PackedArgs &a = b.a[blockIdx.y];
    const int wg_linear = blockIdx.y * gridDim.x + blockIdx.x;
    if ((int)blockIdx.x >= a.S * a.RB) {
        pending_only(pd, wg_linear, a.nwaves);
        return;
    }
    gemv_packed_body<4, false>(a, blockIdx.x, pd, wg_linear);
}

// y[n] = scale[n] * sum_s partial[s][n], slices in ascending order.  MAXS loads are issued unconditionally
// (slices past S re-read the last one) so that none of them waits behind a branch.  One row per thread, one
// wavefront per block: the kernel is one memory round trip long, and the fewer requests queue on a CU the
// shorter it is.
constexpr int kFinalizeRows = 64;
template <int MAXS>
__device__ __forceinline__ void gemv_packed_finalize_body(const float *__restrict__ partial,
                                                          const half_t *__restrict__ scale, half_t *__restrict__ y,
                                                          int N, int S) {
    const int n = blockIdx.x * kFinalizeRows + threadIdx.x;  // (the launch shape is fixed: no load of the hidden arguments)
    if (n >= N) return;
    // (pointers that went through pin_scalar have to be told again that they are global)
    const __attribute__((address_space(1))) float *gp = (const __attribute__((address_space(1))) float *)partial;
    const __attribute__((address_space(1))) half_t *gs = (const __attribute__((address_space(1))) half_t *)scale;
    __attribute__((address_space(1))) half_t *gy = (__attribute__((address_space(1))) half_t *)y;
    float v[MAXS];
#pragma unroll
    for (int k = 0; k < MAXS; ++k) v[k] = gp[partial_index(S, k < S ? k : S - 1, n)];
    const float sc = scale ? (float)gs[n] : 1.f;
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < MAXS; ++k) sum += k < S ? v[k] : 0.f;
    gy[n] = scaled_output(sum, sc);
}
__global__ __launch_bounds__(kFinalizeRows) void gemv_packed_finalize_kernel(const float *__restrict__ partial,
                                                                  const half_t *__restrict__ scale,
                                                                  half_t *__restrict__ y, int N, int S) {
    pin_scalar(partial); pin_scalar(scale); pin_scalar(y); pin_scalar(N); pin_scalar(S);  // one round of argument loads
    gemv_packed_finalize_body<kPackMaxSlices>(partial, scale, y, N, S);
}
struct FinalizeBatch {
    FinalizeArgs a[kPackMaxBatch];
};
__global__ __launch_bounds__(kFinalizeRows) void gemv_packed_finalize_batch_kernel(FinalizeBatch b) {
    FinalizeArgs a = b.a[blockIdx.y];
    pin_scalar(a.partial); pin_scalar(a.scale); pin_scalar(a.y); pin_scalar(a.N); pin_scalar(a.S);
    gemv_packed_finalize_body<kPackMaxSlices>(a.partial, a.scale, a.y, a.N, a.S);
}

// ------------------------------------------------------------------------ pipelined kernel
// Many products in ONE launch of 256 persistent workgroups (one per compute unit).  A launch of the kernel above
// runs its phases in lockstep on all units -- staging (latency bound, LDS and arithmetic idle), gathers (LDS
// bound, memory idle for want of requests), stores -- and at Llama sizes each phase is 1 - 4 us long.  Here a
// workgroup holds TWO LDS images: while its consumer wavefronts gather problem k from one, its producer
// wavefronts stage problem k + 1 into the other, and the atom requests of the consumers run one group ahead,
// across problem boundaries.  Workgroup b of the launch takes block b of EVERY problem.
//
// Synchronisation inside the workgroup is by four LDS counters instead of barriers (a barrier would make
// every wavefront wait for the slowest of each problem):
//   staged[k & 1]: +1 by each producer when its share of problem k has landed   (k staged: >= NP (k/2 + 1))
//   done  [k & 1]: +1 by each consumer when it has left problem k               (k done:   >= NC (k/2 + 1))
// A consumer enters problem k after seeing it staged; a producer stages k after seeing k - 2 done.  No wavefront
// can be two problems ahead of another, so the counters of one parity are never ambiguous.  A consumer leaves the
// sum of a task in an LDS buffer of the image (by row); the producers write the buffer of problem k - 1 out in
// row order, whole lines at a time, before they stage problem k + 1.  (Stores straight from the consumers'
// registers -- 64 scattered 4-byte writes per group -- cost a quarter of the kernel's time: measured 0.74 ms with
// them against 0.56 ms without, gathers switched off in both.)  Every wait is bounded: after
// kPipeSpinLimit looks a wavefront gives up waiting for the rest of the launch and raises the status word,
// so the grid always drains.
// The S partial sums per row of all problems are added by one reduction launch behind it.
constexpr int kPipeWgs = 256;
constexpr int kPipeConsumers = 14, kPipeProducers = 2;   // wavefronts 0 .. 13 and 14, 15
constexpr int kPipeFirstProducer = kPipeConsumers;
constexpr int kPipeOps = 12;                            // staging operations per producer and problem
constexpr uint32_t kPipeImage = 65536;                  // LDS bytes from one image to the other
constexpr uint32_t kPipeFlags = kPipeImage - 64;        // in the tail of image 0: staged[2], done[2], next group to hand
                                                        // out, finished groups per image and row block [2][4]
constexpr uint32_t kPipeGroupsDone = kPipeFlags + 20u;
constexpr uint32_t kPipeAcc = 2 * kPipeImage;           // two buffers (one per image) of one float per task ...
constexpr uint32_t kPipeAccBytes = 16384;               // ... for problems with up to 4096 tasks per image; larger ones
                                                        // keep theirs in the tail of their image
constexpr uint32_t kPipeLds = kPipeAcc + 2 * kPipeAccBytes;   // 160 KiB: all of a compute unit's LDS
constexpr uint32_t kPipeSpinLimit = 1u << 20;

// One problem as the kernel reads it (a table in device memory, written once when the pipeline is created).
struct PipeProblem {
    const unsigned char *atoms, *tasks, *steps;   // the three regions of the packed buffer
    const half_t *cb, *x;
    float *partial;
    const half_t *scale;
    half_t *y;
    int N, J, S, RB, rows_per_block, EB, P, Jp, n_groups;
    uint32_t wg_pitch;
    uint32_t reserved[2];
    uint32_t bpi;          // row blocks per LDS image: a workgroup of the launch takes bpi consecutive row blocks of its slice
    uint32_t rbv;          // RB / bpi
    uint32_t acc_lds;      // LDS byte address of the problem's buffer of task sums: [row block of the image][part][row]
    uint32_t groups_through;   // groups per row block of this and all earlier problems of the lane with the same parity
    // How producer w builds the LDS image, worked out on the host (the kernel's instruction issue is a scarce
    // resource: four wavefronts per SIMD): pairs (source byte offset, PipeOp word), the list ends at a zero word.
    uint32_t ops[kPipeProducers][kPipeOps][2];
    uint32_t group[VQ_PACK_MAX_GROUPS];   // prefix << 16 | common steps
};
static_assert(sizeof(PipeProblem) % 64 == 0 && offsetof(PipeProblem, ops) == 128, "the scout touches the descriptor by 64-byte lines");
// PipeOp word: bits 0..16 LDS byte offset in the image, 17..18 kind, 19..25 lanes (kind 2), 31 valid.
enum : uint32_t {
    kOpSlice4k = 0,   // 4 KiB of the codebook slice (source offset from the slice)
    kOpX4k = 1,       // 4 KiB of x
    kOpX1k = 2,       // up to 1 KiB of x: `lanes` units of 16 bytes
    kOpZero = 3,      // 256 zero bytes (the units behind a part of x that padding atoms point at)
};
__host__ __device__ constexpr uint32_t pipe_op(uint32_t lds_off, uint32_t kind, uint32_t lanes) {
    return lds_off | (kind << 17) | (lanes << 19) | (1u << 31);
}
typedef const __attribute__((address_space(4))) PipeProblem cproblem_t;   // read with scalar loads
typedef __attribute__((address_space(3))) uint32_t lds_u32_t;

struct PipeSync {
    bool broken;          // a wait ran out: no more waiting in this wavefront (it raises the status word when it ends)
};
// Waits until the LDS counter at `addr` has reached `target`.
__device__ __forceinline__ void pipe_wait(uint32_t addr, uint32_t target, PipeSync &sy) {
    if (!sy.broken) {
        uint32_t spin = 0;
        for (;;) {
            const uint32_t v = __builtin_amdgcn_readfirstlane(
                __hip_atomic_load((lds_u32_t *)(uintptr_t)addr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
            if (v >= target) break;
            if (++spin == kPipeSpinLimit) {
                sy.broken = true;   // (no store here: a memory operation inside this loop would keep the compiler
                break;              // from counting the requests in flight around it)
            }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    asm volatile("" ::: "memory");   // what follows reads what the counter announces
}
// +1 on an LDS counter, after everything this wavefront wrote to LDS before.
__device__ __forceinline__ void pipe_signal(uint32_t addr, int lane) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (lane == 0) __hip_atomic_fetch_add((lds_u32_t *)(uintptr_t)addr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// A consumer's unit of work: up to PF consecutive steps of one group of problem i (of this workgroup's blocks),
// all of them requested at once.  A group of more steps is taken in several pieces, one after the other by the
// same wavefront, the sums carried in registers.
template <int PF>
struct PipePiece {
    uint32_t i;          // problem (n: no more work)
    uint32_t meta;       // first step of the piece in its group | row block of the image << 8 | steps of the piece << 12 |
                         // last piece << 16 | valid << 17
    uint32_t slot;
    uint32_t q[PF][2];
};
// The groups of a lane's problems are numbered through ("items").  Consumers take them from an LDS counter as they
// go (each wavefront when it has requests to issue, i.e. two pieces before it works on them): whoever gets
// long groups takes fewer of them.  What a wavefront takes is ascending, so it still passes the problems in order.
struct PipeCursor {
    uint32_t t, h;       // the group being requested (number in the lane's list) and its next piece
    // the group being requested, worked out before the piece before it is worked on
    uint32_t word;       // its entry of the problem's group table (prefix << 16 | common steps)
    uint32_t own;        // steps that this workgroup's tasks of the group really have (<= common steps)
    uint32_t wg, g, jb;  // block in the packed tables, group in the block, row block of the image
    bool none;           // past the last group
    bool advance;        // the piece last requested ended its group
    // two groups taken ahead, so that nothing here waits: the group after the current one with its entry of the
    // table of groups already requested (a scalar load that lands while a piece is worked on), and the one after
    // that still on its way back from the LDS counter (in a vector register until needed)
    uint32_t where_a;
    uint32_t t_b, where_b;
    uint32_t t_c_v;
};
// (take = 0 reads the counter without taking anything: the callers have no branch around this)
__device__ __forceinline__ uint32_t pipe_grab(int lane, uint32_t take) {
    uint32_t v = 0;
    if (lane == 0)
        v = __hip_atomic_fetch_add((lds_u32_t *)(uintptr_t)(kPipeFlags + 16u), take, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return v;
}
// What requesting needs of a problem: read once per problem and wavefront, kept in scalar registers.
struct PipeHead {
    uint32_t i;
    int S, RB, ng, bpi;
    uint32_t wg_pitch;
    const unsigned char *atoms, *tasks, *steps;
    int s, rbv;          // this workgroup's slice and first row block / bpi
    bool in;             // the workgroup has blocks of this problem
};
__device__ __forceinline__ void pipe_head_load(PipeHead &h, cproblem_t *table, uint32_t i, int bid) {
    cproblem_t &pr = table[i];
    h.i = i;
    h.S = pr.S; h.RB = pr.RB; h.ng = pr.n_groups; h.bpi = (int)pr.bpi;
    h.wg_pitch = pr.wg_pitch;
    h.atoms = pr.atoms; h.tasks = pr.tasks; h.steps = pr.steps;
    const int RBv = (int)pr.rbv;
    h.in = bid < h.S * RBv;
    slice_and_block(h.in ? bid : 0, h.S, RBv, h.s, h.rbv);
}

// Moves the cursor behind the piece last requested: to the next piece of the group, or to the next group of this
// wavefront, taken from the counter.  Straight-line code for both cases.  Where group t lies comes from a table
// the host wrote (problem | row block of the image << 16 | group << 20).  Called BEFORE the wavefront works on an
// earlier piece: the scalar loads here (the last one is left in flight) land while it does, instead of standing
// in front of the next requests.  Not called between the requests and the end of the main loop: anything but
// the requests themselves there makes the compiler lose count of the requests in flight at the loop's head (it
// then waits for nearly all of them).
__device__ __forceinline__ void pipe_next(PipeCursor &cu, PipeHead &hd, cproblem_t *table, cu32_t *items, uint32_t total_items, int bid,
                                          int lane) {
    const bool advance = cu.advance;
    // current <- next (its table entry was requested one call ago), next <- the one after (taken from the counter
    // one call ago; its table entry is requested now), and one more is taken from the counter
    const uint32_t where = advance ? cu.where_b : cu.where_a;
    cu.where_a = where;
    cu.t = advance ? cu.t_b : cu.t;
    cu.h = advance ? 0u : cu.h + 1u;
    const uint32_t t_c = __builtin_amdgcn_readfirstlane(cu.t_c_v);
    cu.t_b = advance ? t_c : cu.t_b;
    const uint32_t fresh = pipe_grab(lane, advance ? 1u : 0u);
    cu.t_c_v = advance ? fresh : cu.t_c_v;
    cu.where_b = items[cu.t_b < total_items ? cu.t_b : total_items - 1];   // (past the end: the last group once more, never used)
    cu.none = cu.t >= total_items;
    const uint32_t i = where & 0xFFFFu;
    if (i != hd.i) pipe_head_load(hd, table, i, bid);
    cu.jb = (where >> 16) & 15u;
    cu.g = where >> 20;
    cu.wg = (uint32_t)(hd.s * hd.RB + hd.rbv * hd.bpi) + cu.jb;
    cu.word = table[i].group[cu.g];
    cu.own = ((cu32_t *)hd.steps)[cu.wg * (uint32_t)hd.ng + cu.g];
}

template <int PF>
__device__ __forceinline__ void pipe_fetch(PipePiece<PF> &it, PipeCursor &cu, PipeHead &hd, cproblem_t *table, cu32_t *items,
                                           uint32_t n, uint32_t total_items, int bid, int lane, uint32_t zero_v) {
    const uint32_t first = cu.h * PF;
    const uint32_t left = cu.own > first ? cu.own - first : 0u;          // steps of the group from this piece on
    const uint32_t n_piece = left < (uint32_t)PF ? left : (uint32_t)PF;
    gbyte_t *gbase = (gbyte_t *)hd.atoms + ((size_t)cu.wg * hd.wg_pitch + (cu.word >> 16) + first) * kStepBytes;
    it.slot = ((gu16_t *)hd.tasks)[(size_t)(cu.wg * (uint32_t)hd.ng + cu.g) * 64 + lane];
    // PF requests whatever the piece's length (no branch: the compiler must be able to count them), but those past
    // the piece's last step name that step again: the blocks behind a short group's own steps are padding that
    // nobody needs, or the next group's head, and neither should cross the memory system for this wavefront.
    // (ordinary loads: with a non-temporal hint such repeats come from memory again; measured 7 % slower)
    const uint32_t top = n_piece > 0u ? n_piece - 1u : 0u;
    const uint32_t lane8 = (uint32_t)lane * 8u + zero_v;
#pragma unroll
    for (int st = 0; st < PF; ++st) {
        const uint32_t idx = (uint32_t)st < top ? (uint32_t)st : top;
        gu32_t *p = (gu32_t *)(gbase + (size_t)idx * kStepBytes + lane8);
        it.q[st][0] = p[0]; it.q[st][1] = p[1];
    }
    const uint32_t last = left <= (uint32_t)PF ? 1u : 0u;
    it.i = cu.none ? n : hd.i;
    it.meta = first | (cu.jb << 8) | (n_piece << 12) | (last << 16) | ((hd.in && !cu.none) ? 1u << 17 : 0u);
    cu.advance = last != 0u;
}

// What working on a piece needs of its problem: read when a wavefront enters the problem.
struct PipeBody {
    uint32_t i;
    uint32_t EB, P, Jp, rows_per_block;
    uint32_t acc_lds;     // where the sums of the image's tasks go
};
__device__ __forceinline__ void pipe_body_load(PipeBody &b, cproblem_t *table, uint32_t i) {
    cproblem_t &pr = table[i];
    b.i = i;
    b.EB = (uint32_t)pr.EB; b.P = (uint32_t)pr.P; b.Jp = (uint32_t)pr.Jp; b.rows_per_block = (uint32_t)pr.rows_per_block;
    b.acc_lds = pr.acc_lds;
}

// Where a consumer stands: in problem `cur` (seen staged), all earlier ones left.
struct PipeConsumer {
    uint32_t cur, n;
    PipeSync sy;
};
__device__ __forceinline__ void pipe_enter(PipeConsumer &c, uint32_t k) {
    pipe_wait(kPipeFlags + (k & 1u) * 4u, (uint32_t)kPipeProducers * (k / 2u + 1u), c.sy);
}
// Leaves problems until it stands in problem `to` (n: until the end).
__device__ __forceinline__ void pipe_advance(PipeConsumer &c, uint32_t to, int lane) {
    while (c.cur < to) {
        pipe_signal(kPipeFlags + 8u + (c.cur & 1u) * 4u, lane);
        ++c.cur;
        if (c.cur < c.n) pipe_enter(c, c.cur);
    }
}

template <int PF>
__device__ __forceinline__ void pipe_consume(PipePiece<PF> &it, Acc3 &acc, PipeConsumer &c, PipeBody &bd, cproblem_t *table, int bid,
                                             int lane) {
    static_assert(PF % 2 == 0 && PF <= kPackTailBlocks, "steps in pairs; requests run up to PF - 1 blocks past the end of a group");
    pipe_advance(c, it.i, lane);
    if (it.i >= c.n) return;
    if (bd.i != it.i) pipe_body_load(bd, table, it.i);
    const bool valid = (it.meta >> 17) & 1u;
    const uint32_t first = it.meta & 0xFFu, jb = (it.meta >> 8) & 0xFu;
    const uint32_t n_steps = valid ? (it.meta >> 12) & 15u : 0u;   // of this piece
    const uint32_t slot = valid ? it.slot : 0xFFFFu;
    const uint32_t img = (it.i & 1u) * kPipeImage;
    const uint32_t slice_bytes = 16u << bd.EB, part_pitch = (bd.Jp + kZeroUnits) * 16u;
    uint32_t part = 0;
    for (uint32_t p = 1; p < bd.P; ++p) part += (slot != 0xFFFFu && slot >= p * bd.rows_per_block) ? 1u : 0u;
    AtomDecode dec;
    dec.emask4 = ((1u << bd.EB) - 1u) << 4;
    dec.eb = bd.EB;
    dec.xb = (uint32_t)kAtomBits - bd.EB;
    dec.ebase = img;
    dec.xbase = img + slice_bytes + part * part_pitch;
    if (first == 0) acc = {{0.f, 0.f, 0.f}};
#pragma unroll
    for (int k = 0; k < PF; k += 2) {
        const uint32_t lo[2] = {it.q[k][0], it.q[k + 1][0]}, hi[2] = {it.q[k][1], it.q[k + 1][1]};
        if ((uint32_t)k + 1 < n_steps) {
            steps_dot<2>(lo, hi, dec, acc);
        } else if ((uint32_t)k < n_steps) {
            const uint32_t lo1[1] = {lo[0]}, hi1[1] = {hi[0]};
            steps_dot<1>(lo1, hi1, dec, acc);
        }
    }
    if ((it.meta >> 16) & 1u) {
        if (slot != 0xFFFFu)   // (slot = part * rows_per_block + row inside the block)
            *(__attribute__((address_space(3))) float *)(uintptr_t)(bd.acc_lds + (jb * bd.rows_per_block * bd.P + slot) * 4u) =
                (acc.a[0] + acc.a[1]) + acc.a[2];
        // one more group of this row block is finished: when all are, the producers write the block's rows out
        // (counted also where the workgroup has no block of the problem: the counters run on over all problems)
        pipe_signal(kPipeGroupsDone + ((it.i & 1u) * 4u + jb) * 4u, lane);
    }
}
// Declares every requested step of a piece used.  The steps past the end of a short group are never looked at, and
// the compiler would hand their registers out again while the requests are still in flight -- which costs a wait
// for (nearly) everything in flight, the other piece's requests included.  After this, what is in flight is the
// other piece's requests and nothing else.
template <int PF>
__device__ __forceinline__ void pipe_retire(const PipePiece<PF> &it) {
#pragma unroll
    for (int k = 0; k < PF; ++k) asm volatile("" ::"v"(it.q[k][0]), "v"(it.q[k][1]));
    asm volatile("" ::"v"(it.slot));
}

// Producer w's share of the image of problem k, from the list the host prepared: read (all of it, into scalar
// registers) before the producer starts waiting for its turn, carried out after.
struct PipeStage {
    const uint4 *slice, *x;
    uint32_t op[kPipeOps][2];
};
__device__ __forceinline__ PipeStage pipe_stage_read(cproblem_t *table, uint32_t k, int bid, int pw) {
    cproblem_t &pr = table[k];
    PipeStage st;
    const int S = pr.S, RB = (int)pr.rbv;
    const bool mine = bid < S * RB;
    int s, rb;
    slice_and_block(mine ? bid : 0, S, RB, s, rb);
    st.slice = reinterpret_cast<const uint4 *>(pr.cb) + ((size_t)s << pr.EB);
    st.x = reinterpret_cast<const uint4 *>(pr.x);
    pin_scalar(st.slice); pin_scalar(st.x);
#pragma unroll
    for (int j = 0; j < kPipeOps; ++j) {
        st.op[j][0] = pr.ops[pw][j][0];
        st.op[j][1] = mine ? pr.ops[pw][j][1] : 0u;
        pin_scalar(st.op[j][0]); pin_scalar(st.op[j][1]);
    }
    return st;
}
__device__ __forceinline__ void pipe_stage(const PipeStage &st, int lane, unsigned char *img) {
#pragma unroll
    for (int j = 0; j < kPipeOps; ++j) {
        const uint32_t src = st.op[j][0], w = st.op[j][1];
        if (w == 0u) break;
        unsigned char *dst = img + (w & 0x1FFFFu);
        const uint32_t kind = (w >> 17) & 3u;
        if (kind == kOpSlice4k) {
            dma_4k(st.slice + (src >> 4) + lane, dst);
        } else if (kind == kOpX4k) {
            dma_4k(st.x + (src >> 4) + lane, dst);
        } else if (kind == kOpX1k) {
            if ((uint32_t)lane < ((w >> 19) & 127u)) dma_1k(st.x + (src >> 4) + lane, dst);
        } else {
            reinterpret_cast<uint32_t *>(dst)[lane] = 0u;
        }
    }
}

// The partial sums of problem k of this workgroup, LDS -> global: rows in natural order (whole 256-byte runs per
// store instruction), the parts of a row added in part order -- the additions of the one-problem kernel.  Row
// block by row block, each as soon as the consumers have finished its groups (so that only the last one's rows
// stand between "problem done" and the staging of the next image); the rows are dealt to the producers 64 at a time.
__device__ __forceinline__ void pipe_emit(cproblem_t *table, uint32_t k, int bid, int pw, int lane, PipeSync &sy) {
    cproblem_t &pr = table[k];
    const int S = pr.S, RBv = (int)pr.rbv, bpi = (int)pr.bpi, rpb = pr.rows_per_block, P = pr.P, N = pr.N;
    const uint32_t through = pr.groups_through;
    if (bid >= S * RBv) return;
    int s, rbv;
    slice_and_block(bid, S, RBv, s, rbv);
    __attribute__((address_space(1))) float *out = (__attribute__((address_space(1))) float *)pr.partial;
    const uint32_t acc_lds = pr.acc_lds;
    for (int jb = 0; jb < bpi; ++jb) {
        pipe_wait(kPipeGroupsDone + ((k & 1u) * 4u + (uint32_t)jb) * 4u, through, sy);
        const uint32_t base = acc_lds + (uint32_t)(jb * rpb * P) * 4u;
        const int row0 = (rbv * bpi + jb) * rpb;
#pragma unroll 4
        for (int r = pw * 64 + lane; r < rpb; r += kPipeProducers * 64) {
            const int row = row0 + r;
            float sum = *(const __attribute__((address_space(3))) float *)(uintptr_t)(base + (uint32_t)r * 4u);
            for (int p = 1; p < P; ++p)
                sum += *(const __attribute__((address_space(3))) float *)(uintptr_t)(base + (uint32_t)(p * rpb + r) * 4u);
            if (row < N) out[partial_index(S, s, row)] = sum;
        }
    }
}

// Scouting: between two images a producer reads the descriptor of a coming problem through the scalar cache and
// touches its share of the lines of that problem's codebook slice and x, so that the producers' and consumers'
// scalar loads hit the scalar cache and the staging transfers hit this die's L2.  A first touch of anything costs
// a trip to memory, 1.5 - 2 us under this load: as long as a short problem's gathers.  Returns a value that
// depends on the touches: the caller declares it used after its next full wait (so the touches cost no wait of
// their own).
struct PipeWarm {
    uint32_t w[4];
};
__device__ __forceinline__ PipeWarm pipe_scout(cproblem_t *table, uint32_t k, int bid, int pw, int lane) {
    cu32_t *words = (cu32_t *)&table[k];
    uint32_t acc = 0;
#pragma unroll
    for (int l = 0; l < (int)(sizeof(PipeProblem) / 64); ++l) acc |= words[l * 16];   // (one word per 64-byte line)
    asm volatile("" ::"s"(acc));
    cproblem_t &pr = table[k];
    const int S = pr.S, RB = (int)pr.rbv;
    int s, rb;
    slice_and_block(bid < S * RB ? bid : 0, S, RB, s, rb);
    const uint32_t slice_bytes = 16u << pr.EB, x_bytes = (uint32_t)pr.J * 16u;
    const gbyte_t *slice = (gbyte_t *)pr.cb + (size_t)s * slice_bytes;
    const gbyte_t *x = (gbyte_t *)pr.x;
    // two lines of the slice and two of x per lane (a 32 KiB slice and up to 32 KiB of x with two producers); no
    // conditions and no dependent arithmetic: a lane past the end touches the last line again
    const uint32_t first = (uint32_t)(pw * 64 + lane) * 128u, stride = (uint32_t)kPipeProducers * 64u * 128u;
    PipeWarm r;
    r.w[0] = *(const volatile gu32_t *)(slice + min(first, slice_bytes - 128u));
    r.w[1] = *(const volatile gu32_t *)(slice + min(first + stride, slice_bytes - 128u));
    r.w[2] = *(const volatile gu32_t *)(x + min(first, x_bytes - 16u));
    r.w[3] = *(const volatile gu32_t *)(x + min(first + stride, x_bytes - 16u));
    return r;
}
__device__ __forceinline__ void pipe_warm_done(const PipeWarm &r) {
    asm volatile("" ::"v"(r.w[0]), "v"(r.w[1]), "v"(r.w[2]), "v"(r.w[3]));
}

// The 256 workgroups form 1, 2, 4 or 8 independent lanes, each with a problem list of its own (problem k of the
// pipeline goes to lane k % lanes): a problem whose blocks are taken bpi at a time needs only S RB / bpi
// workgroups, and a workgroup that stages one image for bpi blocks has bpi times the work between two image
// changes -- more groups to spread over its consumers, and more time to stage the next image in.
struct PipeLanes {
    uint32_t first[8], n[8];             // per lane: where its problems start in the table, how many
    uint32_t item_first[8], items[8];    // where its groups start in the table of groups, how many
    uint32_t log2_lanes;
};
__global__ __launch_bounds__(1024) void gemv_pipeline_kernel(const PipeProblem *table_, const uint32_t *items_, PipeLanes lanes,
                                                               uint32_t *status) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    // workgroup number = [index in the lane : lane : die] (the low three bits are the die the workgroup lands on;
    // they stay the low bits of its number within the lane, so that a codebook slice is still staged by one die)
    const uint32_t my_lane = (blockIdx.x >> 3) & ((1u << lanes.log2_lanes) - 1u);
    const int bid = (int)((blockIdx.x & 7u) | ((blockIdx.x >> (3u + lanes.log2_lanes)) << 3));
    uint32_t n = lanes.n[my_lane], total_items = lanes.items[my_lane];
    table_ += lanes.first[my_lane];
    items_ += lanes.item_first[my_lane];
    pin_scalar(table_); pin_scalar(items_); pin_scalar(n); pin_scalar(total_items); pin_scalar(status);
    if (n == 0u) return;
    cproblem_t *table = (cproblem_t *)table_;
    cu32_t *items = (cu32_t *)items_;
    if (threadIdx.x < 13) reinterpret_cast<uint32_t *>(smem + kPipeFlags)[threadIdx.x] = threadIdx.x == 4 ? 2u * (uint32_t)kPipeConsumers : 0u;
    __syncthreads();
    PipeSync sy = {false};
    if (wave >= kPipeFirstProducer) {
        // ---- producer (and scout, two problems ahead, in the slack between two images)
        const int pw = wave - kPipeFirstProducer;
        PipeWarm warm = pipe_scout(table, n > 2u ? 2u : 0u, bid, pw, lane);
        for (uint32_t k = 0; k < n; ++k) {
            const PipeStage st = pipe_stage_read(table, k, bid, pw);
            if (k >= 2) pipe_wait(kPipeFlags + 8u + (k & 1u) * 4u, (uint32_t)kPipeConsumers * ((k - 2u) / 2u + 1u), sy);
            pipe_stage(st, lane, smem + (k & 1u) * kPipeImage);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the transfers of this wavefront (and the touches before them)
            pipe_warm_done(warm);
            pipe_signal(kPipeFlags + (k & 1u) * 4u, lane);
            warm = pipe_scout(table, k + 3u < n ? k + 3u : n - 1u, bid, pw, lane);
            // the sums of the problem before: its buffer is the one that problem k + 1's tasks will write
            if (k >= 1) pipe_emit(table, k - 1u, bid, pw, lane, sy);
        }
        pipe_warm_done(warm);
        pipe_emit(table, n - 1u, bid, pw, lane, sy);
        if (sy.broken && lane == 0) *status = 1u;
        return;
    }
    // ---- consumer: groups wave, wave + NC, ... of the list of all groups; the requests of one piece are in
    //      flight while the piece before it is worked on
    constexpr int PF = 8;
    PipeConsumer c = {0u, n, sy};
    pipe_enter(c, 0u);
    // three pieces in rotation: while one is worked on, the requests of the next two are in flight (a piece is
    // 4 - 8 steps, about a microsecond of this wavefront's time; a request that misses the caches takes two)
    PipePiece<PF> a, b, d;
    // the first three groups of wavefront w are w, w + NC and w + 2 NC (the counter starts behind these)
    PipeCursor cu;
    cu.t = 0u; cu.h = 0u; cu.advance = true; cu.where_a = 0u;
    cu.t_b = (uint32_t)wave;
    cu.where_b = items[cu.t_b < total_items ? cu.t_b : total_items - 1];
    cu.t_c_v = (uint32_t)(wave + kPipeConsumers);
    PipeHead hd;
    pipe_head_load(hd, table, 0u, bid);
    PipeBody bd;
    pipe_body_load(bd, table, 0u);
    Acc3 acc = {{0.f, 0.f, 0.f}};
    uint32_t zero_v = 0u;
    asm volatile("" : "+v"(zero_v));
    pipe_next(cu, hd, table, items, total_items, bid, lane);
    pipe_fetch(a, cu, hd, table, items, n, total_items, bid, lane, zero_v);
    pipe_next(cu, hd, table, items, total_items, bid, lane);
    pipe_fetch(b, cu, hd, table, items, n, total_items, bid, lane, zero_v);
    pipe_next(cu, hd, table, items, total_items, bid, lane);
    pipe_fetch(d, cu, hd, table, items, n, total_items, bid, lane, zero_v);
    for (;;) {
        pipe_next(cu, hd, table, items, total_items, bid, lane);
        pipe_consume(a, acc, c, bd, table, bid, lane);
        pipe_retire(a);
        if (b.i >= n) break;
        pipe_fetch(a, cu, hd, table, items, n, total_items, bid, lane, zero_v);
        pipe_next(cu, hd, table, items, total_items, bid, lane);
        pipe_consume(b, acc, c, bd, table, bid, lane);
        pipe_retire(b);
        if (d.i >= n) break;
        pipe_fetch(b, cu, hd, table, items, n, total_items, bid, lane, zero_v);
        pipe_next(cu, hd, table, items, total_items, bid, lane);
        pipe_consume(d, acc, c, bd, table, bid, lane);
        pipe_retire(d);
        if (a.i >= n) break;
        pipe_fetch(d, cu, hd, table, items, n, total_items, bid, lane, zero_v);
    }
    pipe_advance(c, n, lane);
    if (c.sy.broken && lane == 0) *status = 1u;
}

// y of every problem of a pipeline: blockIdx.y picks the problem.
__global__ __launch_bounds__(kFinalizeRows) void gemv_pipeline_finalize_kernel(const PipeProblem *table_) {
    cproblem_t &pr = ((cproblem_t *)table_)[blockIdx.y];
    const float *partial = pr.partial;
    const half_t *scale = pr.scale;
    half_t *y = pr.y;
    int N = pr.N, S = pr.S;
    pin_scalar(partial); pin_scalar(scale); pin_scalar(y); pin_scalar(N); pin_scalar(S);
    gemv_packed_finalize_body<kPackMaxSlices>(partial, scale, y, N, S);
}

bool gemv_uses_pack(const vq_weight_t *w, int bs) {
    return w->gemv_pack != nullptr && bs == 1 && pack_supported(w);
}

// S partial sums per row in blocks of 64 rows (partial_index), plus the 4 KiB that a block fetch may read past
// the last block.
size_t gemv_packed_workspace(const vq_weight_t *w) {
    return (size_t)w->gemv_pack->S * (((size_t)w->N + 63) / 64) * 64 * sizeof(float) + 4096;
}

int check_pack(const vq_weight_t *w) {
    const vq_gemv_pack_t *p = w->gemv_pack;
    if (!p->data) return VQ_ERR_NULL;
    if (!aligned16(p->data)) return VQ_ERR_ALIGN;
    PackPlan plan;
    if (!pack_plan(w, &plan)) return VQ_ERR_UNSUPPORTED;
    if (p->S != plan.S || p->RB != plan.RB || p->rows_per_block != plan.rows_per_block || p->entry_bits != plan.EB ||
        p->parts != plan.P || p->part_cols != plan.Jp)
        return VQ_ERR_SHAPE;
    if (p->S > (uint32_t)kPackMaxSlices) return VQ_ERR_UNSUPPORTED;
    // every address the kernel derives from the descriptor must lie inside the buffer
    const uint64_t ng = plan.G, nwg = (uint64_t)p->S * p->RB;
    uint64_t sum = 0;
    for (uint64_t g = 0; g < ng; ++g) sum += p->group_steps[g];
    if (sum != p->wg_pitch || sum > 65535 || sum == 0) return VQ_ERR_SHAPE;
    if (p->task_off + nwg * ng * 128 > p->steps_off || p->steps_off + nwg * ng * 4 > p->atom_off ||
        p->atom_off + (nwg * sum + kPackTailBlocks) * kStepBytes > p->bytes)
        return VQ_ERR_SHAPE;
    if ((p->task_off & 1) || (p->steps_off & 3) || (p->atom_off & 7)) return VQ_ERR_ALIGN;
    return VQ_OK;
}

namespace {

struct PackedLaunch {
    PackedArgs a;
    int grid, waves;
    size_t lds;
};

PackedLaunch packed_launch(const vq_weight_t *w, const void *x, void *y, void *partial) {
    const vq_gemv_pack_t *p = w->gemv_pack;
    PackPlan plan;
    (void)pack_plan(w, &plan);   // (checked by check_pack before any launch)
    PackedLaunch l;
    PackedArgs &a = l.a;
    a.data = (const unsigned char *)p->data;
    a.cb = (const half_t *)w->codebooks;
    a.scale = (const half_t *)w->scale;
    a.x = (const half_t *)x;
    a.y = (half_t *)y;
    a.partial = (float *)partial;
    a.N = w->N;
    a.J = w->K / 8;
    a.S = (int)p->S;
    a.RB = (int)p->RB;
    a.rows_per_block = (int)p->rows_per_block;
    a.EB = (int)plan.EB;
    a.P = (int)plan.P;
    a.Jp = (int)plan.Jp;
    a.n_groups = (int)plan.G;
    a.task_off = p->task_off;
    a.steps_off = p->steps_off;
    a.atom_off = p->atom_off;
    a.wg_pitch = p->wg_pitch;
    {
        unsigned at = 0;
        for (int g = 0; g < VQ_PACK_MAX_GROUPS; ++g) {
            a.group[g] = (at << 16) | p->group_steps[g];
            at += p->group_steps[g];
        }
    }
    l.lds = plan.lds;
    // every wavefront the same number of groups (the first, longest ones are dealt first, one to each)
    const int rounds = ((int)plan.G + 15) / 16;
    l.waves = ((int)plan.G + rounds - 1) / rounds;
    if (l.waves < 8) l.waves = 8;   // at least 512 threads, so that slice and x are staged with many loads in flight
    a.nwaves = l.waves;
    l.grid = (int)(p->S * p->RB);
    return l;
}

}  // namespace

namespace {

// The reduction that a main-kernel launch leaves to whoever comes next.
PendingArgs pending_of(const PackedArgs *probs, int count) {
    PendingArgs pd;
    std::memset(&pd, 0, sizeof(pd));
    pd.count = count;
    for (int i = 0; i < kPackMaxBatch; ++i) {
        const PackedArgs &a = probs[i < count ? i : 0];
        pd.a[i] = {a.partial, a.scale, a.y, a.N, a.S};
        pd.first_block[i] = i < count ? pd.blocks_total : 0x7fffffff;
        if (i < count) pd.blocks_total += (a.N + 63) / 64;
    }
    return pd;
}

// The plain reduction kernel for a pending set (after the last launch of a call or sequence, or when the next
// launch has too few workgroups to take the rows along).
int launch_finalize(const PendingArgs &pd, hipStream_t s) {
    if (pd.count == 0) return VQ_OK;
    if (pd.count == 1) {
        const FinalizeArgs &a = pd.a[0];
        gemv_packed_finalize_kernel<<<(a.N + kFinalizeRows - 1) / kFinalizeRows, kFinalizeRows, 0, s>>>(a.partial, a.scale, a.y, a.N, a.S);
        return launch_status();
    }
    FinalizeBatch f;
    int max_n = 0;
    for (int i = 0; i < kPackMaxBatch; ++i) {
        f.a[i] = pd.a[i];
        if (i < pd.count && pd.a[i].N > max_n) max_n = pd.a[i].N;
    }
    gemv_packed_finalize_batch_kernel<<<dim3((max_n + kFinalizeRows - 1) / kFinalizeRows, pd.count), kFinalizeRows, 0, s>>>(f);
    return launch_status();
}

}  // namespace

// Partial sums of the problems of a batch lie back to back in the workspace, each 256-byte aligned.
size_t gemv_packed_batch_workspace(const vq_weight_t *const *w, int count) {
    size_t total = 0;
    for (int i = 0; i < count; ++i) total += (gemv_packed_workspace(w[i]) + 255) & ~(size_t)255;
    return total;
}

// One launch of the main kernel for `count` problems (1 .. kPackMaxBatch).  `in`: the reduction left over by the
// previous launch on this stream, or null; it rides along in this launch when the launch has workgroups enough,
// otherwise it gets the plain reduction kernel first.  `out` receives this launch's own pending reduction.
int launch_gemv_packed_main(const vq_weight_t *const *w, const void *const *x, void *const *y, int count, void *ws,
                            const PendingArgs *in, PendingArgs *out, hipStream_t s) {
    PackedBatch b;
    int grid = 0, waves = 0;
    size_t lds = 0, off = 0;
    for (int i = 0; i < kPackMaxBatch; ++i) {
        const int k = i < count ? i : 0;  // unused slots repeat problem 0 (never launched: grid.y = count)
        PackedLaunch l = packed_launch(w[k], x[k], y[k], (unsigned char *)ws + (i < count ? off : 0));
        b.a[i] = l.a;
        if (i < count) {
            off += (gemv_packed_workspace(w[i]) + 255) & ~(size_t)255;
            grid = l.grid > grid ? l.grid : grid;
            waves = l.waves > waves ? l.waves : waves;
            lds = l.lds > lds ? l.lds : lds;
        }
    }
    for (int i = 0; i < kPackMaxBatch; ++i) b.a[i].nwaves = waves;  // one launch shape for all problems
    PendingArgs pd;
    std::memset(&pd, 0, sizeof(pd));
    if (in && in->count > 0) {
        const int n_wg = grid * count;
        const int per = (in->blocks_total + n_wg - 1) / n_wg;
        if (per <= kFinChunks && per <= waves) {
            pd = *in;
            pd.blocks_per_wg = per;
            lds += (size_t)per * kFinChunkBytes;
        } else if (int st = launch_finalize(*in, s)) {
            return st;
        }
    }
    *out = pending_of(b.a, count);
    if (count == 1) {
        static KernelSetup setup;   // (the atoms hold absolute LDS addresses: no static LDS allowed)
        if (int st = kernel_setup(reinterpret_cast<const void *>(&gemv_packed_kernel), lds, true, setup)) return st;
        gemv_packed_kernel<<<grid, waves * 64, lds, s>>>(b.a[0], pd);
    } else {
        static KernelSetup setup;
        if (int st = kernel_setup(reinterpret_cast<const void *>(&gemv_packed_batch_kernel), lds, true, setup)) return st;
        gemv_packed_batch_kernel<<<dim3(grid, count), waves * 64, lds, s>>>(b, pd);
    }
    return launch_status();
}

int launch_gemv_packed_batch(const vq_weight_t *const *w, const void *const *x, void *const *y, int count, void *ws,
                             hipStream_t s) {
    PendingArgs out;
    if (int st = launch_gemv_packed_main(w, x, y, count, ws, nullptr, &out, s)) return st;
    return launch_finalize(out, s);
}

int launch_gemv_packed(const vq_weight_t *w, const void *x, void *y, void *ws, hipStream_t s) {
    return launch_gemv_packed_batch(&w, &x, &y, 1, ws, s);
}

// A sequence of calls, each a batch of 1 .. kPackMaxBatch problems with re-tiled codes: one launch per call plus one
// reduction launch at the very end.  The partial sums of consecutive calls alternate between the two halves of
// the workspace (a launch reads the previous call's while it writes its own).
size_t gemv_packed_sequence_workspace(const vq_gemv_call_t *calls, int n_calls) {
    size_t half = 0;
    for (int c = 0; c < n_calls; ++c) half = std::max(half, gemv_packed_batch_workspace(calls[c].w, calls[c].count));
    return 2 * ((half + 255) & ~(size_t)255);
}

int launch_gemv_packed_sequence(const vq_gemv_call_t *calls, int n_calls, void *ws, hipStream_t s) {
    const size_t half = gemv_packed_sequence_workspace(calls, n_calls) / 2;
    PendingArgs pending;
    std::memset(&pending, 0, sizeof(pending));
    for (int c = 0; c < n_calls; ++c) {
        PendingArgs next;
        if (int st = launch_gemv_packed_main(calls[c].w, calls[c].x, calls[c].y, calls[c].count,
                                             (unsigned char *)ws + (size_t)(c & 1) * half, &pending, &next, s))
            return st;
        pending = next;
    }
    return launch_finalize(pending, s);
}

// ---- the pipelined launch: host side -----------------------------------------------------------------------
// Workspace: [status word, 256 B][problem table][partial sums of every problem, each 256-byte aligned].
namespace {
constexpr size_t kPipeHeader = 256;
size_t pipe_table_bytes(int n) { return ((size_t)n * sizeof(PipeProblem) + 255) & ~(size_t)255; }
// the table of groups: one word per (problem, row block of an image, group); at most 4 row blocks per image
size_t pipe_items_bytes(const vq_gemv_call_t *calls, int n_calls) {
    size_t groups = 0;
    for (int c = 0; c < n_calls; ++c)
        for (int i = 0; i < calls[c].count; ++i) {
            const vq_gemv_pack_t *p = calls[c].w[i]->gemv_pack;
            groups += 4 * (((size_t)p->rows_per_block * p->parts + 63) / 64);
        }
    return (groups * sizeof(uint32_t) + 255) & ~(size_t)255;
}
int pipe_problems(const vq_gemv_call_t *calls, int n_calls) {
    int n = 0;
    for (int c = 0; c < n_calls; ++c) n += calls[c].count;
    return n;
}
}  // namespace

// The staging operations of a problem's LDS image ([slice][parts of x, kZeroUnits zero units behind each]), dealt to
// the producers in turn.  False if a producer would get more than kPipeOps of them.
static bool pipe_build_ops(PipeProblem &p) {
    std::vector<std::pair<uint32_t, uint32_t>> ops;
    const uint32_t slice_bytes = 16u << p.EB, part_pitch = ((uint32_t)p.Jp + kZeroUnits) * 16u;
    for (uint32_t c = 0; c < slice_bytes / 4096; ++c) ops.push_back({c * 4096, pipe_op(c * 4096, kOpSlice4k, 0)});
    for (int q = 0; q < p.P; ++q) {
        const uint32_t len = (uint32_t)std::min(p.Jp, p.J - q * p.Jp);   // positions of this part
        const uint32_t src0 = (uint32_t)q * (uint32_t)p.Jp * 16u, dst0 = slice_bytes + (uint32_t)q * part_pitch;
        const uint32_t full = len >> 8;
        for (uint32_t c = 0; c < full; ++c) ops.push_back({src0 + c * 4096, pipe_op(dst0 + c * 4096, kOpX4k, 0)});
        for (uint32_t t = full * 4; t * 64 < len; ++t)
            ops.push_back({src0 + t * 1024, pipe_op(dst0 + t * 1024, kOpX1k, std::min(64u, len - t * 64))});
        ops.push_back({0u, pipe_op(dst0 + (uint32_t)p.Jp * 16u, kOpZero, 0)});
    }
    if (ops.size() > (size_t)kPipeProducers * kPipeOps) return false;
    std::memset(p.ops, 0, sizeof(p.ops));
    for (size_t j = 0; j < ops.size(); ++j) {
        p.ops[j % kPipeProducers][j / kPipeProducers][0] = ops[j].first;
        p.ops[j % kPipeProducers][j / kPipeProducers][1] = ops[j].second;
    }
    return true;
}

struct GemvPipeline {
    int device;
    uint32_t n;
    PipeLanes lanes;
    int max_n;
    PipeProblem *table;    // device
    uint32_t *items;       // device
    uint32_t *status;      // device
};

// S partial sums per row in blocks of 64 rows (partial_index), 256-byte aligned.
static size_t pipe_partial_bytes(const vq_weight_t *w) { return (gemv_packed_workspace(w) + 255) & ~(size_t)255; }
size_t gemv_pipeline_workspace(const vq_gemv_call_t *calls, int n_calls) {
    size_t total = kPipeHeader + pipe_table_bytes(pipe_problems(calls, n_calls)) + pipe_items_bytes(calls, n_calls);
    for (int c = 0; c < n_calls; ++c)
        for (int i = 0; i < calls[c].count; ++i) total += pipe_partial_bytes(calls[c].w[i]);
    return total;
}

// Whether the pipelined kernel can take this (already validated) weight: its block fits one workgroup of the
// persistent launch, and its LDS image one of the two slots.
bool gemv_pipeline_supports(const vq_weight_t *w) {
    PackPlan plan;
    if (!pack_plan(w, &plan)) return false;
    const size_t image = ((size_t)plan.slice_entries + (size_t)plan.P * (plan.Jp + kZeroUnits)) * 16;
    return plan.S * plan.RB <= (uint32_t)kPipeWgs && image + 64 <= kPipeImage;   // (64 bytes of counters in the tail of image 0)
}

// Builds the problem table in the workspace (a synchronous copy: the calls' arrays need not outlive this).
int gemv_pipeline_create(const vq_gemv_call_t *calls, int n_calls, void *ws, hipStream_t s, GemvPipeline **out) {
    const int n = pipe_problems(calls, n_calls);
    std::vector<PipeProblem> probs((size_t)n);
    unsigned char *base = (unsigned char *)ws;
    const size_t items_off = kPipeHeader + pipe_table_bytes(n);
    size_t off = items_off + pipe_items_bytes(calls, n_calls);
    int k = 0, max_n = 0;
    if (n > 0xFFFF) return VQ_ERR_UNSUPPORTED;   // (a problem number travels in 16 bits)
    uint32_t bpi = 4, max_vwg = 1;   // blocks per image: the largest of 4, 2, 1 that divides every problem's row blocks
    for (int c = 0; c < n_calls; ++c)
        for (int i = 0; i < calls[c].count; ++i)
            while (calls[c].w[i]->gemv_pack->RB % bpi) bpi >>= 1;
    for (int c = 0; c < n_calls; ++c)
        for (int i = 0; i < calls[c].count; ++i, ++k) {
            const vq_weight_t *w = calls[c].w[i];
            const PackedLaunch l = packed_launch(w, calls[c].x[i], calls[c].y[i], base + off);
            off += pipe_partial_bytes(w);
            const PackedArgs &a = l.a;
            PipeProblem &p = probs[(size_t)k];
            std::memset(&p, 0, sizeof(p));
            p.atoms = a.data + a.atom_off;
            p.tasks = a.data + a.task_off;
            p.steps = a.data + a.steps_off;
            p.cb = a.cb; p.x = a.x; p.partial = a.partial; p.scale = a.scale; p.y = a.y;
            p.N = a.N; p.J = a.J; p.S = a.S; p.RB = a.RB; p.rows_per_block = a.rows_per_block;
            p.EB = a.EB; p.P = a.P; p.Jp = a.Jp; p.n_groups = a.n_groups;
            p.wg_pitch = a.wg_pitch;
            p.bpi = bpi;
            p.rbv = (uint32_t)a.RB / bpi;
            for (int g = 0; g < a.n_groups; ++g)
                if ((a.group[g] & 0xFFFFu) > 255u) return VQ_ERR_UNSUPPORTED;   // (the first step of a piece travels in 8 bits)
            std::memcpy(p.group, a.group, sizeof(p.group));
            if (!pipe_build_ops(p)) return VQ_ERR_UNSUPPORTED;
            if (a.N > max_n) max_n = a.N;
            max_vwg = std::max(max_vwg, (uint32_t)(a.S * a.RB) / bpi);
        }
    // lanes: as many as fit side by side (a power of two; the largest problem decides)
    PipeLanes lanes;
    std::memset(&lanes, 0, sizeof(lanes));
    uint32_t n_lanes = 1;
    while (n_lanes < 8 && max_vwg * n_lanes * 2 <= (uint32_t)kPipeWgs && max_vwg * n_lanes * 2 / 8 * 8 == max_vwg * n_lanes * 2) n_lanes *= 2;
    if (max_vwg % 8) n_lanes = 1;   // (the die bits of a workgroup number must be those of its number within the lane)
    while ((1u << lanes.log2_lanes) < n_lanes) ++lanes.log2_lanes;
    // the table, lane after lane; within a lane the problems keep their order
    std::vector<PipeProblem> table;
    std::vector<uint32_t> items;
    table.reserve((size_t)n);
    for (uint32_t l = 0; l < n_lanes; ++l) {
        lanes.first[l] = (uint32_t)table.size();
        lanes.item_first[l] = (uint32_t)items.size();
        uint32_t through[2] = {0u, 0u};
        for (int q = (int)l; q < n; q += (int)n_lanes) {
            PipeProblem p = probs[(size_t)q];
            const uint32_t i = (uint32_t)table.size() - lanes.first[l];   // its number within the lane
            through[i & 1u] += (uint32_t)p.n_groups;
            p.groups_through = through[i & 1u];
            // where the sums of its tasks wait for the producers: the buffer of its image's parity, or (more than
            // 4096 tasks per image) the tail of the image itself
            const uint32_t acc_bytes = bpi * (uint32_t)p.rows_per_block * (uint32_t)p.P * 4u;
            const uint32_t image = (((16u << p.EB) + (uint32_t)p.P * ((uint32_t)p.Jp + kZeroUnits) * 16u) + 15u) & ~15u;
            if (acc_bytes <= kPipeAccBytes)
                p.acc_lds = kPipeAcc + (i & 1u) * kPipeAccBytes;
            else if (image + acc_bytes + 64u <= kPipeImage)
                p.acc_lds = (i & 1u) * kPipeImage + image;
            else
                return VQ_ERR_UNSUPPORTED;
            for (uint32_t jb = 0; jb < bpi; ++jb)
                for (uint32_t g = 0; g < (uint32_t)p.n_groups; ++g) items.push_back(i | (jb << 16) | (g << 20));
            table.push_back(p);
        }
        lanes.n[l] = (uint32_t)table.size() - lanes.first[l];
        lanes.items[l] = (uint32_t)items.size() - lanes.item_first[l];
    }
    GemvPipeline *h = new (std::nothrow) GemvPipeline;
    if (!h) return VQ_ERR_LAUNCH;
    if (hipGetDevice(&h->device) != hipSuccess) { delete h; return VQ_ERR_LAUNCH; }
    h->n = (uint32_t)n;
    h->lanes = lanes;
    h->max_n = max_n;
    h->status = reinterpret_cast<uint32_t *>(base);
    h->table = reinterpret_cast<PipeProblem *>(base + kPipeHeader);
    h->items = reinterpret_cast<uint32_t *>(base + items_off);
    if (hipMemsetAsync(h->status, 0, kPipeHeader, s) != hipSuccess ||
        hipMemcpyAsync(h->table, table.data(), (size_t)n * sizeof(PipeProblem), hipMemcpyHostToDevice, s) != hipSuccess ||
        hipMemcpyAsync(h->items, items.data(), items.size() * sizeof(uint32_t), hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
        delete h;
        return VQ_ERR_LAUNCH;
    }
    *out = h;
    return VQ_OK;
}

void gemv_pipeline_destroy(GemvPipeline *h) { delete h; }

int launch_gemv_pipeline(const GemvPipeline *h, hipStream_t s) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != h->device) return VQ_ERR_LAUNCH;   // the table lives on another GPU
    static KernelSetup setup;   // (the atoms hold absolute LDS addresses: no static LDS allowed)
    if (int st = kernel_setup(reinterpret_cast<const void *>(&gemv_pipeline_kernel), kPipeLds, true, setup)) return st;
    gemv_pipeline_kernel<<<kPipeWgs, (kPipeConsumers + kPipeProducers) * 64, kPipeLds, s>>>(h->table, h->items, h->lanes, h->status);
    if (int st = launch_status()) return st;
    gemv_pipeline_finalize_kernel<<<dim3((h->max_n + kFinalizeRows - 1) / kFinalizeRows, h->n), kFinalizeRows, 0, s>>>(h->table);
    return launch_status();
}

int gemv_pipeline_status(const GemvPipeline *h, hipStream_t s, int *status) {
    uint32_t v = 0;
    if (hipMemcpyAsync(&v, h->status, sizeof(v), hipMemcpyDeviceToHost, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
        return VQ_ERR_LAUNCH;
    *status = (int)v;
    return VQ_OK;
}

}  // namespace vq

using namespace vq;

extern "C" {

size_t vq_gemv_prepack_bytes(const vq_weight_t *w) {
    if (!w || !w->codes || !pack_supported(w)) return 0;
    return (size_t)pack_build(w, nullptr, nullptr, nullptr);
}

int vq_gemv_prepack(const vq_weight_t *w, void *out_host, size_t out_bytes, vq_gemv_pack_t *pack) {
    if (!w || !w->codes || !out_host || !pack) return VQ_ERR_NULL;
    if (!pack_supported(w)) return VQ_ERR_UNSUPPORTED;
    if (!aligned16(out_host)) return VQ_ERR_ALIGN;
    bool bad_code = false;
    const uint64_t need = pack_build(w, nullptr, nullptr, &bad_code);
    if (bad_code) return VQ_ERR_SHAPE;          // a code >= n_entries
    if (need == 0) return VQ_ERR_UNSUPPORTED;   // codes too uneven for a common shape
    if (out_bytes < need) return VQ_ERR_WORKSPACE;
    pack_build(w, (unsigned char *)out_host, pack, nullptr);
    return VQ_OK;
}

}  // extern "C"
