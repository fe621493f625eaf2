// bs = 1 VQ-gemv from re-tiled ("packed") codes: codebook slices in LDS, dense LDS gathers.
//
// Why: with a 2^16 x 8 fp16 codebook (1 MiB) the entries cannot live in LDS, and random
// 16-byte gathers from L2 run at ~0.44 per clock per CU on MI355X (each one moves a
// 128-byte line), an order of magnitude below what the HBM code stream could feed.  Random
// 16-byte gathers from LDS run at ~5.5 per clock per CU.  So the product is partitioned
// along the codebook itself -- the codebook-centric dataflow of VQ-LLM (arXiv 2503.02236)
// Sec. VI-A pushed from "one codebook per block" to "one codebook slice per block":
//   workgroup (s, rb) holds slice s (E/S entries) and the activation vector in LDS and
//   processes, for the rows of block rb, exactly the codes that point into slice s.
// Those codes are found offline (Sec. II-C: weights are quantized offline; Sec. V-B already
// rewrites indices offline) by vq_gemv_prepack and stored as 24-bit atoms, two 12-bit numbers of
// 16-byte units in the workgroup's LDS image  [slice: E/S units][x: K/8 units][one zero unit]:
//   bits 0..11   unit of the entry   = its index inside the slice
//   bits 12..23  unit of x_j         = E/S + j
// so an address is a shift and a mask away from the atom.  A padding atom names the zero unit twice and
// adds 0 * 0: no validity test per atom (the loop around the gathers is bound by vector ALU issue: 15
// instructions per atom before this format, 9 with it).  The image must fit 4096 units: slices of at most
// 2048 entries, K/8 <= 2047.
// One lane owns one row: it walks that row's atoms (j ascending), gathers entry and x_j from
// LDS and accumulates privately, so there is no cross-lane reduction at all.  Rows of a block
// are sorted by atom count and grouped 64 at a time, so the lanes of a wavefront run nearly the
// same trip count.  The S partial sums of a row are added in slice order by a second small
// kernel (Sec. VI-A "explicit global reduction"), which keeps the result bit-reproducible.
//
// Packed buffer (little endian, offsets from the start of the buffer, 256-byte aligned):
//   row ids      [S*RB][G][64] uint16   row inside the block, 0xFFFF = idle lane; G = ceil(rows_per_block / 64)
//   atoms        blocks of 768 bytes = 64 lanes x 12 bytes = 4 atoms per lane per step; 16 blocks of padding atoms
//                follow the last workgroup's (the kernels read a few blocks past the end of a group without looking)
// Placement of the atom blocks.  A kernel that has to read a table before it can ask for its atoms
// pays two dependent first touches of memory (~1.5 us each) before any work.  Codes that spread evenly
// over the codebook make group g look nearly the same in every workgroup (the g-th 64 rows of a sorted
// list of equally distributed lengths), so all workgroups are padded to one common shape: group g has
// group_steps[g] steps everywhere (the maximum over the workgroups; ~5 % more blocks at Llama-7B shapes)
// and starts at block wg * wg_pitch + sum_{g' < g} group_steps[g'].  Those few numbers travel in the
// descriptor and reach the kernel as launch arguments.  Codes too uneven for that (more than a quarter
// more blocks) are declined: the canonical-code kernels serve them.
#include <algorithm>
#include <cstring>
#include <type_traits>
#include <vector>

#include "vq_common.h"

namespace vq {

constexpr int kPackFieldBits = 12;   // an atom = two LDS unit numbers of 12 bits
// atom blocks behind the last workgroup's: the kernels read up to this many blocks past the end of a group
// without looking (a clamp per load costs more instructions than the load)
constexpr int kPackTailBlocks = 16;

struct PackPlan {
    uint32_t S, RB, rows_per_block, slice_entries;
};

static bool pack_supported(const vq_weight_t *w) {
    if (w->v != 8 || w->code_bits != 16 || w->n_codebooks != 1) return false;
    int E = w->n_entries;
    if (E < 4096 || (E & (E - 1)) != 0) return false;
    if (w->K <= 0 || w->N <= 0 || 2048 + w->K / 8 + 1 > (1 << kPackFieldBits)) return false;  // slice + x + zero unit
    return true;
}

// S * RB = 256 workgroups, one per compute unit.  Slices of 2048 entries (32 KiB); a workgroup with more
// than 16 row groups gives its wavefronts several groups each.  Long rows
// (K > 8192) take 1024-entry slices: the atom list of a (row, slice) cell is K/8 / S long, and a short
// list is what keeps every step of a wavefront in its register prefetch (measured on 4096 x 11008:
// 18.2 -> 14.6 us; on K = 4096 the doubled partial-sum traffic costs more than it saves).
static PackPlan pack_plan(const vq_weight_t *w) {
    PackPlan p;
    p.slice_entries = 2048;
    if (w->K / 8 > 1024 && w->n_entries >= 65536) p.slice_entries = 1024;
    p.S = (uint32_t)w->n_entries / p.slice_entries;
    uint32_t rb = 256 / p.S;
    uint32_t max_rb = ((uint32_t)w->N + 63) / 64;   // at least one full 64-row group per block
    if (rb > max_rb) rb = max_rb;
    if (rb < 1) rb = 1;
    p.RB = rb;
    p.rows_per_block = ((uint32_t)w->N + rb - 1) / rb;
    return p;
}

static inline uint64_t align256(uint64_t x) { return (x + 255) & ~(uint64_t)255; }

// One pass builds everything; `out` == nullptr only measures.
static uint64_t pack_build(const vq_weight_t *w, unsigned char *out, vq_gemv_pack_t *pack) {
    const PackPlan p = pack_plan(w);
    const int J = w->K / 8;
    const uint16_t *codes = reinterpret_cast<const uint16_t *>(w->codes);
    uint32_t lb = 0;  // log2(slice_entries)
    while ((1u << lb) < p.slice_entries) ++lb;
    const uint32_t nwg = p.S * p.RB;

    // counts[rb][s][row_in_block]
    std::vector<uint32_t> cnt((size_t)nwg * p.rows_per_block, 0);
    for (int n = 0; n < w->N; ++n) {
        uint32_t rb = (uint32_t)n / p.rows_per_block, ri = (uint32_t)n % p.rows_per_block;
        const uint16_t *row = codes + (size_t)n * J;
        for (int j = 0; j < J; ++j) cnt[((size_t)(row[j] >> lb) * p.RB + rb) * p.rows_per_block + ri]++;
    }
    // per workgroup: rows sorted by count (descending, ties by row), groups of 64
    const uint32_t ng = (p.rows_per_block + 63) / 64;
    if (ng > VQ_PACK_MAX_GROUPS) return 0;
    std::vector<uint32_t> steps((size_t)nwg * ng, 0);   // steps a group needs
    std::vector<uint16_t> rowids;
    rowids.reserve((size_t)nwg * ng * 64);
    std::vector<uint32_t> order(p.rows_per_block);
    std::vector<uint32_t> max_steps(ng, 0);
    uint64_t needed_blocks = 0;
    for (uint32_t wg = 0; wg < nwg; ++wg) {
        uint32_t rb = wg % p.RB;
        uint32_t rows_here = 0;
        if ((uint64_t)rb * p.rows_per_block < (uint64_t)w->N)
            rows_here = std::min<uint32_t>(p.rows_per_block, (uint32_t)w->N - rb * p.rows_per_block);
        const uint32_t *c = &cnt[(size_t)wg * p.rows_per_block];
        for (uint32_t i = 0; i < rows_here; ++i) order[i] = i;
        std::stable_sort(order.begin(), order.begin() + rows_here, [&](uint32_t a, uint32_t b) { return c[a] > c[b]; });
        for (uint32_t g = 0; g < ng; ++g) {
            const uint32_t st = g * 64 < rows_here ? (c[order[g * 64]] + 3) / 4 : 0;  // a group's first row is its longest
            steps[(size_t)wg * ng + g] = st;
            needed_blocks += st;
            max_steps[g] = std::max(max_steps[g], st);
            for (uint32_t l = 0; l < 64; ++l) {
                uint32_t i = g * 64 + l;
                rowids.push_back(i < rows_here ? (uint16_t)order[i] : (uint16_t)0xFFFF);
            }
        }
    }
    // the common shape of all workgroups (at least one block each: the kernel's wavefronts without work read it)
    if (max_steps[0] == 0) max_steps[0] = 1;
    uint64_t pitch = 0;
    std::vector<uint32_t> prefix(ng, 0);
    for (uint32_t g = 0; g < ng; ++g) {
        prefix[g] = (uint32_t)pitch;
        pitch += max_steps[g];
    }
    // too uneven: more than a quarter more blocks than needed -- unless that is less than 1 MiB (small or
    // ragged matrices, where a group of a few rows is as long as its longest row in the unluckiest workgroup)
    const uint64_t padded = pitch * nwg;
    if (pitch > 65535) return 0;
    if (padded > needed_blocks + needed_blocks / 4 + nwg && (padded - needed_blocks) * 768 > (1u << 20)) return 0;
    const uint64_t atom_blocks = pitch * nwg;
    const uint64_t rowid_off = 0;
    const uint64_t atom_off = align256(rowid_off + rowids.size() * 2);
    const uint64_t total = atom_off + (atom_blocks + kPackTailBlocks) * 768;
    if (pack) {
        pack->data = out;
        pack->bytes = total;
        pack->S = p.S;
        pack->RB = p.RB;
        pack->rows_per_block = p.rows_per_block;
        pack->wg_pitch = (uint32_t)pitch;
        pack->rowid_off = rowid_off;
        pack->atom_off = atom_off;
        for (uint32_t g = 0; g < VQ_PACK_MAX_GROUPS; ++g) pack->group_steps[g] = g < ng ? (uint16_t)max_steps[g] : (uint16_t)0;
    }
    if (!out) return total;

    std::memset(out, 0, (size_t)atom_off);
    std::memcpy(out + rowid_off, rowids.data(), rowids.size() * 2);
    unsigned char *atoms = out + atom_off;
    // padding everywhere first: the zero unit (behind slice and x) as entry and as x_j
    const uint32_t zero_unit = p.slice_entries + (uint32_t)J;
    const uint32_t pad_atom = zero_unit | (zero_unit << kPackFieldBits);
    for (uint64_t i = 0, n_atoms = (atom_blocks + kPackTailBlocks) * 256; i < n_atoms; ++i) {
        atoms[3 * i] = (unsigned char)pad_atom;
        atoms[3 * i + 1] = (unsigned char)(pad_atom >> 8);
        atoms[3 * i + 2] = (unsigned char)(pad_atom >> 16);
    }
    // fill: lane l of group g walks row rowids[wg][g][l]; its k-th atom of slice s goes to step k/4, slot k%4
    for (uint32_t wg = 0; wg < nwg; ++wg) {
        uint32_t s = wg / p.RB, rb = wg % p.RB;
        for (uint32_t g = 0; g < ng; ++g) {
            const uint64_t first_block = (uint64_t)wg * pitch + prefix[g];
            for (uint32_t l = 0; l < 64; ++l) {
                uint16_t ri = rowids[((size_t)wg * ng + g) * 64 + l];
                if (ri == 0xFFFF) continue;
                const uint16_t *row = codes + ((size_t)rb * p.rows_per_block + ri) * J;
                uint32_t k = 0;
                for (int j = 0; j < J; ++j) {
                    if ((uint32_t)(row[j] >> lb) != s) continue;
                    uint32_t atom = (row[j] & ((1u << lb) - 1)) | ((p.slice_entries + (uint32_t)j) << kPackFieldBits);
                    unsigned char *q = atoms + (first_block + k / 4) * 768 + l * 12 + (k % 4) * 3;
                    q[0] = (unsigned char)atom;
                    q[1] = (unsigned char)(atom >> 8);
                    q[2] = (unsigned char)(atom >> 16);
                    ++k;
                }
            }
        }
    }
    return total;
}

// ---------------------------------------------------------------------------------- kernel

// What the main kernel needs of the launch arguments before its first vector load leaves ...
struct PackedCore {
    const unsigned char *data;
    const half_t *cb, *x;
    float *partial;       // [S][N]
    int N, J, S, RB, rows_per_block, slice_entries;
    unsigned long long rowid_off, atom_off;
    unsigned wg_pitch;    // group g of workgroup wg: atom blocks from wg * wg_pitch + prefix[g] on
    int nwaves;           // wavefronts per workgroup of the launch (saves a load of the hidden launch arguments)
};
// ... and the rest: one 32-bit word per group, prefix << 16 | steps, so that a scalar load can fetch it
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

constexpr int kPackMaxSlices = 64;  // 2^16 entries / 1024 per slice
// Steps in flight per wavefront: a ring of 3 (9 registers), 2 of them requested before the barrier.  More
// steps requested ahead do not arrive sooner -- a CU's share of the memory system is ~20 KB per microsecond,
// and what is requested ahead of another wavefront's slice transfer delays that transfer and with it the
// barrier (measured on 4096 x 11008: 12 steps ahead, barrier 2.6 us after the loads were issued, 9.8 us in
// all; 4 steps, 1.5 us and 8.8 us).  Llama-7B stack, (ahead, ring): (2,2) 1206, (2,3) 1217, (2,4) 1214,
// (1,3) 1211, (2,5) 1204 GB/s; nothing ahead of the barrier 1150 - 1166.
constexpr int kPackRing = 3;
constexpr int kPackAhead = 2;   // of these, requested before the barrier

struct Acc4 {
    float a0, a1, a2, a3;
};

// 16 bytes at an absolute LDS address.  The kernels below have no static LDS, so the dynamic region (the
// image the atoms index) starts at address 0 and a unit number is an address after one shift; going through
// a pointer into the region would cost one more add per gather for a base the compiler cannot see is 0.
// (A test compiles this file and checks that these kernels have no static LDS.)
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

// One step = the lane's next four atoms (three dwords).  The LDS gathers (entry and x_j of each atom)
// of CL atoms are issued before the first dot product: taken one atom at a time, as the compiler orders
// them when left alone, every atom waits out a full LDS round trip (~90 clocks per gather with eight
// wavefronts asking) and the gather phase of a 4096 x 4096 launch lasts 3.1 us.  CL = 4 keeps 32
// registers of operands in flight, CL = 2 half of that (for the kernels held to 128 registers).
template <int CL>
__device__ __forceinline__ void step_dot(uint32_t d0, uint32_t d1, uint32_t d2, Acc4 &acc) {
    // the 24 bits of atom k start at bit 24 k of the 96-bit string d2:d1:d0
    const uint32_t at[4] = {d0, __builtin_amdgcn_alignbit(d1, d0, 24), __builtin_amdgcn_alignbit(d2, d1, 16), d2 >> 8};
    float *accs[4] = {&acc.a0, &acc.a1, &acc.a2, &acc.a3};
#pragma unroll
    for (int h = 0; h < 4; h += CL) {
        V16 e[CL], xv[CL];
#pragma unroll
        for (int i = 0; i < CL; ++i) {
            e[i] = lds_unit((at[h + i] << 4) & 0xfff0u);
            xv[i] = lds_unit((at[h + i] >> (kPackFieldBits - 4)) & 0xfff0u);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * CL, 0);  // these LDS reads first,
        __builtin_amdgcn_sched_group_barrier(0x002, 4 * CL, 0);  // then the arithmetic on them
#pragma unroll
        for (int i = 0; i < CL; ++i) *accs[h + i] = atom_fma(e[i], xv[i], *accs[h + i]);
    }
}

// Two steps at once: the sixteen gathers of both are issued before the first dot product (a launch with one
// 8-wavefront workgroup per CU has too few gathers in flight to fill the LDS pipeline otherwise).  The dot
// products run in the order of two single steps, so the sums are the same bit for bit.
__device__ __forceinline__ void step_dot_pair(const uint32_t (&da)[3], const uint32_t (&db)[3], Acc4 &acc) {
    const uint32_t at[8] = {da[0], __builtin_amdgcn_alignbit(da[1], da[0], 24), __builtin_amdgcn_alignbit(da[2], da[1], 16), da[2] >> 8,
                            db[0], __builtin_amdgcn_alignbit(db[1], db[0], 24), __builtin_amdgcn_alignbit(db[2], db[1], 16), db[2] >> 8};
    float *accs[4] = {&acc.a0, &acc.a1, &acc.a2, &acc.a3};
    V16 e[8], xv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        e[i] = lds_unit((at[i] << 4) & 0xfff0u);
        xv[i] = lds_unit((at[i] >> (kPackFieldBits - 4)) & 0xfff0u);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, 32, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) *accs[i & 3] = atom_fma(e[i], xv[i], *accs[i & 3]);
}

// All global loads of a workgroup are issued before anything waits: the kernel is a chain of
// memory latencies (tables -> atoms -> partials), not a bandwidth problem, at these sizes.
template <int PF, int CL, bool PAIR, int AHEAD = kPackAhead>
__device__ __forceinline__ void gemv_packed_body(const PackedArgs &ka, const int bid) {
    extern __shared__ __align__(16) unsigned char smem[];
    // all launch arguments in one round of scalar loads
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: group lookups, block numbers and
                                                                         // addresses derived from it stay scalar
    uint32_t group_word = ka.group[wave];
    PackedCore a = ka;
    pin_scalar(a.data); pin_scalar(a.cb); pin_scalar(a.x); pin_scalar(a.partial);
    pin_scalar(a.N); pin_scalar(a.J); pin_scalar(a.S); pin_scalar(a.RB); pin_scalar(a.rows_per_block);
    pin_scalar(a.slice_entries); pin_scalar(a.rowid_off); pin_scalar(a.atom_off); pin_scalar(a.wg_pitch);
    pin_scalar(a.nwaves); pin_scalar(group_word);
    // the LDS image the atoms index, in 16-byte units: [slice][x][one zero unit]; then one float per row of the block
    unsigned char *slice = smem;
    unsigned char *xl = smem + (size_t)a.slice_entries * 16;
    unsigned char *zero_unit = xl + (size_t)a.J * 16;
    float *accbuf = reinterpret_cast<float *>(zero_unit + 16);

    const int tid = threadIdx.x, lane = tid & 63, nwaves = a.nwaves;
    // Workgroups are dealt round-robin to the 8 compute dies, each with its own L2.  All row blocks of
    // one codebook slice run on the same die, so a slice is fetched from memory by one L2 only
    // (otherwise every die pulls the whole 1 MiB codebook: 8 MiB per launch).
    int s, rb;
    if (a.S % 8 == 0) {  // S is a power of two: shifts instead of a division
        const int die = bid & 7, local = bid >> 3, per_die = a.S >> 3, sh = __builtin_ctz(per_die);
        s = die * per_die + (local & (per_die - 1));
        rb = local >> sh;
    } else {
        s = bid / a.RB;
        rb = bid % a.RB;
    }
    const int wg = s * a.RB + rb;  // index into the packed tables
    // (the pinned pointers went through an asm statement and have to be told again that they are global)
    typedef const __attribute__((address_space(1))) unsigned char gbyte_t;
    typedef const __attribute__((address_space(1))) uint16_t gu16_t;
    typedef const __attribute__((address_space(1))) uint32_t gu32_t;
    gbyte_t *gdata = (gbyte_t *)a.data;
    gu16_t *rowids = (gu16_t *)(gdata + a.rowid_off);
    // atom block b of this lane: a scalar base (block numbers are wave-uniform) plus a 32-bit lane offset
    gbyte_t *atoms = gdata + a.atom_off;
    const uint32_t lane_off = (uint32_t)lane * 12u;

    // (1) codebook slice and x go straight from global memory into LDS (no registers): one
    //     wave-wide 1 KiB transfer per 64 entries, lane l's 16 bytes land at base + 16 l.  Written as an
    //     asm statement: with the builtin the compiler knows that LDS is being written behind its back and
    //     makes the first LDS read wait for every outstanding load, the atoms included, which puts the whole
    //     memory phase of a launch in front of its whole gather phase.  The transfers complete in issue order
    //     with the other loads, and the counted wait below is what orders them against the gathers.
    {
        typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
        auto dma16 = [](const uint4 *src, unsigned char *dst_wave_base) {
            const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_byte_t *)dst_wave_base);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(m0), "v"(src) : "memory");  // (M0 is written and used inside the statement; nothing else in this kernel uses it)
        };
        const uint4 *src = reinterpret_cast<const uint4 *>(a.cb) + (size_t)s * a.slice_entries;
        const uint4 *xs = reinterpret_cast<const uint4 *>(a.x);
        for (int c = wave; c * 64 < a.slice_entries; c += nwaves)  // slices are multiples of 64 entries
            dma16(src + c * 64 + lane, slice + c * 1024);
        for (int c = wave; c * 64 < a.J; c += nwaves)
            if (c * 64 + lane < a.J) dma16(xs + c * 64 + lane, xl + c * 1024);
        if (tid < 4) reinterpret_cast<uint32_t *>(zero_unit)[tid] = 0u;  // what padding atoms point at
    }
    // (2) this wavefront's first group: where its atoms lie follows from the launch arguments alone, so
    //     the row ids and the atoms are requested right behind the slice.  Loads complete in the order
    //     they were issued, so the wait below counts the loads of this step as still in flight and lets
    //     the gathers start as soon as the slice and x are in, while the atoms stream in behind them
    //     (waiting for everything put the whole memory phase of a launch in front of its whole LDS
    //     phase).  The empty statement keeps the compiler from moving a load above the staging transfers.
    asm volatile("" ::: "memory");
    const uint32_t n_groups = (uint32_t)(a.rows_per_block + 63) / 64, first_group = (uint32_t)wg * n_groups;
    auto group_of = [&](uint32_t word) { return make_uint2((uint32_t)wg * a.wg_pitch + (word >> 16), word & 0xffffu); };
    // Step st of the group whose first block this lane sees at `base`.  No look at the group's length: a
    // branch around a load keeps the compiler from counting which loads are in flight (it then waits for
    // all of them before every use), and a clamp costs more instructions than the load.  Blocks past the
    // end of a group belong to the next one, or to the tail of the buffer, and are never used.
    static_assert(2 * PF - 2 <= kPackTailBlocks, "reads run up to 2 PF - 2 blocks past the end of a group");
    auto load_step = [&](uint32_t (&dst)[3], gbyte_t *base, uint32_t st) {
        gu32_t *p = (gu32_t *)(base + (size_t)st * 768);
        dst[0] = p[0]; dst[1] = p[1]; dst[2] = p[2];
    };
    auto lane_base = [&](uint32_t first_block) { return atoms + (size_t)first_block * 768 + lane_off; };
    // Every wavefront issues the same kPackAhead + 1 loads, so the count in the wait holds for all of them: one
    // without a group reads the row ids of the last group and the first blocks of the workgroup and uses
    // neither.
    const bool has_group = (uint32_t)wave < n_groups;
    uint2 gr = make_uint2((uint32_t)wg * a.wg_pitch, 0);  // .x first atom block, .y steps
    if (has_group) gr = group_of(group_word);
    uint32_t ri = rowids[((size_t)first_group + min((uint32_t)wave, n_groups - 1)) * 64 + lane];
    uint32_t q[PF][3];  // the ring: the atoms of the next PF steps
    gbyte_t *gbase = lane_base(gr.x);
#pragma unroll
    for (int st = 0; st < AHEAD; ++st) load_step(q[st], gbase, st);
    // kPackAhead atom loads and the row ids were issued behind the staging transfers: when at most that many
    // loads are pending, the transfers have landed.  (A test compiles this file and counts those loads in each build.)
    // (lgkmcnt: the store of the zero unit)
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(AHEAD + 1) : "memory");
    // (3) the slice and x of this wavefront have landed (direct-to-LDS transfers count as vector memory
    //     loads); after the barrier those of all wavefronts are visible.  A bare s_barrier: __syncthreads()
    //     would wait for the atoms as well.
    asm volatile("s_barrier" ::: "memory");
#pragma unroll
    for (int st = AHEAD; st < PF; ++st) load_step(q[st], gbase, st);  // the rest of the ring

    // (4) gathers and dot products: lane = row; results go to LDS in natural row order.  The ring already
    //     holds the group's first PF steps.
    auto run_group = [&](const uint2 gr, const uint32_t ri, gbyte_t *gbase) {
        Acc4 acc = {0.f, 0.f, 0.f, 0.f};
        // slot k is refilled with step st + PF as soon as step st has been taken out of it -- except in the
        // group's last round: what would be requested there lies past the end of the group (with a refill in
        // every round a group of 5 steps read 9 blocks; the blocks read in vain are the next group's, but
        // they cross the memory system once more all the same).  Measured on the Llama-7B stack: 1163 -> 1214
        // GB/s; refilling exactly up to the group's end (one copy of the round before the last per number of
        // refills) was slower again, 1154 - 1181.
        auto ring_round = [&](uint32_t base, auto refill_tag) {
            if constexpr (PAIR) {
                static_assert(!PAIR || PF % 2 == 0, "steps are taken two at a time");
#pragma unroll
                for (int k = 0; k < PF; k += 2) {
                    const uint32_t da[3] = {q[k][0], q[k][1], q[k][2]}, db[3] = {q[k + 1][0], q[k + 1][1], q[k + 1][2]};
                    if constexpr (decltype(refill_tag)::value) {
                        load_step(q[k], gbase, base + k + PF);
                        load_step(q[k + 1], gbase, base + k + 1 + PF);
                    }
                    if (base + k + 1 < gr.y) step_dot_pair(da, db, acc);
                    else if (base + k < gr.y) step_dot<CL>(da[0], da[1], da[2], acc);
                }
            } else {
#pragma unroll
                for (int k = 0; k < PF; ++k) {
                    const uint32_t d0 = q[k][0], d1 = q[k][1], d2 = q[k][2];
                    if constexpr (decltype(refill_tag)::value) load_step(q[k], gbase, base + k + PF);
                    if (base + k < gr.y) step_dot<CL>(d0, d1, d2, acc);
                }
            }
        };
        // (the first round outside the loop: at a loop head the ring would be copied, and a copy needs
        // all of its data)
        uint32_t base = 0;
        if (gr.y > (uint32_t)PF) {
            ring_round(0, std::true_type{});
            for (base = PF; base + PF < gr.y; base += PF) ring_round(base, std::true_type{});
        }
        if (gr.y > 0) ring_round(base, std::false_type{});
        if (ri != 0xFFFFu) accbuf[ri] = (acc.a0 + acc.a1) + (acc.a2 + acc.a3);
    };
    if (has_group) run_group(gr, ri, gbase);
    for (uint32_t g = wave + nwaves; g < n_groups; g += nwaves) {  // only when a block has more groups than wavefronts
        const uint2 gr2 = group_of(ka.group[g]);
        const uint32_t ri2 = rowids[((size_t)first_group + g) * 64 + lane];
        gbyte_t *gbase2 = lane_base(gr2.x);
#pragma unroll
        for (int k = 0; k < PF; ++k) load_step(q[k], gbase2, k);
        run_group(gr2, ri2, gbase2);
    }
    __syncthreads();

    // (5) this slice's partial sums, in natural row order (coalesced).  A second, tiny kernel adds the
    // S partials of every row in slice order -- the "explicit global reduction" of Sec. VI-A.  It is a
    // kernel of its own because device-wide synchronisation inside one kernel costs more here.  Measured
    // with the "last workgroup of a row block reduces" pattern at the 4096 x 4096 shape (one thread per
    // workgroup takes a ticket): a relaxed device-scope ticket returns after 1.8 us (median), an
    // acquire-release one (L2 write-back and invalidate) after 3.8 us, and the last workgroup then needs
    // 4 us to read the 64 KiB of partials through its emptied L2 -- 9.5 us from the first partial store to
    // the end, against ~3.5 us for the second launch.
    for (uint32_t c = wave; c < n_groups; c += nwaves) {
        const int r = (int)c * 64 + lane;
        const int n = rb * a.rows_per_block + r;
        if (r < a.rows_per_block && n < a.N) ((__attribute__((address_space(1))) float *)a.partial)[(size_t)s * a.N + n] = accbuf[r];
    }
}

// One problem: 8 to 16 wavefronts, one per row group of the block (more groups than that: several each).
__global__ __launch_bounds__(1024) void gemv_packed_kernel(PackedArgs a) { gemv_packed_body<4, 4, true>(a, blockIdx.x); }

// Several independent problems in one launch (blockIdx.y picks the problem): the fixed latencies of a
// launch (ramp-up, first touches of tables and atoms, drain) are paid once for all of them, and
// workgroups of different problems share a CU.
constexpr int kPackMaxBatch = 4;
struct PackedBatch {
    PackedArgs a[kPackMaxBatch];
};
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(6))) void gemv_packed_batch_kernel(PackedBatch b) {
    const PackedArgs &a = b.a[blockIdx.y];
    if ((int)blockIdx.x >= a.S * a.RB) return;
    gemv_packed_body<kPackRing, 4, false>(a, blockIdx.x);
}

// y[n] = scale[n] * sum_s partial[s][n], slices in ascending order.  MAXS loads are issued unconditionally
// (slices past S re-read the last one) so that none of them waits behind a branch.  One row per thread, one
// wavefront per block: the kernel is one memory round trip long, and the fewer requests queue on a CU the
// shorter it is (256 rows per block: 1209 GB/s on the Llama-7B stack, 64 rows: 1220).
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
    for (int k = 0; k < MAXS; ++k) v[k] = gp[(size_t)(k < S ? k : S - 1) * N + n];
    const float sc = scale ? (float)gs[n] : 1.f;
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < MAXS; ++k) sum += k < S ? v[k] : 0.f;
    gy[n] = (half_t)(sum * sc);
}
__global__ __launch_bounds__(kFinalizeRows) void gemv_packed_finalize_kernel(const float *__restrict__ partial,
                                                                  const half_t *__restrict__ scale,
                                                                  half_t *__restrict__ y, int N, int S) {
    pin_scalar(partial); pin_scalar(scale); pin_scalar(y); pin_scalar(N); pin_scalar(S);  // one round of argument loads
    if (S <= 32)
        gemv_packed_finalize_body<32>(partial, scale, y, N, S);
    else
        gemv_packed_finalize_body<kPackMaxSlices>(partial, scale, y, N, S);
}
struct FinalizeArgs {
    const float *partial;
    const half_t *scale;
    half_t *y;
    int N, S;
};
struct FinalizeBatch {
    FinalizeArgs a[kPackMaxBatch];
};
__global__ __launch_bounds__(kFinalizeRows) void gemv_packed_finalize_batch_kernel(FinalizeBatch b) {
    FinalizeArgs a = b.a[blockIdx.y];
    pin_scalar(a.partial); pin_scalar(a.scale); pin_scalar(a.y); pin_scalar(a.N); pin_scalar(a.S);
    if (a.S <= 32)
        gemv_packed_finalize_body<32>(a.partial, a.scale, a.y, a.N, a.S);
    else
        gemv_packed_finalize_body<kPackMaxSlices>(a.partial, a.scale, a.y, a.N, a.S);
}

bool gemv_uses_pack(const vq_weight_t *w, int bs) {
    return w->gemv_pack != nullptr && bs == 1 && pack_supported(w);
}

size_t gemv_packed_workspace(const vq_weight_t *w) {
    return (size_t)w->gemv_pack->S * w->N * sizeof(float);
}

int check_pack(const vq_weight_t *w) {
    const vq_gemv_pack_t *p = w->gemv_pack;
    if (!p->data) return VQ_ERR_NULL;
    if (!aligned16(p->data)) return VQ_ERR_ALIGN;
    if (!pack_supported(w)) return VQ_ERR_UNSUPPORTED;
    PackPlan plan = pack_plan(w);
    if (p->S != plan.S || p->RB != plan.RB || p->rows_per_block != plan.rows_per_block) return VQ_ERR_SHAPE;
    if (p->S > (uint32_t)kPackMaxSlices) return VQ_ERR_UNSUPPORTED;
    // every address the kernel derives from the descriptor must lie inside the buffer
    const uint64_t ng = (plan.rows_per_block + 63) / 64, nwg = (uint64_t)p->S * p->RB;
    if (ng > VQ_PACK_MAX_GROUPS) return VQ_ERR_SHAPE;
    uint64_t sum = 0;
    for (uint64_t g = 0; g < ng; ++g) sum += p->group_steps[g];
    if (sum != p->wg_pitch || sum > 65535 || sum == 0) return VQ_ERR_SHAPE;
    if (p->rowid_off + nwg * ng * 128 > p->atom_off || p->atom_off + (nwg * sum + kPackTailBlocks) * 768 > p->bytes)
        return VQ_ERR_SHAPE;
    if ((p->rowid_off & 1) || (p->atom_off & 3)) return VQ_ERR_ALIGN;
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
    PackPlan plan = pack_plan(w);
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
    a.slice_entries = (int)plan.slice_entries;
    a.rowid_off = p->rowid_off;
    a.atom_off = p->atom_off;
    a.wg_pitch = p->wg_pitch;
    {
        unsigned at = 0;
        for (int g = 0; g < VQ_PACK_MAX_GROUPS; ++g) {
            a.group[g] = (at << 16) | p->group_steps[g];
            at += p->group_steps[g];
        }
    }
    int groups_per_wg = (int)((p->rows_per_block + 63) / 64);
    l.lds = ((size_t)plan.slice_entries + (size_t)a.J + 1) * 16 + (size_t)groups_per_wg * 64 * sizeof(float);
    // every wavefront the same number of groups (the first, longest ones are dealt first, one to each)
    const int rounds = (groups_per_wg + 15) / 16;
    l.waves = (groups_per_wg + rounds - 1) / rounds;
    if (l.waves < 8) l.waves = 8;   // at least 512 threads, so that slice and x are staged with many loads in flight
    a.nwaves = l.waves;
    l.grid = (int)(p->S * p->RB);
    return l;
}


}  // namespace

int launch_gemv_packed(const vq_weight_t *w, const void *x, void *y, void *ws, hipStream_t s) {
    PackedLaunch l = packed_launch(w, x, y, ws);
    static KernelSetup setup;   // (the atoms hold absolute LDS addresses: no static LDS allowed)
    if (int st = kernel_setup(reinterpret_cast<const void *>(&gemv_packed_kernel), l.lds, true, setup)) return st;
    gemv_packed_kernel<<<l.grid, l.waves * 64, l.lds, s>>>(l.a);
    gemv_packed_finalize_kernel<<<(l.a.N + kFinalizeRows - 1) / kFinalizeRows, kFinalizeRows, 0, s>>>(l.a.partial, l.a.scale, l.a.y, l.a.N, l.a.S);
    return launch_status();
}

// Partial sums of the problems of a batch lie back to back in the workspace, each 256-byte aligned.
size_t gemv_packed_batch_workspace(const vq_weight_t *const *w, int count) {
    size_t total = 0;
    for (int i = 0; i < count; ++i) total += (gemv_packed_workspace(w[i]) + 255) & ~(size_t)255;
    return total;
}

int launch_gemv_packed_batch(const vq_weight_t *const *w, const void *const *x, void *const *y, int count, void *ws,
                             hipStream_t s) {
    PackedBatch b;
    int grid = 0, waves = 0, max_n = 0;
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
            max_n = l.a.N > max_n ? l.a.N : max_n;
        }
    }
    static KernelSetup setup;
    if (int st = kernel_setup(reinterpret_cast<const void *>(&gemv_packed_batch_kernel), lds, true, setup)) return st;
    for (int i = 0; i < kPackMaxBatch; ++i) b.a[i].nwaves = waves;  // one launch shape for all problems
    gemv_packed_batch_kernel<<<dim3(grid, count), waves * 64, lds, s>>>(b);
    FinalizeBatch f;
    for (int i = 0; i < kPackMaxBatch; ++i) f.a[i] = {b.a[i].partial, b.a[i].scale, b.a[i].y, b.a[i].N, b.a[i].S};
    gemv_packed_finalize_batch_kernel<<<dim3((max_n + kFinalizeRows - 1) / kFinalizeRows, count), kFinalizeRows, 0, s>>>(f);
    return launch_status();
}

}  // namespace vq

using namespace vq;

extern "C" {

size_t vq_gemv_prepack_bytes(const vq_weight_t *w) {
    if (!w || !w->codes || !pack_supported(w)) return 0;
    return (size_t)pack_build(w, nullptr, nullptr);
}

int vq_gemv_prepack(const vq_weight_t *w, void *out_host, size_t out_bytes, vq_gemv_pack_t *pack) {
    if (!w || !w->codes || !out_host || !pack) return VQ_ERR_NULL;
    if (w->v != 8 && w->v != 4) return VQ_ERR_UNSUPPORTED;
    if (!pack_supported(w)) return VQ_ERR_UNSUPPORTED;
    if (!aligned16(out_host)) return VQ_ERR_ALIGN;
    uint64_t need = pack_build(w, nullptr, nullptr);
    if (out_bytes < need) return VQ_ERR_WORKSPACE;
    pack_build(w, (unsigned char *)out_host, pack);
    return VQ_OK;
}

}  // extern "C"
