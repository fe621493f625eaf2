"""Host-side checks of vq_gemv_prepack (no GPU): the re-tiled buffer is decoded here, by a decoder
written from the format description alone, and must reproduce the canonical codes exactly."""
import ctypes
import time

import numpy as np
import pytest

import paper_2503_02236_amd as vq
from paper_2503_02236_amd import workloads as wl
from paper_2503_02236_amd.binding import vq_gemv_pack_t, vq_weight_t

ATOM_BITS = 21
ZERO_UNITS = 16
_HALF = [[0, 1, 2, 3, 12, 13, 14, 15, 20, 21, 22, 23, 24, 25, 26, 27], [4, 5, 6, 7, 8, 9, 10, 11, 16, 17, 18, 19, 28, 29, 30, 31]]
PASS_LANES = [np.array(g) for g in _HALF] + [np.array(g) + 32 for g in _HALF]


def decode(buf, pack, N, J):
    """Packed buffer -> (codes[N][J], hits[N][J], stats), following the documented layout:
    task table [S*RB][G][64] uint16, step table [S*RB][G] uint32, atom blocks of 64 step words of 64 bits
    (three 21-bit atoms each: entry index in the low entry_bits bits, position inside the part above)."""
    S, RB, RPB = pack.S, pack.RB, pack.rows_per_block
    EB, P, JP = pack.entry_bits, pack.parts, pack.part_cols
    XB = ATOM_BITS - EB
    slice_entries = 1 << EB
    assert JP + ZERO_UNITS <= (1 << XB) and P * JP >= J and (P - 1) * JP < max(J, 1)
    tasks_per_wg = RPB * P
    G = (tasks_per_wg + 63) // 64
    common = [int(pack.group_steps[g]) for g in range(G)]
    assert sum(common) == pack.wg_pitch and all(int(pack.group_steps[g]) == 0 for g in range(G, 128))
    prefix = np.concatenate([[0], np.cumsum(common)])
    nwg = S * RB
    slots = np.frombuffer(buf, dtype=np.uint16, count=64 * G * nwg, offset=pack.task_off).reshape(nwg, G, 64)
    own = np.frombuffer(buf, dtype=np.uint32, count=G * nwg, offset=pack.steps_off).reshape(nwg, G)
    assert pack.task_off % 256 == 0 and pack.steps_off % 256 == 0 and pack.atom_off % 256 == 0
    assert pack.task_off + slots.nbytes <= pack.steps_off and pack.steps_off + own.nbytes <= pack.atom_off
    words = np.frombuffer(buf, dtype=np.uint64, offset=pack.atom_off)
    assert words.size == (nwg * pack.wg_pitch + 16) * 64          # 16 blocks of padding behind the last workgroup's
    assert (own <= np.array(common)[None, :]).all()
    assert (own.max(axis=0) == np.maximum(np.array(common), 0))[1:].all()   # the common shape is the maximum
    mask = (1 << ATOM_BITS) - 1

    def atoms_of(w64):
        """[..., 3] atoms of step words"""
        assert ((w64 >> np.uint64(63)) == 0).all()
        return np.stack([(w64 >> np.uint64(ATOM_BITS * k)) & np.uint64(mask) for k in range(3)], axis=-1).astype(np.int64)

    # everything outside the groups' own steps is padding: any entry, a zero unit of the part as position
    codes = np.zeros((N, J), dtype=np.int64)
    hits = np.zeros((N, J), dtype=np.int32)
    real_atoms = pad_atoms = 0
    conflict_passes = 0       # LDS passes per (16 lanes, position) under the column model, entry + x
    positions = 0
    seen_slots = np.zeros((nwg, tasks_per_wg), dtype=np.int32)
    for w in range(nwg):
        s, rb = divmod(w, RB)
        rows_here = max(0, min(RPB, N - rb * RPB))
        prev_len = None
        blk0 = w * pack.wg_pitch
        wg_words = words[blk0 * 64:(blk0 + pack.wg_pitch) * 64].reshape(pack.wg_pitch, 64)
        for g in range(G):
            st = int(own[w, g])
            a = atoms_of(wg_words[prefix[g]:prefix[g] + st])              # [st][64][3]
            rest = atoms_of(wg_words[prefix[g] + st:prefix[g] + common[g]])
            assert ((rest >> EB) >= JP).all() and ((rest >> EB) < JP + ZERO_UNITS).all()
            lists = a.transpose(1, 0, 2).reshape(64, st * 3)              # lane-major: order of the additions
            e, x = lists & (slice_entries - 1), lists >> EB
            if st:   # padding atoms name entries that codes of the same group use, never an unused one
                assert np.isin(e[x >= JP], e[x < JP]).all()
            assert (x < JP + ZERO_UNITS).all()
            part = np.zeros(64, dtype=np.int64)
            for lane in range(64):
                slot = int(slots[w, g, lane])
                valid = x[lane] < JP
                n_valid = int(valid.sum())
                if slot == 0xFFFF:
                    assert n_valid == 0
                    continue
                p_, r_ = divmod(slot, RPB)
                part[lane] = p_
                assert p_ < P and r_ < rows_here
                seen_slots[w, slot] += 1
                if prev_len is not None:
                    assert n_valid <= prev_len                               # tasks sorted by length inside a workgroup
                prev_len = n_valid
                n = rb * RPB + r_
                js = p_ * JP + x[lane][valid]
                assert (js < J).all() and len(np.unique(js)) == n_valid
                codes[n, js] = s * slice_entries + e[lane][valid]
                hits[n, js] += 1
                real_atoms += n_valid
                pad_atoms += st * 3 - n_valid
            if st:
                assert st == -(-max(int((x[l] < JP).sum()) for l in range(64)) // 3)   # as long as its longest task
                # bank model: the 16-byte reads of these sets of 16 lanes are served together; passes = max
                # multiplicity of a 16-byte column inside a set
                unit_x = slice_entries + part[:, None] * (JP + ZERO_UNITS) + x
                for lanes in PASS_LANES:
                    for col in (e[lanes] % 16, unit_x[lanes] % 16):
                        onehot = (col[:, :, None] == np.arange(16)[None, None, :]).sum(axis=0)   # [pos][16]
                        conflict_passes += int(onehot.max(axis=1).sum())
                    positions += 2 * st * 3
        assert (seen_slots[w, [p_ * RPB + r_ for p_ in range(P) for r_ in range(rows_here)]] == 1).all()
    tail = atoms_of(words[nwg * pack.wg_pitch * 64:])
    assert ((tail >> EB) >= JP).all() and ((tail >> EB) < JP + ZERO_UNITS).all()
    read_bytes = int(own.sum()) * 512 + slots.nbytes + own.nbytes
    return codes, hits, dict(real=real_atoms, pad=pad_atoms, passes=conflict_passes / max(positions, 1),
                             read_bytes=read_bytes)


@pytest.mark.parametrize("N,K,E", [
    (200, 1024, 65536),
    (64, 512, 4096),
    (513, 2048, 65536),
    (1, 64, 65536),
    (70, 16368, 8192),       # long rows: three parts
    (40, 11008, 65536),      # two parts of 688 positions
    (9000, 64, 65536),       # many rows: 18 groups per workgroup
    (20000, 64, 65536),      # 40 groups per workgroup
])
def test_prepack_round_trip(N, K, E):
    w = wl.make_weight(N, K, 8, 16, 1, E, 0.02, seed=77 + N)
    buf, pack = vq.vq_gemv_prepack(w)
    assert buf is not None and pack.bytes == buf.size
    assert pack.S == E // 2048 and pack.S * pack.RB <= 256 and pack.entry_bits == 11
    assert pack.parts == -(-(K // 8) // 1008)
    codes, hits, _ = decode(buf, pack, N, K // 8)
    assert (hits == 1).all()                       # every code appears exactly once
    assert np.array_equal(codes, w.codes[:, :, 0].astype(np.int64))


def test_prepack_declines_uneven_codes():
    """Skewed codes: the slices' loads differ so much that one common workgroup shape would be mostly padding."""
    w = wl.make_weight(513, 2048, 8, 16, 1, 65536, 0.02, seed=590, zipf_s=1.0)
    assert vq.vq_gemv_prepack(w) == (None, None)


def test_prepack_is_deterministic_and_rejects_other_formats():
    w = wl.make_weight(128, 512, 8, 16, 1, 65536, 0.02, seed=5)
    b1, _ = vq.vq_gemv_prepack(w)
    b2, _ = vq.vq_gemv_prepack(w)
    assert np.array_equal(b1, b2)
    for bad in (wl.make_weight(64, 512, 8, 8, 1, 256, 0.02, seed=6),       # uint8 codes
                wl.make_weight(64, 512, 4, 16, 1, 65536, 0.02, seed=6),    # v = 4
                wl.make_weight(64, 512, 8, 16, 2, 4096, 0.02, seed=6),     # two codebooks
                wl.make_weight(64, 512, 8, 16, 1, 1000, 0.02, seed=6),     # E not a power of two
                wl.make_weight(8, 65536, 8, 16, 1, 65536, 0.02, seed=6)):  # rows too long: more than eight parts
        assert vq.vq_gemv_prepack(bad) == (None, None)


def test_prepack_rejects_codes_beyond_the_codebook():
    """A code >= n_entries would index past the packer's tables: it is reported, not assumed away."""
    w = wl.make_weight(64, 512, 8, 16, 1, 4096, 0.02, seed=8)
    codes = np.ascontiguousarray(w.codes).copy()
    codes[17, 3, 0] = 4096
    d = vq_weight_t(w.N, w.K, 8, 16, 1, 4096, codes.ctypes.data, None, None, None)
    lib = vq.lib()
    assert lib.vq_gemv_prepack_bytes(ctypes.byref(d)) == 0
    out = np.empty(1 << 20, dtype=np.uint8)
    off = (-out.ctypes.data) % 16
    pack = vq_gemv_pack_t()
    assert lib.vq_gemv_prepack(ctypes.byref(d), out.ctypes.data + off, out.size - off, ctypes.byref(pack)) == -2


def test_prepack_llama_shape_size_order_and_speed():
    w = wl.config2_layer(0)                        # (4096, 4096)
    t0 = time.time()
    buf, pack = vq.vq_gemv_prepack(w)
    dt = time.time() - t0
    codes, hits, st = decode(buf, pack, w.N, w.K // 8)
    assert (hits == 1).all() and np.array_equal(codes, w.codes[:, :, 0].astype(np.int64))
    ratio = st["read_bytes"] / w.codes.nbytes
    print(f"prepack 4096x4096: {dt:.2f} s, {buf.size / 2**20:.1f} MiB allocated, {st['read_bytes'] / 2**20:.1f} MiB read per "
          f"product = {ratio:.3f} x canonical codes; padding {st['pad'] / st['real']:.3f}; LDS passes per 16 lanes "
          f"and gather {st['passes']:.2f}")
    assert (pack.S, pack.RB, pack.parts) == (32, 8, 1)      # 2048-entry slices, 8 groups per workgroup
    assert 1.3 <= ratio < 1.7                      # 64 bits per three codes, tasks padded to their group's length
    # the offline order of the atoms: 16 lanes with random addresses need ~2.9 passes per gather
    assert st["passes"] < 1.9
