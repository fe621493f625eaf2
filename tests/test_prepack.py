"""Host-side checks of vq_gemv_prepack (no GPU): the re-tiled buffer is decoded here, by a decoder
written from the format description alone, and must reproduce the canonical codes exactly."""
import time

import numpy as np
import pytest

import paper_2503_02236_amd as vq
from paper_2503_02236_amd import workloads as wl



def decode(buf, pack, N, J, SLICE):
    """Packed buffer -> codes[N][J] plus per-position hit counts, following the documented layout."""
    S, RB, RPB = pack.S, pack.RB, pack.rows_per_block
    ng = (RPB + 63) // 64
    steps = [int(pack.group_steps[g]) for g in range(ng)]
    assert sum(steps) == pack.wg_pitch and all(int(pack.group_steps[g]) == 0 for g in range(ng, 128))
    prefix = np.concatenate([[0], np.cumsum(steps)])
    rowids = np.frombuffer(buf, dtype=np.uint16, count=64 * ng * S * RB, offset=pack.rowid_off).reshape(S * RB, ng, 64)
    atoms = np.frombuffer(buf, dtype=np.uint8, offset=pack.atom_off)
    assert atoms.size == (S * RB * pack.wg_pitch + 16) * 768          # 16 blocks of padding behind the last workgroup's
    # an atom = two 12-bit numbers of 16-byte units in the LDS image [slice][x][zero unit]; padding names the zero unit twice
    zero_unit = SLICE + J
    assert zero_unit < 4096
    pad = zero_unit | (zero_unit << 12)
    tail = atoms[S * RB * pack.wg_pitch * 768:].reshape(-1, 3).astype(np.uint32)
    assert ((tail[:, 0] | (tail[:, 1] << 8) | (tail[:, 2] << 16)) == pad).all()
    codes = np.zeros((N, J), dtype=np.int64)
    hits = np.zeros((N, J), dtype=np.int32)
    for w in range(S * RB):
        s, rb = divmod(w, RB)
        prev_len = None
        for g in range(ng):
            blk = w * pack.wg_pitch + int(prefix[g])
            a = atoms[blk * 768:(blk + steps[g]) * 768].reshape(steps[g], 64, 4, 3).astype(np.uint32)
            val = a[..., 0] | (a[..., 1] << 8) | (a[..., 2] << 16)          # [steps][lane][4]
            val = val.transpose(1, 0, 2).reshape(64, steps[g] * 4)          # lane-major atom lists
            for lane in range(64):
                ri = int(rowids[w, g, lane])
                lst = val[lane]
                valid = lst != pad
                n_valid = int(valid.sum())
                assert valid[:n_valid].all()                                       # real atoms first, then padding
                assert ((lst[:n_valid] & 0xFFF) < SLICE).all() and ((lst[:n_valid] >> 12) >= SLICE).all()
                if ri == 0xFFFF:
                    assert n_valid == 0
                    continue
                if prev_len is not None:
                    assert n_valid <= prev_len                               # rows sorted by length inside a workgroup
                prev_len = n_valid
                n = rb * RPB + ri
                assert ri < RPB and n < N
                js = (lst[:n_valid] >> 12) - SLICE
                assert (js < J).all()
                assert (np.diff(js.astype(np.int64)) > 0).all()                # ascending positions: fixed summation order
                codes[n, js] = s * SLICE + (lst[:n_valid] & 0xFFF)
                hits[n, js] += 1
    return codes, hits


@pytest.mark.parametrize("N,K,E", [
    (200, 1024, 65536),
    (64, 512, 4096),
    (513, 2048, 65536),
    (1, 64, 65536),
    (70, 16368, 8192),       # longest supported rows (K/8 = 2046)
    (9000, 64, 65536),       # many rows: 18 groups per workgroup
    (20000, 64, 65536),      # 20 groups per workgroup
])
def test_prepack_round_trip(N, K, E):
    w = wl.make_weight(N, K, 8, 16, 1, E, 0.02, seed=77 + N)
    buf, pack = vq.vq_gemv_prepack(w)
    assert buf is not None and pack.bytes == buf.size
    assert pack.S == E // 2048 and pack.S * pack.RB <= 256
    codes, hits = decode(buf, pack, N, K // 8, E // pack.S)
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
                wl.make_weight(8, 16384, 8, 16, 1, 65536, 0.02, seed=6)):  # rows too long for the position field
        assert vq.vq_gemv_prepack(bad) == (None, None)


def test_prepack_llama_shape_size_and_speed():
    w = wl.config2_layer(1)                        # (11008, 4096)
    t0 = time.time()
    buf, pack = vq.vq_gemv_prepack(w)
    dt = time.time() - t0
    ratio = buf.size / w.codes.nbytes
    print(f"prepack 11008x4096: {dt:.2f} s, {buf.size / 2**20:.1f} MiB = {ratio:.3f} x canonical codes")
    assert (pack.S, pack.RB) == (32, 8)                # 2048-entry slices, 22 groups per workgroup
    assert 1.5 <= ratio < 1.9                      # 3 bytes per code plus padding to whole 4-atom steps and to the common shape
