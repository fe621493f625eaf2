"""Compile-time invariants of hand-scheduled kernels, checked on the compiler's own output (no GPU).

The re-tiled gemv lets its gathers start when the codebook slice has landed while the atoms still stream in:
a counted ``s_waitcnt vmcnt(AHEAD + 1)`` stands between the loads and the barrier.  That is only right if, in every
build of the kernel, at least AHEAD + 1 ordinary vector loads are issued between the last direct-to-LDS transfer
and that wait, in straight-line code (loads complete in issue order)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2503_02236_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_gemv_packed_counted_wait_matches_the_loads_in_front_of_it(tmp_path):
    """Order of a wavefront's vector memory instructions in front of the barrier, in every build of the kernel:
    staging transfers (slice, x) | trip count, task slots, AHEAD atom loads | [the pending block of the previous
    launch: 4 transfers, 4 more when it has more than 16 slices] | scale.  The barrier may open when the staging
    transfers have landed, i.e. when at most AHEAD + 2 (+ 4, + 8) younger instructions are pending: three counted
    waits, one per case.  Loads complete in issue order, so that is right iff the counts match the code."""
    out = tmp_path / "gemv_packed.s"
    cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only", "-S",
           os.path.join(CSRC, "gemv_packed.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    text = out.read_text()
    ahead = int(re.search(r"constexpr int kPackAhead = (\d+);", open(os.path.join(CSRC, "gemv_packed.hip")).read()).group(1))
    is_load = lambda l: re.match(r"global_load_(dword|ushort|ubyte|short)", l) is not None
    is_dma = lambda l: l.startswith("global_load_lds")
    is_flow = lambda l: l.startswith(("s_cbranch", "s_branch")) or l.endswith(":")
    checked = 0
    for name in ("gemv_packed_kernel", "gemv_packed_batch_kernel"):
        m = re.search(r"^(_ZN2vq\d+%sE\w*):[^\n]*\n(.*?)^\.Lfunc_end" % name, text, re.S | re.M)
        assert m, name
        lines = [l.strip() for l in m.group(2).splitlines()]
        barrier = lines.index("s_barrier")
        head = lines[:barrier]
        waits = {c: [i for i, l in enumerate(head) if l == "s_waitcnt vmcnt(%d) lgkmcnt(0)" % c and "ASMSTART" in head[i - 1]]
                 for c in (ahead + 2, ahead + 6, ahead + 10)}
        assert all(len(v) == 1 for v in waits.values()), (name, waits)
        first_wait = min(v[0] for v in waits.values())
        atoms = [i for i, l in enumerate(head[:first_wait]) if l.startswith("global_load_dwordx2")]
        assert len(atoms) == ahead, (name, atoms)
        staging = [i for i in range(atoms[0]) if is_dma(head[i])]
        assert staging and all(head[i].startswith("global_load_lds_dwordx4") for i in staging), name
        # between the last staging transfer and the first atom load: trip count and task slots, straight-line
        mid = head[staging[-1] + 1:atoms[0]]
        assert sum(is_load(l) for l in mid) == 2, (name, mid)
        first_mid_load = next(i for i, l in enumerate(mid) if is_load(l))
        assert not any(is_flow(l) for l in mid[first_mid_load:]), name
        assert not any(is_flow(l) or is_dma(l) for l in head[atoms[0]:atoms[-1] + 1]), name
        # behind the atoms: the pending block (two groups of four transfers, nothing else that counts), then the scale
        tail = head[atoms[-1] + 1:first_wait]
        dmas = [i for i, l in enumerate(tail) if is_dma(l)]
        assert len(dmas) == 8 and all(tail[i].startswith("global_load_lds_dwordx4") for i in dmas), (name, dmas)
        assert dmas[3] == dmas[0] + 3 and dmas[7] == dmas[4] + 3                   # each group in one statement
        assert any(is_flow(l) for l in tail[dmas[3] + 1:dmas[4]])                  # the second group can be skipped
        loads = [i for i, l in enumerate(tail) if is_load(l)]
        assert len(loads) == 1 and loads[0] > dmas[-1], (name, loads)               # the scale, outside the condition
        assert tail[loads[0]].startswith("global_load_ushort")
        checked += 1
        # the atoms hold absolute LDS addresses of the dynamic region: it must start at 0, i.e. no static LDS
        k = re.search(r"\.amdhsa_kernel (_ZN2vq\d+%sE\w*)\n(.*?)\.end_amdhsa_kernel" % name, text, re.S)
        assert k, name
        assert re.search(r"\.amdhsa_group_segment_fixed_size 0\b", k.group(2)), name
    assert checked == 2


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_gemm_dense_ring_wait_matches_the_transfers_of_a_stage(tmp_path):
    """The dense gemm stage waits with ``s_waitcnt vmcnt(12)`` for the older of two stages in flight: right only
    if a stage is exactly twelve direct-to-LDS transfers per wavefront and the main loop issues no other vector
    memory instruction."""
    out = tmp_path / "gemm_dense.s"
    cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only", "-S",
           os.path.join(CSRC, "gemm_dense.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    lines = [l.strip() for l in out.read_text().splitlines()]
    # the main loop: from the loop-head wait to the backward branch
    heads = [i for i, l in enumerate(lines) if l == "s_waitcnt vmcnt(12) lgkmcnt(0)"]
    assert heads, "counted wait not found"
    h = heads[0]
    assert lines[h + 1] == "s_barrier"
    end = next(i for i in range(h, len(lines)) if lines[i].startswith("s_cbranch"))
    body = lines[h:end]
    assert sum(l.startswith("global_load_lds_dwordx4") for l in body) == 12
    assert not any(re.match(r"(global|flat|buffer)_(load|store)", l) and not l.startswith("global_load_lds") for l in body)
    assert sum(l.startswith("v_mfma_f32_32x32x16") for l in body) == 32


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_attention_kernels_have_no_static_lds(tmp_path):
    """The attention kernel forms entry addresses as absolute LDS offsets, which needs its dynamic LDS to start
    at address 0, i.e. no static LDS in any build of it (the launcher checks the same at run time and returns
    an error instead of launching)."""
    out = tmp_path / "attn.s"
    cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only", "-S",
           os.path.join(CSRC, "attn.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    kernels = re.findall(r"\.amdhsa_kernel (\S*attn_decode_kernel\S*)\n(.*?)\.end_amdhsa_kernel", out.read_text(), re.S)
    assert len(kernels) >= 6            # v = 2, 4, 8 x one / several codebooks (x one or two sequences)
    for name, body in kernels:
        assert re.search(r"\.amdhsa_group_segment_fixed_size 0\b", body), name


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_gemv_replica_gathers_form_one_block_and_nothing_lives_in_scratch(tmp_path):
    """The small-codebook list kernel forms absolute LDS addresses (no static LDS allowed), reads its problem list
    with scalar loads (a by-value list indexed with a register would move to scratch memory: none allowed), and issues
    the gathers of an item as asm in blocks, each followed by a full LDS wait that names the block's destinations: no
    instruction reads a gathered register before such a wait."""
    out = tmp_path / "gemv_replica.s"
    cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only", "-S",
           os.path.join(CSRC, "gemv_replica.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    text = out.read_text()
    checked = 0
    for R in (1, 2):
        name = r"_ZN2vq25gemv_replica_table_kernelILi%dEE\w*" % R
        k = re.search(r"\.amdhsa_kernel (%s)\n(.*?)\.end_amdhsa_kernel" % name, text, re.S)
        assert k, R
        assert re.search(r"\.amdhsa_group_segment_fixed_size 0\b", k.group(2)), R
        assert re.search(r"\.amdhsa_private_segment_fixed_size 0\b", k.group(2)), R
        m = re.search(r"^(%s):[^\n]*\n(.*?)^\.Lfunc_end" % name, text, re.S | re.M)
        assert m, R
        lines = [l.strip() for l in m.group(2).splitlines()]
        lines = [l for l in lines if l and not l.startswith(";")]
        assert not any(l.startswith("scratch_") for l in lines), R
        # Every 16-byte LDS read is waited for (a full LDS wait) before the first instruction that names one of its
        # destination registers -- the compiler may move the second block's gathers in between the first block's
        # matrix instructions, but never a use in front of the wait.
        def regs(text):
            out = set()
            for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
                if m.group(3) is not None:
                    out.add(int(m.group(3)))
                else:
                    out.update(range(int(m.group(1)), int(m.group(2)) + 1))
            return out
        gathers = 0
        for i, l in enumerate(lines):
            if not l.startswith("ds_read_b128"):
                continue
            dst = regs(l.split(",")[0])
            waited = False
            for m in lines[i + 1:i + 600]:
                if m.startswith("s_waitcnt") and "lgkmcnt(0)" in m:
                    waited = True
                    break
                assert not (regs(m) & dst), (R, i, l, m)
            assert waited, (R, i, l)
            gathers += 1
        n_mfma = sum(l.startswith("v_mfma_f32_4x4x4") for l in lines)
        assert n_mfma >= 3 * 16 * R and n_mfma % (16 * R) == 0, (R, n_mfma)      # whole items: 16 R per item
        assert gathers >= n_mfma // 2, (R, gathers, n_mfma)                        # a gather per two of them (+ x reads)
        checked += 1
    assert checked == 2
