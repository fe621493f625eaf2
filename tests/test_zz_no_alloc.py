"""vq_gemv_noalloc (the entry point for callers that cannot allocate) against vq_gemv, through the C ABI.

Same kernels, scratch inside the library instead of a caller's workspace: results must be identical bit for
bit, on two calls in a row that share the scratch, the second with a smaller problem."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2503_02236_amd as vq
from paper_2503_02236_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_gemv_noalloc_matches_gemv_on_two_calls_in_a_row(gpu_device):
    lib = vq.lib()
    assert lib.vq_init() == 0
    cases = [wl.make_weight(1000, 4096, 8, 16, 1, 65536, 0.02, seed=8800),   # 32 slices x 1000 rows of partial sums
             wl.make_weight(300, 2048, 8, 16, 1, 4096, 0.02, seed=8801)]     # smaller: two slices, part of the scratch
    results = []
    for i, w in enumerate(cases):
        print(f"case {i}: {w.N}x{w.K} E={w.codebooks.shape[1]}", flush=True)
        wd = vq.weight_to_device(w, gpu_device, prepack=True, keep_codes=False)
        x = wl.make_activations(1, w.K, seed=8810 + i)
        xd = torch.from_numpy(x).to(gpu_device)
        assert 0 < vq.vq_gemv_workspace(wd, 1) <= lib.vq_gemv_noalloc_max_workspace()
        y = torch.full((1, w.N), 7.0, dtype=torch.float16, device=gpu_device)
        vq.vq_gemv_noalloc(wd, xd, y)
        results.append((w, wd, x, xd, y))
    torch.cuda.synchronize()
    for w, wd, x, xd, y in results:
        want = vq.vq_gemv(wd, xd)                       # the existing entry point, workspace from the caller
        torch.cuda.synchronize()
        assert torch.equal(y, want)
        ref = oracle.gemv(w.codes, w.codebooks, w.scale, x)
        got = y.float().cpu().numpy().astype(np.float64)
        assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 2e-3
        assert np.abs(got - ref).max() <= 1e-2 * np.sqrt(np.mean(ref ** 2))


def test_gemv_noalloc_without_scratch_and_beyond_its_size(gpu_device):
    lib = vq.lib()
    # codebooks in LDS: no scratch is used at all
    w = wl.config3_layer(0)
    wd = vq.weight_to_device(w, gpu_device)
    xd = torch.from_numpy(wl.make_activations(4, w.K, seed=8820)).to(gpu_device)
    y = torch.empty((4, w.N), dtype=torch.float16, device=gpu_device)
    vq.vq_gemv_noalloc(wd, xd, y)
    torch.cuda.synchronize()
    assert torch.equal(y, vq.vq_gemv(wd, xd))
    # more partial sums than the built-in scratch holds: refused, nothing launched, y untouched
    big = wl.make_weight(20000, 128, 8, 16, 1, 65536, 0.02, seed=8830)
    bd = vq.weight_to_device(big, gpu_device, prepack=True, keep_codes=False)
    assert vq.vq_gemv_workspace(bd, 1) > lib.vq_gemv_noalloc_max_workspace()
    xb = torch.from_numpy(wl.make_activations(1, 128, seed=8831)).to(gpu_device)
    yb = torch.full((1, 20000), 3.0, dtype=torch.float16, device=gpu_device)
    with pytest.raises(vq.VQError) as e:
        vq.vq_gemv_noalloc(bd, xb, yb)
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert (yb == 3).all()
