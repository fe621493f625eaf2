#!/usr/bin/env python3
"""Benchmark of the fused VQ hot path on one MI355X.

Headline workload (N = 1 GPU): Llama-7B-shaped decode VQ-gemv, bs = 1, one 2^16 x 8 fp16
codebook per matrix, uint16 codes, fp16 per-channel scale.  One "step" is one decode token's
worth of linear layers of the whole 32-block stack: 224 matrices (4 x (4096,4096),
2 x (11008,4096), 1 x (4096,11008) per block) in 128 launches -- the projections of a block that share
their input go through vq_gemv_batch (query/key/value; gate/up), the other two through vq_gemv;
`--no-batch` gives one vq_gemv per matrix -- every matrix with its own codes and codebook
(1.5 GiB + 224 MiB, far beyond the 256 MB last-level cache, so every launch streams from HBM).
All inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is effective bandwidth: algorithmic bytes (codes + codebook
once + x + scale + y) per step divided by the step time.  Secondary objects report the
per-shape gemv times, the prefill VQ-gemm (M = 2048) against the fp16 MFMA peak and the
VQ-attn decode against HBM, each timed outside the headline region.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, vendor figure
MFMA_FP16_PEAK_TFLOPS = 2500.0  # dense fp16 matrix-core peak, vendor figure


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps first; the default is long enough for the clocks to settle (a GPU that comes "
                         "from idle runs its first few launches fast, the next dozen slow, and levels out after that)")
    ap.add_argument("--layers", type=int, default=32, help="decoder blocks in the gemv stack")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a HIP graph replay")
    ap.add_argument("--skip-secondary", action="store_true", help="only the headline gemv stack")
    ap.add_argument("--skip-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--canonical", action="store_true",
                    help="headline gemv from the canonical code layout (L2 gathers) instead of the re-tiled codes")
    ap.add_argument("--no-batch", action="store_true",
                    help="one vq_gemv call per matrix (224 launches) instead of vq_gemv_batch for the projections of "
                         "a block that share their input (query/key/value; gate/up)")
    ap.add_argument("--no-sequence", action="store_true",
                    help="separate vq_gemv_batch / vq_gemv calls (two launches each: product and its reduction) instead "
                         "of one vq_gemv_sequence over the stack (the reduction rides along in the next launch)")
    ap.add_argument("--mode", choices=["pipeline", "streams"], default="pipeline",
                    help="how the stack is issued: 'pipeline' = vq_gemv_pipeline (one persistent launch for all matrices "
                         "plus one reduction launch), 'streams' = vq_gemv_sequence_streams (one launch per call)")
    ap.add_argument("--streams", type=int, default=4,
                    help="HIP streams the sequence is spread over (vq_gemv_sequence_streams; 1 = vq_gemv_sequence)")
    ap.add_argument("--only", default="", help="comma list of sections for profiling runs: gemv,gemm,attn,add,zipf,tile,bit12")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="counter run (wrap in rocprofv3 --pmc FETCH_SIZE or WRITE_SIZE): three plain copies of "
                         "known size as calibration, then one eager pass over the headline gemv stack; no timing")
    ap.add_argument("--pmc-probe-additive", action="store_true",
                    help="counter run like --pmc-probe, over the additive-codebook (2 x 256 x 8) decoder stack through "
                         "vq_gemv_pipeline (one launch)")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "gemv_pipeline_c2_hbm_traffic.md"),
                    help="summary written by paper_2503_02236_amd.profile_summary traffic; its "
                         "'traffic_bytes_per_launch:' line fills roofline.traffic")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding)"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2503_02236_amd as vq
    from paper_2503_02236_amd import workloads as wl
    from paper_2503_02236_amd.binding import _stream

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    lib = vq.lib()
    only = set(s for s in args.only.split(",") if s)

    def want(section):
        return not only or section in only

    def timed_once(fn, iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def timed(fn, iters, warm):
        """Average ms per call of fn() over back-to-back calls, HIP events on the launch stream: at least `iters`
        calls, and as many as it takes to time about 60 ms of GPU work after as much untimed work (steady clocks:
        a GPU that comes from idle runs its first launches fast and the next ones slow before it levels out)."""
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        ms = timed_once(fn, iters)
        if ms < 60.0 and not args.pmc_probe:
            n = min(max(iters, int(iters * 60.0 / max(ms, 1e-3)) + 1), 5000)
            timed_once(fn, n)
            return timed_once(fn, n) / n
        return ms / iters

    def timed_replay(fn, iters, warm):
        """Like timed(), with fn() captured once into a HIP graph and replayed (as the headline stack is timed):
        the host's launch rate stays out of the figure.  Eager with --no-graph."""
        if args.no_graph:
            return timed(fn, iters, warm)
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                fn()
        ms = timed(g.replay, iters, warm)
        del g
        return ms

    class GemvCall:
        """Pre-marshalled vq_gemv call (descriptor built once, so the loop is launch-bound only)."""
        def __init__(self, wd, x, y, ws=None):
            self.keep = (wd, x, y, ws)
            self.desc = wd.desc()
            self.ref = ctypes.byref(self.desc)
            self.x, self.y, self.bs = x.data_ptr(), y.data_ptr(), x.shape[0]
            self.ws = None if ws is None else ws.data_ptr()
            self.ws_bytes = 0 if ws is None else ws.numel()

        def __call__(self):
            st = lib.vq_gemv(self.ref, self.x, self.bs, self.y, self.ws, self.ws_bytes, _stream())
            if st != 0:
                raise vq.VQError(st, "vq_gemv")

    def read_traffic(path):
        """HBM bytes per vq_gemv launch from the committed counter summary (None if there is none)."""
        try:
            for line in open(path):
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1])
        except OSError:
            pass
        return None

    result = {}
    t_setup = time.time()

    def additive_stack():
        """The decoder stack of the additive 2 x 256 x 8 configuration: 32 blocks x (4 + 2 + 1) matrices, every weight
        its own codes and codebooks; (weight, x, y) triples and the algorithmic bytes (as in the headline figure)."""
        stack, nbytes = [], 0
        for layer in range(args.layers):
            for si, cnt in ((0, 4), (1, 2), (2, 1)):
                N, K = wl.LLAMA7B_SHAPES[si]
                for j in range(cnt):
                    wd = vq.weight_to_device(wl.config3_layer(si, layer * 4 + j), dev)
                    x = torch.from_numpy(wl.make_activations(1, K, wl.seed_for(3, 1))).to(dev)
                    stack.append((wd, x, torch.empty((1, N), dtype=torch.float16, device=dev)))
                    nbytes += N * K // 8 * 2 + 2 * 256 * 8 * 2 + K * 2 + N * 4
        return stack, nbytes

    if args.pmc_probe_additive:
        args.pmc_probe = True
    if args.pmc_probe:
        nbytes = 256 << 20
        src = torch.full((nbytes,), 3, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            vq.vq_probe_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
        only = {"gemv"}
        if args.pmc_probe_additive:
            stack, eff = additive_stack()
            pipe = vq.GemvPipeline([[t] for t in stack])
            st = pipe.run()
            if st != 0:
                raise vq.VQError(st, "vq_gemv_pipeline_run")
            torch.cuda.synchronize()
            print(json.dumps({"pmc_probe": True, "probe_copy_bytes": 256 << 20, "probe_copies": 3,
                              "gemv_launches": 1, "effective_bytes": eff}), flush=True)
            return

    # ------------------------------------------------------------------ measured ceilings of this chip
    # (second reference beside the vendor peaks): a plain 128-bit streaming read of 2 GiB, cold, and a
    # register-resident fp16 MFMA loop
    ceil_hbm = ceil_mfma = ceil_mfma_rand = ceil_mfma_lds = None
    if not args.pmc_probe:
        big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
        big.fill_(1)
        sink = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
        ms = timed(lambda: vq.vq_probe_read(big, sink), 10, 2)
        ceil_hbm = big.numel() / ms / 1e6
        del big
        iters = 2000
        ms = timed(lambda: vq.vq_probe_mfma(1024, iters, sink), 5, 1)
        ceil_mfma = 1024 * 4 * iters * 8 * 32768.0 / (ms * 1e-3) / 1e12
        ms = timed(lambda: vq.vq_probe_mfma(1024, iters, sink, random_operands=1), 5, 1)
        ceil_mfma_rand = 1024 * 4 * iters * 8 * 32768.0 / (ms * 1e-3) / 1e12
        ms = timed(lambda: vq.vq_probe_mfma(1024, iters, sink, random_operands=2), 5, 1)
        ceil_mfma_lds = 1024 * 4 * iters * 8 * 32768.0 / (ms * 1e-3) / 1e12
        result["measured_ceilings"] = {"hbm_stream_read_GBps": round(ceil_hbm, 1),
                                       "mfma_fp16_register_loop_TFLOPs": round(ceil_mfma, 1),
                                       "mfma_fp16_register_loop_random_operands_TFLOPs": round(ceil_mfma_rand, 1),
                                       "mfma_fp16_lds_fed_random_operands_TFLOPs": round(ceil_mfma_lds, 1)}
        torch.cuda.empty_cache()

    cpu_secondary = {}   # the oracle timed on bounded samples of the secondary workloads (context beside cpu_baseline)

    # ------------------------------------------------------------------ headline: C2 gemv stack
    if want("gemv"):
        L = args.layers
        x_by_k = {K: torch.from_numpy(wl.make_activations(1, K, wl.seed_for(2, K))).to(dev) for K in (4096, 11008)}
        CPU_BLOCKS = 16   # decoder blocks kept on the host for the CPU baseline (about 10 s of oracle time)
        calls, singles, eff_bytes, per_shape = [], [], 0, {0: [], 1: [], 2: []}
        host_block0 = []
        packed = not args.canonical
        batched = packed and not args.no_batch
        sequenced = batched and not args.no_sequence
        ws = vq.new_workspace(4 << 20, dev) if packed else None   # shared by all launches of the stream
        seq_calls = []

        class BatchCall:
            """Pre-marshalled vq_gemv_batch call."""
            def __init__(self, members):
                self.b = vq.GemvBatch([m.keep[0] for m in members], [m.keep[1] for m in members],
                                      [m.keep[2] for m in members])
                assert self.b.workspace() <= ws.numel()

            def __call__(self):
                st = self.b.run(ws.data_ptr(), ws.numel())
                if st != 0:
                    raise vq.VQError(st, "vq_gemv_batch")

        for layer in range(L):
            block = []
            for slot, si in enumerate(wl.LLAMA7B_BLOCK):
                N, K = wl.LLAMA7B_SHAPES[si]
                w = wl.make_weight(N, K, 8, 16, 1, 65536, 0.02, wl.seed_for(2, layer * 7 + slot))
                wd = vq.weight_to_device(w, dev, prepack=packed, keep_codes=not packed)
                y = torch.empty((1, N), dtype=torch.float16, device=dev)
                c = GemvCall(wd, x_by_k[K], y, ws)
                block.append(c)
                singles.append(c)
                per_shape[si].append(c)
                eff_bytes += w.effective_bytes(1)
                if layer < CPU_BLOCKS:
                    host_block0.append(w)
            if batched:
                # slots: 0-2 query/key/value (one input), 3 output, 4-5 gate/up (one input), 6 down
                calls += [BatchCall(block[0:3]), block[3], BatchCall(block[4:6]), block[6]]
                seq_calls += [[c.keep[:3] for c in grp] for grp in (block[0:3], block[3:4], block[4:6], block[6:7])]
            else:
                calls += block
        torch.cuda.synchronize()

        pipelined = sequenced and args.mode == "pipeline"
        if pipelined:
            # the whole stack as ONE persistent launch: every workgroup walks through all matrices, staging the next
            # one's codebook slice and x while it gathers the current one
            pipe = vq.GemvPipeline(seq_calls)
            n_streams = 1

            def step():
                st = pipe.run()
                if st != 0:
                    raise vq.VQError(st, "vq_gemv_pipeline_run")
        elif sequenced:
            # the whole stack as ONE vq_gemv_sequence: one launch per call, the reduction of each riding along
            # in the next, one reduction launch at the end
            seq = vq.GemvSequence(seq_calls)
            n_streams = max(1, min(args.streams, 8))
            seq_ws = vq.new_workspace(seq.workspace_streams(n_streams), dev)
            seq_side = vq.SideStreams(n_streams - 1, dev)

            def step():
                st = seq.run_streams(seq_ws.data_ptr(), seq_ws.numel(), seq_side)
                if st != 0:
                    raise vq.VQError(st, "vq_gemv_sequence_streams")
        else:
            def step():
                for c in calls:
                    c()

        if args.pmc_probe:
            step()
            torch.cuda.synchronize()
            print(json.dumps({"pmc_probe": True, "probe_copy_bytes": 256 << 20, "probe_copies": 3,
                              "gemv_launches": len(calls), "effective_bytes": eff_bytes}), flush=True)
            return

        graph = None
        if not args.no_graph:
            step()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    step()
            run_step = graph.replay
        else:
            run_step = step

        # the first 20 steps of a GPU that comes from idle, for the record (they are part of no other figure)
        torch.cuda.synchronize()
        time.sleep(0.2)
        ms_from_idle = timed_once(run_step, 20) / 20
        # whatever --warmup says, the clocks get 50 more untimed steps to settle after that start from idle (the
        # default --warmup 50 covers it; a caller's smaller value is topped up, and the JSON line says by how much)
        settle = max(0, 50 - args.warmup)
        for _ in range(settle + args.warmup):
            run_step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            run_step()
        e1.record()
        torch.cuda.synchronize()
        ms_step = e0.elapsed_time(e1) / args.steps
        gbps = eff_bytes / (ms_step * 1e-3) / 1e9

        # per-shape cold times (graph replay, rotating over every matrix of that shape)
        shape_us = {}
        for si, cs in per_shape.items():
            def loop(cs=cs):
                for c in cs:
                    c()
            ms = timed_replay(loop, 5, 1)
            N, K = wl.LLAMA7B_SHAPES[si]
            b = cs[0].keep[0]
            bytes_one = (N * (K // 8) * 2 + b.codebooks.numel() * 2 + K * 2 + N * 2 + N * 2)
            us = ms * 1e3 / len(cs)
            shape_us["%dx%d" % (N, K)] = {"us": round(us, 3), "GBps": round(bytes_one / us / 1e3, 1),
                                          "pct_hbm_peak": round(100 * bytes_one / us / 1e3 / HBM_PEAK_GBPS, 2)}
        # warm (cache-resident) figure for the smallest shape, for context
        def warm_loop(c=per_shape[0][0]):
            for _ in range(20):
                c()
        warm_ms = timed_replay(warm_loop, 10, 2) / 20
        shape_us["4096x4096_warm_us"] = round(warm_ms * 1e3, 3)

        n_launch = len(calls)
        if not sequenced:
            n_streams = 1
        if pipelined and pipe.status() != 0:
            raise RuntimeError("vq_gemv_pipeline: a wavefront gave up a bounded wait; the timed runs are invalid")
        n_dispatch = 2 if pipelined else n_launch + n_streams if sequenced else 2 * n_launch if packed else n_launch
        main_launches = 1 if pipelined else n_launch
        result.update({
            "metric": "VQ-GEMV bs=1 effective HBM bandwidth, Llama-7B shapes, 2^16x8 codebook",
            "value": round(gbps, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f16", "data": "synthetic",
            "first_20_steps_from_idle_ms_per_step": round(ms_from_idle, 5),
            "settle_steps_before_warmup": settle,
            "config": {"workload": "C2: Llama-7B decode VQ-gemv bs=1, %d blocks x 7 matrices, VQ<8,16,1> uint16 codes, "
                                   "fp16 scale" % L,
                       "launches_per_step": n_launch, "matrices_per_step": len(singles),
                       "effective_bytes_per_step": eff_bytes,
                       "kernel_dispatches_per_step": n_dispatch,
                       "streams": n_streams if sequenced else 1,
                       "calls": ("one vq_gemv_pipeline over the stack: a persistent launch of 256 workgroups that walk through "
                                 "all %d matrices, plus one reduction launch" % len(singles)
                                 if pipelined else
                                 "one vq_gemv_sequence_streams over the stack (contiguous runs of calls on %d streams); per "
                                 "block the calls (q,k,v), (o), (gate,up), (down)" % n_streams
                                 if sequenced else
                                 "per block: vq_gemv_batch(q,k,v), vq_gemv(o), vq_gemv_batch(gate,up), vq_gemv(down)"
                                 if batched else "one vq_gemv per matrix"),
                       "code_layout": "re-tiled offline by vq_gemv_prepack (LDS codebook slices)" if packed
                                      else "canonical [N][K/8] (entries gathered from L2)",
                       "timing": "hip-graph replay" if graph is not None else "eager launches"},
            "pct_hbm_peak": round(100 * gbps / HBM_PEAK_GBPS, 2),
            "pct_measured_stream_read": round(100 * gbps / ceil_hbm, 2),
            "gemv_per_shape_cold": shape_us,
            "roofline": {"bound": "hbm", "kernel": ("gemv_pipeline_kernel (one launch = the whole step)" if pipelined else
                                    "gemv_packed_batch_kernel / gemv_packed_kernel (reduction folded into the next launch)" if sequenced else
                                    "gemv_packed_batch_kernel / gemv_packed_kernel (+ finalize)" if batched else
                                    "gemv_packed_kernel (+ finalize)" if packed else "gemv_rows_kernel<uint16,8,1>"),
                         "achieved": round(gbps, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": round(gbps / HBM_PEAK_GBPS, 4),
                         "traffic": read_traffic(args.traffic_file) if batched else None,
                         "bytes_per_launch": eff_bytes // main_launches,
                         "avg_launch_us": round(ms_step * 1e3 / main_launches, 3)},
        })

        # ---- CPU oracle baseline on a bounded sample: one decoder block (7 matrices), bs = 1
        if not args.skip_cpu:
            import oracle
            xs = {K: x_by_k[K].cpu().numpy() for K in x_by_k}
            oracle.gemv(host_block0[0].codes, host_block0[0].codebooks, host_block0[0].scale, xs[host_block0[0].K])
            reps = 3
            t0 = time.perf_counter()
            for _ in range(reps):
                for w in host_block0:
                    oracle.gemv(w.codes, w.codebooks, w.scale, xs[w.K])
            dt = (time.perf_counter() - t0) / reps
            blk_bytes = sum(w.effective_bytes(1) for w in host_block0)
            result["cpu_baseline"] = {"value": round(blk_bytes / dt / 1e9, 3), "unit": "GB/s",
                                      "cores": oracle.threads(), "kind": "oracle",
                                      "sample": "%d of the %d matrices (the first %d decoder blocks), mean of %d passes, "
                                                "%.2f s per pass" % (len(host_block0), len(singles),
                                                                     len(host_block0) // 7, reps, dt)}
            # the same oracle on ONE thread, on the first decoder block
            n_threads = oracle.threads()
            oracle.set_threads(1)
            t0 = time.perf_counter()
            for w in host_block0[:7]:
                oracle.gemv(w.codes, w.codebooks, w.scale, xs[w.K])
            dt1 = time.perf_counter() - t0
            one_thread = oracle.threads()
            oracle.set_threads(n_threads)
            cpu_secondary["gemv_single_thread"] = {
                "value": round(sum(w.effective_bytes(1) for w in host_block0[:7]) / dt1 / 1e9, 4), "unit": "GB/s",
                "cores": one_thread, "kind": "oracle", "sample": "the 7 matrices of the first decoder block, one pass, %.2f s" % dt1}
        del calls, singles, per_shape, graph
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ secondary: C4 prefill gemm
    if want("gemm") and not args.skip_secondary:
        gemm = {}
        X = torch.from_numpy(wl.make_activations(2048, 4096, wl.seed_for(4, 0))).to(dev)
        for N in (4096, 11008):
            for v in (8, 4):
                wd = vq.weight_to_device(wl.config4_layer(N, v), dev)
                Y = torch.empty((2048, N), dtype=torch.float16, device=dev)
                gws = vq.new_workspace(vq.vq_gemm_workspace(wd, 2048), dev)   # the caller's workspace: nothing is allocated in the timed calls
                fn = lambda: vq.vq_gemm(wd, X, Y=Y, ws=gws)
                ms = timed(fn, 10, 2)
                tf = 2.0 * 2048 * N * 4096 / (ms * 1e-3) / 1e12
                gemm["N%d_v%d" % (N, v)] = {"us": round(ms * 1e3, 2), "TFLOPs": round(tf, 1),
                                            "pct_mfma_fp16_peak": round(100 * tf / MFMA_FP16_PEAK_TFLOPS, 2),
                                            "pct_measured_mfma_loop": round(100 * tf / ceil_mfma, 2),
                                            "pct_measured_mfma_loop_random_operands": round(100 * tf / ceil_mfma_rand, 2),
                                            "pct_measured_mfma_lds_fed_random_operands": round(100 * tf / ceil_mfma_lds, 2)}
                del wd, Y, gws
        result["gemm_prefill_M2048_K4096"] = gemm
        if not args.skip_cpu:
            # the oracle on a bounded sample of the same product: 1024 evenly spaced output channels, all 2048 rows of X
            import oracle
            wh = wl.config4_layer(4096, 8)
            rows = list(range(0, 4096, 4))
            xh = X.cpu().numpy()
            t0 = time.perf_counter()
            oracle.gemm(wh.codes, wh.codebooks, wh.scale, xh, rows=rows)
            dt = time.perf_counter() - t0
            cpu_secondary["gemm_prefill_N4096_v8"] = {
                "value": round(2.0 * 2048 * len(rows) * 4096 / dt / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.threads(),
                "kind": "oracle", "sample": "%d of 4096 output channels x 2048 rows, one pass, %.2f s" % (len(rows), dt)}

    # ------------------------------------------------------------------ secondary: C5 attention decode
    if want("attn") and not args.skip_secondary:
        kv = wl.config5_kv()
        ring = [vq.kv_to_device(kv, dev) for _ in range(3)]     # 3 x 128 MiB of codes: beyond the last-level cache
        q = torch.from_numpy(kv.q).to(dev)
        out = torch.empty_like(q)
        wsz = vq.vq_attn_decode_workspace(ring[0])
        ws = torch.empty(max(wsz, 16), dtype=torch.uint8, device=dev)
        sm = 1.0 / np.sqrt(128.0)

        def attn_loop():
            for kd in ring:
                vq.vq_attn_decode(kd, q, sm, out=out, ws=ws)
        ms = timed(attn_loop, 10, 2) / len(ring)
        b = kv.effective_bytes()
        result["attn_decode_B16_H32_T4096"] = {"us": round(ms * 1e3, 2), "GBps": round(b / ms / 1e6, 1),
                                               "pct_hbm_peak": round(100 * b / ms / 1e6 / HBM_PEAK_GBPS, 2),
                                               "pct_measured_stream_read": round(100 * b / ms / 1e6 / ceil_hbm, 2)}
        if not args.skip_cpu:
            # the oracle on the whole workload (16 sequences, all heads, all 4096 tokens): a few seconds
            import oracle
            nb = kv.B
            t0 = time.perf_counter()
            oracle.attn_decode(kv.k_codes[:nb], kv.v_codes[:nb], kv.k_codebooks, kv.v_codebooks, kv.q[:nb], float(sm))
            dt = time.perf_counter() - t0
            cpu_secondary["attn_decode_B16_H32_T4096"] = {
                "value": round(b * nb / kv.B / dt / 1e9, 4), "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
                "sample": "%d of %d sequences, one pass, %.2f s" % (nb, kv.B, dt)}
        # on-the-fly quantization of new tokens into that cache: one decode step, and a 4096-token prefill
        kd = ring[0]
        k1 = torch.randn((kv.B, kv.H, 1, kv.D), device=dev).to(torch.float16)
        kT = torch.randn((kv.B, kv.H, kv.T, kv.D), device=dev).to(torch.float16)
        def quant_decode_loop():          # 20 decode-step calls per graph replay: the host's launch rate stays out
            for _ in range(20):
                vq.vq_kv_quantize(kd, k1, k1, kv.T - 1)
        ms1 = timed_replay(quant_decode_loop, 10, 2) / 20
        msT = timed(lambda: vq.vq_kv_quantize(kd, kT, kT, 0), 5, 1)
        result["kv_quantize_B16_H32"] = {"decode_1_token_us": round(ms1 * 1e3, 2),
                                         "prefill_4096_tokens_us": round(msT * 1e3, 1),
                                         "prefill_input_GBps": round(2 * kT.numel() * 2 / msT / 1e6, 1)}
        del k1, kT, kd, ring
        torch.cuda.empty_cache()
        # same shape with the coupled-quantization layout: 32 codebooks per head and side (64 KiB each)
        kv = wl.config5_kv(G=32)
        ring = [vq.kv_to_device(kv, dev) for _ in range(3)]

        def attn_loop_cq():
            for kd in ring:
                vq.vq_attn_decode(kd, q, sm, out=out, ws=ws)
        ms = timed(attn_loop_cq, 10, 2) / len(ring)
        b = kv.effective_bytes()
        result["attn_decode_B16_H32_T4096_cq32"] = {"us": round(ms * 1e3, 2), "GBps": round(b / ms / 1e6, 1),
                                                    "pct_hbm_peak": round(100 * b / ms / 1e6 / HBM_PEAK_GBPS, 2)}
        # the other side of the paper's trade-off for this layout: channel-parallel workgroups, partial inner products
        # accumulated through global memory (three launches)
        ws_cp = vq.new_workspace(kv.B * kv.H * (kv.D // 32 + 1) * kv.T * 4, dev)

        def attn_loop_cp():
            for kd in ring:
                vq.vq_attn_decode_channel_parallel(kd, q, sm, out=out, ws=ws_cp)
        ms = timed(attn_loop_cp, 10, 2) / len(ring)
        result["attn_decode_B16_H32_T4096_cq32_channel_parallel"] = {
            "us": round(ms * 1e3, 2), "GBps": round(b / ms / 1e6, 1), "pct_hbm_peak": round(100 * b / ms / 1e6 / HBM_PEAK_GBPS, 2)}
        del ws_cp
        del ring
        torch.cuda.empty_cache()
        # CQ-4 (Tbl. III: VQ<2,8,1>): 64 codebooks per head and side, twice the code bytes per token
        kv = wl.config5_kv(G=64, v=2)
        ring = [vq.kv_to_device(kv, dev) for _ in range(2)]     # 2 x 256 MiB of codes

        def attn_loop_cq4():
            for kd in ring:
                vq.vq_attn_decode(kd, q, sm, out=out, ws=ws)
        ms = timed(attn_loop_cq4, 10, 2) / len(ring)
        b = kv.effective_bytes()
        result["attn_decode_B16_H32_T4096_cq4_v2"] = {"us": round(ms * 1e3, 2), "GBps": round(b / ms / 1e6, 1),
                                                      "pct_hbm_peak": round(100 * b / ms / 1e6 / HBM_PEAK_GBPS, 2)}
        del ring
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ secondary: C3 additive gemv
    if want("add") and not args.skip_secondary:
        add = {}
        for si in (0, 1, 2):
            N, K = wl.LLAMA7B_SHAPES[si]
            n_copies = 48 if si == 0 else 24
            wds = [vq.weight_to_device(wl.config3_layer(si, layer), dev) for layer in range(n_copies)]
            for bs in (1, 4, 16):
                x = torch.from_numpy(wl.make_activations(bs, K, wl.seed_for(3, bs))).to(dev)
                y = torch.empty((bs, N), dtype=torch.float16, device=dev)

                cs = [GemvCall(wd, x, y) for wd in wds]

                def loop(cs=cs):
                    for c in cs:
                        c()
                ms = timed_replay(loop, 3, 1) / len(wds)
                b = wds[0].codes.numel() + wds[0].codebooks.numel() * 2 + N * 2 + bs * (K + N) * 2
                add["%dx%d_bs%d" % (N, K, bs)] = {"us": round(ms * 1e3, 2),
                                                   "pct_hbm_peak": round(100 * b / ms / 1e6 / HBM_PEAK_GBPS, 2)}
                if bs == 1:
                    # the same matrices three to a launch (vq_gemv_batch: projections of a decoder block that share
                    # their input, as query/key/value do); per-matrix time
                    ys3 = [torch.empty((1, N), dtype=torch.float16, device=dev) for _ in range(3)]
                    bcs = [vq.GemvBatch(wds[i:i + 3], [x] * 3, ys3) for i in range(0, len(wds) - 2, 3)]

                    def bloop(bcs=bcs):
                        for bc in bcs:
                            st = bc.run(None, 0)
                            if st != 0:
                                raise vq.VQError(st, "vq_gemv_batch")
                    msb = timed_replay(bloop, 3, 1) / (3 * len(bcs))
                    add["%dx%d_bs1_batch_of_3" % (N, K)] = {"us": round(msb * 1e3, 2),
                                                           "pct_hbm_peak": round(100 * b / msb / 1e6 / HBM_PEAK_GBPS, 2)}
            del wds
            torch.cuda.empty_cache()
        # the whole decoder stack of this configuration (32 blocks x (4 + 2 + 1) matrices, every weight its own
        # codes and codebooks): one launch through vq_gemv_pipeline (16 LDS copies of every entry), against the
        # same stack as one vq_gemv call per matrix; algorithmic bytes as in the headline figure
        stack, nbytes = additive_stack()
        pipe = vq.GemvPipeline([[t] for t in stack])

        def stack_pipeline():
            st = pipe.run()
            if st != 0:
                raise vq.VQError(st, "vq_gemv_pipeline_run")
        ms_p = timed_replay(stack_pipeline, 10, 2)
        cs = [GemvCall(wd, x, y) for (wd, x, y) in stack]

        def stack_calls():
            for c in cs:
                c()
        ms_c = timed_replay(stack_calls, 5, 1)
        add["stack_%d_matrices_bs1" % len(stack)] = {
            "algorithmic_bytes": nbytes,
            "vq_gemv_pipeline": {"ms": round(ms_p, 4), "GBps": round(nbytes / ms_p / 1e6, 1),
                                 "pct_hbm_peak": round(100 * nbytes / ms_p / 1e6 / HBM_PEAK_GBPS, 2), "kernel_dispatches": 1},
            "one_vq_gemv_per_matrix": {"ms": round(ms_c, 4), "GBps": round(nbytes / ms_c / 1e6, 1),
                                       "pct_hbm_peak": round(100 * nbytes / ms_c / 1e6 / HBM_PEAK_GBPS, 2),
                                       "kernel_dispatches": len(stack)}}
        pipe.close()
        del pipe, cs, stack
        torch.cuda.empty_cache()
        result["gemv_additive_2x256x8"] = add

    # ------------------------------------------------------------------ secondary: per-tile codebooks (VQ<4,8,1>, 256 x 256 tiles)
    if want("tile") and not args.skip_secondary:
        tile = {}
        for si in (0, 1, 2):
            N, K = wl.LLAMA7B_SHAPES[si]
            n_copies = 24 if si == 0 else 12
            wds = [vq.weight_to_device(wl.gptvq_like_layer(si, layer), dev) for layer in range(n_copies)]
            for bs in (1, 16):
                x = torch.from_numpy(wl.make_activations(bs, K, wl.seed_for(7, bs))).to(dev)
                y = torch.empty((bs, N), dtype=torch.float16, device=dev)
                cs = [GemvCall(wd, x, y) for wd in wds]

                def loop(cs=cs):
                    for c in cs:
                        c()
                ms = timed_replay(loop, 3, 1) / len(wds)
                b = wds[0].codes.numel() + wds[0].codebooks.numel() * 2 + N * 2 + bs * (K + N) * 2
                tile["%dx%d_bs%d" % (N, K, bs)] = {"us": round(ms * 1e3, 2),
                                                    "pct_hbm_peak": round(100 * b / ms / 1e6 / HBM_PEAK_GBPS, 2)}
            del wds
            torch.cuda.empty_cache()
        result["gemv_per_tile_codebooks_256x4_tiles256"] = tile

    # ------------------------------------------------------------------ secondary: packed 12-bit codes (VQ<8,12,2>)
    if want("bit12") and not args.skip_secondary:
        b12 = {}
        for si in (0, 1, 2):
            N, K = wl.LLAMA7B_SHAPES[si]
            n_copies = 24 if si == 0 else 12
            wds = [vq.weight_to_device(wl.aqlm3_like_layer(si, layer), dev) for layer in range(n_copies)]
            for bs in (1, 16):
                x = torch.from_numpy(wl.make_activations(bs, K, wl.seed_for(8, bs))).to(dev)
                y = torch.empty((bs, N), dtype=torch.float16, device=dev)
                cs = [GemvCall(wd, x, y) for wd in wds]

                def loop(cs=cs):
                    for c in cs:
                        c()
                ms = timed_replay(loop, 3, 1) / len(wds)
                b = wds[0].codes.numel() + wds[0].codebooks.numel() * 2 + N * 2 + bs * (K + N) * 2
                b12["%dx%d_bs%d" % (N, K, bs)] = {"us": round(ms * 1e3, 2),
                                                   "pct_hbm_peak": round(100 * b / ms / 1e6 / HBM_PEAK_GBPS, 2)}
            del wds
            torch.cuda.empty_cache()
        result["gemv_12bit_2x4096x8"] = b12

    # ------------------------------------------------------------------ secondary: skewed code usage (Zipf, s = 1)
    if want("zipf") and not args.skip_secondary:
        zipf = {}
        N, K = wl.LLAMA7B_SHAPES[0]
        n_copies = 24
        x = torch.from_numpy(wl.make_activations(1, K, wl.seed_for(2, K))).to(dev)
        y = torch.empty((1, N), dtype=torch.float16, device=dev)
        ws = vq.new_workspace(4 << 20, dev)
        variants = {"canonical_entries_in_quantizer_order": [], "canonical_reordered_by_frequency": []}
        hot_frac = 0.0
        for layer in range(n_copies):
            w = wl.shuffle_entries(wl.make_weight(N, K, 8, 16, 1, 65536, 0.02, wl.seed_for(6, layer), zipf_s=1.0),
                                   seed=layer)
            r = vq.vq_reorder_by_frequency(w)
            hot_frac += float((r.codes < 4096).mean()) / n_copies
            variants["canonical_entries_in_quantizer_order"].append(GemvCall(vq.weight_to_device(w, dev), x, y))
            variants["canonical_reordered_by_frequency"].append(GemvCall(vq.weight_to_device(r, dev), x, y))
            # the re-tiled form needs codes that spread evenly over the codebook slices
            if layer == 0:
                zipf["vq_gemv_prepack_declines_these_codes"] = bool(vq.vq_gemv_prepack(w)[0] is None and
                                                                    vq.vq_gemv_prepack(r)[0] is None)
        for name, cs in variants.items():
            def loop(cs=cs):
                for c in cs:
                    c()
            zipf[name + "_us"] = round(timed(loop, 5, 1) * 1e3 / n_copies, 2)
        zipf["codes_served_by_the_4096_entry_lds_cache"] = round(hot_frac, 3)
        result["gemv_zipf_s1_4096x4096"] = zipf
        del variants
        torch.cuda.empty_cache()

    if cpu_secondary:
        result["cpu_baseline_secondary"] = cpu_secondary
    result["setup_plus_run_s"] = round(time.time() - t_setup, 1)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
