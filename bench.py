#!/usr/bin/env python3
"""Benchmark of the fused LoRA linear layer, forward + backward, on one MI355X.

One "step" is one pass of the whole hot path - lora_fwd (operations 1-2) then lora_bwd
(operations 3-5, dX, dA and dB) - over one batch of synthetic bf16 inputs that are already
resident in HBM.  The default workload is the 8B-style attention projection (M=8192 tokens,
K=N=4096, r=16, s=2, p=0.1), the configuration the headline metric is quoted on.

Prints ONE JSON line: whole-job TFLOP/s on the algorithmic FLOP count 4MKN + 6Mr(K+N), tokens/s,
the roofline record of the dominant kernel (timed live with HIP events on the launch stream) and
the CPU oracle timed on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published


def read_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary
    (profiles/hbm_traffic_<workload>.txt, line 'dominant_kernel_bytes_per_launch: N'); None if absent."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        with open(path) as f:
            for ln in f:
                if ln.startswith("dominant_kernel_bytes_per_launch:"):
                    return float(ln.split(":", 1)[1])
    except OSError:
        pass
    return None


def measure_ceilings(torch, binding, dev, operands):
    """What this GPU sustains with nothing in the way (library diagnostics, timed with events on the launch
    stream): the GEMM kernels' MFMA instruction (and the other bf16 MFMA shape) in a register-resident loop on
    `operands` (values of the workload's distribution), one plain read of a 2 GiB buffer (eight times the memory-side cache), and
    plain reads the size of `operands` (what one streaming kernel of the path reads), one launch each, back to
    back, every launch on a window of the big buffer that has left the memory-side cache."""
    def timed(fn, reps, skip):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        evs[0].record()
        for i in range(reps):
            fn()
            evs[i + 1].record()
        torch.cuda.synchronize()
        ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(reps)][skip:]
        return sum(ms) / len(ms)

    big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    big.fill_(1)
    sink2 = torch.empty(4096 * 256, dtype=torch.int32, device=dev)
    nbytes = [0]

    def read():
        nbytes[0] = binding.ceiling_hbm_read(big, sink2, 4096)
    ms = timed(read, 6, 2)
    read_gbs = nbytes[0] / (ms * 1e-3) / 1e9
    # the same read in launches of the streaming kernels' size: start-up and drain of a launch included
    win = operands.numel() * operands.element_size() // 4096 * 4096
    nwin = min(16, (2 << 30) // win)
    wgs_win = 512                                # two workgroups per compute unit walk the window (the fastest shape found)
    views = [big[i * win:(i + 1) * win] for i in range(nwin)]
    ms_win = None
    if nwin >= 4:
        # three whole-buffer reads go first so that the queue never runs dry while the host enqueues the windows
        # (the events then bracket back-to-back launches, as they do inside a step); the big read ends on the far
        # end of the buffer, the windows start at the near end, so none of them is in the memory-side cache
        for _ in range(3):
            read()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(nwin + 1)]
        evs[0].record()
        for i in range(nwin):
            binding.ceiling_hbm_read(views[i], sink2, wgs_win)
            evs[i + 1].record()
        torch.cuda.synchronize()
        ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(nwin)][nwin // 4:]
        ms_win = sum(ms) / len(ms)
    del views
    del big

    # the matrix loops last: the timed steps then start from the chip's state under its heaviest load
    wgs, iters = 2048, 1536
    sink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
    flops = [0.0]
    rates = {}
    for shape in (32, 16):                      # the GEMM kernels' own instruction (16x16x32) last
        def mfma():
            flops[0] = binding.ceiling_mfma(operands, sink, wgs, iters, shape)
        ms = timed(mfma, 8, 3)                  # about 55 ms in all: the sustained rate, not the first burst
        rates[shape] = flops[0] / (ms * 1e-3) / 1e12
    out = {"mfma_bf16_tflops": round(rates[16], 1), "mfma_bf16_tflops_32x32x16": round(rates[32], 1),
           "hbm_read_gbs": round(read_gbs, 1),
           "how": "register-resident MFMA loops, 256 accumulators per lane in independent chains, 1 wave per SIMD, operands = "
                  "the workload's X values: v_mfma_f32_16x16x32_bf16 (the GEMM kernels' instruction) and, for comparison, "
                  "v_mfma_f32_32x32x16_bf16; plain 16-byte-per-lane read of 2 GiB; the same read in single launches "
                  "of sizeof(X) bytes, back to back, on windows that are not cached"}
    if ms_win:
        out["hbm_read_one_launch_gbs"] = round(win / (ms_win * 1e-3) / 1e9, 1)
        out["hbm_read_one_launch_us"] = round(ms_win * 1e3, 2)
        out["hbm_read_one_launch_bytes"] = win
    return out


def sweep(torch, binding, workloads, dev, args):
    """The axes of the paper's Figure 3 / Figure 17 on this GPU: n = k = 4096, tokens swept, r in {16, 32};
    forward and backward times of the fused LoRA linear, the unfused baseline and the frozen linear."""
    def timed(fn, iters):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / iters * 1e6

    for r in (16, 32):
        for M in (1024, 2048, 4096, 8192, 16384):
            L = workloads.custom_layer(M, 4096, 4096, r, 2.0, 0.1, cfg=6, name=f"sweep_m{M}_r{r}")
            X, W, A, B, dY = (t.to(dev) for t in workloads.make_inputs(L))
            A1, B1 = A[0].contiguous(), B[0].contiguous()
            Y = torch.empty((M, 4096), dtype=torch.bfloat16, device=dev)
            dX = torch.empty((M, 4096), dtype=torch.bfloat16, device=dev)
            S = torch.empty((M, r), dtype=torch.bfloat16, device=dev)
            dA = torch.empty((r, 4096), dtype=torch.float32, device=dev)
            dB = torch.empty((4096, r), dtype=torch.float32, device=dev)
            ws = binding.alloc_workspace(M, 4096, 4096, r, 1, dev)
            uws = binding.unfused_workspace(M, 4096, 4096, r, dev)
            it = max(10, min(args.steps, 200))
            rec = {"sweep": "tokens x rank, K=N=4096", "tokens": M, "r": r,
                   "fused_fwd_us": timed(lambda: binding.lora_fwd(X, W, A1, B1, L.s, L.p, L.seeds[0], Y=Y, S=S), it),
                   "fused_bwd_us": timed(lambda: binding.lora_bwd(X, W, A1, B1, S, dY, L.s, L.p, L.seeds[0], dA=dA, dB=dB,
                                                                  workspace=ws, dX=dX), it),
                   "unfused_fwd_us": timed(lambda: binding.lora_unfused_fwd(X, W, A1, B1, L.s, L.p, L.seeds[0], uws, Y=Y), it),
                   "unfused_bwd_us": timed(lambda: binding.lora_unfused_bwd(W, A1, B1, dY, L.s, L.p, L.seeds[0], uws,
                                                                            dX=dX, dA=dA, dB=dB), it),
                   "frozen_fwd_us": timed(lambda: binding.frozen_fwd(X, W, Y=Y), it),
                   "frozen_bwd_us": timed(lambda: binding.frozen_bwd(dY, W, dX=dX), it)}
            rec = {k: (round(v, 1) if isinstance(v, float) else v) for k, v in rec.items()}
            rec["fused_over_frozen_fwd"] = round(rec["fused_fwd_us"] / rec["frozen_fwd_us"], 3)
            rec["fused_over_frozen_bwd"] = round(rec["fused_bwd_us"] / rec["frozen_bwd_us"], 3)
            rec["unfused_over_fused_fwd"] = round(rec["unfused_fwd_us"] / rec["fused_fwd_us"], 3)
            rec["unfused_over_fused_bwd"] = round(rec["unfused_bwd_us"] / rec["fused_bwd_us"], 3)
            print(json.dumps(rec), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--settle-ms", type=float, default=100.0,
                    help="untimed steps of the workload for about this long before the warm-up steps (0: none)")
    ap.add_argument("--workload", default="c2", help="c1..c5 (default c2, the headline configuration); layer8b, layer70b (decoder-layer "
                         "composites, 7 LoRA linears) and their _qkv variants (q/k/v as one LoRA linear)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rotate", type=int, default=1,
                    help="number of independent buffer sets (inputs, weights, outputs, workspace) used round-robin, "
                         "one per step; with enough sets (> 256 MB in total) no step finds its tensors in the "
                         "memory-side cache.  Default 1: back-to-back steps on the same buffers")
    ap.add_argument("--unfused", action="store_true",
                    help="time the unfused multi-kernel baseline instead of the fused path (comparison runs)")
    ap.add_argument("--sweep", action="store_true",
                    help="token-count x rank sweep at K=N=4096: fused LoRA, unfused baseline and frozen linear (one JSON line each)")
    ap.add_argument("--row-tile", type=int, default=0, choices=(0, 128, 256),
                    help="token rows per GEMM tile: 0 lets every launch choose (default), 128 or 256 fixes it (comparison runs)")
    ap.add_argument("--graph", action="store_true",
                    help="record one step (all layers, forward + backward) into a HIP graph and time replays of it: "
                         "takes the host's launch work out of launch-bound workloads such as c1")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured ceilings (register-resident MFMA loop, plain HBM read) that are otherwise "
                         "taken before the warm-up steps")
    ap.add_argument("--ceilings-only", action="store_true", help="measure and print the ceilings, nothing else")
    ap.add_argument("--gemm-compare", type=int, default=0, metavar="M",
                    help="only time (and, under rocprofv3, expose to the counters) M x 4096 x 4096 bf16 products: the library's "
                         "frozen-linear forward / backward GEMMs and torch.matmul (the vendor library) on the same operands")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a 1 GiB device copy 10 times (reference reading for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_00206_amd import binding, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.load_library()                     # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.lora_set_row_tile(args.row_tile)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4, "launches": 10}))
        return
    if args.gemm_compare:
        M = args.gemm_compare
        L = workloads.custom_layer(M, 4096, 4096, 16, 2.0, 0.1, cfg=2, name="gemm_compare")
        X, W, _, _, dY = (t.to(dev) for t in workloads.make_inputs(L))
        Y, dX = torch.empty_like(dY), torch.empty_like(X)

        def timed(fn, iters=args.steps):
            for _ in range(max(5, iters // 4)):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(iters):
                fn()
            torch.cuda.synchronize()
            return round((time.perf_counter() - t0) / iters * 1e6, 1)
        rec = {"gemm_compare": f"{M} x 4096 x 4096 bf16", "iters": args.steps}
        for rep in range(2):                   # twice: the first pass also settles the clocks
            rec.update({"frozen_fwd_us": timed(lambda: binding.frozen_fwd(X, W, Y=Y)),
                        "vendor_matmul_x_wt_us": timed(lambda: torch.matmul(X, W.t(), out=Y)),
                        "frozen_bwd_us": timed(lambda: binding.frozen_bwd(dY, W, dX=dX)),
                        "vendor_matmul_dy_w_us": timed(lambda: torch.matmul(dY, W, out=dX))})
        print(json.dumps(rec))
        return
    if args.sweep:
        sweep(torch, binding, workloads, dev, args)
        return
    layers = workloads.CONFIGS[args.workload]

    # inputs, outputs and workspaces resident in HBM before the timed region
    def make_state():
        state = []
        for li, L in enumerate(layers):
            X, W, A, B, dY = (t.to(dev) for t in workloads.make_inputs(L, layer_index=li))
            st = dict(L=L, X=X, W=W, A=A, B=B, dY=dY,
                      Y=torch.empty((L.M, L.N), dtype=torch.bfloat16, device=dev),
                      S=torch.empty((L.M, L.r), dtype=torch.bfloat16, device=dev),
                      dX=torch.empty((L.M, L.K), dtype=torch.bfloat16, device=dev),
                      dA=torch.empty((L.G, L.r, L.K), dtype=torch.float32, device=dev),
                      dB=torch.empty((L.G, L.N, L.r), dtype=torch.float32, device=dev),
                      ws=binding.alloc_workspace(L.M, L.K, L.N, L.r, L.G, dev),
                      s=[L.s] * L.G, p=[L.p] * L.G)
            state.append(st)
        return state

    sets = [make_state()]
    for _ in range(1, max(1, args.rotate)):
        # further sets: same values, separate memory
        sets.append([{k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in st.items()} for st in sets[0]])
    state = sets[0]
    step_no = [0]

    if args.unfused:
        for st in (st for one in sets for st in one):
            assert st["L"].G == 1, "the unfused baseline is single-adapter"
            st["uws"] = binding.unfused_workspace(st["L"].M, st["L"].K, st["L"].N, st["L"].r, dev)
            st["A1"], st["B1"] = st["A"][0].contiguous(), st["B"][0].contiguous()

    def step():
        cur = sets[step_no[0] % len(sets)]
        step_no[0] += 1
        for st in cur:
            L = st["L"]
            if args.unfused:
                binding.lora_unfused_fwd(st["X"], st["W"], st["A1"], st["B1"], L.s, L.p, L.seeds[0], st["uws"], Y=st["Y"])
                binding.lora_unfused_bwd(st["W"], st["A1"], st["B1"], st["dY"], L.s, L.p, L.seeds[0], st["uws"],
                                         dX=st["dX"], dA=st["dA"][0], dB=st["dB"][0])
                continue
            binding.multi_lora_fwd(st["X"], st["W"], st["A"], st["B"], L.seg_offsets, st["s"], st["p"], L.seeds,
                                   Y=st["Y"], S=st["S"])
            binding.multi_lora_bwd(st["X"], st["W"], st["A"], st["B"], st["S"], st["dY"], L.seg_offsets,
                                   st["s"], st["p"], L.seeds, dA=st["dA"], dB=st["dB"],
                                   workspace=st["ws"], dX=st["dX"])

    # measured ceilings first (outside the timed region): they also bring the chip to its working clocks
    ceilings = None
    if not args.no_ceilings and not args.unfused:
        ceilings = measure_ceilings(torch, binding, dev, state[0]["X"])
        if args.ceilings_only:
            print(json.dumps({"ceilings": ceilings}))
            return

    eager_step = step
    if args.graph:
        assert len(sets) == 1, "--graph replays one recorded step: use it without --rotate"
        eager_step()                           # first launches (kernel attributes) outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eager_step()
        step = graph.replay

    # The ceiling loops leave the chip well off the state that the step workload itself settles in (the matrix loops
    # run it into its power limit; the clocks then sag for some tens of milliseconds).  Untimed steps of the
    # workload bring it there, whatever --warmup is: about `--settle-ms` of them, before the W warm-up steps.
    settle_steps = 0
    if args.settle_ms > 0:
        torch.cuda.synchronize()
        t_s = time.perf_counter()
        while (time.perf_counter() - t_s) * 1e3 < args.settle_ms:
            for _ in range(8):
                step()
            torch.cuda.synchronize()
            settle_steps += 8
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    # spread of single steps: events on the launch stream (the binding launches on torch's current stream)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    evs[0].record()
    for i in range(args.steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps))
    step_ms = {"median": round(per_step[len(per_step) // 2], 4), "min": round(per_step[0], 4),
               "max": round(per_step[-1], 4)}

    flops = sum(st["L"].flops for st in state)
    tokens = state[0]["L"].M                    # the layers of one configuration share the token batch
    fused_bytes = sum(st["L"].fused_bytes for st in state)
    tflops = flops / (ms_per_step * 1e-3) / 1e12

    if args.unfused:
        print(json.dumps({"metric": "unfused multi-kernel LoRA linear fwd+bwd (baseline for comparison)",
                          "value": round(tflops, 2), "unit": "TFLOP/s", "ms_per_step": round(ms_per_step, 4),
                          "steps": args.steps, "warmup": args.warmup, "config": {"workload": args.workload},
                          "step_ms": step_ms, "buffer_sets": len(sets),
                          "tokens_per_s": round(tokens / (ms_per_step * 1e-3), 1),
                          "algorithmic_hbm_bytes_per_token": round(sum(st["L"].unfused_bytes for st in state) / tokens, 1)}))
        return

    # per-kernel durations: same steps again with HIP events around every launch (on the launch stream)
    binding.profile_begin()
    for _ in range(args.steps):
        eager_step()
    prof = binding.profile_end()
    kernels_us = {k: (ms / n * 1e3 if n else 0.0) for k, (ms, n) in prof.items()}
    launches = {k: n for k, (ms, n) in prof.items()}
    # dominant kernel: the dX GEMM (operation 5); its algorithmic FLOPs per launch = 2MNK + 2MrK,
    # averaged over the launches of one step (one per layer)
    dom = "dx_gemm" if kernels_us["dx_gemm"] >= kernels_us["fwd_gemm"] else "fwd_gemm"
    if dom == "dx_gemm":
        dom_flops = sum(2 * st["L"].M * st["L"].N * st["L"].K + 2 * st["L"].M * st["L"].r * st["L"].K for st in state)
    else:
        dom_flops = sum(2 * st["L"].M * st["L"].N * st["L"].K + 2 * st["L"].M * st["L"].r * st["L"].N for st in state)
    dom_flops /= len(state)
    achieved = dom_flops / (kernels_us[dom] * 1e-6) / 1e12
    traffic = read_traffic(args.workload)
    # the bandwidth-bound kernels: algorithmic bytes (one read of X or dY per launch) over their launch time
    stream_bytes = {"down": sum(2 * st["L"].M * st["L"].K for st in state) / len(state),
                    "ds_db": sum(2 * st["L"].M * st["L"].N for st in state) / len(state),
                    "da": sum(2 * st["L"].M * st["L"].K for st in state) / len(state)}
    stream_gbs = {k: round(b / (kernels_us[k] * 1e-6) / 1e9, 1) for k, b in stream_bytes.items() if kernels_us[k] > 0}

    out = {
        "metric": "fused LoRA linear fwd+bwd TFLOP/s and tokens/s at 1 MI355X; HBM bytes/token",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_steps": settle_steps,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": args.workload + ": " + ", ".join(
            f"{st['L'].name} M={st['L'].M} K={st['L'].K} N={st['L'].N} r={st['L'].r} G={st['L'].G} p={st['L'].p}"
            for st in state)},
        "step_ms": step_ms,
        "buffer_sets": len(sets),
        "launch": "hip graph replay" if args.graph else "eager",
        "tokens_per_s": round(tokens / (ms_per_step * 1e-3), 1),
        "frac_of_bf16_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "algorithmic_hbm_bytes_per_token": round(fused_bytes / tokens, 1),
        "kernel_us": {k: round(v, 2) for k, v in kernels_us.items()},
        "kernel_launches": launches,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under profiles/ (not taken by this run)"},
        "stream_kernels_gbs": stream_gbs,
        "peak_hbm_gbs": PEAK_HBM_GBS,
    }
    if ceilings:
        out["ceilings"] = ceilings
        out["roofline"]["measured_peak"] = ceilings["mfma_bf16_tflops"]
        out["roofline"]["frac_of_measured"] = round(achieved / ceilings["mfma_bf16_tflops"], 4)
        out["frac_of_measured_mfma_peak"] = round(tflops / ceilings["mfma_bf16_tflops"], 4)
        out["stream_kernels_frac_of_measured_read"] = {k: round(v / ceilings["hbm_read_gbs"], 4) for k, v in stream_gbs.items()}
        if "hbm_read_one_launch_gbs" in ceilings:
            out["stream_kernels_frac_of_one_launch_read"] = {k: round(v / ceilings["hbm_read_one_launch_gbs"], 4)
                                                             for k, v in stream_gbs.items()}

    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        L0 = state[0]["L"]
        f64 = lambda t: t.to(torch.float64).cpu().numpy()
        Xd, Wd, Ad, Bd, dYd = (f64(state[0][k]) for k in ("X", "W", "A", "B", "dY"))
        s, p = [L0.s] * L0.G, [L0.p] * L0.G
        # whole passes of the oracle over the layer until about ten seconds of CPU work are on the clock
        passes, t0 = 0, time.perf_counter()
        while passes == 0 or (time.perf_counter() - t0 < 10.0 and passes < 50):
            oracle.multi_lora_fwd(Xd, Wd, Ad, Bd, L0.seg_offsets, s, p, L0.seeds)
            oracle.multi_lora_bwd(Xd, Wd, Ad, Bd, dYd, L0.seg_offsets, s, p, L0.seeds)
            passes += 1
        total_s = time.perf_counter() - t0
        cpu_s = total_s / passes
        try:
            from threadpoolctl import threadpool_info
            cores = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": round(L0.flops / cpu_s / 1e12, 4), "unit": "TFLOP/s", "cores": int(cores),
                               "kind": "oracle", "sample": f"{passes} full fwd+bwd passes of layer {L0.name} "
                               f"(M={L0.M}), fp64 numpy, {total_s:.1f} s in all"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
