#!/usr/bin/env python3
"""Benchmark of the COMP-AMS optimizer step on one MI355X.

A "step" is one call of compams_step(): all n workers' error-feedback compression, the worker-ordered
average and the AMSGrad update, on gradients that already sit in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

The default workload is the one the headline metric is quoted on: n = 16 workers, d = 11 181 642
(ResNet-18-shaped), top-k with k/d = 1 %.  Gradients are seeded synthetic data (a distinct pre-generated
buffer per step, so the residuals evolve as they would in training).

`value` is the headline workload's.  The line also carries, under "workloads", a short run (10 timed steps after
12, a distinct gradient buffer per step) of every other workload of the build and, under "eps_out", the headline
workload with epsilon outside the square root: figures for the record, none of them enters `value`.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
OTHER_WORKLOADS = ["r18_topk01", "r18_blocksign", "r18_none", "r18_topk1_layers", "r50_topk1", "gpt2s_topk01",
                   "gpt2s_blocksign"]


def algorithmic_bytes(w, comp):
    """Minimum bytes one step must move (fp32): per worker-coordinate read g, read e, write e; per coordinate
    read+write theta, m, v, vhat; plus writing and reading the compressed messages."""
    n, d = w.n, w.d
    dense = 12 * n * d + 32 * d
    if comp in ("topk", "topk_blocks"):
        return dense + 16 * n * w.k
    if comp == "blocksign":
        M = len(w.block_offsets()) - 1
        return dense + 2 * n * (d // 8 + 4 * M)
    return 4 * n * d + 32 * d  # identity: g is read once, e does not exist


def dominant_kernel(comp):
    """(kernel slot name, algorithmic bytes per launch as a function of n, d)."""
    if comp in ("topk", "topk_blocks"):
        return "topk_pass_a", lambda n, d: 12 * n * d      # read g, read e, write x in place of e
    if comp == "blocksign":
        return "bs_pass1", lambda n, d: 12 * n * d
    return "none_amsgrad", lambda n, d: 4 * n * d + 32 * d


def load_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 3 and parts[0] == "hbm_bytes_per_launch" and parts[1] == kernel:
            return float(parts[2])
    return None


class Run:
    """One workload set up on the GPU: context, pre-generated gradients, and the timed loop."""

    def __init__(self, name, steps, warmup, grad_buffers=0, eps_mode=None, predict=True, force_dense=False, band=True,
                 cached_arrays=-1):
        import torch
        from paper_2205_05632_amd import binding as B
        from paper_2205_05632_amd import workloads as W
        self.torch, self.B, self.W = torch, B, W
        self.dev = torch.device("cuda:0")
        self.w = w = W.get(name)
        self.steps, self.warmup = steps, warmup
        self.blocks_topk = w.compressor == "topk_blocks"
        self.comp = {"topk": B.TOPK, "blocksign": B.BLOCKSIGN, "none": B.NONE, "topk_blocks": B.TOPK_BLOCKS}[w.compressor]
        self.eps_mode = B.EPS_IN_SQRT if eps_mode is None else eps_mode
        self.ctx = B.Compams(w.n, w.d, W.theta0(w, self.dev), compressor=self.comp, k=w.k,
                             block_offsets=w.block_offsets(), block_k=w.block_k() if self.blocks_topk else None,
                             eps_mode=self.eps_mode, device=self.dev)
        if not predict:
            self.ctx.set_option(B.OPT_PREDICT, 0)
        if force_dense:
            self.ctx.set_option(B.OPT_FORCE_DENSE, 1)
        if not band and self.comp in (B.TOPK, B.TOPK_BLOCKS):
            self.ctx.set_option(B.OPT_BAND, 0)
        if cached_arrays >= 0:
            self.ctx.set_option(B.OPT_CACHED_ARRAYS, cached_arrays)
        total = warmup + steps
        scale = W.coordinate_scale(w, self.dev)
        nbuf = total if grad_buffers <= 0 else min(total, grad_buffers)
        pool = [W.gradients(w, t, device=self.dev, ld=self.ctx.ld, scale=scale) for t in range(nbuf)]
        self.grads = [pool[t % nbuf] for t in range(total)]
        del scale
        torch.cuda.synchronize()

    def timed(self, event_mode=2, stride=4, settle_each_step=False):
        """Warm-up, then the timed steps between two synchronisations.  event_mode 2 brackets the dominant kernel
        with HIP events on the step's stream on every `stride`-th step (their cost is part of the measured time),
        1 brackets every kernel of every step, 0 none."""
        torch, ctx, w = self.torch, self.ctx, self.w
        for t in range(self.warmup):
            ctx.compams_step(self.grads[t], w.lr)
        stride = 1 if event_mode == 1 else max(1, stride)
        ctx.profile_enable(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(self.warmup, self.warmup + self.steps):
            if event_mode:
                ctx.profile_enable(event_mode if (t - self.warmup) % stride == 0 else 0)  # host-side switch only
            ctx.compams_step(self.grads[t], w.lr)
            if settle_each_step:
                ctx.compams_state("e")
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        prof = ctx.profile_read()
        ctx.profile_enable(0)
        sec = t1 - t0
        bmin = algorithmic_bytes(w, w.compressor)
        res = {"ms_per_step": sec / self.steps * 1e3, "steps_per_s": self.steps / sec, "prof": prof,
               "algorithmic_bytes_per_step": bmin, "hbm_gbps": bmin / (sec / self.steps) / 1e9}
        res["hbm_frac_of_peak"] = res["hbm_gbps"] / HBM_PEAK_GBPS
        kname, kbytes = dominant_kernel(w.compressor)
        res["roofline"] = None
        if prof and kname in prof:
            k_ms, k_launches = prof[kname]
            k_avg_s = k_ms / k_launches * 1e-3
            k_gbps = kbytes(w.n, w.d) / k_avg_s / 1e9
            res["roofline"] = {"bound": "hbm", "kernel": kname, "achieved": k_gbps, "peak": HBM_PEAK_GBPS,
                               "unit": "GB/s", "frac": k_gbps / HBM_PEAK_GBPS, "traffic": load_traffic(w.name, kname),
                               "traffic_source": f"profiles/traffic_{w.name}.txt (rocprofv3 --pmc FETCH_SIZE / "
                                                 "WRITE_SIZE runs of this command, committed; not measured in this run)",
                               "avg_launch_us": k_avg_s * 1e6, "launches_timed": k_launches,
                               "algorithmic_bytes_per_launch": kbytes(w.n, w.d)}
        return res

    def counters(self):
        B = self.B
        if self.comp not in (B.TOPK, B.TOPK_BLOCKS):
            return None
        c = self.ctx.compams_state("counters").cpu()
        if self.comp == B.TOPK:
            return {"dense_rereads_per_row_last_step": c[:, 0].tolist(),
                    "candidates_per_row_last_step": c[:, 1].tolist(),
                    "band_entries_per_row_last_step": c[:, 4].tolist(),       # > 0: selected in one launch
                    "problems_on_band_route_last_step": int((c[:, 4] > 0).sum()), "selection_problems": int(c.shape[0])}
        return {"selection_problems": int(c.shape[0]),   # one selection problem per (worker, block): totals
                "problems_on_band_route_last_step": int((c[:, 4] > 0).sum()),
                "problems_without_candidate_list_last_step": int((c[:, 0] == 4).sum()),
                "problems_with_one_reread_last_step": int((c[:, 0] == 1).sum()),
                "candidates_last_step": int(c[:, 1].sum())}

    def close(self):
        self.ctx.close()
        self.grads = None
        self.torch.cuda.empty_cache()


BRIEF_STEPS, BRIEF_WARMUP = 10, 12


def brief(name, eps_mode=None, stride=4):
    """The short run of a workload for the record: 10 timed steps after 12, a distinct gradient buffer per step (the
    selection settles on its steady-state route within about ten steps of a smoothly drifting threshold; a handful
    of buffers in rotation would make the threshold jump back and forth instead)."""
    r = Run(name, steps=BRIEF_STEPS, warmup=BRIEF_WARMUP, grad_buffers=0, eps_mode=eps_mode)
    m = r.timed(event_mode=2, stride=stride)
    c = r.counters()
    out = {"ms_per_step": m["ms_per_step"], "steps_per_s": m["steps_per_s"], "hbm_frac_of_peak": m["hbm_frac_of_peak"],
           "algorithmic_bytes_per_step": m["algorithmic_bytes_per_step"], "n": r.w.n, "d": r.w.d,
           "compressor": r.w.compressor, "steps": BRIEF_STEPS, "warmup": BRIEF_WARMUP,
           "grad_buffers": BRIEF_STEPS + BRIEF_WARMUP}
    if m["roofline"]:
        out["dominant_kernel"] = m["roofline"]["kernel"]
        out["dominant_kernel_us"] = m["roofline"]["avg_launch_us"]
        out["dominant_kernel_frac"] = m["roofline"]["frac"]
    if c and "dense_rereads_per_row_last_step" in c:
        out["dense_rereads_last_step"] = int(sum(c["dense_rereads_per_row_last_step"]))
    if c and "problems_on_band_route_last_step" in c:
        out["problems_on_band_route_last_step"] = c["problems_on_band_route_last_step"]
        out["selection_problems"] = c["selection_problems"]
    r.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="r18_topk1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="leave out the short runs of the other workloads and of the other epsilon form")
    ap.add_argument("--eps-out", action="store_true", help="epsilon outside the square root for the main run")
    ap.add_argument("--cpu-steps", type=int, default=10, help="oracle steps timed for the cpu_baseline leg")
    ap.add_argument("--kernels", action="store_true",
                    help="bracket every kernel with events and print the per-kernel table to stderr")
    ap.add_argument("--no-predict", action="store_true", help="ablation: re-read the row instead of guessing")
    ap.add_argument("--force-dense", action="store_true", help="ablation: no candidate lists at all")
    ap.add_argument("--no-band", action="store_true",
                    help="ablation: every selection by the general kernels (no window carried over for the threshold key)")
    ap.add_argument("--cached-arrays", type=int, default=-1,
                    help="ablation: how many of theta, m, v, vhat the server kernels keep in the memory-side cache "
                         "(0..4; default: the library's choice by size)")
    ap.add_argument("--grad-buffers", type=int, default=0,
                    help="how many distinct gradient buffers to cycle through (0: one per step)")
    ap.add_argument("--settle-each-step", action="store_true",
                    help="ablation: ask for e after every step, so that the residual zeroing is never deferred")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="time the steps without per-kernel events (the roofline object is then left out)")
    ap.add_argument("--event-stride", type=int, default=4,
                    help="bracket the dominant kernel with events on every this-many-th timed step (each bracketed "
                         "launch adds a few microseconds to its step)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the n workers are rows of one buffer); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2205_05632_amd import binding as B
    from paper_2205_05632_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    run = Run(args.workload, args.steps, args.warmup, grad_buffers=args.grad_buffers,
              eps_mode=B.EPS_OUT_SQRT if args.eps_out else B.EPS_IN_SQRT, predict=not args.no_predict,
              force_dense=args.force_dense, band=not args.no_band, cached_arrays=args.cached_arrays)
    w, ctx, comp, grads = run.w, run.ctx, run.comp, run.grads
    event_mode = 0 if args.no_kernel_events else (1 if args.kernels else 2)
    main_res = run.timed(event_mode=event_mode, stride=args.event_stride, settle_each_step=args.settle_each_step)
    prof = main_res["prof"]
    kernel_sum_ms = sum(ms / cnt for ms, cnt in prof.values()) if prof else None
    counters = run.counters()
    if args.kernels:
        for name, (ms, cnt) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
            print(f"  {name:16s} {ms / cnt * 1e3:9.1f} us/launch  x{cnt}", file=sys.stderr)

    # a second look at the same steps, one pair of events per step: median and minimum (each figure includes
    # the cost of its events; `value` above does not)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i, (a, b) in enumerate(ev):
        a.record()
        ctx.compams_step(grads[args.warmup + i], w.lr)
        b.record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in ev)
    step_ms_median, step_ms_min = per_step[len(per_step) // 2], per_step[0]

    # what the box gives a plain copy (1 GiB read + 1 GiB written per launch): the practical ceiling beside the
    # published peak
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        B.compams_copy(dst, src)
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    for _ in range(10):
        B.compams_copy(dst, src)
    torch.cuda.synchronize()
    copy_gbps = 2.0 * (1 << 30) / ((time.perf_counter() - c0) / 10) / 1e9

    # what the box gives the access pattern of the server's lines (theta, m, v, vhat of the workload's size read and
    # written once, in place, nothing else): each launch follows a copy of 2 GiB of traffic, as a step's server
    # kernel follows its first pass; with as many of the four arrays kept in the memory-side cache as the library
    # keeps for this size, and with none and all four beside it
    quads = (w.d + 3) // 4 * 4
    state = [torch.zeros(quads, dtype=torch.float32, device=dev) for _ in range(4)]
    kept = B.compams_cached_state_arrays(w.d)
    server_ceiling = {"arrays": 4, "elements_each": quads, "bytes_per_launch": 32 * quads, "library_caches": kept}
    for cached in sorted({0, kept, 4}):
        pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
        for a, b in pe:
            B.compams_copy(dst, src)
            a.record()
            B.compams_inplace_probe(state, cached)
            b.record()
        torch.cuda.synchronize()
        us = sorted(a.elapsed_time(b) * 1e3 for a, b in pe[2:])
        server_ceiling[f"cached_{cached}"] = {"us_median": us[len(us) // 2], "us_min": us[0],
                                              "gbps_median": 32 * quads / us[len(us) // 2] / 1e3}
    del src, dst, state

    # the last step's messages on the wire: sizes (32 bits per word, the accounting of the paper's experiments
    # section) and the time to pack and unpack them; not part of `value`
    wire = None
    if comp != B.NONE:
        reps = 20
        msgs, words = ctx.compams_encode()      # warm-up: first launches load the kernels
        ctx.compams_decode(msgs, words)
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        for _ in range(reps):
            msgs, words = ctx.compams_encode()
        torch.cuda.synchronize()
        w1 = time.perf_counter()
        for _ in range(reps):
            ctx.compams_decode(msgs, words)
        torch.cuda.synchronize()
        w2 = time.perf_counter()
        bits = 32.0 * float(words.float().mean().item())
        wire = {"bits_per_worker": bits, "full_gradient_bits": 32.0 * w.d, "reduction": 32.0 * w.d / bits,
                "encode_us": (w1 - w0) / reps * 1e6, "decode_us": (w2 - w1) / reps * 1e6}
        if comp in (B.TOPK, B.TOPK_BLOCKS):
            tiles = (w.k + 255) // 256
            wire["gap_bits_mean"] = (bits / 32.0 - 3 - (tiles + 3) // 4 - w.k) * 32.0 / w.k
            wire["reduction_values_only"] = w.d / w.k
        del msgs, words

    # the inputs of the oracle's leg come off the GPU before its memory goes to the other workloads; the leg itself
    # runs last, so that the GPU does not sit idle (and clock down) in front of timed GPU work
    host = None
    if not args.no_cpu_baseline:
        host = [grads[t][:, : w.d].cpu().contiguous().numpy() for t in range(min(args.cpu_steps, len(grads)))]
        theta0_host = W.theta0(w, dev).cpu().numpy()
    blocks_topk, eps_mode_main = run.blocks_topk, run.eps_mode
    run.close()
    del grads, run, ctx

    others, eps_out = None, None
    if not args.no_others:
        eps_out = brief(args.workload, eps_mode=B.EPS_IN_SQRT if args.eps_out else B.EPS_OUT_SQRT,
                        stride=args.event_stride)
        eps_out["eps_mode"] = "in_sqrt" if args.eps_out else "out_sqrt"
        others = {}
        for name in OTHER_WORKLOADS:
            if name != args.workload:
                others[name] = brief(name, stride=args.event_stride)

    cpu = None
    if host is not None:
        from oracle import compams_oracle as O
        ocomp = {"topk": O.TOPK, "blocksign": O.BLOCKSIGN, "none": O.NONE, "topk_blocks": O.TOPK_BLOCKS}[w.compressor]
        orc = O.Oracle(w.n, w.d, theta0_host, compressor=ocomp, k=w.k,
                       block_offsets=w.block_offsets(), block_k=w.block_k() if blocks_topk else None,
                       eps_mode=eps_mode_main)
        c0 = time.perf_counter()
        for g in host:
            orc.step(g, w.lr)
        c1 = time.perf_counter()
        cpu = {"value": len(host) / (c1 - c0), "unit": "steps/s", "cores": 1, "kind": "oracle",
               "sample": f"first {len(host)} steps of the same workload and inputs, single thread"}
        orc.close()
        del host

    out = {
        "metric": "compressed-AMSGrad steps/sec and HBM GB/s (% of peak), n=16, d=11.2M, top-k 1%",
        "value": main_res["steps_per_s"], "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "d": w.d, "compressor": w.compressor, "k": w.k,
                   "num_blocks": (len(w.block_offsets()) - 1) if w.compressor == "blocksign" else 0,
                   "eps_mode": "out_sqrt" if args.eps_out else "in_sqrt",
                   "predict": not args.no_predict, "force_dense": args.force_dense, "band": not args.no_band,
                   "cached_state_arrays": args.cached_arrays if args.cached_arrays >= 0
                   else B.compams_cached_state_arrays(w.d)},
        "hbm_gbps": main_res["hbm_gbps"],
        "hbm_frac_of_peak": main_res["hbm_frac_of_peak"],
        "algorithmic_bytes_per_step": main_res["algorithmic_bytes_per_step"],
        "step_ms_median": step_ms_median, "step_ms_min": step_ms_min,
        "copy_kernel_gbps": copy_gbps, "hbm_frac_of_copy_kernel": main_res["hbm_gbps"] / copy_gbps,
        "server_lines_ceiling": server_ceiling,
        "kernel_ms_per_step": kernel_sum_ms,
        "roofline": main_res["roofline"],
        "kernels_us_per_launch": {k_: v_[0] / v_[1] * 1e3 for k_, v_ in prof.items()},
        "topk_counters": counters,
        "wire": wire,
        "cpu_baseline": cpu,
        "eps_out": eps_out,
        "workloads": others,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
