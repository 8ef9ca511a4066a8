#!/usr/bin/env python3
"""Benchmark of the COMP-AMS optimizer step on one MI355X.

A "step" is one call of compams_step(): all n workers' error-feedback compression, the worker-ordered
average and the AMSGrad update, on gradients that already sit in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

The default workload is the one the headline metric is quoted on: n = 16 workers, d = 11 181 642
(ResNet-18-shaped), top-k with k/d = 1 %.  Gradients are seeded synthetic data (a distinct pre-generated
buffer per step, so the residuals evolve as they would in training).
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
    if comp == "topk":
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="r18_topk1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=10, help="oracle steps timed for the cpu_baseline leg")
    ap.add_argument("--kernels", action="store_true",
                    help="bracket every kernel with events and print the per-kernel table to stderr")
    ap.add_argument("--no-predict", action="store_true", help="ablation: re-read the row instead of guessing")
    ap.add_argument("--force-dense", action="store_true", help="ablation: no candidate lists at all")
    ap.add_argument("--compose-blocks", action="store_true",
                    help="top-k per layer tensor as one context per tensor, stepped one after the other")
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
    w = W.get(args.workload)
    blocks_topk = w.compressor == "topk_blocks"
    # --compose-blocks: one context per layer tensor stepped one after the other (no per-kernel events, no codec)
    per_block = blocks_topk and args.compose_blocks
    if per_block:
        comp = None
        ctx = B.CompamsBlockTopk(w.n, w.d, W.theta0(w, dev), w.block_offsets(), w.block_k(), device=dev)
        args.no_kernel_events = True
    else:
        comp = {"topk": B.TOPK, "blocksign": B.BLOCKSIGN, "none": B.NONE, "topk_blocks": B.TOPK_BLOCKS}[w.compressor]
        ctx = B.Compams(w.n, w.d, W.theta0(w, dev), compressor=comp, k=w.k, block_offsets=w.block_offsets(),
                        block_k=w.block_k() if blocks_topk else None, device=dev)
    if args.no_predict and not per_block:
        ctx.set_option(B.OPT_PREDICT, 0)
    if args.force_dense and not per_block:
        ctx.set_option(B.OPT_FORCE_DENSE, 1)

    total = args.warmup + args.steps
    scale = W.coordinate_scale(w, dev)
    nbuf = total if args.grad_buffers <= 0 else min(total, args.grad_buffers)
    pool = [W.gradients(w, t, device=dev, ld=ctx.ld, scale=scale) for t in range(nbuf)]
    grads = [pool[t % nbuf] for t in range(total)]
    torch.cuda.synchronize()

    for t in range(args.warmup):
        ctx.compams_step(grads[t], w.lr)
    # timed region: the dominant kernel is bracketed by HIP events on the step's stream (their cost is part of
    # the measured time); --kernels brackets every kernel instead, which costs a few microseconds per kernel
    event_mode = 0 if args.no_kernel_events else (1 if args.kernels else 2)
    stride = 1 if args.kernels else max(1, args.event_stride)
    if not per_block:
        ctx.profile_enable(0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.warmup, total):
        if event_mode and stride > 1:
            ctx.profile_enable(event_mode if (t - args.warmup) % stride == 0 else 0)  # host-side switch only
        elif t == args.warmup and not per_block:
            ctx.profile_enable(event_mode)
        ctx.compams_step(grads[t], w.lr)
        if args.settle_each_step:
            ctx.compams_state("e")
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = {} if per_block else ctx.profile_read()
    if not per_block:
        ctx.profile_enable(0)
    sec = t1 - t0
    ms_per_step = sec / args.steps * 1e3
    steps_per_s = args.steps / sec

    bmin = algorithmic_bytes(w, w.compressor)
    kname, kbytes = dominant_kernel("topk" if blocks_topk else w.compressor)
    roofline = None
    kernel_sum_ms = None
    if prof:
        k_ms, k_launches = prof[kname]
        k_avg_s = k_ms / k_launches * 1e-3
        k_gbps = kbytes(w.n, w.d) / k_avg_s / 1e9
        kernel_sum_ms = sum(ms / cnt for ms, cnt in prof.values())
        roofline = {"bound": "hbm", "kernel": kname, "achieved": k_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": k_gbps / HBM_PEAK_GBPS, "traffic": load_traffic(w.name, kname),
                    "avg_launch_us": k_avg_s * 1e6, "launches_timed": k_launches,
                    "algorithmic_bytes_per_launch": kbytes(w.n, w.d)}

    counters = None
    if comp in (B.TOPK, B.TOPK_BLOCKS):
        c = ctx.compams_state("counters").cpu()
        if comp == B.TOPK:
            counters = {"dense_rereads_per_row_last_step": c[:, 0].tolist(),
                        "candidates_per_row_last_step": c[:, 1].tolist()}
        else:   # one selection problem per (worker, block): totals
            counters = {"selection_problems": int(c.shape[0]),
                        "problems_without_candidate_list_last_step": int((c[:, 0] == 4).sum()),
                        "problems_with_one_reread_last_step": int((c[:, 0] == 1).sum()),
                        "candidates_last_step": int(c[:, 1].sum())}
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
    del src, dst

    # the last step's messages on the wire: sizes (32 bits per word, the accounting of the paper's experiments
    # section) and the time to pack and unpack them; not part of `value`
    wire = None
    if comp is not None and comp != B.NONE:
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

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import compams_oracle as O
        ocomp = {"topk": O.TOPK, "blocksign": O.BLOCKSIGN, "none": O.NONE, "topk_blocks": O.TOPK_BLOCKS}[w.compressor]
        orc = O.Oracle(w.n, w.d, W.theta0(w, dev).cpu().numpy(), compressor=ocomp, k=w.k,
                       block_offsets=w.block_offsets(), block_k=w.block_k() if blocks_topk else None)
        host = [grads[t][:, : w.d].cpu().contiguous().numpy() for t in range(args.cpu_steps)]
        c0 = time.perf_counter()
        for g in host:
            orc.step(g, w.lr)
        c1 = time.perf_counter()
        cpu = {"value": args.cpu_steps / (c1 - c0), "unit": "steps/s", "cores": 1, "kind": "oracle",
               "sample": f"first {args.cpu_steps} steps of the same workload and inputs, single thread"}
        orc.close()

    out = {
        "metric": "compressed-AMSGrad steps/sec and HBM GB/s (% of peak), n=16, d=11.2M, top-k 1%",
        "value": steps_per_s, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "d": w.d, "compressor": w.compressor, "k": w.k,
                   "num_blocks": (len(w.block_offsets()) - 1) if w.compressor == "blocksign" else 0,
                   "predict": not args.no_predict, "force_dense": args.force_dense},
        "hbm_gbps": bmin / (sec / args.steps) / 1e9,
        "hbm_frac_of_peak": bmin / (sec / args.steps) / 1e9 / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_step": bmin,
        "step_ms_median": step_ms_median, "step_ms_min": step_ms_min,
        "copy_kernel_gbps": copy_gbps, "hbm_frac_of_copy_kernel": bmin / (sec / args.steps) / 1e9 / copy_gbps,
        "kernel_ms_per_step": kernel_sum_ms,
        "roofline": roofline,
        "kernels_us_per_launch": {k_: v_[0] / v_[1] * 1e3 for k_, v_ in prof.items()},
        "topk_counters": counters,
        "wire": wire,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
