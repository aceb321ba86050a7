#!/usr/bin/env python3
"""Throughput of the DEF / DEF-A compression-and-update step on one MI355X.

One "step" is one pass of the whole hot path (block draw, fused momentum +
error-feedback + residual pass over all W workers, cross-worker average of the
kept block, parameter update) over one set of synthetic per-worker gradients
that is already resident in HBM.

Default workload: the ResNet-50-shaped configuration (d = 25,557,032 parameters
in 161 tensors, W = 16 workers, ratio 1/128, momentum 0.9, weight decay 1e-4).

Prints ONE JSON line.  `value` is the algorithmic HBM traffic of a step divided
by the measured time per step; `roofline` prices the streaming kernel alone
(measured with HIP events around each of its launches, on the stream it runs on)
against the 8 TB/s HBM peak; `cpu_baseline` times the plain C oracle on this
host's cores on a bounded number of steps of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E peak, GB/s

# HBM bytes per launch of the streaming kernel from rocprofv3 FETCH_SIZE + WRITE_SIZE,
# each scaled by what the same counter reads for a 1 GiB copy
# (profiles/def_stream_vec4_kernel_resnet50_shaped_hbm_counters.md).  Keyed by workload
# and by the exact kernel instantiation, so a changed kernel reports null until the
# counters are taken again.
MEASURED_TRAFFIC = {
    ("resnet50_shaped",
     "def_stream_vec4_kernel<mu=1,wd=1,detach=0,tables=0,threads=64,quads=1,nt=1,order=blocked:16384,sweep=alternating,lds=8960>"): 8293526202,
}


def algorithmic_bytes(w, y_out=False, detach=False):
    """Bytes the method itself must move per step (fp32): per (worker, index) one
    gradient read, error memory read+write and, with momentum, momentum read+write;
    plus x: read once everywhere when weight decay needs it, else read on the
    block; written on the block.  The compact staging of the kept block between
    the two kernels is not counted."""
    per_elem = 12 + (8 if w.momentum != 0 else 0)
    stream = w.W * w.d * per_elem
    if w.weight_decay != 0:
        stream_x, block = 4 * w.d, 4 * w.B
    else:
        stream_x, block = 0, 8 * w.B
    extra = 0
    if y_out:
        extra = 4 * w.d + (0 if w.weight_decay != 0 else 4 * w.d)
    if detach:
        # w_k = x - lambda*e_k: one more write per (worker, index); x read once everywhere
        stream += 4 * w.W * w.d
        if w.weight_decay == 0:
            stream_x, block = 4 * w.d, 4 * w.B
    return dict(step=stream + stream_x + block + extra, stream_kernel=stream + stream_x)


def cpu_baseline(w, ld, budget_s=15.0):
    """Time the plain C oracle (oracle/def_oracle.c, as it stands) on this host:
    full d and W of the workload, as many steps as fit the budget."""
    import numpy as np
    from oracle.c_oracle import DefOracleC
    from paper_2004_05298_amd import workloads as wl

    x0 = wl.initial_params(w)
    g = wl.gradient_set(w, 0, ld=w.d, threads=16)
    ora = DefOracleC(x0, w.W, w.R, w.lr, w.momentum, w.weight_decay, w.seed)
    ora.step(g)                     # first touch of the state pages, not timed
    steps, t0 = 0, time.perf_counter()
    while True:
        ora.step(g)
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or steps >= w.T:
            break
    per_step = dt / steps
    ab = algorithmic_bytes(w)["step"]
    # the same oracle on one thread: a couple of steps, bounded by a fifth of the budget
    all_threads = ora.threads
    ora.set_threads(1)
    steps1, t1 = 0, time.perf_counter()
    while True:
        ora.step(g)
        steps1 += 1
        dt1 = time.perf_counter() - t1
        if dt1 >= budget_s / 5 or steps1 >= 3:
            break
    ora.set_threads(all_threads)
    return {
        "value": ab / per_step / 1e9, "unit": "GB/s", "cores": all_threads, "kind": "oracle",
        "steps_per_s": 1.0 / per_step,
        "sample": f"{steps} full steps of {w.name} (d={w.d}, W={w.W}) by the plain C oracle "
                  f"with {all_threads} OpenMP threads, after one untimed step",
        "one_thread": {"value": ab / (dt1 / steps1) / 1e9, "unit": "GB/s",
                       "steps_per_s": steps1 / dt1, "sample": f"{steps1} full steps"},
        "cpu_model": cpu_model(), "host_cpus": os.cpu_count(),
    }


def run_probes(torch, binding, stream, src, n, reps=20):
    """What plain streaming kernels of known traffic sustain on this GPU, right after the
    timed steps: pure read, pure write, copy and in-place update over a buffer of the size
    of one state buffer, the best of seven launch shapes each (among them the streaming
    pass's own, with and without its residency cap).  Context for the roofline fraction,
    not part of the step."""
    n = min(n, 1 << 29) // 256 * 256
    if src is None:
        src = torch.zeros(n, dtype=torch.float32, device="cuda")
    # the destination can sit 12 KiB further than its allocation's alignment: where the two
    # buffers of a copy sit relative to each other matters on this GPU
    SKEW = 12288 // 4
    dst_buf = torch.zeros(n + SKEW, dtype=torch.float32, device="cuda")
    kinds = [("read", binding.PROBE_READ, 4 * n), ("write", binding.PROBE_WRITE, 4 * n),
             ("copy", binding.PROBE_COPY, 8 * n), ("update_in_place", binding.PROBE_UPDATE, 8 * n)]
    out = {"bytes_per_buffer": 4 * n, "launches_each": reps}
    shapes = [(64, 1, 0), (64, 1, 10240), (64, 2, 0), (64, 4, 0), (256, 1, 0), (256, 2, 0), (256, 4, 0)]
    for name, kind, nbytes in kinds:
        best, every = None, {}
        for threads, quads, lds, skew in [sh + (0,) for sh in shapes] + (
                [sh + (SKEW,) for sh in shapes[:1] + shapes[2:5]] if name == "copy" else []):
            dst = dst_buf[skew:skew + n]

            def launch():
                binding.probe_stream(kind, src, dst, n, 1.0, threads, quads, lds, stream)
            launch()
            launch()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                launch()
            b.record()
            torch.cuda.synchronize()
            gbs = nbytes / (a.elapsed_time(b) / reps) / 1e6
            every[f"{threads}x{quads}/{lds}" + ("+12K" if skew else "")] = round(gbs)
            if best is None or gbs > best[0]:
                best = (gbs, f"{threads} threads x {quads} float4, lds {lds}"
                        + (", destination 12 KiB past the source's alignment" if skew else ""))
        out[name] = {"GB/s": round(best[0], 1), "frac_of_peak": round(best[0] / HBM_PEAK_GBS, 4),
                     "best_shape": best[1], "all_shapes_GB/s": every}
    return out


def skewed_rows(torch, W, ld, offset_bytes):
    """A [W][ld] float32 device tensor that starts offset_bytes past its allocation's alignment."""
    assert offset_bytes % 16 == 0
    buf = torch.empty(W * ld + offset_bytes // 4, dtype=torch.float32, device="cuda")
    return buf[offset_bytes // 4:].view(W, ld)


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet50_shaped")
    ap.add_argument("--variant", default=None, choices=[None, "def", "def_a"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=15.0)
    ap.add_argument("--detach", type=float, default=None, metavar="LAMBDA",
                    help="also write the detached evaluation points w_k = x - LAMBDA*e_k in the "
                         "same pass (24 instead of 20 bytes per worker and index)")
    ap.add_argument("--workers", type=int, default=None, metavar="W",
                    help="override the workload's number of workers on this GPU (W = 1 is one GPU's "
                         "share when the workers are spread one per GPU)")
    ap.add_argument("--momentum", type=float, default=None, metavar="MU",
                    help="override the workload's momentum (0 drops the momentum buffer: three streams "
                         "per worker and index instead of five)")
    ap.add_argument("--weight-decay", type=float, default=None, metavar="WD",
                    help="override the workload's weight decay (0: the pass does not read x)")
    ap.add_argument("--split", action="store_true",
                    help="run every iteration as def_pack + def_apply (the two halves between which "
                         "a multi-GPU deployment would all-reduce the kept block), applying the "
                         "local sum with divisor W")
    ap.add_argument("--with-y", action="store_true",
                    help="def_step also writes DEF's output y = x - mean_k e_k every step (a second "
                         "pass over the error memories; the paper needs y only when the model is "
                         "evaluated, so the default step does not)")
    ap.add_argument("--graph", type=int, default=0, metavar="N",
                    help="capture N consecutive steps (device-side block draw) into one HIP graph "
                         "and time replays of it instead of eager launches; for the small, "
                         "launch-bound workloads.  No per-kernel timing in this mode.")
    ap.add_argument("--aux", action="store_true",
                    help="also time the occasional kernels (DEF output y, stand-alone detached "
                         "points, error-memory statistics) and report them under aux_kernels")
    ap.add_argument("--tensors", action="store_true",
                    help="give gradients and parameters per tensor (def_step_tensors with a "
                         "pointer table), each tensor starting on a 256-byte boundary as a "
                         "framework's allocator would place it")
    ap.add_argument("--misaligned", action="store_true",
                    help="offset the gradient buffers by one float (rows 4-byte but not 16-byte "
                         "aligned)")
    ap.add_argument("--kernel-timing", default="two-pass", choices=["two-pass", "inline"],
                    help="two-pass: the K timed steps run without per-launch events (value, ms_per_step), "
                         "then K more steps run with a HIP event pair around every streaming launch "
                         "(roofline); inline: the event pairs are recorded inside the timed steps")
    ap.add_argument("--w-offset", type=int, default=0, metavar="BYTES",
                    help="start the buffer of the detached points this many bytes (a multiple of 16) past "
                         "its allocation's alignment")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="N",
                    help="first run N launches of the library's plain copy probe on a 1 GiB buffer (a "
                         "kernel of known traffic, 2^30 bytes read and 2^30 written per launch, against "
                         "which hardware counters are scaled); not part of the timed region")
    ap.add_argument("--no-probes", action="store_true",
                    help="skip the plain read / write / copy / in-place probes (include/def_probe.h) that "
                         "are timed after the steps to show what this GPU sustains in the same run")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs all W workers' shares on ONE GPU; there is no "
              "multi-GPU path, run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2004_05298_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if not os.path.exists(binding._build.library_path()):
        binding._build.build_library()
    binding.load_library()
    torch.cuda.set_device(0)

    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.copy_calibration):
            binding.probe_stream(binding.PROBE_COPY, src, dst, 1 << 28, 1.0, 64, 1, 0,
                                 torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        del src, dst

    w = wl.by_name(args.workload)
    if args.workers is not None:
        w = w.replace(W=args.workers)
    if args.momentum is not None:
        w = w.replace(momentum=args.momentum)
    if args.weight_decay is not None:
        w = w.replace(weight_decay=args.weight_decay)
    variant = args.variant or ("def_a" if w.variant == "def_a" else "def")
    if args.with_y and variant == "def_a":
        print("bench.py: --with-y asks for DEF's output; DEF-A's output is x itself", file=sys.stderr)
        return 2
    ld = wl.padded_ld(w.d)
    x = torch.from_numpy(wl.initial_params(w)).cuda()
    pool = wl.device_gradient_pool(w, ld)
    if args.misaligned:
        shifted = []
        for g in pool:
            buf = torch.empty(g.numel() + 4, dtype=torch.float32, device="cuda")
            buf[1:1 + g.numel()].copy_(g.view(-1))
            shifted.append(buf[1:1 + g.numel()].view(w.W, ld))
        pool = shifted
    grad_tables = param_tensors = None
    if args.tensors:
        off = [int(v) for v in w.tensor_offsets()]
        starts, pos = [], 0
        for l in range(w.n_tensors):
            starts.append(pos)
            pos += -(-(off[l + 1] - off[l]) // 64) * 64          # next 256-byte boundary
        xbuf = torch.zeros(pos, dtype=torch.float32, device="cuda")
        param_tensors = []
        for l in range(w.n_tensors):
            view = xbuf[starts[l]:starts[l] + off[l + 1] - off[l]]
            view.copy_(x[off[l]:off[l + 1]])
            param_tensors.append(view)
        grad_tables = []
        for g in pool:
            gbuf = torch.zeros((w.W, pos), dtype=torch.float32, device="cuda")
            table = []
            for k in range(w.W):
                for l in range(w.n_tensors):
                    view = gbuf[k, starts[l]:starts[l] + off[l + 1] - off[l]]
                    view.copy_(g[k, off[l]:off[l + 1]])
                    table.append(view)
            grad_tables.append(table)
        pool = None
    side = torch.cuda.Stream() if args.graph else None
    if side is not None:
        side.wait_stream(torch.cuda.current_stream())
        torch.cuda.set_stream(side)
    stream = torch.cuda.current_stream().cuda_stream
    ctx = binding.DefContext(w.d, w.W, w.R, w.lr, w.momentum, w.weight_decay, w.seed,
                             params=None if args.tensors else x, param_tensors=param_tensors,
                             tensor_offsets=w.tensor_offsets(), stream=stream)

    w_out = None
    if args.detach is not None:
        w_out = skewed_rows(torch, w.W, ld, args.w_offset)
        ctx.set_detach(w_out, ld, args.detach)

    y_out = torch.empty(w.d, dtype=torch.float32, device="cuda") if args.with_y else None

    def one_step(t):
        forced = w.forced_start(t)
        if forced is not None:
            ctx.force_next_start(forced)
        if args.split:
            block = (ctx.pack_tensors(grad_tables[t % w.pool]) if grad_tables is not None
                     else ctx.pack(pool[t % w.pool], ld))
            ctx.apply(block, float(w.W), y_out)
        elif grad_tables is not None:
            ctx.step_tensors(grad_tables[t % w.pool], y_out)
        elif variant == "def_a":
            ctx.a_step(pool[t % w.pool], ld)
        else:
            ctx.step(pool[t % w.pool], ld, y_out)

    t = 0
    for _ in range(args.warmup):
        one_step(t)
        t += 1
    torch.cuda.synchronize()
    if args.graph:
        ctx.set_device_draw(True)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for q in range(args.graph):
                one_step(t + q)
        replays = max(1, args.steps // args.graph)
        args.steps = replays * args.graph
        graph.replay()                                   # one untimed replay
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        kernel_ms = None
    else:
        if args.kernel_timing == "inline":
            ctx.profile_begin(args.steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_step(t)
            t += 1
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        if args.kernel_timing == "two-pass":
            # the same K steps again, each streaming launch between two HIP events on its stream
            ctx.profile_begin(args.steps)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                one_step(t)
                t += 1
            torch.cuda.synchronize()
            elapsed_events = time.perf_counter() - t1
        else:
            elapsed_events = elapsed
        kernel_ms = ctx.profile_end(args.steps)
    kernel_name = ctx.last_kernel()
    aux = None
    if args.aux:
        y = torch.empty(w.d, dtype=torch.float32, device="cuda")
        wbuf = w_out if w_out is not None else skewed_rows(torch, w.W, ld, args.w_offset)
        stats = torch.zeros(4, dtype=torch.float64, device="cuda")
        stats_w = torch.zeros(3 * w.W, dtype=torch.float64, device="cuda")
        state = 4 * w.W * w.d

        def timed(fn, nbytes, reps=20):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / reps
            return {"ms": round(ms, 5), "GB/s": round(nbytes / ms / 1e6, 1), "algorithmic_bytes": nbytes}

        aux = {
            "def_output": timed(lambda: ctx.output(y), state + 8 * w.d),
            "def_detach": timed(lambda: ctx.detach(wbuf, ld, 0.3), 2 * state + 4 * w.d),
            "def_diagnostics": timed(lambda: ctx.diagnostics(0.3, stats), state),
            "def_diagnostics_workers": timed(lambda: ctx.diagnostics_workers(stats_w), state * -(-w.W // 16)),
        }
    ctx.destroy()
    probes = None
    if not args.no_probes and not args.graph:
        probes = run_probes(torch, binding, stream, pool[0] if pool is not None else None, w.W * ld)

    ab = algorithmic_bytes(w, y_out=args.with_y, detach=args.detach is not None)
    per_step = elapsed / args.steps
    value = ab["step"] / per_step / 1e9
    if kernel_ms:
        k_avg_ms = sum(kernel_ms) / len(kernel_ms)
        achieved = ab["stream_kernel"] / (k_avg_ms * 1e-3) / 1e9
    else:
        k_avg_ms = achieved = None
    out = {
        "metric": "DEF step throughput: achieved HBM GB/s (% of peak) and steps/s at d, W",
        "value": round(value, 2), "unit": "GB/s",
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "steps_per_s": round(1.0 / per_step, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(per_step * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "d": w.d, "W": w.W, "R": w.R, "B": w.B,
                   "n_tensors": w.n_tensors, "momentum": w.momentum,
                   "weight_decay": w.weight_decay, "lr": w.lr, "variant": variant, "split": bool(args.split), "y_every_step": bool(args.with_y), "detach_lambda": args.detach,
                   "gradient_sets": w.pool, "inputs": "per-tensor pointers" if args.tensors else "flat", "launch": f"hip graph of {args.graph} steps" if args.graph else "eager",
                   "algorithmic_bytes_per_step": ab["step"]},
        "roofline": {"bound": "hbm", "kernel": kernel_name,
                     "achieved": None if achieved is None else round(achieved, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": None if achieved is None else round(achieved / HBM_PEAK_GBS, 4),
                     "avg_launch_ms": None if k_avg_ms is None else round(k_avg_ms, 5),
                     "launches": len(kernel_ms) if kernel_ms else 0,
                     "min_launch_ms": round(min(kernel_ms), 5) if kernel_ms else None,
                     "median_launch_ms": round(sorted(kernel_ms)[len(kernel_ms) // 2], 5) if kernel_ms else None,
                     "algorithmic_bytes_per_launch": ab["stream_kernel"],
                     "timed_in": None if not kernel_ms else (
                         "the timed steps themselves" if args.kernel_timing == "inline" else
                         f"a second pass of {args.steps} steps right after the timed ones, "
                         f"{elapsed_events / args.steps * 1e3:.5f} ms per step with the events"),
                     "traffic": MEASURED_TRAFFIC.get((w.name, kernel_name)),
                     "traffic_source": "rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this kernel "
                                       "on this workload (profiles/), not of this run"
                                       if MEASURED_TRAFFIC.get((w.name, kernel_name)) else None},
    }
    if aux is not None:
        out["aux_kernels"] = aux
    if probes is not None:
        out["probes"] = probes
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, ld, args.cpu_budget)
        for part in (out["cpu_baseline"], out["cpu_baseline"]["one_thread"]):
            for k in ("value", "steps_per_s"):
                part[k] = round(part[k], 3)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
