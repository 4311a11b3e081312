#!/usr/bin/env python3
"""Benchmark of the signature hot path on one MI355X.

A step is one `sig_forward` call over one batch of synthetic paths (increments are
differenced, folded in with the fused multiply-exponentiate and the result stored, all
inside the library).  Inputs and outputs are resident in HBM before the timed region.
Prints ONE JSON line: paths/s, the roofline of the dominant kernel measured live with
HIP events, and the CPU oracle timed on the host cores beside it.

Timing (the paper's protocol, section 6.1: repeat 50 times, take the fastest; here the median is reported as well):
* `value` / `ms_per_step`: exactly `--steps` calls between two device synchronisations, host clock.
* kernel time: `--repeats` (default 50) batches of R back-to-back calls, each batch bracketed by one HIP event pair
  on the stream the kernels run on, R chosen so that a batch lasts at least `--min-batch-ms` (default 2 ms) whatever
  `--steps` is.  The batches are issued twice: call by call through the binding, and as one replay of a HIP graph
  holding the R calls (no host work between the kernels: the GPU-side rate of calls shorter than a Python call).
  The roofline uses the smaller of the two medians per call.
* measured peaks: short microbenchmarks (fp32 matrix-core and vector multiply-adds, HBM fill and copy; libsig_peaks)
  timed the same way, so that the fraction is also stated against what this very device delivers.

`--op backward` times `sig_backward` (the gradient with respect to the path), `--op combine` times `sig_combine` (the
group product of two batches of signatures), `--op logsignature` the forward pass followed by `sig_log` and
`sig_lyndon_gather`, `--op logsignature_backward` the gradient of that (`sig_lyndon_scatter`, `sig_log_backward`,
`sig_backward`), on the same workload shapes instead; the default, and the metric this repository is judged on, is
the forward pass.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Published MI355X peaks used for the roofline fractions.
PEAK_FP32_TFLOPS = 157.3   # fp32 matrix-core peak = fp32 vector peak (packed) = 256 CU x 256 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0


def flops_per_increment(d: int, N: int, fused_fmas: int) -> int:
    """Algorithmic work of one fused multiply-exponentiate: M(d,N) multiply-adds plus the
    d(N-1) scalings z/2..z/N and the dN additions of eq. "fusedterm"."""
    return 2 * fused_fmas + d * (2 * N - 1)


def backward_flops_per_increment(d: int, N: int, fused_fmas: int, channels: int) -> int:
    """Algorithmic work of one backward step: M + N d multiply-adds to undo the increment and form the
    Horner terms, M for the chains contracted with the increment, M + N d for the increment's gradient,
    and M + N d - S additions into the cotangent of the earlier state."""
    return 2 * (3 * fused_fmas + 2 * N * d) + (fused_fmas + N * d - channels)


def recorded_traffic(workload_key: str, kernel: str):
    """HBM bytes per launch (fetched + written) recorded from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    runs of this command (see profiles/); None if no record matches the workload and kernel."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        with open(path) as fh:
            for line in fh:
                parts = line.split()
                if len(parts) == 4 and parts[0] == workload_key and parts[1] == kernel:
                    return int(parts[2]) + int(parts[3])
    except OSError:
        pass
    return None


def event_batches(torch, run_batch, calls_per_batch: int, repeats: int):
    """`repeats` batches, each bracketed by one HIP event pair on torch's current stream (the stream the library
    enqueues on); returns the per-call times in ms, one per batch."""
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(repeats)]
    torch.cuda.synchronize()
    for a, b in pairs:
        a.record()
        run_batch()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) / calls_per_batch for a, b in pairs]


def summary(per_call_ms):
    import numpy as np
    v = np.asarray(per_call_ms, dtype=np.float64)
    return {"min": float(v.min()), "median": float(np.median(v)), "max": float(v.max())}


def measure_peaks(torch, dev):
    """Delivered limits of this device from the microbenchmarks of libsig_peaks (best of five timed launches each)."""
    from paper_2001_00706_amd.build import PEAKS_LIB_PATH
    if not os.path.exists(PEAKS_LIB_PATH):
        from paper_2001_00706_amd.build import build_peaks_lib
        build_peaks_lib()
    lib = ctypes.CDLL(PEAKS_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    for name in ("sig_peak_mfma_f32", "sig_peak_mfma_f32_4x4x1", "sig_peak_valu_f32"):
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = [vp, i32, i32, vp]
    lib.sig_peak_hbm_write.restype = i32
    lib.sig_peak_hbm_write.argtypes = [vp, i64, vp]
    lib.sig_peak_hbm_copy.restype = i32
    lib.sig_peak_hbm_copy.argtypes = [vp, vp, i64, vp]
    wgs = 2048
    sink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
    big = torch.empty(1 << 28, dtype=torch.float32, device=dev)            # 1 GiB
    half = big.numel() * 2                                                 # bytes of half the buffer
    hs = torch.cuda.current_stream().cuda_stream

    def best_ms(fn):
        for _ in range(2):
            assert fn() == 0
        return min(event_batches(torch, lambda: fn(), 1, 5))

    t = best_ms(lambda: lib.sig_peak_mfma_f32(sink.data_ptr(), wgs, 2000, hs))
    mfma = wgs * 4 * 2000 * 8 * 4096 / (t * 1e-3) / 1e12
    t = best_ms(lambda: lib.sig_peak_mfma_f32_4x4x1(sink.data_ptr(), wgs, 8000, hs))
    mfma4 = wgs * 4 * 8000 * 8 * 512 / (t * 1e-3) / 1e12
    t = best_ms(lambda: lib.sig_peak_valu_f32(sink.data_ptr(), wgs, 4000, hs))
    valu = wgs * 256 * 4000 * 16 * 2 / (t * 1e-3) / 1e12
    t = best_ms(lambda: lib.sig_peak_hbm_write(big.data_ptr(), big.numel() * 4, hs))
    write = big.numel() * 4 / (t * 1e-3) / 1e9
    t = best_ms(lambda: lib.sig_peak_hbm_write(big.data_ptr(), 128 << 20, hs))     # fits the 256 MB last-level cache
    write_cached = (128 << 20) / (t * 1e-3) / 1e9
    t = best_ms(lambda: lib.sig_peak_hbm_copy(big.data_ptr() + half, big.data_ptr(), half, hs))
    copy = 2 * half / (t * 1e-3) / 1e9
    # adding into LDS: ns per wavefront operation and compute unit, 8 workgroups of 4 wavefronts on each of 256 units
    lib.sig_peak_lds_add.restype = i32
    lib.sig_peak_lds_add.argtypes = [vp, i32, i32, i32, i32, i32, vp]
    lds = {}
    for key, active, stride, atomic in (("lds_atomic_add_64_lanes_ns", 64, 1, 1), ("lds_atomic_add_16_lanes_ns", 16, 1, 1),
                                        ("lds_atomic_add_4_lanes_ns", 4, 1, 1), ("lds_atomic_add_64_lanes_one_address_ns", 64, 0, 1),
                                        ("lds_read_add_write_64_lanes_ns", 64, 1, 0)):
        t = best_ms(lambda: lib.sig_peak_lds_add(sink.data_ptr(), 256 * 8, 4096, active, stride, atomic, hs))
        lds[key] = t * 1e6 / (8 * 4 * 4096)
    del big, sink
    return {"mfma_f32_32x32x2_tflops": mfma, "mfma_f32_4x4x1_tflops": mfma4, "valu_f32_fma_tflops": valu,
            "hbm_write_1GiB_gbs": write, "write_128MiB_last_level_cache_gbs": write_cached, "hbm_copy_512MiB_gbs": copy, **lds}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=2, help="configuration number 1..5 (default: the metric's)")
    ap.add_argument("--variant", choices=["auto", "generic", "mfma", "mfma_shard", "small", "tree", "mfma_stream", "row_stream", "wide", "depth2"], default="auto")
    ap.add_argument("--shape", default=None, metavar="B,L,d,N[,stream]",
                    help="a shape of your own instead of one of the five workloads (same input recipe, seed index 0), "
                         "e.g. 32,128,7,7 for the largest case of the paper's benchmark grid")
    ap.add_argument("--op", choices=["forward", "backward", "combine", "logsignature", "logsignature_backward"], default="forward")
    ap.add_argument("--repeats", type=int, default=50, help="event-bracketed batches per timing (default 50)")
    ap.add_argument("--min-batch-ms", type=float, default=2.0, help="a batch holds enough calls to last this long")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the microbenchmarks of the device limits")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the batches")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 256 MiB device-to-device copies before the timed region, so that "
                         "a rocprofv3 --pmc run of this command sees a copy kernel of known size next to the "
                         "signature kernel (used to scale FETCH_SIZE / WRITE_SIZE into bytes)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 "
              "(paths are independent, so more GPUs would simply split the batch)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2001_00706_amd as sig
    from paper_2001_00706_amd.inputs import workload, workload_paths

    if not os.path.exists(sig.binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    w = workload(args.workload)
    if args.shape:
        from paper_2001_00706_amd.inputs import Workload
        parts = args.shape.split(",")
        B_, L_, d_, N_ = (int(v) for v in parts[:4])
        w = Workload(0, B=B_, L=L_, d=d_, N=N_, stream=len(parts) > 4 and parts[4] == "stream", basepoint=False)
    variant = {"auto": sig.SIG_VARIANT_AUTO, "generic": sig.SIG_VARIANT_GENERIC, "mfma": sig.SIG_VARIANT_MFMA,
               "mfma_shard": sig.SIG_VARIANT_MFMA_SHARD, "small": sig.SIG_VARIANT_SMALL,
               "tree": sig.SIG_VARIANT_TREE, "mfma_stream": sig.SIG_VARIANT_MFMA_STREAM,
               "row_stream": sig.SIG_VARIANT_ROW_STREAM, "wide": sig.SIG_VARIANT_WIDE, "depth2": sig.SIG_VARIANT_DEPTH2}[args.variant]
    x_host = workload_paths(w)
    dev = torch.device("cuda:0")
    x = torch.from_numpy(x_host).to(dev)
    S = sig.sig_signature_channels(w.d, w.N)
    out_shape = (w.B, w.n_inc, S) if w.stream else (w.B, S)
    out = torch.empty(out_shape, dtype=torch.float32, device=dev)
    kernel = sig.sig_variant_name(w.B, w.L, w.d, w.N, w.stream, w.basepoint, sig.SIG_F32, variant)

    def step():
        # the C call on raw device addresses, on torch's current stream
        st = sig.sig_forward_raw(x.data_ptr(), w.B, w.L, w.d, w.N, int(w.stream), int(w.basepoint), sig.SIG_F32,
                                 out.data_ptr(), sig.current_stream_handle(), variant)
        if st != sig.SIG_OK:
            raise sig.SigError(st, sig.sig_status_string(st))

    if args.op == "backward":
        step()
        grad_out = torch.from_numpy(np.random.default_rng(w.seed).standard_normal(out_shape).astype(np.float32)).to(dev)
        grad_path = torch.empty_like(x)
        need = sig.sig_backward_workspace_bytes(w.B, w.L, w.d, w.N, w.stream, w.basepoint)
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
        kernel = "backward"

        def step():  # noqa: F811
            sig.sig_backward(x, out, grad_out, w.N, stream=w.stream, basepoint=w.basepoint, grad_path=grad_path,
                             workspace=workspace)

        # few long paths: the library's hint asks for the walk back to be cut into stretches, as the autograd op does
        stretches = 1 if w.stream else sig.sig_backward_chunks_hint(w.B, w.L, w.d, w.N, w.basepoint)
        if stretches > 1:
            need = sig.sig_backward_chunked_workspace_bytes(w.B, w.L, w.d, w.N, w.basepoint, stretches)
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
            kernel = f"backward_chunked({stretches})"

            def step():  # noqa: F811
                sig.sig_backward_chunked(x, grad_out, w.N, stretches, basepoint=w.basepoint, grad_path=grad_path,
                                         workspace=workspace)
    elif args.op == "logsignature":
        log_full = torch.empty_like(out)
        n_words = sig.sig_logsignature_channels(w.d, w.N)
        log_words = torch.empty(out_shape[:-1] + (n_words,), dtype=torch.float32, device=dev)
        kernel = kernel + "+log+gather"

        def step():  # noqa: F811
            sig.sig_forward(x, w.N, stream=w.stream, basepoint=w.basepoint, out=out, variant=variant)
            sig.sig_log(out, w.d, w.N, out=log_full)
            sig.sig_lyndon_gather(log_full, w.d, w.N, out=log_words)
    elif args.op == "logsignature_backward":
        step()
        n_words = sig.sig_logsignature_channels(w.d, w.N)
        rows = int(np.prod(out_shape[:-1]))
        grad_words = torch.from_numpy(np.random.default_rng(w.seed).standard_normal(out_shape[:-1] + (n_words,))
                                      .astype(np.float32)).to(dev)
        grad_log = torch.empty_like(out)
        grad_sig = torch.empty_like(out)
        grad_path = torch.empty_like(x)
        ws_log = torch.empty(max(sig.sig_log_backward_workspace_bytes(rows, w.d, w.N), 16), dtype=torch.uint8, device=dev)
        ws_sig = torch.empty(max(sig.sig_backward_workspace_bytes(w.B, w.L, w.d, w.N, w.stream, w.basepoint), 16),
                             dtype=torch.uint8, device=dev)
        kernel = "scatter+log_backward+backward"

        def step():  # noqa: F811
            sig.sig_lyndon_scatter(grad_words, w.d, w.N, out=grad_log)
            sig.sig_log_backward(out, grad_log, w.d, w.N, out=grad_sig, workspace=ws_log)
            sig.sig_backward(x, out, grad_sig, w.N, stream=w.stream, basepoint=w.basepoint, grad_path=grad_path,
                             workspace=ws_sig)
    elif args.op == "combine":
        step()
        lhs = out.reshape(-1, S)
        rhs = torch.flip(lhs, dims=[0]).contiguous()
        prod = torch.empty_like(lhs)
        kernel = "combine"

        def step():  # noqa: F811
            sig.sig_combine(lhs, rhs, w.d, w.N, out=prod)

    measured_peaks = None
    if not args.no_peaks:
        measured_peaks = measure_peaks(torch, dev)

    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)   # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # whole-job timing: exactly K steps between two device synchronisations
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # kernel time: event-bracketed batches of back-to-back calls
    calls = max(1, int(math.ceil(args.min_batch_ms / max(ms_per_step, 1e-4))))
    direct = summary(event_batches(torch, lambda: [step() for _ in range(calls)], calls, args.repeats))
    timings = {"calls_per_batch": calls, "batches": args.repeats, "direct_ms_per_call": direct}
    kern_ms, kern_how = direct["median"], "direct"
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                                    # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(calls):
                step()
        for _ in range(3):
            graph.replay()
        replay = summary(event_batches(torch, graph.replay, calls, args.repeats))
        timings["graph_replay_ms_per_call"] = replay
        if replay["median"] < kern_ms:
            kern_ms, kern_how = replay["median"], "graph_replay"
        del graph

    M = sig.sig_fused_fmas(w.d, w.N)
    flops = w.B * w.n_inc * flops_per_increment(w.d, w.N, M)
    bytes_io = 4 * (w.B * w.L * w.d + int(np.prod(out_shape)))
    units, metric = w.B, "signatures/sec (paths/s)"
    if args.op == "backward":
        flops = w.B * w.n_inc * backward_flops_per_increment(w.d, w.N, M, S)
        if w.N == 2 and not w.stream:
            # closed form, no recurrences: a point's gradient is its row of [points x d] [d x d] with G_2 - G_2^T
            flops = 2 * w.B * w.n_inc * w.d * w.d
        bytes_io = 4 * (2 * w.B * w.L * w.d + 2 * int(np.prod(out_shape)))
        metric = "signature gradients/sec (paths/s)"
    elif args.op == "logsignature":
        rows = int(np.prod(out_shape[:-1]))
        # the logarithm by Horner's rule: pass m forms levels 1..N-m+1, a level-k word costs k-1 multiply-adds
        flops += 2 * rows * sum((k - 1) * w.d ** k for m in range(1, w.N + 1) for k in range(2, w.N - m + 2))
        bytes_io = 4 * (w.B * w.L * w.d + rows * n_words)
        metric = "logsignatures/sec (paths/s)"
    elif args.op == "logsignature_backward":
        # signature gradient, the R_m of Horner's rule again, and two multiply-adds per scalar of every matrix M_l
        flops = w.B * w.n_inc * backward_flops_per_increment(w.d, w.N, M, S)
        flops += 2 * rows * sum((k - 1) * w.d ** k for m in range(2, w.N + 1) for k in range(2, w.N - m + 2))
        flops += 2 * rows * sum(2 * (k - 1) * w.d ** k for m in range(1, w.N) for k in range(2, w.N - m + 2))
        bytes_io = 4 * (2 * w.B * w.L * w.d + int(np.prod(out_shape)) + rows * n_words)
        metric = "logsignature gradients/sec (paths/s)"
    elif args.op == "combine":
        units = int(lhs.shape[0])
        flops = 2 * units * sum((k - 1) * w.d ** k for k in range(2, w.N + 1))
        bytes_io = 4 * 3 * units * S
        metric = "group products/sec"
    # the roof that lies lower for this call: moving its algorithmic bytes at the HBM peak against doing its algorithmic
    # flops at the fp32 peak (final-mode scans and gradients of few channels at low depth move more than they compute)
    memory_bound = args.op in ("forward", "backward") and bytes_io / (PEAK_HBM_GBS * 1e9) > flops / (PEAK_FP32_TFLOPS * 1e12)
    if (w.stream and args.op == "forward") or args.op == "combine" or memory_bound:
        roofline = {"bound": "hbm", "achieved": bytes_io / (kern_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s"}
        if measured_peaks:
            # an output that fits the 256 MB last-level cache is priced against what that cache absorbs
            write_key = "write_128MiB_last_level_cache_gbs" if bytes_io <= 256 * 1000 * 1000 else "hbm_write_1GiB_gbs"
            roofline["peak_measured"] = measured_peaks["hbm_copy_512MiB_gbs" if args.op == "combine" else write_key]
            roofline["peak_measured_is"] = "hbm_copy_512MiB_gbs" if args.op == "combine" else write_key
    else:
        bound = "mfma" if kernel.startswith("mfma") else "alu"
        roofline = {"bound": bound, "achieved": flops / (kern_ms * 1e-3) / 1e12, "peak": PEAK_FP32_TFLOPS,
                    "unit": "TFLOP/s"}
        if measured_peaks:
            roofline["peak_measured"] = (max(measured_peaks["mfma_f32_32x32x2_tflops"],
                                             measured_peaks["mfma_f32_4x4x1_tflops"]) if bound == "mfma"
                                         else measured_peaks["valu_f32_fma_tflops"])
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    if "peak_measured" in roofline:
        roofline["frac_of_measured_peak"] = roofline["achieved"] / roofline["peak_measured"]
    roofline["traffic"] = recorded_traffic(f"cfg{w.index}", kernel)
    roofline["traffic_source"] = ("recorded: profiles/hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, of "
                                  "this command)" if roofline["traffic"] is not None else None)
    roofline["kernel"] = kernel
    roofline["kernel_ms"] = kern_ms
    roofline["kernel_ms_from"] = f"median per call over {args.repeats} event-bracketed batches of {calls} calls ({kern_how})"
    roofline["kernel_ms_min"] = min(direct["min"], timings.get("graph_replay_ms_per_call", direct)["min"])
    roofline["algorithmic_flops_per_launch"] = flops
    roofline["algorithmic_bytes_per_launch"] = bytes_io

    result = {
        "metric": metric,
        "value": units / (ms_per_step * 1e-3),
        "unit": "products/s" if args.op == "combine" else "paths/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "L": w.L, "d": w.d, "N": w.N,
                   "mode": "stream" if w.stream else "final", "op": args.op, "kernel": kernel,
                   "device": torch.cuda.get_device_name(0)},
        "roofline": roofline,
        "timings": timings,
        # the rate the device sustains when nothing on the host sits between the kernels
        "gpu_side_value": units / (kern_ms * 1e-3),
    }
    if measured_peaks:
        result["measured_peaks"] = measured_peaks

    if not args.no_cpu_baseline:
        from oracle import sig_oracle
        # bounded sample: whole paths of the same workload, sized for roughly 1-3 s per pass
        per_path_cost = w.n_inc * (w.N - 1) * w.d ** w.N
        n_sample = int(max(1, min(w.B, 4e9 // max(per_path_cost, 1))))
        xs = x_host[:n_sample]
        # repeat whole passes until about 1.5 s of wall time (some 10-30 core-seconds) is spent
        if args.op == "backward":
            n_sample = max(1, n_sample // 4)
            xs = x_host[:n_sample]
            gs = grad_out[:n_sample].cpu().numpy()
        elif args.op == "logsignature_backward":
            n_sample = max(1, n_sample // 8)
            xs = x_host[:n_sample]
            gs = grad_words[:n_sample].cpu().numpy()
        elif args.op == "combine":
            n_sample = int(max(1, min(units, 4e9 // max((w.N - 1) * w.d ** w.N, 1))))
            la, lb = lhs[:n_sample].cpu().numpy().astype(np.float64), rhs[:n_sample].cpu().numpy().astype(np.float64)
        last = {}

        def oracle_pass(paths=None, threads=0):
            p = xs if paths is None else paths
            if args.op == "backward":
                sig_oracle.signature_backward(p, gs[:len(p)], w.N, stream=w.stream, basepoint=w.basepoint, num_threads=threads)
            elif args.op == "combine":
                for i in range(n_sample):   # the oracle's product is one pair at a time, single-threaded
                    sig_oracle.group_mul(la[i], lb[i], w.d, w.N)
            elif args.op == "logsignature":
                sig_oracle.logsignature(p, w.N, stream=w.stream, basepoint=w.basepoint)
            elif args.op == "logsignature_backward":
                sig_oracle.logsignature_backward(p, gs[:len(p)], w.N, stream=w.stream, basepoint=w.basepoint)
            else:
                last["sig"] = sig_oracle.signature(p, w.N, stream=w.stream, basepoint=w.basepoint, num_threads=threads)

        best, spent, passes = float("inf"), 0.0, 0
        while passes < 3 or (spent < 1.5 and passes < 50):
            t = time.perf_counter()
            oracle_pass()
            dt = time.perf_counter() - t
            best, spent, passes = min(best, dt), spent + dt, passes + 1
        cores = 1 if args.op == "combine" else sig_oracle.max_threads()
        result["cpu_baseline"] = {
            "value": n_sample / best,
            "unit": "products/s" if args.op == "combine" else "paths/s",
            "cores": cores,
            "kind": "oracle",
            "sample": f"first {n_sample} of {units} {'pairs' if args.op == 'combine' else 'paths'} of {w.name}, op {args.op}: " + {
                "forward": "fp64 exp + group product per increment, OpenMP over paths",
                "backward": "fp64 exp + group product per increment and their adjoints over the stored forward, OpenMP over paths",
                "combine": "fp64 group product, one pair at a time on one core",
                "logsignature": "fp64 signature (OpenMP over paths), then the power series of log one row at a time on one core",
                "logsignature_backward": "fp64 signature and its stored-forward gradient (OpenMP over paths), the power series of log and its adjoint one row at a time on one core",
            }[args.op] + f", best of {passes} passes ({best:.3f} s each, {spent:.1f} s in all)",
        }
        if args.op in ("forward", "backward") and cores > 1:
            # the like-for-like figure the paper stresses: the same oracle on one thread, on a proportionally smaller sample
            n_one = max(1, n_sample // cores)
            one = float("inf")
            for _ in range(3):
                t = time.perf_counter()
                oracle_pass(xs[:n_one], threads=1)
                one = min(one, time.perf_counter() - t)
            result["cpu_baseline"]["value_1_thread"] = n_one / one
            result["cpu_baseline"]["sample_1_thread"] = f"first {n_one} paths, best of 3 passes ({one:.3f} s each)"
        if args.op == "forward":
            # the timed output itself against the oracle, on the sample the oracle just computed
            oracle_pass()
            step()
            torch.cuda.synchronize()
            got = out[:n_sample].cpu().numpy().astype(np.float64)
            errs = []
            for sl in sig_oracle.level_slices(w.d, w.N):
                den = np.linalg.norm(last["sig"][..., sl])
                errs.append(float(np.linalg.norm(got[..., sl] - last["sig"][..., sl]) / (den if den > 0 else 1.0)))
            result["rel_l2_per_level"] = errs
            result["rel_l2_max"] = max(errs)
            result["rel_l2_paths"] = n_sample

    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
