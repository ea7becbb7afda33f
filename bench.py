#!/usr/bin/env python3
"""Benchmark of the activation-compression hot path on one MI355X.

One *step* is one pass of the whole path over one batch that is already resident in HBM:
  group_stats -> allocate_bits (greedy) -> quantize_pack -> unpack_dequantize.
By default the allocator runs on the device (actq_allocate_bits_device) and the step never
touches the host; --allocator host runs the host greedy between the kernels instead (widths
and offsets then travel host-to-device in every step).
The default workload is the full ResNet-50 activation sweep at batch 256: the 53 conv-input
tensors (fp32, 10.9 GB), G = 256, one greedy allocation over all 53 x 256 (layer, sample) items
to a 2.0-bit average over widths {1,2,4,8}, multi-tensor launches (one per size class and
kernel).  `value` is input-activation bytes per second through the whole step; the per-kernel
and per-size-class figures and the HBM roofline of the slowest kernel are reported beside it,
the CPU oracle is timed as a baseline, and the single ResNet-50 stage-1 tensor
(--workload r50_stage1) is appended under `r50_stage1`.

Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=40)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--workload", default="r50_sweep", choices=["r50_stage1", "tiny", "r50_stem_f16", "fpn", "r50_sweep", "contexts", "block"])
    p.add_argument("--noise-bits", type=int, default=16, choices=[24, 16])
    p.add_argument("--header", default="f32", choices=["f32", "bf16"],
                   help="group header format: (Z, R/B) binary32, 8 B/group, or (Z, R) bfloat16, 4 B/group")
    p.add_argument("--allocator", default="device", choices=["device", "host"],
                   help="where the greedy bit allocation of each step runs")
    p.add_argument("--launches", default="multi", choices=["multi", "single"],
                   help="r50_sweep: all tensors in a few multi-tensor launches, or one launch per tensor and kernel")
    p.add_argument("--uniform-bits", type=int, default=0, choices=range(0, 9), metavar="B",
                   help="give every sample the width B (1..8) instead of the workload's mixed widths")
    p.add_argument("--event-every", type=int, default=4,
                   help="single-tensor workloads: record the per-kernel HIP events in every n-th timed step")
    p.add_argument("--contexts-dtype", default="f32", choices=["f32", "f16"],
                   help="element type of the `contexts` workload")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--cpu-seconds", type=float, default=12.0,
                   help="r50_sweep: oracle time after which the CPU baseline stops taking further layers")
    p.add_argument("--sweep-batch", type=int, default=256, help="r50_sweep: samples per tensor")
    p.add_argument("--no-secondary", action="store_true",
                   help="r50_sweep: do not append the ResNet-50 stage-1 tensor's figures under `r50_stage1`")
    p.add_argument("--profile-pass", action="store_true",
                   help="for rocprofv3 counter runs: a few launches of each kernel plus a plain device copy "
                        "of the input tensor (known size, calibrates FETCH_SIZE / WRITE_SIZE), then exit")
    return p.parse_args()


def algorithmic_bytes(N, D, ng, elem_bytes, code_bytes, header_group_bytes=8):
    """Bytes each kernel must move per launch: input or output tensor, bit stream, group headers
    (group_stats always writes 4 + 4 bytes per group)."""
    tensor = N * D * elem_bytes
    hdr = N * ng * header_group_bytes
    return {
        "group_stats": tensor + N * ng * 8,
        "quantize_pack": tensor + code_bytes + hdr,
        "unpack_dequantize": code_bytes + hdr + tensor,
    }


def measured_traffic(workload: str, noise_bits: int, kernel: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE,
    each scaled by what the same counter reads for a plain copy of known size), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            table = json.load(f)
        return table[workload][f"noise{noise_bits}"][kernel]["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


SWEEP_NAME = "r50_sweep_f32_53x[256,C,H,W]"


def sweep_traffic(noise_bits: int):
    """HBM bytes per step of every sweep kernel from the committed rocprofv3 counter summary
    (profiles/hbm_traffic.json; a property of that profiling run, not of this one), or None."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            return json.load(f)[SWEEP_NAME][f"noise{noise_bits}"]
    except (OSError, KeyError, ValueError):
        return None


_SWEEP_SINGLE_THREAD_LEG = r'''
import json, sys, time
import numpy as np
sys.path.insert(0, sys.argv[1])
import oracle
from paper_2104_14129_amd import synth
rows, noise_bits = int(sys.argv[2]), int(sys.argv[3])
Dl = [c * h * w for c, h, w in synth.resnet50_conv_input_shapes()]
rng = np.random.default_rng(1)
spent, nbytes = 0.0, 0
for l, D in enumerate(Dl):
    x = np.maximum(rng.standard_normal((rows, D), dtype=np.float32), 0.0)
    bits = np.full(rows, 2, dtype=np.uint8)
    t = time.perf_counter()
    oracle.group_stats(x, 256)
    pk, hd, off = oracle.quantize_pack(x, bits, 15, l, 256, noise_bits)
    oracle.unpack_dequantize(pk, hd, bits, off, rows, D, 256, out_dtype=x.dtype)
    spent += time.perf_counter() - t
    nbytes += x.nbytes
print(json.dumps({"value": nbytes / spent / 1e9, "unit": "GB/s", "cores": oracle.threads(),
                  "sample": f"{rows} samples of each of the 53 layers at 2 bits, {nbytes} input bytes, {spent:.2f} s"}))
'''


def sweep_single_thread(rows, noise_bits):
    """One OpenMP thread of the oracle on a few samples of every layer, in a child process that is
    started before this process touches the GPU (the thread count is fixed when the library loads)."""
    import subprocess
    try:
        out = subprocess.run([sys.executable, "-c", _SWEEP_SINGLE_THREAD_LEG, ROOT, str(rows), str(noise_bits)],
                             env=dict(os.environ, OMP_NUM_THREADS="1"), capture_output=True, text=True,
                             timeout=300, check=True).stdout
        return json.loads(out.strip().splitlines()[-1])
    except Exception as exc:  # the baseline is a report, never a reason for the bench to fail
        return {"error": f"{type(exc).__name__}: {exc}"}


def sweep(args, torch, B, synth, dev, single_thread=None):
    """The 53 conv-input tensors of ResNet-50 at batch 256 (fp32, 10.9 GB).  One step: group_stats on
    every layer, one greedy allocation over all 53 x 256 (layer, sample) items under a 2.0-bit
    average budget, quantize_pack and unpack_dequantize on every layer -- by default as multi-tensor
    launches (one call per size class and kernel), with --launches single as one launch per layer
    and kernel."""
    from paper_2104_14129_amd.plan import TensorSetPlan
    N, G = args.sweep_batch, 256
    shapes = synth.resnet50_conv_input_shapes()
    Dl = [c * h * w for c, h, w in shapes]
    L = len(Dl)
    multi = args.launches == "multi"
    device_alloc = args.allocator == "device"
    gen = torch.Generator(device=dev)
    xs = []
    for l, D in enumerate(Dl):
        gen.manual_seed(1000 + l)
        xs.append(torch.randn((N, D), generator=gen, device=dev, dtype=torch.float32).clamp_min_(0))
    w_host = synth.lognormal_sensitivities(N * L, seed=5)
    D_host = np.repeat(np.array(Dl, dtype=np.int64), N)
    budget = 2 * int(D_host.sum())
    Dmax = max(Dl)
    stream = torch.cuda.current_stream()
    w_dev = torch.from_numpy(w_host).to(dev)
    D_dev = torch.from_numpy(D_host).to(dev)
    bits_pin = torch.empty(N * L, dtype=torch.uint8, pin_memory=True)
    offs_pin = torch.empty(N * L, dtype=torch.int64, pin_memory=True)
    state = {}
    names = ("group_stats", "quantize_pack", "unpack_dequantize")
    lib = B.lib()
    sp = stream.cuda_stream
    every = max(1, args.event_every)

    if multi:
        # one shared bit stream of budget / 8 bytes; every layer keeps its own statistics, header and
        # output arrays, as a training step would
        plan = TensorSetPlan(xs, N, budget // 8 + 4096, noise_bits=args.noise_bits, seed=15, G=G)
        bits_dev, offs_dev, result_dev = plan.bits, plan.offsets, plan.result
        classes = plan.classes
        launches_per_step = 3 * len(classes) + 1
        # boundary events: the end of one launch is the start of the next
        n_ev = 3 * (len(classes) + 1)
    else:
        shared_stream = device_alloc
        packed_buf = torch.empty(budget // 8 + 4096 if shared_stream else N * Dmax, dtype=torch.uint8, device=dev)
        packed_capacity = packed_buf.numel()
        bits_dev = torch.empty(N * L, dtype=torch.uint8, device=dev)
        offs_dev = torch.empty(N * L, dtype=torch.int64, device=dev)
        result_dev = torch.zeros(2, dtype=torch.int64, device=dev)
        classes = [[l] for l in range(L)]
        launches_per_step = 3 * L + 1
        n_ev = 6 * L
    steps_with_events = [i for i in range(args.steps) if i % every == 0]
    pool = {i: [torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for i in steps_with_events}

    def allocate():
        if device_alloc:
            B.allocate_bits_device(w_dev, D_dev, budget, B.ACTQ_WIDTHS_POW2, bits_dev, offs_dev, result_dev, G, stream=stream)
            return
        bits = B.allocate_bits(w_host, D_host, budget)
        totals, base = [], 0
        for l, D in enumerate(Dl):
            offsets, total = B.packed_bytes(N, D, bits[l * N:(l + 1) * N], G)
            offs_pin.numpy()[l * N:(l + 1) * N] = offsets.view(np.int64) + (base if (multi or device_alloc) else 0)
            base += total
            totals.append(total)
        bits_pin.numpy()[:] = bits
        bits_dev.copy_(bits_pin, non_blocking=True)
        offs_dev.copy_(offs_pin, non_blocking=True)
        state["bits"], state["totals"] = bits, totals

    if multi:
        nc = len(classes)

        def step(ev=None):
            # the statistics come first: in training the sensitivities are computed from them (Eq. (8))
            if ev is None:
                plan.group_stats(stream)
                allocate()
                plan.quantize_pack(stream)
                plan.unpack_dequantize(stream)
                return
            ev[0].record(stream)
            plan.group_stats(stream, lambda k: ev[1 + k].record(stream))
            allocate()
            ev[nc + 1].record(stream)
            plan.quantize_pack(stream, lambda k: ev[nc + 2 + k].record(stream))
            ev[2 * nc + 2].record(stream)
            plan.unpack_dequantize(stream, lambda k: ev[2 * nc + 3 + k].record(stream))

        def durations(ev):
            """ms of (kernel j, class k) from the boundary events of one step."""
            starts = (0, nc + 1, 2 * nc + 2)
            return [[ev[starts[j] + k].elapsed_time(ev[starts[j] + k + 1]) for k in range(nc)] for j in range(3)]
    else:
        ngmax = Dmax // G
        gmin = torch.empty(N * ngmax, dtype=torch.float32, device=dev)
        grange = torch.empty(N * ngmax, dtype=torch.float32, device=dev)
        header = torch.empty(N * ngmax * 2, dtype=torch.float32, device=dev)
        out = torch.empty(N * Dmax, dtype=torch.float32, device=dev)
        layer_args = [(xs[l].data_ptr(), D, bits_dev.data_ptr() + l * N, offs_dev.data_ptr() + 8 * l * N)
                      for l, D in enumerate(Dl)]

        def step(ev=None):
            allocate()
            gm, gr, hd, pk, o = gmin.data_ptr(), grange.data_ptr(), header.data_ptr(), packed_buf.data_ptr(), out.data_ptr()
            for l, (xp, D, bp, op) in enumerate(layer_args):
                if ev is not None:
                    ev[6 * l].record(stream)
                rc = lib.actq_group_stats(xp, B.ACTQ_F32, N, D, G, gm, gr, sp)
                if ev is not None:
                    ev[6 * l + 1].record(stream)
                    ev[6 * l + 2].record(stream)
                rc |= lib.actq_quantize_pack(xp, B.ACTQ_F32, N, D, G, bp, op, 15, l, args.noise_bits, pk, packed_capacity, hd, B.ACTQ_HDR_F32, sp)
                if ev is not None:
                    ev[6 * l + 3].record(stream)
                    ev[6 * l + 4].record(stream)
                rc |= lib.actq_unpack_dequantize(pk, packed_capacity, hd, B.ACTQ_HDR_F32, bp, op, N, D, G, o, B.ACTQ_F32, sp)
                if ev is not None:
                    ev[6 * l + 5].record(stream)
                if rc:
                    raise RuntimeError(B.last_error())

        def durations(ev):
            return [[ev[6 * l + 2 * j].elapsed_time(ev[6 * l + 2 * j + 1]) for l in range(L)] for j in range(3)]

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.profile_pass:
        # for rocprofv3 counter runs: two steps and, beside them, plain device copies of the largest
        # tensor (known size: calibrates FETCH_SIZE / WRITE_SIZE)
        big = max(range(L), key=lambda l: Dl[l])
        copy_dst = torch.empty_like(xs[big])
        for _ in range(2):
            copy_dst.copy_(xs[big])
            step()
        torch.cuda.synchronize()
        total, status = (int(v) for v in result_dev.cpu()) if device_alloc else (sum(state["totals"]), 0)
        print(json.dumps({"profile_pass": True, "workload": SWEEP_NAME, "copy_bytes_each_way": 4 * N * Dl[big],
                          "input_bytes": 4 * N * sum(Dl), "packed_bytes": total,
                          "header_bytes": sum(N * (D // G) * 8 for D in Dl), "allocator_status": status}))
        return None
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(pool.get(i))
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    if device_alloc:
        total, status = (int(v) for v in result_dev.cpu())
        if status != 0:
            raise RuntimeError(f"device allocator reported status {status}")
        state["bits"] = bits_dev.cpu().numpy()
    bits_all = state["bits"]
    if N * L <= 20000:
        assert np.array_equal(bits_all, B.allocate_bits(w_host, D_host, budget)), "device and host allocators disagree"

    # per (kernel, class): mean over the instrumented steps
    per = np.mean([durations(pool[i]) for i in steps_with_events], axis=0)        # [3][classes] ms
    in_bytes = 4 * N * sum(Dl)

    def class_bytes(members, j):
        tensor = sum(4 * N * Dl[l] for l in members)
        hdr = sum(N * (Dl[l] // G) * 8 for l in members)
        code = sum(int((bits_all[l * N:(l + 1) * N].astype(np.int64) * (Dl[l] // 8)).sum()) for l in members)
        return tensor + hdr + (0 if j == 0 else code)

    alg = {names[j]: sum(class_bytes(m, j) for m in classes) for j in range(3)}
    kernel_ms = {names[j]: float(per[j].sum()) for j in range(3)}
    per_kernel = {k: {"ms_per_step_all_layers": kernel_ms[k], "input_GBps": in_bytes / kernel_ms[k] / 1e6,
                      "algorithmic_GBps": alg[k] / kernel_ms[k] / 1e6,
                      "frac_of_hbm_peak": alg[k] / kernel_ms[k] / 1e6 / HBM_PEAK_GBS} for k in names}
    class_table = None
    if multi:
        class_table = [{"largest_D": Dl[m[0]], "tensors": len(m), "input_MB": sum(4 * N * Dl[l] for l in m) / 1e6,
                        **{names[j]: {"us": float(per[j][k]) * 1e3,
                                      "frac_of_hbm_peak": class_bytes(m, j) / float(per[j][k]) / 1e6 / HBM_PEAK_GBS}
                           for j in range(3)}} for k, m in enumerate(classes)]
    dominant = max(kernel_ms, key=kernel_ms.get)
    achieved = alg[dominant] / kernel_ms[dominant] / 1e6
    mean_bits = float((bits_all.astype(np.float64) * D_host).sum() / D_host.sum())
    traffic_table = sweep_traffic(args.noise_bits) if (multi and N == 256) else None
    traffic = traffic_table[dominant]["hbm_bytes_per_step"] if traffic_table and dominant in traffic_table else None

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        # The oracle (all OpenMP threads) on whole layers of the same inputs and widths, layer by layer so
        # that host memory stays bounded, until about `--cpu-seconds` of oracle time are spent.
        spent, done_bytes, done_layers = 0.0, 0, 0
        order = sorted(range(L), key=lambda l: Dl[l])          # small layers first: the sample spans every size
        for l in order:
            if spent > args.cpu_seconds:
                break
            x_np = xs[l].cpu().numpy()
            b_np = np.ascontiguousarray(bits_all[l * N:(l + 1) * N])
            t = time.perf_counter()
            oracle.group_stats(x_np, G)
            opk, ohd, ooff = oracle.quantize_pack(x_np, b_np, 15, l, G, args.noise_bits)
            oracle.unpack_dequantize(opk, ohd, b_np, ooff, N, Dl[l], G, out_dtype=x_np.dtype)
            spent += time.perf_counter() - t
            done_bytes += x_np.nbytes
            done_layers += 1
            del x_np, opk, ohd
        cpu_baseline = {"value": done_bytes / spent / 1e9, "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
                        "sample": f"group_stats + quantize_pack + unpack_dequantize on {done_layers} of the {L} layers "
                                  f"(whole layers, smallest first, the step's own inputs and widths), "
                                  f"{done_bytes} input bytes, {spent:.2f} s",
                        "single_thread": single_thread}

    result = {
        "metric": "quantize+pack and unpack+dequant GB/s (fp32 input); % of HBM peak",
        "value": in_bytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": SWEEP_NAME.replace("256", str(N)) if N != 256 else SWEEP_NAME, "G": G, "mean_bits": mean_bits,
                   "noise_bits": args.noise_bits, "launches": args.launches, "launches_per_step": launches_per_step,
                   "allocator": args.allocator, "steps_with_events": len(steps_with_events),
                   "step": f"group_stats + allocate_bits({args.allocator}, M={N * L}) + quantize_pack + unpack_dequantize on every layer"},
        "kernels": per_kernel,
        "size_classes": class_table,
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": "profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE of a separate run of this workload)" if traffic else None,
                     "algorithmic_bytes_per_step": alg[dominant], "sum_launch_ms_per_step": kernel_ms[dominant],
                     "launches_per_step": len(classes)},
        "cpu_baseline": cpu_baseline,
    }
    return result


def contexts(args, torch, B, dev):
    """Exact layer contexts on the ResNet-50 stem at batch 256, fp32 [256,64,112,112]: ReLU forward
    and backward (1-bit mask), then the 3x3 / stride 2 / padding 1 max pooling forward and backward
    (8-bit window positions).  One step is the four launches."""
    N, C, H, W = 256, 64, 112, 112
    k, s_, p = (3, 3), (2, 2), (1, 1)
    tdt = torch.float16 if args.contexts_dtype == "f16" else torch.float32
    eb = 2 if args.contexts_dtype == "f16" else 4
    gen = torch.Generator(device=dev)
    gen.manual_seed(77)
    x = torch.randn((N, C, H, W), generator=gen, device=dev, dtype=torch.float32).to(tdt)
    OH, OW = B.pool2d_output_size(H, W, k, s_, p)
    gy_pool = torch.randn((N, C, OH, OW), generator=gen, device=dev, dtype=torch.float32).to(tdt)
    y = torch.empty_like(x)
    mask = torch.empty(B.relu_mask_bytes(x.numel()), dtype=torch.uint8, device=dev)
    pooled = torch.empty((N, C, OH, OW), dtype=tdt, device=dev)
    arg = torch.empty((N, C, OH, OW), dtype=torch.uint8, device=dev)
    g_act = torch.empty_like(x)
    g_in = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    n_in, n_out = x.numel(), pooled.numel()
    alg = {"relu_forward": n_in * 2 * eb + mask.numel(), "maxpool2d_forward": n_in * eb + n_out * (eb + 1),
           "maxpool2d_backward": n_out * (eb + 1) + n_in * eb, "relu_backward": n_in * 2 * eb + mask.numel()}

    def step(events=None):
        def timed(name, fn):
            if events is None:
                return fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            fn()
            b.record(stream)
            events.setdefault(name, []).append((a, b))
        timed("relu_forward", lambda: B.relu_forward(x, y, mask, stream=stream))
        timed("maxpool2d_forward", lambda: B.maxpool2d_forward(y, k, s_, p, y=pooled, argmax=arg, stream=stream))
        timed("maxpool2d_backward", lambda: B.maxpool2d_backward(arg, gy_pool, H, W, k, s_, p, grad_x=g_act, stream=stream))
        timed("relu_backward", lambda: B.relu_backward(mask, g_act, g_in, stream=stream))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.profile_pass:
        # for rocprofv3 counter runs: three steps and, beside them, plain device copies of the input
        # (known size: calibrates FETCH_SIZE / WRITE_SIZE)
        for _ in range(3):
            g_in.copy_(x)
            step()
        torch.cuda.synchronize()
        print(json.dumps({"profile_pass": True, "workload": f"contexts_r50_stem_{args.contexts_dtype}",
                          "copy_bytes_each_way": n_in * eb, "algorithmic_bytes": alg}))
        return
    events = {}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kernel_ms = {k_: float(np.mean([a.elapsed_time(b) for a, b in v])) for k_, v in events.items()}
    per_kernel = {k_: {"ms": kernel_ms[k_], "algorithmic_GBps": alg[k_] / kernel_ms[k_] / 1e6,
                       "frac_of_hbm_peak": alg[k_] / kernel_ms[k_] / 1e6 / HBM_PEAK_GBS} for k_ in kernel_ms}
    dominant = max(kernel_ms, key=kernel_ms.get)
    achieved = alg[dominant] / kernel_ms[dominant] / 1e6
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        sample = x.cpu().numpy()
        t = time.perf_counter()
        oy, om = oracle.relu_forward(sample.reshape(-1))
        py, pa = oracle.maxpool2d_forward(oy.reshape(sample.shape), k, s_, p)
        gx = oracle.maxpool2d_backward(pa, gy_pool.cpu().numpy(), H, W, k, s_, p)
        oracle.relu_backward(om, gx.reshape(-1))
        cpu_s = time.perf_counter() - t
        cpu_baseline = {"value": sample.nbytes / cpu_s / 1e9, "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
                        "sample": f"the same four calls on the whole workload, {cpu_s:.2f} s "
                                  "(the ReLU loops of the oracle are single-threaded)"}
    print(json.dumps({
        "metric": "exact layer contexts (ReLU mask, max-pool positions): GB/s of input per step; % of HBM peak",
        "value": n_in * eb / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.contexts_dtype, "data": "synthetic",
        "config": {"workload": f"contexts_r50_stem_{args.contexts_dtype}_256x64x112x112", "pool": "3x3 stride 2 padding 1",
                   "step": "relu_forward + maxpool2d_forward + maxpool2d_backward + relu_backward"},
        "kernels": per_kernel,
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": alg[dominant], "avg_launch_ms": kernel_ms[dominant]},
        "cpu_baseline": cpu_baseline}))


def block(args, torch, dev):
    """Layer integration: one ResNet-50 stage-1 bottleneck (1x1-3x3-1x1 convolutions with batch
    norm, ReLU and the residual) at batch 64, fp32, forward + backward, stock layers against their
    activation-compressed versions at a 2.0-bit average: time per iteration and the memory held for
    the backward pass (allocated after the forward pass, minus what was allocated before it and the output).  The convolutions and batch norms themselves are torch's in both runs."""
    import torch.nn as nn
    from paper_2104_14129_amd import layers as L

    class Bottleneck(nn.Module):
        def __init__(self):
            super().__init__()
            self.a = nn.Sequential(nn.Conv2d(256, 64, 1, bias=False), nn.BatchNorm2d(64), nn.ReLU(),
                                   nn.Conv2d(64, 64, 3, padding=1, bias=False), nn.BatchNorm2d(64), nn.ReLU(),
                                   nn.Conv2d(64, 256, 1, bias=False), nn.BatchNorm2d(256))
            self.out = nn.ReLU()

        def forward(self, x):
            return self.out(self.a(x) + x)

    torch.manual_seed(0)
    x = torch.randn(64, 256, 56, 56, device=dev).clamp_min_(0)
    gy = torch.randn(64, 256, 56, 56, device=dev)

    def run(model):
        xin = x.clone().requires_grad_(True)

        def it():
            y = model(xin)
            held = torch.cuda.memory_allocated() - y.numel() * y.element_size()   # contexts only, not the output
            y.backward(gy)
            return held
        for _ in range(args.warmup):
            it()
        torch.cuda.synchronize()
        base = torch.cuda.memory_allocated()
        t0 = time.perf_counter()
        held = 0
        for _ in range(args.steps):
            held = it()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps, held - base

    stock_ms, stock_held = run(Bottleneck().to(dev))
    L.set_optimization_level("L3", bits=2.0)
    q_ms, q_held = run(L.convert(Bottleneck().to(dev)))
    in_bytes = x.numel() * 4
    print(json.dumps({
        "metric": "activation-compressed ResNet-50 bottleneck, forward + backward: GB/s of block input; memory held for backward",
        "value": in_bytes / (q_ms * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": q_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "block_r50_bottleneck_f32_64x256x56x56", "level": "L3", "mean_bits": 2.0},
        "stock": {"ms_per_step": stock_ms, "context_bytes": stock_held},
        "compressed": {"ms_per_step": q_ms, "context_bytes": q_held},
        "memory_ratio": stock_held / max(q_held, 1), "time_ratio": q_ms / stock_ms,
        "roofline": None, "cpu_baseline": None}))


_SINGLE_THREAD_LEG = r'''
import json, sys, time
import numpy as np
sys.path.insert(0, sys.argv[1])
import oracle
d = np.load(sys.argv[2])
x, bits = d["x"], d["bits"]
seed, tag, noise_bits, bf16 = int(d["seed"]), int(d["tag"]), int(d["noise_bits"]), bool(d["bf16"])
rows, D = x.shape
t = time.perf_counter()
oracle.group_stats(x, 256)
if bf16:
    pk, hd, off = oracle.quantize_pack_bf16(x, bits, seed, tag, 256, noise_bits)
    oracle.unpack_dequantize_bf16(pk, hd, bits, off, rows, D, 256, out_dtype=x.dtype)
else:
    pk, hd, off = oracle.quantize_pack(x, bits, seed, tag, 256, noise_bits)
    oracle.unpack_dequantize(pk, hd, bits, off, rows, D, 256, out_dtype=x.dtype)
s = time.perf_counter() - t
print(json.dumps({"value": x.nbytes / s / 1e9, "unit": "GB/s", "cores": oracle.threads(),
                  "sample": f"the same step on the first {rows} samples, {s:.2f} s"}))
'''


def oracle_single_thread(x_np, bits, seed, tag, noise_bits, bf16, rows=8):
    """The oracle's step on the first few samples in a child process limited to one OpenMP thread
    (the thread count is fixed when the library loads); the child never touches the GPU."""
    import subprocess
    import tempfile
    rows = min(rows, x_np.shape[0])
    root = os.path.dirname(os.path.abspath(__file__))
    try:
        with tempfile.TemporaryDirectory() as tmp:
            path = os.path.join(tmp, "sample.npz")
            np.savez(path, x=x_np[:rows], bits=np.ascontiguousarray(bits[:rows]), seed=seed, tag=tag,
                     noise_bits=noise_bits, bf16=bf16)
            out = subprocess.run([sys.executable, "-c", _SINGLE_THREAD_LEG, root, path],
                                 env=dict(os.environ, OMP_NUM_THREADS="1"), capture_output=True, text=True,
                                 timeout=300, check=True).stdout
        return json.loads(out.strip().splitlines()[-1])
    except Exception as exc:  # the baseline is a report, never a reason for the bench to fail
        return {"error": f"{type(exc).__name__}: {exc}"}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (every sample is independent, so data-parallel "
              "ranks would each quantize their own activations with no exchange); --gpus N with N > 1 "
              "is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2104_14129_amd import binding as B
    from paper_2104_14129_amd import synth

    codec = args.workload in ("r50_stage1", "tiny", "r50_stem_f16", "fpn")
    single_thread = None
    wl = x_np = None
    # the one-thread legs of the CPU baseline are child processes: started here, before this
    # process touches the GPU
    if codec:
        wl = {"r50_stage1": synth.r50_stage1, "tiny": synth.tiny, "r50_stem_f16": synth.r50_stem_f16,
              "fpn": synth.fpn}[args.workload]()
        x_np = synth.make_input(wl).reshape(wl.N, wl.D)
        if args.uniform_bits:
            wl.bits = np.full(wl.N, args.uniform_bits, dtype=np.uint8)
        if not args.no_cpu_baseline and not args.profile_pass:
            single_thread = oracle_single_thread(x_np, wl.bits, wl.philox_seed, wl.tag, args.noise_bits,
                                                 args.header == "bf16")
    elif args.workload == "r50_sweep" and not args.no_cpu_baseline and not args.profile_pass:
        single_thread = sweep_single_thread(4, args.noise_bits)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "r50_sweep":
        result = sweep(args, torch, B, synth, dev, single_thread)
        if result is not None and not args.no_secondary and not args.profile_pass:
            # the single ResNet-50 stage-1 tensor (the second configuration), as a secondary figure
            torch.cuda.empty_cache()
            sub = argparse.Namespace(**vars(args))
            sub.workload, sub.no_cpu_baseline, sub.uniform_bits, sub.header, sub.steps, sub.warmup = "r50_stage1", True, 0, "f32", 40, 5
            wl2 = synth.r50_stage1()
            r2 = codec_run(sub, torch, B, synth, dev, wl2, synth.make_input(wl2).reshape(wl2.N, wl2.D), None)
            result["r50_stage1"] = {k: r2[k] for k in ("value", "unit", "ms_per_step", "config", "kernels", "roofline")}
        if result is not None:
            print(json.dumps(result))
        return
    if args.workload == "contexts":
        return contexts(args, torch, B, dev)
    if args.workload == "block":
        return block(args, torch, dev)
    result = codec_run(args, torch, B, synth, dev, wl, x_np, single_thread)
    if result is not None:
        print(json.dumps(result))


def codec_run(args, torch, B, synth, dev, wl, x_np, single_thread):
    """One tensor: group_stats -> sample_sensitivity -> allocate_bits -> quantize_pack -> unpack_dequantize."""
    N, D, ng, G = wl.N, wl.D, wl.ng, wl.G
    x = torch.from_numpy(x_np).to(dev)

    # sensitivities whose greedy allocation at a 2.0-bit budget is the workload's width multiset
    widths = B.ACTQ_WIDTHS_POW2
    if args.uniform_bits:
        widths = 1 << args.uniform_bits           # the only allowed width
        w_host = np.ones(N, dtype=np.float32)
    else:
        w_host = synth.tiered_sensitivities(wl.bits, seed=7)
    D_host = np.full(N, D, dtype=np.int64)
    budget = int(round(float(wl.bits.astype(np.float64).mean()) * N * D))

    gmin = torch.empty((N, ng), dtype=torch.float32, device=dev)
    grange = torch.empty((N, ng), dtype=torch.float32, device=dev)
    _, worst_total = B.packed_bytes(N, D, np.full(N, 8, dtype=np.uint8), G)
    packed_buf = torch.empty(worst_total, dtype=torch.uint8, device=dev)
    hf = B.ACTQ_HDR_BF16 if args.header == "bf16" else B.ACTQ_HDR_F32
    header = torch.empty((N, ng, 2), dtype=torch.int16 if hf == B.ACTQ_HDR_BF16 else torch.float32, device=dev)
    out = torch.empty((N, D), dtype=x.dtype, device=dev)
    bits_pin = torch.empty(N, dtype=torch.uint8, pin_memory=True)
    offs_pin = torch.empty(N, dtype=torch.int64, pin_memory=True)
    bits_dev = torch.empty(N, dtype=torch.uint8, device=dev)
    offs_dev = torch.empty(N, dtype=torch.int64, device=dev)
    stream = torch.cuda.current_stream()

    # Per-sample squared gradient norms (an input of the method, Sec. 4.2) chosen so that the
    # sensitivities computed on the device, (G/6) * grad2_n * sum_g R_ng^2, land on w_host.
    w_dev = torch.empty(N, dtype=torch.float32, device=dev)
    result_dev = torch.zeros(2, dtype=torch.int64, device=dev)
    B.group_stats(x, gmin, grange, G, stream=stream)
    unit = B.sample_sensitivity(grange, None, G=G, stream=stream).cpu().numpy().astype(np.float64)
    grad2 = torch.from_numpy(np.where(unit > 0, w_host / np.maximum(unit, 1e-300), 0.0).astype(np.float32)).to(dev)

    state = {}

    def step(events=None):
        def mark(name, when):
            if events is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record(stream)
                events.setdefault(name, []).append((when, e))

        mark("group_stats", 0)
        B.group_stats(x, gmin, grange, G, stream=stream)
        mark("group_stats", 1)
        if args.allocator == "device":
            mark("sensitivity+allocate", 0)
            B.sample_sensitivity(grange, grad2, w_dev, G, stream=stream)
            B.allocate_bits_device(w_dev, D, budget, widths, bits_dev, offs_dev, result_dev, G, stream=stream)
            mark("sensitivity+allocate", 1)
            packed = packed_buf          # the total is known only on the device: hand over the whole buffer
        else:
            bits = B.allocate_bits(w_host, D_host, budget, widths)
            offsets, total = B.packed_bytes(N, D, bits, G)
            bits_pin.numpy()[:] = bits
            offs_pin.numpy()[:] = offsets.view(np.int64)
            bits_dev.copy_(bits_pin, non_blocking=True)
            offs_dev.copy_(offs_pin, non_blocking=True)
            packed = packed_buf[:total]
            state["bits"], state["total"] = bits, total
        mark("quantize_pack", 0)
        B.quantize_pack(x, bits_dev, offs_dev, packed, header, wl.philox_seed, wl.tag, args.noise_bits, G, stream=stream, hf=hf)
        mark("quantize_pack", 1)
        mark("unpack_dequantize", 0)
        B.unpack_dequantize(packed, header, bits_dev, offs_dev, out, G, stream=stream, hf=hf)
        mark("unpack_dequantize", 1)

    def read_back():
        if args.allocator == "device":
            torch.cuda.synchronize()
            total, status = (int(v) for v in result_dev.cpu())
            if status != 0:
                raise RuntimeError(f"device allocator reported status {status}")
            state["bits"], state["total"] = bits_dev.cpu().numpy(), total

    # The timed steps of the device-allocator path call the C ABI with pointers and sizes worked out
    # once and with events created beforehand, so that the host stays ahead of the GPU (five launches
    # of 5-70 us each); the Python binding, with its checks, runs the first warm-up step and every test.
    if args.allocator == "device":
        binding_step = step
        binding_step()
        lib = B.lib()
        sp = stream.cuda_stream
        dt = B.ACTQ_F16 if wl.dtype == "f16" else B.ACTQ_F32
        xp, gminp, grp, g2p, wp = x.data_ptr(), gmin.data_ptr(), grange.data_ptr(), grad2.data_ptr(), w_dev.data_ptr()
        bp, op, rp = bits_dev.data_ptr(), offs_dev.data_ptr(), result_dev.data_ptr()
        pkp, cap, hp, outp = packed_buf.data_ptr(), packed_buf.numel(), header.data_ptr(), out.data_ptr()
        seed, tag, nb = wl.philox_seed, wl.tag, args.noise_bits
        names = ("group_stats", "sensitivity+allocate", "quantize_pack", "unpack_dequantize")
        # five boundary events per step: the end of one launch is the start of the next
        # (and a sixth right behind the fifth: the interval with nothing in it, which every interval contains)
        pool = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 2)] for _ in range(args.steps)]
        cursor = [0]

        def step(events=None):
            ev = None
            if events is not None:
                ev = pool[cursor[0]]
                cursor[0] += 1
                for i, name in enumerate(names):
                    events.setdefault(name, []).extend([(0, ev[i]), (1, ev[i + 1])])
                ev[0].record(stream)
            rc = lib.actq_group_stats(xp, dt, N, D, G, gminp, grp, sp)
            if ev:
                ev[1].record(stream)
            rc |= lib.actq_sample_sensitivity(grp, N, ng, G, g2p, wp, sp)
            rc |= lib.actq_allocate_bits_device(wp, None, D, N, G, budget, widths, bp, op, rp, sp)
            if ev:
                ev[2].record(stream)
            rc |= lib.actq_quantize_pack(xp, dt, N, D, G, bp, op, seed, tag, nb, pkp, cap, hp, hf, sp)
            if ev:
                ev[3].record(stream)
            rc |= lib.actq_unpack_dequantize(pkp, cap, hp, hf, bp, op, N, D, G, outp, dt, sp)
            if ev:
                ev[4].record(stream)
                ev[5].record(stream)
                events.setdefault("_empty", []).extend([(0, ev[4]), (1, ev[5])])
            if rc:
                raise RuntimeError(B.last_error())

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.profile_pass:
        copy_dst = torch.empty_like(x)
        for _ in range(3):
            copy_dst.copy_(x)          # reads and writes N*D*elem_bytes each: the calibration kernel
            step()
        read_back()
        print(json.dumps({"profile_pass": True, "workload": wl.name, "copy_bytes_each_way": N * D * wl.elem_bytes,
                          "packed_bytes": state["total"], "header_bytes": N * ng * 8}))
        return None
    read_back()
    assert np.array_equal(state["bits"], wl.bits), "allocator did not return the workload's widths"

    # Every `--event-every`-th timed step carries the HIP events that give the per-kernel durations;
    # the steps in between run bare, so that recording events (about 4 us each on the stream) does
    # not dominate the gaps between five short launches.
    events = {}
    every = max(1, args.event_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events if i % every == 0 else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    kernel_ms, kernel_spread = {}, {}
    empty_marks = events.pop("_empty", None)
    empty_interval_ms = None
    if empty_marks:
        empty_interval_ms = float(np.mean([a.elapsed_time(b) for (_, a), (_, b) in zip(empty_marks[0::2], empty_marks[1::2])]))
    for name, marks in events.items():
        starts = [e for when, e in marks if when == 0]
        stops = [e for when, e in marks if when == 1]
        each = [a.elapsed_time(b) for a, b in zip(starts, stops)]
        kernel_ms[name] = float(np.mean(each))
        kernel_spread[name] = {"median_ms": float(np.median(each)), "min_ms": float(np.min(each))}

    # What plain streaming kernels reach on the same bytes (torch's copy and fill, same stream, after
    # the timed region): the practical ceilings beside the 8 TB/s peak.
    ceilings = {}
    other = torch.empty_like(x)
    for label, call, moved in (("device_copy", lambda: other.copy_(x), 2 * N * D * wl.elem_bytes),
                               ("device_fill", lambda: other.fill_(1.0), N * D * wl.elem_bytes)):
        for _ in range(3):
            call()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(20):
            call()
        b.record(stream)
        b.synchronize()
        ceilings[label] = {"ms": a.elapsed_time(b) / 20, "GBps": moved / (a.elapsed_time(b) / 20) / 1e6}
    del other

    read_back()
    assert np.array_equal(state["bits"], wl.bits)
    in_bytes = N * D * wl.elem_bytes
    alg = algorithmic_bytes(N, D, ng, wl.elem_bytes, state["total"], 4 if hf == B.ACTQ_HDR_BF16 else 8)
    per_kernel = {k: {"ms": kernel_ms[k], **kernel_spread[k], "input_GBps": in_bytes / kernel_ms[k] / 1e6,
                      "algorithmic_GBps": alg[k] / kernel_ms[k] / 1e6,
                      "frac_of_hbm_peak": alg[k] / kernel_ms[k] / 1e6 / HBM_PEAK_GBS} for k in alg}
    if "sensitivity+allocate" in kernel_ms:   # two small launches that read N*ng ranges and N sensitivities
        per_kernel["sensitivity+allocate"] = {"ms": kernel_ms["sensitivity+allocate"]}
    dominant = max(alg, key=kernel_ms.get)
    achieved = alg[dominant] / kernel_ms[dominant] / 1e6
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": None if args.uniform_bits else measured_traffic(wl.name, args.noise_bits, dominant),
                "algorithmic_bytes_per_launch": alg[dominant], "avg_launch_ms": kernel_ms[dominant]}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        t = time.perf_counter()
        oracle.group_stats(x_np, G)
        if hf == B.ACTQ_HDR_BF16:
            opacked, oheader, ooff = oracle.quantize_pack_bf16(x_np, wl.bits, wl.philox_seed, wl.tag, G, args.noise_bits)
            oracle.unpack_dequantize_bf16(opacked, oheader, wl.bits, ooff, N, D, G, out_dtype=x_np.dtype)
        else:
            opacked, oheader, ooff = oracle.quantize_pack(x_np, wl.bits, wl.philox_seed, wl.tag, G, args.noise_bits)
            oracle.unpack_dequantize(opacked, oheader, wl.bits, ooff, N, D, G, out_dtype=x_np.dtype)
        cpu_s = time.perf_counter() - t
        cpu_baseline = {"value": in_bytes / cpu_s / 1e9, "unit": "GB/s", "cores": oracle.threads(),
                        "kind": "oracle",
                        "sample": f"one full step (group_stats + quantize_pack + unpack_dequantize) on the whole "
                                  f"workload, {N * D} elements, {cpu_s:.2f} s",
                        "single_thread": single_thread}

    result = {
        "metric": "quantize+pack and unpack+dequant GB/s (fp32 input); % of HBM peak",
        "value": in_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": wl.name, "G": G, "mean_bits": float(wl.bits.astype(np.float64).mean()),
                   "noise_bits": args.noise_bits, "header": args.header,
                   "allocator": args.allocator, "steps_with_events": (args.steps + max(1, args.event_every) - 1) // max(1, args.event_every),
                   "step": ("group_stats + sample_sensitivity + allocate_bits_device + quantize_pack + unpack_dequantize"
                            if args.allocator == "device" else
                            "group_stats + allocate_bits(host) + quantize_pack + unpack_dequantize")},
        "kernels": per_kernel,
        "empty_event_interval_ms": empty_interval_ms,
        "ceilings": ceilings,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
    }
    return result


if __name__ == "__main__":
    main()
