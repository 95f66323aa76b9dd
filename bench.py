#!/usr/bin/env python3
"""Throughput of the K-TanH library on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extra] [--no-cpu] [--probe]

Headline (the JSON line's `value`): ktanh_bf16 over the LSTM gate pre-activation tensor
[50, 128, 4096] BFloat16 ~ N(0, 1.5^2).  One step = one call of the C-ABI entry point over one such
tensor, input already in HBM.  The tensor (105 MB of traffic) would fit the 256 MB last-level cache,
so the steps rotate through 8 distinct input/output pairs (839 MB): what is timed is HBM, not cache.

`roofline` is for the kernel behind that call: algorithmic bytes (4 B per element) over its average
duration, taken with HIP events on the launching stream around the timed steps.  `extra` holds the
same two figures for the other entry points on their own workloads.  `cpu_baseline` times the
reference oracle (plain scalar C, one thread) on repeated passes over the same tensor.

--probe runs a few launches of every kernel plus a plain device copy of known size and exits: it is
the command the rocprofv3 kernel-trace and counter summaries under profiles/ are taken with.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0           # MI355X HBM3E, published peak
ROTATE = 8                      # distinct buffer pairs the headline steps cycle through
HEADLINE_ROLL = 4099            # buffer k holds the seeded tensor rotated by k * this many elements
PAPER_CONTEXT = "paper: 0.28 cycles/TanH, 5.46x over Intel SVML on AVX512 CLX (Table 2) -- other hardware, context only"


def kernel_source_digest():
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1909_07729_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as fh:
            h.update(name.encode() + b"\0" + fh.read())
    return h.hexdigest()[:16]


def measured_traffic(kernel):
    """HBM bytes per launch from the committed counter run, or None once the kernels changed."""
    path = os.path.join(ROOT, "paper_1909_07729_amd", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        rec = json.load(fh)
    if rec.get("kernel_source_digest") != kernel_source_digest():
        return None
    return rec.get("bytes_per_launch", {}).get(kernel)


def time_steps(torch, launch, steps, warmup):
    """(wall seconds, event seconds) for `steps` calls of launch(i) after `warmup` untimed ones."""
    for i in range(warmup):
        launch(i)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start.record()
    for i in range(steps):
        launch(i)
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, start.elapsed_time(stop) * 1e-3


def make_upload(np, torch, dev):
    def upload(a):
        view = {np.dtype(np.uint16): np.int16, np.dtype(np.uint32): np.int32}.get(a.dtype, a.dtype)
        return torch.from_numpy(a.view(view)).to(dev)
    return upload


def make_headline(torch, binding, wl, upload):
    """The timed step: ktanh_bf16 on the [50,128,4096] gate tensor, over ROTATE buffer pairs (buffer k
    is the seeded tensor rotated by k * 4099 elements: distinct memory, same value mix).  Returns the
    step function, with its buffers as attributes, and the host tensor."""
    x_host = wl.lstm_gate_preactivations()
    xs = [upload(x_host)]
    for k in range(1, ROTATE):
        xs.append(xs[0].roll(k * HEADLINE_ROLL))
    ys = [torch.empty_like(x) for x in xs]

    def headline(i):
        binding.ktanh_bf16(xs[i % ROTATE], out=ys[i % ROTATE])
    headline.inputs, headline.outputs = xs, ys
    return headline, x_host


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5000)
    ap.add_argument("--warmup", type=int, default=1000)   # the first ~10 ms after idle run slower
    ap.add_argument("--no-extra", action="store_true", help="headline only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--probe", action="store_true", help="few launches of each kernel + a copy, for rocprofv3")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library is measured on ONE GPU (the op is element-wise and shards "
                 "into independent ranges with no exchange); run with --gpus 1")

    import numpy as np
    import torch
    from paper_1909_07729_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    binding.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    upload = make_upload(np, torch, dev)
    headline, x_host = make_headline(torch, binding, wl, upload)
    xs, ys = headline.inputs, headline.outputs
    n = x_host.size

    if args.probe:
        run_probe(torch, binding, wl, upload, headline, xs[0])
        return

    wall, ev = time_steps(torch, headline, args.steps, args.warmup)
    ms_per_step = wall / args.steps * 1e3
    value = n / (wall / args.steps)
    kernel_s = ev / args.steps
    achieved = 4.0 * n / kernel_s / 1e9
    result = {
        "metric": "K-TanH bf16 elements/sec and achieved HBM GB/s (% of peak) on 1 MI355X",
        "value": value,
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u16",
        "data": "synthetic",
        "config": {
            "workload": "ktanh_bf16 on LSTM gate pre-activations [50,128,4096] bf16 ~ N(0,1.5^2), seed 190902",
            "elements_per_step": n,
            "rotating_buffer_pairs": ROTATE,
            "hbm_gb_per_s": 4.0 * n / (wall / args.steps) / 1e9,
            "context": PAPER_CONTEXT,
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "stream_kernel<bf16, K-TanH>",
            "achieved": achieved,
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": achieved / PEAK_HBM_GBS,
            "traffic": measured_traffic("ktanh_bf16"),
            "algorithmic_bytes_per_launch": 4 * n,
            "avg_launch_us": kernel_s * 1e6,
        },
    }

    if not args.no_extra:
        result["extra"] = run_extras(torch, binding, wl, upload, xs, ys)
        # the same launch shape and accesses with no arithmetic, timed in this run: the memory system's ceiling
        result["roofline"]["copy_same_shape_us"] = result["extra"]["stream_copy_same_shape"]["avg_launch_us"]
    if not args.no_cpu:
        result["cpu_baseline"] = run_cpu_baseline(x_host)
    print(json.dumps(result))


def run_extras(torch, binding, wl, upload, xs, ys):
    """elements/s and GB/s of the other entry points on their own workloads."""
    import numpy as np
    out = {}

    def record(name, workload, launch, units, bytes_per_unit, steps, warmup=5):
        wall, ev = time_steps(torch, launch, steps, warmup)
        gbs = units * bytes_per_unit / (ev / steps) / 1e9
        out[name] = {"workload": workload, "units_per_s": units / (wall / steps),
                     "avg_launch_us": ev / steps * 1e6, "hbm_gb_per_s": gbs,
                     "frac_of_peak": gbs / PEAK_HBM_GBS, "bytes_per_unit": bytes_per_unit}

    # same tensor, same buffers every step: what a cache-resident activation sees
    record("ktanh_bf16_cache_resident", "[50,128,4096] bf16, one buffer pair reused (fits the 256 MB cache)",
           lambda i: binding.ktanh_bf16(xs[0], out=ys[0]), xs[0].numel(), 4, 2000, 500)

    # yardstick: the runtime's own device-to-device copy of the same tensor (same bytes, no arithmetic)
    record("plain_copy_same_size", "hipMemcpyAsync device-to-device of the headline tensor, same 8 rotating pairs",
           lambda i: ys[i % ROTATE].copy_(xs[i % ROTATE]), xs[0].numel(), 4, 2000, 500)
    record("stream_copy_same_shape", "the same launch shape and access policies with no arithmetic (ktanh_stream_copy), same 8 rotating pairs",
           lambda i: binding.ktanh_stream_copy(xs[i % ROTATE], out=ys[i % ROTATE]), xs[0].numel(), 4, 2000, 500)
    record("ktanh64_bf16", "[50,128,4096] bf16 as in the headline, 64-interval table, 8 rotating buffer pairs",
           lambda i: binding.ktanh64_bf16(xs[i % ROTATE], out=ys[i % ROTATE]), xs[0].numel(), 4, 2000, 500)

    record("ktanh_bf16_backward", "dy, y and dx as the headline tensor (6 B per element), 8 rotating triples",
           lambda i: binding.ktanh_bf16_backward(xs[i % ROTATE], ys[(i + 1) % ROTATE], dx=ys[i % ROTATE]),
           xs[0].numel(), 6, 2000, 500)

    for name in ("kswish_backward", "kgelu_backward"):
        record(name, "dy, x and dx as the headline tensor (6 B per element), 8 rotating triples; the K-TanH value is rebuilt from x",
               lambda i, fn=getattr(binding, name): fn(xs[(i + 1) % ROTATE], xs[i % ROTATE], dx=ys[i % ROTATE]),
               xs[0].numel(), 6, 2000, 500)

    # the large tensors rotate as well: a 537 MB working set still keeps part of itself in the cache
    x4 = [upload(wl.mlp_preactivations())]
    for k in range(1, 4):
        x4.append(x4[0].roll(k * 4099))
    y4 = [torch.empty_like(t) for t in x4]
    for name in ("ktanh_bf16", "ksigmoid", "kswish", "kgelu"):
        fn = getattr(binding, name)
        record(f"{name}_mlp", "[8192,16384] bf16 ~ N(0,1), seed 190904, 4 rotating buffer pairs",
               lambda i, fn=fn: fn(x4[i % 4], out=y4[i % 4]), x4[0].numel(), 4, 200, 100)
    del x4, y4

    x3 = [upload(wl.f32_mixture())]
    x3.append(x3[0].roll(4099))
    y3 = [torch.empty_like(t) for t in x3]
    record("ktanh_f32", "2^28 fp32, uniform[-8,8) + 5% N(0,0.01^2), seed 190903, 2 rotating buffer pairs",
           lambda i: binding.ktanh_f32(x3[i % 2], out=y3[i % 2]), x3[0].numel(), 8, 100, 30)
    x3f = [t.view(torch.float32) for t in x3]
    y3f = [t.view(torch.float32) for t in y3]
    for name in ("ksigmoid_f32", "kswish_f32", "kgelu_f32"):
        fn = getattr(binding, name)
        record(name, "same 2^28 fp32 tensor, fp32 in and out, 2 rotating buffer pairs",
               lambda i, fn=fn: fn(x3f[i % 2], out=y3f[i % 2]), x3[0].numel(), 8, 60, 10)
    record("kgelu_f32_backward", "dy, x and dx of 2^28 fp32 each (12 B per element), dx alternating over 2 buffers",
           lambda i: binding.kgelu_f32_backward(x3f[1], x3f[0], dx=y3f[i % 2]), x3[0].numel(), 12, 40, 10)
    y3h = [torch.empty(x3[0].numel(), dtype=torch.bfloat16, device=x3[0].device) for _ in range(2)]
    record("ktanh_f32_to_bf16", "same 2^28 fp32 tensor in, bf16 out (conversion fused into the load)",
           lambda i: binding.ktanh_f32_to_bf16(x3f[i % 2], out=y3h[i % 2]), x3[0].numel(), 6, 60, 4)
    del x3, y3, x3f, y3f, y3h

    gates_h, c0_h = wl.lstm_cell_inputs()
    gates, c0 = upload(gates_h), torch.from_numpy(c0_h).to("cuda:0")
    T, B, H4 = gates.shape
    cells = B * (H4 // 4)
    c = c0.clone()
    gates_rot = [gates, gates.roll(4099), gates.roll(8209)]
    h_rot = [torch.empty((T, B, H4 // 4), dtype=gates.dtype, device=gates.device) for _ in range(3)]
    h = h_rot[0]
    # one call per time step, the way a recurrent network issues it; the 64 launches are captured in
    # a HIP graph so that the host's launch cost does not hide the kernel
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for t in range(T):
            binding.klstm_cell(gates[t:t + 1], c, c_out=c, h_out=h[t:t + 1])
    record("klstm_cell_per_step", "gates [64,256,8192] bf16 ~ N(0,4), c [256,2048] fp32; 64 calls of one "
           "time step each (replayed as a HIP graph), figures per call",
           lambda i: graph.replay(), cells * T, 18, 40, 20)
    out["klstm_cell_per_step"]["avg_launch_us"] /= T
    record("klstm_cell_fused_T64", "same shapes, 3 rotating gate/h buffers; one call carries c through all 64 steps",
           lambda i: binding.klstm_cell(gates_rot[i % 3], c0, c_out=c, h_out=h_rot[i % 3]), cells * T,
           10 + 8.0 / T, 90, 30)
    return out


def run_cpu_baseline(x_host):
    from oracle import ktanh_oracle as oracle
    oracle.ktanh_bf16(x_host[:1024])
    passes, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < 10.0:
        oracle.ktanh_bf16(x_host)
        passes += 1
    dt = time.perf_counter() - t0
    base = {"value": passes * x_host.size / dt, "unit": "elements/s", "cores": 1, "kind": "oracle",
            "sample": f"{passes} passes of oracle_ktanh_bf16 over the same {x_host.size}-element tensor ({dt:.1f} s, scalar C, one thread)"}
    # the same function on disjoint slices from one thread per core of this process's share
    # (the C call releases the interpreter lock); context only
    import concurrent.futures
    import numpy as np
    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    parts = np.array_split(x_host.reshape(-1), threads)
    with concurrent.futures.ThreadPoolExecutor(threads) as pool:
        list(pool.map(oracle.ktanh_bf16, parts))
        rounds, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < 5.0:
            list(pool.map(oracle.ktanh_bf16, parts))
            rounds += 1
        dt = time.perf_counter() - t0
    base["all_cores"] = {"value": rounds * x_host.size / dt, "unit": "elements/s", "cores": threads,
                         "sample": f"{rounds} passes, the tensor cut into {threads} slices, one thread each ({dt:.1f} s)"}
    return base


def run_probe(torch, binding, wl, upload, headline, x):
    """A few launches of every kernel on buffers not touched just before, plus plain device copies
    of known size (the yardstick the HBM counters are scaled by)."""
    for i in range(ROTATE):
        headline(i)
    for i in range(ROTATE):
        binding.ktanh_stream_copy(headline.inputs[i], out=headline.outputs[i])
    for i in range(ROTATE):
        binding.ktanh64_bf16(headline.inputs[i], out=headline.outputs[i])
    for i in range(ROTATE):
        binding.ktanh_bf16_backward(headline.inputs[i], headline.outputs[(i + 1) % ROTATE],
                                    dx=headline.outputs[i])
    for i in range(ROTATE):
        binding.kgelu_backward(headline.inputs[(i + 1) % ROTATE], headline.inputs[i], dx=headline.outputs[i])
    spare = [torch.empty_like(x) for _ in range(4)]
    for k in range(4):
        spare[k].copy_(headline.inputs[k + 4])      # plain copy: 52,428,800 B read + as many written
    torch.cuda.synchronize()
    del spare

    x4 = [upload(wl.mlp_preactivations())]
    x4.append(x4[0].roll(4099))
    y4 = [torch.empty_like(t) for t in x4]
    for name in ("ktanh_bf16", "ksigmoid", "kswish", "kgelu"):
        for k in range(2):
            getattr(binding, name)(x4[k], out=y4[k])
    for k in range(2):
        y4[k].copy_(x4[1 - k])                      # plain copy: 268,435,456 B each way
    torch.cuda.synchronize()
    del x4, y4

    x3 = [upload(wl.f32_mixture())]
    x3.append(x3[0].roll(4099))
    y3 = [torch.empty_like(t) for t in x3]
    for k in range(2):
        binding.ktanh_f32(x3[k], out=y3[k])
    x3f, y3f = [t.view(torch.float32) for t in x3], [t.view(torch.float32) for t in y3]
    for name in ("ksigmoid_f32", "kswish_f32", "kgelu_f32"):
        for k in range(2):
            getattr(binding, name)(x3f[k], out=y3f[k])
    y3h = [torch.empty(x3[0].numel(), dtype=torch.bfloat16, device=x3[0].device) for _ in range(2)]
    for k in range(2):
        binding.ktanh_f32_to_bf16(x3f[k], out=y3h[k])
    torch.cuda.synchronize()
    del x3, y3, x3f, y3f, y3h

    gates_h, c0_h = wl.lstm_cell_inputs()
    gates, c0 = upload(gates_h), torch.from_numpy(c0_h).to("cuda:0")
    for _ in range(2):
        binding.klstm_cell(gates, c0)
    for t in range(8):
        binding.klstm_cell(gates[t:t + 1], c0)
    dh = torch.zeros((c0.shape[0], c0.shape[1]), dtype=gates.dtype, device=gates.device)
    for t in range(8):
        binding.klstm_cell_backward(gates[t], c0, dh, c0)
    torch.cuda.synchronize()
    print("probe done")


if __name__ == "__main__":
    main()
