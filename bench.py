#!/usr/bin/env python3
"""Throughput of the K-TanH library on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extra] [--no-cpu] [--probe]

Headline (the JSON line's `value`): ktanh_bf16 over the LSTM gate pre-activation tensor
[50, 128, 4096] BFloat16 ~ N(0, 1.5^2).  One step = one call of the C-ABI entry point over one such
tensor, input already in HBM.  The tensor (105 MB of traffic) would fit the 256 MB last-level cache,
so the steps rotate through 8 distinct input/output pairs (839 MB): what is timed is HBM, not cache.

Timing: W untimed steps, a synchronisation, then exactly K steps between two readings of the host
clock, and a synchronisation: `value` and `ms_per_step` come from the host clock, and nothing else is
inside that region (the same K steps are then repeated between two HIP events on the launching stream
for `timed_region_launch_us`; recorded inside the timed region, the two events would cost a 20-step
run 7 % of its `value`).  `roofline` is for the kernel behind the call: algorithmic bytes (4 B per
element) over its average duration, taken with HIP events around K launches issued right behind W
others, so that the queue never runs empty -- five such groups of max(K, 200) launches, with their
mean, median and minimum (the timed region itself starts on an idle queue and holds the host's launch
latency once, which is 2 % of a 20-step run, and the two events of a group cost 4-8 us, which is as
much; the timed region's own event figure is reported as `timed_region_launch_us`).  An event between
every two launches is not used for that: it costs microseconds per launch on this runtime (the run
records what it reads and what it costs as `roofline.one_event_pair_per_launch`).  `extra` holds the same figures for the other entry points on their own
workloads, the yardsticks of the measurement library (the same launch with the arithmetic, the
stores or the loads taken out) and a sweep over tensor sizes with its fitted fixed cost per launch.
`cpu_baseline` times the reference oracle (plain scalar C) on every workload, on one thread and on
one thread per core.

--probe launches every kernel at least 20 times on rotating buffers, plus plain device copies of
known size, and exits: it is the command the rocprofv3 kernel-trace and counter summaries under
profiles/ are taken with.
"""
import argparse
import hashlib
import json
import os
import statistics
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
    """HBM bytes per launch from the committed counter runs (profiles/hbm_traffic.json), or None once
    the kernel sources have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        rec = json.load(fh)
    if rec.get("kernel_source_digest") != kernel_source_digest():
        return None
    return rec.get("bytes_per_launch", {}).get(kernel)


GROUPS = 5                      # back-to-back groups of launches behind the kernel figures
GROUP_MIN_LAUNCHES = 200        # the two events of a group cost 4-8 us: too much for 20 launches of 17 us


def time_steps(torch, launch, steps, warmup, groups=GROUPS, group_min=1):
    """The timed region: `warmup` untimed calls of launch(i), a synchronisation, `steps` calls between
    two readings of the host clock, a synchronisation -- and nothing else (an event recorded inside it
    costs more than a microsecond per step of a 20-step region).  The same region once more between
    two events, for the duration as the device saw it.  Then, for the duration of the kernel itself,
    `groups` times: `warmup` calls followed, with the queue still full, by max(`steps`, `group_min`)
    calls between two events -- without the host's launch latency after an idle queue, which a region
    holds once.  The groups follow each other with no synchronisation in between.  Returns (host
    seconds of the timed region, event seconds per launch of the repeated region, [event seconds per
    launch of each group])."""
    for i in range(warmup):
        launch(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        launch(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    first.record()
    for i in range(steps):
        launch(i)
    last.record()
    torch.cuda.synchronize()
    region = first.elapsed_time(last) * 1e-3 / steps
    per_group = max(steps, group_min)
    marks = []
    for _ in range(groups):
        first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(max(warmup, 2)):
            launch(i)
        first.record()
        for i in range(per_group):
            launch(i)
        last.record()
        marks.append((first, last))
    torch.cuda.synchronize()
    return wall, region, [a.elapsed_time(b) * 1e-3 / per_group for a, b in marks]


def one_event_pair_per_launch(torch, launch, n):
    """The other way to time a kernel: an event before and after every single launch.  On this runtime
    each recorded event occupies the queue for microseconds, so both the pairs' own readings and the
    pace of the run they perturb are reported, next to the undisturbed figures."""
    pairs = []
    for i in range(n):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        launch(i)
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    us = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)
    return {"launches": n, "median_us": statistics.median(us), "min_us": us[0], "mean_us": sum(us) / n,
            "us_per_step_of_that_run": pairs[0][0].elapsed_time(pairs[-1][1]) * 1e3 / n}


def launch_stats(region, per_launch):
    """Microseconds per launch: mean, median and minimum over the back-to-back groups, and the figure
    of the timed region itself (which starts on an idle queue)."""
    us = [t * 1e6 for t in per_launch]
    return {"avg_launch_us": sum(us) / len(us), "median_launch_us": statistics.median(us),
            "min_launch_us": min(us), "timed_region_launch_us": region * 1e6}


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
    ap.add_argument("--warmup", type=int, default=1000)
    ap.add_argument("--no-extra", action="store_true", help="headline only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--probe", action="store_true", help="20+ launches of each kernel + plain copies, for rocprofv3")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library is measured on ONE GPU (the op is element-wise and shards "
                 "into independent ranges with no exchange); run with --gpus 1")

    import numpy as np
    import torch
    from paper_1909_07729_amd import binding, probe, workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    binding.load_library()
    probe.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    upload = make_upload(np, torch, dev)
    headline, x_host = make_headline(torch, binding, wl, upload)
    xs, ys = headline.inputs, headline.outputs
    n = x_host.size

    if args.probe:
        run_probe(torch, binding, probe, wl, upload, headline)
        return

    # Bring the device out of its idle clocks before anything is measured: after the uploads above the
    # first 20-50 ms of work run 2-3 % slower than what follows, whatever the kernel (power
    # management, not this library).  60 ms of the headline call on its own buffers, untimed; the W
    # warm-up steps and the K timed steps that follow are the ones the caller asked for.
    settle_until = time.perf_counter() + 0.06
    while time.perf_counter() < settle_until:
        for i in range(64):
            headline(i)
        torch.cuda.synchronize()

    wall, region, per_launch = time_steps(torch, headline, args.steps, args.warmup, group_min=GROUP_MIN_LAUNCHES)
    stats = launch_stats(region, per_launch)
    stats["one_event_pair_per_launch"] = one_event_pair_per_launch(torch, headline, GROUP_MIN_LAUNCHES)
    ms_per_step = wall / args.steps * 1e3
    achieved = 4.0 * n / (stats["avg_launch_us"] * 1e-6) / 1e9
    result = {
        "metric": "K-TanH bf16 elements/sec and achieved HBM GB/s (% of peak) on 1 MI355X",
        "value": n / (wall / args.steps),
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
            **stats,
            "frac_at_median": 4.0 * n / (stats["median_launch_us"] * 1e-6) / 1e9 / PEAK_HBM_GBS,
        },
    }

    if not args.no_extra:
        result["extra"] = run_extras(torch, binding, probe, wl, upload, xs, ys)
        # the same launch with no arithmetic, timed in this run: what the memory system allows for this tensor
        result["roofline"]["copy_same_shape_us"] = result["extra"]["probe_copy_headline"]["median_launch_us"]
    if not args.no_cpu:
        result["cpu_baseline"] = run_cpu_baseline(wl, x_host)
    print(json.dumps(result))


def run_extras(torch, binding, probe, wl, upload, xs, ys):
    """elements/s and GB/s of the other entry points on their own workloads, the yardsticks, and the
    size sweep."""
    import numpy as np
    out = {}

    def record(name, workload, launch, units, bytes_per_unit, steps, warmup=5):
        wall, region, per_launch = time_steps(torch, launch, steps, warmup, groups=3)
        st = launch_stats(region, per_launch)
        gbs = units * bytes_per_unit / (st["avg_launch_us"] * 1e-6) / 1e9
        gbs_med = units * bytes_per_unit / (st["median_launch_us"] * 1e-6) / 1e9
        out[name] = {"workload": workload, "units_per_s": units / (wall / steps), **st,
                     "hbm_gb_per_s": gbs, "frac_of_peak": gbs / PEAK_HBM_GBS,
                     "frac_of_peak_at_median": gbs_med / PEAK_HBM_GBS, "bytes_per_unit": bytes_per_unit}
        return out[name]

    n2 = xs[0].numel()
    # same tensor, same buffers every step: what a cache-resident activation sees
    record("ktanh_bf16_cache_resident", "[50,128,4096] bf16, one buffer pair reused (fits the 256 MB cache)",
           lambda i: binding.ktanh_bf16(xs[0], out=ys[0]), n2, 4, 1000, 200)
    # yardsticks on the headline tensor: the runtime's own device-to-device copy, and the launch of
    # ktanh_bf16 with no arithmetic
    record("plain_copy_same_size", "hipMemcpyAsync device-to-device of the headline tensor, same 8 rotating pairs",
           lambda i: ys[i % ROTATE].copy_(xs[i % ROTATE]), n2, 4, 1000, 200)
    record("probe_copy_headline", "ktanh_probe_copy: the launch of ktanh_bf16 with no arithmetic, same 8 rotating pairs",
           lambda i: probe.ktanh_probe_copy(xs[i % ROTATE], ys[i % ROTATE]), n2, 4, 1000, 200)
    record("ktanh64_bf16", "[50,128,4096] bf16 as in the headline, 64-interval table, 8 rotating buffer pairs",
           lambda i: binding.ktanh64_bf16(xs[i % ROTATE], out=ys[i % ROTATE]), n2, 4, 1000, 200)
    for name in ("kpade32_bf16", "kpade78_bf16"):
        record(name, "Table 2's rational approximant (Float32 arithmetic with a division) on the headline tensor, 8 rotating pairs",
               lambda i, fn=getattr(binding, name): fn(xs[i % ROTATE], out=ys[i % ROTATE]), n2, 4, 1000, 200)
    for name in ("ktaylor2_bf16", "ktaylor3_bf16"):
        record(name, "piecewise Taylor polynomial on K-TanH's 32 intervals (3 or 4 Float32 coefficients per table read) on the headline tensor, 8 rotating pairs",
               lambda i, fn=getattr(binding, name): fn(xs[i % ROTATE], out=ys[i % ROTATE]), n2, 4, 1000, 200)
    record("ktanh_bf16_backward", "dy, y and dx as the headline tensor (6 B per element), 8 rotating triples",
           lambda i: binding.ktanh_bf16_backward(xs[i % ROTATE], ys[(i + 1) % ROTATE], dx=ys[i % ROTATE]),
           n2, 6, 1000, 200)
    for name in ("kswish_backward", "kgelu_backward", "kgelu64_backward"):
        record(name, "dy, x and dx as the headline tensor (6 B per element), 8 rotating triples; the K-TanH value is rebuilt from x",
               lambda i, fn=getattr(binding, name): fn(xs[(i + 1) % ROTATE], xs[i % ROTATE], dx=ys[i % ROTATE]),
               n2, 6, 1000, 200)

    # the large tensors rotate as well: a 537 MB working set still keeps part of itself in the cache
    x4 = [upload(wl.mlp_preactivations())]
    for k in range(1, 4):
        x4.append(x4[0].roll(k * 4099))
    y4 = [torch.empty_like(t) for t in x4]
    n4 = x4[0].numel()
    for name in ("ktanh_bf16", "ksigmoid", "kswish", "kgelu", "kpade32_bf16", "kpade78_bf16", "ktaylor2_bf16",
                 "ktaylor3_bf16"):
        fn = getattr(binding, name)
        record(f"{name}_mlp", "[8192,16384] bf16 ~ N(0,1), seed 190904, 4 rotating buffer pairs",
               lambda i, fn=fn: fn(x4[i % 4], out=y4[i % 4]), n4, 4, 200, 60)
    # what the memory system allows on that tensor in this launch shape: no arithmetic; loads alone;
    # stores alone.  HBM moves one direction at a time, so a stream that reads and writes the same
    # amount cannot beat the harmonic mean of the last two.
    sink = torch.zeros(512, dtype=torch.int16, device=x4[0].device)
    cp = record("probe_copy_mlp", "ktanh_probe_copy on the [8192,16384] bf16 tensor, 4 rotating pairs",
                lambda i: probe.ktanh_probe_copy(x4[i % 4], y4[i % 4]), n4, 4, 200, 60)
    rd = record("probe_read_mlp", "ktanh_probe_read: the loads of that launch alone (2 B per element)",
                lambda i: probe.ktanh_probe_read(x4[i % 4], sink), n4, 2, 200, 60)
    wr = record("probe_write_mlp", "ktanh_probe_write: the stores of that launch alone (2 B per element)",
                lambda i: probe.ktanh_probe_write(y4[i % 4]), n4, 2, 200, 60)
    rdw = record("probe_read_wide_mlp", "ktanh_probe_read_wide: the same loads from 512-thread blocks (an eighth of the blocks to dispatch)",
                 lambda i: probe.ktanh_probe_read(x4[i % 4], sink, wide=True), n4, 2, 200, 60)
    wrw = record("probe_write_wide_mlp", "ktanh_probe_write_wide: the same stores from 512-thread blocks",
                 lambda i: probe.ktanh_probe_write(y4[i % 4], wide=True), n4, 2, 200, 60)
    out["size_sweep"] = run_size_sweep(torch, binding, x4, y4)
    del x4, y4
    out["memory_system"] = {
        "note": "single-wavefront blocks are bound by the dispatcher when they only read or only write "
                "(the read+write stream the library launches needs half the blocks per byte); 512-thread "
                "blocks show what the memory system gives the same accesses in one direction alone",
        "copy_gb_per_s": cp["hbm_gb_per_s"], "read_only_gb_per_s": rd["hbm_gb_per_s"],
        "write_only_gb_per_s": wr["hbm_gb_per_s"], "read_only_wide_gb_per_s": rdw["hbm_gb_per_s"],
        "write_only_wide_gb_per_s": wrw["hbm_gb_per_s"]}

    x3 = [upload(wl.f32_mixture())]
    x3.append(x3[0].roll(4099))
    y3 = [torch.empty_like(t) for t in x3]
    n3 = x3[0].numel()
    record("ktanh_f32", "2^28 fp32, uniform[-8,8) + 5% N(0,0.01^2), seed 190903, 2 rotating buffer pairs",
           lambda i: binding.ktanh_f32(x3[i % 2], out=y3[i % 2]), n3, 8, 80, 20)
    x3f = [t.view(torch.float32) for t in x3]
    y3f = [t.view(torch.float32) for t in y3]
    for name in ("ksigmoid_f32", "kswish_f32", "kgelu_f32"):
        fn = getattr(binding, name)
        record(name, "same 2^28 fp32 tensor, fp32 in and out, 2 rotating buffer pairs",
               lambda i, fn=fn: fn(x3f[i % 2], out=y3f[i % 2]), n3, 8, 50, 10)
    record("kgelu_f32_backward", "dy, x and dx of 2^28 fp32 each (12 B per element), dx alternating over 2 buffers",
           lambda i: binding.kgelu_f32_backward(x3f[1], x3f[0], dx=y3f[i % 2]), n3, 12, 40, 10)
    y3h = [torch.empty(n3, dtype=torch.bfloat16, device=x3[0].device) for _ in range(2)]
    record("ktanh_f32_to_bf16", "same 2^28 fp32 tensor in, bf16 out (conversion fused into the load)",
           lambda i: binding.ktanh_f32_to_bf16(x3f[i % 2], out=y3h[i % 2]), n3, 6, 50, 10)
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
    rec = record("klstm_cell_per_step", "gates [64,256,8192] bf16 ~ N(0,4), c [256,2048] fp32; 64 calls of one "
                 "time step each (replayed as a HIP graph), figures per call",
                 lambda i: graph.replay(), cells * T, 18, 100, 200)  # 45 ms of warm-up: the clocks settle slowly under launch-bound work
    for key in ("avg_launch_us", "median_launch_us", "min_launch_us", "timed_region_launch_us"):
        rec[key] /= T
    record("klstm_cell_fused_T64", "same shapes, 3 rotating gate/h buffers; one call carries c through all 64 steps",
           lambda i: binding.klstm_cell(gates_rot[i % 3], c0, c_out=c, h_out=h_rot[i % 3]), cells * T,
           10 + 8.0 / T, 400, 200)  # long enough for the clocks to settle after the launch-bound graph replays
    # one step backwards per call, the way back-propagation through time issues it (each step's dh needs
    # the recurrent product of the step after it, so the steps cannot share a launch); again as a graph
    dh = h_rot[1][0]
    dgates = torch.empty_like(gates)
    dc_a, dc_b = torch.ones_like(c0), torch.empty_like(c0)
    torch.cuda.synchronize()
    graph_b = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph_b):
        for t in range(T - 1, -1, -1):
            binding.klstm_cell_backward(gates[t], c0, dh, dc_a, dgates=dgates[t], dc_prev=dc_b)
            dc_a, dc_b = dc_b, dc_a
    rec = record("klstm_cell_backward_per_step", "one LSTM-cell step backwards per call on [256,2048] cells (gates, c_prev, dh, dc_next in; "
                 "dgates, dc_prev out: 30 B per cell), 64 calls replayed as a HIP graph, figures per call",
                 lambda i: graph_b.replay(), cells * T, 30, 100, 200)
    for key in ("avg_launch_us", "median_launch_us", "min_launch_us", "timed_region_launch_us"):
        rec[key] /= T
    # the launch of the fused kernel with its arithmetic taken out, on the same buffers
    record("probe_lstm_T64", "ktanh_probe_lstm: the loads, stores, waits and loop of klstm_cell_fused_T64 with no arithmetic, same buffers",
           lambda i: probe.ktanh_probe_lstm(gates_rot[i % 3], c0, c, h_rot[i % 3]), cells * T, 10 + 8.0 / T, 400, 200)
    return out


def run_size_sweep(torch, binding, pool_in, pool_out):
    """ktanh_bf16 on slices of 2^24 .. 2^27 elements (67 .. 537 MB of traffic; below that a call from
    Python takes longer to issue than the kernel to run), each size rotating over distinct slices of
    the big buffers (at least 1 GB touched per cycle), median of three groups of 48 launches; then the
    least-squares line  duration = fixed + bytes / rate  through the points below 256 MiB of output
    (from there on the kernel runs two windows through the tensor, which is faster)."""
    points = []
    whole = pool_in[0].numel()
    pool_in, pool_out = [t.view(-1) for t in pool_in], [t.view(-1) for t in pool_out]
    for n in (1 << 24, 3 << 23, 1 << 25, 3 << 24, 1 << 26, 3 << 25, 1 << 27):
        per = whole // n
        pairs = [(pool_in[k // per][(k % per) * n:(k % per + 1) * n], pool_out[k // per][(k % per) * n:(k % per + 1) * n])
                 for k in range(min(len(pool_in) * per, max(4, (1 << 28) // n)))]
        _, _, per_launch = time_steps(torch, lambda i: binding.ktanh_bf16(pairs[i % len(pairs)][0], out=pairs[i % len(pairs)][1]),
                                      48, 16, groups=3)
        points.append((4.0 * n, statistics.median(per_launch)))
    line = [(b, t) for b, t in points if b < 4.0 * (1 << 27)]
    mx = sum(b for b, _ in line) / len(line)
    my = sum(t for _, t in line) / len(line)
    slope = sum((b - mx) * (t - my) for b, t in line) / sum((b - mx) ** 2 for b, _ in line)
    return {"workload": "ktanh_bf16 on 2^24..2^27 bf16 elements, rotating slices, median of three groups of 48 launches each",
            "points": [{"traffic_mb": b / 1e6, "median_launch_us": t * 1e6, "gb_per_s": b / t / 1e9} for b, t in points],
            "fit_over": "the six sizes below 256 MiB of output",
            "fit_fixed_us_per_launch": (my - slope * mx) * 1e6, "fit_asymptotic_gb_per_s": 1.0 / slope / 1e9}


def run_cpu_baseline(wl, x_host):
    """The oracle as it stands (plain scalar C, gcc -O2), timed on this host: repeated passes over the
    headline tensor on one thread (the baseline `value`), then each workload on one thread and on one
    thread per core of this process's share, on a bounded sample of the workload."""
    import concurrent.futures
    import numpy as np
    from oracle import ktanh_oracle as oracle
    threads = max(1, min(16, len(os.sched_getaffinity(0))))

    def timed(fn, budget):
        fn()
        passes, t0 = 0, time.perf_counter()
        while True:
            fn()
            passes += 1
            dt = time.perf_counter() - t0
            if dt >= budget:
                return passes, dt

    def leg(name, units, sample, one, parts_of, budget=1.2):
        """`one()` runs the whole sample on the calling thread; parts_of(k) gives k closures that
        together run it once."""
        passes, dt = timed(one, budget)
        entry = {"unit": "elements/s", "kind": "oracle", "sample": sample,
                 "one_thread": {"value": passes * units / dt, "cores": 1, "seconds": dt}}
        parts = parts_of(threads)
        with concurrent.futures.ThreadPoolExecutor(threads) as pool:
            passes, dt = timed(lambda: list(pool.map(lambda f: f(), parts)), budget * 0.8)
        entry["all_cores"] = {"value": passes * units / dt, "cores": threads, "seconds": dt}
        return name, entry

    def slices(fn, arr, k):
        return [lambda part=part: fn(part) for part in np.array_split(arr, k)]

    passes, dt = timed(lambda: oracle.ktanh_bf16(x_host), 8.0)
    base = {"value": passes * x_host.size / dt, "unit": "elements/s", "cores": 1, "kind": "oracle",
            "sample": f"{passes} passes of oracle_ktanh_bf16 over the same {x_host.size}-element tensor ({dt:.1f} s, scalar C, one thread)"}
    flat = x_host.reshape(-1)
    with concurrent.futures.ThreadPoolExecutor(threads) as pool:
        parts = slices(oracle.ktanh_bf16, flat, threads)
        rounds, dt = timed(lambda: list(pool.map(lambda f: f(), parts)), 3.0)
    base["all_cores"] = {"value": rounds * x_host.size / dt, "unit": "elements/s", "cores": threads,
                         "sample": f"{rounds} passes, the tensor cut into {threads} slices, one thread each ({dt:.1f} s)"}

    per_config = {}
    n_s = 1 << 23
    x3 = wl.f32_mixture(n_s)
    name, entry = leg("ktanh_f32", n_s, f"the first {n_s} elements of the 2^28-element fp32 workload (seed 190903)",
                      lambda: oracle.ktanh_f32(x3), lambda k: slices(oracle.ktanh_f32, x3, k))
    per_config[name] = entry
    x4 = wl.mlp_preactivations(n_s)
    for op in ("ksigmoid", "kswish", "kgelu"):
        fn = getattr(oracle, op)
        name, entry = leg(op, n_s, f"the first {n_s} elements of the [8192,16384] bf16 workload (seed 190904)",
                          lambda fn=fn: fn(x4), lambda k, fn=fn: slices(fn, x4, k))
        per_config[name] = entry
    T, B, H = 64, 16, 2048
    gates, c0 = wl.lstm_cell_inputs(T, B, H)

    def cell_parts(k):
        rows = np.array_split(np.arange(B), min(k, B))
        return [lambda r=r: oracle.klstm_cell(np.ascontiguousarray(gates[:, r]), np.ascontiguousarray(c0[r])) for r in rows]
    name, entry = leg("klstm_cell", T * B * H, f"64 time steps of {B} of the 256 batch rows, H = 2048 (cell-steps per second)",
                      lambda: oracle.klstm_cell(gates, c0), cell_parts)
    entry["unit"] = "cell-steps/s"
    per_config[name] = entry
    base["per_config"] = per_config
    return base


def run_probe(torch, binding, probe, wl, upload, headline):
    """At least 20 launches of every kernel on rotating buffers, plus plain device copies of known
    size (the yardstick the HBM counters are scaled by)."""
    xs, ys = headline.inputs, headline.outputs
    R = 3 * ROTATE
    for i in range(R):
        headline(i)
    for i in range(R):
        probe.ktanh_probe_copy(xs[i % ROTATE], ys[i % ROTATE])
    for i in range(R):
        binding.ktanh64_bf16(xs[i % ROTATE], out=ys[i % ROTATE])
    for i in range(R):
        binding.ktanh_bf16_backward(xs[i % ROTATE], ys[(i + 1) % ROTATE], dx=ys[i % ROTATE])
    for i in range(R):
        binding.kgelu_backward(xs[(i + 1) % ROTATE], xs[i % ROTATE], dx=ys[i % ROTATE])
    for i in range(R):
        binding.kgelu64_backward(xs[(i + 1) % ROTATE], xs[i % ROTATE], dx=ys[i % ROTATE])
    spare = [torch.empty_like(xs[0]) for _ in range(4)]
    for k in range(4):
        spare[k].copy_(xs[k + 4])                   # plain copy: 52,428,800 B read + as many written
    torch.cuda.synchronize()
    del spare

    x4 = [upload(wl.mlp_preactivations())]
    for k in range(1, 4):
        x4.append(x4[0].roll(k * 4099))
    y4 = [torch.empty_like(t) for t in x4]
    sink = torch.zeros(512, dtype=torch.int16, device=x4[0].device)
    for name in ("ktanh_bf16", "ksigmoid", "kswish", "kgelu", "kpade32_bf16", "kpade78_bf16", "ktaylor2_bf16",
                 "ktaylor3_bf16"):
        for k in range(20):
            getattr(binding, name)(x4[k % 4], out=y4[k % 4])
    for k in range(20):
        probe.ktanh_probe_copy(x4[k % 4], y4[k % 4])
    for k in range(20):
        probe.ktanh_probe_read(x4[k % 4], sink)
    for k in range(20):
        probe.ktanh_probe_write(y4[k % 4])
    for k in range(20):
        probe.ktanh_probe_read(x4[k % 4], sink, wide=True)
    for k in range(20):
        probe.ktanh_probe_write(y4[k % 4], wide=True)
    for k in range(2):
        y4[k].copy_(x4[1 - k])                      # plain copy: 268,435,456 B each way
    torch.cuda.synchronize()
    del x4, y4

    x3 = [upload(wl.f32_mixture())]
    x3.append(x3[0].roll(4099))
    y3 = [torch.empty_like(t) for t in x3]
    for k in range(20):
        binding.ktanh_f32(x3[k % 2], out=y3[k % 2])
    x3f, y3f = [t.view(torch.float32) for t in x3], [t.view(torch.float32) for t in y3]
    for name in ("ksigmoid_f32", "kswish_f32", "kgelu_f32"):
        for k in range(20):
            getattr(binding, name)(x3f[k % 2], out=y3f[k % 2])
    y3h = [torch.empty(x3[0].numel(), dtype=torch.bfloat16, device=x3[0].device) for _ in range(2)]
    for k in range(20):
        binding.ktanh_f32_to_bf16(x3f[k % 2], out=y3h[k % 2])
    for k in range(20):
        binding.kgelu_f32_backward(x3f[1], x3f[0], dx=y3f[k % 2])
    torch.cuda.synchronize()
    del x3, y3, x3f, y3f, y3h

    gates_h, c0_h = wl.lstm_cell_inputs()
    gates, c0 = upload(gates_h), torch.from_numpy(c0_h).to("cuda:0")
    gates_rot = [gates, gates.roll(4099), gates.roll(8209)]
    h_rot = [torch.empty((gates.shape[0], gates.shape[1], gates.shape[2] // 4), dtype=gates.dtype, device=gates.device)
             for _ in range(3)]
    c = torch.empty_like(c0)
    for k in range(21):
        binding.klstm_cell(gates_rot[k % 3], c0, c_out=c, h_out=h_rot[k % 3])
    for t in range(24):
        binding.klstm_cell(gates[t:t + 1], c0, c_out=c, h_out=h_rot[0][t:t + 1])
    for k in range(21):
        probe.ktanh_probe_lstm(gates_rot[k % 3], c0, c, h_rot[k % 3])
    dh = torch.zeros((c0.shape[0], c0.shape[1]), dtype=gates.dtype, device=gates.device)
    dc_next = torch.ones_like(c0)
    for t in range(24):
        binding.klstm_cell_backward(gates[t], c0, dh, dc_next)
    torch.cuda.synchronize()
    print("probe done")


if __name__ == "__main__":
    main()
