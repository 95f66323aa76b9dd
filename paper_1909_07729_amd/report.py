"""Accuracy and throughput of the K-TanH tables on this GPU: the trade-off among table size, accuracy
and throughput that Section 1 of arXiv:1909.07729 describes, measured with the library itself.

    python -m paper_1909_07729_amd.report

For each table (Table 1, the 64-interval fit, the ablation's b_min = 0 fit) every finite BFloat16
input goes through the GPU kernel and the result is compared with TanH in double precision; the
derived Sigmoid, Swish and GELU are compared with their exact forms on |x| <= 16.  Throughput is
taken on a [50, 128, 4096] BFloat16 tensor.  (The ablation's row shows the two error figures that
Table 2 of the paper prints for K-TanH, 1.67e-2 and 3.03 %.)  The rational Pade approximants of
Section 2 and the piecewise Taylor polynomials, which stand for rows of Table 2, are measured the same way.  The reference values are numpy's,
computed here; the library's arithmetic is not repeated on the CPU.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding, workloads as wl


def _values(bits: np.ndarray) -> np.ndarray:
    with np.errstate(invalid="ignore"):  # NaN patterns among the inputs
        return wl.bf16_bits_to_f32(bits).astype(np.float64)


def _on_gpu(fn, bits: np.ndarray, **kw) -> np.ndarray:
    x = torch.from_numpy(bits.view(np.int16)).to("cuda:0")
    return fn(x, **kw).cpu().numpy().view(np.uint16)


def _throughput(fn, **kw) -> float:
    """Elements per second over rotating buffers of the [50, 128, 4096] gate tensor."""
    xs = [torch.from_numpy(wl.lstm_gate_preactivations().view(np.int16)).to("cuda:0")]
    xs += [xs[0].roll(4099 * k) for k in range(1, 8)]
    ys = [torch.empty_like(x) for x in xs]
    for i in range(200):
        fn(xs[i % 8], out=ys[i % 8], **kw)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    steps = 2000
    torch.cuda.synchronize()
    start.record()
    for i in range(steps):
        fn(xs[i % 8], out=ys[i % 8], **kw)
    stop.record()
    torch.cuda.synchronize()
    return xs[0].numel() * steps / (start.elapsed_time(stop) * 1e-3)


def error_rows() -> list[dict]:
    """One row per table: errors of K-TanH against TanH over all finite BFloat16 inputs."""
    bits = wl.all_bf16_patterns()
    bits = bits[(bits & 0x7FFF) < 0x7F80]
    x = _values(bits)
    want = np.tanh(x)
    region = (np.abs(x) >= 0.25) & (np.abs(x) < 4.0)
    tables = [
        ("Table 1 (32 intervals)", binding.ktanh_bf16, {}),
        ("fitted, 64 intervals", binding.ktanh64_bf16, {}),
        ("ablation b_min = 0 (32 intervals)", binding.ktanh_bf16, {"lut": binding.ktanh_fit_lut_bmin0()}),
    ]
    rows = []
    for name, fn, kw in tables:
        err = np.abs(_values(_on_gpu(fn, bits, **kw)) - want)
        worst = int(np.argmax(err))
        nz = want != 0
        rows.append({
            "table": name,
            "max_abs": float(err.max()),
            "at": f"0x{int(bits[worst]):04X}",
            "max_rel": float(np.max(err[nz] / np.abs(want[nz]))),
            "mean_abs_region": float(err[region].mean()),
            "elements_per_s": _throughput(fn, **kw),
        })
    return rows


def comparator_rows() -> list[dict]:
    """The approximants that Table 2 of the paper sets against K-TanH and that this library builds
    (the rational Pade approximants; piecewise Taylor polynomials on K-TanH's intervals for the Taylor
    rows): the same error figures and throughput, measured with this library's kernels."""
    bits = wl.all_bf16_patterns()
    bits = bits[(bits & 0x7FFF) < 0x7F80]
    x = _values(bits)
    want = np.tanh(x)
    nz = want != 0
    rows = []
    for name, fn in (("Pade[3/2]", binding.kpade32_bf16), ("Pade[7/8]", binding.kpade78_bf16),
                     ("Taylor degree 2, 32 intervals", binding.ktaylor2_bf16),
                     ("Taylor degree 3, 32 intervals", binding.ktaylor3_bf16)):
        err = np.abs(_values(_on_gpu(fn, bits)) - want)
        rows.append({"approximant": name, "max_abs": float(err.max()), "at": f"0x{int(bits[int(np.argmax(err))]):04X}",
                     "max_rel": float(np.max(err[nz] / np.abs(want[nz]))), "elements_per_s": _throughput(fn)})
    return rows


def derived_rows() -> list[dict]:
    """Errors of the derived activations against their exact forms on |x| <= 16, 32 and 64 intervals."""
    bits = wl.all_bf16_patterns()
    x_all = _values(bits)
    keep = np.isfinite(x_all) & (np.abs(x_all) <= 16)
    bits, x = bits[keep], x_all[keep]
    sig = 1.0 / (1.0 + np.exp(-x))
    exact = {
        "Sigmoid": sig,
        "Swish": x * sig,
        "GELU (tanh form)": 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3))),
    }
    fns = {"Sigmoid": ("ksigmoid", "ksigmoid64"), "Swish": ("kswish", "kswish64"),
           "GELU (tanh form)": ("kgelu", "kgelu64")}
    rows = []
    for name, want in exact.items():
        row = {"op": name}
        for width, fn_name in zip((32, 64), fns[name]):
            err = np.abs(_values(_on_gpu(getattr(binding, fn_name), bits)) - want)
            row[f"max_abs_{width}"] = float(err.max())
            row[f"mean_abs_{width}"] = float(err.mean())
        rows.append(row)
    return rows


def main() -> None:
    if not torch.cuda.is_available():
        raise SystemExit("report: no GPU visible")
    binding.load_library()
    print("K-TanH against TanH (double), all finite BFloat16 inputs")
    print(f"{'table':36s} {'max abs':>9s} {'at':>7s} {'max rel':>8s} {'mean abs [0.25,4)':>18s} {'Gelem/s':>9s}")
    for r in error_rows():
        print(f"{r['table']:36s} {r['max_abs']:9.5f} {r['at']:>7s} {100 * r['max_rel']:7.2f}% "
              f"{r['mean_abs_region']:18.5f} {r['elements_per_s'] / 1e9:9.1f}")
    print()
    print("Table 2's comparison approximants (Float32 arithmetic, BFloat16 in and out) against TanH (double)")
    print(f"{'approximant':36s} {'max abs':>9s} {'at':>7s} {'max rel':>8s} {'Gelem/s':>9s}")
    for r in comparator_rows():
        print(f"{r['approximant']:36s} {r['max_abs']:9.5f} {r['at']:>7s} {100 * r['max_rel']:7.2f}% "
              f"{r['elements_per_s'] / 1e9:9.1f}")
    print()
    print("Derived activations against their exact forms, |x| <= 16")
    print(f"{'operation':20s} {'max abs (32)':>13s} {'mean abs (32)':>14s} {'max abs (64)':>13s} {'mean abs (64)':>14s}")
    for r in derived_rows():
        print(f"{r['op']:20s} {r['max_abs_32']:13.5f} {r['mean_abs_32']:14.6f} {r['max_abs_64']:13.5f} "
              f"{r['mean_abs_64']:14.6f}")


if __name__ == "__main__":
    main()
