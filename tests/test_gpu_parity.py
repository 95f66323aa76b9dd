"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded
bytes.  Integer paths (ktanh_bf16, ktanh_f32) must match bit for bit.  The derived activations and
the LSTM cell do their Float32 steps in the oracle's order, so they are held to the same bar --
identical bits -- which is tighter than the 1 BFloat16 ulp they are allowed; only a NaN may differ
in sign or payload (compared as a class).
"""
import numpy as np
import pytest

from paper_1909_07729_amd import workloads as wl

pytestmark = pytest.mark.gpu

BF16_OPS = ("ktanh_bf16", "ksigmoid", "kswish", "kgelu")


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1909_07729_amd import binding
    binding.load_library()          # no fallback: a missing library fails the whole module
    torch.cuda.set_device(0)
    return binding, torch


def _to_dev(torch, a):
    view = {np.dtype(np.uint16): np.int16, np.dtype(np.uint32): np.int32}.get(a.dtype, a.dtype)
    return torch.from_numpy(np.ascontiguousarray(a).view(view)).to("cuda:0")


def _to_host(t, dtype):
    return t.cpu().numpy().view(dtype)


def _assert_bf16_equal(got, want, exact_nan, what):
    if exact_nan:
        bad = np.nonzero(got != want)[0]
    else:
        gn, wn = (got & 0x7FFF) > 0x7F80, (want & 0x7FFF) > 0x7F80
        assert np.array_equal(gn, wn), f"{what}: NaN positions differ"
        bad = np.nonzero((got != want) & ~wn)[0]
    assert bad.size == 0, (f"{what}: {bad.size} mismatches, first at {bad[0]}: "
                           f"got {int(got[bad[0]]):04X} want {int(want[bad[0]]):04X}")


def _run_bf16(gpu, oracle, name, x, lut_rows=None):
    binding, torch = gpu
    klut = binding.KtanhLut.from_tuples(lut_rows) if lut_rows else None
    olut = oracle.OracleLut.from_tuples(lut_rows) if lut_rows else None
    got = _to_host(getattr(binding, name)(_to_dev(torch, x), lut=klut), np.uint16)
    want = getattr(oracle, name)(x, olut)
    _assert_bf16_equal(got, want, name == "ktanh_bf16", f"{name} n={x.size}")


# ------------------------------------------------------------------ all 65,536 patterns
@pytest.mark.parametrize("name", BF16_OPS)
def test_exhaustive_bf16_patterns(gpu, oracle, name):
    _run_bf16(gpu, oracle, name, wl.all_bf16_patterns())


def test_exhaustive_bf16_patterns_shuffled_and_custom_lut(gpu, oracle):
    rng = np.random.Generator(np.random.PCG64(11))
    x = rng.permutation(wl.all_bf16_patterns())
    rows = oracle.table1().as_tuples()
    rows[24] = (126, 0, 60); rows[9] = (125, 1, 3); rows[7] = (127, 7, 0); rows[16] = (124, 3, 100)
    for name in BF16_OPS:
        _run_bf16(gpu, oracle, name, x, rows)


def test_f32_structured_patterns(gpu, oracle):
    binding, torch = gpu
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    rng = np.random.Generator(np.random.PCG64(12))
    u = np.concatenate([hi, hi | 0xFFFF, hi | 0x8000, hi | 1,
                        rng.integers(0, 1 << 32, size=(1 << 22) + 3, dtype=np.uint64).astype(np.uint32)])
    got = _to_host(binding.ktanh_f32(_to_dev(torch, u)), np.uint32)
    assert np.array_equal(got, oracle.ktanh_f32(u))


# ------------------------------------------------------------------ ragged sizes, alignment, aliasing
@pytest.mark.parametrize("n", [1, 2, 7, 8, 9, 63, 64, 65, 1023, 8191, 8192, 8193, 8192 * 3 + 5,
                               256 * 4 * 8 * 7 + 8 * 300 + 3])
def test_ragged_sizes(gpu, oracle, n):
    x = wl.lstm_gate_preactivations(n, seed=1000 + n)
    x[:: max(1, n // 7)] = wl.edge_bf16_patterns()[: len(x[:: max(1, n // 7)])]
    for name in BF16_OPS:
        _run_bf16(gpu, oracle, name, x)
    binding, torch = gpu
    u = wl.f32_mixture(n, seed=2000 + n)
    got = _to_host(binding.ktanh_f32(_to_dev(torch, u)), np.uint32)
    assert np.array_equal(got, oracle.ktanh_f32(u))


@pytest.mark.parametrize("in_off,out_off", [(0, 0), (1, 1), (3, 3), (7, 7), (0, 1), (5, 2), (1, 0)])
def test_unaligned_views(gpu, oracle, in_off, out_off):
    """Element offsets into 16-byte aligned buffers: congruent offsets take the vector body with
    peeled ends, different ones the element-wise kernel.  Guard bytes around `out` stay intact."""
    binding, torch = gpu
    n = 8192 * 2 + 11
    x = wl.mlp_preactivations(n + 16, seed=31)
    xd = _to_dev(torch, x)
    for name in BF16_OPS:
        outd = torch.full((n + 32,), 0x5A5A, dtype=torch.int16, device="cuda:0")
        getattr(binding, name)(xd[in_off:in_off + n], out=outd[8 + out_off:8 + out_off + n])
        res = _to_host(outd, np.uint16)
        want = getattr(oracle, name)(x[in_off:in_off + n])
        _assert_bf16_equal(res[8 + out_off:8 + out_off + n], want, name == "ktanh_bf16", name)
        assert np.all(res[:8 + out_off] == 0x5A5A) and np.all(res[8 + out_off + n:] == 0x5A5A)
    u = wl.f32_mixture(n + 8, seed=32)
    ud = _to_dev(torch, u)
    i4, o4 = in_off % 4, out_off % 4
    outd = torch.full((n + 16,), 0x5A5A5A5A, dtype=torch.int32, device="cuda:0")
    binding.ktanh_f32(ud[i4:i4 + n], out=outd[4 + o4:4 + o4 + n])
    res = _to_host(outd, np.uint32)
    assert np.array_equal(res[4 + o4:4 + o4 + n], oracle.ktanh_f32(u[i4:i4 + n]))
    assert np.all(res[:4 + o4] == 0x5A5A5A5A) and np.all(res[4 + o4 + n:] == 0x5A5A5A5A)


def test_in_place_and_empty_and_stream(gpu, oracle):
    binding, torch = gpu
    x = wl.lstm_gate_preactivations(300007, seed=41)
    for name in BF16_OPS:
        xd = _to_dev(torch, x)
        getattr(binding, name)(xd, out=xd)
        _assert_bf16_equal(_to_host(xd, np.uint16), getattr(oracle, name)(x), name == "ktanh_bf16", name)
    empty = torch.empty(0, dtype=torch.bfloat16, device="cuda:0")
    assert binding.ktanh_bf16(empty).numel() == 0
    side = torch.cuda.Stream()
    xd = _to_dev(torch, x)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        yd = binding.ktanh_bf16(xd)
    side.synchronize()
    assert np.array_equal(_to_host(yd, np.uint16), oracle.ktanh_bf16(x))
    # bfloat16-typed tensors go through unchanged
    xb = _to_dev(torch, x).view(torch.bfloat16)
    assert np.array_equal(_to_host(binding.ktanh_bf16(xb).view(torch.int16), np.uint16), oracle.ktanh_bf16(x))


def test_rejected_calls_raise(gpu):
    binding, torch = gpu
    x = torch.zeros(64, dtype=torch.bfloat16, device="cuda:0")
    bad = binding.KtanhLut.from_tuples([(126, 9, 0)] * 32)
    with pytest.raises(binding.KtanhError) as e:
        binding.ktanh_bf16(x, lut=bad)
    assert e.value.status == 3
    g = torch.zeros((1, 2, 4 * 12), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(binding.KtanhError) as e:
        binding.klstm_cell(g, torch.zeros((2, 12), device="cuda:0"))
    assert e.value.status == 4


# ------------------------------------------------------------------ the named workloads, full size
def test_bench_headline_step_matches_oracle_on_every_buffer(gpu, oracle):
    """The step bench.py times, built by bench.py itself: same buffers, same call, every one of the
    rotating outputs against the oracle (element-wise, so the rotated input gives the rotated output)."""
    binding, torch = gpu
    import bench
    headline, x_host = bench.make_headline(torch, binding, wl, bench.make_upload(np, torch, torch.device("cuda:0")))
    for i in range(2 * bench.ROTATE):
        headline(i)
    torch.cuda.synchronize()
    want = oracle.ktanh_bf16(x_host)
    for k in range(bench.ROTATE):
        got = _to_host(headline.outputs[k], np.uint16)
        assert np.array_equal(got, np.roll(want, k * bench.HEADLINE_ROLL)), f"buffer pair {k}"


def test_lstm_gate_preactivations_full(gpu, oracle):
    """[50, 128, 4096] BFloat16 ~ N(0, 1.5^2): the tensor the throughput figure is quoted on."""
    _run_bf16(gpu, oracle, "ktanh_bf16", wl.lstm_gate_preactivations())


def test_f32_mixture_full(gpu, oracle):
    """2^28 Float32: uniform [-8, 8) with 5 % N(0, 0.01^2)."""
    binding, torch = gpu
    u = wl.f32_mixture()
    got = _to_host(binding.ktanh_f32(_to_dev(torch, u)), np.uint32)
    want = oracle.ktanh_f32(u)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, f"{bad.size} mismatches, first {bad[:1]}"


def test_mlp_preactivations_full(gpu, oracle):
    """[8192, 16384] BFloat16 ~ N(0, 1) through Sigmoid, Swish and GELU."""
    x = wl.mlp_preactivations()
    for name in ("ksigmoid", "kswish", "kgelu"):
        _run_bf16(gpu, oracle, name, x)


# ------------------------------------------------------------------ LSTM cell
def _lstm_check(gpu, oracle, gates, c0, per_step):
    binding, torch = gpu
    T = gates.shape[0]
    gd, cd = _to_dev(torch, gates), torch.from_numpy(c0).to("cuda:0")
    if per_step:
        hs = []
        for t in range(T):
            cd, h = binding.klstm_cell(gd[t:t + 1], cd, c_out=cd)      # state updated in place
            hs.append(h)
        hd = torch.cat(hs, dim=0)
    else:
        cd, hd = binding.klstm_cell(gd, cd)
    c_ref, h_ref = oracle.klstm_cell(gates, c0)
    c_got, h_got = cd.cpu().numpy(), _to_host(hd, np.uint16)
    cn = np.isnan(c_ref)
    assert np.array_equal(np.isnan(c_got), cn)
    assert np.array_equal(c_got.view(np.uint32)[~cn], c_ref.view(np.uint32)[~cn])
    _assert_bf16_equal(h_got.ravel(), h_ref.ravel(), False, "h_out")


# T below, at and above the depth of the gate prefetch ring and twice that depth (the kernel switches
# from its start-up path to the steady loop there), with lane counts that leave ragged last blocks.
@pytest.mark.parametrize("T,B,H", [(1, 1, 8), (3, 5, 24), (4, 7, 2048 + 8), (2, 300, 64), (5, 3, 40),
                                   (7, 2, 264), (8, 3, 72), (9, 5, 24), (11, 2, 520), (12, 1, 8),
                                   (13, 3, 136), (16, 2, 72), (23, 2, 200)])
def test_lstm_cell_small(gpu, oracle, T, B, H):
    gates, c0 = wl.lstm_cell_inputs(T, B, H)
    _lstm_check(gpu, oracle, gates, c0, per_step=False)
    _lstm_check(gpu, oracle, gates, c0, per_step=True)


def test_lstm_cell_special_values(gpu, oracle):
    T, B, H = 2, 2, 16
    gates, c0 = wl.lstm_cell_inputs(T, B, H)
    edge = wl.edge_bf16_patterns()
    gates.reshape(-1)[: edge.size] = edge
    c0.reshape(-1)[:6] = [np.inf, -np.inf, np.nan, 0.0, -0.0, 1e-40]
    _lstm_check(gpu, oracle, gates, c0, per_step=False)


def test_lstm_cell_special_values_late_in_a_long_sequence(gpu, oracle):
    """NaN and infinite gates first appear at steps inside the steady loop and inside the last steps;
    every earlier step must be unaffected and every later one must carry the poisoned state."""
    T, B, H = 19, 3, 72
    gates, c0 = wl.lstm_cell_inputs(T, B, H)
    edge = wl.edge_bf16_patterns()
    for t, b in ((2, 0), (6, 1), (9, 2), (13, 0), (17, 1), (18, 2)):
        row = gates[t, b]
        row[(7 * t) % 40: (7 * t) % 40 + edge.size] = edge[: row.size - (7 * t) % 40]
    c0.reshape(-1)[:4] = [np.inf, -np.inf, np.nan, 3.0e38]
    _lstm_check(gpu, oracle, gates, c0, per_step=False)
    _lstm_check(gpu, oracle, gates, c0, per_step=True)


def test_lstm_cell_full(gpu, oracle):
    """gates [64, 256, 4 x 2048] ~ N(0, 2^2), c0 [256, 2048] ~ N(0, 1): one call over all 64 steps
    and 64 calls of one step, both against the oracle."""
    gates, c0 = wl.lstm_cell_inputs()
    _lstm_check(gpu, oracle, gates, c0, per_step=False)
    _lstm_check(gpu, oracle, gates, c0, per_step=True)


def test_lstm_cell_just_below_the_size_limit(gpu, oracle):
    """B * H / 2 = 2^28 - 16384 cell pairs: the byte offsets inside one time step come within 256 KiB of
    2^32.  Inputs are drawn on the GPU; the first, middle and last batch rows go through the oracle."""
    binding, torch = gpu
    T, B, H = 2, 16383, 32768
    assert B * H // 2 < (1 << 28) <= (B + 1) * H // 2
    gen = torch.Generator(device="cuda:0").manual_seed(190908)
    gates = torch.empty((T, B, 4 * H), dtype=torch.bfloat16, device="cuda:0")
    for t in range(T):
        for b0 in range(0, B, 2048):                      # in slabs: the Float32 draw is twice the size
            rows = min(2048, B - b0)
            gates[t, b0:b0 + rows] = (torch.randn((rows, 4 * H), generator=gen, device="cuda:0") * 2).to(torch.bfloat16)
    c0 = torch.randn((B, H), generator=gen, device="cuda:0")
    c1, h = binding.klstm_cell(gates, c0)
    rows = [0, 1, B // 2, B - 2, B - 1]
    g_host = gates[:, rows, :].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    c_ref, h_ref = oracle.klstm_cell(g_host, c0[rows].cpu().numpy())
    assert np.array_equal(c1[rows].cpu().numpy().view(np.uint32), c_ref.view(np.uint32))
    assert np.array_equal(h[:, rows, :].contiguous().view(torch.int16).cpu().numpy().view(np.uint16), h_ref)
    del gates, h
    with pytest.raises(binding.KtanhError):               # one more row crosses the limit
        binding.klstm_cell(torch.empty((1, B + 1, 4 * H), dtype=torch.bfloat16, device="cuda:0"),
                           torch.empty((B + 1, H), device="cuda:0"))


def test_calls_captured_in_a_hip_graph_replay_correctly(gpu, oracle):
    """Every entry point only enqueues kernels, so a stream capture records them; each replay is
    checked against the oracle, with eager work and synchronisation between the replays."""
    binding, torch = gpu
    x = wl.lstm_gate_preactivations(200000, seed=77)
    gates, c0 = wl.lstm_cell_inputs(6, 8, 64)
    xd, gd = _to_dev(torch, x), _to_dev(torch, gates)
    cd = torch.from_numpy(c0).to("cuda:0")
    yd, sd = torch.empty_like(xd), torch.empty_like(xd)
    hd = torch.empty((6, 8, 64), dtype=torch.int16, device="cuda:0")
    cw = torch.empty_like(cd)
    binding.ktanh_bf16(xd, out=yd)                       # warm up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.ktanh_bf16(xd, out=yd)
        binding.kgelu(xd, out=sd)
        cw.copy_(cd)
        for t in range(6):
            binding.klstm_cell(gd[t:t + 1], cw, c_out=cw, h_out=hd[t:t + 1])
    want_y, want_s = oracle.ktanh_bf16(x), oracle.kgelu(x)
    want_c, want_h = oracle.klstm_cell(gates, c0)
    for replay in range(3):
        yd.fill_(0); sd.fill_(0); hd.fill_(0); cw.fill_(0)          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(_to_host(yd, np.uint16), want_y), f"replay {replay}"
        _assert_bf16_equal(_to_host(sd, np.uint16), want_s, False, f"kgelu replay {replay}")
        assert np.array_equal(cw.cpu().numpy(), want_c), f"replay {replay}"
        assert np.array_equal(_to_host(hd, np.uint16), want_h), f"replay {replay}"


def test_probe_yardsticks(gpu):
    """The measurement library: ktanh_probe_copy moves bits unchanged (NaN payloads included) for any
    alignment and in place; ktanh_probe_write fills exactly its range; ktanh_probe_read writes nothing;
    ktanh_probe_lstm writes the XOR of the words it loads."""
    binding, torch = gpu
    from paper_1909_07729_amd import probe
    x = np.concatenate([wl.all_bf16_patterns(), wl.lstm_gate_preactivations(100003, seed=73)])
    xd = _to_dev(torch, x)
    assert np.array_equal(_to_host(probe.ktanh_probe_copy(xd, torch.empty_like(xd)), np.uint16), x)
    n = x.size - 16
    for off_in, off_out in ((0, 0), (1, 1), (3, 0), (0, 5), (7, 2)):
        outd = torch.full((x.size + 16,), 0x5A5A, dtype=torch.int16, device="cuda:0")
        probe.ktanh_probe_copy(xd[off_in:off_in + n], outd[8 + off_out:8 + off_out + n])
        res = _to_host(outd, np.uint16)
        assert np.array_equal(res[8 + off_out:8 + off_out + n], x[off_in:off_in + n]), (off_in, off_out)
        assert np.all(res[:8 + off_out] == 0x5A5A) and np.all(res[8 + off_out + n:] == 0x5A5A)
    probe.ktanh_probe_copy(xd, xd)
    assert np.array_equal(_to_host(xd, np.uint16), x)
    # write: 1 KiB-aligned start inside a guarded buffer, a length that ends inside a tile
    buf = torch.full((4096 + 40000,), 0x5A5A, dtype=torch.int16, device="cuda:0")
    start = (-buf.data_ptr() % 1024) // 2 + 512
    probe.ktanh_probe_write(buf[start:start + 30008])
    res = _to_host(buf, np.uint16)
    assert np.all(res[start:start + 30008] == 0x3F80) and np.all(res[:start] == 0x5A5A) and np.all(res[start + 30008:] == 0x5A5A)
    sink = torch.full((512,), 0x5A5A, dtype=torch.int16, device="cuda:0")
    probe.ktanh_probe_read(buf[start:start + 30008], sink)
    torch.cuda.synchronize()
    assert np.all(_to_host(sink, np.uint16) == 0x5A5A) and np.array_equal(_to_host(buf, np.uint16), res)
    # the 512-thread forms: a length that ends inside a block of eight tiles
    buf.fill_(0x5A5A)
    probe.ktanh_probe_write(buf[start:start + 30008], wide=True)
    res = _to_host(buf, np.uint16)
    assert np.all(res[start:start + 30008] == 0x3F80) and np.all(res[:start] == 0x5A5A) and np.all(res[start + 30008:] == 0x5A5A)
    probe.ktanh_probe_read(buf[start:start + 30008], sink, wide=True)
    torch.cuda.synchronize()
    assert np.all(_to_host(sink, np.uint16) == 0x5A5A) and np.array_equal(_to_host(buf, np.uint16), res)
    # the LSTM kernel's launch without its arithmetic: output word = XOR of the step's four gate words and
    # the bits of the lane's first state value; the state passes through (ragged last block, short and long T)
    for T, B, H in ((1, 3, 8), (5, 3, 40), (8, 2, 1032), (19, 5, 264)):
        rng = np.random.Generator(np.random.PCG64(T * 1000 + H))
        g = rng.integers(0, 1 << 16, size=(T, B, 4 * H), dtype=np.uint16)
        c = rng.standard_normal((B, H), dtype=np.float32)
        gd, cd = _to_dev(torch, g), torch.from_numpy(c).to("cuda:0")
        c_out = torch.zeros_like(cd)
        hd = torch.full((T, B, H), 0x5A5A, dtype=torch.int16, device="cuda:0")
        probe.ktanh_probe_lstm(gd, cd, c_out, hd)
        words = g.reshape(T, B, 4, H // 2, 2).astype(np.uint32)
        words = words[..., 0] | (words[..., 1] << 16)                       # [T, B, 4, H/2]
        want = words[:, :, 0] ^ words[:, :, 1] ^ words[:, :, 2] ^ words[:, :, 3] ^ c.view(np.uint32)[None, :, 0::2]
        got = _to_host(hd, np.uint16).reshape(T, B, H // 2, 2).astype(np.uint32)
        assert np.array_equal(got[..., 0] | (got[..., 1] << 16), want), (T, B, H)
        assert np.array_equal(c_out.cpu().numpy().view(np.uint32), c.view(np.uint32))


def test_graph_replay_of_the_later_entry_points(gpu, oracle):
    """64-interval, Float32-tensor, fused-conversion and gradient calls (aligned and unaligned
    inputs) recorded into one HIP graph and replayed three times with eager work in between."""
    binding, torch = gpu
    x = wl.mlp_preactivations(40009, seed=70)
    dy = wl.f32_to_bf16_bits(np.random.Generator(np.random.PCG64(71)).standard_normal(x.size, dtype=np.float32))
    xf = wl.f32_mixture(40009, seed=72).view(np.float32)
    xd, dyd = _to_dev(torch, x), _to_dev(torch, dy)
    xfd = torch.from_numpy(xf).to("cuda:0")
    n = x.size - 5
    outs = {k: torch.empty_like(xd) for k in ("t64", "gb", "gb_unaligned")}
    outs["sf"] = torch.empty_like(xfd)
    outs["nb"] = torch.empty(xf.size, dtype=torch.int16, device="cuda:0")
    outs["gf"] = torch.empty_like(xfd)
    binding.ktanh64_bf16(xd, out=outs["t64"])                         # warm up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.ktanh64_bf16(xd, out=outs["t64"])
        binding.kgelu_backward(dyd, xd, dx=outs["gb"])
        binding.kgelu_backward(dyd[3:3 + n], xd[2:2 + n], dx=outs["gb_unaligned"][:n])
        binding.kswish64_f32(xfd, out=outs["sf"])
        binding.ktanh_f32_to_bf16(xfd, out=outs["nb"])
        binding.kswish_f32_backward(xfd, xfd, dx=outs["gf"])
    with np.errstate(all="ignore"):
        want = {"t64": oracle.ktanh64_bf16(x), "gb": oracle.kgelu_backward(dy, x),
                "gb_unaligned": oracle.kgelu_backward(dy[3:3 + n], x[2:2 + n]),
                "sf": oracle.kswish64_f32(xf), "nb": oracle.ktanh_f32_to_bf16(xf),
                "gf": oracle.kswish_f32_backward(xf, xf)}
    for replay in range(3):
        for t in outs.values():
            t.zero_()                                                 # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(_to_host(outs["t64"], np.uint16), want["t64"]), f"replay {replay}"
        _assert_bf16_equal(_to_host(outs["gb"], np.uint16), want["gb"], False, f"kgelu_backward replay {replay}")
        _assert_bf16_equal(_to_host(outs["gb_unaligned"], np.uint16)[:n], want["gb_unaligned"], False, f"unaligned replay {replay}")
        _assert_f32_equal(outs["sf"].cpu().numpy(), want["sf"], f"kswish64_f32 replay {replay}")
        _assert_bf16_equal(_to_host(outs["nb"], np.uint16), want["nb"], False, f"ktanh_f32_to_bf16 replay {replay}")
        _assert_f32_equal(outs["gf"].cpu().numpy(), want["gf"], f"kswish_f32_backward replay {replay}")


# ------------------------------------------------------------------ 64-interval variant
def test_ktanh64_exhaustive_ragged_and_custom_table(gpu, oracle):
    binding, torch = gpu
    x = np.concatenate([wl.all_bf16_patterns(), wl.lstm_gate_preactivations(100003, seed=64)])
    got = _to_host(binding.ktanh64_bf16(_to_dev(torch, x)), np.uint16)
    assert np.array_equal(got, oracle.ktanh64_bf16(x))
    rows = oracle.fit_lut64().as_tuples()
    rows[48] = (126, 0, 60); rows[17] = (125, 1, 4); rows[15] = (127, 7, 0); rows[32] = (124, 3, 100)
    got = _to_host(binding.ktanh64_bf16(_to_dev(torch, x), lut=binding.KtanhLut64.from_tuples(rows)), np.uint16)
    assert np.array_equal(got, oracle.ktanh64_bf16(x, oracle.OracleLut64.from_tuples(rows)))
    xd = _to_dev(torch, x)
    outd = torch.full((x.size + 16,), 0x5A5A, dtype=torch.int16, device="cuda:0")
    binding.ktanh64_bf16(xd[3:], out=outd[5:5 + x.size - 3])          # element-wise fallback path
    res = _to_host(outd, np.uint16)
    assert np.array_equal(res[5:5 + x.size - 3], oracle.ktanh64_bf16(x[3:]))
    assert np.all(res[:5] == 0x5A5A) and np.all(res[5 + x.size - 3:] == 0x5A5A)
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    u = np.concatenate([hi, hi | 0xFFFF, hi | 0x8000, wl.f32_mixture((1 << 20) + 5, seed=65)])
    got = _to_host(binding.ktanh64_f32(_to_dev(torch, u)), np.uint32)
    assert np.array_equal(got, oracle.ktanh64_f32(u))


def test_ktanh64_full_size(gpu, oracle):
    binding, torch = gpu
    x = wl.lstm_gate_preactivations()
    got = _to_host(binding.ktanh64_bf16(_to_dev(torch, x)), np.uint16)
    assert np.array_equal(got, oracle.ktanh64_bf16(x))
    u = wl.f32_mixture(1 << 26)
    got = _to_host(binding.ktanh64_f32(_to_dev(torch, u)), np.uint32)
    assert np.array_equal(got, oracle.ktanh64_f32(u))


# ------------------------------------------------------------------ Float32 tensors
def _assert_f32_equal(got, want, what):
    gn, wn = np.isnan(got), np.isnan(want)
    assert np.array_equal(gn, wn), f"{what}: NaN positions differ"
    bad = np.nonzero((got.view(np.uint32) != want.view(np.uint32)) & ~wn)[0]
    assert bad.size == 0, (f"{what}: {bad.size} mismatches, first at {bad[0]}: "
                           f"got {got.view(np.uint32)[bad[0]]:08X} want {want.view(np.uint32)[bad[0]]:08X}")


def _f32_cases():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    rng = np.random.Generator(np.random.PCG64(14))
    return np.concatenate([hi, hi | 0xFFFF, hi | 0x8000, hi | 0x7FFF, hi | 0x8001,
                           rng.integers(0, 1 << 32, size=(1 << 21) + 7, dtype=np.uint64).astype(np.uint32),
                           wl.f32_mixture((1 << 21) + 3, seed=15)])


@pytest.mark.parametrize("name", ["ksigmoid_f32", "kswish_f32", "kgelu_f32"])
def test_f32_derived_ops(gpu, oracle, name):
    """Same Float32 operations in the same order on both sides: identical bits (the budget is 1e-6
    relative), NaN by position."""
    binding, torch = gpu
    u = _f32_cases()
    xf = u.view(np.float32)
    with np.errstate(all="ignore"):
        want = getattr(oracle, name)(xf)
    got = getattr(binding, name)(torch.from_numpy(xf).to("cuda:0")).cpu().numpy()
    _assert_f32_equal(got, want, name)
    # ragged, unaligned, in place
    n = 8192 * 3 + 5
    xd = torch.from_numpy(xf[: n + 8].copy()).to("cuda:0")
    for off_in, off_out in ((0, 0), (1, 1), (3, 2)):
        outd = torch.full((n + 16,), 7.0, dtype=torch.float32, device="cuda:0")
        getattr(binding, name)(xd[off_in:off_in + n], out=outd[4 + off_out:4 + off_out + n])
        res = outd.cpu().numpy()
        with np.errstate(all="ignore"):
            _assert_f32_equal(res[4 + off_out:4 + off_out + n], getattr(oracle, name)(xf[off_in:off_in + n]), name)
        assert np.all(res[:4 + off_out] == 7.0) and np.all(res[4 + off_out + n:] == 7.0)
    getattr(binding, name)(xd, out=xd)
    with np.errstate(all="ignore"):
        _assert_f32_equal(xd.cpu().numpy(), getattr(oracle, name)(xf[: n + 8]), name + " in place")


def test_f32_derived_ops_on_64_interval_tables(gpu, oracle):
    """ksigmoid64_f32, kswish64_f32, kgelu64_f32 on the fitted table and on random valid tables."""
    binding, torch = gpu
    xf = _f32_cases().view(np.float32)
    xd = torch.from_numpy(xf).to("cuda:0")
    rng = np.random.Generator(np.random.PCG64(66))
    for rows in (None, _random_valid_table(rng, 64), _random_valid_table(rng, 64)):
        k64 = binding.KtanhLut64.from_tuples(rows) if rows else None
        o64 = oracle.OracleLut64.from_tuples(rows) if rows else None
        for name in ("ksigmoid64_f32", "kswish64_f32", "kgelu64_f32"):
            with np.errstate(all="ignore"):
                want = getattr(oracle, name)(xf, o64)
            _assert_f32_equal(getattr(binding, name)(xd, lut=k64).cpu().numpy(), want, name)


def test_f32_to_bf16(gpu, oracle):
    binding, torch = gpu
    u = _f32_cases()
    xf = u.view(np.float32)
    got = _to_host(binding.ktanh_f32_to_bf16(torch.from_numpy(xf).to("cuda:0")).view(torch.int16), np.uint16)
    _assert_bf16_equal(got, oracle.ktanh_f32_to_bf16(xf), False, "ktanh_f32_to_bf16")
    n = 8192 * 3 + 5
    xd = torch.from_numpy(xf[: n + 8].copy()).to("cuda:0")
    for off_in, off_out in ((0, 0), (1, 1), (3, 3), (0, 1), (2, 0), (1, 3), (0, 4)):
        outd = torch.full((n + 24,), 0x5A5A, dtype=torch.int16, device="cuda:0")
        binding.ktanh_f32_to_bf16(xd[off_in:off_in + n], out=outd[8 + off_out:8 + off_out + n])
        res = _to_host(outd, np.uint16)
        _assert_bf16_equal(res[8 + off_out:8 + off_out + n], oracle.ktanh_f32_to_bf16(xf[off_in:off_in + n]),
                           False, f"offsets {off_in},{off_out}")
        assert np.all(res[:8 + off_out] == 0x5A5A) and np.all(res[8 + off_out + n:] == 0x5A5A)
    for n_small in (1, 3, 4, 5, 7, 8, 9, 511, 513):
        got = _to_host(binding.ktanh_f32_to_bf16(xd[:n_small]).view(torch.int16), np.uint16)
        _assert_bf16_equal(got, oracle.ktanh_f32_to_bf16(xf[:n_small]), False, f"n={n_small}")


def test_f32_tensor_ops_full_size(gpu, oracle):
    binding, torch = gpu
    xf = wl.f32_mixture(1 << 26).view(np.float32)
    xd = torch.from_numpy(xf).to("cuda:0")
    for name in ("ksigmoid_f32", "kswish_f32", "kgelu_f32"):
        _assert_f32_equal(getattr(binding, name)(xd).cpu().numpy(), getattr(oracle, name)(xf), name)
    got = _to_host(binding.ktanh_f32_to_bf16(xd).view(torch.int16), np.uint16)
    _assert_bf16_equal(got, oracle.ktanh_f32_to_bf16(xf), False, "ktanh_f32_to_bf16")


# ------------------------------------------------------------------ sizes beyond 32-bit offsets
def test_more_than_2_to_the_32_elements(gpu, oracle):
    """8.6 GB tensors: element indices and byte offsets no longer fit 32 bits.  The input repeats the
    65,536 BFloat16 patterns, so the expected output is the oracle's 65,536 answers repeated; the
    comparison itself runs on the GPU (torch is only the ruler here)."""
    binding, torch = gpu
    base = wl.all_bf16_patterns()
    n = (1 << 32) + 8 * 5 + 3
    reps = n // base.size + 1
    xd = _to_dev(torch, base).repeat(reps)[:n]
    want = _to_dev(torch, oracle.ktanh_bf16(base)).repeat(reps)[:n]
    got = binding.ktanh_bf16(xd)
    assert got.numel() == n and torch.equal(got, want)
    got = binding.ktanh_bf16(xd[1:])                     # peeled head, body beyond 4 GiB, ragged tail
    assert torch.equal(got, want[1:])
    del got, want
    # Float32: the same patterns in the upper half of each word, 2^31 + 7 elements (8.6 GB)
    n32 = (1 << 31) + 7
    ud = (xd[:n32].to(torch.int32) << 16)
    want32 = _to_dev(torch, oracle.ktanh_f32(base.astype(np.uint32) << 16)).repeat(n32 // base.size + 1)[:n32]
    got32 = binding.ktanh_f32(ud)
    assert torch.equal(got32, want32)


def test_concurrent_host_threads_on_their_own_streams(gpu, oracle):
    """The entry points keep no mutable state: four host threads, each with its own stream, tables
    and tensors, interleave their calls freely."""
    import threading
    binding, torch = gpu
    x = wl.mlp_preactivations(1 << 20, seed=91)
    rows = oracle.table1().as_tuples()
    results, errors = {}, []

    def worker(k):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            my_rows = list(rows)
            my_rows[24] = (126, 0, 60 + k)              # a different table per thread
            klut, olut = binding.KtanhLut.from_tuples(my_rows), oracle.OracleLut.from_tuples(my_rows)
            with torch.cuda.stream(stream):
                xd = _to_dev(torch, x)
                outs = [binding.kgelu(binding.ktanh_bf16(xd, lut=klut, stream=stream), lut=klut, stream=stream)
                        for _ in range(20)]
            stream.synchronize()
            want = oracle.kgelu(oracle.ktanh_bf16(x, olut), olut)
            results[k] = all(np.array_equal(_to_host(o, np.uint16), want) for o in outs)
        except Exception as exc:                          # surfaced below, in the main thread
            errors.append(repr(exc))

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert results == {0: True, 1: True, 2: True, 3: True}


# ------------------------------------------------------------------ arbitrary valid tables
def _random_valid_table(rng, intervals):
    """Any (E, r, b) the validator accepts: E in 1..254, r in 0..7, b such that (M >> r) + b stays in
    0..127 over the interval -- including the extremes on purpose."""
    per = 512 // intervals                           # 16 or 8 mantissas per interval
    rows = []
    for t in range(intervals):
        j = t % (128 // per)
        E = int(rng.choice([1, 2, 60, 124, 125, 126, 127, 128, 200, 254, int(rng.integers(1, 255))]))
        r = int(rng.integers(0, 8))
        lo, hi = -((j * per) >> r), 127 - ((j * per + per - 1) >> r)
        b = int(rng.choice([lo, hi, int(rng.integers(lo, hi + 1))]))
        rows.append((E, r, b))
    return rows


def test_ablation_table_on_the_gpu(gpu, oracle):
    """The b_min = 0 table of the ablation study, fitted by the library, fed to the kernels."""
    binding, torch = gpu
    klut, olut = binding.ktanh_fit_lut_bmin0(), oracle.fit_lut_bmin0()
    x = np.concatenate([wl.all_bf16_patterns(), wl.lstm_gate_preactivations(100003, seed=62)])
    for name in BF16_OPS:
        got = _to_host(getattr(binding, name)(_to_dev(torch, x), lut=klut), np.uint16)
        _assert_bf16_equal(got, getattr(oracle, name)(x, olut), name == "ktanh_bf16", name + " ablation table")


def test_random_valid_tables(gpu, oracle):
    """The packed slots (folded input exponent, saturation slot, Float32 base) must reproduce
    Algorithm 1 for every table the validator lets through, not just for Table 1."""
    binding, torch = gpu
    rng = np.random.Generator(np.random.PCG64(2024))
    x = np.concatenate([wl.all_bf16_patterns(), wl.lstm_gate_preactivations(20011, seed=5)])
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    u = np.concatenate([hi, hi | 0xFFFF, hi | rng.integers(0, 1 << 16, size=1 << 16, dtype=np.uint32)])
    xd, ud = _to_dev(torch, x), _to_dev(torch, u)
    gates, c0 = wl.lstm_cell_inputs(6, 3, 64)
    gd, cd = _to_dev(torch, gates), torch.from_numpy(c0).to("cuda:0")
    for trial in range(12):
        rows = _random_valid_table(rng, 32)
        klut, olut = binding.KtanhLut.from_tuples(rows), oracle.OracleLut.from_tuples(rows)
        assert binding.ktanh_lut_validate(klut) == 0, rows
        for name in BF16_OPS:
            got = _to_host(getattr(binding, name)(xd, lut=klut), np.uint16)
            with np.errstate(all="ignore"):
                want = getattr(oracle, name)(x, olut)
            _assert_bf16_equal(got, want, name == "ktanh_bf16", f"{name} trial {trial}")
        assert np.array_equal(_to_host(binding.ktanh_f32(ud, lut=klut), np.uint32), oracle.ktanh_f32(u, olut))
        c_got, h_got = binding.klstm_cell(gd, cd, lut=klut)
        with np.errstate(all="ignore"):
            c_ref, h_ref = oracle.klstm_cell(gates, c0, olut)
        cn = np.isnan(c_ref)
        assert np.array_equal(np.isnan(c_got.cpu().numpy()), cn), f"lstm trial {trial}"
        assert np.array_equal(c_got.cpu().numpy().view(np.uint32)[~cn], c_ref.view(np.uint32)[~cn])
        _assert_bf16_equal(_to_host(h_got, np.uint16).ravel(), h_ref.ravel(), False, f"lstm h trial {trial}")
        rows64 = _random_valid_table(rng, 64)
        k64, o64 = binding.KtanhLut64.from_tuples(rows64), oracle.OracleLut64.from_tuples(rows64)
        assert binding.ktanh_lut64_validate(k64) == 0, rows64
        assert np.array_equal(_to_host(binding.ktanh64_bf16(xd, lut=k64), np.uint16), oracle.ktanh64_bf16(x, o64))
        assert np.array_equal(_to_host(binding.ktanh64_f32(ud, lut=k64), np.uint32), oracle.ktanh64_f32(u, o64))


def test_derived_ops_and_lstm_on_64_interval_tables(gpu, oracle):
    binding, torch = gpu
    rng = np.random.Generator(np.random.PCG64(640))
    x = np.concatenate([wl.all_bf16_patterns(), wl.mlp_preactivations(300007, seed=66)])
    xd = _to_dev(torch, x)
    gates, c0 = wl.lstm_cell_inputs(5, 7, 72)
    edge = wl.edge_bf16_patterns()
    gates.reshape(-1)[: edge.size] = edge
    gd, cd = _to_dev(torch, gates), torch.from_numpy(c0).to("cuda:0")
    tables = [None, _random_valid_table(rng, 64), _random_valid_table(rng, 64)]
    for rows in tables:
        k64 = None if rows is None else binding.KtanhLut64.from_tuples(rows)
        o64 = None if rows is None else oracle.OracleLut64.from_tuples(rows)
        for name in ("ksigmoid64", "kswish64", "kgelu64"):
            got = _to_host(getattr(binding, name)(xd, lut=k64), np.uint16)
            with np.errstate(all="ignore"):
                want = getattr(oracle, name)(x, o64)
            _assert_bf16_equal(got, want, False, name)
        c_got, h_got = binding.klstm_cell64(gd, cd, lut=k64)
        with np.errstate(all="ignore"):
            c_ref, h_ref = oracle.klstm_cell64(gates, c0, o64)
        cn = np.isnan(c_ref)
        assert np.array_equal(np.isnan(c_got.cpu().numpy()), cn)
        assert np.array_equal(c_got.cpu().numpy().view(np.uint32)[~cn], c_ref.view(np.uint32)[~cn])
        _assert_bf16_equal(_to_host(h_got, np.uint16).ravel(), h_ref.ravel(), False, "klstm_cell64 h")


# ------------------------------------------------------------------ gradients
def test_backward_of_ktanh_and_ksigmoid(gpu, oracle):
    binding, torch = gpu
    rng = np.random.Generator(np.random.PCG64(51))
    base = wl.all_bf16_patterns()
    fwd = np.concatenate([base, base, wl.mlp_preactivations(100003, seed=52)])
    dy = np.concatenate([rng.permutation(base), wl.f32_to_bf16_bits(rng.standard_normal(base.size + 100003, dtype=np.float32))])
    for name in ("ktanh_bf16_backward", "ksigmoid_backward"):
        with np.errstate(all="ignore"):
            want = getattr(oracle, name.replace("_bf16", ""))(dy, fwd)
        got = _to_host(getattr(binding, name)(_to_dev(torch, dy), _to_dev(torch, fwd)), np.uint16)
        _assert_bf16_equal(got, want, False, name)
        # ragged length, unaligned views (element-wise kernel), result written over dy
        n = 8192 + 13
        dyd, fd = _to_dev(torch, dy), _to_dev(torch, fwd)
        for off in (0, 1, 5):
            outd = torch.full((n + 16,), 0x5A5A, dtype=torch.int16, device="cuda:0")
            getattr(binding, name)(dyd[off:off + n], fd[off:off + n], dx=outd[8:8 + n])
            res = _to_host(outd, np.uint16)
            _assert_bf16_equal(res[8:8 + n], want[off:off + n], False, f"{name} offset {off}")
            assert np.all(res[:8] == 0x5A5A) and np.all(res[8 + n:] == 0x5A5A)
        getattr(binding, name)(dyd, fd, dx=dyd)
        _assert_bf16_equal(_to_host(dyd, np.uint16), want, False, name + " in place")


def test_backward_of_kswish_and_kgelu(gpu, oracle):
    """Gradients from the forward input: every BFloat16 pattern as x (twice, against shuffled and
    random upstream gradients), ragged and unaligned views, in place over dy and over x, and a
    caller's table."""
    binding, torch = gpu
    rng = np.random.Generator(np.random.PCG64(59))
    base = wl.all_bf16_patterns()
    x = np.concatenate([base, base, wl.mlp_preactivations(100003, seed=60)])
    dy = np.concatenate([rng.permutation(base), wl.f32_to_bf16_bits(rng.standard_normal(base.size + 100003, dtype=np.float32))])
    rows = _random_valid_table(np.random.Generator(np.random.PCG64(61)), 32)
    for name in ("kswish_backward", "kgelu_backward"):
        with np.errstate(all="ignore"):
            want = getattr(oracle, name)(dy, x)
            want_custom = getattr(oracle, name)(dy, x, oracle.OracleLut.from_tuples(rows))
        dyd, xd = _to_dev(torch, dy), _to_dev(torch, x)
        _assert_bf16_equal(_to_host(getattr(binding, name)(dyd, xd), np.uint16), want, False, name)
        got = getattr(binding, name)(dyd, xd, lut=binding.KtanhLut.from_tuples(rows))
        _assert_bf16_equal(_to_host(got, np.uint16), want_custom, False, name + " custom table")
        n = 8192 + 13
        for off in (0, 1, 5):
            outd = torch.full((n + 16,), 0x5A5A, dtype=torch.int16, device="cuda:0")
            getattr(binding, name)(dyd[off:off + n], xd[off:off + n], dx=outd[8:8 + n])
            res = _to_host(outd, np.uint16)
            _assert_bf16_equal(res[8:8 + n], want[off:off + n], False, f"{name} offset {off}")
            assert np.all(res[:8] == 0x5A5A) and np.all(res[8 + n:] == 0x5A5A)
        for n_small in (1, 7, 8, 9, 511, 512, 513):
            got = getattr(binding, name)(dyd[:n_small].clone(), xd[:n_small].clone())
            _assert_bf16_equal(_to_host(got, np.uint16), want[:n_small], False, f"{name} n={n_small}")
        over_dy, over_x = dyd.clone(), xd.clone()
        getattr(binding, name)(over_dy, xd, dx=over_dy)
        _assert_bf16_equal(_to_host(over_dy, np.uint16), want, False, name + " over dy")
        getattr(binding, name)(dyd, over_x, dx=over_x)
        _assert_bf16_equal(_to_host(over_x, np.uint16), want, False, name + " over x")


def test_backward_on_float32_tensors(gpu, oracle):
    """The four Float32 gradients: structured and random bit patterns as the second input, random
    upstream gradients, ragged and unaligned views, in place, and a caller's table."""
    binding, torch = gpu
    rng = np.random.Generator(np.random.PCG64(67))
    vf = _f32_cases().view(np.float32)
    dy = rng.standard_normal(vf.size, dtype=np.float32)
    dy[: 1 << 16] = vf[rng.permutation(1 << 16)]          # non-finite upstream values too
    vd, dyd = torch.from_numpy(vf).to("cuda:0"), torch.from_numpy(dy).to("cuda:0")
    rows = _random_valid_table(np.random.Generator(np.random.PCG64(68)), 32)
    for name in ("ktanh_f32_backward", "ksigmoid_f32_backward", "kswish_f32_backward", "kgelu_f32_backward"):
        with np.errstate(all="ignore"):
            want = getattr(oracle, name)(dy, vf)
        _assert_f32_equal(getattr(binding, name)(dyd, vd).cpu().numpy(), want, name)
        if name in ("kswish_f32_backward", "kgelu_f32_backward"):
            with np.errstate(all="ignore"):
                want_custom = getattr(oracle, name)(dy, vf, oracle.OracleLut.from_tuples(rows))
            got = getattr(binding, name)(dyd, vd, lut=binding.KtanhLut.from_tuples(rows))
            _assert_f32_equal(got.cpu().numpy(), want_custom, name + " custom table")
        n = 4096 * 3 + 3
        for off_dy, off_v, off_out in ((0, 0, 0), (1, 1, 1), (0, 1, 2), (3, 0, 0)):
            outd = torch.full((n + 16,), 7.0, dtype=torch.float32, device="cuda:0")
            shifted = torch.empty(n + 8, dtype=torch.float32, device="cuda:0")
            shifted[off_dy:off_dy + n] = dyd[off_v:off_v + n]
            getattr(binding, name)(shifted[off_dy:off_dy + n], vd[off_v:off_v + n], dx=outd[4 + off_out:4 + off_out + n])
            res = outd.cpu().numpy()
            _assert_f32_equal(res[4 + off_out:4 + off_out + n], want[off_v:off_v + n], f"{name} offsets {off_dy},{off_v},{off_out}")
            assert np.all(res[:4 + off_out] == 7.0) and np.all(res[4 + off_out + n:] == 7.0)
        for n_small in (1, 3, 4, 5, 255, 256, 257):
            got = getattr(binding, name)(dyd[:n_small].clone(), vd[:n_small].clone())
            _assert_f32_equal(got.cpu().numpy(), want[:n_small], f"{name} n={n_small}")
        over = dyd.clone()
        getattr(binding, name)(over, vd, dx=over)
        _assert_f32_equal(over.cpu().numpy(), want, name + " over dy")
        over = vd.clone()
        getattr(binding, name)(dyd, over, dx=over)
        _assert_f32_equal(over.cpu().numpy(), want, name + " over the second input")


@pytest.mark.parametrize("B,H", [(1, 8), (5, 24), (3, 2056), (256, 2048)])
def test_lstm_cell_backward(gpu, oracle, B, H):
    binding, torch = gpu
    g3, c0 = wl.lstm_cell_inputs(1, B, H)
    gates = g3[0]
    rng = np.random.Generator(np.random.PCG64(53))
    dh = wl.f32_to_bf16_bits(rng.standard_normal((B, H), dtype=np.float32))
    dcn = rng.standard_normal((B, H), dtype=np.float32)
    if B * H >= 64:
        edge = wl.edge_bf16_patterns()
        gates.reshape(-1)[: edge.size] = edge                 # zeros, thresholds, Inf, NaN in the i-gate
        c0.reshape(-1)[:4] = [np.inf, -np.inf, np.nan, 1e-40]
    with np.errstate(all="ignore"):
        dg_ref, dc_ref = oracle.klstm_cell_backward(gates, c0, dh, dcn)
    dg, dc = binding.klstm_cell_backward(_to_dev(torch, gates), torch.from_numpy(c0).to("cuda:0"), _to_dev(torch, dh),
                                         torch.from_numpy(dcn).to("cuda:0"))
    _assert_bf16_equal(_to_host(dg, np.uint16).ravel(), dg_ref.ravel(), False, "dgates")
    dc = dc.cpu().numpy()
    nanp = np.isnan(dc_ref)
    assert np.array_equal(np.isnan(dc), nanp)
    assert np.array_equal(dc.view(np.uint32)[~nanp], dc_ref.view(np.uint32)[~nanp])


def test_gradients_on_64_interval_tables(gpu, oracle):
    """kswish64_backward, kgelu64_backward, their Float32 forms and klstm_cell64_backward against the
    oracle: every BFloat16 pattern as x, structured and random Float32 patterns, the fitted table and a
    random valid one, ragged sizes, in place."""
    binding, torch = gpu
    rng = np.random.Generator(np.random.PCG64(81))
    base = wl.all_bf16_patterns()
    x = np.concatenate([base, base, wl.mlp_preactivations(100003, seed=82)])
    dy = np.concatenate([rng.permutation(base), wl.f32_to_bf16_bits(rng.standard_normal(base.size + 100003, dtype=np.float32))])
    rows = _random_valid_table(np.random.Generator(np.random.PCG64(83)), 64)
    klut, olut = binding.KtanhLut64.from_tuples(rows), oracle.OracleLut64.from_tuples(rows)
    dyd, xd = _to_dev(torch, dy), _to_dev(torch, x)
    for name in ("kswish64_backward", "kgelu64_backward"):
        with np.errstate(all="ignore"):
            want, want_custom = getattr(oracle, name)(dy, x), getattr(oracle, name)(dy, x, olut)
        _assert_bf16_equal(_to_host(getattr(binding, name)(dyd, xd), np.uint16), want, False, name)
        _assert_bf16_equal(_to_host(getattr(binding, name)(dyd, xd, lut=klut), np.uint16), want_custom, False, name + " custom table")
        for n_small in (1, 7, 8, 9, 511, 512, 513, 8192 + 13):
            got = getattr(binding, name)(dyd[3:3 + n_small], xd[3:3 + n_small])
            _assert_bf16_equal(_to_host(got, np.uint16), want[3:3 + n_small], False, f"{name} n={n_small}")
        over = dyd.clone()
        getattr(binding, name)(over, xd, dx=over)
        _assert_bf16_equal(_to_host(over, np.uint16), want, False, name + " over dy")
    vf = _f32_cases().view(np.float32)
    dyf = rng.standard_normal(vf.size, dtype=np.float32)
    vd, dyfd = torch.from_numpy(vf).to("cuda:0"), torch.from_numpy(dyf).to("cuda:0")
    for name in ("kswish64_f32_backward", "kgelu64_f32_backward"):
        with np.errstate(all="ignore"):
            want, want_custom = getattr(oracle, name)(dyf, vf), getattr(oracle, name)(dyf, vf, olut)
        _assert_f32_equal(getattr(binding, name)(dyfd, vd).cpu().numpy(), want, name)
        _assert_f32_equal(getattr(binding, name)(dyfd, vd, lut=klut).cpu().numpy(), want_custom, name + " custom table")
        for n_small in (1, 3, 4, 5, 255, 257, 4096 * 3 + 3):
            got = getattr(binding, name)(dyfd[1:1 + n_small], vd[1:1 + n_small])
            _assert_f32_equal(got.cpu().numpy(), want[1:1 + n_small], f"{name} n={n_small}")
    for B, H in ((5, 24), (256, 2048)):
        g3, c0 = wl.lstm_cell_inputs(1, B, H)
        gates = g3[0]
        edge = wl.edge_bf16_patterns()
        gates.reshape(-1)[: edge.size] = edge
        dh = wl.f32_to_bf16_bits(rng.standard_normal((B, H), dtype=np.float32))
        dcn = rng.standard_normal((B, H), dtype=np.float32)
        for kl, ol in ((None, None), (klut, olut)):
            with np.errstate(all="ignore"):
                dg_ref, dc_ref = oracle.klstm_cell64_backward(gates, c0, dh, dcn, ol)
            dg, dc = binding.klstm_cell64_backward(_to_dev(torch, gates), torch.from_numpy(c0).to("cuda:0"),
                                                   _to_dev(torch, dh), torch.from_numpy(dcn).to("cuda:0"), lut=kl)
            _assert_bf16_equal(_to_host(dg, np.uint16).ravel(), dg_ref.ravel(), False, "dgates, 64 intervals")
            dc = dc.cpu().numpy()
            nanp = np.isnan(dc_ref)
            assert np.array_equal(np.isnan(dc), nanp)
            assert np.array_equal(dc.view(np.uint32)[~nanp], dc_ref.view(np.uint32)[~nanp])


def test_lstm_cell_tensors_need_only_pair_alignment(gpu, oracle):
    """gates and h 4-byte aligned, the state 8-byte aligned: views that start 4 (8) bytes into a
    16-byte aligned buffer give the oracle's results, forward (T = 1 and T = 9) and backward."""
    binding, torch = gpu
    rng = np.random.Generator(np.random.PCG64(84))
    B, H = 6, 40
    for T in (1, 9):
        gates, c0 = wl.lstm_cell_inputs(T, B, H)
        c_ref, h_ref = oracle.klstm_cell(gates, c0)
        gbuf = torch.zeros(gates.size + 8, dtype=torch.int16, device="cuda:0")
        gbuf[2:2 + gates.size] = _to_dev(torch, gates).reshape(-1)
        cbuf = torch.zeros(c0.size + 4, dtype=torch.float32, device="cuda:0")
        cbuf[2:2 + c0.size] = torch.from_numpy(c0).to("cuda:0").reshape(-1)
        hbuf = torch.full((T * B * H + 16,), 0x5A5A, dtype=torch.int16, device="cuda:0")
        cout = torch.full((c0.size + 8,), 7.0, dtype=torch.float32, device="cuda:0")
        gv, cv = gbuf[2:2 + gates.size].view(T, B, 4 * H), cbuf[2:2 + c0.size].view(B, H)
        assert gv.data_ptr() % 16 == 4 and cv.data_ptr() % 16 == 8
        binding.klstm_cell(gv, cv, c_out=cout[2:2 + c0.size].view(B, H), h_out=hbuf[6:6 + T * B * H].view(T, B, H))
        res_h, res_c = _to_host(hbuf, np.uint16), cout.cpu().numpy()
        assert np.array_equal(res_h[6:6 + T * B * H], h_ref.ravel()) and np.all(res_h[:6] == 0x5A5A) and np.all(res_h[6 + T * B * H:] == 0x5A5A)
        assert np.array_equal(res_c[2:2 + c0.size], c_ref.ravel()) and np.all(res_c[:2] == 7.0) and np.all(res_c[2 + c0.size:] == 7.0)
    g3, c0 = wl.lstm_cell_inputs(1, B, H)
    dh = wl.f32_to_bf16_bits(rng.standard_normal((B, H), dtype=np.float32))
    dcn = rng.standard_normal((B, H), dtype=np.float32)
    dg_ref, dc_ref = oracle.klstm_cell_backward(g3[0], c0, dh, dcn)
    gbuf = torch.zeros(g3[0].size + 8, dtype=torch.int16, device="cuda:0")
    gbuf[2:2 + g3[0].size] = _to_dev(torch, g3[0]).reshape(-1)
    dhbuf = torch.zeros(dh.size + 8, dtype=torch.int16, device="cuda:0")
    dhbuf[6:6 + dh.size] = _to_dev(torch, dh).reshape(-1)
    sbuf = torch.zeros(2 * (c0.size + 4), dtype=torch.float32, device="cuda:0")
    sbuf[2:2 + c0.size] = torch.from_numpy(c0).to("cuda:0").reshape(-1)
    sbuf[c0.size + 6:2 * c0.size + 6] = torch.from_numpy(dcn).to("cuda:0").reshape(-1)
    dgbuf = torch.full((g3[0].size + 8,), 0x5A5A, dtype=torch.int16, device="cuda:0")
    dcbuf = torch.full((c0.size + 8,), 7.0, dtype=torch.float32, device="cuda:0")
    binding.klstm_cell_backward(gbuf[2:2 + g3[0].size].view(B, 4 * H), sbuf[2:2 + c0.size].view(B, H),
                                dhbuf[6:6 + dh.size].view(B, H), sbuf[c0.size + 6:2 * c0.size + 6].view(B, H),
                                dgates=dgbuf[2:2 + g3[0].size].view(B, 4 * H), dc_prev=dcbuf[2:2 + c0.size].view(B, H))
    res_g, res_c = _to_host(dgbuf, np.uint16), dcbuf.cpu().numpy()
    assert np.array_equal(res_g[2:2 + g3[0].size], dg_ref.ravel()) and np.all(res_g[:2] == 0x5A5A) and np.all(res_g[2 + g3[0].size:] == 0x5A5A)
    assert np.array_equal(res_c[2:2 + c0.size], dc_ref.ravel()) and np.all(res_c[:2] == 7.0) and np.all(res_c[2 + c0.size:] == 7.0)


def test_autograd_functions_chain_the_gradient_entry_points(gpu, oracle):
    """torch.autograd through ktanh, ksigmoid and two LSTM-cell steps: the gradients that reach the
    leaves must be the oracle's, chained by hand in the same order."""
    binding, torch = gpu
    from paper_1909_07729_amd import autograd as kt
    rng = np.random.Generator(np.random.PCG64(57))

    def bf16_leaf(bits):
        return _to_dev(torch, bits).view(torch.bfloat16).requires_grad_()

    x = wl.mlp_preactivations(50021, seed=58)
    dy = wl.f32_to_bf16_bits(rng.standard_normal(x.size, dtype=np.float32))
    for fn, fwd, bwd, from_input in ((kt.ktanh, oracle.ktanh_bf16, oracle.ktanh_backward, False),
                                     (kt.ksigmoid, oracle.ksigmoid, oracle.ksigmoid_backward, False),
                                     (kt.kswish, oracle.kswish, oracle.kswish_backward, True),
                                     (kt.kgelu, oracle.kgelu, oracle.kgelu_backward, True)):
        xd = bf16_leaf(x)
        yd = fn(xd)
        yd.backward(_to_dev(torch, dy).view(torch.bfloat16))
        y_ref = fwd(x, None)
        _assert_bf16_equal(_to_host(yd.detach().view(torch.int16), np.uint16), y_ref, False, fn.__name__)
        _assert_bf16_equal(_to_host(xd.grad.view(torch.int16), np.uint16), bwd(dy, x if from_input else y_ref),
                           False, fn.__name__ + " grad")

    # the same four functions on Float32 tensors
    xf = wl.f32_mixture(40009, seed=69).view(np.float32)
    dyf = rng.standard_normal(xf.size, dtype=np.float32)
    for fn, fwd, bwd, from_input in ((kt.ktanh, lambda v: oracle.ktanh_f32(v.view(np.uint32)).view(np.float32), oracle.ktanh_f32_backward, False),
                                     (kt.ksigmoid, oracle.ksigmoid_f32, oracle.ksigmoid_f32_backward, False),
                                     (kt.kswish, oracle.kswish_f32, oracle.kswish_f32_backward, True),
                                     (kt.kgelu, oracle.kgelu_f32, oracle.kgelu_f32_backward, True)):
        xd = torch.from_numpy(xf).to("cuda:0").requires_grad_()
        yd = fn(xd)
        yd.backward(torch.from_numpy(dyf).to("cuda:0"))
        y_ref = fwd(xf)
        _assert_f32_equal(yd.detach().cpu().numpy(), y_ref, fn.__name__ + " f32")
        _assert_f32_equal(xd.grad.cpu().numpy(), bwd(dyf, xf if from_input else y_ref), fn.__name__ + " f32 grad")

    # two cell steps; the loss sees h of both steps and the final state
    B, H = 5, 24
    gates, c0 = wl.lstm_cell_inputs(2, B, H)
    dh = [wl.f32_to_bf16_bits(rng.standard_normal((B, H), dtype=np.float32)) for _ in range(2)]
    dc2 = rng.standard_normal((B, H), dtype=np.float32)
    g = [bf16_leaf(gates[t]) for t in range(2)]
    c0d = torch.from_numpy(c0).to("cuda:0").requires_grad_()
    h1, c1 = kt.klstm_cell(g[0], c0d)
    h2, c2 = kt.klstm_cell(g[1], c1)
    torch.autograd.backward([h1, h2, c2], [_to_dev(torch, dh[0]).view(torch.bfloat16),
                                           _to_dev(torch, dh[1]).view(torch.bfloat16),
                                           torch.from_numpy(dc2).to("cuda:0")])
    c1_ref, _ = oracle.klstm_cell(gates[:1], c0)
    dg2_ref, dc1_ref = oracle.klstm_cell_backward(gates[1], c1_ref, dh[1], dc2)
    dg1_ref, dc0_ref = oracle.klstm_cell_backward(gates[0], c0, dh[0], dc1_ref)
    _assert_bf16_equal(_to_host(g[1].grad.view(torch.int16), np.uint16).ravel(), dg2_ref.ravel(), False, "dgates step 2")
    _assert_bf16_equal(_to_host(g[0].grad.view(torch.int16), np.uint16).ravel(), dg1_ref.ravel(), False, "dgates step 1")
    assert np.array_equal(c0d.grad.cpu().numpy().view(np.uint32), dc0_ref.view(np.uint32))

    # 64-interval tables: the fitted one through intervals=64, a caller's one through its type
    rows = _random_valid_table(np.random.Generator(np.random.PCG64(85)), 64)
    klut, olut = binding.KtanhLut64.from_tuples(rows), oracle.OracleLut64.from_tuples(rows)
    for kwargs, ol in (({"intervals": 64}, None), ({"lut": klut}, olut)):
        for fn, fwd, bwd, from_input in ((kt.ktanh, oracle.ktanh64_bf16, oracle.ktanh_backward, False),
                                         (kt.ksigmoid, oracle.ksigmoid64, oracle.ksigmoid_backward, False),
                                         (kt.kswish, oracle.kswish64, oracle.kswish64_backward, True),
                                         (kt.kgelu, oracle.kgelu64, oracle.kgelu64_backward, True)):
            xd = bf16_leaf(x)
            yd = fn(xd, **kwargs)
            yd.backward(_to_dev(torch, dy).view(torch.bfloat16))
            with np.errstate(all="ignore"):
                y_ref = fwd(x, ol)
                g_ref = bwd(dy, x, ol) if from_input else bwd(dy, y_ref)
            _assert_bf16_equal(_to_host(yd.detach().view(torch.int16), np.uint16), y_ref, False, fn.__name__ + " 64")
            _assert_bf16_equal(_to_host(xd.grad.view(torch.int16), np.uint16), g_ref, False, fn.__name__ + " 64 grad")
        xd = torch.from_numpy(xf).to("cuda:0").requires_grad_()
        yd = kt.kgelu(xd, **kwargs)
        yd.backward(torch.from_numpy(dyf).to("cuda:0"))
        with np.errstate(all="ignore"):
            _assert_f32_equal(yd.detach().cpu().numpy(), oracle.kgelu64_f32(xf, ol), "kgelu f32 64")
            _assert_f32_equal(xd.grad.cpu().numpy(), oracle.kgelu64_f32_backward(dyf, xf, ol), "kgelu f32 64 grad")
        g0 = bf16_leaf(gates[0])
        c0d = torch.from_numpy(c0).to("cuda:0").requires_grad_()
        h1, c1 = kt.klstm_cell(g0, c0d, **kwargs)
        torch.autograd.backward([h1, c1], [_to_dev(torch, dh[0]).view(torch.bfloat16), torch.from_numpy(dc2).to("cuda:0")])
        with np.errstate(all="ignore"):
            dg_ref, dc_ref = oracle.klstm_cell64_backward(gates[0], c0, dh[0], dc2, ol)
        _assert_bf16_equal(_to_host(g0.grad.view(torch.int16), np.uint16).ravel(), dg_ref.ravel(), False, "dgates 64")
        cn = np.isnan(dc_ref)
        assert np.array_equal(c0d.grad.cpu().numpy().view(np.uint32)[~cn], dc_ref.view(np.uint32)[~cn])
    with pytest.raises(TypeError):
        kt.ktanh(bf16_leaf(x), lut=binding.ktanh_default_lut(), intervals=64)


# ------------------------------------------------------------------ random LSTM shapes
def test_lstm_random_shapes_and_special_values(gpu, oracle):
    """60 seeded draws of (T, B, H) -- every start-up and last-steps length of the kernel, ragged last
    blocks -- with infinities, NaNs, zeros and threshold values sprinkled into gates and state: fused
    and one call per step, 32- and 64-interval tables, and one step backwards, against the oracle."""
    binding, torch = gpu
    rng = np.random.Generator(np.random.PCG64(97))
    special = np.array([0x7F80, 0xFF80, 0x7FC0, 0xFFC1, 0x7F7F, 0x0000, 0x8000, 0x0001, 0x4080, 0xC080, 0x3E80, 0x3E7F],
                       dtype=np.uint16)

    def same(c_got, h_got, c_ref, h_ref, what):
        cn = np.isnan(c_ref)
        assert np.array_equal(np.isnan(c_got), cn), what
        assert np.array_equal(c_got.view(np.uint32)[~cn], c_ref.view(np.uint32)[~cn]), what
        _assert_bf16_equal(h_got.ravel(), h_ref.ravel(), False, what)

    for trial in range(60):
        T, B, H = int(rng.integers(1, 23)), int(rng.integers(1, 8)), 8 * int(rng.integers(1, 70))
        gates = wl.f32_to_bf16_bits(rng.standard_normal((T, B, 4 * H), dtype=np.float32) * 2)
        c0 = rng.standard_normal((B, H), dtype=np.float32)
        if trial % 3 == 0:
            k = int(rng.integers(1, 6))
            gates.reshape(-1)[rng.integers(0, gates.size, size=k)] = special[rng.integers(0, special.size, size=k)]
        if trial % 7 == 0:
            c0.reshape(-1)[int(rng.integers(0, c0.size))] = [np.inf, -np.inf, np.nan, 3e38][trial % 4]
        what = f"trial {trial} T={T} B={B} H={H}"
        gd, cd = _to_dev(torch, gates), torch.from_numpy(c0).to("cuda:0")
        with np.errstate(all="ignore"):
            for fn, ref in ((binding.klstm_cell, oracle.klstm_cell), (binding.klstm_cell64, oracle.klstm_cell64)):
                c_ref, h_ref = ref(gates, c0)
                c1, h1 = fn(gd, cd)
                same(c1.cpu().numpy(), _to_host(h1, np.uint16), c_ref, h_ref, f"{what} fused {fn.__name__}")
                cc, hs = cd.clone(), []
                for t in range(T):
                    cc, h = fn(gd[t:t + 1], cc, c_out=cc)
                    hs.append(h)
                same(cc.cpu().numpy(), _to_host(torch.cat(hs), np.uint16), c_ref, h_ref, f"{what} per step {fn.__name__}")
            dh = wl.f32_to_bf16_bits(rng.standard_normal((B, H), dtype=np.float32))
            dc = rng.standard_normal((B, H), dtype=np.float32)
            for fn, ref in ((binding.klstm_cell_backward, oracle.klstm_cell_backward),
                            (binding.klstm_cell64_backward, oracle.klstm_cell64_backward)):
                dg_ref, dcp_ref = ref(gates[0], c0, dh, dc)
                dg, dcp = fn(gd[0], cd, _to_dev(torch, dh), torch.from_numpy(dc).to("cuda:0"))
                same(dcp.cpu().numpy(), _to_host(dg, np.uint16), dcp_ref, dg_ref, f"{what} backward {fn.__name__}")


# ------------------------------------------------------------------ random sizes and alignments
def test_random_sizes_and_alignments_over_every_elementwise_entry_point(gpu, oracle):
    """400 seeded draws of (entry point, n, offset of each tensor): the peeled heads and tails, the
    switch to the element-wise kernel on mismatched alignment, and the guard bands around the output
    must hold for any of them, not only for the hand-picked cases above."""
    binding, torch = gpu
    rng = np.random.Generator(np.random.PCG64(63))
    N = 40000
    xb = np.concatenate([wl.all_bf16_patterns()[rng.permutation(1 << 16)[: N // 2]],
                         wl.mlp_preactivations(N - N // 2 + 64, seed=64)])
    db = wl.f32_to_bf16_bits(rng.standard_normal(xb.size, dtype=np.float32))
    xu = np.concatenate([rng.integers(0, 1 << 32, size=N // 2, dtype=np.uint64).astype(np.uint32),
                         wl.f32_mixture(N - N // 2 + 64, seed=65)])
    xf = xu.view(np.float32)
    df = rng.standard_normal(xf.size, dtype=np.float32)
    xbd, dbd, xud = _to_dev(torch, xb), _to_dev(torch, db), _to_dev(torch, xu)
    xfd, dfd = xud.view(torch.float32), torch.from_numpy(df).to("cuda:0")
    with np.errstate(all="ignore"):
        yb, sb = oracle.ktanh_bf16(xb), oracle.ksigmoid(xb)
        cases = {
            "kpade32_bf16": ("bf16", oracle.kpade32(xb)), "kpade78_bf16": ("bf16", oracle.kpade78(xb)),
            "ktaylor2_bf16": ("bf16", oracle.ktaylor2(xb)), "ktaylor3_bf16": ("bf16", oracle.ktaylor3(xb)),
            "ktanh_bf16": ("bf16", yb), "ksigmoid": ("bf16", sb), "kswish": ("bf16", oracle.kswish(xb)),
            "kgelu": ("bf16", oracle.kgelu(xb)), "ktanh64_bf16": ("bf16", oracle.ktanh64_bf16(xb)),
            "ksigmoid64": ("bf16", oracle.ksigmoid64(xb)), "kswish64": ("bf16", oracle.kswish64(xb)),
            "kgelu64": ("bf16", oracle.kgelu64(xb)),
            "ktanh_f32": ("u32", oracle.ktanh_f32(xu)), "ktanh64_f32": ("u32", oracle.ktanh64_f32(xu)),
            "ksigmoid_f32": ("f32", oracle.ksigmoid_f32(xf)), "kswish_f32": ("f32", oracle.kswish_f32(xf)),
            "kgelu_f32": ("f32", oracle.kgelu_f32(xf)),
            "ksigmoid64_f32": ("f32", oracle.ksigmoid64_f32(xf)), "kswish64_f32": ("f32", oracle.kswish64_f32(xf)),
            "kgelu64_f32": ("f32", oracle.kgelu64_f32(xf)),
            "ktanh_f32_to_bf16": ("f32->bf16", oracle.ktanh_f32_to_bf16(xf)),
            "ktanh_bf16_backward": ("grad", oracle.ktanh_backward(db, yb)),
            "ksigmoid_backward": ("grad", oracle.ksigmoid_backward(db, sb)),
            "kswish_backward": ("grad", oracle.kswish_backward(db, xb)),
            "kgelu_backward": ("grad", oracle.kgelu_backward(db, xb)),
            "kswish64_backward": ("grad", oracle.kswish64_backward(db, xb)),
            "kgelu64_backward": ("grad", oracle.kgelu64_backward(db, xb)),
            "kswish64_f32_backward": ("grad32", oracle.kswish64_f32_backward(df, xf)),
            "kgelu64_f32_backward": ("grad32", oracle.kgelu64_f32_backward(df, xf)),
            "kswish_f32_backward": ("grad32", oracle.kswish_f32_backward(df, xf)),
            "kgelu_f32_backward": ("grad32", oracle.kgelu_f32_backward(df, xf)),
            "ktanh_f32_backward": ("grad32", oracle.ktanh_f32_backward(df, xf)),
            "ksigmoid_f32_backward": ("grad32", oracle.ksigmoid_f32_backward(df, xf)),
        }
    ybd, sbd = _to_dev(torch, yb), _to_dev(torch, sb)
    names = sorted(cases)
    for trial in range(400):
        name = names[int(rng.integers(len(names)))]
        kind, want = cases[name]
        n = int(rng.choice([int(rng.integers(1, 40)), int(rng.integers(40, 3000)), int(rng.integers(3000, N))]))
        a, o, g = (int(v) for v in rng.integers(0, 17, size=3))      # element offsets of in, out, dy
        a = min(a, xb.size - n)
        what = f"trial {trial}: {name} n={n} offsets in={a} out={o} dy={g}"
        fn = getattr(binding, name)
        if kind in ("bf16", "grad", "f32->bf16"):
            guard = torch.full((n + 48,), 0x5A5A, dtype=torch.int16, device="cuda:0")
            out = guard[16 + o:16 + o + n]
            if kind == "bf16":
                fn(xbd[a:a + n], out=out)
            elif kind == "f32->bf16":
                fn(xfd[a:a + n], out=out)
            else:
                # dy needs its own offset: a shifted copy of the slice the expected values were made from
                dyd = torch.empty(n + 32, dtype=torch.int16, device="cuda:0")
                dyd[g:g + n] = dbd[a:a + n]
                second = {"ktanh_bf16_backward": ybd, "ksigmoid_backward": sbd}.get(name, xbd)
                fn(dyd[g:g + n], second[a:a + n], dx=out)
            res = _to_host(guard, np.uint16)
            _assert_bf16_equal(res[16 + o:16 + o + n], want[a:a + n], False, what)
            assert np.all(res[:16 + o] == 0x5A5A) and np.all(res[16 + o + n:] == 0x5A5A), what
        else:
            guard = torch.full((n + 48,), 0x5A5A5A5A, dtype=torch.int32, device="cuda:0")
            if kind == "grad32":
                dyd = torch.empty(n + 32, dtype=torch.float32, device="cuda:0")
                dyd[g:g + n] = dfd[a:a + n]
                fn(dyd[g:g + n], xfd[a:a + n], dx=guard.view(torch.float32)[16 + o:16 + o + n])
                res = guard.cpu().numpy().view(np.uint32)
                _assert_f32_equal(res[16 + o:16 + o + n].view(np.float32), want[a:a + n], what)
            elif kind == "u32":
                fn(xud[a:a + n], out=guard[16 + o:16 + o + n])
                res = guard.cpu().numpy().view(np.uint32)
                assert np.array_equal(res[16 + o:16 + o + n], want[a:a + n]), what
            else:
                fn(xfd[a:a + n], out=guard.view(torch.float32)[16 + o:16 + o + n])
                res = guard.cpu().numpy().view(np.uint32)
                _assert_f32_equal(res[16 + o:16 + o + n].view(np.float32), want[a:a + n], what)
            assert np.all(res[:16 + o] == 0x5A5A5A5A) and np.all(res[16 + o + n:] == 0x5A5A5A5A), what


# ------------------------------------------------------------------ Table 2's comparison approximants
def test_table2_comparators(gpu, oracle):
    """kpade32_bf16, kpade78_bf16, ktaylor2_bf16 and ktaylor3_bf16 against the oracle, bit for bit
    (same Float32 operations in the same order, correctly rounded division on both sides, the Taylor
    coefficients formed separately on each side): every BFloat16 pattern, a ragged sample of the
    transformer-MLP tensor at an odd offset, in place."""
    binding, torch = gpu
    x = np.concatenate([wl.all_bf16_patterns(), wl.mlp_preactivations(100003, seed=86)])
    xd = _to_dev(torch, x)
    for name, ref in (("kpade32_bf16", oracle.kpade32), ("kpade78_bf16", oracle.kpade78),
                      ("ktaylor2_bf16", oracle.ktaylor2), ("ktaylor3_bf16", oracle.ktaylor3)):
        want = ref(x)
        assert np.array_equal(_to_host(getattr(binding, name)(xd), np.uint16), want), name
        n = 50021
        outd = torch.full((n + 24,), 0x5A5A, dtype=torch.int16, device="cuda:0")
        getattr(binding, name)(xd[3:3 + n], out=outd[9:9 + n])
        res = _to_host(outd, np.uint16)
        assert np.array_equal(res[9:9 + n], want[3:3 + n]) and np.all(res[:9] == 0x5A5A) and np.all(res[9 + n:] == 0x5A5A), name
        over = xd.clone()
        getattr(binding, name)(over, out=over)
        assert np.array_equal(_to_host(over, np.uint16), want), name + " in place"


# ------------------------------------------------------------------ the accuracy report
def test_accuracy_report_figures_equal_the_oracle_s(gpu, oracle):
    """paper_1909_07729_amd.report measures the three tables with the GPU kernels; the error figures
    it prints must be the ones the oracle gives for the same tables."""
    from paper_1909_07729_amd import report
    bits = wl.all_bf16_patterns()
    bits = bits[(bits & 0x7FFF) < 0x7F80]
    x = wl.bf16_bits_to_f32(bits).astype(np.float64)
    want = [oracle.ktanh_bf16(bits), oracle.ktanh64_bf16(bits), oracle.ktanh_bf16(bits, oracle.fit_lut_bmin0())]
    rows = report.error_rows()
    assert len(rows) == 3
    for row, y in zip(rows, want):
        err = np.abs(wl.bf16_bits_to_f32(y).astype(np.float64) - np.tanh(x))
        assert row["max_abs"] == float(err.max()), row["table"]
        assert row["at"] == f"0x{int(bits[int(np.argmax(err))]):04X}"
        assert row["elements_per_s"] > 1e11
    assert rows[0]["max_abs"] < rows[1]["max_abs"] < rows[2]["max_abs"]
    assert rows[1]["mean_abs_region"] < rows[0]["mean_abs_region"] < rows[2]["mean_abs_region"]
    comp = report.comparator_rows()
    assert [r["approximant"] for r in comp] == ["Pade[3/2]", "Pade[7/8]", "Taylor degree 2, 32 intervals",
                                                "Taylor degree 3, 32 intervals"]
    for row, ref in zip(comp, (oracle.kpade32, oracle.kpade78, oracle.ktaylor2, oracle.ktaylor3)):
        err = np.abs(wl.bf16_bits_to_f32(ref(bits)).astype(np.float64) - np.tanh(x))
        assert row["max_abs"] == float(err.max()) and row["elements_per_s"] > 1e11
    derived = report.derived_rows()
    assert [r["op"] for r in derived] == ["Sigmoid", "Swish", "GELU (tanh form)"]
    assert all(r["mean_abs_64"] < r["mean_abs_32"] for r in derived)


# ------------------------------------------------------------------ the C ABI without Python
def test_native_consumer_of_the_c_abi(gpu):
    """tests/host_c/gpu_consumer.cpp: hipMalloc'd buffers, a stream of its own, the entry points called
    from C++, results checked in the same program against the CPU checker."""
    import os
    import subprocess
    import __graft_entry__ as entry
    exe = entry.NATIVE_CONSUMER
    assert os.path.exists(exe), f"{exe} is not built; run __graft_entry__.build()"
    res = subprocess.run([exe], capture_output=True, text=True, timeout=150)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip().endswith("all match"), res.stdout
