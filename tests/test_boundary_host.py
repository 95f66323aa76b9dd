"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what the header
declares, carries the paper's table, validates tables, and rejects bad arguments before any launch."""
import ctypes
import os
import re
import subprocess

import pytest

from conftest import ROOT, read_golden


@pytest.fixture(scope="module")
def binding():
    from paper_1909_07729_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_1909_07729_amd import build
        build.build_library()
    b.load_library()
    return b


def _declarations(header):
    """{function name: number of parameters} for every function a header declares."""
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    found = {}
    for name, params in re.findall(r"\b(k\w+)\s*\(([^)]*)\)\s*;", text):
        params = params.strip()
        found[name] = 0 if params in ("", "void") else params.count(",") + 1
    return found


@pytest.fixture(scope="module")
def probe(binding):
    from paper_1909_07729_amd import probe as p
    if not os.path.exists(p.LIB_PATH):
        from paper_1909_07729_amd import build
        build.build_probe_library()
    p.load_library()
    return p


def test_every_declared_symbol_is_exported(binding, probe):
    for module, header in ((binding, "ktanh.h"), (probe, "ktanh_probe.h")):
        declared = _declarations(header)
        assert set(declared) == set(module.EXPORTS), header
        lib = module.load_library()
        for name in declared:
            assert getattr(lib, name) is not None
    # the yardsticks stay out of the product library
    assert not any(hasattr(binding.load_library(), name) for name in probe.EXPORTS)


def test_prototypes_match_the_header(binding, probe):
    """Every ctypes prototype has as many parameters as the header's declaration, and pointer, size and
    table kinds where the header has them."""
    for module, header in ((binding, "ktanh.h"), (probe, "ktanh_probe.h")):
        lib = module.load_library()
        for name, count in _declarations(header).items():
            fn = getattr(lib, name)
            assert len(fn.argtypes) == count == len(module.SIGNATURES[name]), name
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "ktanh.h")).read(), flags=re.S)
    for name, params in re.findall(r"\b(k\w+)\s*\(([^)]*)\)\s*;", text):
        kinds = binding.SIGNATURES[name]
        for kind, param in zip(kinds, [q.strip() for q in params.split(",")] if params.strip() not in ("", "void") else []):
            if kind == "l":
                assert "ktanh_lut_t" in param, (name, param)
            elif kind == "L":
                assert "ktanh_lut64_t" in param, (name, param)
            elif kind == "n":
                assert param.startswith("size_t"), (name, param)
            elif kind == "s":
                assert param.startswith("ktanh_stream_t"), (name, param)
            elif kind == "p":
                assert "*" in param and "lut" not in param, (name, param)


def test_a_failed_call_raises_ktanh_error(binding, monkeypatch):
    """The error path of the table fits: a non-zero status becomes a KtanhError that names the call."""
    class Failing:
        def __getattr__(self, name):
            if name == "ktanh_status_string":
                return lambda status: b"KT_ERR_NULL: a required pointer is NULL"
            return lambda *args: 1
    monkeypatch.setattr(binding, "_lib", Failing())
    for name in ("ktanh_fit_lut", "ktanh_fit_lut_bmin0", "ktanh_fit_lut64"):
        with pytest.raises(binding.KtanhError) as err:
            getattr(binding, name)()
        assert err.value.status == 1 and name in str(err.value)


def test_struct_layout_is_96_bytes(binding):
    assert ctypes.sizeof(binding.KtanhLut) == 96


def test_default_lut_is_table1(binding):
    want = [None] * 32
    for bits, E, r, b in read_golden("table1_bf16.txt"):
        want[int(bits, 2)] = (int(E), int(r), int(b))
    assert binding.ktanh_default_lut().as_tuples() == want
    assert binding.ktanh_lut_validate(binding.ktanh_default_lut()) == 0


def test_lut_validation(binding):
    assert binding.ktanh_lut_validate(None) == 1
    rows = binding.ktanh_default_lut().as_tuples()

    def status(t, row):
        bad = list(rows); bad[t] = row
        return binding.ktanh_lut_validate(binding.KtanhLut.from_tuples(bad))

    assert status(0, (126, 2, 120)) == 0          # still inside 0..127: (15 >> 2) + 120 = 123
    assert status(7, (126, 6, 127)) == 3          # (127 >> 6) + 127 = 128 overflows the mantissa
    assert status(9, (125, 0, -17)) == 3          # (16 >> 0) - 17 < 0 underflows
    assert status(3, (126, 8, 0)) == 3            # shift beyond the mantissa width
    assert status(3, (0, 1, 0)) == 3 and status(3, (255, 1, 0)) == 3   # exponent field out of range
    assert status(15, (125, 0, -112)) == 0        # b_min of the interval with mantissa_idx_val 7
    assert status(15, (125, 0, -113)) == 3


def test_argument_errors_are_returned_before_any_launch(binding):
    lib = binding.load_library()
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(0x1000)                # never dereferenced: rejected on the host
    for name in ("ktanh_bf16", "ktanh_f32", "ksigmoid", "kswish", "kgelu", "ksigmoid_f32", "kswish_f32",
                 "kgelu_f32", "ktanh_f32_to_bf16"):
        fn = getattr(lib, name)
        assert fn(null, null, 0, None, null) == 0             # n == 0: nothing to do
        assert fn(null, fake, 8, None, null) == 1
        assert fn(fake, null, 8, None, null) == 1
        assert fn(ctypes.c_void_p(0x1001), fake, 8, None, null) == 2
    assert lib.ktanh_f32(ctypes.c_void_p(0x1002), fake, 8, None, null) == 2
    bad = binding.KtanhLut.from_tuples([(126, 9, 0)] * 32)
    assert lib.ktanh_bf16(fake, fake, 8, ctypes.byref(bad), null) == 3
    # LSTM cell
    assert lib.klstm_cell(null, null, null, null, 0, 4, 8, None, null) == 0
    assert lib.klstm_cell(null, fake, fake, fake, 1, 4, 8, None, null) == 1
    assert lib.klstm_cell(fake, fake, fake, fake, 1, 4, 12, None, null) == 4
    # BFloat16 pairs need 4-byte alignment, Float32 pairs 8-byte alignment; nothing more
    assert lib.klstm_cell(ctypes.c_void_p(0x1002), fake, fake, fake, 1, 4, 8, None, null) == 2
    assert lib.klstm_cell(fake, ctypes.c_void_p(0x1004), fake, fake, 1, 4, 8, None, null) == 2
    assert lib.klstm_cell(fake, fake, fake, ctypes.c_void_p(0x1006), 1, 4, 8, None, null) == 2
    assert lib.klstm_cell(fake, fake, fake, fake, 1, 4, 8, ctypes.byref(bad), null) == 3
    assert b"KT_ERR_LUT" in lib.ktanh_status_string(3)


def test_binding_refuses_host_tensors(binding):
    import torch
    with pytest.raises(ValueError):
        binding.ktanh_bf16(torch.zeros(8, dtype=torch.bfloat16))


def test_library_fit_reproduces_table1_and_matches_the_oracle_fit64(binding, oracle):
    """The library carries its own implementation of Section 2.4's optimisation (no code shared with
    the oracle): 32 intervals must give Table 1, 64 intervals what the oracle's fit gives."""
    want = [None] * 32
    for bits, E, r, b in read_golden("table1_bf16.txt"):
        want[int(bits, 2)] = (int(E), int(r), int(b))
    assert binding.ktanh_fit_lut().as_tuples() == want
    lut64 = binding.ktanh_fit_lut64()
    assert lut64.as_tuples() == oracle.fit_lut64().as_tuples()
    assert binding.ktanh_lut64_validate(lut64) == 0
    ablation = binding.ktanh_fit_lut_bmin0()
    assert ablation.as_tuples() == oracle.fit_lut_bmin0().as_tuples()
    assert binding.ktanh_lut_validate(ablation) == 0
    lib = binding.load_library()
    assert lib.ktanh_fit_lut(None) == 1 and lib.ktanh_fit_lut64(None) == 1 and lib.ktanh_fit_lut_bmin0(None) == 1


def test_lut64_validation(binding):
    assert binding.ktanh_lut64_validate(None) == 1
    rows = binding.ktanh_fit_lut64().as_tuples()

    def status(t, row):
        bad = list(rows); bad[t] = row
        return binding.ktanh_lut64_validate(binding.KtanhLut64.from_tuples(bad))

    assert status(15, (126, 6, 126)) == 0         # (127 >> 6) + 126 = 127: the last value allowed
    assert status(15, (126, 6, 127)) == 3
    assert status(17, (125, 0, -8)) == 0          # interval 17 starts at mantissa 8
    assert status(17, (125, 0, -9)) == 3
    assert status(40, (126, 8, 0)) == 3 and status(40, (0, 1, 0)) == 3
    lib = binding.load_library()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    bad = binding.KtanhLut64.from_tuples([(126, 9, 0)] * 64)
    for name in ("ktanh64_bf16", "ktanh64_f32"):
        fn = getattr(lib, name)
        assert fn(null, null, 0, None, null) == 0
        assert fn(null, fake, 8, None, null) == 1
        assert fn(ctypes.c_void_p(0x1001), fake, 8, None, null) == 2
        assert fn(fake, fake, 8, ctypes.byref(bad), null) == 3


def test_header_is_valid_c_and_host_entry_points_work_from_c(binding, tmp_path):
    """include/ktanh.h compiled as strict C99 by gcc, linked against the built library."""
    exe = tmp_path / "abi_check"
    libdir = os.path.dirname(binding.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                    "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "host_c", "abi_check.c"),
                    "-o", str(exe), "-L", libdir, "-lktanh", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert out.strip() == "KT_OK"


def test_host_sources_under_address_and_ub_sanitizers(tmp_path):
    """Table, validation, packing and fit are plain host C++: run them under ASan + UBSan."""
    exe = tmp_path / "sanitize_host"
    csrc = os.path.join(ROOT, "paper_1909_07729_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                    "-I", os.path.join(ROOT, "include"), "-I", csrc,
                    os.path.join(ROOT, "tests", "host_c", "sanitize_host.cpp"),
                    os.path.join(csrc, "ktanh_lut.cpp"), os.path.join(csrc, "ktanh_fit.cpp"), "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1")
    res = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "host sources clean" in res.stdout


def test_sizes_beyond_the_grid_limit_are_rejected_on_the_host(binding):
    """A launch holds fewer than 2^32 work-items, i.e. at most 2^26 - 1 single-wavefront tiles of
    1 KiB of output; larger tensors are refused (status 4) before anything is launched, so the fake
    pointers are never touched."""
    lib = binding.load_library()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    for name in ("ktanh_bf16", "ksigmoid", "kswish", "kgelu", "ktanh64_bf16"):
        assert getattr(lib, name)(fake, fake, (1 << 40) + 8, None, null) == 4
        assert getattr(lib, name)(fake, fake, 1 << 35, None, null) == 4      # 2^26 tiles: one too many
    for name in ("ktanh_f32", "ksigmoid_f32", "ktanh64_f32"):
        assert getattr(lib, name)(fake, fake, 1 << 34, None, null) == 4
    assert lib.ktanh_f32_to_bf16(fake, fake, 1 << 34, None, null) == 4       # 512-byte tiles of output
    for name in ("ktanh_bf16_backward", "ksigmoid_backward"):
        assert getattr(lib, name)(fake, fake, fake, 1 << 35, null) == 4
    # LSTM cell: B * H / 2 lane pairs must stay below 2^28; T below 2^31
    assert lib.klstm_cell(fake, fake, fake, fake, 1, 1 << 20, 1 << 9, None, null) == 4
    assert lib.klstm_cell(fake, fake, fake, fake, 1 << 31, 1, 8, None, null) == 4
    assert lib.klstm_cell64(fake, fake, fake, fake, 1, 1 << 20, 1 << 9, None, null) == 4


def test_gradient_entry_points_reject_bad_arguments(binding):
    lib = binding.load_library()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    for name in ("ktanh_bf16_backward", "ksigmoid_backward"):
        fn = getattr(lib, name)
        assert fn(null, null, null, 0, null) == 0
        assert fn(fake, null, fake, 8, null) == 1
        assert fn(fake, fake, ctypes.c_void_p(0x1001), 8, null) == 2
        assert fn(fake, fake, fake, (1 << 40) + 8, null) == 4
    bad = binding.ktanh_default_lut()
    bad.r[5] = 9
    for name in ("kswish_backward", "kgelu_backward"):
        fn = getattr(lib, name)
        assert fn(null, null, null, 0, None, null) == 0
        assert fn(fake, fake, null, 8, None, null) == 1
        assert fn(ctypes.c_void_p(0x1001), fake, fake, 8, None, null) == 2
        assert fn(fake, fake, fake, (1 << 40) + 8, None, null) == 4
        assert fn(fake, fake, fake, 8, ctypes.byref(bad), null) == 3
    for name in ("ktanh_f32_backward", "ksigmoid_f32_backward"):
        fn = getattr(lib, name)
        assert fn(null, null, null, 0, null) == 0
        assert fn(fake, null, fake, 8, null) == 1
        assert fn(fake, fake, ctypes.c_void_p(0x1002), 8, null) == 2
        assert fn(fake, fake, fake, (1 << 40) + 8, null) == 4
    for name in ("kswish_f32_backward", "kgelu_f32_backward"):
        fn = getattr(lib, name)
        assert fn(null, null, null, 0, None, null) == 0
        assert fn(null, fake, fake, 8, None, null) == 1
        assert fn(fake, ctypes.c_void_p(0x1001), fake, 8, None, null) == 2
        assert fn(fake, fake, fake, 8, ctypes.byref(bad), null) == 3
    bw = lib.klstm_cell_backward
    assert bw(null, null, null, null, null, null, 0, 8, None, null) == 0
    assert bw(fake, fake, fake, null, fake, fake, 2, 8, None, null) == 1
    assert bw(fake, fake, fake, fake, fake, fake, 2, 12, None, null) == 4
    assert bw(fake, fake, ctypes.c_void_p(0x1002), fake, fake, fake, 2, 8, None, null) == 2
    assert bw(fake, ctypes.c_void_p(0x1004), fake, fake, fake, fake, 2, 8, None, null) == 2
    assert bw(fake, fake, fake, fake, fake, fake, 1 << 20, 1 << 9, None, null) == 4
    bad64 = binding.KtanhLut64.from_tuples([(126, 9, 0)] * 64)
    for name in ("kswish64_backward", "kgelu64_backward", "kswish64_f32_backward", "kgelu64_f32_backward"):
        fn = getattr(lib, name)
        assert fn(null, null, null, 0, None, null) == 0
        assert fn(fake, fake, null, 8, None, null) == 1
        assert fn(ctypes.c_void_p(0x1001), fake, fake, 8, None, null) == 2
        assert fn(fake, fake, fake, 8, ctypes.byref(bad64), null) == 3
    bw64 = lib.klstm_cell64_backward
    assert bw64(null, null, null, null, null, null, 0, 8, None, null) == 0
    assert bw64(fake, fake, fake, null, fake, fake, 2, 8, None, null) == 1
    assert bw64(fake, fake, fake, fake, fake, fake, 2, 12, None, null) == 4
    assert bw64(fake, fake, fake, fake, fake, fake, 2, 8, ctypes.byref(bad64), null) == 3


def test_probe_library_rejects_bad_arguments(probe):
    lib = probe.load_library()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    aligned = ctypes.c_void_p(0x10000)
    assert lib.ktanh_probe_copy(null, null, 0, null) == 0
    assert lib.ktanh_probe_copy(fake, null, 8, null) == 1
    assert lib.ktanh_probe_copy(ctypes.c_void_p(0x1001), fake, 8, null) == 2
    assert lib.ktanh_probe_read(null, fake, 1024, null) == 1 and lib.ktanh_probe_read(aligned, null, 1024, null) == 1
    assert lib.ktanh_probe_read(ctypes.c_void_p(0x1010), fake, 1024, null) == 2 and lib.ktanh_probe_read(aligned, fake, 1000, null) == 4
    assert lib.ktanh_probe_write(null, 1024, null) == 1 and lib.ktanh_probe_write(ctypes.c_void_p(0x1010), 1024, null) == 2
    assert lib.ktanh_probe_write(aligned, 1 << 37, null) == 4 and lib.ktanh_probe_write(null, 0, null) == 0
    assert lib.ktanh_probe_read_wide(null, fake, 1024, null) == 1 and lib.ktanh_probe_read_wide(aligned, fake, 1000, null) == 4
    assert lib.ktanh_probe_read_wide(ctypes.c_void_p(0x1010), fake, 1024, null) == 2 and lib.ktanh_probe_read_wide(aligned, null, 1024, null) == 1
    assert lib.ktanh_probe_write_wide(null, 1024, null) == 1 and lib.ktanh_probe_write_wide(ctypes.c_void_p(0x1010), 1024, null) == 2
    assert lib.ktanh_probe_write_wide(aligned, 1 << 37, null) == 4 and lib.ktanh_probe_write_wide(null, 0, null) == 0
    cell = lib.ktanh_probe_lstm
    assert cell(null, null, null, null, 0, 4, 8, null) == 0 and cell(fake, fake, null, fake, 1, 4, 8, null) == 1
    assert cell(fake, fake, fake, fake, 1, 4, 12, null) == 4 and cell(ctypes.c_void_p(0x1002), fake, fake, fake, 1, 4, 8, null) == 2
    assert cell(fake, ctypes.c_void_p(0x1004), fake, fake, 1, 4, 8, null) == 2
