"""What the compiler made of the kernels, read from the gfx950 assembly of the shipped sources built
with the shipped flags: no packed Float32 arithmetic, no register spills to scratch memory, and the
table reads are the cross-lane instruction the design rests on."""
import os
import re
import subprocess

import pytest

from paper_1909_07729_amd import build

HIP_SOURCES = [s for s in build.SOURCES + build.PROBE_SOURCES if s.endswith(".hip")]


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    out = {}
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    tmp = tmp_path_factory.mktemp("asm")
    procs = []
    for src in HIP_SOURCES:
        dst = str(tmp / (src + ".s"))
        cmd = [hipcc, *flags, "-S", "--cuda-device-only", "-I", os.path.join(build.ROOT, "include"),
               "-I", build.CSRC, os.path.join(build.CSRC, src), "-o", dst]
        procs.append((src, dst, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE)))
    for src, dst, p in procs:
        _, err = p.communicate(timeout=600)
        assert p.returncode == 0, err.decode()
        out[src] = open(dst).read()
    return out


def test_no_packed_float32_arithmetic(assembly):
    for src, text in assembly.items():
        hits = re.findall(r"v_pk_(?:add|mul|fma)_f32", text)
        assert not hits, f"{src}: {len(hits)} packed Float32 instructions"


def test_no_kernel_spills_registers(assembly):
    for src, text in assembly.items():
        sizes = [int(v) for v in re.findall(r"\.amdhsa_private_segment_fixed_size\s+(\d+)", text)]
        assert sizes and all(v == 0 for v in sizes), f"{src}: private segment sizes {sizes}"
        assert "scratch_load" not in text and "scratch_store" not in text, src


def test_table_reads_are_cross_lane_and_stores_stream(assembly):
    for src, store in (("ktanh_stream.hip", r"global_store_dwordx4 .* sc0 sc1 nt"),
                       ("ktanh_lstm.hip", r"global_store_dword .* sc1$")):
        text = assembly[src]
        assert "ds_bpermute_b32" in text, src
        assert "ds_read" not in text and "ds_write" not in text, f"{src}: the table must not live in LDS"
        assert re.search(store, text, flags=re.M), src
    assert re.search(r"global_load_dwordx4 .* nt", assembly["ktanh_stream.hip"])


def test_lstm_steady_loop_waits_for_its_own_gate_words_only(assembly):
    """With four register stages of four loads each, and the gate words of a step consumed one step
    early (its activations are formed under the previous step's wait), a step must wait for its four
    words with eight to eleven younger memory operations still in flight; a wait for everything
    (vmcnt(0)) inside the steady loop would serialise memory and arithmetic."""
    text = assembly["ktanh_lstm.hip"]
    loop = text[text.index("Inner Loop Header"):]
    loop = loop[:loop.index("s_endpgm")]
    for count in (11, 10, 9, 8):
        assert f"s_waitcnt vmcnt({count})" in loop, count
    steady = loop[:loop.index("ds_bpermute_b32")]          # the unrolled body up to the first out-of-line path
    assert "vmcnt(0)" not in steady


def test_wide_stores_written_as_statements_keep_their_data_registers(assembly):
    """A store of more than 64 bits reads its data registers for a few cycles after issue; the
    compiler inserts the wait for stores it emits itself but cannot see into a statement, so each such
    statement carries its own two idle slots."""
    seen = 0
    for src, text in assembly.items():
        lines = text.splitlines()
        for i, line in enumerate(lines):
            if "global_store_dwordx4" in line and "sc0 sc1 nt" in line:
                seen += 1
                assert lines[i + 1].strip() == "s_nop 1", f"{src}: {line.strip()} is followed by {lines[i + 1].strip()}"
    assert seen > 20


def test_leading_scalar_arguments_are_preloaded(assembly):
    """Every streaming kernel gets the pointers and sizes it needs for its first load in registers."""
    for src in ("ktanh_stream.hip", "ktanh_backward.hip", "ktanh_probe.hip"):
        lengths = [int(v) for v in re.findall(r"\.amdhsa_user_sgpr_kernarg_preload_length\s+(\d+)", assembly[src])]
        assert lengths and min(lengths) >= 4, (src, sorted(set(lengths)))
