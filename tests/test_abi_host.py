"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, rejects bad arguments before any launch and
reports its configurations."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2108_13191_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2108_13191_amd import build
        build.build()
    return binding.load()


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "gemm_f16.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(gemm_\w+)\s*\(", text)
    assert {"gemm_f16_f32acc", "gemm_f16_f16acc", "gemm_strerror", "gemm_f16_query_config"} <= set(names)
    raw = ctypes.CDLL(binding.LIB_PATH)
    for n in set(names):
        assert hasattr(raw, n), f"{n} declared in the header but not exported"


def test_argument_errors_without_launch(lib):
    f32, f16 = binding.gemm_f16_f32acc, binding.gemm_f16_f16acc
    for fn in (f32, f16):
        assert fn(-1, 8, 8, 16, 8, 16, 8, 16, 8) == binding.ERR_SIZE
        assert fn(8, 8, 2**31, 16, 2**31, 16, 8, 16, 8) == binding.ERR_SIZE
        assert fn(8, 8, 8, 16, 7, 16, 8, 16, 8) == binding.ERR_PITCH
        assert fn(8, 8, 8, 16, 8, 16, 7, 16, 8) == binding.ERR_PITCH
        assert fn(8, 8, 8, 16, 8, 16, 8, 16, 7) == binding.ERR_PITCH
        assert fn(8, 8, 8, 0, 8, 16, 8, 16, 8) == binding.ERR_NULL
        assert fn(8, 8, 8, 16, 8, 0, 8, 16, 8) == binding.ERR_NULL
        assert fn(8, 8, 8, 16, 8, 16, 8, 0, 8) == binding.ERR_NULL
        assert fn(8, 8, 8, 17, 8, 16, 8, 16, 8) == binding.ERR_ALIGN
        # empty problems succeed without touching anything, whatever the pointers
        assert fn(0, 8, 8, 0, 8, 0, 8, 0, 8) == binding.OK
        assert fn(8, 0, 8, 0, 8, 0, 0, 0, 0) == binding.OK
    assert f32(8, 8, 8, 16, 8, 16, 8, 18, 8) == binding.ERR_ALIGN     # f32 C needs 4-byte alignment
    # f16 C needs 2-byte alignment only (asked through the query, which launches nothing)
    assert binding.query_config(1, 8, 8, 8, 16, 8, 16, 8, 18, 8)["id"] >= 0
    with pytest.raises(binding.GemmError) as e:
        binding.query_config(0, 8, 8, 8, 16, 8, 16, 8, 18, 8)
    assert e.value.code == binding.ERR_ALIGN


def test_strerror_texts(lib):
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        s = binding.strerror(code)
        assert isinstance(s, str) and s
        seen.add(s)
    assert len(seen) == 8


def test_config_table_and_selection(lib):
    n = binding.num_configs()
    assert n >= 2
    for i in range(n):
        d = binding.describe_config(i)
        assert d["id"] == i and d["block_m"] % d["wave_m"] == 0 and d["block_n"] % d["wave_n"] == 0
        assert d["waves"] == (d["block_m"] // d["wave_m"]) * (d["block_n"] // d["wave_n"])
        assert d["lds_bytes"] <= 160 * 1024
    with pytest.raises(binding.GemmError):
        binding.describe_config(n)
    big = binding.query_config(0, 8192, 8192, 8192, 16, 8192, 16, 8192, 16, 8192)
    tiles = (8192 // big["block_m"]) * (8192 // big["block_n"])
    # (the chained form of the large tile runs one workgroup per compute unit, 256 on an MI355X and without a GPU)
    assert big["block_m"] * big["block_n"] >= 128 * 128 and big["grid"] == (256 if big["name"].endswith("_chain") else tiles)
    small = binding.query_config(0, 256, 256, 256, 16, 256, 16, 256, 16, 256)
    assert small["block_m"] <= 128     # small problems take small tiles (more workgroups)
    # anything unaligned goes to the any-shape kernel
    for args in [(255, 256, 256, 16, 256, 16, 256), (256, 255, 256, 16, 256, 16, 255), (256, 256, 252, 16, 252, 16, 256),
                 (256, 256, 256, 18, 256, 16, 256), (256, 256, 256, 16, 260, 16, 256)]:
        M, N, K, A, lda, B, ldb = args
        got = binding.query_config(0, M, N, K, A, lda, B, ldb, 16, N)
        want = 0 if (N % 8 or K % 8 or A % 16 or lda % 8) else got["id"]
        assert got["id"] == want
    assert binding.force_config(n) == binding.ERR_CONFIG
    assert binding.force_config(0) == 0
    assert binding.query_config(0, 8192, 8192, 8192, 16, 8192, 16, 8192, 16, 8192)["id"] == 0
    binding.force_config(-1)


def test_large_pitches_take_64_bit_addressing(lib):
    """The tuned kernels keep tile-relative offsets in 32 bits; a pitch beyond what that covers
    (for any of A, B, C) must select the any-shape kernel, whose addresses are all 64-bit."""
    ok = binding.query_config(0, 512, 512, 512, 256, 512, 256, 512, 256, 1 << 22)
    assert ok["id"] != 0
    for mode in (0, 1):
        for ldc in (1 << 26, 1 << 28, 2**31 - 8):
            q = binding.query_config(mode, 512, 512, 512, 256, 512, 256, 512, 256, ldc)
            assert q["id"] == 0 and q["name"].startswith("generic"), (mode, ldc, q)
        for big in ((1 << 22) + 8, 1 << 28, 2**31 - 8):
            assert binding.query_config(mode, 512, 512, 512, 256, big, 256, 512, 256, 512)["id"] == 0
            assert binding.query_config(mode, 512, 512, 512, 256, 512, 256, big, 256, 512)["id"] == 0
    # a forced tuned configuration does not override that
    tuned = [i for i in range(binding.num_configs()) if binding.describe_config(i)["name"].startswith("t64")][0]
    binding.force_config(tuned)
    try:
        assert binding.query_config(0, 512, 512, 512, 256, 512, 256, 512, 256, 512)["id"] == tuned
        assert binding.query_config(0, 512, 512, 512, 256, 512, 256, 512, 256, 1 << 28)["id"] == 0
    finally:
        binding.force_config(-1)


def test_header_is_plain_c(tmp_path):
    """include/gemm_f16.h compiles as C99 on its own, and a C program that calls
    the host-only entry points links against the library and runs (no GPU)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    hdr = os.path.join(root, "include", "gemm_f16.h")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", hdr], check=True)
    src = tmp_path / "use.c"
    src.write_text('''
#include <stdio.h>
#include <string.h>
#include "gemm_f16.h"
int main(void) {
    gemm_f16_config c;
    if (gemm_f16_num_configs() < 1) return 1;
    if (gemm_f16_describe_config(0, &c) != GEMM_F16_OK || strlen(c.name) == 0) return 2;
    if (gemm_f16_query_config(0, 8192, 8192, 8192, (void*)256, 8192, (void*)256, 8192, (void*)256, 8192, &c) != GEMM_F16_OK) return 3;
    if (c.block_m != 256 || (c.grid != 1024 && c.grid != 256)) return 4;
    if (gemm_f16_f32acc(-1, 1, 1, 0, 1, 0, 1, 0, 1, 0) != GEMM_F16_ERR_SIZE) return 5;
    if (gemm_f16_f32acc_bias_act(4, 4, 4, (void*)256, 4, (void*)256, 4, (float*)256, 4, 0, 9, 0) != GEMM_F16_ERR_CONFIG) return 6;
    printf("%s\\n", gemm_strerror(GEMM_F16_ERR_PITCH));
    return 0;
}
''')
    exe = tmp_path / "use"
    libdir = os.path.join(root, "paper_2108_13191_amd")
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(root, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-lgemm_f16", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True)
    assert "leading dimension" in out.stdout


def test_overlap_kernel_keeps_in_flight_registers_untouched():
    """gemm_overlap.hip uses loaded registers two k steps after the load without a wait the
    compiler knows of; the generated code must not touch them in between."""
    import shutil
    if shutil.which("hipcc") is None:
        pytest.skip("no hipcc")
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location(
        "check_overlap_asm", os.path.join(root, "paper_2108_13191_amd", "csrc", "ladder", "check_overlap_asm.py"))
    check_overlap_asm = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(check_overlap_asm)
    # the scanner itself: a planted use of an in-flight register is found, a use after the marker is not
    planted = ("_Zk:\n\tglobal_load_dwordx4 v[10:13], v[2:3], off ; C slab load\n\tv_add_f32_e32 v1, v11, v1\n"
               "\t; C slab arrived v[10:13]\n\tv_add_f32_e32 v1, v12, v1\n")
    loads, bad = check_overlap_asm.hazards(planted)
    assert loads == 1 and [b[0] for b in bad] == [3]
    loads, bad = check_overlap_asm.hazards(check_overlap_asm.compile_to_asm())
    assert loads >= 64 and not bad, bad[:3]


def test_plan_invariants_on_random_shapes(lib):
    """Whatever the selector picks, the plan is well formed: the rows are covered once, a cut
    lies on a 256-row boundary, every launch has workgroups, and the launch forms with
    conditions are only chosen where they apply."""
    rng = np.random.default_rng(12345)
    n = n_product = binding.num_configs()
    names = [binding.describe_config(i)["name"] for i in range(n)]
    for _ in range(3000):
        M = int(rng.integers(1, 20000))
        N = int(rng.integers(1, 2500)) * 8
        K = int(rng.integers(1, 1200)) * 8
        q = binding.query_config(int(rng.integers(0, 2)), M, N, K, 256, K, 256, N, 256, N)
        assert 0 < q["id"] < n and q["name"] == names[q["id"]] and q["grid"] >= 1, (M, N, K, q)
        if q["split_rows"]:
            assert 0 < q["split_rows"] < M and q["split_rows"] % 256 == 0 and 0 < q["id2"] < n, (M, N, K, q)
            assert q["block_m"] == 256 and q["block_n"] == 256
        else:
            assert q["id2"] == -1
        tiles256 = ((M + 255) // 256) * ((N + 255) // 256)
        if q["name"].endswith("_chain"):
            rows = q["split_rows"] or M
            assert K % 64 == 0 and ((rows + 255) // 256) * ((N + 255) // 256) > 256 and (q["split_rows"] or q["grid"] == 256)
        if q["name"].endswith("_stag"):
            assert K <= 1024 and tiles256 >= 512 and 0 < tiles256 % 256 <= 128 and q["grid"] == tiles256 + 128
        assert q["id"] < n_product                                                   # comparison kernels are never selected


def test_split_k_plan_invariants(lib):
    """The k loop is cut only in f32 mode, only for the five-stage 128 x 128 kernel, into parts
    of at least 16 k steps, with at most one workgroup per compute unit and at most four million
    additions; the f16 query of the same shape never reports it."""
    rng = np.random.default_rng(777)
    seen = 0
    for _ in range(3000):
        M = int(rng.integers(1, 600))
        N = int(rng.integers(1, 1200)) * 8
        K = int(rng.integers(16, 4000)) * 8
        tiles = ((M + 127) // 128) * ((N + 127) // 128)
        q = binding.query_config(0, M, N, K, 256, K, 256, N, 256, N)
        q16 = binding.query_config(1, M, N, K, 256, K, 256, N, 256, N)
        if q["name"] == "w4a_128x128x64" and q["grid"] != tiles:
            parts = q["grid"] // tiles
            assert q["grid"] == parts * tiles and 2 <= parts <= 16 and q["grid"] <= 256 and not q["split_rows"], (M, N, K, q)
            assert parts * M * N <= 4194304 and (K + 63) // 64 >= 16 * parts, (M, N, K, q)
            seen += 1
        if q16["name"] == "w4a_128x128x64":
            assert q16["grid"] == tiles, (M, N, K, q16)
    assert seen > 300
