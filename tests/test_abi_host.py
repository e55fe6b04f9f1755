"""CPU-only checks of the C-ABI library: it loads, exports what include/duqpp.h declares, and
its host-side argument validation returns the documented codes without touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "duqpp.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2604_17789_amd as duqpp
    return duqpp.lib


def _declared_symbols():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(duqpp_[a-z0-9_]+)\s*\(", src)))


def test_header_declares_the_four_entry_points():
    names = _declared_symbols()
    for n in ("duqpp_quantize_weights", "duqpp_rotate_quantize", "duqpp_mxfp4_gemm", "duqpp_rotq_gemm"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    for name in _declared_symbols():
        assert hasattr(lib, name), name


def test_status_strings_and_version(lib):
    assert lib.duqpp_status_string(0) == b"ok"
    seen = {lib.duqpp_status_string(-i) for i in range(0, 8)}
    assert len(seen) == 8
    assert lib.duqpp_status_string(-99) == b"unknown status"
    assert b"gfx950" in lib.duqpp_version()


OK, NULL, SHAPE, ALIGN, DTYPE, WORKSPACE = 0, -1, -2, -3, -4, -5
P = 0x10000   # a fake, well-aligned, never dereferenced device address


def test_validate_rotate_quantize(lib):
    v = lib.duqpp_validate_rotate_quantize
    assert v(P, 4, 64, 64, P, 2, P, P) == OK
    assert v(P, 4, 64, 64, P, 1, P, P) == OK            # shared block
    assert v(None, 4, 64, 64, P, 2, P, P) == NULL
    assert v(P, 4, 64, 64, None, 2, P, P) == NULL
    assert v(P, 4, 64, 64, P, 2, None, P) == NULL
    assert v(P, 4, 64, 64, P, 2, P, None) == NULL
    assert v(P, 0, 64, 64, P, 2, P, P) == SHAPE
    assert v(P, 4, 48, 64, P, 1, P, P) == SHAPE         # K % 32
    assert v(P, 4, 0, 64, P, 1, P, P) == SHAPE
    assert v(P, 4, 64, 32, P, 2, P, P) == SHAPE         # ld < K
    assert v(P, 4, 64, 64, P, 3, P, P) == SHAPE         # n_rblocks not in {1, K/32}
    assert v(P + 2, 4, 64, 64, P, 2, P, P) == ALIGN
    assert v(P, 4, 64, 68, P, 2, P, P) == ALIGN         # row stride not 16-byte aligned
    assert v(P, 4, 64, 64, P, 2, P + 8, P) == ALIGN


def test_validate_gemm(lib):
    v = lib.duqpp_validate_mxfp4_gemm
    assert v(P, P, P, P, 8, 16, 64, P, 0, 16, None, 0, 0) == OK
    assert v(P, P, P, P, 8, 16, 64, P, 1, 16, None, 0, 0) == OK
    assert v(None, P, P, P, 8, 16, 64, P, 0, 16, None, 0, 0) == NULL
    assert v(P, None, P, P, 8, 16, 64, P, 0, 16, None, 0, 0) == NULL
    assert v(P, P, P, P, 8, 16, 64, None, 0, 16, None, 0, 0) == NULL
    assert v(P, P, P, P, 0, 16, 64, P, 0, 16, None, 0, 0) == SHAPE
    assert v(P, P, P, P, 8, 16, 40, P, 0, 16, None, 0, 0) == SHAPE
    assert v(P, P, P, P, 8, 16, 64, P, 0, 8, None, 0, 0) == SHAPE     # ldy < N
    assert v(P, P, P, P, 8, 16, 64, P, 7, 16, None, 0, 0) == DTYPE
    assert v(P, P, P + 4, P, 8, 16, 64, P, 0, 16, None, 0, 0) == ALIGN
    assert v(P, P, P, P, 8, 16, 64, P + 2, 0, 16, None, 0, 0) == ALIGN
    # the fused call needs room for the A-side codes and scales
    need = lib.duqpp_gemm_workspace_bytes(8, 16, 64, 1)
    assert need >= 8 * 32 + 8 * 2
    assert v(P, None, P, P, 8, 16, 64, P, 0, 16, None, 0, 1) == WORKSPACE
    assert v(P, None, P, P, 8, 16, 64, P, 0, 16, P, need - 1, 1) == WORKSPACE
    assert v(P, None, P, P, 8, 16, 64, P, 0, 16, P + 64, need, 1) == ALIGN
    assert v(P, None, P, P, 8, 16, 64, P, 0, 16, P, need, 1) == OK


def test_entry_points_reject_bad_arguments_before_any_launch(lib):
    # these return from the host-side checks, so they are safe without a device
    assert lib.duqpp_rotate_quantize(None, 4, 64, 64, P, 2, P, P, None, None) == NULL
    assert lib.duqpp_quantize_weights(P, 4, 50, 64, P, 2, P, P, None) == SHAPE
    assert lib.duqpp_mxfp4_gemm(P, P, P, P, 8, 16, 64, P, 9, 16, None, 0, None) == DTYPE
    assert lib.duqpp_rotq_gemm(P, 64, P, 2, P, P, 8, 16, 64, P, 0, 16, None, 0, None) == WORKSPACE
    assert lib.duqpp_quantize_f32_dbg(None, 4, 64, 64, P, P, None) == NULL
    assert lib.duqpp_group_error(None, 4, 64, 64, P, 2, P, None, None) == NULL
    assert lib.duqpp_group_error(P, 4, 64, 64, P, 2, None, None, None) == NULL
    assert lib.duqpp_group_error(P, 4, 64, 64, P, 3, P, None, None) == SHAPE      # n_rblocks not in {1, K/32}
    assert lib.duqpp_group_error(P, 4, 48, 64, None, 0, P, None, None) == SHAPE   # K % 32, also without rotation
    assert lib.duqpp_group_error(P, 32 * 65535 + 1, 64, 64, None, 0, P, None, None) == -8   # too many token tiles
    assert lib.duqpp_group_error(P, 4, 64, 68, None, 0, P, None, None) == ALIGN   # row stride not a multiple of 8
    assert lib.duqpp_group_error(P, 4, 64, 64, None, 0, P, P + 4, None) == ALIGN  # mean not 8-byte aligned
    assert lib.duqpp_fold_smoothing(P, 2, None, 64, P, P, None) == NULL
    assert lib.duqpp_fold_smoothing(P, 3, P, 64, P, P, None) == SHAPE      # n_rblocks not in {1, K/32}
    assert lib.duqpp_fold_smoothing(P, 2, P, 48, P, P, None) == SHAPE
    assert lib.duqpp_fold_smoothing(P, 2, P + 2, 64, P, P, None) == ALIGN


def test_kernel_choice_for_the_benchmark_shapes(lib):
    """Host-side rule that picks the GEMM kernel: weight streaming up to 64 tokens, 64 x 128 tiles when there are too
    few 128 x 256 tiles for the chip, 256 x 256 tiles when enough of them make up whole rounds over the 256 CUs."""
    DECODE, SMALL, MID, LARGE = 1, 2, 3, 4
    F32, BF16 = 0, 1
    k = lib.duqpp_gemm_kernel_for
    assert k(64, 4096, 4096, F32) == DECODE                # q_proj reference shape
    assert k(1, 14336, 4096, F32) == DECODE and k(16, 4096, 14336, F32) == DECODE
    assert k(48, 14336, 4096, BF16) == DECODE and k(64, 8192, 28672, F32) == DECODE
    assert k(48, 28672, 8192, BF16) == SMALL and k(32, 28672, 8192, BF16) == DECODE   # 224 tiles of 64 x 128 fill the chip
    assert k(512, 4096, 4096, BF16) == SMALL               # 64 tiles of 128 x 256
    assert k(2048, 4096, 14336, BF16) == MID               # 8B down_proj prefill: 256 tiles of 128 x 256, 128 of 256 x 256
    assert k(8192, 1024, 4096, BF16) == MID                # k / v projections of the layer set
    assert k(4096, 8192, 28672, F32) == LARGE              # 70B down_proj prefill: 512 tiles of 256 x 256
    for N, K in ((4096, 4096), (14336, 4096), (4096, 14336)):
        assert k(8192, N, K, BF16) == LARGE                # q / o, gate / up, down of the layer set
    assert k(8192, 4100, 4096, BF16) == MID                # bf16 rows leave in 16-byte pieces: N must be a multiple of 8
    assert k(8192, 4100, 4096, F32) == MID                 # ... and the fp32 result comes from the same kernel as the bf16 one
    assert k(0, 16, 64, F32) == SHAPE and k(8, 16, 48, F32) == SHAPE and k(8, 16, 64, 7) == DTYPE
    # forcing a kernel goes through the same host-side checks first
    assert lib.duqpp_mxfp4_gemm_tiled_on(9, P, P, P, P, 8, 16, 64, P, 0, 16, None) == SHAPE
    assert lib.duqpp_mxfp4_gemm_tiled_on(DECODE, P, P, P, P, 200, 16, 64, P, 0, 16, None) == SHAPE
    assert lib.duqpp_mxfp4_gemm_tiled_on(LARGE, P, P, P, P, 200, 20, 64, P, 1, 20, None) == SHAPE
    assert lib.duqpp_mxfp4_gemm_tiled_on(MID, None, P, P, P, 200, 16, 64, P, 0, 16, None) == NULL


def test_construct_rotation_host_checks(lib):
    ws = lib.duqpp_construct_rotation_workspace_bytes
    assert ws(0, 4) == 0 and ws(8, -1) == 0 and ws(8, 5000) == 0
    assert ws(100, 128) == 64 + 129 * 256 + 129 * 8192 + 100 * 256
    c = lib.duqpp_construct_rotation
    big = 1 << 30
    assert c(None, 8, 64, 64, P, 2, P, P, None, P, big, None) == NULL
    assert c(P, 8, 64, 64, None, 2, P, P, None, P, big, None) == NULL
    assert c(P, 8, 48, 64, P, 2, P, P, None, P, big, None) == SHAPE
    assert c(P, 8, 64, 64, P, 5000, P, P, None, P, big, None) == SHAPE
    assert c(P, 8, 64, 60, P, 2, P, P, None, P, big, None) == SHAPE           # stride shorter than a row
    assert c(P, 8, 64, 68, P, 2, P, P, None, P, big, None) == ALIGN           # stride not a multiple of 8
    assert c(P, 8, 64, 64, P + 4, 2, P, P, None, P, big, None) == ALIGN
    assert c(P, 8, 64, 64, P, 2, P, P, None, None, 0, None) == WORKSPACE
    assert c(P, 8, 64, 64, P, 2, P, P, None, P, 100, None) == WORKSPACE
    assert c(P, 8, 64, 64, P, 2, P, P, None, P + 16, big, None) == ALIGN


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import importlib

    import paper_2604_17789_amd.binding as b
    monkeypatch.setattr(b, "_HERE", str(tmp_path))
    with pytest.raises(ImportError):
        b._load()
    importlib.reload(b)


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """The boundary is a C ABI: include/duqpp.h compiles as C99 with -pedantic, and a C program linked against
    the library calls its host-side entry points (no device needed)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    lib_dir = os.path.join(ROOT, "paper_2604_17789_amd")
    src = tmp_path / "abi.c"
    calls = ("    typedef void (*fn)(void);\n    fn table[] = {" + ", ".join(f"(fn){name}" for name in _declared_symbols())
             + "};\n    for (i = 0; i < sizeof table / sizeof table[0]; ++i) if (table[i] == 0) return 100;")
    src.write_text(f"""
#include <stdio.h>
#include <string.h>
#include "duqpp.h"
int main(void) {{
    size_t i;
{calls}
    if (strstr(duqpp_version(), "gfx950") == 0) return 1;
    if (duqpp_gemm_workspace_bytes(64, 4096, 4096, 1) == 0) return 2;
    if (duqpp_validate_rotate_quantize((const void*)0, 4, 64, 64, (const float*)0, 2, (const uint8_t*)0, (const uint8_t*)0) != DUQPP_ERR_NULL) return 3;
    if (duqpp_gemm_kernel_for(2048, 4096, 14336, DUQPP_BF16) != DUQPP_GEMM_KERNEL_MID) return 4;
    if (duqpp_construct_rotation_workspace_bytes(8, 2) == 0) return 5;
    printf("%s\\n", duqpp_status_string(DUQPP_ERR_WORKSPACE));
    return 0;
}}
""")
    exe = tmp_path / "abi"
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
           "-L", lib_dir, "-lduqpp", "-Wl,-rpath," + lib_dir, "-Wl,-rpath-link,/opt/rocm/lib", "-o", str(exe)]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    env = dict(os.environ, LD_LIBRARY_PATH="/opt/rocm/lib:" + os.environ.get("LD_LIBRARY_PATH", ""))
    run = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env)
    assert run.returncode == 0, (run.returncode, run.stdout)
    assert "workspace" in run.stdout


def test_bench_refuses_more_than_one_gpu():
    """The bench measures one GPU's share; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True, timeout=300)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr)
    assert "{" not in p.stdout                               # no result line
