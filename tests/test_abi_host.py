"""Host-side checks that need no GPU: the shared library loads, exports every symbol the
header declares, and rejects bad arguments before enqueuing anything."""
import ctypes
import os
import re

import pytest

from paper_2603_05232_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_05232_amd.build import build
        build()
    return binding.load()


def test_header_symbols_are_exported(lib):
    with open(os.path.join(ROOT, "include", "slidesparse.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    declared = set(re.findall(r"\b(\w+)\s*\([^;{]*\)\s*;", text))
    declared -= {"defined"}
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_lifted_k(lib):
    assert binding.slide_lifted_k(512, 4) == 768
    assert binding.slide_lifted_k(3584, 4) == 5376
    assert binding.slide_lifted_k(6144, 3) == 8192
    assert binding.slide_lifted_k(5120, 5) == 8192
    assert binding.slide_lifted_k(64, 2) == 64
    assert binding.slide_lifted_k(100, 4) == 13 * 12         # ceil(100 / 8) blocks (Alg. 1's n_g)
    assert binding.slide_lifted_k(3584, 3) == 598 * 8
    assert binding.slide_lifted_k((1 << 24) + 1, 4) == -1
    assert binding.slide_lifted_k(64, 1) == -1 and binding.slide_lifted_k(64, 9) == -1
    assert binding.slide_lifted_k(0, 4) == -1


def test_lifted_ld(lib):
    # stored width: K' rounded up to whole 128-byte units
    assert binding.slide_lifted_ld(512, 4, "i8") == 768 and binding.slide_lifted_ld(3584, 4, "i8") == 5376
    assert binding.slide_lifted_ld(100, 4, "i8") == 256 and binding.slide_lifted_ld(100, 4, "bf16") == 192
    assert binding.slide_lifted_ld(3584, 3, "fp8") == 4864     # K' = 4784
    assert binding.slide_lifted_ld(6912, 4, "i8") == 10368 and binding.slide_lifted_ld(6912, 5, "i8") == 11136   # K' = 11072 = 86.5 units
    assert binding.slide_lifted_ld(1, 2, "fp16") == 64
    assert binding.slide_lifted_ld(64, 9, "i8") == -1 and binding.slide_lifted_ld(0, 4, "i8") == -1
    assert binding.load().slide_lifted_ld(64, 4, 7) == -1


def test_gemm_workspace_bytes(lib):
    # 64 KiB (128 x 128 partial sums of 4 bytes) per tile and k range; 0 where the k range is not split
    w = binding.slide_gemm_workspace_bytes
    assert w(16, 4608, 5376, "i8") == 0                       # few tokens: weights streamed once
    # ... long rows on few panels (28 panels of 128 channels, 222 units): whole panels in 6 k ranges, also for one token
    assert w(16, 3584, 28416, "i8") == 6 * 112 * 4096 and w(1, 3584, 28416, "i8") == 6 * 112 * 4096
    assert w(8192, 4608, 5376, "i8") == 0                     # enough 256 x 256 tiles
    assert w(128, 4608, 5376, "i8") % (36 * 65536) == 0 and w(128, 4608, 5376, "i8") > 0
    assert w(256, 3584, 28416, "i8") % (56 * 65536) == 0 and w(256, 3584, 28416, "i8") > 0
    assert w(48, 3584, 28416, "fp8") > 0 and w(48, 4608, 5376, "fp8") == 0    # 32 < M <= 64: only long rows
    assert w(128, 4608, 100, "i8") == 0 and w(0, 4608, 5376, "i8") == 0 and w(128, 4608, 5376, "i8") == w(128, 4608, 2688, "bf16")


def test_packed_sizes(lib):
    v, m = binding.slide_packed_sizes(512, 512, 4, "i8")
    assert (v, m) == (512 * 384, 512 * 96)
    v, m = binding.slide_packed_sizes(37888, 3584, 4, "i8")
    assert v + m == int(0.9375 * 37888 * 3584)            # values 0.75x + index 0.1875x of dense bytes
    v, m = binding.slide_packed_sizes(130, 512, 4, "i8")    # rows padded to a multiple of 128
    assert v == 256 * 384
    assert binding.slide_packed_sizes(512, 512, 4, "fp8") == (512 * 384, 512 * 96)
    v, m = binding.slide_packed_sizes(512, 512, 4, "bf16")  # 2-byte values; one 4-byte index word per 16 value bytes
    assert (v, m) == (512 * 384 * 2, 512 * 96 * 2)
    assert binding.slide_packed_sizes(128, 128, 4, "bf16")[0] == 128 * 96 * 2   # K' = 192: 384 lifted bytes per row
    assert binding.slide_packed_sizes(512, 512, 4, "fp16") == (v, m)
    assert binding.slide_packed_sizes(512, 520, 4, "i8") == (512 * 448, 512 * 112)   # K' = 780 stored as 896
    assert binding.slide_packed_sizes(128, 100, 4, "i8") == (128 * 128, 128 * 32)    # partial last block


def test_argument_errors_return_codes(lib):
    vp = ctypes.c_void_p
    one = ctypes.c_void_p(16)                               # non-null, never dereferenced: validation fails first
    # bad N
    assert lib.act_lift_quant(one, 0, 4, 64, 64, 1, 0, one, one, None) == 2
    assert lib.slide_decompose(one, 4, 64, 9, 0, one, one, None, None) == 2
    # ldx < K, output not 16-byte aligned, row too long for on-chip staging
    assert lib.act_lift_quant(one, 0, 4, 64, 32, 4, 0, one, one, None) == 3
    assert lib.act_lift_quant(one, 0, 4, 64, 64, 4, 0, ctypes.c_void_p(8), one, None) == 3
    assert lib.act_lift_quant(one, 0, 4, 65536, 65536, 4, 0, one, one, None) == 3
    # bad dtypes
    assert lib.act_lift_quant(one, 7, 4, 64, 64, 4, 0, one, one, None) == 4
    assert lib.act_lift_quant(one, 0, 4, 64, 64, 4, 5, one, one, None) == 4
    # null pointers
    assert lib.act_lift_quant(None, 0, 4, 64, 64, 4, 0, one, one, None) == 1
    assert lib.act_lift_quant(one, 0, 4, 64, 64, 4, 0, one, None, None) == 1
    assert lib.slide_prune_quant(None, 0, 4, 64, 4, 0, one, one, None) == 1
    assert lib.slide_decompose(None, 128, 512, 4, 0, one, one, None, None) == 1
    assert lib.slide_decompose_canonical(one, 4, 64, 4, 0, None, one, None, None) == 1
    # GEMMs: K' must be a multiple of 128, ldy >= O, pointers non-null and 16-byte aligned
    assert lib.slide_sparse_gemm(one, one, one, one, one, 16, 128, 100, 0, one, 128, None) == 3
    assert lib.dense_gemm(one, one, one, one, 16, 128, 128, 0, one, 64, None) == 3
    assert lib.dense_gemm(None, one, one, one, 16, 128, 128, 0, one, 128, None) == 1
    assert lib.dense_gemm(ctypes.c_void_p(8), one, one, one, 16, 128, 128, 0, one, 128, None) == 3
    assert lib.dense_gemm(one, one, one, one, 16, 128, 128, 9, one, 128, None) == 4
    # bf16 rows are counted in bytes: K = 64 is a whole 128-byte line, K = 32 is not; scales may be NULL only for bf16
    assert lib.dense_gemm(one, None, one, None, 16, 128, 32, 2, one, 128, None) == 3
    assert lib.dense_gemm(one, None, one, None, 16, 128, 128, 0, one, 128, None) == 1
    # workspace variants: unaligned workspace, NULL workspace with a size
    assert lib.dense_gemm_ws(one, one, one, one, 16, 128, 128, 0, one, 128, ctypes.c_void_p(24), 1024, None) == 5
    assert lib.dense_gemm_ws(one, one, one, one, 16, 128, 128, 0, one, 128, None, 1024, None) == 1
    assert lib.slide_sparse_gemm_ws(one, one, one, one, one, 16, 128, 128, 0, one, 128, ctypes.c_void_p(8), 64, None) == 5
    assert lib.slide_sparse_gemm_ws(one, one, one, one, one, 16, 128, 100, 0, one, 128, one, 64, None) == 3
    # fused lifting: 6:8 only, whole 128-byte rows, ldx >= K; workspace rules as above
    assert lib.slide_sparse_gemm_fused(one, one, one, one, one, 16, 128, 128, 128, 3, 0, one, 128, None) == 2
    assert lib.slide_sparse_gemm_fused(one, one, one, one, one, 16, 128, 200, 200, 4, 0, one, 128, None) == 3
    assert lib.slide_sparse_gemm_fused(one, one, one, one, one, 16, 128, 128, 64, 4, 0, one, 128, None) == 3
    assert lib.slide_sparse_gemm_fused(None, one, one, one, one, 16, 128, 128, 128, 4, 0, one, 128, None) == 1
    assert lib.slide_sparse_gemm_fused_ws(one, one, one, one, one, 16, 128, 128, 128, 4, 0, one, 128, ctypes.c_void_p(8), 64, None) == 5
    assert lib.slide_sparse_gemm_fused_ws(one, one, one, one, one, 16, 128, 128, 128, 4, 0, one, 128, None, 64, None) == 1
    assert lib.slide_sparse_gemm_fused_ws(None, None, None, None, None, 0, 128, 128, 128, 4, 0, None, 128, None, 0, None) == 0
    assert lib.slide_decompose_fused(one, 128, 512, 3, 0, one, one, None, None) == 2
    # empty problems are fine and touch nothing
    assert lib.act_lift_quant(None, 0, 0, 64, 64, 4, 0, None, None, None) == 0
    assert lib.dense_gemm(None, None, None, None, 0, 128, 128, 0, None, 128, None) == 0
    assert binding.status_string(0) == "ok" and "N" in binding.status_string(2)
    assert lib.slide_format_version() >= 1


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own (no C++ or HIP types in it)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text('#include "slidesparse.h"\n'
                   'int main(void) { size_t v = 0, m = 0; ss_dtype d = SS_FP16; (void)d;\n'
                   '  return (int)slide_packed_sizes(128, 512, 4, SS_I8, &v, &m) + (int)slide_lifted_ld(512, 4, SS_BF16) * 0; }\n')
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
