"""The C-ABI library loads and exports every symbol include/tinykg.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tinykg.h")
LIB = os.path.join(ROOT, "paper_2212_04540_amd", "libtinykg.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tinykg_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for want in ("tinykg_quantize", "tinykg_dequantize", "tinykg_kg_aggregate_fwd",
                 "tinykg_kg_aggregate_bwd", "tinykg_graph_create"):
        assert want in names


def test_library_exports_every_declared_symbol():
    assert os.path.exists(LIB), "build the library first: python -m paper_2212_04540_amd.build"
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in tinykg.h but not exported"


def test_binding_lists_the_same_names():
    from paper_2212_04540_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()


def test_host_only_helpers():
    from paper_2212_04540_amd import binding
    assert binding.tinykg_packed_bytes(4096, 64, 2) == 4096 * 16      # 16 B per 64-wide INT2 row
    assert binding.tinykg_packed_bytes(8, 64, 1) == 64
    assert binding.tinykg_num_groups(4096, 64, 64) == 4096
    assert binding.tinykg_num_groups(4096, 64, 256) == 1024
    assert binding.lib().tinykg_status_string(0) == b"ok"
    assert binding.lib().tinykg_status_string(2) == b"shape mismatch"
    # bytes per activation: b/8 + 8/G
    for bits, group in [(2, 64), (4, 128), (8, 64)]:
        n = 1 << 16
        total = binding.tinykg_packed_bytes(n // 64, 64, bits) + 8 * binding.tinykg_num_groups(n // 64, 64, group)
        assert total / n == bits / 8 + 8 / group


def test_argument_errors_need_no_gpu():
    import ctypes as C
    from paper_2212_04540_amd import binding
    L = binding.lib()
    null = C.c_void_p(0)
    fake = C.c_void_p(4096)       # aligned, never dereferenced: the call must fail first
    assert L.tinykg_quantize(fake, 3, 50, 2, 64, 0, fake, fake, fake, null) == 2      # 150 % 64
    assert L.tinykg_quantize(fake, 4, 64, 3, 64, 0, fake, fake, fake, null) == 1      # bits = 3
    assert L.tinykg_quantize(fake, 4, 64, 2, 48, 0, fake, fake, fake, null) == 1      # group = 48
    assert L.tinykg_quantize(null, 4, 64, 2, 64, 0, fake, fake, fake, null) == 1      # null input
    assert L.tinykg_quantize(C.c_void_p(4100), 4, 64, 2, 64, 0, fake, fake, fake, null) == 1  # misaligned
    assert L.tinykg_quantize(fake, -1, 64, 2, 64, 0, fake, fake, fake, null) == 2
    assert L.tinykg_quantize(null, 0, 64, 2, 64, 0, null, null, null, null) == 0      # empty: ok
    assert L.tinykg_quantize_ex(fake, 4, 64, 2, 64, 0, 32, 0, fake, fake, fake, null) == 2  # first_index
    assert L.tinykg_quantize_ex(fake, 4, 64, 2, 64, 0, 0, 7, fake, fake, fake, null) == 1   # rounding
    assert L.tinykg_dequantize(fake, fake, fake, 3, 50, 2, 64, fake, null) == 2
    assert L.tinykg_dequantize(null, null, null, 0, 64, 2, 64, null, null) == 0


def test_bench_refuses_more_than_one_gpu():
    # this build is one GPU: bench.py --gpus N > 1 must say so and exit non-zero (no GPU needed)
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
