"""CPU-only checks of the C ABI: the library loads, exports what include/ecq.h declares, and
its host-side helpers and argument checks behave as documented (no kernel is launched)."""
import ctypes as C
import os
import re

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def E():
    import paper_1806_08054_amd as E
    if not os.path.exists(E.library_path()):
        from paper_1806_08054_amd import build
        build.build()
    return E


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ecq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ecq_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(E):
    names = declared_symbols()
    assert {"ecq_quantize", "ecq_error_update", "ecq_dequant_aggregate", "ecq_quantize_update"} <= set(names)
    lib = E.lib()
    for name in names:
        assert hasattr(lib, name), name
    assert lib.ecq_version() >= 100


def test_size_helpers_match_the_cost_formula(E):
    """r = ceil(log2(2s+1)), row = ceil(N r / 8) bytes (Section 4, cost paragraph)."""
    for s in range(1, 128):
        assert E.code_bits(s) == oracle.code_bits(s)
    for n, s in [(1, 1), (3, 1), (4096, 1), (25_557_032, 1), (1_048_576, 3), (61_100_840, 7), (5, 127)]:
        assert E.row_bytes(n, s) == oracle.row_bytes(n, s) == (n * E.code_bits(s) + 7) // 8
    assert E.num_buckets(25_557_032, 512) == 49_917
    assert E.num_buckets(138_357_544, 8192) == 16_890
    for bad in (0, -1, 128):
        with pytest.raises(E.EcqError):
            E.code_bits(bad)
    with pytest.raises(E.EcqError):
        E.num_buckets(100, 12)


def test_check_shape_status_codes(E):
    lib = E.lib()

    def st(**kw):
        sh = E.Shape.packed(4096, 4, 512, 1)
        for k, v in kw.items():
            setattr(sh, k, v)
        return lib.ecq_check_shape(C.byref(sh))

    assert st() == 0
    assert lib.ecq_check_shape(None) == -1
    assert st(n=0) == -2 and st(n=(1 << 34) + 1, gh_stride=(1 << 34) + 4) == -2 and st(workers=0) == -2
    assert st(s=0) == -3 and st(s=128) == -3
    assert st(bucket=0) == -4 and st(bucket=20) == -4 and st(bucket=-8) == -4
    assert st(gh_stride=4095) == -5 and st(gh_stride=4098) == -5
    assert st(code_stride=1020) == -5 and st(code_stride=1026) == -5
    assert st(scale_stride=7) == -5
    assert st(norm=1) == 0 and st(norm=3) == -8 and st(norm=-1) == -8
    for code in range(0, -9, -1):
        assert E.status_string(code) != "unknown status"
    assert E.status_string(-99) == "unknown status"


def test_entry_points_reject_bad_arguments_before_any_launch(E):
    """NULL pointers and bad scalars are refused on the host (nothing is enqueued)."""
    lib = E.lib()
    sh = E.Shape.packed(4096, 4, 512, 1)
    assert lib.ecq_quantize_update(C.byref(sh), None, None, 1.0, 1.0, 1, 0, None, None, None) == -1
    assert lib.ecq_quantize(C.byref(sh), None, None, 1.0, 1, 0, None, None, None) == -1
    assert lib.ecq_error_update(C.byref(sh), None, None, None, 1.0, None, None) == -1
    assert lib.ecq_dequant_aggregate(C.byref(sh), None, None, None, None) == -1
    assert lib.ecq_philox_words(1, 0, 0, 0, 16, None, None) == -1
    assert lib.ecq_calib_add(None, None, None, 16, None) == -1
    assert lib.ecq_calib_gather(C.byref(sh), None, None, None) == -1
    fake = C.c_void_p(0x1000)
    assert lib.ecq_quantize_update(C.byref(sh), fake, fake, -1.0, 1.0, 1, 0, fake, fake, None) == -8
    assert lib.ecq_quantize_update(C.byref(sh), fake, fake, 1.0, 2.0, 1, 0, fake, fake, None) == -8
    assert lib.ecq_quantize_update(C.byref(sh), C.c_void_p(0x1004), fake, 1.0, 1.0, 1, 0, fake, fake, None) == -6
    l2_bad = E.Shape.packed(4096, 4, 24, 1, norm=1)        # buckets are multiples of 8 for either norm
    l2_bad.bucket = 20
    assert lib.ecq_quantize_update(C.byref(l2_bad), fake, fake, 1.0, 1.0, 1, 0, fake, fake, None) == -4
    assert lib.ecq_huffman_build(2, 1, None, 3, None, None, None) == -1
    assert lib.ecq_huffman_build(2, 1, fake, 2, fake, fake, None) == -5
    assert lib.ecq_huffman_build(0, 1, fake, 3, fake, fake, None) == -2
    assert lib.ecq_huffman_build(2, 200, fake, 3, fake, fake, None) == -3
    assert lib.ecq_huffman_encode(C.byref(sh), fake, fake, fake, 3, fake, 1024, fake, 4, None) == -5   # 4 tiles + 1
    assert lib.ecq_huffman_encode(C.byref(sh), fake, fake, fake, 3, fake, 1020, fake, 5, None) == -5
    assert lib.ecq_huffman_encode(C.byref(sh), fake, fake, fake, 2, fake, 1024, fake, 5, None) == -5
    assert lib.ecq_huffman_encode(C.byref(sh), fake, fake, fake, 3, None, 1024, fake, 5, None) == -1
    assert lib.ecq_huffman_decode(C.byref(sh), fake, 1024, C.c_void_p(0x1004), 5, fake, fake, 3, fake, None) == -6
    tiles = C.c_int64(0)
    assert lib.ecq_huffman_num_tiles(4097, C.byref(tiles)) == 0 and tiles.value == 5
    tu = E.Tuning(1, 3, 0, 0)
    assert lib.ecq_quantize_update_ex(C.byref(sh), fake, fake, 1.0, 1.0, 1, 0, fake, fake, C.byref(tu), None) == -8


def test_header_is_plain_c_and_the_library_links_from_c(E, tmp_path):
    """include/ecq.h compiles as C99 and as C++ without warnings, and a C program linked against
    the library gets the documented answers from its host-side helpers."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    inc = os.path.join(ROOT, "include")
    src = os.path.join(ROOT, "tests", "abi_check.c")
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, src],
                   check=True)
    gxx = shutil.which("g++")
    if gxx:
        subprocess.run([gxx, "-std=c++11", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc,
                        os.path.join(inc, "ecq.h")], check=True)
    libdir = os.path.dirname(E.library_path())
    exe = str(tmp_path / "abi_check")
    subprocess.run([gcc, "-std=c99", "-I", inc, src, "-o", exe, "-L", libdir, "-lecq", "-Wl,-rpath," + libdir,
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split("\n")
    n, r = 25557032, 2
    tiles = (n + 4095) // 4096
    assert out[:10] == [
        "code_bits 2 4 8",
        f"row_bytes 0 {(n * r + 7) // 8}",
        f"num_buckets 0 {(n + 511) // 512}",
        "check_shape 0",
        "check_shape_bad_bucket 1",
        "zrun_symbols 0 31 249",
        f"zrun_num_tiles 0 {tiles} {(tiles + 63) // 64}",
        f"zrun_stream_bytes 0 {((n * 2 + tiles * 2 * 127 + 7) // 8 + 3) // 4 * 4}",
        "null_pointer 1",
        "status_string text",
    ], out


def test_no_cpu_fallback_in_the_product():
    """The package never imports the oracle (or anything else that could stand in for the
    kernels)."""
    pkg = os.path.join(ROOT, "paper_1806_08054_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
