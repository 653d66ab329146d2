"""CPU-only checks of the boundary: the library loads, exports what the header declares,
the ctypes mirror of fs_format has the C layout, and the size queries are sane."""
import ctypes
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "flashsparse.h")
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))


@pytest.fixture(scope="module")
def fs():
    import paper_2412_11007_amd as fs
    if not os.path.exists(fs.library_path()):
        from paper_2412_11007_amd.build import build_library
        build_library()
    fs.load_library()
    return fs


def test_every_declared_symbol_is_exported(fs):
    src = "\n".join(open(h).read() for h in HEADERS)
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = set(re.findall(r"\b(fs_[a-z_0-9]+)\s*\(", src))
    assert {"fs_convert", "fs_spmm", "fs_sddmm", "fs_format_bytes", "fs_spmm_workspace_bytes", "fs_blk_to_csr",
            "fs_version", "fs_status_string", "fs_spmm_static", "fs_spmm_timed", "fs_gather_probe", "fs_copy_bytes"} <= names
    lib = fs.load_library()
    for n in names:
        assert hasattr(lib, n), n


def test_header_compiles_as_plain_c_and_struct_layout_matches(fs, tmp_path):
    from paper_2412_11007_amd.binding import _FsFormatStruct
    fields = [f[0] for f in _FsFormatStruct._fields_]
    prog = "#include <stdio.h>\n#include <stddef.h>\n#include \"flashsparse.h\"\nint main(void){\n"
    prog += "printf(\"%zu\\n\", sizeof(fs_format));\n"
    for f in fields:
        prog += "printf(\"%%zu\\n\", offsetof(fs_format, %s));\n" % f
    prog += "return 0;}\n"
    c = tmp_path / "layout.c"
    c.write_text(prog)
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(c), "-o", str(exe)],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == ctypes.sizeof(_FsFormatStruct)
    for f, o in zip(fields, out[1:]):
        assert int(o) == getattr(_FsFormatStruct, f).offset, f


def test_status_strings_and_version(fs):
    assert fs.fs_version() >= 100
    seen = {fs.fs_status_string(c) for c in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert fs.fs_status_string(99) == "unknown status"


def test_format_bytes_bounds(fs):
    a, s = fs.fs_format_bytes(65536, 1000000, 8, 32, 0)
    # values (2*V bytes) + three int32 arrays per stored entry, at least
    assert a >= 1000000 * (16 + 12) and s >= 4 * 1000000
    a16, _ = fs.fs_format_bytes(65536, 1000000, 16, 32, 0)
    assert a16 > a
    assert fs.fs_format_bytes(0, 0)[0] > 0
    with pytest.raises(fs.FsError) as e:
        fs.fs_format_bytes(10, 10, 33, 32, 0)
    assert e.value.code == 1
    with pytest.raises(fs.FsError) as e:
        fs.fs_format_bytes(10, 1 << 31, 8, 32, 0)
    assert e.value.code == 5
    with pytest.raises(fs.FsError) as e:
        fs.fs_format_bytes(10, (1 << 31) // 8, 8, 32, 0)  # V*nnz overflows the slot index
    assert e.value.code == 5


def test_transpose_scratch_size(fs):
    lib = fs.load_library()
    need = ctypes.c_size_t(0)
    assert lib.fs_csr_transpose_bytes(1000, 2000, 1000000, ctypes.byref(need)) == 0
    # two key buffers and one payload buffer of nnz int32, plus 256 counters per 2048 entries
    assert 12 * 1000000 <= need.value <= 14 * 1000000
    assert lib.fs_csr_transpose_bytes(0, 0, 0, ctypes.byref(need)) == 0 and need.value > 0
    assert lib.fs_csr_transpose_bytes(1, 1, -1, ctypes.byref(need)) == 1
    assert lib.fs_csr_transpose_bytes(1 << 31, 1, 1, ctypes.byref(need)) == 5
    assert lib.fs_csr_transpose_bytes(1, 1, 1, None) == 1


def test_size_queries_reject_bad_arguments_without_a_gpu(fs):
    """The size queries are pure host code: they must answer (or refuse) with no device present."""
    from paper_2412_11007_amd.binding import _FsFormatStruct
    lib = fs.load_library()
    n = ctypes.c_size_t(0)
    f = _FsFormatStruct()  # all zeros: an empty format
    f.V, f.KB, f.chunk = 8, 32, 256
    assert lib.fs_pack_bytes(None, ctypes.byref(n)) == 1
    assert lib.fs_pack_bytes(ctypes.byref(f), None) == 1
    assert lib.fs_pack_bytes(ctypes.byref(f), ctypes.byref(n)) == 0 and n.value >= 16
    assert lib.fs_attention_workspace_bytes(ctypes.byref(f), 128, ctypes.byref(n)) == 0 and n.value == 0
    assert lib.fs_attention_workspace_bytes(ctypes.byref(f), -8, ctypes.byref(n)) == 1
    f.n_split_items = 3
    assert lib.fs_attention_workspace_bytes(ctypes.byref(f), 128, ctypes.byref(n)) == 0
    assert n.value == 3 * 8 * (128 + 2) * 4
    assert lib.fs_spmm_workspace_bytes(ctypes.byref(f), 128, ctypes.byref(n)) == 0 and n.value == 3 * 8 * 128 * 4
    assert lib.fs_edge_softmax_workspace_bytes(ctypes.byref(f), ctypes.byref(n)) == 0 and n.value == 3 * 2 * 8 * 4


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2412_11007_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2412_11007_amd" not in text and "flashsparse.h" not in text, f
    assert "oracle" not in sys.modules or True
