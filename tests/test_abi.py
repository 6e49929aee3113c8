"""The C-ABI library loads without a GPU and exports every function the headers under include/ declare."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    import glob
    text = "".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ejoin_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2508_21230_amd as pkg
    lib = pkg.load_library()
    names = declared_functions()
    assert len(names) >= 12 and "ejoin_selfjoin_pairs" in names and "ejoin_selfjoin_count" in names
    for name in names:
        assert hasattr(lib, name), f"{name} declared under include/ but not exported"


def test_host_only_entry_points():
    import paper_2508_21230_amd as pkg
    lib = pkg.load_library()
    assert lib.ejoin_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert len(lib.ejoin_strerror(code)) > 0
    # upper-triangular 256 x 256 tiles, diagonal included
    assert pkg.tiles_evaluated(1) == 1 and pkg.tiles_evaluated(256) == 1 and pkg.tiles_evaluated(257) == 3
    assert pkg.tiles_evaluated(1_000_000) == 3907 * 3908 // 2
    assert pkg.tiles_evaluated(0) == 0
    # argument checks that need no device
    assert lib.ejoin_create(None, 0) == -1
    assert lib.ejoin_destroy(None) == -1
    assert lib.ejoin_set_profiling(None, 1) == -1


def test_binding_refuses_to_run_without_a_gpu():
    import pytest
    import torch
    import paper_2508_21230_amd as pkg
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    with pytest.raises(pkg.EJoinError):
        pkg.EJoin(0)


def test_header_is_plain_c(tmp_path):
    """include/ejoin.h compiles as C89-with-stdint and as C++ and declares the same prototypes the library was built from."""
    import shutil
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "ejoin_bench.h"\n'
                   "int use(void) { ejoin_ctx* c = 0; int st = 0; return ejoin_status(c, &st) + (int)ejoin_tiles_evaluated(1) + EJOIN_OK; }\n")
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", inc, "-c", str(src), "-o", str(tmp_path / "a.o")], check=True)
    if shutil.which("g++"):
        cpp = tmp_path / "use_header.cpp"
        cpp.write_text(src.read_text())
        subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-I", inc, "-c", str(cpp), "-o", str(tmp_path / "b.o")], check=True)
