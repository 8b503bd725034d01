"""The C-ABI library loads and exports every symbol the header declares; host-side argument
validation fails cleanly without a GPU (no compute is launched here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in sorted(os.listdir(os.path.join(ROOT, "include"))) if n.endswith(".h")]


@pytest.fixture(scope="module")
def lib():
    import paper_1709_03708_amd as pq

    if not os.path.exists(pq.lib_path()):
        from paper_1709_03708_amd import build

        build.build()
    return pq.load()


def _declared():
    src = "".join(open(h).read() for h in HEADERS)
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pqkm_[a-z_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert {"pqkm_build_tables", "pqkm_assign", "pqkm_update", "pqkm_fit", "pqkm_workspace_bytes",
            "pqkm_status_string", "pqkm_set_option", "pqkm_profile_read", "pqkm_fit_until",
            "pqkm_fit_until_workspace_bytes", "pqkm_encode", "pqkm_decode", "pqkm_update_naive"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings(lib):
    seen = {lib.pqkm_status_string(i).decode() for i in range(6)}
    assert len(seen) == 6 and "ok" in seen
    assert lib.pqkm_status_string(99).decode() == "unknown status"


def test_workspace_bytes_is_host_arithmetic(lib):
    import paper_1709_03708_amd as pq

    assert pq.workspace_bytes(10, 0, 5) == 0 and pq.workspace_bytes(-1, 4, 5) == 0 and pq.workspace_bytes(1, 4, 0) == 0
    # M = 4: one 128 KB tile image per 32 centers + histogram + counts
    b = pq.workspace_bytes(10**6, 4, 1000)
    assert b >= 32 * 131072 + 1000 * 4 * 256 * 4 + 1000 * 4
    assert b % 256 == 0
    # config 5: 4 bytes per code of sorted indices and 4 of ranks inside the clusters, two copies of the tile
    # images, one launch of regrouped codes
    assert 8 * 10**9 <= pq.workspace_bytes(10**9, 4, 10**5) < 10 * 2**30
    assert pq.fit_until_workspace_bytes(10**6, 4, 1000) >= b + 8 * 10**6
    # a generic M needs no tile images
    assert pq.workspace_bytes(100, 5, 10) < 131072


def test_bad_arguments_are_rejected_before_any_gpu_work(lib):
    vp = ctypes.c_void_p
    one = vp(256)        # a non-NULL, aligned dummy address; never dereferenced on these paths
    null = vp(0)
    OK, NULL, SHAPE, WS = 0, 1, 2, 3
    assert lib.pqkm_assign(one, 10, 4, null, 5, one, one, null, one, 1 << 30, null) == NULL
    assert lib.pqkm_assign(one, 10, 4, one, 5, null, one, null, one, 1 << 30, null) == NULL
    assert lib.pqkm_assign(null, 10, 4, one, 5, one, one, null, one, 1 << 30, null) == NULL
    assert lib.pqkm_assign(one, -1, 4, one, 5, one, one, null, one, 1 << 30, null) == SHAPE
    assert lib.pqkm_assign(one, 10, 0, one, 5, one, one, null, one, 1 << 30, null) == SHAPE
    assert lib.pqkm_assign(one, 10, 65, one, 5, one, one, null, one, 1 << 30, null) == SHAPE
    assert lib.pqkm_assign(one, 10, 4, one, 0, one, one, null, one, 1 << 30, null) == SHAPE
    assert lib.pqkm_assign(one, 10, 4, one, 5, one, one, null, null, 1 << 30, null) == WS
    assert lib.pqkm_assign(one, 10, 4, one, 5, one, one, null, one, 16, null) == WS
    assert lib.pqkm_assign(one, 10, 4, one, 5, one, one, null, vp(260), 1 << 30, null) == WS
    assert lib.pqkm_update(one, 10, 4, null, 5, one, one, null, null, one, 1 << 30, null) == NULL
    assert lib.pqkm_update(one, 10, 4, one, 5, one, null, null, null, one, 1 << 30, null) == NULL
    assert lib.pqkm_update(one, 10, 4, one, 5, one, one, null, null, one, 8, null) == WS
    assert lib.pqkm_fit(one, 10, 4, one, 5, one, -1, one, null, null, one, 1 << 30, null) == SHAPE
    assert lib.pqkm_fit(one, 10, 4, null, 5, one, 1, one, null, null, one, 1 << 30, null) == NULL
    lib.pqkm_fit_until.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, vp, ctypes.c_int32, vp, vp,
                                   vp, vp, vp, vp, ctypes.c_size_t, vp]
    assert lib.pqkm_fit_until(one, 10, 4, one, 5, one, -1, one, null, null, null, null, one, 1 << 30, null) == SHAPE
    assert lib.pqkm_fit_until(one, 10, 4, null, 5, one, 3, one, null, null, null, null, one, 1 << 30, null) == NULL
    assert lib.pqkm_fit_until(one, 10, 4, one, 5, one, 3, one, null, null, null, null, one, 64, null) == WS
    for f in (lib.pqkm_encode, lib.pqkm_decode):
        f.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, vp, vp, vp]
        f.restype = ctypes.c_int
        assert f(one, 10, 0, 32, one, one, null) == SHAPE
        assert f(one, 10, 4, 0, one, one, null) == SHAPE
        assert f(one, -1, 4, 32, one, one, null) == SHAPE
        assert f(one, 10, 4, 32, null, one, null) == NULL
        assert f(null, 10, 4, 32, one, one, null) == NULL
    assert lib.pqkm_build_tables(null, 4, 32, one, null) == NULL
    assert lib.pqkm_build_tables(one, 4, 0, one, null) == SHAPE
    assert lib.pqkm_build_tables(one, 0, 32, one, null) == SHAPE
    assert lib.pqkm_set_option(b"no_such_option", 1) == SHAPE
    assert lib.pqkm_set_option(b"assign_kernel", 7) == SHAPE
    assert lib.pqkm_set_option(b"assign_kernel", 0) == OK
    assert lib.pqkm_set_option(None, 0) == NULL


def test_binding_fails_loudly_without_the_library(monkeypatch):
    import paper_1709_03708_amd.binding as b

    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libpqkm.so")
    with pytest.raises(ImportError):
        b.load()


def test_microbenchmark_library_loads_and_rejects_bad_arguments():
    """The measurement library behind `bench.py --microbench` (not part of the method): it loads, exports its one
    entry point, and refuses null outputs before touching a device."""
    from paper_1709_03708_amd import build

    if not os.path.exists(build.MICROBENCH_LIB):
        build.build()
    import torch  # noqa: F401  (its HIP runtime first, as in the binding: a process must not end up with two)
    mb = ctypes.CDLL(build.MICROBENCH_LIB)
    mb.pqkm_microbench.restype = ctypes.c_int
    mb.pqkm_microbench.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
    assert mb.pqkm_microbench(0, None, None) == 1


def test_header_is_plain_c_and_a_c_program_links(lib, tmp_path):
    """include/pqkm.h compiles as strict C99 and as C++, and a C caller links against libpqkm.so (argument
    checks only: nothing here touches a GPU)."""
    import shutil
    import subprocess

    from paper_1709_03708_amd.binding import lib_path

    gcc = shutil.which("gcc")
    gxx = shutil.which("g++")
    if gcc is None or gxx is None:
        pytest.skip("no host C/C++ compiler")
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "caller.c"
    src.write_text(
        '#include "pqkm.h"\n'
        "#include <stdio.h>\n"
        "int main(void) {\n"
        "    /* invalid shapes and NULL pointers are rejected on the host, before any HIP call */\n"
        "    if (pqkm_workspace_bytes(-1, 4, 10) != 0) return 1;\n"
        "    if (pqkm_workspace_bytes(1000, 4, 10) == 0) return 2;\n"
        "    if (pqkm_assign(NULL, -1, 4, NULL, 10, NULL, NULL, NULL, NULL, 0, NULL) != PQKM_ERR_SHAPE) return 3;\n"
        "    if (pqkm_assign(NULL, 10, 4, NULL, 10, NULL, NULL, NULL, NULL, 0, NULL) != PQKM_ERR_NULL) return 4;\n"
        '    printf("%s\\n", pqkm_status_string(PQKM_OK));\n'
        "    return 0;\n"
        "}\n")
    exe = tmp_path / "caller"
    libdir = os.path.dirname(lib_path())
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe),
                    "-L", libdir, "-lpqkm", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True)
    assert out.stdout.strip() == "ok"
    cpp = tmp_path / "caller.cpp"
    cpp.write_text('#include "pqkm.h"\nint main() { return pqkm_workspace_bytes(-1, 4, 10) == 0 ? 0 : 1; }\n')
    subprocess.run([gxx, "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(cpp)], check=True)
