"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="kvl.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)            # drop comments
    names = re.findall(r"^\s*(?:const\s+)?[A-Za-z_][\w\s]*?[\s\*]+(kvl_\w+)\s*\(", text, flags=re.M)
    return sorted(set(n for n in names if not n.endswith("_fn")))


def test_header_lists_the_entry_points():
    fns = declared_functions()
    for must in ("kvl_plan", "kvl_pack_layer", "kvl_unpack_layer", "kvl_h2d_unpack_layer", "kvl_stream_layers"):
        assert must in fns
    assert len(fns) >= 15


def test_library_exports_every_declared_symbol():
    from paper_2602_21548_amd import binding as B
    assert os.path.exists(B.LIB_PATH)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in kvl.h but not exported"
    # and the binding wraps exactly the declared set
    assert sorted(B._SIGNATURES) == declared_functions()
    from paper_2602_21548_amd import sched
    for name in declared_functions("kvl_sched.h"):
        assert hasattr(lib, name), f"{name} declared in kvl_sched.h but not exported"
    assert sorted(sched.SIGNATURES) == declared_functions("kvl_sched.h")


def test_strerror_and_versions():
    import paper_2602_21548_amd as K
    assert K.kvl_strerror(0) == "ok"
    for code in (K.KVL_EINVAL, K.KVL_ERANGE, K.KVL_EALIAS, K.KVL_ESPACE, K.KVL_EHIP, K.KVL_ENOMEM, K.KVL_ENOSYS):
        assert K.kvl_strerror(code) not in ("ok", "unknown kvl error")
    assert K.kvl_strerror(-99) == "unknown kvl error"
    assert "gfx950" in K.kvl_version()
    assert K.kvl_variant_name(0) == "default" and K.kvl_variant_name(128) and K.kvl_variant_name(256).startswith("flat")
    assert K.kvl_variant_name(257).startswith("pipe") and K.kvl_variant_name(512) and K.kvl_variant_name(513) is None


def test_struct_sizes_match_the_header():
    from paper_2602_21548_amd import binding as B
    assert ctypes.sizeof(B.kvl_unit_t) == 16
    assert ctypes.sizeof(B.kvl_layout_t) == 40
    assert ctypes.sizeof(B.kvl_request_t) == 24
    assert ctypes.sizeof(B.kvl_chunk_t) == 32
    assert ctypes.sizeof(B.kvl_probe_t) == 16
    assert ctypes.sizeof(B.kvl_tuning_t) == 16


def test_missing_library_fails_loudly():
    """No fallback: if the shared library is absent and cannot be built, importing the binding raises."""
    import subprocess
    import sys
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_2602_21548_amd.build as b\n"
        "b.LIB = '/nonexistent/dir/libkvl.so'\n"
        "b.hipcc = lambda: '/nonexistent/hipcc'\n"
        "try:\n"
        "    import paper_2602_21548_amd.binding\n"
        "except Exception as e:\n"
        "    print('raised', type(e).__name__); sys.exit(7)\n"
        "sys.exit(0)\n" % ROOT)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True)
    assert r.returncode == 7, r.stdout + r.stderr


def test_headers_are_plain_c_and_link_from_c(tmp_path):
    """include/*.h compile as strict C99 and the library can be driven from a C program (no GPU)."""
    import subprocess
    import sysconfig
    import torch
    from paper_2602_21548_amd import binding as B
    exe = str(tmp_path / "c_abi_check")
    libdir = os.path.dirname(B.LIB_PATH)
    torch_lib = os.path.join(os.path.dirname(torch.__file__), "lib")
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I" + os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "host_sanitize", "c_abi_check.c"), "-o", exe,
           "-L" + libdir, "-lkvl", "-Wl,-rpath," + libdir, "-Wl,-rpath," + torch_lib, "-Wl,--allow-shlib-undefined"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0 and "c abi ok" in out.stdout, (out.returncode, out.stdout, out.stderr[-2000:])
