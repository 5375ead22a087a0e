"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

import paper_2510_18586_amd as K
from paper_2510_18586_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


HEADERS = ("tokencake_kv.h", "tokencake_kv_bench.h")


def _declared_functions(headers=HEADERS):
    names = []
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(tc_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_header_declares_the_expected_calls():
    names = _declared_functions(("tokencake_kv.h",))
    # the serving boundary carries no measurement helper
    for helper in ("tc_copy_contiguous", "tc_copy_via_lds", "tc_hbm_stream", "tc_naive_transfer", "tc_hbm_write",
                   "tc_hbm_read", "tc_stage_on_device"):
        assert helper not in names and helper in _declared_functions(("tokencake_kv_bench.h",))
    for must in ("tc_create", "tc_destroy", "tc_alloc", "tc_free", "tc_offload", "tc_upload",
                 "tc_offload_batch", "tc_upload_batch", "tc_poll", "tc_sync", "tc_stats"):
        assert must in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(K.library_path()) if os.path.exists(K.library_path()) else binding._load()
    for name in _declared_functions():
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"


def test_binding_covers_every_declared_symbol():
    for name in _declared_functions():
        assert hasattr(K, name), f"the Python binding lacks {name}"


def test_error_strings_and_struct_layout():
    assert K.tc_strerror(K.TC_OK) == "ok"
    for code in range(-9, 0):
        assert K.tc_strerror(code) and "unknown" not in K.tc_strerror(code)
    assert "unknown" in K.tc_strerror(-99)
    # the ctypes mirrors must match the C layout (checked against sizes the compiler would give)
    assert ctypes.sizeof(K.tc_pool_desc) == 40
    assert ctypes.sizeof(K.tc_opts) == 56
    assert ctypes.sizeof(K.tc_xfer_desc) == 32
    assert ctypes.sizeof(K.tc_gate_input) == 40 and ctypes.sizeof(K.tc_upload_cand) == 24
    assert ctypes.sizeof(K.tc_index_hit) == 24
    assert ctypes.sizeof(K.tc_stats_t) == 24 + 16 + 48 + 32 + 16 + 24 + 48 + 8 + 8


def test_null_arguments_are_rejected_without_a_gpu():
    lib = binding._load()
    assert lib.tc_create(None, None, None) == K.TC_ERR_INVAL
    assert K.tc_sync(None) == K.TC_ERR_INVAL
    # descriptions that are refused before any device call: 2^31 work items in one launch, bad options
    assert K.tc_create(0x1000, None, 64, 1 << 24, 32768, 16)[0] == K.TC_ERR_INVAL
    assert K.tc_create(0x1000, None, 1 << 19, 4096, 16, 1)[0] == K.TC_ERR_INVAL
    assert K.tc_create(0x1000, None, 2, 16, 4096, 16, direct_offload=4)[0] == K.TC_ERR_INVAL
    assert K.tc_create(0x1000, None, 2, 16, 4096, 16, direct_upload=2)[0] == K.TC_ERR_INVAL
    assert K.tc_create(0x1000, None, 2, 16, 4096, 16, overlap_kernels=2)[0] == K.TC_ERR_INVAL
    assert K.tc_create(0x1010, None, 2, 16, 4096, 16)[0] == K.TC_ERR_INVAL          # base not 256-B aligned
    assert K.tc_create(0x1000, None, 2, 16, 4100, 16)[0] == K.TC_ERR_INVAL          # page not a multiple of 16
    assert K.tc_destroy(None) == K.TC_OK
    assert K.tc_record_bytes(None) == 0


def test_header_is_plain_c_and_cxx(tmp_path):
    """The boundary is a C header: it must compile on its own as C11 and as C++17, warnings as errors."""
    import subprocess
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "use_header.c"
    src.write_text('#include "tokencake_kv.h"\n#include "tokencake_kv_bench.h"\nint main(void) { tc_pool_desc d; tc_opts o; (void)d; (void)o; return TC_OK; }\n')
    subprocess.run(["gcc", "-std=c11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    subprocess.run(["g++", "-std=c++17", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)],
                   check=True)


def test_a_plain_c_program_links_and_runs(tmp_path):
    """tests/csrc/abi_smoke.c, built with gcc against the shared library, runs its host-only calls."""
    import subprocess
    lib = K.library_path()
    exe = str(tmp_path / "abi_smoke")
    libdir = os.path.dirname(lib)
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "csrc", "abi_smoke.c"), "-o", exe,
                    "-L", libdir, "-ltokencake_kv", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib",
                    "-Wl,--allow-shlib-undefined"], check=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0 and out.stdout.strip() == "ok", (out.returncode, out.stdout, out.stderr)
