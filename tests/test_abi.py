"""The C-ABI library loads and exports every symbol include/dsk.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dsk.h")).read()
    return re.findall(r"DSK_API\s+[\w\s\*]+?\b(dsk_\w+)\s*\(", text)


def test_header_declares_the_path():
    names = declared_symbols()
    for required in ("dsk_model_create", "dsk_partial_prefill", "dsk_suffix_prefill"):
        assert required in names
    assert len(names) == len(set(names)) >= 10


def test_library_exports_every_declared_symbol():
    from paper_2411_02820_amd import binding as B
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert set(declared_symbols()) == set(B.EXPORTS)


def test_diag_library_exports_what_its_header_declares():
    from paper_2411_02820_amd import diag
    text = open(os.path.join(ROOT, "include", "dsk_diag.h")).read()
    names = re.findall(r"DSK_DIAG_API\s+[\w\s\*]+?\b(dsk_\w+)\s*\(", text)
    lib = ctypes.CDLL(diag.LIB_PATH)
    assert names and set(names) == set(diag.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name


def test_error_strings_without_gpu():
    from paper_2411_02820_amd import binding as B
    assert B.lib.dsk_strerror(B.DSK_OK) == b"ok"
    assert B.lib.dsk_strerror(B.DSK_EINVAL) == b"invalid argument"
    # null arguments are rejected before any device call
    assert B.lib.dsk_model_create(None, 1, 1, None) == B.DSK_EINVAL
    assert B.lib.dsk_partial_prefill(None, None, 0, 0, 0, None, None, None, None, 0, None) == B.DSK_EINVAL


def test_binding_declares_the_argument_types_of_every_export():
    # without argtypes ctypes passes a Python int as a 32-bit C int: a device pointer would arrive truncated
    from paper_2411_02820_amd import binding as B
    text = open(os.path.join(ROOT, "include", "dsk.h")).read()
    for name in B.EXPORTS:
        fn = getattr(B.lib, name)
        assert fn.argtypes is not None, name
        decl = re.search(r"\b" + name + r"\s*\(([^;]*?)\)\s*;", text, re.S).group(1)
        n_params = 0 if decl.strip() in ("", "void") else decl.count(",") + 1
        assert len(fn.argtypes) == n_params, (name, len(fn.argtypes), n_params)


def test_header_is_valid_c_and_the_c_demo_compiles():
    # the boundary is a C ABI: the header must compile as plain C (not only as C++), and so must the demo that uses it
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    assert gcc, "gcc is part of the toolchain this build expects"
    inc = os.path.join(ROOT, "include")
    for hdr in ("dsk.h", "dsk_diag.h"):
        r = subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", "-I", inc, "-"],
                           input=f'#include "{hdr}"\nint main(void) {{ return 0; }}\n', capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
    rocm_inc = "/opt/rocm/include"
    if os.path.isdir(rocm_inc):
        demo = os.path.join(ROOT, "paper_2411_02820_amd", "examples", "c_abi_demo.c")
        r = subprocess.run([gcc, "-std=c11", "-Wall", "-fsyntax-only", "-D__HIP_PLATFORM_AMD__", "-I", rocm_inc, "-I", inc, demo],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
