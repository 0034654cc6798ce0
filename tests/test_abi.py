"""The C-ABI library loads and exports every symbol that include/lkv.h declares.  No GPU needed."""
import os
import re

from paper_2605_06676_amd import lkv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "lkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lkv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = lkv.load_library()
    names = _declared()
    assert set(names) == set(lkv.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_calls_that_need_no_gpu():
    lib = lkv.load_library()
    assert b"gfx950" in lib.lkv_version()
    # workspace sizing is host arithmetic: one slot per segment plus one per chunk of packed rows,
    # (128 + 2) floats per query head of the group; it must at least hold one slot per segment
    n = lkv.lkv_decode_workspace_bytes(256, 1258291, 32, 8)
    assert n % 256 == 0 and n >= 256 * 4 * 130 * 4
    assert n <= (256 + 1258291 // 128 + 1) * 4 * 130 * 4 + 256
    assert lkv.lkv_decode_workspace_bytes(256, 0, 32, 8) >= 256 * 4 * 130 * 4
    assert lkv.lkv_decode_workspace_bytes(-1, 10, 32, 8) == 0
    # the backward pass of the training-time attention keeps one float per query row and, when the key-side
    # kernel is split by query head (grouped heads, short sequences), partial dK, dV and dm per query head
    d_only = 32 * 16384 * 4
    assert lkv.lkv_masked_attn_backward_workspace_bytes(32, 32, 16384) == d_only        # no groups: never split
    n = lkv.lkv_masked_attn_backward_workspace_bytes(32, 8, 4096)
    assert n in (32 * 4096 * 4, 32 * 4096 * 4 * (1 + 2 * 128 + 1))
    assert lkv.lkv_masked_attn_backward_workspace_bytes(3, 3, 5) == 256                 # rounded up to 256 bytes
    assert lkv.lkv_masked_attn_backward_workspace_bytes(0, 1, 5) == 0
    assert lkv.lkv_masked_attn_backward_workspace_bytes(4, 3, 5) == 0                   # 4 query heads, 3 KV heads
    # calls that need a context refuse a null one without touching the GPU
    assert lib.lkv_masked_attn_forward(None, 4, 2, 8, 128, None, None, None, None, 1.0, None, None, None) == 1
    assert lib.lkv_last_error(None) == b"context is NULL"


def test_header_is_plain_c_and_links_from_c(tmp_path):
    # the header must compile as strict C99 and as C++; a C client built against it links with the library and runs
    import subprocess

    inc = os.path.join(ROOT, "include")
    hdr = os.path.join(inc, "lkv.h")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", hdr], check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", hdr], check=True)
    lkv.load_library()                                    # raises if the library has not been built
    libdir = os.path.dirname(lkv.LIB_PATH)
    exe = str(tmp_path / "c_abi_check")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", inc, os.path.join(ROOT, "tests", "c_abi_check.c"),
                    "-L", libdir, "-llkv", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True)
    assert "c abi ok" in out.stdout


def test_missing_library_is_an_error_not_a_fallback(tmp_path):
    # the binding has no CPU route: without the built library it raises, in a fresh interpreter so that the
    # library already loaded by this process plays no part
    import subprocess
    import sys

    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2605_06676_amd import lkv\n"
            "try:\n"
            "    lkv.load_library()\n"
            "except FileNotFoundError as e:\n"
            "    print('raised:', e)\n"
            "else:\n"
            "    print('loaded')\n") % ROOT
    env = dict(os.environ, LKV_LIBRARY=str(tmp_path / "no_such_liblkv.so"))
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, check=True).stdout
    assert out.startswith("raised:") and "no_such_liblkv.so" in out
