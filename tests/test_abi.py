"""The C-ABI library loads and exports every symbol include/wagma.h declares; host-only
argument checks answer without a GPU.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_2005_00124_amd import wagma as libwagma

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(libwagma.LIB_PATH):
        from paper_2005_00124_amd import build
        build.build()
    return libwagma.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "wagma.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wagma_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    names = declared_symbols()
    assert "wagma_step" in names and "wagma_create" in names and len(names) >= 12
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(libwagma.SYMBOLS) == names


def test_header_constants_match_binding():
    text = open(os.path.join(ROOT, "include", "wagma.h")).read()
    for name in ("WAGMA_OK", "WAGMA_EINVAL", "WAGMA_EHIP", "WAGMA_ENOMEM", "WAGMA_MAX_P",
                 "WAGMA_GROUPING_DYNAMIC", "WAGMA_GROUPING_FIXED", "WAGMA_OPT_NONTEMPORAL", "WAGMA_OPT_PLACEMENT",
                 "WAGMA_STATIC_TABLE_BYTES",
                 "WAGMA_PLACE_PLAIN", "WAGMA_PLACE_ARRAYS", "WAGMA_PLACE_CHUNKS", "WAGMA_PLACE_AUTO", "WAGMA_PLACE_SEARCH"):
        value = re.search(r"#define\s+%s\s+\(?(-?\d+)\)?" % name, text).group(1)
        assert int(value) == getattr(libwagma, name), name


def test_debug_switches_are_exported_but_not_in_the_public_header(lib):
    text = open(os.path.join(ROOT, "include", "wagma.h")).read()
    internal = open(os.path.join(ROOT, "paper_2005_00124_amd", "csrc", "wagma_internal.h")).read()
    for name in libwagma.DEBUG_SYMBOLS:
        assert hasattr(lib, name) and name not in text and name in internal
    for name in ("WAGMA_DEBUG_FORCE_STREAM", "WAGMA_DEBUG_STRIPE_LOG2", "WAGMA_DEBUG_XCD_CHUNK_LOG2",
                 "WAGMA_DEBUG_PLACED_SHAPE", "WAGMA_DEBUG_MAP", "WAGMA_DEBUG_PLACED_COOP_SHAPE",
                 "WAGMA_DEBUG_TENSOR_TABLES"):
        value = re.search(r"#define\s+%s\s+(\d+)" % name, internal).group(1)
        assert int(value) == getattr(libwagma, name) and name not in text
    assert lib.wagma_debug_set_option(None, 3, 1) == libwagma.WAGMA_EINVAL
    assert lib.wagma_debug_get_option(None, 3, None) == libwagma.WAGMA_EINVAL


def test_host_side_argument_checks(lib):
    out = ctypes.c_void_p()
    bad = [(6, 2, 10, 1), (8, 3, 10, 1), (4, 8, 10, 1), (0, 1, 10, 1), (2048, 2, 10, 1),
           (4, 2, 0, 1), (4, 2, 10, -1), (4, 0, 10, 1)]
    for P, S, n, tau in bad:
        assert lib.wagma_create(ctypes.byref(out), P, S, n, tau) == libwagma.WAGMA_EINVAL
        assert out.value is None
    assert lib.wagma_create(None, 4, 2, 10, 1) == libwagma.WAGMA_EINVAL
    assert lib.wagma_destroy(None) == libwagma.WAGMA_OK
    assert lib.wagma_row_stride(None) == libwagma.WAGMA_EINVAL
    assert lib.wagma_schedule_period(None) == libwagma.WAGMA_EINVAL
    assert lib.wagma_is_global_iteration(None, 0) == libwagma.WAGMA_EINVAL
    assert lib.wagma_step(None, None, None, None, None, None, 0.1, 0.9, 0, None) == libwagma.WAGMA_EINVAL
    assert lib.wagma_set_option(None, 2, 1) == libwagma.WAGMA_EINVAL
    assert lib.wagma_step_static(4, 2, 16, 0, 16, None, None, None, None, None, 0.1, 0.9, 0, None) == libwagma.WAGMA_EINVAL
    assert lib.wagma_set_grouping(None, 0) == libwagma.WAGMA_EINVAL
    assert lib.wagma_tensors_create(None, None, 1, None, None, None, None, None) == libwagma.WAGMA_EINVAL
    assert lib.wagma_tensors_destroy(None) == libwagma.WAGMA_OK
    assert lib.wagma_step_tensors(None, None, None, 0.1, 0.9, 0, None) == libwagma.WAGMA_EINVAL
    assert lib.wagma_alloc_buffers(None, None, None, None, None) == libwagma.WAGMA_EINVAL
    assert lib.wagma_free_buffers(None) == libwagma.WAGMA_EINVAL
    assert lib.wagma_placement_info(None, None, None, None, None, None, None) == libwagma.WAGMA_EINVAL
    assert lib.wagma_strerror(0) == b"success"
    assert b"invalid" in lib.wagma_strerror(libwagma.WAGMA_EINVAL)
    assert b"unknown" in lib.wagma_strerror(-99)


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(libwagma, "_lib", None)
    monkeypatch.setattr(libwagma, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        libwagma.load()


def test_bench_refuses_more_than_one_gpu():
    """Every box has one GPU and the P workers live in its memory: --gpus N > 1 says so and stops."""
    import subprocess
    import sys
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, cwd=ROOT, timeout=120)
    assert out.returncode != 0 and "ONE GPU" in out.stderr and not out.stdout.strip()


def test_device_code_has_no_packed_fp32_instructions(tmp_path):
    """The kernels are built with packed-fp32 instruction selection switched off; the device
    assembly of our own source must hold none of v_pk_add/mul/fma_f32."""
    import subprocess
    from paper_2005_00124_amd import build
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    text = ""
    for k, source in enumerate(build.SOURCES):
        asm = tmp_path / ("unit%d.s" % k)
        subprocess.run([build.hipcc(), *flags, "--cuda-device-only", "-S", "-o", str(asm), source],
                       check=True, capture_output=True, timeout=600)
        text += asm.read_text()
    assert "step_rows_in_registers" in text and "placement_probe" in text and "global_load_dwordx4" in text
    assert not re.search(r"\bv_pk_(add|mul|fma)_f32\b", text)


def test_header_is_plain_c_and_links_against_the_library(lib, tmp_path):
    """include/wagma.h compiles as strict C99 (no C++ or HIP in the boundary), and a C program
    that names every entry point links against libwagma.so (built here, not run: no GPU)."""
    import subprocess
    names = declared_symbols()
    src = tmp_path / "uses_wagma.c"
    src.write_text('#include "wagma.h"\n#include <stddef.h>\n'
                   "typedef void (*fn)(void);\n"
                   "fn table[] = {\n" + "".join("    (fn)%s,\n" % n for n in names) + "};\n"
                   "int main(void) { return table[0] == NULL; }\n")
    exe = tmp_path / "uses_wagma"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-Wno-cast-function-type",
                    "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src),
                    "-L", os.path.dirname(libwagma.LIB_PATH), "-lwagma",
                    "-Wl,--allow-shlib-undefined"], check=True, timeout=120)
    subprocess.run(["gcc", "-std=c99", "-pedantic-errors", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                    "-x", "c", os.path.join(ROOT, "include", "wagma.h")], check=True, timeout=120)
