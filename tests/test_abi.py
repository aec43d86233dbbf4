"""The C-ABI library loads and exports every symbol include/bc.h declares (no GPU needed)."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header="bc.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bc_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    from paper_2510_13797_amd import bc
    lib = bc.load()                       # raises if libbc.so is missing: no fallback exists
    names = _declared()
    assert "bc_decode_attn" in names and "bc_compress_evict" in names and "bc_prefill_attn" in names
    for n in names:
        assert hasattr(lib, n), n
        assert n in bc.EXPORTS, n
        assert hasattr(bc, n), "python binding lacks %s" % n
    assert sorted(bc.EXPORTS) == names
    assert bc.bc_version() >= 100
    assert bc.bc_status_str(0) == "ok" and "shape" in bc.bc_status_str(-2)
    # the measurement aids live in a library of their own, not in the product library
    diag = bc.load_diag()
    dnames = _declared("bc_diag.h")
    assert dnames == sorted(bc.DIAG_EXPORTS)
    for n in dnames:
        assert hasattr(diag, n) and hasattr(bc, n) and not hasattr(lib, n), n


def test_struct_layouts_match_header():
    import ctypes as C
    from paper_2510_13797_amd import bc
    assert C.sizeof(bc.bc_shape) == 24
    assert bc.bc_shape.scale.offset == 20
    assert C.sizeof(bc.bc_cache) == 104 and bc.bc_cache.max_cap.offset == 72
    assert bc.bc_cache.order.offset == 80
    assert bc.bc_cache.uniform_P.offset == 88 and bc.bc_cache.uniform_cap.offset == 92
    assert bc.bc_cache.rows_per_workgroup.offset == 96 and bc.bc_cache.plan.offset == 100


def test_header_is_plain_c_and_agrees_with_the_binding(tmp_path):
    # compile a C program against include/bc.h with the host C compiler and compare the struct
    # layouts it prints with the ctypes declarations
    import ctypes as C
    import shutil
    import subprocess
    from paper_2510_13797_amd import bc
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        import pytest
        pytest.skip("no host C compiler")
    src = tmp_path / "layout.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "bc.h"\n#include "bc_diag.h"\n'
        'int main(void) {\n'
        '  printf("%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\\n", sizeof(bc_shape), offsetof(bc_shape, scale),\n'
        '         sizeof(bc_cache), offsetof(bc_cache, base), offsetof(bc_cache, err),\n'
        '         offsetof(bc_cache, max_cap), offsetof(bc_cache, order),\n'
        '         offsetof(bc_cache, uniform_P), offsetof(bc_cache, uniform_cap),\n'
        '         offsetof(bc_cache, rows_per_workgroup), offsetof(bc_cache, plan));\n'
        '  return 0;\n}\n')
    exe = tmp_path / "layout"
    subprocess.check_call([cc, "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                           str(src), "-o", str(exe)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    want = [C.sizeof(bc.bc_shape), bc.bc_shape.scale.offset, C.sizeof(bc.bc_cache),
            bc.bc_cache.base.offset, bc.bc_cache.err.offset, bc.bc_cache.max_cap.offset,
            bc.bc_cache.order.offset, bc.bc_cache.uniform_P.offset, bc.bc_cache.uniform_cap.offset,
            bc.bc_cache.rows_per_workgroup.offset, bc.bc_cache.plan.offset]
    assert got == want, (got, want)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2510_13797_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("the CPU oracle", ""), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            src = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2510_13797_amd" not in src and "libbc" not in src, f
