"""The C-ABI library loads without a GPU and exports every symbol include/hbp.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_in_header():
    header = open(os.path.join(ROOT, "include", "hbp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    return set(re.findall(r"\b(hbp_[a-z_0-9]+)\s*\(", header))


def _exported_by_library(path):
    """The hbp_* functions in the library's dynamic symbol table (what a C caller can link against)."""
    import subprocess
    out = subprocess.check_output(["nm", "-D", "--defined-only", path]).decode()
    names = set()
    for line in out.splitlines():
        parts = line.split()
        if len(parts) >= 3 and parts[1] in ("T", "W") and parts[2].startswith("hbp_"):
            names.add(parts[2].split("@")[0])
    return names


def test_header_symbols_are_exported():
    import paper_2504_08860_amd as H
    if not os.path.exists(H.LIB_PATH):
        from paper_2504_08860_amd.build import build_library
        build_library()
    lib = ctypes.CDLL(H.LIB_PATH)
    declared = _declared_in_header()
    assert declared == set(H.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name
    # and nothing else: every extern "C" hbp_* entry point of the built library is declared in the header
    assert _exported_by_library(H.LIB_PATH) == declared


def test_host_only_calls():
    import paper_2504_08860_amd as H
    p = H.hbp_default_params()
    assert (p.rows_per_block, p.cols_per_block, p.group_width) == (0, 0, 64)   # block sizes chosen from the matrix, wave64
    assert H.hbp_status_string(0) == "ok" and "column" in H.hbp_status_string(-3)
    assert H.lib().hbp_free(None) == 0
    assert H.lib().hbp_get_info(None, None) == -1
    assert H.lib().hbp_build(None, None, None, 1, 1, None, None, None) == -1
    assert ctypes.sizeof(H.hbp_params_t) == 64


def test_struct_layout_matches_header(tmp_path):
    """The ctypes mirrors of hbp_params_t / hbp_info_t have the C compiler's sizes and offsets."""
    import subprocess
    import paper_2504_08860_amd as H
    src = tmp_path / "layout.c"
    fields_p = [f[0] for f in H.hbp_params_t._fields_]
    fields_i = [f[0] for f in H.hbp_info_t._fields_]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "hbp.h"', 'int main(void){',
             'printf("%zu %zu\\n", sizeof(hbp_params_t), sizeof(hbp_info_t));']
    lines += [f'printf("%zu\\n", offsetof(hbp_params_t, {f}));' for f in fields_p]
    lines += [f'printf("%zu\\n", offsetof(hbp_info_t, {f}));' for f in fields_i]
    lines += ['return 0;}']
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I" + os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    out = subprocess.check_output([str(exe)]).decode().split()
    assert [int(out[0]), int(out[1])] == [ctypes.sizeof(H.hbp_params_t), ctypes.sizeof(H.hbp_info_t)]
    want = [getattr(H.hbp_params_t, f).offset for f in fields_p] + [getattr(H.hbp_info_t, f).offset for f in fields_i]
    assert [int(v) for v in out[2:]] == want
