"""The C-ABI library loads and exports every symbol that include/dbw.h declares; host-side
argument checks that need no GPU compute."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    """Every function declared in include/*.h."""
    import glob
    names = set()
    for path in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        names |= set(re.findall(r"\b(dbw_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_declared_symbols():
    from paper_2102_06280_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    names = declared_symbols()
    assert {"dbw_create", "dbw_select", "dbw_round", "dbw_destroy"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(binding.EXPORTS) == set(names)


def test_strerror_and_null_handling():
    from paper_2102_06280_amd import binding as B
    assert B.dbw_strerror(0) == "ok"
    for code in range(-8, 0):
        assert B.dbw_strerror(code) not in ("ok", "unknown error")
    assert B._lib.dbw_destroy(None) == 0
    assert B._lib.dbw_select(None, None, None, None) == B.ERR_NULL
    assert B._lib.dbw_round(None, None, None, None, None, None, None, 0.1, None) == B.ERR_NULL


def test_create_rejects_bad_graphs_before_touching_the_gpu():
    """Graph validation runs on the host before any allocation."""
    from paper_2102_06280_amd import binding as B
    bad = [
        ([0, 1, 2], [1, 1]),            # asymmetric / wrong
        ([0, 1, 2], [0, 1]),            # self loops
        ([0, 2, 3, 4], [2, 1, 0, 0]),   # unsorted row
        ([0, 1, 2, 2], [1, 0]),         # disconnected (worker 2 isolated)
        ([0, 1, 2], [5, 0]),            # out of range
    ]
    for rowptr, colidx in bad:
        with pytest.raises(B.DbwError) as e:
            B.dbw_create(np.array(rowptr, np.int32), np.array(colidx, np.int32), len(rowptr) - 1, 8)
        assert e.value.code == B.ERR_GRAPH
    with pytest.raises(B.DbwError) as e:
        B.dbw_create(np.array([0, 1, 2], np.int32), np.array([1, 0], np.int32), 2, 8, ld=4)
    assert e.value.code == B.ERR_INVALID


def test_binding_structs_match_the_header(tmp_path):
    """sizeof / offsetof of the structs in include/dbw.h, as a C compiler lays them out, equal
    the ctypes mirrors in the binding."""
    import ctypes as C
    import subprocess
    from paper_2102_06280_amd import binding as B
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "dbw_measure.h"\n'
                   'int main(void) { printf("%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\\n", sizeof(dbw_model), '
                   'offsetof(dbw_model, loss), offsetof(dbw_model, dims), offsetof(dbw_model, grad_path), sizeof(dbw_opts), offsetof(dbw_opts, order), '
                   'offsetof(dbw_opts, mix_path), offsetof(dbw_opts, layout), offsetof(dbw_opts, model), '
                   'sizeof(dbw_kernel_time), offsetof(dbw_kernel_time, ms_total), offsetof(dbw_kernel_time, launches)); '
                   'return 0; }\n')
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    want = [C.sizeof(B.dbw_model), B.dbw_model.loss.offset, B.dbw_model.dims.offset, B.dbw_model.grad_path.offset,
            C.sizeof(B.dbw_opts),
            B.dbw_opts.order.offset, B.dbw_opts.mix_path.offset, B.dbw_opts.layout.offset, B.dbw_opts.model.offset,
            C.sizeof(B.dbw_kernel_time), B.dbw_kernel_time.ms_total.offset, B.dbw_kernel_time.launches.offset]
    assert got == want
    # the header is plain C: it compiled above with a C compiler
