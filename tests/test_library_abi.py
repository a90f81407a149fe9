"""CPU-side checks of the C ABI: the library loads, exports what include/atomo.h and include/atomo_bench.h
declare, and the host-side argument validation answers without touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_1806_04090_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header="atomo.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(atomo_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_symbols()
    assert {"atomo_encode_svd", "atomo_encode_entrywise", "atomo_probabilities", "atomo_decode"} <= set(names)
    bench = declared_symbols("atomo_bench.h")
    assert {"atomo_profile_enable", "atomo_profile_read", "atomo_measure_mfma_fp32", "atomo_last_counters"} == set(bench)
    assert not set(bench) & set(names)                       # the method's header holds no measurement call
    L = binding.lib()
    for name in names + bench:
        assert hasattr(L, name), name


def test_strerror_and_null_arguments():
    L = binding.lib()
    assert L.atomo_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert L.atomo_strerror(code) not in (b"ok", b"unknown status")
    assert L.atomo_create(None, 0) == binding.ATOMO_EINVAL
    assert L.atomo_destroy(None) == binding.ATOMO_EINVAL
    assert L.atomo_reserve(None, 10) == binding.ATOMO_EINVAL
    assert L.atomo_status(None, None, None) == binding.ATOMO_EINVAL
    offs = (C.c_int64 * 2)(0, 4)
    assert L.atomo_probabilities(None, None, offs, 1, 1.0, None, None) == binding.ATOMO_EINVAL
    assert L.atomo_encode_svd(None, None, 1, 1.0, 0, 0, None, None, None, None, None) == binding.ATOMO_EINVAL
    assert L.atomo_encode_entrywise(None, None, 1.0, 0, 0, None, None, None) == binding.ATOMO_EINVAL
    assert L.atomo_decode(None, 0, None, 1, 1.0, None, 0, None) == binding.ATOMO_EINVAL


def test_workspace_queries_are_host_only():
    L = binding.lib()
    mats = (binding.atomo_mat * 2)(binding.atomo_mat(512, 4608, 4608, None), binding.atomo_mat(64, 27, 27, None))
    nbytes = C.c_size_t(0)
    assert L.atomo_svd_workspace_bytes(mats, 2, C.byref(nbytes)) == 0
    assert nbytes.value > 512 * (4608 + 512) * 4
    bad = (binding.atomo_mat * 1)(binding.atomo_mat(4096, 4096, 4096, None))
    assert L.atomo_svd_workspace_bytes(bad, 1, C.byref(nbytes)) == binding.ATOMO_EINVAL
    assert L.atomo_entrywise_workspace_bytes(11_173_962, C.byref(nbytes)) == 0
    assert nbytes.value > 70_000
    assert L.atomo_entrywise_workspace_bytes(0, C.byref(nbytes)) == binding.ATOMO_EINVAL
    assert L.atomo_entrywise_workspace_bytes(1 << 32, C.byref(nbytes)) == binding.ATOMO_EINVAL


def test_no_fallback_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    with pytest.raises(RuntimeError):
        binding.Context(0)


def test_struct_layouts_match_the_header(tmp_path):
    """The ctypes mirrors in the binding against include/atomo.h as the host C compiler lays it out."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no host C compiler")
    structs = [binding.atomo_mat, binding.atomo_svd_msg, binding.atomo_ew_msg, binding.atomo_lq_msg,
               binding.atomo_svd_options]
    lines = ["#include <stdio.h>", "#include <stddef.h>", '#include "atomo.h"', "int main(void) {"]
    for st in structs:
        lines.append(f'  printf("{st.__name__} size %zu\\n", sizeof({st.__name__}));')
        for name, _ in st._fields_:
            lines.append(f'  printf("{st.__name__} {name} %zu\\n", offsetof({st.__name__}, {name}));')
    lines += ["  return 0;", "}"]
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run([cc, "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    seen = {}
    for line in out:
        if line:
            st, field, value = line.split()
            seen[(st, field)] = int(value)
    for st in structs:
        assert seen[(st.__name__, "size")] == C.sizeof(st), st.__name__
        for name, _ in st._fields_:
            assert seen[(st.__name__, name)] == getattr(st, name).offset, (st.__name__, name)
    # and the header declares no field that the binding leaves out
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "atomo.h")).read(), flags=re.S)
    for st in structs:
        body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (st.__name__, st.__name__), text, flags=re.S).group(1)
        declared = [part.replace("*", " ").split()[-1] for stmt in body.split(";") if stmt.strip()
                    for part in stmt.split(",")]
        assert declared == [name for name, _ in st._fields_], st.__name__
