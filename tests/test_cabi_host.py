"""CPU-side checks of the C-ABI library: it loads, exports every symbol include/nz.h declares, and its pure
host functions (bounds, workspace sizes, argument checks that need no GPU) behave.  No compute call is made."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def nz():
    from paper_2605_12396_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_12396_amd import build
        build.build()
    binding.lib()
    return binding


def test_exports_every_declared_symbol(nz):
    inc = os.path.join(ROOT, "include")
    hdr = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(nz_[a-z_]+)\s*\(", hdr))
    assert {"nz_compress", "nz_decompress", "nz_reduce_frames", "nz_reduce_local", "nz_compress_bound", "nz_workspace_bytes",
            "nz_reduce_workspace_bytes", "nz_version", "nz_trace_events", "nz_trace_recorded"} <= names
    L = nz.lib()
    for n in names:
        assert hasattr(L, n), n
    assert L.nz_version() >> 16 == 1


def test_struct_layouts_match_header(nz):
    assert C.sizeof(nz.Opts) == 32 == C.sizeof(oracle.Opts) and nz.RESULT_BYTES == 32 == C.sizeof(oracle.Result)


def test_compress_bound_equals_oracle_bound(nz):
    for n in (1, 37, 16384, 100000, (1 << 20) + 1, 1 << 26):
        for kw in (dict(), dict(chunk_elems=16384), dict(chunk_elems=1000, force_codec=2), dict(chunk_elems=1 << 20),
                   dict(alphabet=1024, force_codec=2)):
            assert nz.nz_compress_bound(n, nz.make_opts(**kw)) == oracle.compress_bound(n, oracle.make_opts(**kw))
    assert nz.nz_compress_bound(0) == 0
    assert nz.nz_compress_bound(100, nz.make_opts(alphabet=3)) == 0
    assert nz.nz_compress_bound(100, nz.make_opts(seg_syms=64)) == 0       # the HIP build decodes 256-symbol segments
    assert nz.nz_compress_bound(100, nz.make_opts(chunk_elems=(1 << 20) + 1)) == 0


def test_workspace_sizes(nz):
    n = 1 << 26
    w = nz.nz_workspace_bytes(n)
    wr = nz.nz_reduce_workspace_bytes(n)
    assert 0 < w < 32 << 20                      # per-frame tables and partial histograms only
    # operand A and the sums, each staged as 16-bit codes with a 32-bit spill array
    assert wr >= 12 * n and wr < 12 * n + (32 << 20)
    assert nz.nz_workspace_bytes(0) == 0


def test_missing_library_fails_loudly(nz, monkeypatch, tmp_path):
    from paper_2605_12396_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        binding.lib()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_12396_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src and "nz_oracle" not in src, f


def test_public_headers_are_plain_c_and_agree_with_the_bindings(tmp_path):
    """include/*.h must compile as C99 on their own (no HIP or C++ types in the boundary), and the structures the
    Python bindings mirror must have the sizes the C compiler gives them."""
    import ctypes as C
    import subprocess
    import oracle
    from paper_2605_12396_amd import binding as nz
    src = tmp_path / "h.c"
    src.write_text('#include "nz.h"\n#include "nz_trace.h"\n#include <stdio.h>\n'
                   'int main(void) { printf("%zu %zu %zu %zu\\n", sizeof(nz_opts), sizeof(nz_result), sizeof(nz_rea_opts), '
                   'sizeof(nz_rea_result)); return 0; }\n')
    exe = tmp_path / "h"
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-o", str(exe), str(src)], check=True)
    sizes = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert sizes == [C.sizeof(nz.Opts), nz.RESULT_BYTES, C.sizeof(nz.ReaOpts), nz.REA_RESULT_BYTES]
    assert sizes == [C.sizeof(oracle.Opts), C.sizeof(oracle.Result), C.sizeof(oracle.ReaOpts), C.sizeof(oracle.ReaResult)]
