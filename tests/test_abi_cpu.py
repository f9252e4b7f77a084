"""Host-side checks that need no GPU: the C-ABI library loads and exports every symbol that
include/ozdgemm.h declares; the calls that do not touch a device behave."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2511_13778_amd import ozdgemm as g
    if not os.path.exists(g.LIB_PATH):
        from paper_2511_13778_amd.build import build_library
        build_library(verbose=False)
    return g, g.load_library()


def declared_functions(header="ozdgemm.h", prefix="oz_"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(%s[a-z0-9_]+)\s*\(" % prefix, text)))


def test_every_declared_symbol_is_exported(lib):
    g, dll = lib
    names = declared_functions()
    assert set(names) == set(g.EXPORTS), names
    for name in names:
        assert getattr(dll, name) is not None


def test_every_header_has_its_library(lib):
    # every header under include/ is covered by one of the two symbol checks
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["ozdgemm.h", "ozprobe.h"]


def test_probe_library_exports_its_header(lib):
    from paper_2511_13778_amd import ozprobe as p
    dll = p.load_library()
    names = declared_functions("ozprobe.h", "ozp_")
    assert set(names) == set(p.EXPORTS), names
    for name in names:
        assert getattr(dll, name) is not None
    # argument errors are reported without touching a device
    assert dll.ozp_launch_mfma_i8(None, None, None, 1, 1) == 1
    assert dll.ozp_launch_copy(None, None, None, 16) == 1
    assert dll.ozp_launch_read(None, None, 0, None) == 1


def test_struct_sizes_match_header(lib):
    g, _ = lib
    assert C.sizeof(g.oz_opts_t) == 28
    assert C.sizeof(g.oz_result_t) == 40 == 4 * g.RESULT_INT32_WORDS
    assert C.sizeof(g.oz_heuristic_t) == 32
    assert C.sizeof(g.oz_layout_t) == 6 * 8 + 9 * C.sizeof(C.c_size_t)


def test_host_only_calls(lib):
    g, dll = lib
    o = g.oz_opts_t()
    dll.oz_default_opts(C.byref(o))
    assert (o.mode, o.target_bits, o.max_bits, o.slices, o.esc_block, o.heuristic, o.tile_slices) == (0, 53, 200, 0, 0, 1, 1)
    assert dll.oz_status_string(0) == b"ok"
    assert b"workspace" in dll.oz_status_string(2)
    # null handle / null pointers are argument errors, not crashes
    assert dll.oz_destroy(None) == 1
    assert dll.oz_create(None, 0) == 1
    assert dll.oz_dgemm_workspace_bytes(None, b"N", b"N", 8, 8, 8, C.byref(o)) == 0
    assert dll.oz_profile_enable(None, 4) == 1


def test_no_cpu_fallback_in_binding():
    # the product path must not import the oracle
    for name in ("ozdgemm.py", "ozprobe.py", "qr.py", "build.py", "workloads.py", "__init__.py"):
        src = open(os.path.join(ROOT, "paper_2511_13778_amd", name)).read()
        assert "oracle" not in src.replace("CPU oracle's tests", ""), name


def test_only_the_allowed_places_use_the_oracle():
    # the oracle is test infrastructure: besides tests/, only smoke() and bench.py's cpu_baseline leg import it
    import ast
    def oracle_imports(path):
        tree = ast.parse(open(path).read())
        hits = []
        for node in ast.walk(tree):
            if isinstance(node, ast.ImportFrom) and (node.module or "").split(".")[0] == "oracle":
                hits.append(node.lineno)
            if isinstance(node, ast.Import) and any(a.name.split(".")[0] == "oracle" for a in node.names):
                hits.append(node.lineno)
        return hits
    for folder in ("experiments", "paper_2511_13778_amd"):
        for name in sorted(os.listdir(os.path.join(ROOT, folder))):
            if name.endswith(".py"):
                assert oracle_imports(os.path.join(ROOT, folder, name)) == [], (folder, name)
    # bench.py: only inside cpu_baseline; __graft_entry__.py: only inside smoke
    for fname, func in (("bench.py", "cpu_baseline"), ("__graft_entry__.py", "smoke")):
        tree = ast.parse(open(os.path.join(ROOT, fname)).read())
        allowed = set()
        for node in tree.body:
            if isinstance(node, ast.FunctionDef) and node.name == func:
                allowed = {n.lineno for n in ast.walk(node) if isinstance(n, (ast.Import, ast.ImportFrom))}
        assert set(oracle_imports(os.path.join(ROOT, fname))) <= allowed, fname
    # and the oracle never reaches for the product
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith(".py"):
            src = open(os.path.join(ROOT, "oracle", name)).read()
            assert "paper_2511_13778_amd" not in src and "ctypes" not in src, name


def test_headers_are_plain_c_and_struct_layouts_match_the_binding(tmp_path):
    # the boundary is a C ABI: both headers must compile as C99 on their own, and the structs the Python
    # binding mirrors must have the sizes and field offsets the C compiler gives them
    import ctypes as C
    import subprocess
    from paper_2511_13778_amd import ozdgemm as g
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "abi.c"
    src.write_text(r'''
#include <stdio.h>
#include <stddef.h>
#include "ozdgemm.h"
#include "ozprobe.h"
int main(void) {
    printf("opts %zu %zu %zu\n", sizeof(oz_opts_t), offsetof(oz_opts_t, esc_block), offsetof(oz_opts_t, tile_slices));
    printf("result %zu %zu %zu\n", sizeof(oz_result_t), offsetof(oz_result_t, slices_min), offsetof(oz_result_t, pair_tiles));
    printf("heur %zu %zu\n", sizeof(oz_heuristic_t), offsetof(oz_heuristic_t, fixed_ns));
    printf("layout %zu %zu %zu %zu\n", sizeof(oz_layout_t), offsetof(oz_layout_t, nkb), offsetof(oz_layout_t, off_T),
           offsetof(oz_layout_t, total_bytes));
    printf("consts %d %d %u\n", OZ_NUM_STAGES, OZ_BATCH_LANES, (unsigned)OZ_STATIC_SCRATCH_BYTES);
    return 0;
}
''')
    exe = tmp_path / "abi"
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(root, "include"), str(src), "-o", str(exe)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    out = dict((ln.split()[0], [int(v) for v in ln.split()[1:]]) for ln in subprocess.run([str(exe)], capture_output=True, text=True).stdout.splitlines())
    assert out["opts"] == [C.sizeof(g.oz_opts_t), g.oz_opts_t.esc_block.offset, g.oz_opts_t.tile_slices.offset]
    assert out["result"] == [C.sizeof(g.oz_result_t), g.oz_result_t.slices_min.offset, g.oz_result_t.pair_tiles.offset]
    assert out["heur"] == [C.sizeof(g.oz_heuristic_t), g.oz_heuristic_t.fixed_ns.offset]
    assert out["layout"] == [C.sizeof(g.oz_layout_t), g.oz_layout_t.nkb.offset, g.oz_layout_t.off_T.offset,
                             g.oz_layout_t.total_bytes.offset]
    assert out["consts"] == [g.OZ_NUM_STAGES, 4, 256 << 20]
