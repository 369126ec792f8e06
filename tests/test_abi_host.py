"""Host-side checks of the C ABI that need no GPU: the library loads and exports what the header
declares.  No compute call is made here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "harp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(harp_[a-z0-9_]+)\s*\(", text)))


def _library():
    from paper_2509_24859_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_library()
    return ctypes.CDLL(binding.LIB_PATH)


def test_every_declared_symbol_is_exported():
    lib = _library()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n


def test_binding_lists_the_same_symbols():
    from paper_2509_24859_amd import binding
    assert sorted(binding.EXPORTS) == _declared()


def test_tables_bytes_rejects_malformed_headers():
    from paper_2509_24859_amd import binding
    lib = binding.load_library()
    tp = (ctypes.c_int32 * 2)(1, 2)
    good = dict(L=8, T=2, G=2, M=4, ar_count=4, flags=0, n_tp=2)

    def size(**kw):
        f = dict(good, **kw)
        p = binding.harp_problem(f["L"], f["T"], f["G"], f["M"], f["ar_count"], f["flags"],
                                 f["n_tp"], ctypes.addressof(tp))
        return lib.harp_tables_bytes(ctypes.byref(p))

    assert size() > 0
    for bad in (dict(L=0), dict(T=0), dict(G=0), dict(M=0), dict(ar_count=-1), dict(flags=1),
                dict(n_tp=0), dict(n_tp=9)):
        assert size(**bad) == 0, bad
    tp[0] = 2
    assert size() == 0                  # first degree must be 1
    tp[0], tp[1] = 1, 1
    assert size() == 0                  # degrees must rise
    assert lib.harp_tables_bytes(None) == 0


def test_null_context_is_refused_without_touching_the_gpu():
    from paper_2509_24859_amd import binding
    lib = binding.load_library()
    assert lib.harp_set_plan_path(None, 0) == binding.ERR_INVALID_ARG
    assert lib.harp_tables_finalize(None, None) == binding.ERR_INVALID_ARG
    assert lib.harp_last_error(None) == b"null context"
    assert lib.harp_create(None, 0) == binding.ERR_INVALID_ARG


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2509_24859_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "harp_oracle" not in text, f


def test_header_is_plain_c99(tmp_path):
    """The boundary is a C interface: the header must compile as strict C99 with no warnings, and a
    C translation unit must be able to name every struct in it by value."""
    import subprocess
    src = tmp_path / "uses_header.c"
    src.write_text('#include "harp.h"\n'
                   "int main(void) {\n"
                   "    harp_problem p; harp_candidates c; harp_plans o; harp_orderings g;\n"
                   "    (void)p; (void)c; (void)o; (void)g;\n"
                   "    return (int)(sizeof(p) + sizeof(c) + sizeof(o) + sizeof(g)) == 0;\n"
                   "}\n")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                        "-I", os.path.join(ROOT, "include"), "-fsyntax-only", str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_a_c_program_links_and_calls_the_library(tmp_path):
    """A plain C translation unit, compiled with gcc, links against the shared library and calls
    entry points that need no GPU (argument checks and the table-size query)."""
    import subprocess
    from paper_2509_24859_amd import binding
    _library()
    src = tmp_path / "client.c"
    src.write_text('#include <stdio.h>\n#include "harp.h"\n'
                   "int main(void) {\n"
                   "    int32_t tp[2] = {1, 2};\n"
                   "    harp_problem p = {0};\n"
                   "    p.L = 8; p.T = 2; p.G = 2; p.M = 4; p.ar_count = 4; p.n_tp = 2; p.tp_degrees = tp;\n"
                   '    printf("%zu %d %s\\n", harp_tables_bytes(&p), harp_set_plan_path(NULL, 0), harp_last_error(NULL));\n'
                   "    p.L = 0;\n"
                   '    printf("%zu\\n", harp_tables_bytes(&p));\n'
                   "    return 0;\n"
                   "}\n")
    exe = tmp_path / "client"
    libdir = os.path.dirname(binding.LIB_PATH)
    libname = os.path.basename(binding.LIB_PATH)
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
                        "-o", str(exe), "-L", libdir, "-l:" + libname, "-Wl,-rpath," + libdir,
                        "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    first, second = r.stdout.strip().splitlines()
    size, rc, msg = first.split(" ", 2)
    assert int(size) > 0 and int(rc) == binding.ERR_INVALID_ARG and msg == "null context"
    assert int(second) == 0


def test_the_c_only_client_builds_against_the_library(tmp_path):
    """tests/c_client/plan_tiny.c drives the hot path through the C ABI and the HIP runtime's C
    interface alone (no Python, no torch).  Here it is compiled and linked with gcc; on a GPU machine it
    prints "0 2 4 4 20 0" for the hand example and exits 0."""
    import subprocess
    from paper_2509_24859_amd import binding
    _library()
    if not os.path.exists("/opt/rocm/include/hip/hip_runtime_api.h"):
        pytest.skip("no ROCm headers on this machine")
    libdir, libname = os.path.dirname(binding.LIB_PATH), os.path.basename(binding.LIB_PATH)
    exe = tmp_path / "plan_tiny"
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
                        os.path.join(ROOT, "tests", "c_client", "plan_tiny.c"), "-o", str(exe), "-L", libdir,
                        "-l:" + libname, "-L", "/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath," + libdir,
                        "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    assert exe.exists()


def test_recorded_counters_belong_to_the_current_kernel_sources():
    """bench.py quotes HBM traffic and issued instructions from the rocprofv3 record in profiles/ only
    while the record's hash of the planner kernel sources matches the tree; a source edit without a
    new counter run would silently turn those fields into null."""
    import json
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    with open(bench.COUNTER_FILE) as f:
        rec = json.load(f)
    assert rec["workload"] == "stress"
    assert rec["kernel_source_hash"] == bench.kernel_source_hash()
    traffic, issued = bench.counter_figures("stress", True)
    assert 0.28e9 < traffic < 1.5e9                # above the algorithmic bytes, within the budget set for it
    assert 0.5 < issued["k2_fast_valu_issue_utilisation"] <= 1.0
    assert bench.counter_figures("tiny", True) == (None, None)       # another workload: nothing to quote
    assert bench.counter_figures("stress", False) == (None, None)    # part of the batch: nothing to quote


def test_recorded_table_build_counters_belong_to_the_current_kernel_source():
    """The same for the table build: its HBM traffic is quoted from profiles/ only for the length the
    counters were taken at and while k1_tables.hip is unchanged."""
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    traffic = bench.tables_traffic(1 << 20)
    assert traffic is not None and 1.317e9 < traffic < 1.7e9      # above the algorithmic bytes, one re-read of the inputs
    assert bench.tables_traffic(1 << 19) is None
