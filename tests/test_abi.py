"""The C-ABI library loads without a GPU and exports every function the public header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hcspmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hcspmm_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_named_entry_points():
    names = declared_functions()
    for must in ("hcspmm_prepare", "hcspmm_spmm", "hcspmm_gcn_layer"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import paper_2412_08902_amd.binding as hc
    lib = hc.load_library()
    names = declared_functions()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(hc.EXPORTED_SYMBOLS) == names


def test_host_only_calls():
    import paper_2412_08902_amd.binding as hc
    assert hc.hcspmm_version() >= 100
    o = hc.hcspmm_default_options()
    assert o.struct_size == ctypes.sizeof(hc.HcspmmOptions) and o.window_rows == 16 and o.route_mode == 0
    for dt in (hc.HCSPMM_F32, hc.HCSPMM_BF16, hc.HCSPMM_F16):
        for d in (0, 16, 32, 64, 128, 602):
            for nnz in (0, 10 ** 6, 10 ** 8):
                c = hc.hcspmm_default_selector(dt, d, nnz)
                assert len(c) == 3 and c[0] >= 0 and c[1] >= 0 and c[2] < 0  # monotone in the paper's directions
    lib = hc.load_library()
    assert lib.hcspmm_status_string(0) == b"ok"
    assert lib.hcspmm_status_string(2) == b"invalid CSR"
    # argument errors that are detected before any device work
    out = ctypes.c_void_p()
    st = lib.hcspmm_prepare(-1, 4, 0, None, None, None, None, None, ctypes.byref(out))
    assert st == hc.HCSPMM_EINVAL and out.value is None
    st = lib.hcspmm_prepare(4, 1 << 27, 0, ctypes.c_void_p(16), None, None, None, None, ctypes.byref(out))
    assert st == hc.HCSPMM_EUNSUPPORTED
    assert b"2^27" in lib.hcspmm_last_error()
    assert lib.hcspmm_spmm(None, None, 0, 4, 0, None, 0, 0, None) == hc.HCSPMM_EINVAL
    assert lib.hcspmm_gcn_layer(None, None, 0, 4, None, 0, 4, None, 0, 1, None, 0, None) == hc.HCSPMM_EINVAL
    assert lib.hcspmm_gcn_workspace_bytes(None, 4, 4) == 0
    lib.hcspmm_plan_destroy(None)


def test_header_is_plain_c(tmp_path):
    """The public header must compile as C (no C++ constructs, no HIP or torch types) and link against the library."""
    import shutil
    import subprocess
    import paper_2412_08902_amd.binding as hc
    gcc = shutil.which("gcc")
    assert gcc, "gcc is part of the image"
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include "hcspmm.h"\n'
        "#include <stdio.h>\n"
        "int main(void) {\n"
        "    hcspmm_options o;\n"
        "    hcspmm_default_options(&o);\n"
        "    hcspmm_plan* plan = NULL;\n"
        "    hcspmm_status st = hcspmm_prepare(-1, 1, 0, NULL, NULL, NULL, &o, NULL, &plan);\n"
        "    size_t ws = hcspmm_layer_backward_workspace_bytes(NULL, 4, 4);\n"
        '    printf("%d %d %s %d\\n", (int)st, (int)ws, hcspmm_status_string(st), (int)hcspmm_version());\n'
        "    return (st == HCSPMM_EINVAL && plan == NULL && ws == 0) ? 0 : 1;\n"
        "}\n")
    exe = tmp_path / "use_header"
    lib_dir = os.path.dirname(hc.LIB_PATH)
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src), "-o",
                        str(exe), "-L", lib_dir, "-lhcspmm", "-Wl,-rpath," + lib_dir], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, (r.stdout, r.stderr)
    assert r.stdout.split()[0] == "1"


def test_new_entry_points_reject_bad_arguments_on_the_host():
    import paper_2412_08902_amd.binding as hc
    lib = hc.load_library()
    assert lib.hcspmm_layer_backward(None, None, 0, 4, None, 0, None, 0, 4, None, 0, None, 0, None, 0, 0, None, 0, None) == hc.HCSPMM_EINVAL
    assert lib.hcspmm_aggregate_update(None, None, 0, 4, 0, None, 0, 4, None, 0, 0, 1, None, 0, None) == hc.HCSPMM_EINVAL
    assert lib.hcspmm_gcn_layer_ex(None, None, 0, 4, None, 0, 4, None, 0, 0, 1, 0, None, 0, None) == hc.HCSPMM_EINVAL
    assert lib.hcspmm_spmm_noalloc(None, None, 0, 4, 0, None, 0, 0, None) == hc.HCSPMM_EINVAL
    assert lib.hcspmm_plan_export_runs(None, None, None, None) == hc.HCSPMM_EINVAL
    assert lib.hcspmm_probe_gather(None, -1, None, 0, 4, 1, None, 0, None) == hc.HCSPMM_EINVAL
    assert lib.hcspmm_layer_backward_workspace_bytes(None, 4, 4) == 0
    assert lib.hcspmm_aggregate_update_workspace_bytes(None, 4, 4) == 0
