"""The C-ABI library loads without a GPU and exports every function include/epp.h declares."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


def declared_functions():
    text = (ROOT / "include" / "epp.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(epp_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_documented_entry_points():
    names = declared_functions()
    for must in ("epp_prepare", "epp_backward_aggregate", "epp_full_aggregate", "epp_prepare_full",
                 "epp_path_export", "epp_active_set_export", "epp_select_group_size", "epp_last_error",
                 "epp_path_prepare_width"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import paper_2204_02662_amd as epp

    lib = epp.load_library()  # no compute call is made: loading needs no GPU
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    assert not missing, missing
    assert sorted(epp.EXPORTED) == declared_functions()
    assert isinstance(lib.epp_last_error(), bytes)


def test_host_side_argument_checks_need_no_gpu():
    import paper_2204_02662_amd as epp

    lib = epp.load_library()
    assert lib.epp_num_layers(None) == epp.EPP_ERR_INVALID_ARG
    assert b"NULL" in lib.epp_last_error()
    out = ctypes.c_void_p()
    assert lib.epp_prepare(None, None, 0, 1, None, None, ctypes.byref(out)) == epp.EPP_ERR_INVALID_ARG
    assert lib.epp_select_group_size(None, 16) == epp.EPP_ERR_INVALID_ARG
    assert lib.epp_path_prepare_width(None, 16, None) == epp.EPP_ERR_INVALID_ARG
    # size limits are checked before anything is dereferenced or sent to the GPU
    dummy = ctypes.c_void_p(16)
    for n, nnz, want in ((1 << 29, 10, epp.EPP_ERR_TOO_LARGE), (10, (1 << 31) - 1, epp.EPP_ERR_TOO_LARGE),
                         (-1, 0, epp.EPP_ERR_INVALID_ARG)):
        csr = epp._Csr(n, nnz, dummy, dummy, dummy)
        assert lib.epp_prepare(ctypes.byref(csr), None, 0, 2, None, None, ctypes.byref(out)) == want
        assert lib.epp_prepare_full(ctypes.byref(csr), None, None, ctypes.byref(out)) == want
    # combination stage: NULL handles and NULL matrices are refused on the host
    assert lib.epp_weight_gradient_workspace(None, 0, 16, 16) == epp.EPP_ERR_INVALID_ARG
    assert lib.epp_weight_gradient(None, 0, dummy, 16, dummy, 16, dummy, dummy, 1 << 20, None) == epp.EPP_ERR_INVALID_ARG
    assert lib.epp_input_gradient(None, 0, dummy, 16, dummy, 16, dummy, None) == epp.EPP_ERR_INVALID_ARG
    csr = epp._Csr(10, 10, dummy, dummy, dummy)
    assert lib.epp_prepare(ctypes.byref(csr), None, 0, 0, None, None, ctypes.byref(out)) == epp.EPP_ERR_INVALID_ARG  # L < 1
    assert lib.epp_prepare(ctypes.byref(csr), None, 5, 1, None, None, ctypes.byref(out)) == epp.EPP_ERR_INVALID_ARG  # ids NULL


def test_paper_linear_regression_group_size():
    """Sec. 5 regression evaluated on the rows of Table 3 (whole graphs, as printed).  Only the
    coefficients and the table are printed in the paper, not the resulting group sizes, so this
    checks plain arithmetic (parity unpinned beyond that)."""
    import paper_2204_02662_amd as epp

    table3 = [(2708, 5278), (3327, 4552), (19717, 44324), (81306, 1342296), (88784, 2093195),
              (410236, 2439437), (875713, 4322051), (1134890, 2987624)]
    b = (0.65538, 1.67431e-5, -2.24342e-6, 0.63641)
    got = [epp.epp_paper_linreg_group_size(v, e) for v, e in table3]
    want = [max(1, int(b[0] + b[1] * v + b[2] * e + b[3] * e / v + 0.5)) for v, e in table3]
    assert got == want == [2, 2, 2, 10, 12, 6, 9, 15]
    # far outside the fitted domain the value clamps to 1 (e.g. a path of configuration 4)
    assert epp.epp_paper_linreg_group_size(2_449_029, 61_900_000) == 1


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """include/epp.h compiles as C99 and a C program linked against libepp.so runs the host-side
    argument checks (no GPU involved)."""
    import subprocess

    import paper_2204_02662_amd as epp

    epp.load_library()
    exe = tmp_path / "abi_host_checks"
    so_dir = epp.SO.parent
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", str(ROOT / "include"),
                           str(ROOT / "tests" / "c" / "abi_host_checks.c"), "-o", str(exe),
                           "-L", str(so_dir), "-lepp", f"-Wl,-rpath,{so_dir}"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stdout + out.stderr


def test_built_library_is_from_the_current_sources():
    """The library file in the tree is what the GPU tests and the benchmark load; build.py leaves the
    hash of the sources beside it.  A file built from other sources (an edit without a rebuild, a
    left-over experiment) would make every GPU result describe something else."""
    from paper_2204_02662_amd import build
    if not build.SO.exists():
        pytest.skip("library not built")
    assert build.STAMP.exists(), "libepp.so has no source stamp: rebuild (python -m paper_2204_02662_amd.build)"
    assert build.STAMP.read_text().strip() == build.source_hash(), "libepp.so was built from other sources: rebuild"
