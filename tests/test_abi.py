"""The C-ABI library loads without a GPU and exports every function include/epp.h declares."""
import ctypes
import re
from pathlib import Path

ROOT = Path(__file__).resolve().parent.parent


def declared_functions():
    text = (ROOT / "include" / "epp.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(epp_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_documented_entry_points():
    names = declared_functions()
    for must in ("epp_prepare", "epp_backward_aggregate", "epp_full_aggregate", "epp_prepare_full",
                 "epp_path_export", "epp_active_set_export", "epp_select_group_size", "epp_last_error"):
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
    assert lib.epp_prepare(None, None, 0, 1, None, ctypes.byref(out)) == epp.EPP_ERR_INVALID_ARG
    assert lib.epp_select_group_size(None, 16) == epp.EPP_ERR_INVALID_ARG
