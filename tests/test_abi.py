"""The C-ABI library loads without a GPU and exports every function include/ca_attention.h declares."""
import ctypes
import os
import re

from paper_2510_18121_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "ca_attention.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b(ca_[a-z_0-9]+)\s*\(", src)
    return sorted(set(names))


def test_header_functions_are_exported():
    names = declared_functions()
    assert {"ca_plan", "ca_plan_host", "ca_plan_upload", "ca_forward", "ca_backward", "ca_plan_destroy",
            "ca_plan_workspace_bytes", "ca_error_string", "ca_last_error", "ca_profile_enable",
            "ca_profile_read", "ca_plan_info", "ca_plan_rows", "ca_plan_fwd_units", "ca_plan_bwd_units",
            "ca_merge_partials", "ca_sum_partial_dq", "ca_mfma_stream"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_error_strings():
    lib = B.lib()
    seen = set()
    for code in (0, -1, -2, -3, -4, -5):
        s = lib.ca_error_string(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert "unknown" in lib.ca_error_string(-99).decode()


def test_calls_without_plan_fail_cleanly():
    lib = B.lib()
    assert lib.ca_forward(None, None, None, None, None, None, None, 0, None) == B.CA_ERR_INVALID_ARG
    assert lib.ca_plan_workspace_bytes(None, None, None) == B.CA_ERR_INVALID_ARG
    assert lib.ca_plan_host(None, None) == B.CA_ERR_INVALID_ARG
    lib.ca_plan_destroy(None)  # no-op


def test_merge_entry_points_reject_bad_arguments_on_the_host():
    lib = B.lib()
    # counts and head_dim are checked before anything touches a device
    assert lib.ca_merge_partials(None, 4, 0, None, None, 4, None, None, None, None, 2, 64, None) == B.CA_ERR_INVALID_ARG
    assert b"n_parts" in lib.ca_last_error()
    assert lib.ca_merge_partials(None, 4, 65, None, None, 4, None, None, None, None, 2, 64, None) == B.CA_ERR_INVALID_ARG
    assert lib.ca_merge_partials(None, 4, 2, None, None, 4, None, None, None, None, 2, 96, None) == B.CA_ERR_UNSUPPORTED
    assert lib.ca_merge_partials(None, 4, 2, None, None, 4, None, None, None, None, 2, 64, None) == B.CA_ERR_INVALID_ARG
    assert b"null" in lib.ca_last_error()
    assert lib.ca_sum_partial_dq(None, -1, 2, None, 4, None, 2, 64, None) == B.CA_ERR_INVALID_ARG
    assert lib.ca_sum_partial_dq(None, 4, 2, None, 4, None, 2, 64, None) == B.CA_ERR_INVALID_ARG
    # nothing to do: no launch, no error
    assert lib.ca_merge_partials(None, 0, 1, None, None, 0, None, None, None, None, 2, 64, None) == B.CA_OK


def test_mfma_stream_rejects_bad_arguments_on_the_host():
    lib = B.lib()
    assert lib.ca_mfma_stream(None, 65, 4, 0, None, None) == B.CA_ERR_INVALID_ARG
    assert b"multiple of 64" in lib.ca_last_error()
    assert lib.ca_mfma_stream(None, -64, 4, 0, None, None) == B.CA_ERR_INVALID_ARG
    assert lib.ca_mfma_stream(None, 64, -1, 0, None, None) == B.CA_ERR_INVALID_ARG
    assert lib.ca_mfma_stream(None, 64, 4, 3, None, None) == B.CA_ERR_INVALID_ARG
    assert b"side_work" in lib.ca_last_error()
    assert lib.ca_mfma_stream(None, 64, 4, 0, None, None) == B.CA_ERR_INVALID_ARG
    assert b"null" in lib.ca_last_error()
    assert lib.ca_mfma_stream(None, 64, 0, 0, None, None) == B.CA_OK
