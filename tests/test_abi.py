"""CPU-side checks of the C ABI: the library loads and exports every symbol pcpp.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    from paper_2511_23227_amd import binding
    L = binding.library()
    header = open(os.path.join(ROOT, "include", "pcpp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(pcpp_[a-z_]+)\s*\(", header))
    assert {"pcpp_build_triplets", "pcpp_mvmr_fwd", "pcpp_mvmr_bwd_input", "pcpp_mvmr_bwd_weight"} <= declared
    for name in declared:
        assert hasattr(L, name), name
    assert set(binding.EXPORTS) <= declared
    assert L.pcpp_version() >= 100


def test_size_queries_and_argument_errors_without_gpu():
    from paper_2511_23227_amd import binding
    L = binding.library()
    assert L.pcpp_build_triplets_workspace_bytes(1000, 1000, 3) > 0
    assert L.pcpp_build_triplets_workspace_bytes(-1, 10, 3) == 0
    assert L.pcpp_build_triplets_workspace_bytes(10, 10, 99) == 0
    a = L.pcpp_plan_bytes(1000, 500, 3, 20000, 1)
    b = L.pcpp_plan_bytes(1000, 500, 3, 20000, 3)
    assert 0 < a < b and a % 256 == 0 and b % 256 == 0
    assert L.pcpp_mvmr_workspace_bytes(1, 10, 10, 50, 8, 4, 27, 1) >= 27 * 8 * 4 * 2
    # argument validation happens before any GPU call
    n = ctypes.c_int64(-7)
    rc = L.pcpp_build_triplets(None, 5, None, 5, 0.1, 3, None, None, None, 0, None, ctypes.byref(n), None, 0, 0,
                               None, 0, None)
    assert rc == -1 and b"null" in L.pcpp_last_error()
    rc = L.pcpp_mvmr_fwd(None, None, None, 0, 0, 1, 1, 4, 4, 27, None, None, None, None, 0, None, None, 0, None)
    assert rc == -1
