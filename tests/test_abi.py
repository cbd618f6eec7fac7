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
    # and nothing else: every dynamic symbol the library defines is declared in the header (the toolchain's own
    # per-file identifiers aside)
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", binding.LIB_PATH], capture_output=True, text=True, check=True)
    exported = {line.split()[-1] for line in out.stdout.splitlines() if line.strip()}
    exported = {s for s in exported if not s.startswith("__hip_")}
    assert exported == declared, exported ^ declared


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
    rc = L.pcpp_mvmr_fwd(None, None, None, 0, 0, 1, 1, 4, 4, 27, None, None, None, None, 0, None, 0, 1, None, 0, None)
    assert rc == -1
    # a plan without the part a call reads, or smaller than these sizes need, is refused before anything is launched
    buf = ctypes.create_string_buffer(4096 + 256)
    p = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    args = (p, p, p, 0, 0, 100, 100, 4, 4, 27, p, p, p, p, 10)
    assert L.pcpp_mvmr_bwd_input(*args, p, 1 << 30, binding.PLAN_FWD, p, 1 << 20, None) == -1
    assert b"plan_flags" in L.pcpp_last_error()
    assert L.pcpp_mvmr_fwd(*args, p, 1024, binding.PLAN_FWD, p, 1 << 20, None) == -3
    assert L.pcpp_mvmr_fwd_static(p, p, p, 0, 0, 100, 100, 1024, 1024, 27, p, p, p, p, 10, p, 1 << 30, 1, None) == -4
    assert L.pcpp_static_scratch_bytes() == 24 << 20
    # spatial plans are larger (a permutation per side and a private gather array for the forward side)
    c = L.pcpp_plan_bytes(1000, 500, 3, 20000, 7)
    assert c >= b + 4 * (1000 + 500 + 20000)
    assert L.pcpp_build_triplets(p, 5, p, 5, 0.1, 3, None, None, None, 0, None, ctypes.byref(n), None, 0, 0x1000,
                                 p, 1 << 20, None) == -1
