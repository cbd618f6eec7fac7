"""The entry point that allocates nothing (pcpp_mvmr_fwd_static) against pcpp_mvmr_fwd, through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pcpp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2511_23227_amd as m
    m.library()
    return m


def run_pair(m, n, c_in, c_out, dt, r, t, seed):
    """One forward pass through each entry point on the same inputs; returns both outputs."""
    from paper_2511_23227_amd import binding as B
    L = m.library()
    rng = np.random.default_rng(seed)
    p = torch.from_numpy(rng.uniform(0, 1, (n, 3)).astype(np.float32)).cuda()
    K = t ** 3
    x = torch.from_numpy(rng.standard_normal((n, c_in)).astype(np.float32)).cuda().to(dt)
    w = torch.from_numpy((rng.standard_normal((K, c_out, c_in)) / np.sqrt(K * c_in)).astype(np.float32)).cuda().to(dt)
    T = m.pcpp_build_triplets(p, p, r, t)
    code = B._dtype_code(x)
    need = L.pcpp_mvmr_workspace_bytes(0, n, n, T.n_triplets, c_in, c_out, K, code)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    ref = torch.full((n, c_out), 7.0, dtype=torch.float32, device="cuda")
    got = torch.full((n, c_out), -7.0, dtype=torch.float32, device="cuda")
    common = (n, n, c_in, c_out, K, B._ptr(T.tri_o), B._ptr(T.tri_i), B._ptr(T.tri_k), B._ptr(T.seg_offsets),
              T.n_triplets, B._ptr(T.plan), T.plan.numel(), T.plan_flags)
    rc = L.pcpp_mvmr_fwd(B._ptr(x), B._ptr(w), B._ptr(ref), code, 0, *common, B._ptr(ws), ws.numel(), B._stream())
    assert rc == 0, L.pcpp_last_error()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = L.pcpp_mvmr_fwd_static(B._ptr(x), B._ptr(w), B._ptr(got), code, 0, *common, B._stream())
    assert rc == 0, L.pcpp_last_error()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return ref, got, T


def test_static_entry_point_matches_twice(pcpp):
    """Two calls in a row, the second with a smaller input: the library's own scratch keeps the first call's
    contents, and the second result must still be bit-identical to the ordinary entry point's."""
    for n, c_in, c_out, dt, r, t, seed in ((3000, 64, 128, torch.bfloat16, 0.09, 3, 1),
                                           (900, 64, 64, torch.bfloat16, 0.12, 3, 2),
                                           (2500, 32, 32, torch.float32, 0.1, 3, 3),
                                           (700, 32, 32, torch.float32, 0.15, 3, 4),
                                           (1500, 256, 256, torch.bfloat16, 0.12, 3, 5),
                                           (400, 256, 256, torch.bfloat16, 0.2, 2, 6)):
        ref, got, T = run_pair(pcpp, n, c_in, c_out, dt, r, t, seed)
        assert T.n_triplets > 0
        assert torch.equal(ref, got), (n, c_in, c_out)


def test_static_entry_point_rejects_what_does_not_fit(pcpp):
    from paper_2511_23227_amd import binding as B
    L = pcpp.library()
    assert L.pcpp_static_scratch_bytes() == 24 << 20
    n, c, t = 200, 512, 5                         # 125 * 512 * 512 * 2 bytes = 65 MB of packed weights
    p = torch.rand((n, 3), device="cuda")
    T = pcpp.pcpp_build_triplets(p, p, 0.2, t)
    x = torch.zeros((n, c), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((t ** 3, c, c), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((n, c), dtype=torch.float32, device="cuda")
    with pytest.raises(pcpp.PcppError) as e:
        pcpp.pcpp_mvmr_fwd_static(x, w, T, out)
    assert e.value.code == -4 and "scratch" in str(e.value)
