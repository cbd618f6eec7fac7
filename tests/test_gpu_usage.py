"""GPU tests of how the library is used rather than of one kernel: one build serving several layers, builds from
two host threads on two streams, the documented behaviour with non-finite features."""
import threading

import numpy as np
import pytest
import torch

import oracle
import scenes
from parity_util import TOL, assert_close, oracle_bwd_input, oracle_bwd_weight, oracle_fwd

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pcpp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2511_23227_amd as m
    m.library()
    return m


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(dtype) if dtype is not None else t


@pytest.mark.parametrize("spatial", [False, True])
def test_one_build_serves_several_layers(pcpp, spatial):
    """The triplets and the plan depend on the coordinates, the radius and t only (Sec. 3.2), so the convolutions of
    a residual block that share them (the ResNet-18 stacks of Sec. 4.1 / 4.2) reuse one build: three channel shapes,
    fp32 and bf16, all three operations each, against the oracle."""
    rng = np.random.default_rng(31)
    n, r, t = 3000, 0.09, 3
    p = rng.uniform(0, 1, (n, 3)).astype(np.float32)
    K = t ** 3
    d = dev(p)
    flags = pcpp.PLAN_FWD | pcpp.PLAN_BWD_INPUT | (pcpp.PLAN_SPATIAL if spatial else 0)
    T = pcpp.pcpp_build_triplets(d, d, r, t, plan_flags=flags)
    o, i, k, seg = oracle.build_triplets(p, p, np.float32(r), t)
    assert np.array_equal(T.tri_o.cpu().numpy(), o) and np.array_equal(T.tri_i.cpu().numpy(), i)
    plan_before = T.plan.clone()
    for cin, cout, dt in ((32, 32, "f32"), (64, 128, "bf16"), (128, 64, "bf16"), (256, 256, "bf16"), (20, 36, "f32")):
        x = rng.standard_normal((n, cin)).astype(np.float32)
        w = (rng.standard_normal((K, cout, cin)) / np.sqrt(K * cin)).astype(np.float32)
        dy = rng.standard_normal((n, cout)).astype(np.float32)
        tdt = torch.float32
        if dt == "bf16":
            x, w, dy, tdt = scenes.round_to_bf16(x), scenes.round_to_bf16(w), scenes.round_to_bf16(dy), torch.bfloat16
        what = f"shared build {cin}->{cout} {dt}"
        ref, scale = oracle_fwd(x, w, o, i, k, n)
        assert_close(pcpp.pcpp_mvmr_fwd(dev(x, tdt), dev(w, tdt), T).cpu().numpy(), ref, scale, TOL[dt], what + " fwd")
        ref, scale = oracle_bwd_input(dy, w, o, i, k, n)
        assert_close(pcpp.pcpp_mvmr_bwd_input(dev(dy, tdt), dev(w, tdt), T).cpu().numpy(), ref, scale, TOL[dt],
                     what + " bwd_input")
        ref, scale = oracle_bwd_weight(x, dy, o, i, k, K)
        assert_close(pcpp.pcpp_mvmr_bwd_weight(dev(x, tdt), dev(dy, tdt), T).cpu().numpy(), ref, scale, TOL[dt],
                     what + " bwd_weight")
    assert torch.equal(plan_before, T.plan)           # the compute calls only read the plan


def test_builds_from_two_threads_on_two_streams(pcpp):
    """The build keeps nothing between calls: two host threads, each on a stream of its own with buffers of its own,
    give the oracle's triplets."""
    rng = np.random.default_rng(17)
    clouds = [rng.uniform(0, 1, (4000, 3)).astype(np.float32), rng.uniform(0, 1, (2500, 3)).astype(np.float32)]
    radii = [0.08, 0.11]
    refs = [oracle.build_triplets(c, c, np.float32(r), 3) for c, r in zip(clouds, radii)]
    devs = [dev(c) for c in clouds]
    torch.cuda.synchronize()
    results, errors = [None, None], []

    def work(j):
        try:
            torch.cuda.set_device(0)
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                for _ in range(5):
                    T = pcpp.pcpp_build_triplets(devs[j], devs[j], radii[j], 3)
                st.synchronize()
            results[j] = T
        except Exception as e:              # noqa: BLE001 - reported by the main thread
            errors.append(e)

    threads = [threading.Thread(target=work, args=(j,)) for j in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    for T, (o, i, k, seg) in zip(results, refs):
        assert T.n_triplets == len(o)
        assert np.array_equal(T.tri_o.cpu().numpy(), o) and np.array_equal(T.tri_i.cpu().numpy(), i)
        assert np.array_equal(T.tri_k.cpu().numpy(), k) and np.array_equal(T.seg_offsets.cpu().numpy(), seg)


def test_pageable_count_word(pcpp):
    """n_triplets in pageable host memory: the documented slower path gives the same result."""
    import ctypes
    from paper_2511_23227_amd import binding as B
    rng = np.random.default_rng(2)
    p = rng.uniform(0, 1, (3000, 3)).astype(np.float32)
    o, i, k, seg = oracle.build_triplets(p, p, np.float32(0.1), 3)
    L = pcpp.library()
    d = dev(p)
    flags = B.PLAN_FWD | B.PLAN_BWD_INPUT
    tri = [torch.empty(len(o), dtype=torch.int32, device="cuda") for _ in range(3)]
    sg = torch.empty(28, dtype=torch.int64, device="cuda")
    plan = torch.zeros(L.pcpp_plan_bytes(len(p), len(p), 3, len(o), flags), dtype=torch.uint8, device="cuda")
    ws = torch.empty(L.pcpp_build_triplets_workspace_bytes_for(len(p), len(p), 3, len(o)), dtype=torch.uint8, device="cuda")
    n = ctypes.c_int64(-1)
    rc = L.pcpp_build_triplets(B._ptr(d), len(p), B._ptr(d), len(p), 0.1, 3, B._ptr(tri[0]), B._ptr(tri[1]),
                               B._ptr(tri[2]), len(o), B._ptr(sg), ctypes.byref(n), B._ptr(plan), plan.numel(), flags,
                               B._ptr(ws), ws.numel(), B._stream())
    assert rc == 0, L.pcpp_last_error()
    torch.cuda.synchronize()
    assert n.value == len(o)
    assert np.array_equal(tri[0].cpu().numpy(), o) and np.array_equal(tri[1].cpu().numpy(), i)
    T = pcpp.pcpp_build_triplets(d, d, 0.1, 3, capacity=len(o), buffers={"plan": torch.zeros_like(plan)})
    assert torch.equal(T.plan[256:], plan[256:])


@pytest.mark.parametrize("c,dt", [(32, "f32"), (64, "bf16"), (256, "bf16"), (20, "f32")])
def test_non_finite_source_row_stays_local(pcpp, c, dt):
    """The header's contract for non-finite features: an Inf in one source row may reach destination rows of the
    same group of up to 128 consecutive centres, never further; rows with a triplet to it are non-finite."""
    rng = np.random.default_rng(c)
    n, r, t = 2000, 0.1, 3
    p = rng.uniform(0, 1, (n, 3)).astype(np.float32)
    o, i, k, seg = oracle.build_triplets(p, p, np.float32(r), t)
    bad = 777
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    x = rng.standard_normal((n, c)).astype(np.float32)
    x[bad, 3] = np.inf
    w = (rng.standard_normal((27, c, c)) / np.sqrt(27 * c)).astype(np.float32)
    d = dev(p)
    T = pcpp.pcpp_build_triplets(d, d, r, t)
    out = pcpp.pcpp_mvmr_fwd(dev(x, tdt), dev(w, tdt), T).cpu().numpy()
    linked = np.unique(o[i == bad])
    assert not np.isfinite(out[linked]).all(axis=1).any()
    groups = np.unique(linked // 128)
    far = ~np.isin(np.arange(n) // 128, groups)
    assert np.isfinite(out[far]).all()


@pytest.mark.parametrize("c, dt, voxel", [(32, torch.float32, False), (256, torch.bfloat16, False), (64, torch.bfloat16, True)])
def test_tune_plan_order(pcpp, c, dt, voxel):
    """The tuner of the plan's order (Sec. 3.3.2, closing remark): it reports positive times for both orders, returns
    flags that differ from the request by PCPP_PLAN_SPATIAL at most and match the faster time, leaves nothing behind
    that a later build depends on, and the plan built with its answer gives the oracle's result."""
    rng = np.random.default_rng(77)
    n, t = 6000, 3
    r = 0.08 if not voxel else 0.05
    p = rng.uniform(0, 1, (n, 3)).astype(np.float32)
    K = t ** 3
    d = dev(p)
    bflags = pcpp.BUILD_VOXEL if voxel else 0
    n_t = pcpp.pcpp_build_triplets(d, d, r, t, plan_flags=pcpp.PLAN_FWD | bflags).n_triplets
    ops = pcpp.PLAN_FWD | pcpp.PLAN_BWD_INPUT
    best, ms_index, ms_spatial = pcpp.pcpp_tune_plan_order(d, d, r, t, n_t, c, c, dt, ops, bflags)
    assert ms_index > 0 and ms_spatial > 0
    assert best & ~pcpp.PLAN_SPATIAL == ops
    assert bool(best & pcpp.PLAN_SPATIAL) == (ms_spatial < ms_index)
    with pytest.raises(pcpp.PcppError):
        pcpp.pcpp_tune_plan_order(d, d, r, t, n_t + 1, c, c, dt, ops, bflags)        # not this cloud's |T|
    with pytest.raises(pcpp.PcppError):
        pcpp.pcpp_tune_plan_order(d, d, r, t, n_t, c, c, dt, pcpp.PLAN_BWD_INPUT, bflags)   # forward side missing
    T = pcpp.pcpp_build_triplets(d, d, r, t, plan_flags=best | bflags)
    if voxel:
        o, i, k, seg = oracle.build_triplets_general(p, p, np.float32(r), t, mode=oracle.MODE_VOXEL)
    else:
        o, i, k, seg = oracle.build_triplets(p, p, np.float32(r), t)
    assert T.n_triplets == n_t == len(o)
    x = rng.standard_normal((n, c)).astype(np.float32)
    w = (rng.standard_normal((K, c, c)) / np.sqrt(K * c)).astype(np.float32)
    name = "f32"
    if dt == torch.bfloat16:
        x, w, name = scenes.round_to_bf16(x), scenes.round_to_bf16(w), "bf16"
    ref, scale = oracle_fwd(x, w, o, i, k, n)
    assert_close(pcpp.pcpp_mvmr_fwd(dev(x, dt), dev(w, dt), T).cpu().numpy(), ref, scale, TOL[name], "fwd on the tuned plan")
