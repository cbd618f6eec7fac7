"""GPU parity of plans built with PLAN_SPATIAL: the library orders the centres along a space-filling curve itself;
the public triplet arrays and every result must be what the plain plan gives (and what the oracle gives)."""
import zlib

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


def spatial_flags(m):
    return m.PLAN_FWD | m.PLAN_BWD_INPUT | m.PLAN_SPATIAL


def check_all(m, T, pin, pout, r, t, x, w, dy, dt, what):
    o, i, k, seg = oracle.build_triplets(pin, pout, np.float32(r), t)
    assert T.n_triplets == len(o)
    assert np.array_equal(T.seg_offsets.cpu().numpy(), seg)
    assert np.array_equal(T.tri_k.cpu().numpy(), k)
    assert np.array_equal(T.tri_o.cpu().numpy(), o)
    assert np.array_equal(T.tri_i.cpu().numpy(), i)
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    K = t ** 3
    out = m.pcpp_mvmr_fwd(dev(x, tdt), dev(w, tdt), T).cpu().numpy()
    ref, scale = oracle_fwd(x, w, o, i, k, len(pout))
    assert_close(out, ref, scale, TOL[dt], what + " fwd")
    gx = m.pcpp_mvmr_bwd_input(dev(dy, tdt), dev(w, tdt), T).cpu().numpy()
    ref, scale = oracle_bwd_input(dy, w, o, i, k, len(pin))
    assert_close(gx, ref, scale, TOL[dt], what + " bwd_input")
    gw = m.pcpp_mvmr_bwd_weight(dev(x, tdt), dev(dy, tdt), T).cpu().numpy()
    ref, scale = oracle_bwd_weight(x, dy, o, i, k, K)
    assert_close(gw, ref, scale, TOL[dt], what + " bwd_weight")


def test_permutation_is_a_space_filling_order(pcpp):
    """The plan's slot order is a permutation of the centres, and consecutive slots are close in space."""
    rng = np.random.default_rng(3)
    p = rng.uniform(0, 1, (20000, 3)).astype(np.float32)
    d = dev(p)
    T = pcpp.pcpp_build_triplets(d, d, 0.03, 3, plan_flags=spatial_flags(pcpp))
    perm = T.plan[256:256 + 4 * len(p)].view(torch.int32).cpu().numpy()
    assert np.array_equal(np.sort(perm), np.arange(len(p)))
    step = np.linalg.norm(np.diff(p[perm], axis=0), axis=1)
    rand = np.linalg.norm(np.diff(p, axis=0), axis=1)
    assert np.median(step) < 0.2 * np.median(rand)
    # a pure function of the coordinates: the same cloud in another index order gives the same order of points
    shuffle = rng.permutation(len(p))
    d2 = dev(p[shuffle])
    T2 = pcpp.pcpp_build_triplets(d2, d2, 0.03, 3, plan_flags=spatial_flags(pcpp))
    perm2 = T2.plan[256:256 + 4 * len(p)].view(torch.int32).cpu().numpy()
    a, b = p[perm], p[shuffle][perm2]
    inv_pitch = 1.0 / (0.5 * float(np.float32(0.03)))          # the sort's cells: half the radius as the library sees it
    same_cell = np.floor(a.astype(np.float64) * inv_pitch) == np.floor(b.astype(np.float64) * inv_pitch)
    assert same_cell.all()


@pytest.mark.parametrize("case", [
    dict(n_in=700, n_out=333, r=0.17, t=3, cin=5, cout=7, dt="f32"),          # generic kernels
    dict(n_in=1501, n_out=1333, r=0.12, t=3, cin=32, cout=32, dt="f32"),      # matrix-core rows kernels
    dict(n_in=1300, n_out=1501, r=0.12, t=3, cin=64, cout=64, dt="bf16"),
    dict(n_in=2100, n_out=700, r=0.15, t=3, cin=64, cout=128, dt="bf16"),
    dict(n_in=1500, n_out=1300, r=0.15, t=5, cin=256, cout=256, dt="bf16"),   # wide kernel
    dict(n_in=1000, n_out=1000, r=0.2, t=6, cin=48, cout=24, dt="bf16"),
    dict(n_in=300, n_out=2000, r=0.15, t=4, cin=16, cout=130, dt="bf16"),
])
def test_small_shapes_spatial(pcpp, case):
    rng = np.random.default_rng(zlib.crc32(repr(sorted(case.items())).encode()))
    pin = rng.uniform(0, 1, (case["n_in"], 3)).astype(np.float32)
    same = case["n_in"] == case["n_out"]
    pout = pin if same else rng.uniform(0, 1, (case["n_out"], 3)).astype(np.float32)
    K = case["t"] ** 3
    x = rng.standard_normal((case["n_in"], case["cin"])).astype(np.float32)
    w = (rng.standard_normal((K, case["cout"], case["cin"])) / np.sqrt(K * case["cin"])).astype(np.float32)
    dy = rng.standard_normal((case["n_out"], case["cout"])).astype(np.float32)
    if case["dt"] == "bf16":
        x, w, dy = scenes.round_to_bf16(x), scenes.round_to_bf16(w), scenes.round_to_bf16(dy)
    din = dev(pin)
    dout = din if same else dev(pout)
    T = pcpp.pcpp_build_triplets(din, dout, case["r"], case["t"], plan_flags=spatial_flags(pcpp))
    check_all(pcpp, T, pin, pout, case["r"], case["t"], x, w, dy, case["dt"], repr(case))


def test_wide_layer_clustered_spatial(pcpp):
    """256 -> 256 on a clustered cloud: long runs, many triplets per (cell, block), empty cells for whole blocks."""
    rng = np.random.default_rng(21)
    p = np.concatenate([rng.normal(0.5, 0.03, (500, 3)), rng.uniform(0, 1, (600, 3)),
                        np.c_[rng.uniform(0, 1, (700, 2)), np.full(700, 0.25)]]).astype(np.float32)
    r, t, c = 0.12, 3, 256
    K = t ** 3
    x = scenes.round_to_bf16(rng.standard_normal((len(p), c)).astype(np.float32))
    w = scenes.round_to_bf16((rng.standard_normal((K, c, c)) / np.sqrt(K * c)).astype(np.float32))
    dy = scenes.round_to_bf16(rng.standard_normal((len(p), c)).astype(np.float32))
    d = dev(p)
    T = pcpp.pcpp_build_triplets(d, d, r, t, plan_flags=spatial_flags(pcpp))
    check_all(pcpp, T, p, p, r, t, x, w, dy, "bf16", "clustered 256")


@pytest.mark.parametrize("sid", [2, 4])
def test_scene_spatial_matches_plain_plan(pcpp, sid):
    """Full scenes: same public arrays as the plain build, results within tolerance of the oracle."""
    s = scenes.make_scene(sid)
    x, w, dy = scenes.make_features(s)
    din = dev(s.in_xyz)
    dout = din if s.out_xyz is s.in_xyz else dev(s.out_xyz)
    T = pcpp.pcpp_build_triplets(din, dout, s.radius, s.t, plan_flags=spatial_flags(pcpp))
    check_all(pcpp, T, s.in_xyz, s.out_xyz, s.radius, s.t, x, w, dy, s.dtype, s.name)


def test_determinism_spatial_wide(pcpp):
    rng = np.random.default_rng(8)
    p = rng.uniform(0, 1, (1500, 3)).astype(np.float32)
    c, t = 256, 3
    x = dev(rng.standard_normal((len(p), c)).astype(np.float32), torch.bfloat16)
    w = dev((rng.standard_normal((27, c, c)) / 80).astype(np.float32), torch.bfloat16)
    d = dev(p)
    runs = []
    n_t = pcpp.pcpp_count_triplets(d, d, 0.15, t)
    nbytes = pcpp.library().pcpp_plan_bytes(len(p), len(p), t, n_t, spatial_flags(pcpp))
    for _ in range(2):
        T = pcpp.pcpp_build_triplets(d, d, 0.15, t, plan_flags=spatial_flags(pcpp), capacity=n_t,
                                     buffers={"plan": torch.zeros(nbytes, dtype=torch.uint8, device="cuda")})
        runs.append([pcpp.pcpp_mvmr_fwd(x, w, T).cpu().numpy(), pcpp.pcpp_mvmr_bwd_input(x, w, T).cpu().numpy(),
                     T.plan.cpu().numpy()[256:]])
    for a, b in zip(*runs):
        assert np.array_equal(a, b)


def test_scene5_spatial_sampled(pcpp):
    """Scene 5 at full size with the plan the benchmark times (PLAN_SPATIAL): forward and input gradient on sampled
    rows against the oracle, element by element; the public arrays must equal those of the plain build."""
    s = scenes.make_scene(5)
    x, w, dy = scenes.make_features(s)
    rng = np.random.default_rng(56)
    xyz = dev(s.in_xyz)
    T = pcpp.pcpp_build_triplets(xyz, xyz, s.radius, s.t, plan_flags=spatial_flags(pcpp))
    T0 = pcpp.pcpp_build_triplets(xyz, xyz, s.radius, s.t, plan_flags=pcpp.PLAN_FWD)
    assert T.n_triplets == T0.n_triplets
    assert torch.equal(T.tri_o, T0.tri_o) and torch.equal(T.tri_i, T0.tri_i) and torch.equal(T.tri_k, T0.tri_k)
    del T0
    n = s.n_in
    bf = torch.bfloat16
    dx_, dw_, ddy = dev(x, bf), dev(w, bf), dev(dy, bf)
    so = np.sort(rng.choice(n, 2048, replace=False))
    o, i, k, _ = oracle.build_triplets(s.in_xyz, s.out_xyz[so], s.radius, s.t)
    out = pcpp.pcpp_mvmr_fwd(dx_, dw_, T)
    ui, inv = np.unique(i, return_inverse=True)
    ref, scale = oracle_fwd(x[ui], w, o, inv.astype(np.int32), k, len(so))
    assert_close(out[torch.from_numpy(so).cuda()].cpu().numpy(), ref, scale, TOL["bf16"], "scene5 spatial fwd")
    del out
    si = np.sort(rng.choice(n, 2048, replace=False))
    o2, i2, k2, _ = oracle.build_triplets(s.in_xyz[si], s.out_xyz, s.radius, s.t)
    gx = pcpp.pcpp_mvmr_bwd_input(ddy, dw_, T)
    uo, inv = np.unique(o2, return_inverse=True)
    ref, scale = oracle_bwd_input(dy[uo], w, inv.astype(np.int32), i2, k2, len(si))
    assert_close(gx[torch.from_numpy(si).cuda()].cpu().numpy(), ref, scale, TOL["bf16"], "scene5 spatial bwd_input")
