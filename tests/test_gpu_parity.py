"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
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


def feat_dtype(scene):
    return torch.bfloat16 if scene.dtype == "bf16" else torch.float32


def build_gpu(pcpp, in_xyz, out_xyz, r, t, same=False):
    din = dev(in_xyz)
    dout = din if same else dev(out_xyz)
    return pcpp.pcpp_build_triplets(din, dout, r, t)


def check_triplets(T, o, i, k, seg):
    assert T.n_triplets == len(o)
    assert np.array_equal(T.seg_offsets.cpu().numpy(), seg)
    assert np.array_equal(T.tri_k.cpu().numpy(), k)
    assert np.array_equal(T.tri_o.cpu().numpy(), o)
    assert np.array_equal(T.tri_i.cpu().numpy(), i)


def run_ops(pcpp, scene, T, x, w, dy, o, i, k, ops):
    tol = TOL[scene.dtype]
    dt = feat_dtype(scene)
    dx_, dw_, ddy = dev(x, dt), (dev(w, dt) if w is not None else None), dev(dy, dt)
    if "fwd" in ops:
        out = pcpp.pcpp_mvmr_fwd(dx_, dw_, T).cpu().numpy()
        ref, scale = oracle_fwd(x, w, o, i, k, scene.n_out)
        assert_close(out, ref, scale, tol, f"{scene.name} fwd")
    if "bwd_input" in ops:
        gx = pcpp.pcpp_mvmr_bwd_input(ddy, dw_, T).cpu().numpy()
        ref, scale = oracle_bwd_input(dy, w, o, i, k, scene.n_in)
        assert_close(gx, ref, scale, tol, f"{scene.name} bwd_input")
    if "bwd_weight" in ops:
        gw = pcpp.pcpp_mvmr_bwd_weight(dx_, ddy, T).cpu().numpy()
        ref, scale = oracle_bwd_weight(x, dy, o, i, k, scene.K)
        assert_close(gw, ref, scale, tol, f"{scene.name} bwd_weight")
        assert not gw[np.diff(T.seg_offsets.cpu().numpy()) == 0].any()      # unused cells: exact zeros


@pytest.mark.parametrize("sid", [1, 2, 3, 4])
def test_scene_full(pcpp, sid):
    """Scenes 1-4 at full size: triplets bit-exact, every op within tolerance on every element."""
    s = scenes.make_scene(sid)
    x, w, dy = scenes.make_features(s)
    o, i, k, seg = oracle.build_triplets(s.in_xyz, s.out_xyz, s.radius, s.t)
    T = build_gpu(pcpp, s.in_xyz, s.out_xyz, s.radius, s.t, same=s.out_xyz is s.in_xyz)
    check_triplets(T, o, i, k, seg)
    run_ops(pcpp, s, T, x, w, dy, o, i, k, ("fwd", "bwd_input", "bwd_weight"))


@pytest.mark.parametrize("case", [
    dict(n_in=700, n_out=333, r=0.17, t=3, cin=5, cout=7, dt="f32"),
    dict(n_in=1000, n_out=1000, r=0.12, t=2, cin=24, cout=8, dt="bf16"),
    dict(n_in=900, n_out=129, r=0.2, t=5, cin=70, cout=33, dt="f32"),
    dict(n_in=64, n_out=64, r=0.5, t=1, cin=3, cout=3, dt="f32"),
    dict(n_in=300, n_out=2000, r=0.15, t=4, cin=16, cout=130, dt="bf16"),
    # shapes served by the matrix-core kernels, with ragged point counts
    dict(n_in=1501, n_out=1333, r=0.12, t=3, cin=32, cout=32, dt="f32"),
    dict(n_in=1300, n_out=1501, r=0.12, t=3, cin=64, cout=64, dt="bf16"),
    dict(n_in=2100, n_out=700, r=0.15, t=3, cin=64, cout=128, dt="bf16"),
    dict(n_in=999, n_out=999, r=0.2, t=5, cin=32, cout=32, dt="bf16"),
    dict(n_in=800, n_out=31, r=0.2, t=2, cin=64, cout=64, dt="f32"),
    # the largest kernel the library accepts: K = 216 (the search tables need more LDS than the default limit)
    dict(n_in=1100, n_out=900, r=0.22, t=6, cin=12, cout=20, dt="f32"),
    dict(n_in=1000, n_out=1000, r=0.2, t=6, cin=64, cout=64, dt="bf16"),
    # wide layers (W shared through LDS), K = 125 and K = 27, ragged point counts
    dict(n_in=1500, n_out=1300, r=0.15, t=5, cin=256, cout=256, dt="bf16"),
    dict(n_in=700, n_out=900, r=0.2, t=3, cin=128, cout=128, dt="bf16"),
    # enough triplets for the weight gradient to balance its chunks over the CUs (two sub-block waves per chunk)
    dict(n_in=5000, n_out=5000, r=0.15, t=3, cin=128, cout=128, dt="bf16"),
])
def test_small_shapes(pcpp, case):
    """Ragged sizes: n_out != n_in, partial tiles, channel counts that are not multiples of anything."""
    rng = np.random.default_rng(zlib.crc32(repr(sorted(case.items())).encode()))
    pin = rng.uniform(0, 1, (case["n_in"], 3)).astype(np.float32)
    pout = rng.uniform(0, 1, (case["n_out"], 3)).astype(np.float32)
    K = case["t"] ** 3
    x = rng.standard_normal((case["n_in"], case["cin"])).astype(np.float32)
    w = (rng.standard_normal((K, case["cout"], case["cin"])) / np.sqrt(K * case["cin"])).astype(np.float32)
    dy = rng.standard_normal((case["n_out"], case["cout"])).astype(np.float32)
    if case["dt"] == "bf16":
        x, w, dy = scenes.round_to_bf16(x), scenes.round_to_bf16(w), scenes.round_to_bf16(dy)
    s = scenes.Scene(0, "small", pin, pout, float(np.float32(case["r"])), case["t"], case["cin"], case["cout"], case["dt"])
    o, i, k, seg = oracle.build_triplets(pin, pout, s.radius, s.t)
    T = build_gpu(pcpp, pin, pout, s.radius, s.t)
    check_triplets(T, o, i, k, seg)
    run_ops(pcpp, s, T, x, w, dy, o, i, k, ("fwd", "bwd_input", "bwd_weight"))


def test_edge_cases(pcpp):
    m = pcpp
    # no inputs, some outputs: zero triplets, zero output rows
    pin = np.zeros((0, 3), np.float32)
    pout = np.random.default_rng(0).uniform(0, 1, (10, 3)).astype(np.float32)
    T = build_gpu(m, pin, pout, 0.3, 3)
    assert T.n_triplets == 0 and not T.seg_offsets.cpu().numpy().any()
    out = m.pcpp_mvmr_fwd(torch.zeros((0, 4), device="cuda"), torch.ones((27, 6, 4), device="cuda"), T)
    assert out.shape == (10, 6) and not out.cpu().numpy().any()
    # no outputs
    T = build_gpu(m, pout, pin, 0.3, 3)
    assert T.n_triplets == 0
    # coincident points: every pair is a triplet in the centre cell
    q = np.tile(np.array([[0.25, 0.5, 0.75]], np.float32), (70, 1))
    T = build_gpu(m, q, q, 0.1, 3, same=True)
    o, i, k, seg = oracle.build_triplets(q, q, np.float32(0.1), 3)
    check_triplets(T, o, i, k, seg)
    assert T.n_triplets == 4900 and np.all(k == 13)
    # far-apart points: only self pairs; outputs with no neighbour give zero rows
    far = (np.arange(30, dtype=np.float32)[:, None] * np.array([[10.0, 0, 0]], np.float32))
    T = build_gpu(m, far[:20], far, 0.5, 3)
    o, i, k, seg = oracle.build_triplets(far[:20], far, np.float32(0.5), 3)
    check_triplets(T, o, i, k, seg)
    x = torch.ones((20, 2), device="cuda")
    out = m.pcpp_mvmr_fwd(x, torch.ones((27, 2, 2), device="cuda"), T).cpu().numpy()
    assert np.array_equal(out[:20], np.full((20, 2), 2.0)) and not out[20:].any()


def test_boundary_ties_and_large_coordinates(pcpp):
    """Points on a coarse binary grid produce exact ties at |d| = r and on cell faces."""
    rng = np.random.default_rng(9)
    p = (rng.integers(0, 64, (3000, 3)) / 16.0).astype(np.float32)          # spacing 1/16
    for shift in (0.0, 4096.0):
        q = (p + np.float32(shift)).astype(np.float32)
        for r, t in ((0.25, 4), (0.1875, 3), (0.3125, 5)):
            o, i, k, seg = oracle.build_triplets(q, q, np.float32(r), t)
            T = build_gpu(pcpp, q, q, r, t, same=True)
            check_triplets(T, o, i, k, seg)


def test_dense_cluster_uses_rescan_path(pcpp):
    """More neighbours per centre than the on-chip list holds: ranks come from a second scan."""
    rng = np.random.default_rng(4)
    p = rng.normal(0.5, 0.02, (1500, 3)).astype(np.float32)
    o, i, k, seg = oracle.build_triplets(p, p, np.float32(0.05), 3)
    d = dev(p)
    flags = pcpp.PLAN_FWD | pcpp.PLAN_BWD_INPUT | pcpp.BUILD_TEST_SHORT_LISTS
    nbytes = pcpp.library().pcpp_plan_bytes(len(p), len(p), 3, len(o), pcpp.PLAN_FWD | pcpp.PLAN_BWD_INPUT)
    zeros = lambda: {"plan": torch.zeros(nbytes, dtype=torch.uint8, device="cuda")}
    T = pcpp.pcpp_build_triplets(d, d, 0.05, 3, plan_flags=flags, capacity=len(o), buffers=zeros())
    assert np.bincount(o).max() > 40
    check_triplets(T, o, i, k, seg)
    # the same plan as the ordinary paths write
    T2 = pcpp.pcpp_build_triplets(d, d, 0.05, 3, capacity=len(o), buffers=zeros())
    assert torch.equal(T.plan[256:], T2.plan[256:])


def test_wide_key_path(pcpp):
    """Lists of more than 160 neighbours when cell and index do not share a word (as for clouds of 2^24 points):
    per-cell buckets filled with wave ballots.  Same triplets and same plan as the packed-key path."""
    rng = np.random.default_rng(5)
    p = np.concatenate([rng.normal(0.5, 0.02, (900, 3)), rng.uniform(0, 1, (600, 3))]).astype(np.float32)
    r, t = 0.05, 5
    o, i, k, seg = oracle.build_triplets(p, p, np.float32(r), t)
    cnt = np.bincount(o)
    assert ((cnt > 160) & (cnt <= 512)).any()
    d = dev(p)
    flags = pcpp.PLAN_FWD | pcpp.PLAN_BWD_INPUT
    nbytes = pcpp.library().pcpp_plan_bytes(len(p), len(p), t, len(o), flags)
    zeros = lambda: {"plan": torch.zeros(nbytes, dtype=torch.uint8, device="cuda")}
    T = pcpp.pcpp_build_triplets(d, d, r, t, plan_flags=flags | pcpp.BUILD_TEST_WIDE_KEYS, capacity=len(o), buffers=zeros())
    check_triplets(T, o, i, k, seg)
    T2 = pcpp.pcpp_build_triplets(d, d, r, t, plan_flags=flags, capacity=len(o), buffers=zeros())
    assert torch.equal(T.plan[256:], T2.plan[256:])


def test_error_paths(pcpp):
    m = pcpp
    p = dev(np.random.default_rng(1).uniform(0, 1, (500, 3)).astype(np.float32))
    n = m.binding.pcpp_count_triplets(p, p, 0.2, 3)
    assert n == oracle.count_triplets(p.cpu().numpy(), p.cpu().numpy(), np.float32(0.2), 3)
    with pytest.raises(m.PcppError) as e:
        m.pcpp_build_triplets(p, p, 0.2, 3, capacity=n - 1)
    assert e.value.code == -2 and str(n) in str(e.value)
    with pytest.raises(m.PcppError) as e:
        m.pcpp_build_triplets(p, p, -1.0, 3)
    assert e.value.code == -1
    with pytest.raises(m.PcppError):
        m.pcpp_build_triplets(p, p, 0.2, 9)
    T = m.pcpp_build_triplets(p, p, 0.2, 3, plan_flags=m.PLAN_FWD)
    with pytest.raises(m.PcppError):
        m.pcpp_mvmr_bwd_input(torch.zeros((500, 4), device="cuda"), torch.zeros((27, 4, 4), device="cuda"), T)


def test_determinism(pcpp):
    """Two runs give identical triplet arrays and identical float bits (no atomics on the data path)."""
    s = scenes.make_scene(1)
    x, w, dy = scenes.make_features(s)
    outs = []
    for _ in range(2):
        T = build_gpu(pcpp, s.in_xyz, s.out_xyz, s.radius, s.t, same=True)
        out = pcpp.pcpp_mvmr_fwd(dev(x), dev(w), T)
        gx = pcpp.pcpp_mvmr_bwd_input(dev(dy), dev(w), T)
        gw = pcpp.pcpp_mvmr_bwd_weight(dev(x), dev(dy), T)
        outs.append([T.tri_o.cpu().numpy(), T.tri_i.cpu().numpy(), T.tri_k.cpu().numpy(), out.cpu().numpy(),
                     gx.cpu().numpy(), gw.cpu().numpy()])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_scene5_full_size_sampled(pcpp):
    """Scene 5 (1M points, K = 125, 256 -> 256 bf16) at full size.  The oracle cannot finish the whole scene
    in a test, so: global invariants of the triplet list, bit-exact triplets for sampled outputs (and, with the
    roles swapped, for sampled inputs), and every float op on those samples element by element."""
    s = scenes.make_scene(5)
    x, w, dy = scenes.make_features(s)
    tol = TOL[s.dtype]
    rng = np.random.default_rng(55)
    xyz = dev(s.in_xyz)
    T = pcpp.pcpp_build_triplets(xyz, xyz, s.radius, s.t)
    n = s.n_in
    # invariants on the whole list
    assert T.n_triplets == pcpp.binding.pcpp_count_triplets(xyz, xyz, s.radius, s.t)
    key = (T.tri_k.long() * n + T.tri_o.long()) * n + T.tri_i.long()
    assert bool((key[1:] > key[:-1]).all())                       # strictly ascending (k, o, i)
    seg = T.seg_offsets.cpu().numpy()
    assert seg[0] == 0 and seg[-1] == T.n_triplets
    bounds = torch.searchsorted(T.tri_k.long().contiguous(), torch.arange(s.K + 1, device="cuda"))
    assert np.array_equal(bounds.cpu().numpy(), seg)
    cnt = np.diff(seg).reshape(5, 5, 5)
    assert all(cnt[a, b, c] == 0 for a in (0, 4) for b in (0, 4) for c in (0, 4))   # corner cells lie outside the ball
    assert abs(T.n_triplets / n - 32.0) <= 1.0
    del key
    tri_o, tri_i, tri_k = (t.cpu().numpy() for t in (T.tri_o, T.tri_i, T.tri_k))

    # sampled outputs: triplets and forward
    so = np.sort(rng.choice(n, 4096, replace=False))
    o, i, k, _ = oracle.build_triplets(s.in_xyz, s.out_xyz[so], s.radius, s.t)
    sel = np.isin(tri_o, so)
    assert np.array_equal(np.searchsorted(so, tri_o[sel]), o)
    assert np.array_equal(tri_i[sel], i) and np.array_equal(tri_k[sel], k)
    dt = feat_dtype(s)
    dx_, dw_, ddy = dev(x, dt), (dev(w, dt) if w is not None else None), dev(dy, dt)
    out = pcpp.pcpp_mvmr_fwd(dx_, dw_, T)
    ui, inv = np.unique(i, return_inverse=True)
    ref, scale = oracle_fwd(x[ui], w, o, inv.astype(np.int32), k, len(so))
    assert_close(out[torch.from_numpy(so).cuda()].cpu().numpy(), ref, scale, tol, "scene5 fwd (sampled outputs)")
    # weight gradient with dy restricted to the sampled outputs: only their triplets contribute
    dy_m = np.zeros_like(dy)
    dy_m[so] = dy[so]
    gw = pcpp.pcpp_mvmr_bwd_weight(dx_, dev(dy_m, dt), T).cpu().numpy()
    ref, scale = oracle_bwd_weight(x[ui], dy[so], o, inv.astype(np.int32), k, s.K)
    assert_close(gw, ref, scale, tol, "scene5 bwd_weight (dy on sampled outputs)")
    del out, gw

    # sampled inputs: all triplets that touch them, and the input gradient
    si = np.sort(rng.choice(n, 4096, replace=False))
    o2, i2, k2, _ = oracle.build_triplets(s.in_xyz[si], s.out_xyz, s.radius, s.t)
    sel = np.isin(tri_i, si)
    got = sorted(zip(tri_k[sel].tolist(), tri_o[sel].tolist(), np.searchsorted(si, tri_i[sel]).tolist()))
    assert got == sorted(zip(k2.tolist(), o2.tolist(), i2.tolist()))
    gx = pcpp.pcpp_mvmr_bwd_input(ddy, dw_, T)
    uo, inv = np.unique(o2, return_inverse=True)
    ref, scale = oracle_bwd_input(dy[uo], w, inv.astype(np.int32), i2, k2, len(si))
    assert_close(gx[torch.from_numpy(si).cuda()].cpu().numpy(), ref, scale, tol, "scene5 bwd_input (sampled inputs)")


@pytest.mark.parametrize("spatial,same", [(False, False), (True, False), (True, True)])
def test_build_with_and_without_kept_neighbours(pcpp, spatial, same):
    """The second pass either ranks the neighbours the count pass kept (large workspace) or searches again
    (minimal workspace, or lists longer than the kept part), and the second count of a plan in spatial order either
    regroups the first one's lists or searches again: same triplets and same plan either way, and both equal to the
    oracle's list.  Separate centres, and a cloud against itself (one count pass for both sides of the plan)."""
    rng = np.random.default_rng(77)
    # a dense blob among sparse points: some centres have far more neighbours than twice the mean
    pts = np.concatenate([rng.random((3000, 3)) * 2.0, 0.9 + rng.random((500, 3)) * 0.08]).astype(np.float32)
    out = pts if same else pts[::3].copy()
    r, t = 0.12, 3
    o, i, k, seg = oracle.build_triplets(pts, out, r, t)
    L = pcpp.library()
    din = dev(pts)
    dout = din if same else dev(out)
    small = torch.empty(L.pcpp_build_triplets_workspace_bytes(len(pts), len(out), t), dtype=torch.uint8, device="cuda")
    large = torch.empty(L.pcpp_build_triplets_workspace_bytes_for(len(pts), len(out), t, len(o)), dtype=torch.uint8,
                        device="cuda")
    assert large.numel() > small.numel()
    # capacity given: the binding keeps a workspace that is large enough, so the minimal one is passed through
    # the C ABI directly
    import ctypes
    from paper_2511_23227_amd import binding as B
    results = []
    for ws in (small, large):
        tri = [torch.empty(len(o), dtype=torch.int32, device="cuda") for _ in range(3)]
        sg = torch.empty(t ** 3 + 1, dtype=torch.int64, device="cuda")
        flags = B.PLAN_FWD | B.PLAN_BWD_INPUT | (B.PLAN_SPATIAL if spatial else 0)
        plan = torch.zeros(L.pcpp_plan_bytes(len(pts), len(out), t, len(o), flags), dtype=torch.uint8, device="cuda")
        n = ctypes.c_int64(0)
        rc = L.pcpp_build_triplets(B._ptr(din), len(pts), B._ptr(dout), len(out), float(r), t, B._ptr(tri[0]),
                                   B._ptr(tri[1]), B._ptr(tri[2]), len(o), B._ptr(sg), ctypes.byref(n), B._ptr(plan),
                                   plan.numel(), flags, B._ptr(ws), ws.numel(), B._stream())
        assert rc == 0, L.pcpp_last_error()
        torch.cuda.synchronize()
        assert n.value == len(o)
        assert np.array_equal(tri[0].cpu().numpy(), o) and np.array_equal(tri[1].cpu().numpy(), i)
        assert np.array_equal(tri[2].cpu().numpy(), k) and np.array_equal(sg.cpu().numpy(), seg)
        results.append(plan.cpu().numpy()[256:])         # everything after the header
    assert np.array_equal(results[0], results[1])


@pytest.mark.parametrize("case", [
    dict(n=1400, r=0.12, t=3, c=32, dt="f32"),        # split-bf16 rows kernel, 16x16x4 weight kernel
    dict(n=1200, r=0.12, t=3, c=64, dt="bf16"),
    dict(n=900, r=0.16, t=5, c=256, dt="bf16"),       # wide kernels
])
def test_determinism_matrix_core_paths(pcpp, case):
    """The tuned kernels add partial results in a fixed order: two runs give identical bits."""
    rng = np.random.default_rng(case["n"])
    p = rng.uniform(0, 1, (case["n"], 3)).astype(np.float32)
    K, c = case["t"] ** 3, case["c"]
    dt = torch.bfloat16 if case["dt"] == "bf16" else torch.float32
    x = dev(rng.standard_normal((case["n"], c)).astype(np.float32), dt)
    w = dev((rng.standard_normal((K, c, c)) / np.sqrt(K * c)).astype(np.float32), dt)
    dy = dev(rng.standard_normal((case["n"], c)).astype(np.float32), dt)
    runs = []
    for _ in range(2):
        T = build_gpu(pcpp, p, p, case["r"], case["t"], same=True)
        runs.append([pcpp.pcpp_mvmr_fwd(x, w, T).cpu().numpy(), pcpp.pcpp_mvmr_bwd_input(dy, w, T).cpu().numpy(),
                     pcpp.pcpp_mvmr_bwd_weight(x, dy, T).cpu().numpy()])
    for a, b in zip(*runs):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("c", [64, 256])
def test_bf16_outputs(pcpp, c):
    """out / dx emitted as bf16: the fp32 result rounded once (tolerance of the bf16 inputs plus one rounding)."""
    rng = np.random.default_rng(c)
    n, r, t = 1100, 0.15, 3
    p = rng.uniform(0, 1, (n, 3)).astype(np.float32)
    K = t ** 3
    x = scenes.round_to_bf16(rng.standard_normal((n, c)).astype(np.float32))
    w = scenes.round_to_bf16((rng.standard_normal((K, c, c)) / np.sqrt(K * c)).astype(np.float32))
    dy = scenes.round_to_bf16(rng.standard_normal((n, c)).astype(np.float32))
    o, i, k, seg = oracle.build_triplets(p, p, np.float32(r), t)
    T = build_gpu(pcpp, p, p, r, t, same=True)
    check_triplets(T, o, i, k, seg)
    bf = torch.bfloat16
    out = pcpp.pcpp_mvmr_fwd(dev(x, bf), dev(w, bf), T, out_dtype=bf)
    assert out.dtype == bf
    ref, scale = oracle_fwd(x, w, o, i, k, n)
    assert_close(out.float().cpu().numpy(), ref, scale, TOL["bf16"] + 2.0 ** -8, f"bf16 out c={c}")
    gx = pcpp.pcpp_mvmr_bwd_input(dev(dy, bf), dev(w, bf), T, out_dtype=bf)
    assert gx.dtype == bf
    ref, scale = oracle_bwd_input(dy, w, o, i, k, n)
    assert_close(gx.float().cpu().numpy(), ref, scale, TOL["bf16"] + 2.0 ** -8, f"bf16 dx c={c}")


def test_wide_layer_long_lists(pcpp):
    """256 -> 256 with hundreds of triplets per (cell, 32-centre block): the wide kernel's path for lists longer
    than its prefetch ring, and runs that straddle its 64-triplet groups."""
    rng = np.random.default_rng(21)
    p = np.concatenate([rng.normal(0.5, 0.03, (500, 3)), rng.uniform(0, 1, (300, 3))]).astype(np.float32)
    r, t, c = 0.12, 3, 256
    K = t ** 3
    x = scenes.round_to_bf16(rng.standard_normal((len(p), c)).astype(np.float32))
    w = scenes.round_to_bf16((rng.standard_normal((K, c, c)) / np.sqrt(K * c)).astype(np.float32))
    dy = scenes.round_to_bf16(rng.standard_normal((len(p), c)).astype(np.float32))
    s = scenes.Scene(0, "dense256", p, p, float(np.float32(r)), t, c, c, "bf16")
    o, i, k, seg = oracle.build_triplets(p, p, s.radius, t)
    per_block_cell = np.bincount(k.astype(np.int64) * (len(p) // 32 + 1) + o // 32)
    assert per_block_cell.max() > 256
    T = build_gpu(pcpp, p, p, r, t, same=True)
    check_triplets(T, o, i, k, seg)
    run_ops(pcpp, s, T, x, w, dy, o, i, k, ("fwd", "bwd_input", "bwd_weight"))


@pytest.mark.parametrize("c", [64, 256])
def test_weight_gradient_short_lists(pcpp, c):
    """Weight gradient of the bf16 kernels on lists shorter than their pipelines: 1 to 196 triplets in one cell
    (coincident points), and a sparse cloud in which every cell of a 5^3 kernel holds a handful of triplets."""
    rng = np.random.default_rng(77 + c)
    cases = []
    for n in (1, 2, 5, 6, 8, 11, 14):
        q = np.tile(np.array([[0.25, 0.5, 0.75]], np.float32), (n, 1))
        cases.append((q, 0.1, 3))
    cases.append((rng.uniform(0, 1, (60, 3)).astype(np.float32), 0.3, 5))
    cases.append((rng.uniform(0, 1, (300, 3)).astype(np.float32), 0.12, 5))
    for q, r, t in cases:
        n = len(q)
        o, i, k, seg = oracle.build_triplets(q, q, np.float32(r), t)
        T = build_gpu(pcpp, q, q, r, t, same=True)
        check_triplets(T, o, i, k, seg)
        x = scenes.round_to_bf16(rng.standard_normal((n, c)).astype(np.float32))
        dy = scenes.round_to_bf16(rng.standard_normal((n, c)).astype(np.float32))
        s = scenes.Scene(0, f"short{n}", q, q, float(np.float32(r)), t, c, c, "bf16")
        run_ops(pcpp, s, T, x, None, dy, o, i, k, ("bwd_weight",))


RANDOM_SHAPES = [(32, 32, "f32"), (64, 64, "f32"), (16, 16, "f32"), (64, 64, "bf16"), (64, 128, "bf16"),
                 (128, 64, "bf16"), (128, 128, "bf16"), (256, 256, "bf16"), (48, 24, "bf16")]


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_small_scenes(pcpp, seed):
    """Seeded random draws of everything at once: kernel size 1..6, radius, point counts, uniform / clustered /
    lattice-with-ties clouds, self-convolution or separate centres, and a channel shape from every kernel family.
    Triplets bit-exact and all three ops within tolerance on every element, twelve cases per seed."""
    rng = np.random.default_rng(seed)
    for case in range(12):
        t = int(rng.integers(1, 7))
        n_in = int(rng.integers(1, 2500))
        same = bool(rng.random() < 0.5)
        n_out = n_in if same else int(rng.integers(1, 2500))
        kind = int(rng.integers(0, 3))

        def cloud(n):
            if kind == 0:
                return rng.uniform(0, 1, (n, 3))
            if kind == 1:       # half the points in a blob far denser than the rest
                return np.concatenate([rng.normal(0.5, 0.03, (n // 2, 3)), rng.uniform(0, 1, (n - n // 2, 3))])
            return rng.integers(0, 24, (n, 3)) / 16.0      # many points exactly on the ball and on cell faces

        pin = cloud(n_in).astype(np.float32)
        pout = pin if same else cloud(n_out).astype(np.float32)
        r = float(np.float32(rng.choice([0.0625, 0.1, 0.15, 0.25])))
        cin, cout, dt = RANDOM_SHAPES[int(rng.integers(0, len(RANDOM_SHAPES)))]
        what = f"seed {seed} case {case}: t={t} n_in={n_in} n_out={n_out} same={same} kind={kind} r={r} " \
               f"{cin}->{cout} {dt}"
        print(what, flush=True)
        K = t ** 3
        o, i, k, seg = oracle.build_triplets(pin, pout, np.float32(r), t)
        T = build_gpu(pcpp, pin, pout, r, t, same=same)
        check_triplets(T, o, i, k, seg)
        x = rng.standard_normal((n_in, cin)).astype(np.float32)
        w = (rng.standard_normal((K, cout, cin)) / np.sqrt(K * cin)).astype(np.float32)
        dy = rng.standard_normal((n_out, cout)).astype(np.float32)
        tdt = torch.float32
        if dt == "bf16":
            x, w, dy, tdt = scenes.round_to_bf16(x), scenes.round_to_bf16(w), scenes.round_to_bf16(dy), torch.bfloat16
        out = pcpp.pcpp_mvmr_fwd(dev(x, tdt), dev(w, tdt), T).cpu().numpy()
        ref, scale = oracle_fwd(x, w, o, i, k, n_out)
        assert_close(out, ref, scale, TOL[dt], what + " fwd")
        gx = pcpp.pcpp_mvmr_bwd_input(dev(dy, tdt), dev(w, tdt), T).cpu().numpy()
        ref, scale = oracle_bwd_input(dy, w, o, i, k, n_in)
        assert_close(gx, ref, scale, TOL[dt], what + " bwd_input")
        gw = pcpp.pcpp_mvmr_bwd_weight(dev(x, tdt), dev(dy, tdt), T).cpu().numpy()
        ref, scale = oracle_bwd_weight(x, dy, o, i, k, K)
        assert_close(gw, ref, scale, TOL[dt], what + " bwd_weight")
