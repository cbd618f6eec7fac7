"""Pins of the oracle's variants (voxel mode, batches, voxel-grid down-sampling) against things other than
itself: a dense conv3d on the occupancy lattice, a dictionary-based sparse convolution written here, numpy.unique,
and the main oracle where the two must coincide.  CPU only."""
import itertools

import numpy as np
import pytest
import torch

import oracle


def lattice_cloud(rng, n, pitch, fill, jitter=True, per_voxel=1):
    """Points inside randomly chosen voxels of an n^3 block of a global voxel grid of the given pitch."""
    occ = rng.random((n, n, n)) < fill
    idx = np.argwhere(occ)
    idx = np.repeat(idx, per_voxel, axis=0)
    u = rng.uniform(0.1, 0.9, idx.shape) if jitter else np.full(idx.shape, 0.5)
    pts = ((idx + u) * pitch).astype(np.float32)
    perm = rng.permutation(len(pts))
    return pts[perm], idx[perm], occ


@pytest.mark.parametrize("t", [3, 5])
def test_voxel_mode_equals_dense_conv3d_on_the_occupancy_lattice(t):
    """Sec. 3.2: with the three degradations the operator is sparse voxel convolution.  One point somewhere inside
    each occupied voxel of a lattice with holes: the result at the occupied sites must equal a zero-padded dense
    3-D cross-correlation of the occupancy-masked feature volume (torch.nn.functional.conv3d)."""
    rng = np.random.default_rng(100 + t)
    n, pitch, ci, co = 7, 0.25, 3, 4
    pts, vox, occ = lattice_cloud(rng, n, pitch, 0.6)
    K = t ** 3
    x = rng.standard_normal((len(pts), ci))
    w = rng.standard_normal((K, co, ci))
    o, i, k, seg = oracle.build_triplets_general(pts, pts, pitch, t, oracle.MODE_VOXEL)
    out = oracle.mvmr_fwd(x, w, o, i, k, len(pts))
    vol = np.zeros((1, ci, n, n, n))
    vol[0, :, vox[:, 0], vox[:, 1], vox[:, 2]] = x
    wd = torch.from_numpy(w.reshape(t, t, t, co, ci).transpose(3, 4, 0, 1, 2).copy())   # [co, ci, kx, ky, kz]
    dense = torch.nn.functional.conv3d(torch.from_numpy(vol), wd, padding=t // 2)[0].numpy()
    ref = dense[:, vox[:, 0], vox[:, 1], vox[:, 2]].T
    assert np.allclose(out, ref, rtol=1e-11, atol=1e-11)
    assert seg[-1] == len(o) and (np.diff(k) >= 0).all()


def test_voxel_mode_against_a_dictionary_sparse_convolution():
    """Several points per voxel, separate output points, an independent implementation: voxel -> points dictionary,
    explicit loop over the t^3 offsets."""
    rng = np.random.default_rng(7)
    pitch, t = 0.2, 3
    pin, vin, _ = lattice_cloud(rng, 6, pitch, 0.5, per_voxel=2)
    pout, vout, _ = lattice_cloud(rng, 6, pitch, 0.4)
    o, i, k, seg = oracle.build_triplets_general(pin, pout, pitch, t, oracle.MODE_VOXEL)
    table = {}
    for j, v in enumerate(map(tuple, vin)):
        table.setdefault(v, []).append(j)
    want = []
    for oo, v in enumerate(vout):
        for cx, cy, cz in itertools.product(range(t), repeat=3):
            nb = (v[0] + cx - 1, v[1] + cy - 1, v[2] + cz - 1)          # offset = input voxel - output voxel
            for j in table.get(nb, ()):
                want.append(((cx * t + cy) * t + cz, oo, j))
    want.sort()
    assert list(zip(k.tolist(), o.tolist(), i.tolist())) == want
    assert np.array_equal(seg, np.searchsorted(k, np.arange(t ** 3 + 1)))


def test_voxel_mode_depends_on_the_voxels_only():
    """Degradation 1 (centres snapped to their voxels): moving every point inside its voxel changes nothing; points
    at the voxel centres give the same list."""
    rng = np.random.default_rng(8)
    pitch = 0.5
    pts, vox, _ = lattice_cloud(rng, 5, pitch, 0.7)
    a = oracle.build_triplets_general(pts, pts, pitch, 3, oracle.MODE_VOXEL)
    centred = ((vox + 0.5) * pitch).astype(np.float32)
    b = oracle.build_triplets_general(centred, centred, pitch, 3, oracle.MODE_VOXEL)
    moved = ((vox + rng.uniform(0.01, 0.99, vox.shape)) * pitch).astype(np.float32)
    c = oracle.build_triplets_general(moved, moved, pitch, 3, oracle.MODE_VOXEL)
    for u, v, z in zip(a, b, c):
        assert np.array_equal(u, v) and np.array_equal(u, z)
    # the self pair sits in the centre cell, and the list is symmetric under (o, i, k) -> (i, o, K-1-k)
    o, i, k, _ = a
    assert set(zip(o[o == i].tolist(), k[o == i].tolist())) == {(j, 13) for j in range(len(pts))}
    assert set(zip(o.tolist(), i.tolist(), k.tolist())) == set(zip(i.tolist(), o.tolist(), (26 - k).tolist()))


def test_voxel_mode_hand_example_and_even_t():
    # pitch 1: voxels are the unit cubes.  Output in voxel (2,2,2); inputs in voxels (1,2,2), (2,2,2), (3,3,3), (4,2,2).
    pout = np.array([[2.9, 2.1, 2.5]], np.float32)
    pin = np.array([[1.01, 2.99, 2.0], [2.0, 2.0, 2.0], [3.5, 3.5, 3.99], [4.0, 2.5, 2.5]], np.float32)
    o, i, k, seg = oracle.build_triplets_general(pin, pout, 1.0, 3, oracle.MODE_VOXEL)
    # offsets (-1,0,0) -> k = (0*3+1)*3+1 = 4; (0,0,0) -> 13; (1,1,1) -> 26; (2,0,0) outside
    assert list(zip(k.tolist(), o.tolist(), i.tolist())) == [(4, 0, 0), (13, 0, 1), (26, 0, 2)]
    # t = 5 reaches two voxels: (2,0,0) -> c = (4,2,2) -> k = (4*5+2)*5+2 = 112
    o, i, k, seg = oracle.build_triplets_general(pin, pout, 1.0, 5, oracle.MODE_VOXEL)
    assert 112 in k.tolist() and len(k) == 4
    # negative coordinates: floor, not truncation
    o, i, k, _ = oracle.build_triplets_general(np.array([[-0.1, 0.5, 0.5]], np.float32), np.array([[0.1, 0.5, 0.5]], np.float32),
                                               1.0, 3, oracle.MODE_VOXEL)
    assert k.tolist() == [4]
    with pytest.raises(ValueError):
        oracle.build_triplets_general(pin, pout, 1.0, 4, oracle.MODE_VOXEL)


def test_general_oracle_reduces_to_the_main_oracle():
    """One cloud, ball mode: the same list as pcpp_oracle.c, including ties on the ball and on cell faces."""
    rng = np.random.default_rng(9)
    for pts in (rng.uniform(0, 1, (400, 3)), rng.integers(0, 16, (500, 3)) / 8.0):
        pts = pts.astype(np.float32)
        out = pts[::3]
        for r, t in ((0.25, 3), (0.3, 4), (0.375, 5)):
            a = oracle.build_triplets(pts, out, r, t)
            b = oracle.build_triplets_general(pts, out, r, t, oracle.MODE_BALL)
            for u, v in zip(a, b):
                assert np.array_equal(u, v)


@pytest.mark.parametrize("mode", [oracle.MODE_BALL, oracle.MODE_VOXEL])
def test_batches_do_not_see_each_other(mode):
    """Sec. 4.1 (batches as one concatenated array with offsets): the triplets of a batch are the union of the
    clouds' own triplets with indices shifted; clouds that overlap in space share nothing."""
    rng = np.random.default_rng(10 + mode)
    sizes_in, sizes_out = [150, 0, 260, 90], [100, 20, 0, 90]
    clouds_in = [rng.uniform(0, 1, (n, 3)).astype(np.float32) for n in sizes_in]
    clouds_out = [rng.uniform(0, 1, (n, 3)).astype(np.float32) for n in sizes_out]
    clouds_out[3] = clouds_in[3]
    io, oo = np.cumsum([0] + sizes_in), np.cumsum([0] + sizes_out)
    size, t = 0.2, 3
    o, i, k, seg = oracle.build_triplets_general(np.concatenate(clouds_in), np.concatenate(clouds_out), size, t, mode, io, oo)
    want = set()
    for b in range(4):
        if mode == oracle.MODE_BALL:
            bo, bi, bk, _ = oracle.build_triplets(clouds_in[b], clouds_out[b], size, t)
        else:
            bo, bi, bk, _ = oracle.build_triplets_general(clouds_in[b], clouds_out[b], size, t, mode)
        want |= {(int(kk), int(a + oo[b]), int(c + io[b])) for a, c, kk in zip(bo, bi, bk)}
    got = list(zip(k.tolist(), o.tolist(), i.tolist()))
    assert got == sorted(want) and len(got) == len(want)
    assert np.array_equal(seg, np.searchsorted(k, np.arange(t ** 3 + 1)))


def test_voxel_subsample_against_numpy_unique():
    rng = np.random.default_rng(11)
    pts = np.concatenate([rng.uniform(-1, 1, (1500, 3)), rng.normal(0.3, 0.02, (500, 3))]).astype(np.float32)
    for pitch in (0.05, 0.11, 0.5):
        kept = oracle.voxel_subsample(pts, pitch)
        cell = np.floor(pts.astype(np.float64) / float(np.float32(pitch))).astype(np.int64)
        _, first = np.unique(cell, axis=0, return_index=True)
        assert np.array_equal(kept, np.sort(first))
    assert oracle.voxel_subsample(np.zeros((0, 3), np.float32), 0.1).size == 0
