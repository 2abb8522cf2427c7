"""Pins for the oracle's adaptive voxel down-sampling (Sec. 3.2.1).

Expectations: hand-worked voxel sizes (tests/golden/voxel_cases.txt), a hand-worked point set, a numpy evaluation of
voxel down-sampling built from library routines (floor, unique, add.at), a lattice whose answer is itself, and the
property the section is about: the number of sampled points does not change with the scale of the object."""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "voxel_cases.txt")


def test_hand_worked_voxel_sizes(orc):
    rows = [l for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 9
    for line in rows:
        lo, hi, nt, s, dims = [c.strip() for c in line.split("|")]
        got_s, got_dims = orc.voxel_grid(np.array(lo.split(), np.float32), np.array(hi.split(), np.float32), int(nt))
        assert np.isclose(got_s, float(s), rtol=1e-6), line       # 0.1 is not an fp32 number
        assert list(got_dims) == [int(x) for x in dims.split()], line


def test_hand_worked_point_set(orc):
    # box 0..2 cubed, N_target 8: unit voxels.  Two points share the first voxel; (1.5, 0.2, 0.2) is in voxel (1, 0, 0),
    # the corner (2, 2, 2) in voxel (2, 2, 2); the list is ordered by (z * 3 + y) * 3 + x
    xyz = np.array([[0, 0, 0], [0.5, 0.25, 0.125], [2, 2, 2], [1.5, 0.25, 0.25], [0.25, 0.5, 0.75]], np.float32)
    r = orc.voxel_downsample(xyz, 8)
    assert np.array_equal(r["xyz"], [[0.25, 0.25, 0.875 / 3], [1.5, 0.25, 0.25], [2, 2, 2]])
    assert list(r["count"]) == [3, 1, 1] and list(r["voxel_of_point"]) == [0, 0, 2, 1, 0] and list(r["offsets"]) == [0, 3]


def _numpy_reference(xyz, lo, hi, n_target):
    e = (hi - lo).astype(np.float32)
    vol = float(e[0]) * float(e[1]) * float(e[2])
    s = np.float32(np.cbrt(vol / n_target))
    dims = np.floor(e / s).astype(np.int64) + 1
    q = np.floor((xyz - lo).astype(np.float32) / s).astype(np.int64)
    q = np.clip(q, 0, dims - 1)
    lin = (q[:, 2] * dims[1] + q[:, 1]) * dims[0] + q[:, 0]
    keys, inv, cnt = np.unique(lin, return_inverse=True, return_counts=True)
    sums = np.zeros((len(keys), 3))
    np.add.at(sums, inv, xyz.astype(np.float64))
    return sums / cnt[:, None], cnt, inv


@pytest.mark.parametrize("seed,n,n_target", [(1, 5000, 150), (2, 777, 30), (3, 20000, 1000), (4, 50, 150)])
def test_against_library_routines(orc, seed, n, n_target):
    rng = np.random.default_rng(seed)
    xyz = (rng.normal(size=(n, 3)) * [1.0, 0.4, 0.7] + [3, -2, 0.5]).astype(np.float32)
    lo, hi = xyz.min(0), xyz.max(0)
    r = orc.voxel_downsample(xyz, n_target)
    want_xyz, want_cnt, want_inv = _numpy_reference(xyz, lo, hi, n_target)
    assert np.array_equal(r["count"], want_cnt) and np.array_equal(r["voxel_of_point"], want_inv)
    assert np.allclose(r["xyz"], want_xyz, rtol=1e-13, atol=1e-13)
    assert r["count"].sum() == n and r["offsets"][-1] == len(want_cnt)
    # the count lands near the target (the section: "slightly lower than N_target" for a filled box; a cloud that
    # does not fill its box occupies fewer voxels)
    assert len(want_cnt) <= min(n, np.prod(orc.voxel_grid(lo, hi, n_target)[1]))


def test_lattice_is_its_own_sample(orc):
    # centres of a 5 x 4 x 3 lattice of unit cubes, box = the lattice's hull grown by half a cube: one point per voxel
    g = np.stack(np.meshgrid(np.arange(5), np.arange(4), np.arange(3), indexing="ij"), -1).reshape(-1, 3).astype(np.float32)
    pts = g + 0.5
    r = orc.voxel_downsample(pts, 60, box_lo=[[0, 0, 0]], box_hi=[[5, 4, 3]])
    assert len(r["xyz"]) == 60 and (r["count"] == 1).all()
    order = np.lexsort((pts[:, 0], pts[:, 1], pts[:, 2]))            # z slowest, x fastest
    assert np.array_equal(r["xyz"], pts[order].astype(np.float64))
    # every point doubled: same sample, counts 2
    r2 = orc.voxel_downsample(np.concatenate([pts, pts]), 60, box_lo=[[0, 0, 0]], box_hi=[[5, 4, 3]])
    assert np.array_equal(r2["xyz"], r["xyz"]) and (r2["count"] == 2).all()


def test_sample_count_does_not_follow_object_scale(orc):
    """The point of Sec. 3.2.1: with s_voxel tied to the box, a larger copy of the object yields the same sample."""
    rng = np.random.default_rng(9)
    xyz = rng.uniform(-1, 1, (4000, 3)).astype(np.float32)
    base = orc.voxel_downsample(xyz, 150)
    for scale in (0.125, 4.0, 64.0):                 # powers of two: every fp32 operation scales exactly
        r = orc.voxel_downsample(xyz * np.float32(scale), 150)
        assert np.array_equal(r["count"], base["count"]) and np.array_equal(r["voxel_of_point"], base["voxel_of_point"])
        assert np.allclose(r["xyz"], base["xyz"] * scale, rtol=1e-15, atol=0)
    # while a fixed voxel size would not: the same cloud scaled by 4 in a grid made for the small one has more voxels
    fixed = orc.voxel_downsample(xyz * np.float32(4.0), 150 * 64)
    assert len(fixed["xyz"]) > 3 * len(base["xyz"])
    # a higher target gives a finer grid: s scales with the cube root
    s150, _ = orc.voxel_grid([-1, -1, -1], [1, 1, 1], 150)
    s1200, _ = orc.voxel_grid([-1, -1, -1], [1, 1, 1], 1200)
    assert np.isclose(s150 / s1200, 2.0, rtol=1e-6)


def test_objects_capacity_and_degenerate_boxes(orc):
    rng = np.random.default_rng(2)
    a = rng.uniform(0, 1, (300, 3)).astype(np.float32)
    b = rng.uniform(5, 9, (500, 3)).astype(np.float32)
    po = np.array([0, 300, 300, 800], np.int64)                    # the middle object is empty
    both = orc.voxel_downsample(np.concatenate([a, b]), 40, pt_offsets=po)
    ra, rb = orc.voxel_downsample(a, 40), orc.voxel_downsample(b, 40)
    assert list(both["offsets"]) == [0, len(ra["xyz"]), len(ra["xyz"]), len(ra["xyz"]) + len(rb["xyz"])]
    assert np.array_equal(both["xyz"], np.concatenate([ra["xyz"], rb["xyz"]]))
    assert np.array_equal(both["voxel_of_point"], np.concatenate([ra["voxel_of_point"], rb["voxel_of_point"] + len(ra["xyz"])]))
    # fewer slots than voxels: the first ones are written, the total is still reported
    cut = orc.voxel_downsample(a, 40, capacity=5)
    assert len(cut["xyz"]) == 5 and cut["offsets"][-1] == len(ra["xyz"]) and np.array_equal(cut["xyz"], ra["xyz"][:5])
    # points on a plane: the flat-box rule; identical points: one voxel
    flat = np.concatenate([rng.uniform(0, 4, (200, 2)), np.full((200, 1), 7.0)], 1).astype(np.float32)
    rf = orc.voxel_downsample(flat, 64)
    assert 10 < len(rf["xyz"]) <= 36 and (rf["xyz"][:, 2] == 7.0).all()
    same = orc.voxel_downsample(np.full((10, 3), 2.5, np.float32), 150)
    assert len(same["xyz"]) == 1 and same["count"][0] == 10 and np.array_equal(same["xyz"][0], [2.5, 2.5, 2.5])
    # points outside a given box are binned into its border voxels
    out = orc.voxel_downsample(np.array([[-5, 0.5, 0.5], [9, 0.5, 0.5]], np.float32), 8, box_lo=[[0, 0, 0]], box_hi=[[2, 2, 2]])
    assert list(out["voxel_of_point"]) == [0, 1] and len(out["xyz"]) == 2
