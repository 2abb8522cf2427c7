"""Pins for the oracle's normal estimation (Sec. 3.2.2: normals of the sampled points, needed by S_angle).

Expectations: surfaces whose normal is known in closed form (plane, sphere, cylinder), scipy's k-d tree as an
independent nearest-neighbour search, and invariants.  None comes from the oracle or from the GPU library."""
import numpy as np
import pytest
from scipy.spatial import cKDTree


def _rot(axis, deg):
    a = np.deg2rad(deg)
    c, s = np.cos(a), np.sin(a)
    x, y, z = np.asarray(axis, float) / np.linalg.norm(axis)
    K = np.array([[0, -z, y], [z, 0, -x], [-y, x, 0]])
    return np.eye(3) + s * K + (1 - c) * (K @ K)


def test_plane(orc):
    rng = np.random.default_rng(1)
    Q = _rot([1, 2, 0.5], 33)
    flat = np.concatenate([rng.uniform(-1, 1, (3000, 2)), np.zeros((3000, 1))], 1)
    pts = (flat @ Q.T + [0.3, -0.2, 1.0]).astype(np.float32)
    n_true = Q[:, 2]
    centre = (np.array([0.3, -0.2, 1.0]) - 2.0 * n_true).astype(np.float32)     # the object's inside is below the plane
    r = orc.estimate_normals(pts, pts[:50], centre, 20)
    assert np.abs(r["normals"] @ n_true - 1.0).max() < 1e-6                     # fp32 coordinates
    assert np.allclose(np.linalg.norm(r["normals"], axis=1), 1.0, atol=1e-12)
    assert (r["evals"][:, 0] < 1e-12).all()
    # the centre on the other side turns every normal over
    r2 = orc.estimate_normals(pts, pts[:50], centre + 4.0 * n_true.astype(np.float32), 20)
    assert np.allclose(r2["normals"], -r["normals"], atol=1e-12)


def test_sphere_and_cylinder(orc):
    rng = np.random.default_rng(2)
    d = rng.standard_normal((40000, 3))
    d /= np.linalg.norm(d, axis=1, keepdims=True)
    c = np.array([1.0, 2.0, -0.5])
    pts = (c + 0.8 * d).astype(np.float32)
    r = orc.estimate_normals(pts, pts[:200], c.astype(np.float32), 30)
    cosang = np.einsum("ij,ij->i", r["normals"], d[:200])
    assert cosang.min() > np.cos(np.deg2rad(3.0))            # 30 of 40 000 neighbours: a cap of about 2.5 degrees
    # cylinder along z: the normal has no z component and points away from the axis
    ang, h = rng.uniform(0, 2 * np.pi, 40000), rng.uniform(-1, 1, 40000)
    cyl = np.stack([0.5 * np.cos(ang), 0.5 * np.sin(ang), h], 1).astype(np.float32)
    q = np.nonzero(np.abs(h) < 0.8)[0][:200]
    r = orc.estimate_normals(cyl, cyl[q], [0, 0, 0], 30)
    radial = np.stack([np.cos(ang[q]), np.sin(ang[q]), np.zeros(len(q))], 1)
    assert np.einsum("ij,ij->i", r["normals"], radial).min() > np.cos(np.deg2rad(4.0))
    assert np.abs(r["normals"][:, 2]).max() < 0.1


def test_neighbours_against_a_kd_tree(orc):
    rng = np.random.default_rng(3)
    pts = rng.uniform(-1, 1, (5000, 3)).astype(np.float32)
    qs = rng.uniform(-1, 1, (100, 3)).astype(np.float32)
    k = 16
    r = orc.estimate_normals(pts, qs, [0, 0, 0], k)
    dist, idx = cKDTree(pts.astype(np.float64)).query(qs.astype(np.float64), k=k + 1)
    clear = (dist[:, k] ** 2 - dist[:, k - 1] ** 2) > 1e-6      # the k-th and the next one apart by more than fp32 rounding
    assert clear.mean() > 0.95
    assert np.array_equal(np.sort(r["nn_idx"][clear], 1), np.sort(idx[clear, :k], 1))
    for m in np.nonzero(clear)[0][:20]:                         # and the normal is the smallest eigenvector of their covariance
        nb = pts[idx[m, :k]].astype(np.float64)
        w, v = np.linalg.eigh(np.cov(nb.T, bias=True))
        assert abs(abs(r["normals"][m] @ v[:, 0]) - 1.0) < 1e-9 and np.allclose(r["evals"][m], w, rtol=1e-9, atol=1e-15)


def test_ties_small_clouds_objects_and_rotation(orc):
    # four points at the same distance from the query: the lower indices are taken first
    pts = np.array([[1, 0, 0], [0, 1, 0], [-1, 0, 0], [0, -1, 0], [0, 0, 0.5], [3, 3, 3]], np.float32)
    r = orc.estimate_normals(pts, [[0, 0, 0]], [0, 0, -1], 3)
    assert list(r["nn_idx"][0]) == [4, 0, 1] and r["gap"][0] == 0.0
    # fewer points than k: all of them; a square in the plane z = 0 seen from below
    r = orc.estimate_normals(pts[:4], [[0, 0, 0]], [0, 0, -1], 30)
    assert list(r["nn_idx"][0][:4]) == [0, 1, 2, 3] and (r["nn_idx"][0][4:] == -1).all()
    assert np.allclose(r["normals"][0], [0, 0, 1], atol=1e-12)
    # two objects: neighbours come from the query's own object only
    rng = np.random.default_rng(5)
    a = np.concatenate([rng.uniform(-1, 1, (500, 2)), np.zeros((500, 1))], 1).astype(np.float32)              # plane z = 0
    b = np.concatenate([np.zeros((500, 1)), rng.uniform(-1, 1, (500, 2))], 1).astype(np.float32)              # plane x = 0
    both = orc.estimate_normals(np.concatenate([a, b]), np.array([[0.1, 0.1, 0], [0, 0.1, 0.1]], np.float32),
                                [[0, 0, -1], [-1, 0, 0]], 10, pt_offsets=[0, 500, 1000], q_offsets=[0, 1, 2])
    assert np.allclose(both["normals"], [[0, 0, 1], [1, 0, 0]], atol=1e-6) and both["nn_idx"].max() < 500
    # a rotation of everything rotates the normals
    Q = _rot([0.3, 1, 0.2], 50)
    d = rng.standard_normal((3000, 3)) * [1.0, 0.6, 0.3]
    surf = (d / np.linalg.norm(d, axis=1, keepdims=True) * [1.0, 0.6, 0.3]).astype(np.float32)                 # an ellipsoid
    base = orc.estimate_normals(surf, surf[:40], [0, 0, 0], 12)
    turned = orc.estimate_normals((surf.astype(np.float64) @ Q.T).astype(np.float32), (surf[:40].astype(np.float64) @ Q.T).astype(np.float32),
                                  [0, 0, 0], 12)
    stable = (base["gap"] > 1e-5) & ((base["evals"][:, 1] - base["evals"][:, 0]) > 0.05 * base["evals"][:, 2])
    assert stable.sum() > 20
    assert np.abs(np.einsum("ij,ij->i", turned["normals"][stable], base["normals"][stable] @ Q.T) - 1.0).max() < 1e-4
