"""Pins for the oracle's similarity scores, Eq. 4 kernel regression (Sec. 3.4.1) and the
voxel-volume integration to mass (Sec. 3.4.2).

Expectations: hand-worked softmax cases (tests/golden/softmax_cases.txt), library routines the
steps reduce to (numpy matmul, scipy softmax), closed forms (two-material logistic form, solid
sphere mass) and invariants.  None comes from the oracle or from the GPU library.
"""
import os

import numpy as np
import pytest
from scipy.special import expit, softmax

GOLD = os.path.join(os.path.dirname(__file__), "golden", "softmax_cases.txt")


def _unit(x):
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


def _scores_setup(omega):
    """fused/temb pair whose inner products are exactly the requested scores (K <= D)."""
    omega = np.asarray(omega, np.float64)
    K = len(omega)
    temb = np.eye(K, dtype=np.float32)
    return omega[None, :], temb


def test_hand_worked_softmax_cases(orc):
    rows = [l for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 7
    for line in rows:
        T_s, om_s, y_s, rho_s = line.split("|")
        T = float(T_s)
        om = np.array(om_s.split(), np.float64) * T * np.log(2.0)
        y = np.array(y_s.split(), np.float32)
        fused, temb = _scores_setup(om)
        r = orc.material_scores(fused, temb, y[:, None], T=T)
        # T arrives as fp32 (0.1f is 1.5e-8 off 0.1), hence the 1e-6 slack on a relative scale
        assert r["prop"][0, 0] == pytest.approx(float(rho_s), rel=1e-6), line


def test_scores_are_the_matrix_product(orc):
    rng = np.random.default_rng(0)
    N, D, K = 40, 96, 7
    fused = _unit(rng.standard_normal((N, D)))
    temb = _unit(rng.standard_normal((K, D))).astype(np.float32)
    r = orc.material_scores(fused, temb)
    assert np.allclose(r["scores"], fused @ temb.astype(np.float64).T, rtol=0, atol=1e-14)
    assert np.all(np.abs(r["scores"]) <= 1 + 1e-6)
    # operand order: scores[i][k] pairs point i with material k, not the transpose
    assert r["scores"].shape == (N, K)
    assert np.allclose(r["scores"][3, 5], fused[3] @ temb[5].astype(np.float64), atol=1e-14)


def test_identical_and_orthogonal_embeddings(orc):
    D = 16
    fused = np.zeros((2, D)); fused[0, 3] = 1.0; fused[1, 7] = 1.0
    temb = np.zeros((3, D), np.float32); temb[0, 3] = 1.0; temb[1, 7] = 1.0; temb[2, 9] = 1.0
    r = orc.material_scores(fused, temb)
    assert np.array_equal(r["scores"], np.array([[1.0, 0, 0], [0, 1.0, 0]]))
    assert r["label"].tolist() == [0, 1]
    assert np.array_equal(r["margin"], np.array([1.0, 1.0]))


def test_regression_matches_library_softmax_and_is_bounded(orc):
    rng = np.random.default_rng(1)
    N, D, K, P = 60, 32, 9, 3
    fused = _unit(rng.standard_normal((N, D)))
    temb = _unit(rng.standard_normal((K, D))).astype(np.float32)
    y = rng.uniform(100, 8000, (K, P)).astype(np.float32)
    for T in (0.1, 0.02, 1.0):
        r = orc.material_scores(fused, temb, y, T=T)
        w = softmax(r["scores"] / float(np.float32(T)), axis=1)
        assert np.allclose(r["prop"], w @ y.astype(np.float64), rtol=1e-12)
        assert np.all(r["prop"] >= y.min(0) - 1e-9) and np.all(r["prop"] <= y.max(0) + 1e-9)
        assert np.array_equal(r["label"], np.argmax(r["scores"], 1))


def test_two_material_logistic_closed_form(orc):
    y = np.array([[800.0], [2700.0]], np.float32)
    for delta in (-0.3, -0.05, 0.0, 0.01, 0.2):
        fused, temb = _scores_setup([0.4 + delta, 0.4])
        r = orc.material_scores(fused, temb, y, T=0.1)
        T = float(np.float32(0.1))
        exp = 800.0 * expit(delta / T) + 2700.0 * expit(-delta / T)
        assert r["prop"][0, 0] == pytest.approx(exp, rel=1e-12)


def test_temperature_limits_and_shift_invariance(orc):
    rng = np.random.default_rng(2)
    om = rng.uniform(-0.2, 0.6, 6)
    y = rng.uniform(0, 1, (6, 2)).astype(np.float32)
    fused, temb = _scores_setup(om)
    hot = orc.material_scores(fused, temb, y, T=1e6)["prop"][0]
    assert np.allclose(hot, y.astype(np.float64).mean(0), atol=1e-6)
    cold = orc.material_scores(fused, temb, y, T=1e-4)["prop"][0]
    assert np.allclose(cold, y[np.argmax(om)].astype(np.float64), atol=1e-9)
    a = orc.material_scores(fused, temb, y, T=0.1)["prop"][0]
    b = orc.material_scores(fused + 0.125, temb, y, T=0.1)["prop"][0]
    assert np.allclose(a, b, rtol=1e-12)


def test_label_takes_lowest_index_on_exact_ties_and_zero_feature_is_uniform(orc):
    fused, temb = _scores_setup([0.25, 0.5, 0.5, 0.125])
    r = orc.material_scores(fused, temb)
    assert r["label"][0] == 1 and r["margin"][0] == 0.0
    y = np.array([[1.0], [2.0], [6.0]], np.float32)
    z = orc.material_scores(np.zeros((1, 3)), np.eye(3, dtype=np.float32), y)
    assert z["label"][0] == 0 and z["prop"][0, 0] == pytest.approx(3.0, rel=1e-15)


def test_unseen_policy_zeroes_only_all_zero_rows(orc):
    """Sec. 3.1 Eq. 2 is 0 / 0 for a point no view sees; the two readings of its property: Eq. 4 on an all-zero row (the
    mean of y: hand value 3 for y = 1, 2, 6) and zero.  A row with any non-zero element, however small, and a non-zero
    row orthogonal to every embedding (equal scores, but an observation) keep Eq. 4's value."""
    y = np.array([[1.0, 10.0], [2.0, 20.0], [6.0, 60.0]], np.float32)
    temb = np.eye(3, 4, dtype=np.float32)
    rows = np.array([[0, 0, 0, 0], [0, 0, 1e-300, 0], [0, 0, 0, 1.0], [0.5, 0.25, 0.125, 0]], np.float64)
    prior = orc.material_scores(rows, temb, y, T=0.1)
    zero = orc.material_scores(rows, temb, y, T=0.1, unseen_zero=True)
    assert np.allclose(prior["prop"][0], [3.0, 30.0], rtol=1e-15)
    assert np.array_equal(zero["prop"][0], [0.0, 0.0])
    assert np.array_equal(zero["prop"][1:], prior["prop"][1:])
    assert np.allclose(zero["prop"][2], [3.0, 30.0], rtol=1e-15)       # orthogonal but observed: still the mean
    for k in ("scores", "label", "margin"):
        assert np.array_equal(zero[k], prior[k])


# ------------------------------------------------------------------------------------ mass

def _sphere_voxels(res, r):
    h = 2.0 / res
    g = -1.0 + (np.arange(res) + 0.5) * h
    X, Y, Z = np.meshgrid(g, g, g, indexing="ij")
    m = X * X + Y * Y + Z * Z < r * r
    return np.c_[X[m], Y[m], Z[m]].astype(np.float32), h


@pytest.mark.parametrize("res,tol", [(64, 0.01), (128, 0.003)])
def test_solid_sphere_mass(orc, res, tol):
    rho0, r = 2700.0, 0.8
    pts, h = _sphere_voxels(res, r)
    prop = np.full((len(pts), 1), rho0)
    out = orc.property_integrate(prop, vol_uniform=h ** 3)
    # brute force: an integer count of voxel centres times one voxel's mass
    assert out["n_used"][0] == len(pts)
    assert out["mass"][0] == pytest.approx(len(pts) * float(np.float32(h ** 3)) * rho0, rel=1e-12)
    # closed form within the discretisation error of the grid
    assert out["mass"][0] == pytest.approx(4.0 / 3.0 * np.pi * r ** 3 * rho0, rel=tol)


def test_mass_scales_with_the_cube_of_the_scene(orc):
    rng = np.random.default_rng(3)
    pts, h = _sphere_voxels(32, 0.7)
    prop = rng.uniform(100, 8000, (len(pts), 1))
    a = orc.property_integrate(prop, vol_uniform=h ** 3)["mass"][0]
    b = orc.property_integrate(prop, vol_uniform=(2.0 * h) ** 3)["mass"][0]    # scene scaled by 2
    assert b == pytest.approx(8.0 * a, rel=1e-6)


def test_mass_is_additive_over_objects_and_skips_unseen_points(orc):
    rng = np.random.default_rng(4)
    N = 5000
    prop = rng.uniform(100, 8000, (N, 2))
    vol = rng.uniform(1e-6, 2e-6, N).astype(np.float32)
    count = rng.integers(0, 3, N).astype(np.int32)
    off = np.array([0, 100, 100, 2500, N], np.int64)            # one empty object
    whole = orc.property_integrate(prop, p_index=1, count=count, vol=vol)
    parts = orc.property_integrate(prop, p_index=1, count=count, vol=vol, pt_offsets=off)
    assert parts["mass"].shape == (4,) and parts["mass"][1] == 0 and parts["n_used"][1] == 0
    assert parts["mass"].sum() == pytest.approx(whole["mass"][0], rel=1e-12)
    assert parts["n_used"].sum() == whole["n_used"][0] == int((count > 0).sum())
    used = count > 0
    assert whole["mass"][0] == pytest.approx(float(np.sum(prop[used, 1] * vol[used].astype(np.float64))), rel=1e-12)


def test_grid_mode_averages_within_a_voxel(orc):
    lo = np.zeros((1, 3), np.float32)
    h = np.array([0.5], np.float32)                      # 4^3 grid over [0,2)^3
    pts = np.array([[0.1, 0.1, 0.1], [0.4, 0.3, 0.2],    # same voxel (0,0,0): densities 1 and 3 -> 2
                    [1.9, 0.1, 0.1],                     # voxel (3,0,0): 10
                    [0.6, 1.2, 1.7]], np.float32)        # voxel (1,2,3): 100
    prop = np.array([[1.0], [3.0], [10.0], [100.0]])
    out = orc.property_integrate(prop, xyz=pts, grid_lo=lo, grid_h=h, G=4)
    assert out["mass"][0] == pytest.approx(0.125 * (2.0 + 10.0 + 100.0), rel=1e-15)
    # points outside the cube are clamped into the border voxels
    pts2 = np.array([[-5.0, 0.1, 0.1], [0.2, 0.2, 0.2], [9.0, 9.0, 9.0]], np.float32)
    out = orc.property_integrate(np.array([[4.0], [8.0], [1.0]]), xyz=pts2, grid_lo=lo, grid_h=h, G=4)
    assert out["mass"][0] == pytest.approx(0.125 * (6.0 + 1.0), rel=1e-15)


def test_grid_mode_with_one_point_per_voxel_equals_point_volume_mode(orc):
    rng = np.random.default_rng(5)
    G = 16
    h = np.float32(0.125)
    idx = rng.choice(G ** 3, 700, replace=False)
    ijk = np.stack([idx % G, (idx // G) % G, idx // (G * G)], 1)
    pts = ((ijk + rng.uniform(0.1, 0.9, ijk.shape)) * float(h) - 1.0).astype(np.float32)
    prop = rng.uniform(100, 8000, (700, 1))
    count = rng.integers(0, 2, 700).astype(np.int32)
    a = orc.property_integrate(prop, count=count, xyz=pts, grid_lo=np.full((1, 3), -1.0, np.float32),
                               grid_h=np.array([h]), G=G)
    b = orc.property_integrate(prop, count=count, vol_uniform=float(h) ** 3)
    assert a["mass"][0] == pytest.approx(b["mass"][0], rel=1e-12)
    assert a["n_used"][0] == b["n_used"][0]


def test_grid_mode_per_object_grids(orc):
    rng = np.random.default_rng(6)
    pts = rng.uniform(0, 1, (300, 3)).astype(np.float32)
    pts[150:] += 10.0
    prop = rng.uniform(1, 2, (300, 1))
    off = np.array([0, 150, 300], np.int64)
    lo = np.array([[0, 0, 0], [10, 10, 10]], np.float32)
    h = np.array([0.25, 0.125], np.float32)
    both = orc.property_integrate(prop, pt_offsets=off, xyz=pts, grid_lo=lo, grid_h=h, G=8)
    one = orc.property_integrate(prop[150:], xyz=pts[150:], grid_lo=lo[1:], grid_h=h[1:], G=8)
    assert both["mass"][1] == pytest.approx(one["mass"][0], rel=1e-15)


def test_end_to_end_recovers_planted_materials(orc):
    # composition of the pinned parts on a generated scene: most seen points must be labelled
    # with the material planted in the views' feature maps, and the mass must sit between the
    # lightest and heaviest material filling the occupied voxels
    from workloads.scenes import make_scene
    s = make_scene("c1", n_points=4000)
    f = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, s.xyz, tau=s.tau)
    m = orc.material_scores(f["fused"], s.temb, s.y, T=s.temperature)
    seen = f["count"] > 0
    assert (m["label"][seen] == s.material_of_point[seen]).mean() > 0.8
    out = orc.property_integrate(m["prop"], count=f["count"], xyz=s.xyz, grid_lo=s.grid_lo, grid_h=s.grid_h, G=s.G)
    n_occ = len(np.unique(np.floor((s.xyz[seen] - s.grid_lo[0]) / s.grid_h[0]).astype(int), axis=0))
    v = float(s.grid_h[0]) ** 3
    assert s.y.min() * v * n_occ * 0.99 <= out["mass"][0] <= s.y.max() * v * n_occ * 1.01
