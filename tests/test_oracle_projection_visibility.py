"""Pins for the oracle's projection (pi, proj_depth) and visibility mask (Sec. 3.1, Eq. 1).

None of these expectations comes from the oracle or from the GPU library: they are closed
forms worked by hand (tests/golden/pinhole_cases.txt), geometric constructions whose answer
is known in advance, and invariants of the definitions.
"""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "pinhole_cases.txt")


def _rot(axis, deg):
    a = np.deg2rad(deg)
    c, s = np.cos(a), np.sin(a)
    x, y, z = axis / np.linalg.norm(axis)
    K = np.array([[0, -z, y], [z, 0, -x], [-y, x, 0]])
    return np.eye(3) + s * K + (1 - c) * (K @ K)


def _cam(R, C, fx=250.0, fy=250.0, cx=112.0, cy=112.0):
    return np.concatenate([R.ravel(), -R @ C, [fx, fy, cx, cy]]).astype(np.float32)


def test_hand_worked_pinhole_cases(orc):
    rows = [l for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 6
    for line in rows:
        cam_s, pt_s, exp_s = line.split("|")
        cam = np.array(cam_s.split(), np.float32)
        pt = np.array(pt_s.split(), np.float32)
        exp = np.array(exp_s.split(), np.float64)
        u32, u64 = orc.project_point(cam, pt)
        assert np.array_equal(u32.astype(np.float64), exp), line   # dyadic values: exact in fp32
        assert np.array_equal(u64, exp), line


def test_point_on_principal_axis_hits_principal_point(orc):
    rng = np.random.default_rng(1)
    for _ in range(50):
        R = _rot(rng.standard_normal(3), rng.uniform(0, 180))
        C = rng.uniform(-3, 3, 3)
        s = rng.uniform(0.1, 10.0)
        cam = _cam(R, C, 250.0, 300.0, 112.0, 96.0)
        p = C + s * R[2]                      # R[2] is the forward axis in world coordinates
        u32, u64 = orc.project_point(cam, p)
        assert abs(u64[0] - 112.0) < 2e-3 and abs(u64[1] - 96.0) < 2e-3   # fp32 inputs, f = 300
        assert abs(u32[0] - 112.0) < 2e-3 and abs(u32[1] - 96.0) < 2e-3
        assert abs(u64[2] - s) < 1e-5 * max(1, s) and abs(u32[2] - s) < 1e-5 * max(1, s)


def test_offaxis_point_matches_camera_frame_closed_form(orc):
    # a point given directly in the camera frame (X, Y, Z) must land at (fx X/Z + cx, fy Y/Z + cy)
    rng = np.random.default_rng(2)
    for _ in range(50):
        R = _rot(rng.standard_normal(3), rng.uniform(0, 180))
        C = rng.uniform(-2, 2, 3)
        Xc = np.array([rng.uniform(-1, 1), rng.uniform(-1, 1), rng.uniform(1, 5)])
        p = R.T @ Xc + C
        cam = _cam(R, C, 250.0, 260.0, 112.0, 110.0)
        u32, u64 = orc.project_point(cam, p)
        exp = np.array([250.0 * Xc[0] / Xc[2] + 112.0, 260.0 * Xc[1] / Xc[2] + 110.0, Xc[2]])
        assert np.allclose(u64, exp, atol=5e-4)
        assert np.allclose(u32, exp, atol=5e-4)


def test_rigid_motion_of_scene_and_camera_leaves_projection_unchanged(orc):
    rng = np.random.default_rng(3)
    R = _rot(np.array([1.0, 2.0, 3.0]), 40.0)
    C = np.array([0.5, -2.0, 0.3])
    pts = rng.uniform(-0.5, 0.5, (20, 3))
    Q = _rot(rng.standard_normal(3), 77.0)
    s = np.array([0.3, 0.1, -0.7])
    for p in pts:
        a = orc.project_point(_cam(R, C), p)[1]
        # moved world: x' = Q x + s ; camera orientation R Q^T, centre Q C + s
        b = orc.project_point(_cam(R @ Q.T, Q @ C + s), Q @ p + s)[1]
        assert np.allclose(a, b, rtol=0, atol=2e-3)


def _plane_scene(H=32, W=32, d0=2.0):
    cam = _cam(np.eye(3), np.zeros(3), 20.0, 20.0, W / 2.0, H / 2.0)[None]
    depth = np.full((1, H, W), d0, np.float32)
    return cam, depth


def test_depth_test_is_less_or_equal_as_in_eq1(orc):
    cam, depth = _plane_scene()
    pts = np.array([[0.1, 0.1, 1.5],      # in front of the surface -> visible
                    [0.1, 0.1, 2.0],      # exactly on it: Eq. 1 is <=, so visible
                    [0.1, 0.1, 2.5],      # behind the surface -> occluded
                    [0.1, 0.1, 2.0009765625]], np.float32)   # 2 + 2^-10
    r = orc.project_visibility(cam, depth, pts, tau=0.0)
    assert r["vis"][:, 0].tolist() == [1, 1, 0, 0]
    assert r["count"].tolist() == [1, 1, 0, 0]
    r = orc.project_visibility(cam, depth, pts, tau=0.0009765625)
    assert r["vis"][:, 0].tolist() == [1, 1, 0, 1]


def test_point_behind_a_front_plane_gets_zero_weight(orc):
    # a dense fronto-parallel wall at z = 1 in front of points at z = 3: fully occluded
    cam, depth = _plane_scene(d0=1.0)
    rng = np.random.default_rng(4)
    pts = np.c_[rng.uniform(-1, 1, (100, 2)), np.full(100, 3.0)].astype(np.float32)
    r = orc.project_visibility(cam, depth, pts, tau=1e-3)
    assert r["vis"].sum() == 0 and r["count"].sum() == 0


def test_outside_behind_and_invalid_depth_are_invisible(orc):
    cam, depth = _plane_scene(d0=5.0)
    depth[0, 3, 5] = 0.0
    depth[0, 4, 5] = -1.0
    depth[0, 5, 5] = np.nan
    depth[0, 6, 5] = np.inf
    def at(px, py, z=1.0):     # a point projecting to the centre of pixel (col px, row py)
        return [(px + 0.5 - 16.0) / 20.0 * z, (py + 0.5 - 16.0) / 20.0 * z, z]
    pts = np.array([at(5, 3), at(5, 4), at(5, 5), at(5, 6), at(5, 7),
                    at(5, 7, -1.0),                # behind the camera
                    [0.0, 0.0, 0.0],               # at the camera centre
                    at(-1, 7), at(32, 7), at(5, -1), at(5, 32),     # outside each border
                    at(0, 0), at(31, 31)], np.float32)
    r = orc.project_visibility(cam, depth, pts, tau=0.0)
    assert r["vis"][:, 0].tolist() == [0, 0, 0, 1, 1, 0, 0, 0, 0, 0, 0, 1, 1]
    # without the depth test only the frustum conditions remain
    r = orc.project_visibility(cam, depth, pts, tau=0.0, flags=orc.FLAG_FRUSTUM_ONLY)
    assert r["vis"][:, 0].tolist() == [1, 1, 1, 1, 1, 0, 0, 0, 0, 0, 0, 1, 1]


def test_half_open_pixel_bounds(orc):
    # focal length 16 keeps every coordinate a dyadic rational, so the borders are hit exactly
    cam = _cam(np.eye(3), np.zeros(3), 16.0, 16.0, 16.0, 16.0)[None]
    depth = np.full((1, 32, 32), 5.0, np.float32)
    def at_uv(u, v):
        return [(u - 16.0) / 16.0, (v - 16.0) / 16.0, 1.0]
    pts = np.array([at_uv(0.0, 0.0), at_uv(31.75, 31.75), at_uv(32.0, 5.0), at_uv(5.0, 32.0),
                    at_uv(-0.25, 5.0), at_uv(5.0, -0.25)], np.float32)
    r = orc.project_visibility(cam, depth, pts, want_uvz=True)
    assert r["vis"][:, 0].tolist() == [1, 1, 0, 0, 0, 0]
    assert np.array_equal(r["uvz"][:, 0, :2],
                          np.array([[0, 0], [31.75, 31.75], [32, 5], [5, 32], [-0.25, 5], [5, -0.25]], np.float32))


def test_the_depth_texel_read_is_row_floor_v_col_floor_u(orc):
    # one far texel in an otherwise near map: only a point projecting into that texel sees through
    cam, depth = _plane_scene(d0=1.0)
    depth[0, 9, 20] = 10.0            # row 9, column 20
    z = 4.0
    def at_uv(u, v):
        return [(u - 16.0) / 20.0 * z, (v - 16.0) / 20.0 * z, z]
    pts = np.array([at_uv(20.5, 9.5), at_uv(9.5, 20.5), at_uv(20.99, 9.01), at_uv(21.01, 9.5), at_uv(20.5, 10.01)],
                   np.float32)
    r = orc.project_visibility(cam, depth, pts)
    assert r["vis"][:, 0].tolist() == [1, 0, 1, 0, 0]


def test_count_is_row_sum_and_views_permute(orc):
    from workloads.scenes import make_scene
    s = make_scene("c1", n_points=1500)
    r = orc.project_visibility(s.cam, s.depth, s.xyz, tau=s.tau)
    assert np.array_equal(r["count"], r["vis"].sum(1))
    assert 0.05 < r["vis"].mean() < 0.9
    perm = np.random.default_rng(5).permutation(s.n_views)
    r2 = orc.project_visibility(s.cam[perm], s.depth[perm], s.xyz, tau=s.tau)
    assert np.array_equal(r2["vis"], r["vis"][:, perm])
    assert np.array_equal(r2["count"], r["count"])


def test_mask_agrees_with_vectorised_float64_evaluation_away_from_thresholds(orc):
    # an independent, matrix-form float64 evaluation of Eq. 1; compared wherever the oracle's own
    # diagnostics say the pair is not within rounding of a threshold or a pixel edge
    from workloads.scenes import make_scene
    s = make_scene("c1", n_points=3000)
    r = orc.project_visibility(s.cam, s.depth, s.xyz, tau=s.tau, want_diag=True)
    X = s.xyz.astype(np.float64)
    tau = float(np.float32(s.tau))
    checked = 0
    for v in range(s.n_views):
        c = s.cam[v].astype(np.float64)
        Xc = X @ c[:9].reshape(3, 3).T + c[9:12]
        u = c[12] * Xc[:, 0] / Xc[:, 2] + c[14]
        w = c[13] * Xc[:, 1] / Xc[:, 2] + c[15]
        inside = (Xc[:, 2] > 1e-6) & (u >= 0) & (u < s.W) & (w >= 0) & (w < s.H)
        px = np.clip(np.floor(u), 0, s.W - 1).astype(int)
        py = np.clip(np.floor(w), 0, s.H - 1).astype(int)
        d = s.depth[v][py, px].astype(np.float64)
        exp = inside & (d > 0) & (Xc[:, 2] <= d + tau)
        safe = r["diag"][:, v] == 0
        assert np.array_equal(r["vis"][safe, v].astype(bool), exp[safe])
        checked += int(safe.sum())
    assert checked > 0.9 * s.N * s.n_views


def test_ragged_objects_use_their_own_views(orc):
    from workloads.scenes import make_scene
    s = make_scene("c5", n_points=400, n_objects=3, ragged_views=True)
    r = orc.project_visibility(s.cam, s.depth, s.xyz, tau=s.tau, pt_offsets=s.pt_offsets,
                               view_offsets=s.view_offsets, vis_pitch=s.vis_pitch)
    for b in range(s.B):
        p0, p1 = s.pt_offsets[b], s.pt_offsets[b + 1]
        v0, v1 = s.view_offsets[b], s.view_offsets[b + 1]
        solo = orc.project_visibility(s.cam[v0:v1], s.depth[v0:v1], s.xyz[p0:p1], tau=s.tau)
        assert np.array_equal(r["vis"][p0:p1, :v1 - v0], solo["vis"])
        assert not r["vis"][p0:p1, v1 - v0:].any()
        assert np.array_equal(r["count"][p0:p1], solo["count"])
