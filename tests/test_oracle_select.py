"""Pins for the oracle's view importance-based filtering (Sec. 3.2.2) and the mean over the kept views (Sec. 3.2.3).

Expectations: hand-worked 3-4-5 cases (tests/golden/view_score_cases.txt), camera rigs whose ranking is known in
advance, a numpy evaluation of the definition, and invariants.  None comes from the oracle's selection code or
from the GPU library (the visibility gate used by the numpy evaluation is the Eq. 1 mask pinned in
test_oracle_projection_visibility.py)."""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "view_score_cases.txt")
FRUSTUM_ONLY = 1


def _rot(axis, deg):
    a = np.deg2rad(deg)
    c, s = np.cos(a), np.sin(a)
    x, y, z = np.asarray(axis, float) / np.linalg.norm(axis)
    K = np.array([[0, -z, y], [z, 0, -x], [-y, x, 0]])
    return np.eye(3) + s * K + (1 - c) * (K @ K)


def _cam(R, C, f=100.0, c=500.0):
    return np.concatenate([np.asarray(R, float).ravel(), -np.asarray(R, float) @ np.asarray(C, float), [f, f, c, c]]).astype(np.float32)


def test_hand_worked_scores(orc):
    rows = [l for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 9
    for line in rows:
        name, cam, pt, nrm, sd, sa, st = [c.strip() for c in line.split("|")]
        cam = np.array(cam.split(), np.float32)
        r = orc.select_views(cam, None, np.array(pt.split(), np.float32), np.array(nrm.split(), np.float32), 1,
                             flags=FRUSTUM_ONLY, H=1000, W=1000)
        assert r["n_sel"][0] == 1 and r["sel_view"][0, 0] == 0, name
        assert np.isclose(r["sel_score"][0, 0], float(st), rtol=1e-6, atol=1e-7), (name, r["sel_score"])   # fp32 inputs
        assert np.isclose(float(sd) * float(sa), float(st), rtol=1e-12), name


def _line_of_cameras(dists):
    """Cameras on the -z axis at the given distances from the origin, all looking along +z."""
    return np.stack([_cam(np.eye(3), [0, 0, -d]) for d in dists])


def test_nearer_views_rank_first(orc):
    # the point at the origin faces the cameras: S_total = 1 / (1 + distance)
    dists = [4.0, 1.0, 3.0, 0.5, 2.0]
    r = orc.select_views(_line_of_cameras(dists), None, [0, 0, 0], [0, 0, -1], 3, flags=FRUSTUM_ONLY, H=1000, W=1000)
    assert list(r["sel_view"][0]) == [3, 1, 4]
    assert np.allclose(r["sel_score"][0], [1 / 1.5, 1 / 2.0, 1 / 3.0], rtol=1e-7)
    assert list(r["sel_mask"][0]) == [0, 1, 0, 1, 1] and r["n_sel"][0] == 3
    assert np.isclose(r["gap"][0], 1 / 3.0 - 1 / 4.0, rtol=1e-6)


def test_equal_scores_keep_the_lower_index_and_zero_scores_come_last(orc):
    front = _line_of_cameras([2.0, 2.0, 1.0])
    behind = _cam(_rot([0, 1, 0], 180), [0, 0, 1.0])[None]      # on the far side, looking back at the point
    cams = np.concatenate([behind, front])
    r = orc.select_views(cams, None, [0, 0, 0], [0, 0, -1], 4, flags=FRUSTUM_ONLY, H=1000, W=1000)
    # view 0 sees the back of the surface: score 0, still visible, ranked after every positive score
    assert list(r["sel_view"][0]) == [3, 1, 2, 0]
    assert np.allclose(r["sel_score"][0], [0.5, 1 / 3, 1 / 3, 0.0], rtol=1e-7)
    r = orc.select_views(cams, None, [0, 0, 0], [0, 0, -1], 2, flags=FRUSTUM_ONLY, H=1000, W=1000)
    assert list(r["sel_view"][0]) == [3, 1] and np.isclose(r["gap"][0], 0.0, atol=1e-12)


def test_only_visible_views_compete(orc):
    cams = _line_of_cameras([0.5, 1.0, 2.0, 3.0])
    depth = np.full((4, 1000, 1000), np.inf, np.float32)
    depth[0] = 0.25                        # a wall in front of the nearest camera: Eq. 1 fails there
    depth[2] = 2.0                         # the surface itself
    depth[1] = np.nan                      # invalid depth
    r = orc.select_views(cams, depth, [0, 0, 0], [0, 0, -1], 3)
    assert list(r["sel_view"][0]) == [2, 3, -1] and r["n_sel"][0] == 2
    assert list(r["sel_mask"][0]) == [0, 0, 1, 1]
    assert np.allclose(r["sel_score"][0], [1 / 3, 1 / 4, 0.0], rtol=1e-7) and r["gap"][0] == np.inf
    # a point no camera sees keeps nothing
    r = orc.select_views(cams, depth, [0, 0, -10], [0, 0, -1], 3)
    assert list(r["sel_view"][0]) == [-1, -1, -1] and r["n_sel"][0] == 0 and not r["sel_mask"].any()


def _numpy_scores(cam, xyz, normals):
    """S_total of every pair from the definition, vectorised: [N][V]."""
    cam = cam.astype(np.float64)
    R, t = cam[:, :9].reshape(-1, 3, 3), cam[:, 9:12]
    C = -np.einsum("vji,vj->vi", R, t)
    ray = xyz[:, None, :].astype(np.float64) - C[None]
    z = xyz.astype(np.float64) @ R[:, 2].T + t[:, 2]          # depth in the camera frame Xc = R x + t
    v = ray / np.linalg.norm(ray, axis=2, keepdims=True)
    s_angle = np.maximum(0.0, -np.einsum("nvj,nj->nv", v, normals.astype(np.float64)))
    return s_angle / (1.0 + z)


@pytest.mark.parametrize("name,k", [("c1", 3), ("c5", 2), ("c1", 8)])
def test_against_numpy_on_a_scene(orc, name, k):
    from workloads.scenes import make_scene, synthetic_normals
    s = make_scene(name, n_points=3000, n_objects=3) if name == "c5" else make_scene(name, n_points=3000)
    nrm = synthetic_normals(s.xyz, s.pt_offsets, 3)
    single = s.B == 1
    po, vo = (None, None) if single else (s.pt_offsets, s.view_offsets)
    r = orc.select_views(s.cam, s.depth, s.xyz, nrm, k, tau=s.tau, z_near=s.z_near, pt_offsets=po, view_offsets=vo)
    vis = orc.project_visibility(s.cam, s.depth, s.xyz, tau=s.tau, z_near=s.z_near, pt_offsets=po, view_offsets=vo,
                                 vis_pitch=s.vis_pitch)["vis"]
    assert vis.mean() > 0.2
    for b in range(s.B):
        ps = slice(int(s.pt_offsets[b]), int(s.pt_offsets[b + 1]))
        vs = slice(int(s.view_offsets[b]), int(s.view_offsets[b + 1]))
        nv = vs.stop - vs.start
        S = _numpy_scores(s.cam[vs], s.xyz[ps], nrm[ps])
        S = np.where(vis[ps, :nv] > 0, S, -1.0)
        order = np.argsort(-S, axis=1, kind="stable")[:, :k]
        top = np.take_along_axis(S, order, 1)
        want_view = np.where(top >= 0, order, -1)
        if want_view.shape[1] < k:
            want_view = np.pad(want_view, ((0, 0), (0, k - nv)), constant_values=-1)
            top = np.pad(top, ((0, 0), (0, k - nv)), constant_values=-1)
        # away from near-ties the ranking is identical (exactly equal scores, e.g. several views that see the back
        # of the surface, go by view index on both sides); the scores agree to rounding everywhere
        srt = -np.sort(-S, axis=1)
        d = srt[:, :-1] - srt[:, 1:]
        clear = ~((d[:, :k] > 0) & (d[:, :k] <= 1e-9)).any(1)
        assert clear.mean() > 0.95
        assert np.array_equal(r["sel_view"][ps][clear], want_view[clear])
        assert np.allclose(r["sel_score"][ps], np.maximum(top, 0.0), rtol=1e-9, atol=1e-12)
        assert np.allclose(r["score_all"][ps, :nv], S, rtol=1e-9, atol=1e-12)
        assert np.array_equal(r["n_sel"][ps], np.minimum(k, (vis[ps] > 0).sum(1)))
    # structure: the mask marks exactly the kept views, all of them visible, in descending score order
    assert np.array_equal(r["sel_mask"].sum(1), r["n_sel"])
    assert not (r["sel_mask"] & ~(vis > 0)).any()
    assert (np.diff(r["sel_score"], axis=1) <= 0).all() and (r["gap"] >= 0).all()
    rows, cols = np.nonzero(r["sel_view"] >= 0)
    assert r["sel_mask"][rows, r["sel_view"][rows, cols]].all()


def test_invariants(orc):
    rng = np.random.default_rng(4)
    V, N = 6, 200
    cams = np.stack([_cam(_rot(rng.standard_normal(3), rng.uniform(-25, 25)), rng.uniform(-0.5, 0.5, 3) + [0, 0, -4]) for _ in range(V)])
    xyz = rng.uniform(-0.8, 0.8, (N, 3)).astype(np.float32)
    nrm = rng.standard_normal((N, 3))
    nrm = (nrm / np.linalg.norm(nrm, axis=1, keepdims=True)).astype(np.float32)
    base = orc.select_views(cams, None, xyz, nrm, 3, flags=FRUSTUM_ONLY, H=1000, W=1000)
    assert (base["n_sel"] == 3).all()
    # a rigid motion of points, normals and cameras together changes nothing (to fp32 rounding of the moved inputs)
    Q, shift = _rot([1, 2, 3], 40), np.array([0.5, -1.0, 2.0])
    cams2 = np.stack([_cam(c[:9].reshape(3, 3).astype(np.float64) @ Q.T,
                           Q @ (-c[:9].reshape(3, 3).astype(np.float64).T @ c[9:12]) + shift) for c in cams])
    moved = orc.select_views(cams2, None, xyz @ Q.T + shift, nrm @ Q.T, 3, flags=FRUSTUM_ONLY, H=1000, W=1000)
    assert np.allclose(moved["score_all"], base["score_all"], rtol=0, atol=2e-6)
    # turning every surface away leaves only zero scores; the kept views are then the first visible ones
    away = orc.select_views(cams, None, xyz, -nrm, 3, flags=FRUSTUM_ONLY, H=1000, W=1000)
    both = np.minimum(base["score_all"], away["score_all"])
    assert (both == 0).all()                                   # a view cannot face both sides of a surface
    # reordering the views permutes the result
    perm = rng.permutation(V)
    pr = orc.select_views(cams[perm], None, xyz, nrm, 3, flags=FRUSTUM_ONLY, H=1000, W=1000)
    assert np.allclose(pr["score_all"], base["score_all"][:, perm], rtol=0, atol=0)
    clear = base["gap"] > 1e-9
    assert np.array_equal(np.sort(perm[pr["sel_view"][clear]], 1), np.sort(base["sel_view"][clear], 1))
    # k beyond the number of views keeps every visible view
    allv = orc.select_views(cams, None, xyz, nrm, V + 2, flags=FRUSTUM_ONLY, H=1000, W=1000)
    assert (allv["n_sel"] == V).all() and (allv["sel_view"][:, V:] == -1).all() and (allv["gap"] == np.inf).all()


def test_fusion_over_the_kept_views(orc):
    """Sec. 3.2.3: the fused feature is the mean over the kept views.  With every visible view kept it is Eq. 2;
    with one view kept it is that view's sample, normalised."""
    from workloads.scenes import make_scene, synthetic_normals
    s = make_scene("c1", n_points=400)
    nrm = synthetic_normals(s.xyz, s.pt_offsets, 5)
    plain = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, s.xyz, tau=s.tau, z_near=s.z_near)
    vis = orc.project_visibility(s.cam, s.depth, s.xyz, tau=s.tau, z_near=s.z_near)["vis"]
    everything = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, s.xyz, tau=s.tau, z_near=s.z_near, sel_mask=vis)
    assert np.array_equal(everything["fused"], plain["fused"]) and np.array_equal(everything["count"], plain["count"])
    sel = orc.select_views(s.cam, s.depth, s.xyz, nrm, 1, tau=s.tau, z_near=s.z_near)
    one = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, s.xyz, tau=s.tau, z_near=s.z_near, sel_mask=sel["sel_mask"])
    assert np.array_equal(one["count"], sel["n_sel"])
    for i in np.nonzero(sel["n_sel"] == 1)[0][:50]:
        v = sel["sel_view"][i, 0]
        u32, _ = orc.project_point(s.cam[v], s.xyz[i])
        f = orc.sample_bilinear(s.feat[v], s.feat_dtype, s.H, s.W, u32[0], u32[1])
        assert np.allclose(one["fused"][i], f / np.linalg.norm(f), rtol=1e-12, atol=1e-15)
    # two kept views: the normalised mean of the two samples
    sel2 = orc.select_views(s.cam, s.depth, s.xyz, nrm, 2, tau=s.tau, z_near=s.z_near)
    two = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, s.xyz, tau=s.tau, z_near=s.z_near, sel_mask=sel2["sel_mask"],
                            flags=2)   # mean only
    for i in np.nonzero(sel2["n_sel"] == 2)[0][:50]:
        fs = []
        for v in sel2["sel_view"][i]:
            u32, _ = orc.project_point(s.cam[v], s.xyz[i])
            fs.append(orc.sample_bilinear(s.feat[v], s.feat_dtype, s.H, s.W, u32[0], u32[1]))
        assert np.allclose(two["fused"][i], 0.5 * (fs[0] + fs[1]), rtol=1e-12, atol=1e-15)
