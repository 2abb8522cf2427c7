"""Pins for the oracle's feature sampling and aggregation (Sec. 3.1, Eq. 2).

Expectations are closed forms of bilinear interpolation, a library routine that the sampling
reduces to (torch.nn.functional.grid_sample), exact element-widening by numpy/torch, and
invariants of Eq. 2.  None comes from the oracle or from the GPU library.
"""
import numpy as np
import pytest
import torch

from workloads.scenes import make_scene, store, stored_to_f32


def _front_cam(H, W, f=20.0):
    return np.array([1, 0, 0, 0, 1, 0, 0, 0, 1, 0, 0, 0, f, f, W / 2.0, H / 2.0], np.float32)[None]


def _pt(u, v, H, W, f=20.0, z=1.0):
    return [(u - W / 2.0) / f * z, (v - H / 2.0) / f * z, z]


def test_cell_centre_returns_that_cell(orc):
    rng = np.random.default_rng(0)
    Hf, Wf, D, H, W = 4, 8, 5, 56, 112          # pitch 14 in both axes
    F = rng.standard_normal((Hf, Wf, D)).astype(np.float32)
    for r in range(Hf):
        for c in range(Wf):
            out = orc.sample_bilinear(F, "f32", H, W, (c + 0.5) * 14.0, (r + 0.5) * 14.0)
            assert np.array_equal(out, F[r, c].astype(np.float64))


def test_affine_map_is_reproduced_between_cell_centres(orc):
    # F = a*col + b*row + c is linear, so bilinear blending must return the same affine function
    # of the continuous grid coordinate g = u/pitch - 0.5 (this pins the half-cell alignment)
    Hf, Wf, H, W = 6, 5, 48, 40                  # pitch 8
    col, row = np.meshgrid(np.arange(Wf), np.arange(Hf))
    F = np.stack([2.0 * col - 3.0 * row + 1.0, 0.5 * col + 0.25 * row - 4.0], -1).astype(np.float32)
    rng = np.random.default_rng(1)
    for _ in range(200):
        u = float(np.float32(rng.uniform(4.0, W - 4.0)))     # between the first and last cell centres
        v = float(np.float32(rng.uniform(4.0, H - 4.0)))
        gx, gy = u / 8.0 - 0.5, v / 8.0 - 0.5
        out = orc.sample_bilinear(F, "f32", H, W, u, v)
        exp = [2.0 * gx - 3.0 * gy + 1.0, 0.5 * gx + 0.25 * gy - 4.0]
        assert np.allclose(out, exp, rtol=0, atol=1e-5)


def test_one_hot_map_returns_the_four_bilinear_weights(orc):
    Hf, Wf, H, W = 4, 4, 32, 32                  # pitch 8
    u, v = 13.0, 18.0                            # g = (1.125, 1.75): cells x 1|2, y 1|2
    got = np.zeros((Hf, Wf))
    for r in range(Hf):
        for c in range(Wf):
            F = np.zeros((Hf, Wf, 1), np.float32)
            F[r, c, 0] = 1.0
            got[r, c] = orc.sample_bilinear(F, "f32", H, W, u, v)[0]
    exp = np.zeros((Hf, Wf))
    exp[1, 1], exp[1, 2], exp[2, 1], exp[2, 2] = 0.25 * 0.875, 0.25 * 0.125, 0.75 * 0.875, 0.75 * 0.125
    assert np.array_equal(got, exp)
    assert got.min() >= 0 and got.sum() == 1.0


def test_border_is_replicated(orc):
    Hf, Wf, H, W = 3, 3, 24, 24
    F = np.arange(9, dtype=np.float32).reshape(3, 3, 1)
    assert orc.sample_bilinear(F, "f32", H, W, 0.0, 0.0)[0] == 0.0
    assert orc.sample_bilinear(F, "f32", H, W, 23.9, 23.9)[0] == 8.0
    assert orc.sample_bilinear(F, "f32", H, W, 1.0, 12.0)[0] == 3.0       # left of the first centre: row 1, col 0
    assert orc.sample_bilinear(F, "f32", H, W, 12.0, 23.0)[0] == 7.0      # below the last centre


def test_pixel_aligned_map_sampled_at_pixel_centres(orc):
    rng = np.random.default_rng(2)
    F = rng.standard_normal((7, 9, 3)).astype(np.float32)
    for r in range(7):
        for c in range(9):
            assert np.array_equal(orc.sample_bilinear(F, "f32", 7, 9, c + 0.5, r + 0.5), F[r, c].astype(np.float64))


@pytest.mark.parametrize("Hf,Wf,H,W", [(16, 16, 224, 224), (5, 7, 40, 56), (9, 9, 9, 9)])
def test_sampling_reduces_to_grid_sample_border_mode(orc, Hf, Wf, H, W):
    # library routine: bilinear grid_sample with align_corners=False and border padding uses the
    # same cell-centre alignment and clamps the coordinate to the outermost cell centres
    rng = np.random.default_rng(3)
    D = 6
    F = rng.standard_normal((Hf, Wf, D))
    uv = np.c_[rng.uniform(0, W, 300), rng.uniform(0, H, 300)].astype(np.float32)
    grid = torch.from_numpy(np.c_[2.0 * uv[:, 0].astype(np.float64) / W - 1.0,
                                  2.0 * uv[:, 1].astype(np.float64) / H - 1.0]).reshape(1, 1, -1, 2)
    ref = torch.nn.functional.grid_sample(torch.from_numpy(F).permute(2, 0, 1)[None], grid, mode="bilinear",
                                          padding_mode="border", align_corners=False)[0, :, 0].T.numpy()
    F32 = F.astype(np.float32)
    ref32 = torch.nn.functional.grid_sample(torch.from_numpy(F32.astype(np.float64)).permute(2, 0, 1)[None], grid,
                                            mode="bilinear", padding_mode="border",
                                            align_corners=False)[0, :, 0].T.numpy()
    for i, (u, v) in enumerate(uv):
        out = orc.sample_bilinear(F32, "f32", H, W, float(u), float(v))
        assert np.allclose(out, ref32[i], rtol=0, atol=2e-5), (i, u, v)
    assert np.allclose(ref, ref32, atol=1e-5)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_half_precision_elements_widen_exactly(orc, dtype):
    rng = np.random.default_rng(4)
    x = (rng.standard_normal((3, 3, 64)) * np.exp(rng.uniform(-12, 4, (3, 3, 64)))).astype(np.float32)
    x[0, 0, :4] = [0.0, -0.0, 6.0e-8, -6.1e-5]           # zero and fp16 subnormals
    st = store(x, dtype)
    if dtype == "bf16":      # torch's own bf16 -> fp32 widening
        ref = torch.from_numpy(st.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
        assert np.array_equal(torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy(), ref)  # RNE storage
    else:
        ref = st.astype(np.float32)
    for r in range(3):
        for c in range(3):
            out = orc.sample_bilinear(st, dtype, 3, 3, c + 0.5, r + 0.5)
            assert np.array_equal(out, ref[r, c].astype(np.float64))


def _two_view_scene(H=32, W=32, Hf=4, Wf=4, D=8):
    cam = np.repeat(_front_cam(H, W), 2, 0)
    depth = np.full((2, H, W), 5.0, np.float32)
    rng = np.random.default_rng(5)
    c1, c2 = rng.standard_normal(D).astype(np.float32), rng.standard_normal(D).astype(np.float32)
    feat = np.stack([np.broadcast_to(c1, (Hf, Wf, D)), np.broadcast_to(c2, (Hf, Wf, D))]).copy()
    return cam, depth, feat, c1.astype(np.float64), c2.astype(np.float64)


def test_eq2_is_the_mean_over_visible_views_only(orc):
    cam, depth, feat, c1, c2 = _two_view_scene()
    pts = np.array([_pt(10.3, 20.7, 32, 32, z=2.0)], np.float32)
    r = orc.fuse_features(cam, depth, feat, "f32", pts, flags=orc.FLAG_MEAN_ONLY)
    assert r["count"][0] == 2 and np.allclose(r["fused"][0], 0.5 * (c1 + c2), atol=1e-12)
    depth[1] = 1.0                                   # second view now has a wall in front of the point
    r = orc.fuse_features(cam, depth, feat, "f32", pts, flags=orc.FLAG_MEAN_ONLY)
    assert r["count"][0] == 1 and np.allclose(r["fused"][0], c1, atol=1e-12)
    r = orc.fuse_features(cam, depth, feat, "f32", pts)
    assert np.allclose(r["fused"][0], c1 / np.linalg.norm(c1), atol=1e-12)
    depth[0] = 1.0                                   # occluded everywhere: zero weight, zero feature
    r = orc.fuse_features(cam, depth, feat, "f32", pts)
    assert r["count"][0] == 0 and not r["fused"].any()


def test_three_views_weights_are_one_over_count(orc):
    # distinct constant maps per view; mean-only output must be the arithmetic mean of the seen ones
    H = W = 32
    cam = np.repeat(_front_cam(H, W), 3, 0)
    depth = np.full((3, H, W), 5.0, np.float32)
    depth[1] = 0.5
    feat = np.stack([np.full((2, 2, 4), a, np.float32) for a in (1.0, 10.0, 100.0)])
    pts = np.array([_pt(16, 16, H, W)], np.float32)
    r = orc.fuse_features(cam, depth, feat, "f32", pts, flags=orc.FLAG_MEAN_ONLY)
    assert r["count"][0] == 2 and np.allclose(r["fused"][0], 50.5)


def test_uniform_map_fuses_to_that_feature(orc):
    s = make_scene("c1", n_points=1200)
    c = np.random.default_rng(6).standard_normal(s.D).astype(np.float32)
    feat = np.broadcast_to(c, s.feat.shape).copy()
    r = orc.fuse_features(s.cam, s.depth, feat, "f32", s.xyz, tau=s.tau)
    seen = r["count"] > 0
    assert seen.sum() > 100
    unit = c.astype(np.float64) / np.linalg.norm(c.astype(np.float64))
    assert np.allclose(r["fused"][seen], unit, atol=1e-12)
    assert not r["fused"][~seen].any()
    m = orc.fuse_features(s.cam, s.depth, feat, "f32", s.xyz, tau=s.tau, flags=orc.FLAG_MEAN_ONLY)
    assert np.allclose(m["fused"][seen], c.astype(np.float64), atol=1e-12)


def test_fused_is_unit_norm_or_zero_and_scale_invariant(orc):
    s = make_scene("c1", n_points=800)
    r = orc.fuse_features(s.cam, s.depth, s.feat, "f32", s.xyz, tau=s.tau)
    n = np.linalg.norm(r["fused"], axis=1)
    seen = r["count"] > 0
    assert np.allclose(n[seen], 1.0, atol=1e-12) and np.all(n[~seen] == 0)
    r2 = orc.fuse_features(s.cam, s.depth, s.feat * np.float32(4.0), "f32", s.xyz, tau=s.tau)   # exact scaling
    assert np.allclose(r2["fused"], r["fused"], atol=1e-12)


def test_duplicating_every_view_changes_nothing(orc):
    s = make_scene("c1", n_points=600)
    r = orc.fuse_features(s.cam, s.depth, s.feat, "f32", s.xyz, tau=s.tau, flags=orc.FLAG_MEAN_ONLY)
    r2 = orc.fuse_features(np.r_[s.cam, s.cam], np.r_[s.depth, s.depth], np.r_[s.feat, s.feat], "f32", s.xyz,
                           tau=s.tau, flags=orc.FLAG_MEAN_ONLY)
    assert np.array_equal(r2["count"], 2 * r["count"])
    assert np.allclose(r2["fused"], r["fused"], atol=1e-12)


def test_fused_equals_mask_weighted_mean_of_independent_samples(orc):
    # composition check: Eq. 2 assembled in numpy from the mask (pinned in the visibility tests)
    # and grid_sample (library routine) must give the oracle's fused feature
    s = make_scene("c2", n_points=500)
    pv = orc.project_visibility(s.cam, s.depth, s.xyz, tau=s.tau, want_uvz=True)
    r = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, s.xyz, tau=s.tau, flags=orc.FLAG_MEAN_ONLY)
    F = torch.from_numpy(stored_to_f32(s.feat, s.feat_dtype).astype(np.float64))
    acc = np.zeros((s.N, s.D))
    for v in range(s.n_views):
        uv = pv["uvz"][:, v, :2].astype(np.float64)
        uv[~pv["vis"][:, v].astype(bool)] = 0.0
        grid = torch.from_numpy(np.c_[2 * uv[:, 0] / s.W - 1, 2 * uv[:, 1] / s.H - 1]).reshape(1, 1, -1, 2)
        smp = torch.nn.functional.grid_sample(F[v].permute(2, 0, 1)[None], grid, mode="bilinear",
                                              padding_mode="border", align_corners=False)[0, :, 0].T.numpy()
        acc += smp * pv["vis"][:, v:v + 1]
    seen = pv["count"] > 0
    exp = acc[seen] / pv["count"][seen, None]
    assert np.array_equal(pv["count"], r["count"])
    assert np.allclose(r["fused"][seen], exp, rtol=0, atol=1e-6)
