"""Pins for the oracle's multi-scale patch batch (Sec. 3.2.3): squares of several sizes around the projection of a
point in its kept views, resampled to the encoder's resolution.

Expectations: crops that coincide with the pixel grid (the patch is the image block itself), constant and affine
images (bilinear resampling reproduces them exactly), and `torch.nn.functional.grid_sample` over the whole image as
an independent library evaluation of the same sampling rule.  None comes from the oracle or from the GPU library."""
import numpy as np
import pytest
import torch

CAM = np.array([1, 0, 0, 0, 1, 0, 0, 0, 1, 0, 0, 0, 1, 1, 0, 0], np.float32)   # u = x / z, v = y / z


def _point_for(u, v):
    """A point that the camera above projects exactly to pixel coordinates (u, v): z = 1."""
    return np.array([u, v, 1.0], np.float32)


def test_aligned_crop_is_the_image_block(orc):
    rng = np.random.default_rng(1)
    img = rng.integers(0, 256, (1, 40, 50, 3), dtype=np.uint8)
    # centre (20, 16), side 8, R = 8: output pixel (i, j) samples pixel centre (16.5 + j, 12.5 + i): pixels 16..23 x 12..19
    r = orc.patch_batch(CAM, img, _point_for(20.0, 16.0), [[0]], [8.0], 8)
    assert r["valid"][0, 0] == 1
    want = img[0, 12:20, 16:24].transpose(2, 0, 1) / 255.0
    assert np.allclose(r["patches"][0, 0, 0], want, rtol=0, atol=1e-15)
    # side 16 at R = 8: every output pixel is the mean of a 2 x 2 block's centre, i.e. the average of its four pixels
    r = orc.patch_batch(CAM, img, _point_for(20.0, 16.0), [[0]], [16.0], 8)
    blk = img[0, 8:24, 12:28].astype(np.float64).reshape(8, 2, 8, 2, 3).mean((1, 3)).transpose(2, 0, 1) / 255.0
    assert np.allclose(r["patches"][0, 0, 0], blk, rtol=0, atol=1e-15)


def test_constant_and_affine_images_are_reproduced(orc):
    H, W = 64, 80
    yy, xx = np.mgrid[0:H, 0:W]
    img = np.stack([np.full((H, W), 77), xx + 2 * yy, 250 - 3 * xx + yy // 1 * 0], -1).astype(np.uint8)[None]
    u, v, R = 37.25, 30.5, 12
    for side in (5.0, 20.0, 33.0):
        r = orc.patch_batch(CAM, img, _point_for(u, v), [[0]], [side], R)["patches"][0, 0, 0] * 255.0
        x = u - side / 2 + (np.arange(R) + 0.5) * side / R
        y = v - side / 2 + (np.arange(R) + 0.5) * side / R
        assert x.min() > 1 and x.max() < W - 1 and y.min() > 1 and y.max() < H - 1      # interior: no border effect
        assert np.allclose(r[0], 77.0, atol=1e-12)
        assert np.allclose(r[1], (x[None, :] - 0.5) + 2 * (y[:, None] - 0.5), atol=1e-10)
        assert np.allclose(r[2], 250 - 3 * (x[None, :] - 0.5) + 0 * y[:, None], atol=1e-10)


def _grid_sample_reference(img, u, v, side, R):
    H, W, _ = img.shape
    x = u - side / 2 + (np.arange(R) + 0.5) * side / R
    y = v - side / 2 + (np.arange(R) + 0.5) * side / R
    gx, gy = np.meshgrid(2 * x / W - 1, 2 * y / H - 1)
    grid = torch.from_numpy(np.stack([gx, gy], -1)[None])
    t = torch.from_numpy(img.astype(np.float64).transpose(2, 0, 1)[None])
    return torch.nn.functional.grid_sample(t, grid, mode="bilinear", padding_mode="border", align_corners=False)[0].numpy() / 255.0


def test_against_grid_sample_including_the_image_border(orc):
    rng = np.random.default_rng(2)
    img = rng.integers(0, 256, (3, 48, 56, 3), dtype=np.uint8)
    cams = np.stack([CAM, CAM, CAM])
    centres = [(20.0, 20.0), (1.5, 3.25), (55.0, 47.0), (28.125, 0.0), (-4.0, 60.0)]     # the last ones hang over the edge
    pts = np.stack([_point_for(u, v) for u, v in centres])
    sel = np.array([[2, 0]] * len(pts), np.int32)
    scales = [6.0, 20.0, 40.0]
    r = orc.patch_batch(cams, img, pts, sel, scales, 16)["patches"]
    for s, (u, v) in enumerate(centres):
        for rank, view in enumerate(sel[s]):
            for l, side in enumerate(scales):
                want = _grid_sample_reference(img[view], u, v, side, 16)
                assert np.allclose(r[s, rank, l], want, rtol=0, atol=1e-12), (s, rank, l)


def test_missing_views_normalisation_and_objects(orc):
    rng = np.random.default_rng(3)
    img = rng.integers(0, 256, (4, 32, 32, 3), dtype=np.uint8)
    cams = np.stack([CAM] * 4)
    pts = np.stack([_point_for(10.0, 12.0), _point_for(20.0, 8.0), _point_for(16.0, 16.0)])
    sel = np.array([[1, -1], [0, 1], [1, 0]], np.int32)
    po, vo = np.array([0, 2, 3], np.int64), np.array([0, 2, 4], np.int32)       # object 1 owns views 2 and 3
    mean, inv_std = np.array([0.5, 0.25, 0.125], np.float32), np.array([2.0, 4.0, 8.0], np.float32)
    r = orc.patch_batch(cams, img, pts, sel, [8.0], 8, mean=mean, inv_std=inv_std, pt_offsets=po, view_offsets=vo)
    plain = orc.patch_batch(cams, img, pts, sel, [8.0], 8, pt_offsets=po, view_offsets=vo)
    assert list(r["valid"].ravel()) == [1, 0, 1, 1, 1, 1] and (r["patches"][0, 1] == 0).all()
    want = (plain["patches"] - mean[None, None, None, :, None, None]) * inv_std[None, None, None, :, None, None]
    want[0, 1] = 0
    assert np.allclose(r["patches"], want, atol=1e-15)
    # the third point belongs to object 1: its view 1 is view 3 of the call
    alone = orc.patch_batch(cams[3:], img[3:], pts[2:], [[0]], [8.0], 8)
    assert np.array_equal(plain["patches"][2, 0], alone["patches"][0, 0])
