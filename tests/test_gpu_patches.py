"""GPU parity of aura_patch_batch (Sec. 3.2.3) against the CPU oracle on the same seeded inputs.  Bar: valid flags
exact; patch values within 2e-4 (fp32 output; the sample positions are fp32 on the device, double in the oracle: a
position error of 3e-5 pixel at u ~ 400 times a slope of at most one grey range per pixel) and 2e-3 for fp16 output, in
units of the normalised value times inv_std."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _inputs(name, kw, M, k, seed=0):
    from workloads.scenes import make_scene, synthetic_images, synthetic_normals
    s = make_scene(name, **kw)
    images = synthetic_images(s.n_views, s.H, s.W, s.meta["seed"])
    # M source points per object, evenly spaced through the object's (spatially sorted) points
    idx = np.concatenate([np.linspace(s.pt_offsets[b], s.pt_offsets[b + 1] - 1, M).astype(np.int64) for b in range(s.B)])
    xyz = s.xyz[idx]
    po = np.arange(s.B + 1, dtype=np.int64) * M
    nrm = synthetic_normals(s.xyz, s.pt_offsets, s.meta["seed"])[idx]
    return s, images, xyz, po, nrm


def _gpu(s, images, xyz, po, sel, scales, R, dtype=torch.float32, mean=None, inv_std=None):
    import paper_2511_03126_amd as aura
    dev = "cuda:0"
    M, k = sel.shape
    out = torch.full((M, k, len(scales), 3, R, R), float("nan"), dtype=dtype, device=dev)
    valid = torch.full((M, k), 9, dtype=torch.uint8, device=dev)
    single = s.B == 1
    aura.patch_batch(torch.from_numpy(s.cam).to(dev), torch.from_numpy(images).to(dev), torch.from_numpy(xyz).to(dev),
                     torch.from_numpy(sel).to(dev), scales, out, mean, inv_std, valid,
                     None if single else po, None if single else s.view_offsets)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), valid.cpu().numpy()


@pytest.mark.parametrize("name,kw,M,k,R,dtype,tol", [
    ("c1", dict(n_points=4000), 40, 3, 32, torch.float32, 2e-4),
    ("c1", dict(n_points=4000), 40, 3, 30, torch.float32, 2e-4),          # R not a multiple of 4: scalar stores
    ("c1", dict(n_points=4000), 24, 2, 32, torch.float16, 2e-3),
    ("c2", dict(n_points=20_000), 30, 3, 56, torch.float32, 2e-4),
    ("c5", dict(n_points=2_000, n_objects=5), 12, 2, 32, torch.float32, 2e-4),
])
def test_patches_match_oracle(orc, name, kw, M, k, R, dtype, tol):
    s, images, xyz, po, nrm = _inputs(name, kw, M, k)
    single = s.B == 1
    sel = orc.select_views(s.cam, s.depth, xyz, nrm, k, tau=s.tau, z_near=s.z_near, pt_offsets=None if single else po,
                           view_offsets=None if single else s.view_offsets)["sel_view"]
    sel[::7, -1] = -1                                  # some points with a view missing, whatever the scene gave
    assert (sel >= 0).mean() > 0.5
    scales = np.array([20.0, 40.0, 60.0], np.float32)
    mean, inv_std = np.array([0.48, 0.46, 0.41], np.float32), np.array([3.7, 3.8, 3.6], np.float32)
    g, valid = _gpu(s, images, xyz, po, sel, scales, R, dtype, mean, inv_std)
    ref = orc.patch_batch(s.cam, images, xyz, sel, scales, R, mean=mean, inv_std=inv_std, pt_offsets=None if single else po,
                          view_offsets=None if single else s.view_offsets)
    assert np.array_equal(valid, ref["valid"]) and np.array_equal(valid, (sel >= 0).astype(np.uint8))
    err = np.abs(g - ref["patches"]).max()
    assert err <= tol * inv_std.max(), f"patch err {err}"
    assert (g[sel < 0] == 0).all()


def test_pixel_aligned_crop_and_the_image_border():
    """Hand-known answers through the library: a crop that coincides with the pixel grid is the image block itself;
    a patch that hangs over the edge repeats the border pixels."""
    import paper_2511_03126_amd as aura
    dev = "cuda:0"
    rng = np.random.default_rng(1)
    img = rng.integers(0, 256, (1, 40, 52, 3), dtype=np.uint8)
    cam = torch.tensor([[1, 0, 0, 0, 1, 0, 0, 0, 1, 0, 0, 0, 1, 1, 0, 0]], dtype=torch.float32, device=dev)   # u = x / z
    xyz = torch.tensor([[20.0, 16.0, 1.0], [0.0, 0.0, 1.0]], device=dev)
    sel = torch.zeros((2, 1), dtype=torch.int32, device=dev)
    out = torch.empty((2, 1, 1, 3, 8, 8), device=dev)
    aura.patch_batch(cam, torch.from_numpy(img).to(dev), xyz, sel, [8.0], out)
    torch.cuda.synchronize()
    o = out.cpu().numpy() * 255.0
    assert np.allclose(o[0, 0, 0], img[0, 12:20, 16:24].transpose(2, 0, 1), atol=1e-4)
    # centred on the corner (0, 0): the lower right quarter is the image's first 4 x 4 block, the rest its border
    assert np.allclose(o[1, 0, 0][:, 4:, 4:], img[0, 0:4, 0:4].transpose(2, 0, 1), atol=1e-4)
    assert np.allclose(o[1, 0, 0][:, :4, :4], img[0, 0, 0][:, None, None], atol=1e-4)
    assert np.allclose(o[1, 0, 0][:, :4, 4:], img[0, 0, 0:4].T[:, None, :], atol=1e-4)


def test_encoder_sized_batch_c2(orc):
    """The paper's configuration on C2's views: about 150 source points x 3 views x 3 scales (20, 40, 60 pixels) at the
    encoder resolution 224; the oracle recomputes the patches of 6 of the points."""
    s, images, xyz, po, nrm = _inputs("c2", {}, 150, 3)
    sel = orc.select_views(s.cam, s.depth, xyz, nrm, 3, tau=s.tau, z_near=s.z_near)["sel_view"]
    scales = np.array([20.0, 40.0, 60.0], np.float32)
    g, valid = _gpu(s, images, xyz, po, sel, scales, 224)
    assert np.array_equal(valid, (sel >= 0).astype(np.uint8))
    pick = np.array([0, 31, 62, 93, 124, 149])
    ref = orc.patch_batch(s.cam, images, xyz[pick], sel[pick], scales, 224)
    err = np.abs(g[pick] - ref["patches"]).max()
    assert err <= 2e-4, f"patch err {err}"
    assert not np.isnan(g).any()
