"""The calls of the library strung together in the order of the paper's pipeline (Sec. 3.2 - 3.4), on the device and
in the oracle, each side feeding its own intermediate results forward:

  adaptive sampling (3.2.1) -> normals, view importance filtering (3.2.2) -> fusion over the kept views (3.2.3; the
  stored feature maps stand in for the encoder) -> material scores of the sampled points (3.4.1) -> dense per-point
  features (3.1) -> feature-space k-NN densification (Eq. 5) -> thickness-based mass and centre of mass (3.4.2).

Every call has its own element-by-element parity test; this one checks that the outputs of one call are what the
next one expects (layouts, index conventions, offsets) by comparing the ends of the two chains."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_chain_c2(orc):
    import gpu_harness as H
    import paper_2511_03126_amd as aura
    from paper_2511_03126_amd import binding
    from workloads.scenes import make_scene, material_thickness
    s = make_scene("c2", n_points=30_000)
    d = H.DeviceScene(s)
    dev = d.dev
    theta = material_thickness(s.K, s.meta["seed"])
    lo, hi = s.xyz.min(0, keepdims=True), s.xyz.max(0, keepdims=True)
    centre = s.xyz.mean(0, keepdims=True).astype(np.float32)
    n_target, k_nrm, k_views, k_nn = 150, 30, 3, 5

    # ---- device chain
    q = torch.empty((4096, 3), device=dev)
    off = torch.empty(2, dtype=torch.int32, device=dev)
    work = torch.empty(aura.voxel_workspace_bytes(lo, hi, n_target), dtype=torch.uint8, device=dev)
    aura.voxel_downsample(d.xyz, lo, hi, n_target, q, off, workspace=work)
    M = int(off[1].item())
    q = q[:M].contiguous()
    nrm = torch.empty_like(q)
    aura.estimate_normals(d.xyz, q, centre, k_nrm, nrm)
    sel_view = torch.empty((M, k_views), dtype=torch.int32, device=dev)
    sel_mask = torch.empty((M, s.vis_pitch), dtype=torch.uint8, device=dev)
    aura.select_views(d.views, d.params, q, nrm, k_views, sel_view, None, sel_mask)
    ws_q = torch.empty(max(aura.fuse_workspace_bytes(d.views, M), 1), dtype=torch.uint8, device=dev)
    clip_q = torch.empty((M, s.D), device=dev)
    aura.fuse_selected(d.views, d.params, q, sel_mask, clip_q, None, workspace=ws_q)
    scores_q = torch.empty((M, s.K), device=dev)
    aura.material_scores(clip_q, d.temb, d.y, d.params, scores_q, workspace=d.ws_scores)
    dino_q = torch.empty((M, s.D), device=dev)
    aura.fuse_features(d.views, d.params, q, dino_q, None, workspace=ws_q)
    d.fuse_features()                                   # dense features and view counts of every point
    wq = torch.empty((s.N, s.K), device=dev)
    ws_knn = torch.empty(aura.workspace_bytes(binding.CALL_KNN_DENSIFY, D=s.D, Ns=M), dtype=torch.uint8, device=dev)
    aura.knn_densify(d.fused, dino_q, scores_q, k_nn, None, d.params, wq, workspace=ws_knn)
    mass, com = torch.empty(1, device=dev), torch.empty((1, 3), device=dev)
    ws_th = torch.empty(aura.workspace_bytes(binding.CALL_THICKNESS_INTEGRATE, N=s.N, B=1), dtype=torch.uint8, device=dev)
    aura.thickness_integrate(wq, d.y, torch.from_numpy(theta).to(dev), d.xyz, d.params, mass, count=d.count_fuse, com=com,
                             workspace=ws_th)
    torch.cuda.synchronize()

    # ---- oracle chain
    o_q = orc.voxel_downsample(s.xyz, n_target, box_lo=lo, box_hi=hi)["xyz"].astype(np.float32)
    assert len(o_q) == M and np.abs(q.cpu().numpy() - o_q).max() < 1e-6
    o_nrm = orc.estimate_normals(s.xyz, o_q, centre, k_nrm)["normals"].astype(np.float32)
    o_sel = orc.select_views(s.cam, s.depth, o_q, o_nrm, k_views, tau=s.tau, z_near=s.z_near, mask_pitch=s.vis_pitch)
    same_sel = (sel_mask.cpu().numpy() == o_sel["sel_mask"]).all(1)
    assert same_sel.mean() > 0.95
    o_clip = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, o_q, tau=s.tau, z_near=s.z_near, sel_mask=o_sel["sel_mask"])
    o_scores_q = orc.material_scores(o_clip["fused"], s.temb, s.y, T=s.temperature)["scores"]
    assert np.abs(scores_q.cpu().numpy()[same_sel] - o_scores_q[same_sel]).max() < H.tol_for(s)
    o_dino_q = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, o_q, tau=s.tau, z_near=s.z_near)["fused"]
    o_dense = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, s.xyz, tau=s.tau, z_near=s.z_near)
    o_wq = orc.knn_densify(o_dense["fused"], o_dino_q, o_scores_q, k_nn)["wq"]
    o_th = orc.thickness_integrate(o_wq, s.y[:, 0], theta, s.xyz, count=o_dense["count"], T=s.temperature)
    g_mass, g_com = float(mass.item()), com.cpu().numpy()[0]
    # the ends of the chains: a few sampled points may keep other views and a few dense points other neighbours
    # (near-ties), which moves the sums by far less than the bar of the hot path
    assert abs(g_mass - o_th["mass"][0]) <= H.tol_for(s) * o_th["mass"][0], (g_mass, o_th["mass"][0])
    assert np.abs(g_com - o_th["com"][0]).max() <= H.tol_for(s) * np.abs(s.xyz).max()
    close = np.abs(wq.cpu().numpy() - o_wq).max(1) < H.tol_for(s)
    assert close.mean() > 0.97
