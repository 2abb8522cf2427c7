"""Helpers shared by the GPU parity tests: upload a generated scene, run the four library calls
through the binding, bring results back as numpy, compare against the oracle."""
from __future__ import annotations

import numpy as np
import torch

import paper_2511_03126_amd as aura
from paper_2511_03126_amd import binding


def _feat_tensor(scene, dev):
    if scene.feat_dtype == "bf16":
        return torch.from_numpy(scene.feat.view(np.int16)).to(dev).view(torch.bfloat16)
    return torch.from_numpy(scene.feat).to(dev)


class DeviceScene:
    """Device-resident copy of a scene plus preallocated outputs and workspaces."""

    def __init__(self, scene, dev="cuda:0", want_uvz=False, flags=0):
        s = self.scene = scene
        self.dev = dev
        self.xyz = torch.from_numpy(s.xyz).to(dev)
        self.views = aura.Views(cam=torch.from_numpy(s.cam).to(dev), depth=torch.from_numpy(s.depth).to(dev),
                                feat=_feat_tensor(s, dev))
        self.params = aura.Params(tau=s.tau, z_near=s.z_near, temperature=s.temperature, norm_eps=1e-12, flags=flags)
        # the same with the matrix-core fusion forced into its two-kernel form (AURA_FUSE_TWO_KERNELS)
        self.params_two = aura.Params(tau=s.tau, z_near=s.z_near, temperature=s.temperature, norm_eps=1e-12, flags=flags | 8)
        self.temb = torch.from_numpy(s.temb).to(dev)
        self.y = torch.from_numpy(s.y).to(dev)
        N, V = s.N, s.vis_pitch
        self.single = s.B == 1
        self.pt_offsets = None if self.single else s.pt_offsets
        self.view_offsets = None if self.single else s.view_offsets
        self.vis = torch.empty((N, V), dtype=torch.uint8, device=dev)
        self.count = torch.empty(N, dtype=torch.int32, device=dev)
        self.count_fuse = torch.empty(N, dtype=torch.int32, device=dev)
        self.uvz = torch.empty((N, V, 3), dtype=torch.float32, device=dev) if want_uvz else None
        self.fused = torch.empty((N, s.D), dtype=torch.float32, device=dev)
        self.scores = torch.empty((N, s.K), dtype=torch.float32, device=dev)
        self.prop = torch.empty((N, s.P), dtype=torch.float32, device=dev)
        self.label = torch.empty(N, dtype=torch.int32, device=dev)
        self.mass = torch.empty(s.B, dtype=torch.float32, device=dev)
        self.n_used = torch.empty(s.B, dtype=torch.int64, device=dev)
        nb = aura.fuse_workspace_bytes(self.views, N, s.B)
        self.ws_fuse = torch.empty(nb, dtype=torch.uint8, device=dev) if nb else None
        self.ws_scores = torch.empty(aura.workspace_bytes(binding.CALL_MATERIAL_SCORES, D=s.D, K=s.K),
                                     dtype=torch.uint8, device=dev)
        self.ws_fuse_scores = torch.empty(aura.fuse_scores_workspace_bytes(self.views, N, s.K, s.B), dtype=torch.uint8,
                                          device=dev)
        self.ws_mass = torch.empty(aura.workspace_bytes(binding.CALL_PROPERTY_INTEGRATE, N=N, B=s.B, G=s.G),
                                   dtype=torch.uint8, device=dev)

    def project_visibility(self):
        aura.project_visibility(self.views, self.params, self.xyz, self.vis, self.count, self.uvz,
                                self.pt_offsets, self.view_offsets)

    def fuse_features(self, two_kernels=False):
        aura.fuse_features(self.views, self.params_two if two_kernels else self.params, self.xyz, self.fused,
                           self.count_fuse, self.pt_offsets, self.view_offsets, self.ws_fuse)

    def material_scores(self):
        aura.material_scores(self.fused, self.temb, self.y, self.params, self.scores, self.prop, self.label,
                             self.ws_scores)

    def fuse_scores(self, with_vis=False, two_kernels=False):
        aura.fuse_scores(self.views, self.params_two if two_kernels else self.params, self.xyz, self.temb, self.y,
                         self.fused, self.scores,
                         count=self.count_fuse, prop=self.prop, label=self.label, pt_offsets=self.pt_offsets,
                         view_offsets=self.view_offsets, workspace=self.ws_fuse_scores,
                         vis=self.vis if with_vis else None)

    def fuse_scores_vis(self):
        self.fuse_scores(with_vis=True)

    def property_integrate(self):
        s = self.scene
        aura.property_integrate(self.prop, self.mass, p_index=0, count=self.count_fuse, vol_uniform=s.vol_uniform,
                                pt_offsets=None if self.single else s.pt_offsets,
                                xyz=self.xyz if s.G > 0 else None, grid_lo=s.grid_lo, grid_h=s.grid_h, G=s.G,
                                n_used=self.n_used, workspace=self.ws_mass)

    def step(self):
        """One pass of the whole path, one library call per stage."""
        self.project_visibility()
        self.fuse_features()
        self.material_scores()
        self.property_integrate()

    def step_combined(self):
        """One pass of the whole path with visibility mask, fusion and scoring in one call (the mask and the view
        counts come out of the fusion; `count` is filled from its count output)."""
        self.fuse_scores(with_vis=True)
        self.count.copy_(self.count_fuse)
        self.property_integrate()

    def step_two_kernels(self):
        """`step` with the matrix-core fusion as two kernels (lists, then products)."""
        self.project_visibility()
        self.fuse_features(two_kernels=True)
        self.material_scores()
        self.property_integrate()

    def step_combined_two_kernels(self):
        """`step_combined` with the matrix-core fusion as two kernels."""
        self.fuse_scores(with_vis=True, two_kernels=True)
        self.count.copy_(self.count_fuse)
        self.property_integrate()

    def clear_outputs(self):
        for t in (self.fused, self.scores, self.prop, self.mass):
            t.fill_(float("nan"))
        for t in (self.count_fuse, self.count, self.label, self.n_used):
            t.fill_(-7)
        self.vis.fill_(9)      # uvz (debug output of aura_project_visibility alone) is left as it is

    def results(self):
        torch.cuda.synchronize()
        out = {k: getattr(self, k).cpu().numpy() for k in
               ("vis", "count", "count_fuse", "fused", "scores", "prop", "label", "mass", "n_used")}
        if self.uvz is not None:
            out["uvz"] = self.uvz.cpu().numpy()
        return out


def tol_for(scene):
    """Tolerance of the parity bar: 1e-4 for fp32 feature maps, 2e-2 for bf16 / fp16 maps."""
    return 1e-4 if scene.feat_dtype == "f32" else 2e-2


def oracle_points(orc, scene, idx=None, flags=0, want_uvz=False):
    """Oracle outputs for all points (idx None) or for a subset of point indices (single object)."""
    s = scene
    xyz = s.xyz if idx is None else s.xyz[idx]
    single = s.B == 1 or idx is not None
    po = None if single else s.pt_offsets
    vo = None if single else s.view_offsets
    pv = orc.project_visibility(s.cam, s.depth, xyz, tau=s.tau, z_near=s.z_near, flags=flags & 1, pt_offsets=po,
                                view_offsets=vo, vis_pitch=s.vis_pitch, want_diag=True, want_uvz=want_uvz)
    fu = orc.fuse_features(s.cam, s.depth, s.feat, s.feat_dtype, xyz, tau=s.tau, z_near=s.z_near, flags=flags & 3,
                           pt_offsets=po, view_offsets=vo)
    sc = orc.material_scores(fu["fused"], s.temb, s.y, T=s.temperature)
    return {**pv, "fused": fu["fused"], "count_fuse": fu["count"], **sc}


def compare_points(gpu, ref, scene, idx=None, report=None, mean_only=False):
    """Element-by-element comparison of per-point outputs; returns a dict of error figures."""
    tol = tol_for(scene)
    sel = slice(None) if idx is None else idx
    g = {k: v[sel] for k, v in gpu.items() if k not in ("mass", "n_used")}
    # masks and counts: bit exact, except pairs the oracle flags as within rounding of a threshold
    diff = g["vis"] != ref["vis"]
    allowed = (ref["diag"] & 3) != 0
    assert not (diff & ~allowed).any(), f"{int((diff & ~allowed).sum())} mask mismatches outside the diagnostic sets"
    n_mis = int(diff.sum())
    rows_ok = ~diff.any(1)
    assert np.array_equal(g["count"][rows_ok], ref["count"][rows_ok])
    assert np.array_equal(g["count_fuse"], g["count"])
    if "uvz" in g and ref.get("uvz") is not None:
        assert np.array_equal(g["uvz"].view(np.uint32), ref["uvz"].view(np.uint32)), "projection not bit exact"
    # fused: relative L2 per point
    fr = ref["fused"][rows_ok]
    fg = g["fused"][rows_ok].astype(np.float64)
    err_f = np.linalg.norm(fg - fr, axis=1) / np.maximum(np.linalg.norm(fr, axis=1), 1e-12)
    err_f[(np.linalg.norm(fr, axis=1) == 0) & (np.linalg.norm(fg, axis=1) == 0)] = 0.0
    assert err_f.max(initial=0.0) <= tol, f"fused rel err {err_f.max()}"
    out = dict(mask_mismatch=n_mis, fused_rel=float(err_f.max(initial=0.0)))
    if not mean_only:
        err_s = np.abs(g["scores"][rows_ok] - ref["scores"][rows_ok])
        assert err_s.max(initial=0.0) <= tol, f"scores abs err {err_s.max()}"
        ymax = np.abs(scene.y).max(0)
        err_p = np.abs(g["prop"][rows_ok] - ref["prop"][rows_ok]) / ymax
        assert err_p.max(initial=0.0) <= tol, f"prop err {err_p.max()}"
        lab_bad = (g["label"][rows_ok] != ref["label"][rows_ok])
        near_tie = ref["margin"][rows_ok] <= 2 * tol
        assert not (lab_bad & ~near_tie).any(), "label mismatch away from a tie"
        out.update(scores_abs=float(err_s.max(initial=0.0)), prop_rel=float(err_p.max(initial=0.0)),
                   label_mismatch_near_tie=int(lab_bad.sum()))
    if report is not None:
        report.update(out)
    return out
