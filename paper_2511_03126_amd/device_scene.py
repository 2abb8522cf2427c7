"""A generated scene resident on the GPU, with preallocated outputs and workspaces, and the library's calls strung into
steps of the hot path.  Used by the benchmark, the smoke run and the GPU tests; argument plumbing only."""
from __future__ import annotations

import numpy as np
import torch

from . import binding
from . import binding as aura


def _feat_tensor(scene, dev):
    if scene.feat_dtype == "bf16":
        return torch.from_numpy(scene.feat.view(np.int16)).to(dev).view(torch.bfloat16)
    return torch.from_numpy(scene.feat).to(dev)


class DeviceScene:
    """Device-resident copy of a scene plus preallocated outputs and workspaces."""

    def __init__(self, scene, dev="cuda:0", want_uvz=False, flags=0, want_fused=True, temb_dtype=None):
        s = self.scene = scene
        self.dev = dev
        self.xyz = torch.from_numpy(s.xyz).to(dev)
        self.views = aura.Views(cam=torch.from_numpy(s.cam).to(dev), depth=torch.from_numpy(s.depth).to(dev),
                                feat=_feat_tensor(s, dev))
        self.params = aura.Params(tau=s.tau, z_near=s.z_near, temperature=s.temperature, norm_eps=1e-12, flags=flags)
        # the same with the matrix-core fusion forced into its two-kernel form (AURA_FUSE_TWO_KERNELS)
        self.params_two = aura.Params(tau=s.tau, z_near=s.z_near, temperature=s.temperature, norm_eps=1e-12, flags=flags | 8)
        self.temb = torch.from_numpy(s.temb).to(dev)
        if temb_dtype is not None:      # text embeddings handed over as 16-bit values (the scene's must be exact in it)
            self.temb = self.temb.to(temb_dtype)
        self.y = torch.from_numpy(s.y).to(dev)
        N, V = s.N, s.vis_pitch
        self.single = s.B == 1
        self.pt_offsets = None if self.single else s.pt_offsets
        self.view_offsets = None if self.single else s.view_offsets
        self.vis = torch.empty((N, V), dtype=torch.uint8, device=dev)
        self.count = torch.empty(N, dtype=torch.int32, device=dev)
        self.count_fuse = torch.empty(N, dtype=torch.int32, device=dev)
        self.uvz = torch.empty((N, V, 3), dtype=torch.float32, device=dev) if want_uvz else None
        self.fused = torch.empty((N, s.D), dtype=torch.float32, device=dev) if want_fused else None
        self.scores = torch.empty((N, s.K), dtype=torch.float32, device=dev)
        self.prop = torch.empty((N, s.P), dtype=torch.float32, device=dev)
        self.label = torch.empty(N, dtype=torch.int32, device=dev)
        self.mass = torch.empty(s.B, dtype=torch.float32, device=dev)
        self.n_used = torch.empty(s.B, dtype=torch.int64, device=dev)
        nb = aura.fuse_workspace_bytes(self.views, N, s.B)
        self.ws_fuse = torch.empty(nb, dtype=torch.uint8, device=dev) if nb and want_fused else None
        self.ws_scores = torch.empty(aura.workspace_bytes(binding.CALL_MATERIAL_SCORES, D=s.D, K=s.K),
                                     dtype=torch.uint8, device=dev)
        self.ws_fuse_scores = torch.empty(aura.fuse_scores_workspace_bytes(self.views, N, s.K, s.B), dtype=torch.uint8,
                                          device=dev) if want_fused else None
        self.ws_mass = torch.empty(aura.workspace_bytes(binding.CALL_PROPERTY_INTEGRATE, N=N, B=s.B, G=s.G),
                                   dtype=torch.uint8, device=dev)
        self.ws_single = None      # workspace of fuse_score_integrate, allocated on first use
        self._ran = set()          # fusion calls made so far (their workspaces hold a status word)

    def free_fused(self):
        """Drops the [N][D] output (and the workspaces of the calls that write it): what is left serves
        fuse_score_integrate only."""
        self.fused = self.ws_fuse = self.ws_fuse_scores = None

    def project_visibility(self):
        aura.project_visibility(self.views, self.params, self.xyz, self.vis, self.count, self.uvz,
                                self.pt_offsets, self.view_offsets)

    def fuse_features(self, two_kernels=False):
        self._ran.add("fuse_features")
        aura.fuse_features(self.views, self.params_two if two_kernels else self.params, self.xyz, self.fused,
                           self.count_fuse, self.pt_offsets, self.view_offsets, self.ws_fuse)

    def material_scores(self):
        aura.material_scores(self.fused, self.temb, self.y, self.params, self.scores, self.prop, self.label,
                             self.ws_scores)

    def fuse_scores(self, with_vis=False, two_kernels=False):
        self._ran.add("fuse_scores")
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

    def fuse_score_integrate(self, with_vis=True, two_kernels=False):
        """The whole path in one call, without the fused rows."""
        s = self.scene
        self._ran.add("fuse_score_integrate")
        if self.ws_single is None:
            self.ws_single = torch.empty(aura.fuse_score_integrate_workspace_bytes(self.views, s.N, s.K, s.P, s.B, s.G),
                                         dtype=torch.uint8, device=self.dev)
        aura.fuse_score_integrate(self.views, self.params_two if two_kernels else self.params, self.xyz, self.temb, self.y,
                                  self.scores, self.mass, p_index=0, count=self.count_fuse,
                                  vis=self.vis if with_vis else None, prop=self.prop, label=self.label, n_used=self.n_used,
                                  vol_uniform=s.vol_uniform, pt_offsets=self.pt_offsets, view_offsets=self.view_offsets,
                                  grid_lo=s.grid_lo, grid_h=s.grid_h, G=s.G, workspace=self.ws_single)

    def step_single_pass_call(self):
        """`step_single_pass` without the copy of the view counts (what the benchmark times)."""
        self.fuse_score_integrate()

    def step_single_pass(self):
        """One pass of the whole path as one call that never writes the fused rows."""
        self.fuse_score_integrate()
        self.count.copy_(self.count_fuse)

    def step_single_pass_two_kernels(self):
        self.fuse_score_integrate(two_kernels=True)
        self.count.copy_(self.count_fuse)

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
            if t is not None:
                t.fill_(float("nan"))
        for t in (self.count_fuse, self.count, self.label, self.n_used):
            t.fill_(-7)
        self.vis.fill_(9)      # uvz (debug output of aura_project_visibility alone) is left as it is

    def status_words(self, word=0):
        """The status words of the fusion workspaces that exist (all zero unless a kernel had something to report);
        word = 1: the counts of tiles fused point by point."""
        s = self.scene
        out = {}
        for name, call, ws in (("fuse_features", binding.CALL_FUSE_FEATURES, self.ws_fuse),
                               ("fuse_scores", binding.CALL_FUSE_SCORES, self.ws_fuse_scores),
                               ("fuse_score_integrate", binding.CALL_FUSE_SCORE_INTEGRATE, self.ws_single)):
            if name not in self._ran:
                continue
            w = binding.fuse_status_word(call, self.views, s.N, ws, B=s.B, K=s.K, P=s.P, G=s.G, word=word)
            if w is not None:
                out[name] = w
        return out

    def results(self):
        torch.cuda.synchronize()
        bad = {k: v for k, v in self.status_words().items() if v != 0}
        if bad:
            raise RuntimeError(f"fusion kernels reported a problem in their status word: {bad}")
        out = {k: getattr(self, k).cpu().numpy() for k in
               ("vis", "count", "count_fuse", "fused", "scores", "prop", "label", "mass", "n_used")
               if getattr(self, k) is not None}
        if self.uvz is not None:
            out["uvz"] = self.uvz.cpu().numpy()
        return out
