"""ctypes binding of libaura_fuse.so: same names as the C ABI (include/aura_fuse.h), argument
marshalling only.  Tensors are torch CUDA(HIP) tensors owned by the caller; work is enqueued on
torch's current stream and nothing synchronises.  There is no fallback: if the shared library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from pathlib import Path

import numpy as np
import torch

_LIB_PATH = Path(__file__).resolve().parent / "libaura_fuse.so"

F32, BF16, F16 = 0, 1, 2
VIS_FRUSTUM_ONLY, FUSE_MEAN_ONLY, FUSE_GATHER, FUSE_TWO_KERNELS, UNSEEN_ZERO = 1, 2, 4, 8, 16
CALL_MATERIAL_SCORES, CALL_PROPERTY_INTEGRATE, CALL_FUSE_FEATURES, CALL_FUSE_SCORES, CALL_KNN_DENSIFY = 1, 2, 3, 4, 5
CALL_THICKNESS_INTEGRATE = 6
CALL_FUSE_SCORE_INTEGRATE = 7

_TORCH_DTYPE = {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16}


class AuraError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = lib().aura_strerror(status).decode()
        if status == -6:
            msg += f" [hipError {lib().aura_last_hip_error()}]"
        super().__init__(f"{what}: {msg} ({status})")


class _ViewsT(C.Structure):
    _fields_ = [("n_views", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("Hf", C.c_int32), ("Wf", C.c_int32),
                ("D", C.c_int32), ("feat_dtype", C.c_int32), ("cam", C.c_void_p), ("depth", C.c_void_p),
                ("feat", C.c_void_p)]


class _SizesT(C.Structure):
    _fields_ = [("N", C.c_int64), ("B", C.c_int32), ("n_views", C.c_int32), ("Hf", C.c_int32), ("Wf", C.c_int32),
                ("D", C.c_int32), ("feat_dtype", C.c_int32), ("K", C.c_int32), ("G", C.c_int32), ("Ns", C.c_int32),
                ("P", C.c_int32)]


class _ParamsT(C.Structure):
    _fields_ = [("tau", C.c_float), ("z_near", C.c_float), ("temperature", C.c_float), ("norm_eps", C.c_float),
                ("flags", C.c_uint32)]


_lib = None


def lib():
    """Loads the shared library (built by paper_2511_03126_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise FileNotFoundError(f"{_LIB_PATH} is missing: run `python -m paper_2511_03126_amd.build` first")
        L = C.CDLL(str(_LIB_PATH))
        L.aura_version.restype = C.c_int32
        L.aura_strerror.restype = C.c_char_p
        L.aura_strerror.argtypes = [C.c_int32]
        L.aura_last_hip_error.restype = C.c_int32
        L.aura_workspace_bytes.restype = C.c_int32
        L.aura_workspace_bytes.argtypes = [C.c_int32, C.POINTER(_SizesT), C.POINTER(C.c_size_t)]
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.aura_fuse_status_offset.restype = C.c_int32
        L.aura_fuse_status_offset.argtypes = [C.c_int32, C.POINTER(_SizesT), C.POINTER(C.c_size_t), C.POINTER(C.c_int32)]
        L.aura_project_visibility.restype = C.c_int32
        L.aura_project_visibility.argtypes = [C.POINTER(_ViewsT), C.POINTER(_ParamsT), vp, i64, vp, vp, i32,
                                              vp, i32, vp, vp, vp]
        L.aura_fuse_features.restype = C.c_int32
        L.aura_fuse_features.argtypes = [C.POINTER(_ViewsT), C.POINTER(_ParamsT), vp, i64, vp, vp, i32, vp, vp,
                                         vp, C.c_size_t, vp]
        L.aura_material_scores.restype = C.c_int32
        L.aura_material_scores.argtypes = [vp, i64, i32, vp, i32, i32, vp, i32, C.POINTER(_ParamsT), vp, vp, vp,
                                           vp, C.c_size_t, vp]
        L.aura_material_scores_static.restype = C.c_int32
        L.aura_material_scores_static.argtypes = [vp, i64, i32, vp, i32, i32, vp, i32, C.POINTER(_ParamsT), vp, vp, vp, vp]
        L.aura_fuse_scores.restype = C.c_int32
        L.aura_fuse_scores.argtypes = [C.POINTER(_ViewsT), C.POINTER(_ParamsT), vp, i64, vp, vp, i32, vp, i32, i32, vp,
                                       i32, vp, vp, vp, i32, vp, vp, vp, vp, C.c_size_t, vp]
        L.aura_fuse_score_integrate.restype = C.c_int32
        L.aura_fuse_score_integrate.argtypes = [C.POINTER(_ViewsT), C.POINTER(_ParamsT), vp, i64, vp, vp, i32, vp, i32, i32,
                                                vp, i32, i32, vp, f32, vp, vp, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp,
                                                C.c_size_t, vp]
        L.aura_time_next_fusion.restype = C.c_int32
        L.aura_time_next_fusion.argtypes = [vp, vp]
        L.aura_knn_densify.restype = C.c_int32
        L.aura_knn_densify.argtypes = [vp, i64, i32, vp, i32, vp, i32, i32, vp, i32, C.POINTER(_ParamsT), vp, vp, vp, vp,
                                       vp, C.c_size_t, vp]
        L.aura_property_integrate.restype = C.c_int32
        L.aura_property_integrate.argtypes = [vp, i64, i32, i32, vp, vp, f32, vp, i32, vp, vp, vp, i32, vp, vp,
                                              vp, C.c_size_t, vp]
        L.aura_calibration_copy.restype = C.c_int32
        L.aura_voxel_grid.restype = C.c_int32
        L.aura_voxel_grid.argtypes = [vp, vp, i32, C.POINTER(C.c_float), vp]
        L.aura_voxel_workspace_bytes.restype = C.c_int32
        L.aura_voxel_workspace_bytes.argtypes = [vp, vp, i32, i32, C.POINTER(C.c_size_t)]
        L.aura_voxel_downsample.restype = C.c_int32
        L.aura_voxel_downsample.argtypes = [vp, i64, vp, i32, vp, vp, i32, vp, vp, i64, vp, vp, vp, C.c_size_t, vp]
        L.aura_patch_batch.restype = C.c_int32
        L.aura_patch_batch.argtypes = [vp, i32, i32, i32, vp, vp, i64, vp, vp, i32, vp, i32, vp, i32, i32, vp, vp, vp, i32,
                                       vp, vp]
        L.aura_estimate_normals.restype = C.c_int32
        L.aura_estimate_normals.argtypes = [vp, i64, vp, vp, i64, vp, i32, vp, i32, vp, vp, vp]
        L.aura_select_views.restype = C.c_int32
        L.aura_select_views.argtypes = [C.POINTER(_ViewsT), C.POINTER(_ParamsT), vp, vp, i64, vp, vp, i32, i32, vp, vp, vp,
                                        i32, vp, vp]
        L.aura_fuse_selected.restype = C.c_int32
        L.aura_fuse_selected.argtypes = [C.POINTER(_ViewsT), C.POINTER(_ParamsT), vp, i64, vp, vp, i32, vp, i32, vp, vp,
                                         vp, C.c_size_t, vp]
        L.aura_thickness_integrate.restype = C.c_int32
        L.aura_thickness_integrate.argtypes = [vp, i64, i32, vp, i32, i32, vp, vp, vp, vp, i32, vp, C.POINTER(_ParamsT),
                                               f32, f32, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.aura_calibration_copy.argtypes = [vp, vp, C.c_size_t, vp]
        L.aura_calibration_fill.restype = C.c_int32
        L.aura_calibration_fill.argtypes = [vp, C.c_size_t, C.c_uint32, vp]
        _lib = L
    return _lib


@dataclass
class Params:
    tau: float = 0.0
    z_near: float = 1e-6
    temperature: float = 0.1
    norm_eps: float = 1e-12
    flags: int = 0

    def c(self):
        return _ParamsT(self.tau, self.z_near, self.temperature, self.norm_eps, self.flags)


@dataclass
class Views:
    """Device tensors of one view set: cam [V][16] f32, depth [V][H][W] f32, feat [V][Hf][Wf][D]."""
    cam: torch.Tensor
    depth: torch.Tensor | None
    feat: torch.Tensor | None = None
    H: int | None = None
    W: int | None = None

    def c(self):
        cam = _dev(self.cam, torch.float32, "cam")
        V = cam.shape[0]
        if self.depth is not None:
            depth = _dev(self.depth, torch.float32, "depth")
            H, W = depth.shape[1], depth.shape[2]
        else:
            H, W = self.H, self.W
        v = _ViewsT(V, H, W, 0, 0, 0, 0, cam.data_ptr(), _ptr(self.depth), None)
        if self.feat is not None:
            f = self.feat
            if not (f.is_cuda and f.is_contiguous() and f.dtype in _TORCH_DTYPE):
                raise TypeError("feat must be a contiguous device tensor of float32, bfloat16 or float16")
            v.Hf, v.Wf, v.D, v.feat_dtype, v.feat = f.shape[1], f.shape[2], f.shape[3], _TORCH_DTYPE[f.dtype], f.data_ptr()
        return v


def _dev(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{name} must be a contiguous device tensor of {dtype}")
    return t


def _ptr(t):
    return None if t is None else t.data_ptr()


def _temb(t):
    """Text embeddings [K][D]: float32, bfloat16 or float16."""
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype in _TORCH_DTYPE):
        raise TypeError("temb must be a contiguous device tensor of float32, bfloat16 or float16")
    return t


def _host(a, dtype):
    """Object offsets and grid descriptions live in host memory (numpy)."""
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _hptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, what):
    if status != 0:
        raise AuraError(status, what)


def workspace_bytes(call: int, N: int = 0, B: int = 1, D: int = 1, K: int = 1, G: int = 0, n_views: int = 1,
                    Hf: int = 1, Wf: int = 1, feat_dtype: int = F32, Ns: int = 1, P: int = 1) -> int:
    out = C.c_size_t(0)
    sz = _SizesT(N, B, n_views, Hf, Wf, D, feat_dtype, K, G, Ns, P)
    _check(lib().aura_workspace_bytes(call, C.byref(sz), C.byref(out)), "aura_workspace_bytes")
    return int(out.value)


def fuse_status_word(call: int, views: "Views", N: int, workspace, B: int = 1, K: int = 1, P: int = 1, G: int = 0,
                     word: int = 0):
    """The status word that the fusion kernels of `call` keep in `workspace` (read back, which synchronises): 0 =
    nothing to report; None where the sizes run kernels without one.  word = 1: the word after it, the number of
    tiles that were fused point by point because their cell lists outgrew their storage."""
    f = views.feat
    sz = _SizesT(N, B, f.shape[0], f.shape[1], f.shape[2], f.shape[3], _TORCH_DTYPE[f.dtype], K, G, 1, P)
    off, present = C.c_size_t(0), C.c_int32(0)
    _check(lib().aura_fuse_status_offset(call, C.byref(sz), C.byref(off), C.byref(present)), "aura_fuse_status_offset")
    if not present.value or workspace is None:
        return None
    return int(workspace[off.value + 4 * word:off.value + 4 * word + 4].view(torch.int32).item())


def fuse_workspace_bytes(views: "Views", N: int, B: int = 1) -> int:
    """Workspace size of fuse_features for these views (0 when the per-point gather kernel is used)."""
    f = views.feat
    return workspace_bytes(CALL_FUSE_FEATURES, N=N, B=B, D=f.shape[3], n_views=f.shape[0], Hf=f.shape[1],
                           Wf=f.shape[2], feat_dtype=_TORCH_DTYPE[f.dtype])


def _objects(pt_offsets, view_offsets):
    po, vo = _host(pt_offsets, np.int64), _host(view_offsets, np.int32)
    B = 1 if po is None else len(po) - 1
    return po, vo, B


def project_visibility(views: Views, params: Params, xyz, vis, count=None, uvz=None, pt_offsets=None,
                       view_offsets=None):
    """vis [N][vis_pitch] uint8, count [N] int32, uvz [N][vis_pitch][3] f32 are filled in place."""
    xyz = _dev(xyz, torch.float32, "xyz")
    _dev(vis, torch.uint8, "vis")
    po, vo, B = _objects(pt_offsets, view_offsets)
    v, p = views.c(), params.c()
    _check(lib().aura_project_visibility(C.byref(v), C.byref(p), xyz.data_ptr(), xyz.shape[0], _hptr(po), _hptr(vo),
                                         B, vis.data_ptr(), vis.shape[1], _ptr(count), _ptr(uvz), _stream()),
           "aura_project_visibility")


def fuse_features(views: Views, params: Params, xyz, fused, count=None, pt_offsets=None, view_offsets=None,
                  workspace=None):
    """fused [N][D] f32 and count [N] int32 are filled in place; workspace is a uint8 device tensor or None."""
    xyz = _dev(xyz, torch.float32, "xyz")
    _dev(fused, torch.float32, "fused")
    po, vo, B = _objects(pt_offsets, view_offsets)
    v, p = views.c(), params.c()
    _check(lib().aura_fuse_features(C.byref(v), C.byref(p), xyz.data_ptr(), xyz.shape[0], _hptr(po), _hptr(vo), B,
                                    fused.data_ptr(), _ptr(count), _ptr(workspace),
                                    0 if workspace is None else workspace.numel(), _stream()), "aura_fuse_features")


def material_scores(fused, temb, y, params: Params, scores, prop=None, label=None, workspace=None):
    """scores [N][K], prop [N][P], label [N] are filled in place; workspace is a uint8 device tensor."""
    fused = _dev(fused, torch.float32, "fused")
    temb = _temb(temb)
    N, D = fused.shape
    K = temb.shape[0]
    P = 0 if y is None else y.shape[1]
    p = params.c()
    _check(lib().aura_material_scores(fused.data_ptr(), N, D, temb.data_ptr(), _TORCH_DTYPE[temb.dtype], K, _ptr(y), P, C.byref(p),
                                      scores.data_ptr(), _ptr(prop), _ptr(label), _ptr(workspace),
                                      0 if workspace is None else workspace.numel(), _stream()),
           "aura_material_scores")


def material_scores_static(fused, temb, y, params: Params, scores, prop=None, label=None):
    """material_scores without a workspace: the scratch is a fixed array inside the library (nothing is allocated)."""
    fused = _dev(fused, torch.float32, "fused")
    temb = _temb(temb)
    N, D = fused.shape
    K = temb.shape[0]
    P = 0 if y is None else y.shape[1]
    p = params.c()
    _check(lib().aura_material_scores_static(fused.data_ptr(), N, D, temb.data_ptr(), _TORCH_DTYPE[temb.dtype], K, _ptr(y), P, C.byref(p),
                                             scores.data_ptr(), _ptr(prop), _ptr(label), _stream()),
           "aura_material_scores_static")


def fuse_scores_workspace_bytes(views: "Views", N: int, K: int, B: int = 1) -> int:
    """Workspace size of fuse_scores for these views and K materials."""
    f = views.feat
    return workspace_bytes(CALL_FUSE_SCORES, N=N, B=B, D=f.shape[3], K=K, n_views=f.shape[0], Hf=f.shape[1],
                           Wf=f.shape[2], feat_dtype=_TORCH_DTYPE[f.dtype])


def fuse_scores(views: Views, params: Params, xyz, temb, y, fused, scores, count=None, prop=None, label=None,
                pt_offsets=None, view_offsets=None, workspace=None, vis=None):
    """fuse_features followed by material_scores in one call; fused, count, scores, prop, label (and the
    visibility mask vis [N][vis_pitch] uint8, if given) filled in place."""
    xyz = _dev(xyz, torch.float32, "xyz")
    _dev(fused, torch.float32, "fused")
    temb = _temb(temb)
    po, vo, B = _objects(pt_offsets, view_offsets)
    v, p = views.c(), params.c()
    K = temb.shape[0]
    P = 0 if y is None else y.shape[1]
    _check(lib().aura_fuse_scores(C.byref(v), C.byref(p), xyz.data_ptr(), xyz.shape[0], _hptr(po), _hptr(vo), B,
                                  temb.data_ptr(), _TORCH_DTYPE[temb.dtype], K, _ptr(y), P, fused.data_ptr(), _ptr(count),
                                  _ptr(vis), 0 if vis is None else vis.shape[1], scores.data_ptr(), _ptr(prop), _ptr(label), _ptr(workspace),
                                  0 if workspace is None else workspace.numel(), _stream()), "aura_fuse_scores")


def fuse_score_integrate_workspace_bytes(views: "Views", N: int, K: int, P: int, B: int = 1, G: int = 0) -> int:
    """Workspace size of fuse_score_integrate for these views, K materials, P properties and a G^3 mass grid."""
    f = views.feat
    return workspace_bytes(CALL_FUSE_SCORE_INTEGRATE, N=N, B=B, D=f.shape[3], K=K, n_views=f.shape[0], Hf=f.shape[1],
                           Wf=f.shape[2], feat_dtype=_TORCH_DTYPE[f.dtype], P=P, G=G)


def fuse_score_integrate(views: Views, params: Params, xyz, temb, y, scores, mass, p_index=0, count=None, vis=None,
                         prop=None, label=None, n_used=None, vol=None, vol_uniform=1.0, pt_offsets=None,
                         view_offsets=None, grid_lo=None, grid_h=None, G=0, workspace=None):
    """The whole path in one call without the fused rows: scores [N][K] and mass [B] (and count, vis, prop, label,
    n_used when given) are filled in place."""
    xyz = _dev(xyz, torch.float32, "xyz")
    temb = _temb(temb)
    y = _dev(y, torch.float32, "y")
    _dev(scores, torch.float32, "scores")
    _dev(mass, torch.float32, "mass")
    po, vo, B = _objects(pt_offsets, view_offsets)
    glo, gh = _host(grid_lo, np.float32), _host(grid_h, np.float32)
    v, p = views.c(), params.c()
    _check(lib().aura_fuse_score_integrate(C.byref(v), C.byref(p), xyz.data_ptr(), xyz.shape[0], _hptr(po), _hptr(vo), B,
                                           temb.data_ptr(), _TORCH_DTYPE[temb.dtype], temb.shape[0], y.data_ptr(), y.shape[1],
                                           p_index,
                                           _ptr(vol), vol_uniform, _hptr(glo), _hptr(gh), G, _ptr(count), _ptr(vis),
                                           0 if vis is None else vis.shape[1], scores.data_ptr(), _ptr(prop), _ptr(label),
                                           mass.data_ptr(), _ptr(n_used), _ptr(workspace),
                                           0 if workspace is None else workspace.numel(), _stream()),
           "aura_fuse_score_integrate")


def time_next_fusion(start: "torch.cuda.Event | None", stop: "torch.cuda.Event | None"):
    """The next fusion call of this thread records the two events around its fusion kernel (both None: withdraw).
    The events must have been recorded once before, so that their handles exist."""
    h = lambda e: None if e is None else C.c_void_p(e.cuda_event)
    _check(lib().aura_time_next_fusion(h(start), h(stop)), "aura_time_next_fusion")


def knn_densify(fq, fs, ws, k, y, params: Params, wq, prop=None, label=None, nn_idx=None, workspace=None):
    """wq [Nq][K], prop [Nq][P], label [Nq], nn_idx [Nq][k] are filled in place; workspace is a uint8 device tensor."""
    fq = _dev(fq, torch.float32, "fq")
    fs = _dev(fs, torch.float32, "fs")
    ws = _dev(ws, torch.float32, "ws")
    Nq, D = fq.shape
    Ns, K = ws.shape
    P = 0 if y is None else y.shape[1]
    p = params.c()
    _check(lib().aura_knn_densify(fq.data_ptr(), Nq, D, fs.data_ptr(), Ns, ws.data_ptr(), K, k, _ptr(y), P, C.byref(p),
                                  wq.data_ptr(), _ptr(prop), _ptr(label), _ptr(nn_idx), _ptr(workspace),
                                  0 if workspace is None else workspace.numel(), _stream()), "aura_knn_densify")


def property_integrate(prop, mass, p_index=0, count=None, vol=None, vol_uniform=1.0, pt_offsets=None, xyz=None,
                       grid_lo=None, grid_h=None, G=0, n_used=None, workspace=None):
    """mass [B] f32 and n_used [B] int64 are filled in place."""
    prop = _dev(prop, torch.float32, "prop")
    N, P = prop.shape
    po = _host(pt_offsets, np.int64)
    B = 1 if po is None else len(po) - 1
    glo, gh = _host(grid_lo, np.float32), _host(grid_h, np.float32)
    _check(lib().aura_property_integrate(prop.data_ptr(), N, P, p_index, _ptr(count), _ptr(vol), vol_uniform,
                                         _hptr(po), B, _ptr(xyz), _hptr(glo), _hptr(gh), G, mass.data_ptr(),
                                         _ptr(n_used), _ptr(workspace),
                                         0 if workspace is None else workspace.numel(), _stream()),
           "aura_property_integrate")


def voxel_grid(box_lo, box_hi, n_target):
    """Sec. 3.2.1 (host only): s_voxel and the voxels per axis of one boundary box."""
    lo, hi = _host(box_lo, np.float32), _host(box_hi, np.float32)
    s, dims = C.c_float(0.0), np.zeros(3, np.int32)
    _check(lib().aura_voxel_grid(_hptr(lo), _hptr(hi), n_target, C.byref(s), _hptr(dims)), "aura_voxel_grid")
    return float(s.value), dims


def voxel_workspace_bytes(box_lo, box_hi, n_target):
    lo, hi = _host(box_lo, np.float32).reshape(-1, 3), _host(box_hi, np.float32).reshape(-1, 3)
    out = C.c_size_t(0)
    _check(lib().aura_voxel_workspace_bytes(_hptr(lo), _hptr(hi), lo.shape[0], n_target, C.byref(out)),
           "aura_voxel_workspace_bytes")
    return int(out.value)


def voxel_downsample(xyz, box_lo, box_hi, n_target, out_xyz, out_offsets, out_count=None, voxel_of_point=None,
                     pt_offsets=None, workspace=None):
    """Sec. 3.2.1: out_xyz [capacity][3] f32, out_offsets [B+1] int32 (and out_count [capacity], voxel_of_point [N]
    int32 when given) are filled in place; the boxes are host arrays [B][3]."""
    xyz = _dev(xyz, torch.float32, "xyz")
    lo, hi = _host(box_lo, np.float32).reshape(-1, 3), _host(box_hi, np.float32).reshape(-1, 3)
    po = _host(pt_offsets, np.int64)
    B = 1 if po is None else len(po) - 1
    _check(lib().aura_voxel_downsample(_ptr(xyz), xyz.shape[0], _hptr(po), B, _hptr(lo), _hptr(hi), n_target,
                                       _ptr(out_xyz), _ptr(out_count), 0 if out_xyz is None else out_xyz.shape[0],
                                       out_offsets.data_ptr(), _ptr(voxel_of_point), _ptr(workspace),
                                       0 if workspace is None else workspace.numel(), _stream()),
           "aura_voxel_downsample")


def patch_batch(cam, images, xyz, sel_view, scales, out, mean=None, inv_std=None, valid=None, pt_offsets=None,
                view_offsets=None):
    """Sec. 3.2.3: out [M][k][L][3][R][R] (float32 or float16) and valid [M][k] uint8 are filled in place; images
    [V][H][W][3] uint8 and cam [V][16] f32 are device tensors, scales / mean / inv_std host arrays."""
    cam = _dev(cam, torch.float32, "cam")
    images = _dev(images, torch.uint8, "images")
    xyz = _dev(xyz, torch.float32, "xyz")
    sel_view = _dev(sel_view, torch.int32, "sel_view")
    if not (out.is_cuda and out.is_contiguous() and out.dtype in (torch.float32, torch.float16)):
        raise TypeError("out must be a contiguous device tensor of float32 or float16")
    sc, mu, isd = _host(scales, np.float32), _host(mean, np.float32), _host(inv_std, np.float32)
    po, vo, B = _objects(pt_offsets, view_offsets)
    V, H, W, _ = images.shape
    M, k = sel_view.shape
    _check(lib().aura_patch_batch(cam.data_ptr(), V, H, W, images.data_ptr(), _ptr(xyz), M, _hptr(po), _hptr(vo), B,
                                  sel_view.data_ptr(), k, _hptr(sc), len(sc), out.shape[-1], _hptr(mu), _hptr(isd),
                                  out.data_ptr(), _TORCH_DTYPE[out.dtype], _ptr(valid), _stream()), "aura_patch_batch")


def estimate_normals(xyz, queries, centre, k, normals, evals=None, pt_offsets=None, q_offsets=None):
    """Sec. 3.2.2: normals [M][3] f32 (and evals [M][3] f32 when given) are filled in place; centre is a host array
    [B][3]."""
    xyz = _dev(xyz, torch.float32, "xyz")
    queries = _dev(queries, torch.float32, "queries")
    po, qo = _host(pt_offsets, np.int64), _host(q_offsets, np.int64)
    B = 1 if po is None else len(po) - 1
    ce = _host(centre, np.float32).reshape(B, 3)
    _check(lib().aura_estimate_normals(_ptr(xyz), xyz.shape[0], _hptr(po), _ptr(queries), queries.shape[0], _hptr(qo), B,
                                       _hptr(ce), k, normals.data_ptr(), _ptr(evals), _stream()), "aura_estimate_normals")


def select_views(views: "Views", params: "Params", xyz, normals, k, sel_view, sel_score=None, sel_mask=None, n_sel=None,
                 pt_offsets=None, view_offsets=None):
    """Sec. 3.2.2: sel_view [N][k] int32 (and sel_score [N][k] f32, sel_mask [N][pitch] uint8, n_sel [N] int32 when
    given) are filled in place."""
    xyz = _dev(xyz, torch.float32, "xyz")
    normals = _dev(normals, torch.float32, "normals")
    po, vo, B = _objects(pt_offsets, view_offsets)
    v, p = views.c(), params.c()
    _check(lib().aura_select_views(C.byref(v), C.byref(p), xyz.data_ptr(), normals.data_ptr(), xyz.shape[0], _hptr(po),
                                   _hptr(vo), B, k, sel_view.data_ptr(), _ptr(sel_score), _ptr(sel_mask),
                                   0 if sel_mask is None else sel_mask.shape[1], _ptr(n_sel), _stream()),
           "aura_select_views")


def fuse_selected(views: "Views", params: "Params", xyz, sel_mask, fused, count=None, pt_offsets=None, view_offsets=None,
                  workspace=None):
    """Sec. 3.2.3: Eq. 2 over the views marked in sel_mask [N][pitch] uint8; fused [N][D] f32 and count [N] int32
    are filled in place."""
    xyz = _dev(xyz, torch.float32, "xyz")
    _dev(sel_mask, torch.uint8, "sel_mask")
    po, vo, B = _objects(pt_offsets, view_offsets)
    v, p = views.c(), params.c()
    _check(lib().aura_fuse_selected(C.byref(v), C.byref(p), xyz.data_ptr(), xyz.shape[0], _hptr(po), _hptr(vo), B,
                                    sel_mask.data_ptr(), sel_mask.shape[1], fused.data_ptr(), _ptr(count),
                                    _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream()),
           "aura_fuse_selected")


def thickness_integrate(scores, y, theta, xyz, params: "Params", total, p_index=0, count=None, pt_offsets=None,
                        box_len=None, lam=0.6, scale_factor=1.0, zeta=None, com=None, b_adap=None, n_used=None,
                        workspace=None):
    """Sec. 3.4.2, thickness-based integration: total [B] f32 (and zeta [N], com [B][3], b_adap [B] f32, n_used [B]
    int64 when given) are filled in place."""
    scores = _dev(scores, torch.float32, "scores")
    N, K = scores.shape
    y = _dev(y, torch.float32, "y")
    P = y.shape[1]
    po = _host(pt_offsets, np.int64)
    B = 1 if po is None else len(po) - 1
    bl = _host(box_len, np.float32)
    p = params.c()
    _check(lib().aura_thickness_integrate(scores.data_ptr(), N, K, y.data_ptr(), P, p_index, _ptr(theta), _ptr(xyz),
                                          _ptr(count), _hptr(po), B, _hptr(bl), C.byref(p), lam, scale_factor,
                                          _ptr(zeta), total.data_ptr(), _ptr(com), _ptr(b_adap), _ptr(n_used),
                                          _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream()),
           "aura_thickness_integrate")


def calibration_copy(dst, src):
    """Plain device copy of src into dst (uint8 device tensors of equal size, a multiple of 16 bytes)."""
    _check(lib().aura_calibration_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), _stream()),
           "aura_calibration_copy")


def calibration_fill(dst, value=0):
    """Plain device fill of dst with a 32-bit pattern."""
    _check(lib().aura_calibration_fill(dst.data_ptr(), dst.numel() * dst.element_size(), value, _stream()),
           "aura_calibration_fill")
