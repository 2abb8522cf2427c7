"""ctypes front end of the CPU oracle (oracle/aura_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing here touches the GPU library, and the GPU
library never imports this module.  Arrays in, numpy arrays out; the arithmetic
is in the C file (see its header for the passages of the paper each part follows),
except estimate_normals, which is written out here with numpy (float64 covariance,
numpy.linalg.eigh).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "aura_oracle.c"
_LIB = _HERE / "libaura_oracle.so"

F32, BF16, F16 = 0, 1, 2
FLAG_FRUSTUM_ONLY, FLAG_MEAN_ONLY = 1, 2
DIAG_NEAR_THRESHOLD, DIAG_NEAR_PIXEL_EDGE, DIAG_F64_DIFFERS = 1, 2, 4

_DTYPES = {"f32": F32, "bf16": BF16, "f16": F16}


def build(force: bool = False) -> Path:
    """Compiles the oracle with gcc (no fast-math, no contraction, portable ISA)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", str(_LIB), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(str(_LIB))
        _lib.orc_max_threads.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _feat(feat, feat_dtype):
    """Stored feature maps: float32, or uint16 holding bf16 bits, or float16."""
    code = _DTYPES[feat_dtype]
    want = {F32: np.float32, BF16: np.uint16, F16: np.float16}[code]
    feat = np.ascontiguousarray(feat)
    if feat.dtype != want:
        raise TypeError(f"feat for {feat_dtype} must be {want}, got {feat.dtype}")
    return feat, code


def _csr(N, n_views, pt_offsets, view_offsets):
    if pt_offsets is None and view_offsets is None:
        return None, None, 1
    po = np.ascontiguousarray(pt_offsets, dtype=np.int64)
    vo = np.ascontiguousarray(view_offsets, dtype=np.int32)
    return po, vo, len(po) - 1


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def max_threads() -> int:
    return int(lib().orc_max_threads())


def set_threads(n: int) -> None:
    lib().orc_set_threads(C.c_int(n))


def project_point(cam16, xyz3):
    """One point, one camera -> (uvz fp32 chain, uvz double)."""
    cam16 = _f32(cam16).reshape(16)
    xyz3 = _f32(xyz3).reshape(3)
    o32 = np.zeros(3, np.float32)
    o64 = np.zeros(3, np.float64)
    _check(lib().orc_project_point(_p(cam16), _p(xyz3), _p(o32), _p(o64)), "project_point")
    return o32, o64


def sample_bilinear(feat_v, feat_dtype, H, W, u, v):
    """Bilinear sample of one view's [Hf][Wf][D] map at image location (u, v)."""
    feat_v, code = _feat(feat_v, feat_dtype)
    Hf, Wf, D = feat_v.shape
    out = np.zeros(D, np.float64)
    _check(lib().orc_sample_bilinear(_p(feat_v), C.c_int(code), C.c_int(Hf), C.c_int(Wf), C.c_int(D),
                                     C.c_int(H), C.c_int(W), C.c_float(u), C.c_float(v), _p(out)),
           "sample_bilinear")
    return out


def project_visibility(cam, depth, xyz, tau=0.0, z_near=1e-6, flags=0, pt_offsets=None,
                       view_offsets=None, vis_pitch=None, want_uvz=False, want_diag=False):
    cam = _f32(cam).reshape(-1, 16)
    depth = _f32(depth)
    xyz = _f32(xyz).reshape(-1, 3)
    n_views, H, W = depth.shape
    N = xyz.shape[0]
    po, vo, B = _csr(N, n_views, pt_offsets, view_offsets)
    if vis_pitch is None:
        vis_pitch = n_views if vo is None else int(np.max(np.diff(vo)))
    vis = np.zeros((N, vis_pitch), np.uint8)
    count = np.zeros(N, np.int32)
    uvz = np.zeros((N, vis_pitch, 3), np.float32) if want_uvz else None
    diag = np.zeros((N, vis_pitch), np.uint8) if want_diag else None
    rc = lib().orc_project_visibility(_p(cam), _p(depth), C.c_int(n_views), C.c_int(H), C.c_int(W),
                                      C.c_float(tau), C.c_float(z_near), C.c_uint(flags),
                                      _p(xyz), C.c_int64(N), _p(po), _p(vo), C.c_int(B), C.c_int(vis_pitch),
                                      _p(vis), _p(count), _p(uvz), _p(diag))
    _check(rc, "project_visibility")
    return {"vis": vis, "count": count, "uvz": uvz, "diag": diag}


def fuse_features(cam, depth, feat, feat_dtype, xyz, tau=0.0, z_near=1e-6, norm_eps=1e-12, flags=0,
                  pt_offsets=None, view_offsets=None, sel_mask=None):
    cam = _f32(cam).reshape(-1, 16)
    depth = _f32(depth)
    xyz = _f32(xyz).reshape(-1, 3)
    feat, code = _feat(feat, feat_dtype)
    n_views, H, W = depth.shape
    _, Hf, Wf, D = feat.shape
    if feat.shape[0] != n_views:
        raise ValueError("feat and depth disagree on the number of views")
    N = xyz.shape[0]
    po, vo, B = _csr(N, n_views, pt_offsets, view_offsets)
    fused = np.zeros((N, D), np.float64)
    count = np.zeros(N, np.int32)
    if sel_mask is not None:
        sel_mask = np.ascontiguousarray(sel_mask, dtype=np.uint8).reshape(N, -1)
    rc = lib().orc_fuse_features(_p(cam), _p(depth), _p(feat), C.c_int(code), C.c_int(n_views),
                                 C.c_int(H), C.c_int(W), C.c_int(Hf), C.c_int(Wf), C.c_int(D),
                                 C.c_float(tau), C.c_float(z_near), C.c_float(norm_eps), C.c_uint(flags),
                                 _p(xyz), C.c_int64(N), _p(po), _p(vo), C.c_int(B), _p(sel_mask),
                                 C.c_int(0 if sel_mask is None else sel_mask.shape[1]), _p(fused), _p(count))
    _check(rc, "fuse_features")
    return {"fused": fused, "count": count}


def material_scores(fused, temb, y=None, T=0.1, unseen_zero=False):
    fused = np.ascontiguousarray(fused, dtype=np.float64)
    temb = _f32(temb)
    N, D = fused.shape
    K = temb.shape[0]
    if temb.shape[1] != D:
        raise ValueError("temb and fused disagree on D")
    y = None if y is None else _f32(y).reshape(K, -1)
    P = 0 if y is None else y.shape[1]
    scores = np.zeros((N, K), np.float64)
    prop = np.zeros((N, P), np.float64) if y is not None else None
    label = np.zeros(N, np.int32)
    margin = np.zeros(N, np.float64)
    rc = lib().orc_material_scores(_p(fused), C.c_int64(N), C.c_int(D), _p(temb), C.c_int(K), _p(y), C.c_int(P),
                                   C.c_float(T), C.c_int(1 if unseen_zero else 0), _p(scores), _p(prop), _p(label),
                                   _p(margin))
    _check(rc, "material_scores")
    return {"scores": scores, "prop": prop, "label": label, "margin": margin}


def property_integrate(prop, p_index=0, count=None, vol=None, vol_uniform=1.0, pt_offsets=None,
                       xyz=None, grid_lo=None, grid_h=None, G=0):
    prop = np.ascontiguousarray(prop, dtype=np.float64)
    if prop.ndim == 1:
        prop = prop[:, None]
    N, P = prop.shape
    po = None if pt_offsets is None else np.ascontiguousarray(pt_offsets, dtype=np.int64)
    B = 1 if po is None else len(po) - 1
    count = None if count is None else np.ascontiguousarray(count, dtype=np.int32)
    vol = _f32(vol)
    xyz = None if xyz is None else _f32(xyz).reshape(-1, 3)
    grid_lo = None if grid_lo is None else _f32(grid_lo).reshape(B, 3)
    grid_h = None if grid_h is None else _f32(grid_h).reshape(B)
    mass = np.zeros(B, np.float64)
    n_used = np.zeros(B, np.int64)
    rc = lib().orc_property_integrate(_p(prop), C.c_int64(N), C.c_int(P), C.c_int(p_index), _p(count), _p(vol),
                                      C.c_float(vol_uniform), _p(po), C.c_int(B), _p(xyz), _p(grid_lo),
                                      _p(grid_h), C.c_int(G), _p(mass), _p(n_used))
    _check(rc, "property_integrate")
    return {"mass": mass, "n_used": n_used}


def knn_densify(fq, fs, ws, k, y=None, T=0.1):
    """Eq. 5: material vectors of the queries from their k nearest sources in feature space, then Eq. 4."""
    fq = np.ascontiguousarray(fq, dtype=np.float64)
    fs = np.ascontiguousarray(fs, dtype=np.float64)
    ws = np.ascontiguousarray(ws, dtype=np.float64)
    Nq, D = fq.shape
    Ns, K = ws.shape
    if fs.shape != (Ns, D):
        raise ValueError("fs must be [Ns][D]")
    y = None if y is None else _f32(y).reshape(K, -1)
    P = 0 if y is None else y.shape[1]
    wq = np.zeros((Nq, K), np.float64)
    prop = np.zeros((Nq, P), np.float64) if y is not None else None
    label = np.zeros(Nq, np.int32)
    nn_idx = np.zeros((Nq, k), np.int32)
    nn_sim = np.zeros((Nq, k), np.float64)
    gap = np.zeros(Nq, np.float64)
    rc = lib().orc_knn_densify(_p(fq), C.c_int64(Nq), _p(fs), C.c_int(Ns), C.c_int(D), _p(ws), C.c_int(K), C.c_int(k),
                               _p(y), C.c_int(P), C.c_float(T), _p(wq), _p(prop), _p(label), _p(nn_idx), _p(nn_sim),
                               _p(gap))
    _check(rc, "knn_densify")
    return {"wq": wq, "prop": prop, "label": label, "nn_idx": nn_idx, "nn_sim": nn_sim, "gap": gap}


def thickness_integrate(omega, y_col, theta, xyz, count=None, pt_offsets=None, box_len=None, T=0.1, lam=0.6,
                        scale_factor=1.0):
    """Sec. 3.4.2: thickness-based voxel integration (voxel b_adap x b_adap x theta_k, factor lambda) and the
    centre of mass of the integrated quantity."""
    omega = np.ascontiguousarray(omega, dtype=np.float64)
    N, K = omega.shape
    y_col, theta = _f32(y_col).reshape(K), _f32(theta).reshape(K)
    xyz = _f32(xyz).reshape(N, 3)
    po = None if pt_offsets is None else np.ascontiguousarray(pt_offsets, dtype=np.int64)
    B = 1 if po is None else len(po) - 1
    count = None if count is None else np.ascontiguousarray(count, dtype=np.int32)
    box_len = None if box_len is None else _f32(box_len).reshape(B)
    zeta = np.zeros(N, np.float64)
    total = np.zeros(B, np.float64)
    com = np.zeros((B, 3), np.float64)
    b_adap = np.zeros(B, np.float64)
    n_used = np.zeros(B, np.int64)
    rc = lib().orc_thickness_integrate(_p(omega), C.c_int64(N), C.c_int(K), _p(y_col), _p(theta), _p(xyz), _p(count),
                                       _p(po), C.c_int(B), _p(box_len), C.c_float(T), C.c_float(lam),
                                       C.c_float(scale_factor), _p(zeta), _p(total), _p(com), _p(b_adap), _p(n_used))
    _check(rc, "thickness_integrate")
    return {"zeta": zeta, "mass": total, "com": com, "b_adap": b_adap, "n_used": n_used}


def select_views(cam, depth, xyz, normals, k, tau=0.0, z_near=1e-6, flags=0, pt_offsets=None, view_offsets=None,
                 mask_pitch=None, H=None, W=None):
    """Sec. 3.2.2: S_total = S_dist * S_angle of every visible pair, the k best views per point."""
    cam = _f32(cam).reshape(-1, 16)
    depth = _f32(depth)
    xyz = _f32(xyz).reshape(-1, 3)
    normals = _f32(normals).reshape(-1, 3)
    n_views = cam.shape[0]
    if depth is not None:
        _, H, W = depth.shape
    N = xyz.shape[0]
    po, vo, B = _csr(N, n_views, pt_offsets, view_offsets)
    if mask_pitch is None:
        mask_pitch = n_views if vo is None else int(np.diff(vo).max())
    sel_view = np.zeros((N, k), np.int32)
    sel_score = np.zeros((N, k), np.float64)
    sel_mask = np.zeros((N, mask_pitch), np.uint8)
    n_sel = np.zeros(N, np.int32)
    gap = np.zeros(N, np.float64)
    score_all = np.zeros((N, mask_pitch), np.float64)
    rc = lib().orc_select_views(_p(cam), _p(depth), C.c_int(n_views), C.c_int(H), C.c_int(W), C.c_float(tau),
                                C.c_float(z_near), C.c_uint(flags), _p(xyz), _p(normals), C.c_int64(N), _p(po), _p(vo),
                                C.c_int(B), C.c_int(k), C.c_int(mask_pitch), _p(sel_view), _p(sel_score), _p(sel_mask),
                                _p(n_sel), _p(gap), _p(score_all))
    _check(rc, "select_views")
    return {"sel_view": sel_view, "sel_score": sel_score, "sel_mask": sel_mask, "n_sel": n_sel, "gap": gap,
            "score_all": score_all}


def voxel_grid(box_lo, box_hi, n_target):
    """Sec. 3.2.1: s_voxel = cbrt(V_bound / N_target) and the number of voxels per axis."""
    lo, hi = _f32(box_lo).reshape(3), _f32(box_hi).reshape(3)
    s = C.c_float(0.0)
    dims = np.zeros(3, np.int32)
    _check(lib().orc_voxel_grid(_p(lo), _p(hi), C.c_int(n_target), C.byref(s), _p(dims)), "voxel_grid")
    return float(s.value), dims


def voxel_downsample(xyz, n_target, box_lo=None, box_hi=None, pt_offsets=None, capacity=None):
    """Sec. 3.2.1: adaptive voxel down-sampling; the box defaults to the bounding box of each object's points."""
    xyz = _f32(xyz).reshape(-1, 3)
    N = xyz.shape[0]
    po = None if pt_offsets is None else np.ascontiguousarray(pt_offsets, dtype=np.int64)
    B = 1 if po is None else len(po) - 1
    if box_lo is None:
        rng = [(0, N)] if po is None else [(int(po[b]), int(po[b + 1])) for b in range(B)]
        box_lo = np.stack([xyz[a:b].min(0) if b > a else np.zeros(3, np.float32) for a, b in rng])
        box_hi = np.stack([xyz[a:b].max(0) if b > a else np.zeros(3, np.float32) for a, b in rng])
    lo, hi = _f32(box_lo).reshape(B, 3), _f32(box_hi).reshape(B, 3)
    cap = N if capacity is None else int(capacity)
    out_xyz = np.zeros((max(cap, 1), 3), np.float64)
    out_count = np.zeros(max(cap, 1), np.int32)
    out_offsets = np.zeros(B + 1, np.int64)
    voxel_of_point = np.zeros(max(N, 1), np.int64)
    _check(lib().orc_voxel_downsample(_p(xyz), C.c_int64(N), _p(po), C.c_int(B), _p(lo), _p(hi), C.c_int(n_target),
                                      _p(out_xyz), _p(out_count), C.c_int64(cap), _p(out_offsets), _p(voxel_of_point)),
           "voxel_downsample")
    M = min(int(out_offsets[B]), cap)
    return {"xyz": out_xyz[:M], "count": out_count[:M], "offsets": out_offsets, "voxel_of_point": voxel_of_point[:N],
            "box_lo": lo, "box_hi": hi}


def patch_batch(cam, images, xyz, sel_view, scales, R, mean=None, inv_std=None, pt_offsets=None, view_offsets=None):
    """Sec. 3.2.3: the multi-scale patches of every (point, kept view) as one batch [M][k][L][3][R][R]."""
    cam = _f32(cam).reshape(-1, 16)
    images = np.ascontiguousarray(images, dtype=np.uint8)
    n_views, H, W, _ = images.shape
    xyz = _f32(xyz).reshape(-1, 3)
    M = xyz.shape[0]
    sel_view = np.ascontiguousarray(sel_view, dtype=np.int32).reshape(M, -1)
    k = sel_view.shape[1]
    scales = _f32(scales).reshape(-1)
    L = len(scales)
    po, vo, B = _csr(M, n_views, pt_offsets, view_offsets)
    mean, inv_std = _f32(mean), _f32(inv_std)
    out = np.zeros((M, k, L, 3, R, R), np.float64)
    valid = np.zeros((M, k), np.uint8)
    rc = lib().orc_patch_batch(_p(cam), C.c_int(n_views), C.c_int(H), C.c_int(W), _p(images), _p(xyz), C.c_int64(M),
                               _p(po), _p(vo), C.c_int(B), _p(sel_view), C.c_int(k), _p(scales), C.c_int(L), C.c_int(R),
                               _p(mean), _p(inv_std), _p(out), _p(valid))
    _check(rc, "patch_batch")
    return {"patches": out, "valid": valid}


def estimate_normals(xyz, queries, centre, k, pt_offsets=None, q_offsets=None):
    """Sec. 3.2.2 (the normals of the sampled points, which the view importance score needs): for every query the
    plane through its k nearest points of the object's cloud, i.e. the eigenvector of the smallest eigenvalue of their
    covariance, turned to point away from the object's centre.

    Which points are nearest is decided in fp32 with one fixed operation order, d = (dx * dx + dy * dy) + dz * dz with
    dx = p_x - q_x and every operation rounded to fp32 (numpy float32 arithmetic), and of equal distances the lower
    index first, so that an fp32 implementation selects the same neighbours; means, covariance (numpy, float64) and the eigenvectors (numpy.linalg.eigh) are double.
    Returns normals [M][3], the neighbour indices [M][k] (within the object, -1 beyond its size), the eigenvalues
    [M][3] ascending, and the gap between the k-th distance and the next one."""
    xyz = _f32(xyz).reshape(-1, 3)
    queries = _f32(queries).reshape(-1, 3)
    N, M = len(xyz), len(queries)
    po = np.array([0, N], np.int64) if pt_offsets is None else np.asarray(pt_offsets, np.int64)
    qo = np.array([0, M], np.int64) if q_offsets is None else np.asarray(q_offsets, np.int64)
    B = len(po) - 1
    centre = _f32(centre).reshape(B, 3)
    normals = np.zeros((M, 3), np.float64)
    nn = np.full((M, k), -1, np.int64)
    evals = np.zeros((M, 3), np.float64)
    gap = np.full(M, np.inf)
    for b in range(B):
        P = xyz[po[b]:po[b + 1]]
        for m in range(int(qo[b]), int(qo[b + 1])):
            q = queries[m]
            if len(P) == 0:
                continue
            d = P - q                                                    # fp32 throughout
            t = (d[:, 0] * d[:, 0] + d[:, 1] * d[:, 1]) + d[:, 2] * d[:, 2]
            assert t.dtype == np.float32
            order = np.argsort(t, kind="stable")
            kk = min(k, len(P))
            sel = order[:kk]
            nn[m, :kk] = sel
            if kk < len(P):
                gap[m] = float(t[order[kk]]) - float(t[order[kk - 1]])
            pts = P[sel].astype(np.float64)
            c = pts.mean(0)
            cov = (pts - c).T @ (pts - c) / kk
            w, v = np.linalg.eigh(cov)
            n = v[:, 0]
            out = q.astype(np.float64) - centre[b].astype(np.float64)
            if n @ out < 0:
                n = -n
            normals[m] = n
            evals[m] = w
    return {"normals": normals, "nn_idx": nn, "evals": evals, "gap": gap}
