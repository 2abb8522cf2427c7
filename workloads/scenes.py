"""Seeded synthetic scenes shaped like the paper's workloads.

This module only MAKES INPUTS: point sets on unions of ellipsoids, pinhole cameras on
a sphere (or a frontal arc), depth maps rendered by a z-buffer splat of the points,
patch-feature maps built from per-material prototype vectors plus noise, and a material
dictionary (unit text embeddings, density, hardness).  It stands in for the paper's
captured objects (ABO catalogue objects, smart-glasses captures), which are not
reproduced.  It holds none of the fusion / scoring / integration arithmetic: the depth
splat below is scene rendering done independently in float64, and neither the GPU
library nor the CPU oracle imports anything from here except through the arrays.

Every scene is a pure function of (preset name, seed, size overrides).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20251103


@dataclass
class Scene:
    name: str
    xyz: np.ndarray            # [N][3] float32, world frame, objects concatenated
    pt_offsets: np.ndarray     # [B+1] int64
    view_offsets: np.ndarray   # [B+1] int32
    cam: np.ndarray            # [V][16] float32: R row-major, t, fx, fy, cx, cy
    depth: np.ndarray          # [V][H][W] float32, +inf where nothing was splatted
    feat: np.ndarray           # [V][Hf][Wf][D] float32 | uint16 (bf16 bits) | float16
    feat_dtype: str            # "f32" | "bf16" | "f16"
    temb: np.ndarray           # [K][D] float32 unit vectors
    y: np.ndarray              # [K][P] float32: column 0 density kg/m^3, column 1 hardness
    tau: float
    z_near: float = 1e-6
    temperature: float = 0.1
    G: int = 0                 # 0 = point-volume integration
    grid_lo: np.ndarray | None = None   # [B][3] float32
    grid_h: np.ndarray | None = None    # [B] float32
    vol_uniform: float = 1.0
    material_of_point: np.ndarray | None = None   # [N] int32 ground-truth material (logging only)
    meta: dict = field(default_factory=dict)

    @property
    def N(self): return int(self.xyz.shape[0])
    @property
    def B(self): return int(len(self.pt_offsets) - 1)
    @property
    def n_views(self): return int(self.cam.shape[0])
    @property
    def H(self): return int(self.depth.shape[1])
    @property
    def W(self): return int(self.depth.shape[2])
    @property
    def Hf(self): return int(self.feat.shape[1])
    @property
    def Wf(self): return int(self.feat.shape[2])
    @property
    def D(self): return int(self.feat.shape[3])
    @property
    def K(self): return int(self.temb.shape[0])
    @property
    def P(self): return int(self.y.shape[1])
    @property
    def point_views(self):
        return int(np.sum(np.diff(self.pt_offsets) * np.diff(self.view_offsets).astype(np.int64)))
    @property
    def vis_pitch(self): return int(np.max(np.diff(self.view_offsets)))


PRESETS = {
    # the five benchmark configurations, index 0..4
    "c1": dict(index=0, N=20_000, n_ell=1, V=8, radius=2.5, HW=224, f=250.0, grid=16, D=512, dtype="f32",
               K=12, parts=3, P=1, sigma=0.3, G=64, footprint=1, axes=(0.3, 1.0)),
    "c2": dict(index=1, N=200_000, n_ell=4, V=16, radius=3.0, HW=448, f=500.0, grid=32, D=768, dtype="bf16",
               K=32, parts=8, P=2, sigma=0.3, G=128, footprint=0, axes=(0.3, 1.0)),
    "c3": dict(index=2, N=1_000_000, n_ell=6, V=32, radius=3.0, HW=224, f=250.0, grid=224, D=512, dtype="f16",
               K=64, parts=16, P=1, sigma=0.2, G=128, footprint=0, axes=(0.3, 1.0), smooth=True),
    "c4": dict(index=3, voxel_res=256, n_ell=8, V=24, radius=4.5, HW=448, f=500.0, grid=56, D=1024, dtype="bf16",
               K=128, parts=8, P=2, sigma=0.3, G=0, footprint=0, axes=(0.3, 1.0), occupancy=0.10),
    "c5": dict(index=4, B=64, N=100_000, n_ell=(1, 3), V=4, radius=1.5, HW=224, f=250.0, grid=16, D=512,
               dtype="f16", K=24, parts=(1, 3), P=1, sigma=0.3, G=64, footprint=1, axes=(0.15, 0.5), arc=True),
}


# ----------------------------------------------------------------------------- storage dtypes

def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return to_bf16_bits(x)
    if dtype == "f16":
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16)
    raise ValueError(dtype)


def stored_to_f32(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_to_f32(a)
    return a.astype(np.float32)


# ----------------------------------------------------------------------------- geometry

def _random_rotation(rng):
    q, r = np.linalg.qr(rng.standard_normal((3, 3)))
    q = q * np.sign(np.diag(r))
    if np.linalg.det(q) < 0:
        q[:, 0] = -q[:, 0]
    return q


def _make_ellipsoids(rng, n, axes_range, spread=0.4):
    ells = []
    for e in range(n):
        centre = np.zeros(3) if e == 0 else rng.uniform(-spread, spread, 3)
        ells.append(dict(c=centre, R=_random_rotation(rng), a=rng.uniform(axes_range[0], axes_range[1], 3)))
    return ells


def _inside(ell, pts, shrink=1.0):
    loc = (pts - ell["c"]) @ ell["R"]          # coordinates in the ellipsoid's frame
    return np.sum((loc / (ell["a"] * shrink)) ** 2, axis=1) < 1.0


def _bands(loc_first_axis, a0, nb):
    t = np.clip((loc_first_axis / a0 + 1.0) * 0.5, 0.0, 1.0 - 1e-9)
    return np.floor(t * nb).astype(np.int32)


def _split_parts(n_parts, n_ell):
    base = [n_parts // n_ell] * n_ell
    for e in range(n_parts - sum(base)):
        base[e] += 1
    return [max(1, b) for b in base]


def _sample_union_surface(rng, ells, N, n_parts):
    """N points on the boundary of the union; returns xyz (float64) and a part id per point."""
    n_ell = len(ells)
    area = np.array([(e["a"][0] * e["a"][1] + e["a"][1] * e["a"][2] + e["a"][0] * e["a"][2]) / 3.0 for e in ells])
    bands = _split_parts(n_parts, n_ell)
    part_base = np.concatenate([[0], np.cumsum(bands)])
    pts, parts = [], []
    have = 0
    while have < N:
        want = int((N - have) * 1.6) + 64
        which = rng.choice(n_ell, size=want, p=area / area.sum())
        d = rng.standard_normal((want, 3))
        d /= np.linalg.norm(d, axis=1, keepdims=True)
        p = np.empty((want, 3))
        part = np.empty(want, np.int32)
        for e, ell in enumerate(ells):
            m = which == e
            loc = d[m] * ell["a"]
            p[m] = loc @ ell["R"].T + ell["c"]
            part[m] = part_base[e] + _bands(loc[:, 0], ell["a"][0], bands[e])
        keep = np.ones(want, bool)
        for e, ell in enumerate(ells):
            keep &= ~(_inside(ell, p) & (which != e))
        pts.append(p[keep])
        parts.append(part[keep])
        have += int(keep.sum())
    return np.concatenate(pts)[:N], np.concatenate(parts)[:N]


def _voxel_centres(rng, ells, res, occupancy, n_parts):
    """Centres of the voxels of a res^3 grid over [-1,1]^3 that fall inside the union, after
    scaling all semi-axes by one common factor so that the solid occupancy hits the target."""
    def occ(scale, r):
        h = 2.0 / r
        g = -1.0 + (np.arange(r) + 0.5) * h
        cnt = 0
        for iz in range(r):
            X, Y = np.meshgrid(g, g, indexing="xy")
            p = np.stack([X.ravel(), Y.ravel(), np.full(r * r, g[iz])], 1)
            m = np.zeros(r * r, bool)
            for ell in ells:
                m |= _inside(ell, p, scale)
            cnt += int(m.sum())
        return cnt / float(r ** 3)
    lo, hi = 0.05, 2.0
    coarse = min(res, 64)
    for _ in range(24):
        mid = 0.5 * (lo + hi)
        if occ(mid, coarse) > occupancy:
            hi = mid
        else:
            lo = mid
    scale = 0.5 * (lo + hi)
    for ell in ells:
        ell["a"] = ell["a"] * scale
    h = 2.0 / res
    g = -1.0 + (np.arange(res) + 0.5) * h
    pts, parts = [], []
    bands = _split_parts(n_parts, len(ells))
    part_base = np.concatenate([[0], np.cumsum(bands)])
    for iz in range(res):
        X, Y = np.meshgrid(g, g, indexing="xy")
        p = np.stack([X.ravel(), Y.ravel(), np.full(res * res, g[iz])], 1)
        owner = np.full(res * res, -1, np.int32)
        part = np.zeros(res * res, np.int32)
        for e in reversed(range(len(ells))):
            ell = ells[e]
            m = _inside(ell, p)
            owner[m] = e
            loc = (p[m] - ell["c"]) @ ell["R"]
            part[m] = part_base[e] + _bands(loc[:, 0], ell["a"][0], bands[e])
        sel = owner >= 0
        pts.append(p[sel])
        parts.append(part[sel])
    return np.concatenate(pts), np.concatenate(parts), h


def morton_order(xyz: np.ndarray) -> np.ndarray:
    """Permutation that sorts points along a 3-D Z-order curve (10 bits per axis)."""
    lo = xyz.min(0)
    span = np.maximum(xyz.max(0) - lo, 1e-12)
    q = np.minimum(((xyz - lo) / span * 1024.0).astype(np.uint64), np.uint64(1023))
    def spread(v):
        v = (v | (v << np.uint64(16))) & np.uint64(0x030000FF)
        v = (v | (v << np.uint64(8))) & np.uint64(0x0300F00F)
        v = (v | (v << np.uint64(4))) & np.uint64(0x030C30C3)
        v = (v | (v << np.uint64(2))) & np.uint64(0x09249249)
        return v
    key = spread(q[:, 0]) | (spread(q[:, 1]) << np.uint64(1)) | (spread(q[:, 2]) << np.uint64(2))
    return np.argsort(key, kind="stable")


# ----------------------------------------------------------------------------- cameras

def _look_at(centre, f, cx, cy):
    fwd = -centre / np.linalg.norm(centre)
    up = np.array([0.0, 0.0, 1.0])
    if abs(float(fwd @ up)) > np.cos(np.deg2rad(1.0)):
        up = np.array([0.0, 1.0, 0.0])
    right = np.cross(fwd, up)
    right /= np.linalg.norm(right)
    down = np.cross(fwd, right)
    R = np.stack([right, down, fwd])
    t = -R @ centre
    return np.concatenate([R.ravel(), t, [f, f, cx, cy]])


def cameras_on_sphere(V, radius, f, HW):
    """V cameras on a golden-angle lattice of the sphere, all looking at the origin."""
    cams = []
    ga = np.pi * (3.0 - np.sqrt(5.0))
    for i in range(V):
        z = 1.0 - (2.0 * i + 1.0) / V
        r = np.sqrt(max(0.0, 1.0 - z * z))
        c = radius * np.array([r * np.cos(i * ga), r * np.sin(i * ga), z])
        cams.append(_look_at(c, f, HW / 2.0, HW / 2.0))
    return np.array(cams)


def cameras_on_arc(V, radius, f, HW, arc_deg=60.0):
    """V cameras on a frontal arc at elevation 0, looking at the origin."""
    az = np.deg2rad(np.linspace(-arc_deg / 2.0, arc_deg / 2.0, V)) if V > 1 else np.array([0.0])
    return np.array([_look_at(radius * np.array([np.sin(a), -np.cos(a), 0.0]), f, HW / 2.0, HW / 2.0) for a in az])


# ----------------------------------------------------------------------------- rendering inputs

def _project64(cam, pts):
    R = cam[:9].reshape(3, 3)
    Xc = pts @ R.T + cam[9:12]
    z = Xc[:, 2]
    with np.errstate(divide="ignore", invalid="ignore"):
        u = cam[12] * Xc[:, 0] / z + cam[14]
        v = cam[13] * Xc[:, 1] / z + cam[15]
    return u, v, z


def splat_depth(cam, pts, H, W, footprint):
    """z-buffer splat: every point writes min z into its pixel and a (2r+1)^2 footprint."""
    u, v, z = _project64(cam, pts)
    ok = (z > 1e-6) & (u >= 0) & (u < W) & (v >= 0) & (v < H)
    px = np.floor(u[ok]).astype(np.int64)
    py = np.floor(v[ok]).astype(np.int64)
    zz = z[ok]
    d = np.full(H * W, np.inf)
    for dy in range(-footprint, footprint + 1):
        for dx in range(-footprint, footprint + 1):
            x, yy = px + dx, py + dy
            m = (x >= 0) & (x < W) & (yy >= 0) & (yy < H)
            np.minimum.at(d, yy[m] * W + x[m], zz[m])
    return d.reshape(H, W)


def _cell_materials(cam, pts, mats, depth64, tau, H, W, Hf, Wf, K):
    """Per feature cell, the majority material of the points seen there (-1: none)."""
    u, v, z = _project64(cam, pts)
    ok = (z > 1e-6) & (u >= 0) & (u < W) & (v >= 0) & (v < H)
    idx = np.nonzero(ok)[0]
    px = np.floor(u[idx]).astype(np.int64)
    py = np.floor(v[idx]).astype(np.int64)
    seen = z[idx] <= depth64[py, px] + tau
    idx, px, py = idx[seen], px[seen], py[seen]
    cx = np.minimum((u[idx] * (Wf / W)).astype(np.int64), Wf - 1)
    cy = np.minimum((v[idx] * (Hf / H)).astype(np.int64), Hf - 1)
    votes = np.bincount((cy * Wf + cx) * K + mats[idx], minlength=Hf * Wf * K).reshape(Hf * Wf, K)
    best = votes.argmax(1).astype(np.int32)
    best[votes.sum(1) == 0] = -1
    return best.reshape(Hf, Wf)


def _box3(w):
    p = np.pad(w, ((1, 1), (1, 1), (0, 0)), mode="edge")
    out = np.zeros_like(w)
    for dy in range(3):
        for dx in range(3):
            out += p[dy:dy + w.shape[0], dx:dx + w.shape[1]]
    return out / 9.0


def _feature_map(rng, cell_mat, proto, sigma, smooth):
    Hf, Wf = cell_mat.shape
    K, D = proto.shape
    if smooth:
        w = np.zeros((Hf, Wf, K), np.float32)
        yy, xx = np.nonzero(cell_mat >= 0)
        w[yy, xx, cell_mat[yy, xx]] = 1.0
        base = (_box3(w).reshape(-1, K) @ proto).reshape(Hf, Wf, D)
    else:
        base = np.where((cell_mat >= 0)[..., None], proto[np.maximum(cell_mat, 0)], np.float32(0.0))
    f = base.astype(np.float32) + np.float32(sigma) * rng.standard_normal((Hf, Wf, D), dtype=np.float32)
    f /= np.maximum(np.linalg.norm(f, axis=2, keepdims=True), 1e-12)
    return f


def _materials(rng, K, D, P):
    proto = rng.standard_normal((K, D)).astype(np.float32)
    proto /= np.linalg.norm(proto, axis=1, keepdims=True)
    y = np.empty((K, P), np.float32)
    y[:, 0] = rng.uniform(100.0, 8000.0, K)
    if P > 1:
        y[:, 1] = rng.uniform(0.0, 1.0, K)
    for p in range(2, P):
        y[:, p] = rng.uniform(0.0, 1.0, K)
    return proto, y


def material_thickness(K: int, seed: int) -> np.ndarray:
    """Thickness theta_k of each candidate material in scene units (2 mm to 5 cm, as a language model would
    propose for shells of everyday objects): the per-material input of the thickness-based integration."""
    rng = np.random.default_rng([seed, 77])
    return rng.uniform(0.002, 0.05, K).astype(np.float32)


def synthetic_images(n_views: int, H: int, W: int, seed: int) -> np.ndarray:
    """[n_views][H][W][3] uint8 pictures: smooth colour gradients and blobs plus pixel noise (stand in for the RGB
    captures that the patches of Sec. 3.2.3 are cut from)."""
    rng = np.random.default_rng([seed, 55])
    yy, xx = np.mgrid[0:H, 0:W].astype(np.float32)
    out = np.empty((n_views, H, W, 3), np.uint8)
    for v in range(n_views):
        img = np.empty((H, W, 3), np.float32)
        for c in range(3):
            fx, fy, ph = rng.uniform(0.01, 0.08, 2).tolist() + [rng.uniform(0, 6.28)]
            img[..., c] = 128 + 70 * np.sin(fx * xx + fy * yy + ph) + 30 * np.sin(3.1 * fx * yy - 2.3 * fy * xx)
        img += rng.normal(0, 12, img.shape).astype(np.float32)
        out[v] = np.clip(np.rint(img), 0, 255).astype(np.uint8)
    return out


def synthetic_normals(xyz: np.ndarray, pt_offsets: np.ndarray, seed: int, noise: float = 0.2) -> np.ndarray:
    """Unit "outward" normals for a scene's points: the direction from the object's centroid to the point, perturbed
    by Gaussian noise and renormalised (stands in for normals estimated from the reconstructed cloud)."""
    rng = np.random.default_rng([seed, 91])
    out = np.empty_like(xyz, dtype=np.float32)
    for b in range(len(pt_offsets) - 1):
        s_ = slice(int(pt_offsets[b]), int(pt_offsets[b + 1]))
        if s_.stop == s_.start:
            continue
        d = xyz[s_].astype(np.float64) - xyz[s_].astype(np.float64).mean(0)
        d /= np.maximum(np.linalg.norm(d, axis=1, keepdims=True), 1e-12)
        d += noise * rng.standard_normal(d.shape)
        d /= np.maximum(np.linalg.norm(d, axis=1, keepdims=True), 1e-12)
        out[s_] = d.astype(np.float32)
    return out


def _grid_for(points, G):
    lo, hi = points.min(0), points.max(0)
    h = 1.001 * max(float(np.max(hi - lo)), 1e-6) / G
    glo = 0.5 * (lo + hi) - 0.5 * G * h
    return glo.astype(np.float32), np.float32(h)


# ----------------------------------------------------------------------------- scene assembly

def make_scene(name: str, *, n_points: int | None = None, n_objects: int | None = None,
               voxel_res: int | None = None, ragged_views: bool = False, order: str = "morton",
               seed: int | None = None, overrides: dict | None = None) -> Scene:
    """Builds preset `name` ("c1".."c5").  n_points / n_objects / voxel_res shrink it for quick
    runs; ragged_views draws 2..V views per object (batched preset); order is "morton" or "random"."""
    cfg = dict(PRESETS[name])
    if overrides:
        cfg.update(overrides)
    seed = BASE_SEED + cfg["index"] if seed is None else seed
    B = int(n_objects if n_objects is not None else cfg.get("B", 1))
    HW, f, Gf, D, K, P = cfg["HW"], cfg["f"], cfg["grid"], cfg["D"], cfg["K"], cfg["P"]
    G = cfg["G"]
    mrng = np.random.default_rng([seed, 7])
    proto, y = _materials(mrng, K, D, P)

    xyz_all, mat_all, cams, depths, feats = [], [], [], [], []
    pt_off, view_off = [0], [0]
    glo, gh, taus = [], [], []
    vol_uniform = 1.0
    for b in range(B):
        rng = np.random.default_rng([seed + 1000 * b, 11])
        n_ell = cfg["n_ell"] if isinstance(cfg["n_ell"], int) else int(rng.integers(cfg["n_ell"][0], cfg["n_ell"][1] + 1))
        n_parts = cfg["parts"] if isinstance(cfg["parts"], int) else n_ell
        ells = _make_ellipsoids(rng, n_ell, cfg["axes"], spread=0.4 if not cfg.get("arc") else 0.15)
        if "voxel_res" in cfg:
            res = int(voxel_res or cfg["voxel_res"])
            pts, part, h = _voxel_centres(rng, ells, res, cfg["occupancy"], n_parts)
            vol_uniform = float(np.float32(h) ** 3)
        else:
            pts, part = _sample_union_surface(rng, ells, int(n_points or cfg["N"]), n_parts)
        part_mat = rng.choice(K, size=int(part.max()) + 1, replace=(int(part.max()) + 1 > K)).astype(np.int32)
        mats = part_mat[part]
        perm = morton_order(pts) if order == "morton" else rng.permutation(len(pts))
        pts, mats = pts[perm], mats[perm]
        pts = pts.astype(np.float32).astype(np.float64)     # what the consumers will see

        V = cfg["V"]
        if ragged_views:
            V = int(rng.integers(2, cfg["V"] + 1))
        cam = cameras_on_arc(V, cfg["radius"], f, HW) if cfg.get("arc") else cameras_on_sphere(V, cfg["radius"], f, HW)
        cam = cam.astype(np.float32).astype(np.float64)
        radius = 0.5 * float(np.linalg.norm(pts.max(0) - pts.min(0)))
        # depth tolerance: 1e-3 of the scene radius, plus the depth a surface tilted by 45 degrees
        # gains across the splat footprint (1.5 pixels per footprint ring) where a footprint is used
        tau = 1e-3 * radius + 1.5 * cfg["footprint"] * cfg["radius"] / f
        for v in range(V):
            d64 = splat_depth(cam[v], pts, HW, HW, cfg["footprint"])
            cell_mat = _cell_materials(cam[v], pts, mats, d64, tau, HW, HW, Gf, Gf, K)
            depths.append(d64.astype(np.float32))
            feats.append(store(_feature_map(rng, cell_mat, proto, cfg["sigma"], cfg.get("smooth", False)), cfg["dtype"]))
        cams.append(cam.astype(np.float32))
        xyz_all.append(pts.astype(np.float32))
        mat_all.append(mats)
        pt_off.append(pt_off[-1] + len(pts))
        view_off.append(view_off[-1] + V)
        taus.append(tau)
        if G > 0:
            lo_b, h_b = _grid_for(pts, G)
            glo.append(lo_b)
            gh.append(h_b)

    return Scene(
        name=name,
        xyz=np.concatenate(xyz_all), pt_offsets=np.array(pt_off, np.int64), view_offsets=np.array(view_off, np.int32),
        cam=np.concatenate(cams), depth=np.stack(depths), feat=np.stack(feats), feat_dtype=cfg["dtype"],
        temb=proto, y=y, tau=float(np.float32(np.mean(taus))), G=G,
        grid_lo=np.array(glo, np.float32) if G > 0 else None, grid_h=np.array(gh, np.float32) if G > 0 else None,
        vol_uniform=vol_uniform, material_of_point=np.concatenate(mat_all),
        meta=dict(seed=seed, order=order, preset=name, ragged_views=ragged_views),
    )
