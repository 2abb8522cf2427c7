"""CPU-only checks of the C ABI: the shared library loads, exports every function the header
declares, and rejects bad arguments with the documented status before touching the GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "aura_fuse.h")


@pytest.fixture(scope="module")
def B():
    from paper_2511_03126_amd import binding
    if not binding._LIB_PATH.exists():
        from paper_2511_03126_amd.build import build
        build()
    binding.lib()
    return binding


def _declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(aura_[a-z_]+)\s*\(", text)))


def test_every_declared_function_is_exported(B):
    names = _declared_functions()
    assert {"aura_project_visibility", "aura_fuse_features", "aura_material_scores", "aura_property_integrate",
            "aura_workspace_bytes", "aura_version", "aura_strerror", "aura_last_hip_error",
            "aura_calibration_copy", "aura_calibration_fill", "aura_fuse_scores", "aura_knn_densify"} <= set(names)
    for n in names:
        assert hasattr(B.lib(), n), n


def test_version_and_error_strings(B):
    assert B.lib().aura_version() >= 100
    for code in range(0, -8, -1):
        assert len(B.lib().aura_strerror(code)) > 1
    assert B.lib().aura_last_hip_error() == 0


def test_workspace_sizes(B):
    # split embeddings (4096 bytes per 32 channels and 32 materials), then room for an fp32 copy of 16-bit embeddings
    copy = lambda D, K: -(-4 * D * K // 256) * 256
    assert B.workspace_bytes(B.CALL_MATERIAL_SCORES, D=768, K=32) == 24 * 1 * 4096 + copy(768, 32)
    assert B.workspace_bytes(B.CALL_MATERIAL_SCORES, D=1024, K=128) == 32 * 4 * 4096 + copy(1024, 128)
    assert B.workspace_bytes(B.CALL_MATERIAL_SCORES, D=33, K=65) == 2 * 4 * 4096 + copy(33, 65)     # 3 tiles round up to 4
    small = B.workspace_bytes(B.CALL_PROPERTY_INTEGRATE, N=1000, B=1, G=0)
    grid = B.workspace_bytes(B.CALL_PROPERTY_INTEGRATE, N=1000, B=2, G=64)
    assert 0 < small < 4096 and grid >= 2 * 64 ** 3 * 12
    with pytest.raises(B.AuraError) as e:
        B.workspace_bytes(B.CALL_MATERIAL_SCORES, D=64, K=129)
    assert e.value.status == -7
    with pytest.raises(B.AuraError) as e:
        B.workspace_bytes(99)
    assert e.value.status == -7
    with pytest.raises(B.AuraError) as e:
        B.workspace_bytes(B.CALL_PROPERTY_INTEGRATE, N=-1)
    assert e.value.status == -2
    # fusion: only 16-bit maps with D a multiple of 256 use the matrix-core path and need scratch
    fuse = lambda **kw: B.workspace_bytes(B.CALL_FUSE_FEATURES, **{**dict(N=200_000, B=1, n_views=16, Hf=32, Wf=32), **kw})
    assert fuse(D=512, feat_dtype=B.F32) == 0
    assert fuse(D=100, feat_dtype=B.BF16) == 0
    assert fuse(D=1280, feat_dtype=B.F16) == 0
    tiles = 200_000 // 32 + 1
    # tile headers, ticket counters, the status word, then the tiles' k-steps
    assert fuse(D=768, feat_dtype=B.BF16) == -(-tiles * 144 // 256) * 256 + 256 + 256 + tiles * 32 * 2112
    assert fuse(D=768, feat_dtype=B.BF16, n_views=4) == -(-tiles * 144 // 256) * 256 + 256 + 256 + tiles * 8 * 2112
    # where the status word of these calls lies (right behind the counters), and which sizes have none
    off, present = C.c_size_t(99), C.c_int32(9)
    sz = B._SizesT(200_000, 1, 16, 32, 32, 768, B.BF16, 33, 0, 1, 1)
    for call in (B.CALL_FUSE_FEATURES, B.CALL_FUSE_SCORES, B.CALL_FUSE_SCORE_INTEGRATE):
        assert B.lib().aura_fuse_status_offset(call, C.byref(sz), C.byref(off), C.byref(present)) == 0
        assert present.value == 1 and off.value == -(-tiles * 144 // 256) * 256 + 256
    sz32 = B._SizesT(200_000, 1, 16, 32, 32, 768, B.F32, 33, 0, 1, 1)
    assert B.lib().aura_fuse_status_offset(B.CALL_FUSE_FEATURES, C.byref(sz32), C.byref(off), C.byref(present)) == 0
    assert present.value == 0
    assert B.lib().aura_fuse_status_offset(B.CALL_KNN_DENSIFY, C.byref(sz), C.byref(off), C.byref(present)) == -7
    assert B.lib().aura_fuse_status_offset(B.CALL_FUSE_FEATURES, None, C.byref(off), C.byref(present)) == -1
    with pytest.raises(B.AuraError) as e:
        fuse(D=768, feat_dtype=9)
    assert e.value.status == -3
    assert B.lib().aura_workspace_bytes(B.CALL_FUSE_FEATURES, None, C.byref(C.c_size_t())) == -1
    # fusion + scoring in one call: fusion scratch, then (fewer cells than points, matrix-core fusion) one
    # factor per point and one packed similarity per cell and padded material, then the scoring scratch
    both = lambda **kw: B.workspace_bytes(B.CALL_FUSE_SCORES, **{**dict(N=200_000, B=1, n_views=16, Hf=32, Wf=32, K=33), **kw})
    r256 = lambda x: -(-x // 256) * 256
    sc = lambda D, K: B.workspace_bytes(B.CALL_MATERIAL_SCORES, D=D, K=K)
    assert both(D=512, feat_dtype=B.F32) == r256(sc(512, 33))
    assert both(D=768, feat_dtype=B.BF16) == (r256(fuse(D=768, feat_dtype=B.BF16)) + r256(200_000 * 4)
                                              + r256(16 * 32 * 32 * 64 * 4) + 96 * 2 * 2048    # + the split embeddings
                                              + r256(sc(768, 33)))
    assert both(D=768, feat_dtype=B.BF16, N=1000) == r256(fuse(D=768, feat_dtype=B.BF16, N=1000)) + r256(sc(768, 33))
    with pytest.raises(B.AuraError) as e:
        both(D=768, feat_dtype=B.BF16, K=129)
    assert e.value.status == -7


def _views(B, **kw):
    fake = 0x1000      # never dereferenced: validation fails first
    v = B._ViewsT(4, 32, 32, 4, 4, 64, B.F32, fake, fake, fake)
    for k, val in kw.items():
        setattr(v, k, val)
    return v


def test_argument_validation_returns_status_codes(B):
    L = B.lib()
    p = B.Params().c()
    fake = C.c_void_p(0x1000)
    po = np.array([0, 5, 10], np.int64)
    vo = np.array([0, 2, 4], np.int32)
    hp = lambda a: a.ctypes.data_as(C.c_void_p)
    pv = lambda v, N=10, po_=None, vo_=None, B_=1, pitch=4, xyz=fake, vis=fake: L.aura_project_visibility(
        C.byref(v), C.byref(p), xyz, N, po_, vo_, B_, vis, pitch, None, None, None)
    assert pv(_views(B), xyz=None) == -1
    assert pv(_views(B), vis=None) == -1
    assert pv(_views(B, cam=None)) == -1
    assert pv(_views(B, depth=None)) == -1
    assert pv(_views(B, n_views=0)) == -2
    assert pv(_views(B), N=-1) == -2
    assert pv(_views(B), pitch=3) == -2                                    # fewer columns than views
    assert pv(_views(B), po_=hp(po), vo_=None, B_=2) == -1                 # only one of the offset arrays
    assert pv(_views(B), po_=None, vo_=None, B_=2) == -1
    assert pv(_views(B), po_=hp(po), vo_=hp(vo), B_=2, N=11) == -2         # offsets do not end at N
    bad = np.array([0, 7, 5], np.int64)
    assert pv(_views(B), po_=hp(bad), vo_=hp(vo), B_=2, N=5) == -2         # not monotone
    assert pv(_views(B), N=0, xyz=None, vis=None) == 0                     # empty input is fine

    ff = lambda v, fused=fake, ws=None, wsb=0: L.aura_fuse_features(C.byref(v), C.byref(p), fake, 10, None, None, 1,
                                                                  fused, None, ws, wsb, None)
    assert ff(_views(B, feat=None)) == -1
    assert ff(_views(B, feat_dtype=7)) == -3
    assert ff(_views(B, feat=0x1004)) == -4
    assert ff(_views(B), fused=C.c_void_p(0x1004)) == -4
    assert ff(_views(B, D=0)) == -2
    assert ff(_views(B), fused=None) == -1
    half = dict(feat_dtype=B.BF16, D=256)                                  # a shape the matrix-core path takes
    assert ff(_views(B, **half), ws=C.c_void_p(0x1010), wsb=1 << 30) == -5 # workspace not 256-byte aligned
    assert ff(_views(B, **half), ws=C.c_void_p(0x1000), wsb=64) == -5      # workspace too small

    ms = lambda N=10, D=64, K=8, P=1, temb=fake, dt=B.F32, y=fake, prop=fake, ws=C.c_void_p(0x1000), wsb=1 << 20, par=p: \
        L.aura_material_scores(fake, N, D, temb, dt, K, y, P, C.byref(par) if par is not None else None, fake, prop,
                               None, ws, wsb, None)
    assert ms(temb=None) == -1
    assert ms(par=None) == -1
    assert ms(D=0) == -2
    assert ms(K=129) == -7
    assert ms(P=9) == -7
    assert ms(dt=5) == -3
    assert ms(y=None) == -1                                                # prop wanted but no y
    assert ms(ws=None) == -5
    assert ms(wsb=16) == -5
    assert ms(ws=C.c_void_p(0x1010)) == -5
    cold = B.Params(temperature=0.0).c()
    assert ms(par=cold) == -2

    fs = lambda v=None, N=10, K=8, P=1, temb=fake, dt=B.F32, y=fake, fused=fake, scores=fake, prop=fake, vis=None, pitch=0, \
        ws=C.c_void_p(0x1000), wsb=1 << 30, par=p: L.aura_fuse_scores(
            C.byref(v if v is not None else _views(B)), C.byref(par), fake, N, None, None, 1, temb, dt, K, y, P, fused, None,
            vis, pitch, scores, prop, None, ws, wsb, None)
    assert fs(temb=None) == -1
    assert fs(fused=None) == -1
    assert fs(scores=None) == -1
    assert fs(y=None) == -1                                                # prop wanted but no y
    assert fs(v=_views(B, feat=None)) == -1
    assert fs(v=_views(B, feat_dtype=7)) == -3
    assert fs(dt=5) == -3
    assert fs(K=0) == -2
    assert fs(K=129) == -7
    assert fs(P=9) == -7
    assert fs(par=cold) == -2
    assert fs(fused=C.c_void_p(0x1004)) == -4
    assert fs(ws=None) == -5
    assert fs(wsb=16) == -5
    assert fs(ws=C.c_void_p(0x1010)) == -5
    assert fs(N=0, fused=None, scores=None) == 0
    assert fs(vis=fake, pitch=3) == -2                                     # fewer mask columns than views

    kd = lambda Nq=10, D=64, Ns=20, K=8, k=3, P=1, fq=fake, fs=fake, ws_=fake, y=fake, wq=fake, prop=fake, \
        ws=C.c_void_p(0x1000), wsb=1 << 24, par=p: L.aura_knn_densify(fq, Nq, D, fs, Ns, ws_, K, k, y, P, C.byref(par), wq, prop,
                                                                    None, None, ws, wsb, None)
    assert kd(fs=None) == -1
    assert kd(ws_=None) == -1
    assert kd(fq=None) == -1
    assert kd(wq=None) == -1
    assert kd(y=None) == -1
    assert kd(D=0) == -2
    assert kd(Ns=0) == -2
    assert kd(k=0) == -2
    assert kd(par=cold) == -2
    assert kd(Ns=257) == -7
    assert kd(k=17) == -7
    assert kd(K=129) == -7
    assert kd(P=9) == -7
    assert kd(ws=None) == -5
    assert kd(wsb=16) == -5
    assert kd(ws=C.c_void_p(0x1010)) == -5
    assert kd(Nq=0, fq=None, wq=None) == 0
    assert B.workspace_bytes(B.CALL_KNN_DENSIFY, D=768, Ns=150) == 24 * 5 * 2 * 2 * 64 * 16 + 768   # 5 tiles of 32 sources
    with pytest.raises(B.AuraError) as e:
        B.workspace_bytes(B.CALL_KNN_DENSIFY, D=768, Ns=300)
    assert e.value.status == -7

    sv = lambda v=None, N=10, k=3, xyz=fake, nrm=fake, sel=fake, mask=None, pitch=0, po_=None, vo_=None, B_=1: \
        L.aura_select_views(C.byref(v if v is not None else _views(B)), C.byref(p), xyz, nrm, N, po_, vo_, B_, k, sel, None,
                            mask, pitch, None, None)
    assert sv(xyz=None) == -1 and sv(nrm=None) == -1 and sv(sel=None) == -1
    assert sv(v=_views(B, cam=None)) == -1
    assert sv(v=_views(B, depth=None)) == -1                               # the depth test needs depth maps
    assert sv(k=0) == -2
    assert sv(k=9) == -7
    assert sv(N=-1) == -2
    assert sv(mask=fake, pitch=3) == -2                                    # fewer mask columns than views
    assert sv(po_=hp(po), vo_=None, B_=2) == -1
    assert sv(N=0, xyz=None, nrm=None, sel=None) == 0

    fsel = lambda v=None, N=10, xyz=fake, mask=fake, pitch=4, fused=fake, ws=None, wsb=0: L.aura_fuse_selected(
        C.byref(v if v is not None else _views(B)), C.byref(p), xyz, N, None, None, 1, mask, pitch, fused, None, ws, wsb, None)
    assert fsel(mask=None) == -1
    assert fsel(xyz=None) == -1 and fsel(fused=None) == -1
    assert fsel(pitch=3) == -2
    assert fsel(v=_views(B, feat=None)) == -1
    assert fsel(v=_views(B, feat_dtype=7)) == -3
    assert fsel(fused=C.c_void_p(0x1004)) == -4
    assert fsel(v=_views(B, **half), ws=C.c_void_p(0x1000), wsb=64) == -5
    assert fsel(N=0, xyz=None, mask=None, fused=None) == 0

    box = lambda lo, hi: (hp(np.array(lo, np.float32)), hp(np.array(hi, np.float32)))
    keep = [np.array([0, 0, 0], np.float32), np.array([2, 2, 2], np.float32), np.array([2, 2, 1], np.float32)]
    s_out, dims = C.c_float(0), np.zeros(3, np.int32)
    assert L.aura_voxel_grid(hp(keep[0]), hp(keep[1]), 8, C.byref(s_out), hp(dims)) == 0
    assert s_out.value == 1.0 and list(dims) == [3, 3, 3]
    assert L.aura_voxel_grid(None, hp(keep[1]), 8, C.byref(s_out), hp(dims)) == -1
    assert L.aura_voxel_grid(hp(keep[1]), hp(keep[2]), 8, C.byref(s_out), hp(dims)) == -2   # upper corner below lower
    assert L.aura_voxel_grid(hp(keep[0]), hp(keep[1]), 0, C.byref(s_out), hp(dims)) == -2
    big = np.array([1e4, 1e4, 1e-20], np.float32)
    assert L.aura_voxel_grid(hp(keep[0]), hp(big), 150, C.byref(s_out), hp(dims)) == -7        # too many voxels
    nb = C.c_size_t(0)
    assert L.aura_voxel_workspace_bytes(hp(keep[0]), hp(keep[1]), 1, 8, C.byref(nb)) == 0
    assert nb.value == 2048 * 32 + 2048 * 4 + 256 + 256
    assert L.aura_voxel_workspace_bytes(hp(keep[0]), hp(keep[1]), 65, 8, C.byref(nb)) == -7    # more than 64 objects
    vd = lambda N=10, xyz=fake, lo=keep[0], hi=keep[1], nt=8, out=fake, cap=10, offs=fake, po_=None, B_=1, \
        ws=C.c_void_p(0x1000), wsb=1 << 20: L.aura_voxel_downsample(xyz, N, po_, B_, hp(lo), hp(hi), nt, out, None, cap, offs,
                                                                  None, ws, wsb, None)
    assert vd(xyz=None) == -1 and vd(out=None) == -1 and vd(offs=None) == -1
    assert vd(N=-1) == -2 and vd(nt=0) == -2 and vd(cap=-1) == -2
    assert vd(lo=keep[1], hi=keep[2]) == -2
    assert vd(B_=2) == -1
    assert vd(ws=None) == -5 and vd(wsb=16) == -5 and vd(ws=C.c_void_p(0x1010)) == -5

    ctr = np.zeros((2, 3), np.float32)
    qo2 = np.array([0, 1, 3], np.int64)
    en = lambda xyz=fake, N=10, po_=None, q=fake, M=3, qo_=None, B_=1, c=ctr, k=8, nrm=fake: L.aura_estimate_normals(
        xyz, N, po_, q, M, qo_, B_, None if c is None else hp(c), k, nrm, None, None)
    assert en(xyz=None) == -1 and en(q=None) == -1 and en(nrm=None) == -1 and en(c=None) == -1
    assert en(k=0) == -2 and en(N=-1) == -2 and en(M=-1) == -2
    assert en(B_=2) == -1                                                  # two objects need both offset arrays
    assert en(po_=hp(po), B_=2) == -1
    assert en(po_=hp(po), qo_=hp(qo2), B_=2, N=11) == -2
    assert en(po_=hp(po), qo_=hp(qo2), B_=2, M=4) == -2
    assert en(c=np.full((1, 3), np.nan, np.float32)) == -2
    assert en(M=0, q=None, nrm=None) == 0

    sc3 = np.array([20, 40, 60], np.float32)
    pb = lambda cam=fake, V=4, H=32, W=32, img=fake, xyz=fake, M=10, sel=fake, k=3, sc=sc3, L=3, R=16, out=fake, dt=B.F32: \
        L_.aura_patch_batch(cam, V, H, W, img, xyz, M, None, None, 1, sel, k, None if sc is None else hp(sc), L, R, None, None,
                            out, dt, None, None)
    L_ = L
    assert pb(cam=None) == -1 and pb(img=None) == -1 and pb(xyz=None) == -1 and pb(sel=None) == -1 and pb(out=None) == -1
    assert pb(sc=None) == -1
    assert pb(V=0) == -2 and pb(k=0) == -2 and pb(L=0) == -2 and pb(R=0) == -2 and pb(M=-1) == -2
    assert pb(sc=np.array([20, 0, 60], np.float32)) == -2
    assert pb(L=9, sc=np.ones(9, np.float32)) == -7
    assert pb(dt=B.BF16) == -7 and pb(dt=9) == -3
    assert pb(out=C.c_void_p(0x1002)) == -4
    assert pb(M=0, xyz=None, sel=None, out=None) == 0

    ti = lambda N=10, K=8, P=2, pi=0, scores=fake, y=fake, theta=fake, xyz=fake, po_=None, B_=1, blen=None, par=p, lam=0.6, \
        scale=1.0, total=fake, ws=C.c_void_p(0x1000), wsb=1 << 20: L.aura_thickness_integrate(
            scores, N, K, y, P, pi, theta, xyz, None, po_, B_, blen, C.byref(par) if par is not None else None, lam, scale,
            None, total, None, None, None, ws, wsb, None)
    assert ti(scores=None) == -1 and ti(y=None) == -1 and ti(theta=None) == -1 and ti(xyz=None) == -1
    assert ti(total=None) == -1
    assert ti(par=None) == -1
    assert ti(K=0) == -2
    assert ti(pi=2) == -2                                                  # property column outside y
    assert ti(N=-1) == -2
    assert ti(par=cold) == -2
    assert ti(scale=-1.0) == -2
    assert ti(K=129) == -7
    assert ti(B_=2) == -1                                                  # two objects need offsets
    assert ti(po_=hp(po), B_=2, N=11) == -2
    assert ti(po_=hp(bad), B_=2, N=5) == -2
    assert ti(blen=hp(np.array([-1.0], np.float32))) == -2                 # a given length must not be negative
    assert ti(ws=None) == -5
    assert ti(wsb=16) == -5
    assert ti(ws=C.c_void_p(0x1010)) == -5
    r256 = lambda x: -(-x // 256) * 256
    slices = -(-200_000 // 256) + 3
    assert B.workspace_bytes(B.CALL_THICKNESS_INTEGRATE, N=200_000, B=3) == (r256(slices * 24) + r256(slices * 32)
                                                                             + r256(slices * 8) + 256)
    with pytest.raises(B.AuraError) as e:
        B.workspace_bytes(B.CALL_THICKNESS_INTEGRATE, N=10, B=5000)
    assert e.value.status == -7

    cc = lambda dst=fake, src=fake, n=1024: L.aura_calibration_copy(dst, src, n, None)
    assert cc(dst=None) == -1 and cc(src=None) == -1
    assert cc(n=1000) == -2                                                # not a multiple of 16 bytes
    assert cc(dst=C.c_void_p(0x1004)) == -4
    assert cc(n=0, dst=None, src=None) == 0
    cf = lambda dst=fake, n=1024: L.aura_calibration_fill(dst, n, 7, None)
    assert cf(dst=None) == -1 and cf(n=24) == -2 and cf(dst=C.c_void_p(0x1008)) == -4 and cf(n=0, dst=None) == 0

    pi = lambda N=10, P=1, pidx=0, B_=1, G=0, mass=fake, ws=C.c_void_p(0x1000), wsb=1 << 30, po_=None, glo=None, gh=None, xyz=None: \
        L.aura_property_integrate(fake, N, P, pidx, None, None, 1.0, po_, B_, xyz, glo, gh, G, mass, None, ws, wsb, None)
    assert pi(mass=None) == -1
    assert pi(pidx=1) == -2
    assert pi(B_=2) == -1
    assert pi(G=8) == -1                                                   # grid mode without a grid
    assert pi(G=600, glo=fake, gh=fake) == -7
    assert pi(ws=None) == -5
    assert pi(wsb=8) == -5
    glo = np.zeros((1, 3), np.float32)
    gh = np.zeros(1, np.float32)
    assert pi(G=8, glo=hp(glo), gh=hp(gh), xyz=fake) == -2                 # voxel size must be positive
    assert pi(po_=hp(np.array([0, 4], np.int64))) == -2                    # offsets do not end at N


def test_single_pass_call_validation_and_workspace(B):
    """aura_fuse_score_integrate: the checks of aura_fuse_scores and aura_property_integrate, no fused argument at all."""
    L = B.lib()
    p = B.Params().c()
    cold = B.Params(temperature=0.0).c()
    fake = C.c_void_p(0x1000)
    hp = lambda a: a.ctypes.data_as(C.c_void_p)
    fsi = lambda v=None, N=10, K=8, P=1, pidx=0, temb=fake, dt=B.F32, y=fake, scores=fake, mass=fake, vis=None, pitch=0, G=0, \
        glo=None, gh=None, xyz=fake, ws=C.c_void_p(0x1000), wsb=1 << 30, par=p, po_=None, vo_=None, B_=1: \
        L.aura_fuse_score_integrate(C.byref(v if v is not None else _views(B)), C.byref(par), xyz, N, po_, vo_, B_, temb, dt, K,
                                    y, P, pidx, None, 1.0, glo, gh, G, None, vis, pitch, scores, None, None, mass, None, ws,
                                    wsb, None)
    assert fsi(temb=None) == -1 and fsi(y=None) == -1 and fsi(mass=None) == -1
    assert fsi(xyz=None) == -1 and fsi(scores=None) == -1
    assert fsi(v=_views(B, feat=None)) == -1
    assert fsi(v=_views(B, feat_dtype=7)) == -3
    assert fsi(dt=5) == -3
    assert fsi(K=0) == -2 and fsi(K=129) == -7 and fsi(P=9) == -7
    assert fsi(P=0) == -2                                                  # the integration needs a property column
    assert fsi(pidx=1) == -2
    assert fsi(par=cold) == -2
    assert fsi(vis=fake, pitch=3) == -2
    assert fsi(G=8) == -1                                                  # grid mode without a grid
    assert fsi(G=600, glo=fake, gh=fake) == -7
    assert fsi(G=8, glo=hp(np.zeros((1, 3), np.float32)), gh=hp(np.zeros(1, np.float32))) == -2   # voxel size must be positive
    assert fsi(B_=2) == -1                                                 # two objects need offsets
    assert fsi(ws=None) == -5 and fsi(wsb=16) == -5 and fsi(ws=C.c_void_p(0x1010)) == -5
    # workspace: that of aura_fuse_scores (per-cell scores up to four times as many cells as points), view counts,
    # properties, the integration's scratch and one chunk of fused rows
    r256 = lambda x: -(-x // 256) * 256
    kw = dict(N=200_000, B=1, n_views=16, Hf=32, Wf=32, D=768, feat_dtype=B.BF16, K=33)
    both = B.workspace_bytes(B.CALL_FUSE_SCORES, **kw)
    mass = B.workspace_bytes(B.CALL_PROPERTY_INTEGRATE, N=200_000, B=1, G=128)
    assert B.workspace_bytes(B.CALL_FUSE_SCORE_INTEGRATE, P=2, G=128, **kw) == (
        both + r256(200_000 * 4) + r256(200_000 * 2 * 4) + r256(mass) + r256(32768 * 768 * 4))
    few = dict(kw, N=5000)       # 16384 cells, 5000 points: per-cell scores here, not in aura_fuse_scores
    assert B.workspace_bytes(B.CALL_FUSE_SCORE_INTEGRATE, P=1, **few) > B.workspace_bytes(B.CALL_FUSE_SCORES, **few) + \
        16 * 32 * 32 * 64 * 4
    with pytest.raises(B.AuraError) as e:
        B.workspace_bytes(B.CALL_FUSE_SCORE_INTEGRATE, P=0, **kw)
    assert e.value.status == -2
    with pytest.raises(B.AuraError) as e:
        B.workspace_bytes(B.CALL_FUSE_SCORE_INTEGRATE, P=9, **kw)
    assert e.value.status == -7


def test_timing_request_takes_both_events_or_none(B):
    L = B.lib()
    fake = C.c_void_p(0x1000)
    assert L.aura_time_next_fusion(fake, None) == -1
    assert L.aura_time_next_fusion(None, fake) == -1
    assert L.aura_time_next_fusion(fake, fake) == 0
    assert L.aura_time_next_fusion(None, None) == 0      # withdrawn again: nothing is ever recorded on the fake handles


def test_static_scratch_call_refuses_what_does_not_fit(B):
    binding = B
    L = binding.lib()
    p = binding.Params().c()
    fake = C.c_void_p(0x1000)
    call = lambda N=10, D=64, K=8, P=1, temb=fake, dt=binding.F32, y=fake, prop=fake, fused=fake, scores=fake: \
        L.aura_material_scores_static(fused, N, D, temb, dt, K, y, P, C.byref(p), scores, prop, None, None)
    # 128 channel steps x 4 material tiles x 4096 bytes of split embeddings + 2 MiB for an fp32 copy: beyond the 2 MiB array
    assert call(D=4096, K=128) == -7
    assert call(temb=None) == -1 and call(y=None) == -1
    assert call(K=129) == -7 and call(P=9) == -7 and call(D=0) == -2
    assert call(dt=5) == -3
    assert call(N=0, fused=None, scores=None) == 0       # (every call above is refused before anything is launched)
