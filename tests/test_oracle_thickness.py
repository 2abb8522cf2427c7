"""Pins for the oracle's thickness-based integration and centre of mass (Sec. 3.4.2).

Expectations: hand-worked cases (tests/golden/thickness_cases.txt), a numpy / scipy evaluation of the definition
built from library routines, closed forms (a plate of known volume, two point masses) and invariants.  None
comes from the oracle or from the GPU library.
"""
import os

import numpy as np
import pytest
from scipy.special import softmax

GOLD = os.path.join(os.path.dirname(__file__), "golden", "thickness_cases.txt")


def _vecs(text):
    return np.array([[float(x) for x in part.split()] for part in text.split(";")], np.float64)


def _opt(text):
    return None if text.strip() == "-" else _vecs(text)[0]


def test_hand_worked_cases(orc):
    rows = [l for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 7
    for line in rows:
        name, par, pts, om, y, th, cnt, blen, total, com, b = [c.strip() for c in line.split("|")]
        T, lam, scale = [float(x) for x in par.split()]
        cnt = _opt(cnt)
        r = orc.thickness_integrate(_vecs(om), _vecs(y)[0], _vecs(th)[0], _vecs(pts),
                                    count=None if cnt is None else cnt.astype(np.int32), box_len=_opt(blen), T=T, lam=lam,
                                    scale_factor=scale)
        assert np.allclose(r["mass"], float(total), rtol=1e-12, atol=1e-12), (name, r["mass"])
        assert np.allclose(r["com"][0], _vecs(com)[0], rtol=1e-12, atol=1e-12), (name, r["com"])
        assert np.allclose(r["b_adap"], float(b), rtol=1e-12, atol=1e-12), (name, r["b_adap"])
        assert r["n_used"][0] == (len(_vecs(pts)) if cnt is None else int((cnt > 0).sum())), name


def _scene(rng, sizes, K):
    N = int(sum(sizes))
    po = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    xyz = (rng.normal(size=(N, 3)) * rng.uniform(0.2, 2.0, size=3)).astype(np.float32)
    omega = rng.uniform(-0.3, 0.4, size=(N, K))
    y = rng.uniform(100, 8000, K).astype(np.float32)
    theta = rng.uniform(0.001, 0.05, K).astype(np.float32)
    count = (rng.uniform(size=N) < 0.8).astype(np.int32) * rng.integers(1, 5, N).astype(np.int32)
    return po, xyz, omega, y, theta, count


def _numpy_reference(po, xyz, omega, y, theta, count, T, lam, scale):
    """The definition with library routines: scipy's softmax, numpy's ptp / matmul / sums."""
    out = []
    for b in range(len(po) - 1):
        s = slice(po[b], po[b + 1])
        x = xyz[s].astype(np.float64)
        L = np.ptp(x, axis=0).max()
        area = (L * scale) ** 2 / len(x)
        zeta = softmax(omega[s] / T, axis=1) @ (y.astype(np.float64) * theta.astype(np.float64)) * area * lam
        zeta = zeta * (count[s] > 0)
        out.append((zeta, zeta.sum(), zeta @ x / zeta.sum() if zeta.sum() > 0 else np.zeros(3), np.sqrt(area)))
    return out


@pytest.mark.parametrize("seed,K", [(1, 1), (2, 7), (3, 32)])
def test_against_library_routines(orc, seed, K):
    rng = np.random.default_rng(seed)
    po, xyz, omega, y, theta, count = _scene(rng, [57, 1, 300, 12], K)
    T, lam, scale = 0.1, np.float32(0.6), np.float32(1.25)
    r = orc.thickness_integrate(omega, y, theta, xyz, count=count, pt_offsets=po, T=T, lam=lam, scale_factor=scale)
    ref = _numpy_reference(po, xyz, omega, y, theta, count, np.float64(np.float32(T)), float(lam), float(scale))
    for b, (zeta, total, com, b_adap) in enumerate(ref):
        assert np.allclose(r["zeta"][po[b]:po[b + 1]], zeta, rtol=1e-12, atol=0)
        assert np.isclose(r["mass"][b], total, rtol=1e-12)
        assert np.isclose(r["b_adap"][b], b_adap, rtol=1e-13)
        if total > 0:
            assert np.allclose(r["com"][b], com, rtol=1e-11, atol=1e-13)
        assert r["n_used"][b] == (count[po[b]:po[b + 1]] > 0).sum()


def test_plate_of_known_volume(orc):
    """A flat L x L sheet sampled on any regular grid: the sum is density * (L^2 * theta) * lambda, whatever
    the number of samples; the centre of mass is the centre of the sheet."""
    L, rho, theta, lam = 0.75, 2700.0, 0.0078125, 0.5
    for n in (2, 5, 32):
        g = np.linspace(0.0, L, n)
        xyz = np.stack([*np.meshgrid(g, g, indexing="ij"), np.full((n, n), 3.0)], -1).reshape(-1, 3) + [1.0, -2.0, 0.0]
        r = orc.thickness_integrate(np.zeros((n * n, 1)), [rho], [theta], xyz, lam=lam)
        assert np.isclose(r["mass"][0], rho * L * L * theta * lam, rtol=1e-6)     # fp32 coordinates carry L
        assert np.allclose(r["com"][0], [1.0 + L / 2, -2.0 + L / 2, 3.0], rtol=1e-6)


def test_matches_eq4_when_all_thicknesses_are_one(orc):
    """With theta_k = 1 the bracket of the integration formula is the kernel regression of Eq. 4."""
    rng = np.random.default_rng(11)
    N, D, K = 256, 24, 6      # sqrt(N) is exact in fp32
    fused = rng.normal(size=(N, D))
    fused /= np.linalg.norm(fused, axis=1, keepdims=True)
    temb = rng.normal(size=(K, D)).astype(np.float32)
    temb /= np.linalg.norm(temb, axis=1, keepdims=True)
    y = rng.uniform(100, 8000, (K, 2)).astype(np.float32)
    xyz = rng.normal(size=(N, 3)).astype(np.float32)
    sc = orc.material_scores(fused, temb, y, T=0.1)
    r = orc.thickness_integrate(sc["scores"], y[:, 0], np.ones(K), xyz, T=0.1, lam=1.0, box_len=[np.sqrt(N)])
    assert np.allclose(r["zeta"], sc["prop"][:, 0], rtol=1e-12)       # A_bar = 1
    assert np.isclose(r["mass"][0], sc["prop"][:, 0].sum(), rtol=1e-12)


def test_sharp_temperature_picks_the_best_material(orc):
    rng = np.random.default_rng(5)
    N, K = 64, 9
    omega = rng.uniform(-1, 1, (N, K))
    best = omega.argmax(1)
    omega[np.arange(N), best] += 0.5          # a clear winner: the others weigh exp(-5000) or less
    y, theta = rng.uniform(1, 9, K).astype(np.float32), rng.uniform(0.5, 2, K).astype(np.float32)
    xyz = rng.normal(size=(N, 3)).astype(np.float32)
    r = orc.thickness_integrate(omega, y, theta, xyz, T=1e-4, lam=1.0, box_len=[np.sqrt(N)])
    assert np.allclose(r["zeta"], y[best].astype(np.float64) * theta[best], rtol=1e-9)


def test_invariants(orc):
    rng = np.random.default_rng(7)
    po, xyz, omega, y, theta, count = _scene(rng, [40, 90], 5)
    base = orc.thickness_integrate(omega, y, theta, xyz, count=count, pt_offsets=po, lam=0.5, scale_factor=1.0)
    # scale_factor enters squared, lambda linearly; neither moves the centre of mass
    r = orc.thickness_integrate(omega, y, theta, xyz, count=count, pt_offsets=po, lam=0.25, scale_factor=4.0)
    assert np.allclose(r["mass"], base["mass"] * 8.0, rtol=1e-12)
    assert np.allclose(r["com"], base["com"], rtol=1e-12)
    assert np.allclose(r["b_adap"], base["b_adap"] * 4.0, rtol=1e-12)
    # a shift of every score of a point changes nothing (softmax)
    r = orc.thickness_integrate(omega + rng.uniform(-1, 1, (len(omega), 1)), y, theta, xyz, count=count, pt_offsets=po,
                                lam=0.5)
    assert np.allclose(r["zeta"], base["zeta"], rtol=1e-9)
    # a translation (by amounts exact in fp32) moves the centre of mass and nothing else
    shift = np.array([8.0, -16.0, 4.0])
    r = orc.thickness_integrate(omega, y, theta, (xyz.astype(np.float64) * 0.0 + np.round(xyz * 64) / 64 + shift), count=count,
                                pt_offsets=po, lam=0.5)
    r0 = orc.thickness_integrate(omega, y, theta, np.round(xyz * 64) / 64, count=count, pt_offsets=po, lam=0.5)
    assert np.allclose(r["mass"], r0["mass"], rtol=1e-12)
    assert np.allclose(r["com"], r0["com"] + shift, rtol=1e-12)
    # the order of the points inside an object does not matter
    perm = np.concatenate([rng.permutation(40), 40 + rng.permutation(90)])
    r = orc.thickness_integrate(omega[perm], y, theta, xyz[perm], count=count[perm], pt_offsets=po, lam=0.5)
    assert np.allclose(r["mass"], base["mass"], rtol=1e-12)
    assert np.allclose(r["com"], base["com"], rtol=1e-11)
    assert np.allclose(r["zeta"], base["zeta"][perm], rtol=1e-12)
    # material order does not matter either
    pk = rng.permutation(5)
    r = orc.thickness_integrate(omega[:, pk], y[pk], theta[pk], xyz, count=count, pt_offsets=po, lam=0.5)
    assert np.allclose(r["zeta"], base["zeta"], rtol=1e-12)


def test_degenerate_inputs(orc):
    # an object without points, an object whose points are all unseen
    po = np.array([0, 0, 3], np.int64)
    xyz = np.array([[0, 0, 0], [1, 0, 0], [0, 2, 0]], np.float32)
    r = orc.thickness_integrate(np.zeros((3, 2)), [1, 2], [1, 1], xyz, count=np.zeros(3, np.int32), pt_offsets=po)
    assert (r["mass"] == 0).all() and (r["com"] == 0).all() and (r["n_used"] == 0).all()
    assert r["b_adap"][0] == 0 and np.isclose(r["b_adap"][1], np.sqrt(4.0 / 3.0))
    # large scores do not overflow
    r = orc.thickness_integrate(np.array([[80.0, 79.0]]), [1, 2], [1, 1], [[0, 0, 0]], box_len=[1.0], lam=1.0)
    assert np.isfinite(r["mass"]).all() and np.isclose(r["mass"][0], 1.0, rtol=1e-4)
