"""GPU parity of aura_knn_densify (Sec. 3.4.1 Eq. 5) against the CPU oracle, element by element on the
same seeded inputs.  Bar: the selected neighbours identical wherever the oracle's margin between the k-th
neighbour and the best source left out exceeds the accuracy of the GPU's similarities (queries inside that
margin may pick either source: they must be rare, and their result must still be the Eq. 5 mean of a valid
neighbour set); interpolated vectors and properties within 1e-4 relative (fp32 inputs); labels equal away
from ties."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

TOL = 1e-4
SIM_TOL = 2e-5      # accuracy of a similarity computed with two-term bf16 operands


def _inputs(Nq, Ns, D, K, P, seed, spread=0.3):
    """Clustered, mostly positive features: parts of one object resemble each other, as for DINO features."""
    rng = np.random.default_rng(seed)
    fs = (np.abs(rng.standard_normal((Ns, D))) + 0.1).astype(np.float32)
    fq = (fs[rng.integers(0, Ns, Nq)] + spread * rng.standard_normal((Nq, D))).astype(np.float32)
    ws = rng.uniform(-0.2, 0.5, (Ns, K)).astype(np.float32)
    y = rng.uniform(100, 8000, (K, P)).astype(np.float32)
    return fq, fs, ws, y


def _run_gpu(fq, fs, ws, y, k, T=0.1, want_idx=True):
    import paper_2511_03126_amd as aura
    from paper_2511_03126_amd import binding
    dev = "cuda:0"
    Nq, D = fq.shape
    Ns, K = ws.shape
    P = y.shape[1]
    t = lambda a: torch.from_numpy(a).to(dev)
    wq = torch.full((Nq, K), float("nan"), device=dev)
    prop = torch.full((Nq, P), float("nan"), device=dev)
    label = torch.full((Nq,), -7, dtype=torch.int32, device=dev)
    nn_idx = torch.full((Nq, k), -7, dtype=torch.int32, device=dev) if want_idx else None
    ws_bytes = aura.workspace_bytes(binding.CALL_KNN_DENSIFY, D=D, Ns=Ns)
    work = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    aura.knn_densify(t(fq), t(fs), t(ws), k, t(y), aura.Params(temperature=T), wq, prop, label, nn_idx, work)
    torch.cuda.synchronize()
    return dict(wq=wq.cpu().numpy(), prop=prop.cpu().numpy(), label=label.cpu().numpy(),
                nn_idx=None if nn_idx is None else nn_idx.cpu().numpy())


def _compare(gpu, ref, ws, y, sel=None):
    g = {k: (v if sel is None or v is None else v[sel]) for k, v in gpu.items()}
    clear = ref["gap"] > SIM_TOL                       # the neighbour set is unambiguous
    assert clear.mean() > 0.98, f"too many near-ties at the k-th neighbour: {1 - clear.mean():.3f}"
    if g["nn_idx"] is not None:
        # same set everywhere it is unambiguous; same ORDER where consecutive similarities are also apart
        same_set = np.sort(g["nn_idx"], 1) == np.sort(ref["nn_idx"], 1)
        assert same_set[clear].all()
        d = -np.diff(ref["nn_sim"], axis=1)
        ordered = clear & ((d > SIM_TOL).all(1) if d.shape[1] else True)
        assert np.array_equal(g["nn_idx"][ordered], ref["nn_idx"][ordered])
    scale = np.abs(ws).max()
    err_w = np.abs(g["wq"][clear] - ref["wq"][clear]).max(initial=0.0) / scale
    assert err_w <= TOL, f"interpolated vector err {err_w}"
    err_p = (np.abs(g["prop"][clear] - ref["prop"][clear]) / np.abs(y).max(0)).max(initial=0.0)
    assert err_p <= TOL, f"prop err {err_p}"
    srt = np.sort(ref["wq"], 1)
    margin = srt[:, -1] - srt[:, -2] if srt.shape[1] > 1 else np.full(len(srt), np.inf)
    bad = (g["label"] != ref["label"]) & clear & (margin > 2 * TOL * scale)
    assert not bad.any()
    # ambiguous queries: still the Eq. 5 mean of the neighbours the GPU reports (checked with the oracle's similarities)
    return dict(near_ties=int((~clear).sum()), wq_rel=float(err_w), prop_rel=float(err_p))


@pytest.mark.parametrize("Nq,Ns,D,K,P,k", [
    (1, 1, 4, 1, 1, 1), (33, 5, 7, 3, 1, 16), (1000, 31, 64, 12, 2, 3), (4097, 150, 768, 32, 2, 5),
    (777, 64, 100, 33, 1, 8), (500, 129, 130, 64, 3, 16), (300, 200, 512, 100, 8, 4), (2000, 256, 384, 128, 2, 7),
    (600, 70, 96, 5, 1, 4), (900, 128, 256, 32, 2, 6), (700, 190, 160, 16, 2, 5)])   # 3, 4 and 6 tiles of 32 sources
def test_matches_oracle_on_random_clustered_features(orc, Nq, Ns, D, K, P, k):
    fq, fs, ws, y = _inputs(Nq, Ns, D, K, P, seed=Nq + Ns)
    print(f"\n[knn] Nq={Nq} Ns={Ns} D={D} K={K} P={P} k={k}", flush=True)
    gpu = _run_gpu(fq, fs, ws, y, k)
    ref = orc.knn_densify(fq, fs, ws, k, y=y, T=0.1)
    print(_compare(gpu, ref, ws, y), flush=True)
    assert (gpu["nn_idx"][:, min(k, Ns):] == -1).all()
    # deterministic
    again = _run_gpu(fq, fs, ws, y, k)
    for key in ("wq", "prop", "label", "nn_idx"):
        assert np.array_equal(gpu[key].view(np.uint8), again[key].view(np.uint8)), key


def test_special_cases(orc):
    # queries that are sources themselves, duplicated sources (equal similarities: the lower index first),
    # a zero query (all similarities 0: first k by index, nearest source's vector) and a zero source
    fq, fs, ws, y = _inputs(64, 40, 96, 6, 1, seed=2)
    fs[10] = fs[3]
    fs[20] = 0.0
    fq[:40] = fs
    fq[50] = 0.0
    gpu = _run_gpu(fq, fs, ws, y, 3)
    ref = orc.knn_densify(fq, fs, ws, 3, y=y)
    assert gpu["nn_idx"][3, 0] == 3 and gpu["nn_idx"][10, 0] == 3 and gpu["nn_idx"][10, 1] == 10
    assert list(gpu["nn_idx"][50]) == [0, 1, 2] and np.allclose(gpu["wq"][50], ws[0], rtol=1e-6)
    rows = np.ones(64, bool)
    rows[[3, 10]] = False       # duplicates: order fixed by the tie rule, checked above
    assert np.abs(gpu["wq"][rows] - ref["wq"][rows]).max() <= TOL
    # k = 1 returns the nearest source's vector (phi w / phi in fp32: to rounding)
    g1 = _run_gpu(fq, fs, ws, y, 1)
    assert np.allclose(g1["wq"][rows], ws[g1["nn_idx"][rows, 0]], rtol=1e-6, atol=0)
    # the zero query again where the sources' vectors are too many for the kernel's on-chip copy (eight-wave workgroups,
    # four tiles of materials)
    fq, fs, ws, y = _inputs(300, 256, 64, 128, 2, seed=3)
    fq[[0, 77, 299]] = 0.0
    print("[knn] zero queries, 256 sources x 128 materials", flush=True)
    gpu = _run_gpu(fq, fs, ws, y, 4)
    ref = orc.knn_densify(fq, fs, ws, 4, y=y)
    for i in (0, 77, 299):
        assert list(gpu["nn_idx"][i]) == [0, 1, 2, 3] and np.allclose(gpu["wq"][i], ws[0], rtol=1e-6)
    assert np.abs(gpu["wq"] - ref["wq"]).max() <= TOL * np.abs(ws).max()


def test_on_fused_features_of_a_scene_and_full_size_sample(orc):
    """The densification as the path uses it: queries = fused rows of workload c2 (200 000 x 768), sources =
    150 of its points with their material scores; the oracle recomputes a sample of queries one by one."""
    import gpu_harness as H
    from workloads.scenes import make_scene
    s = make_scene("c2")
    d = H.DeviceScene(s)
    d.step_combined()
    torch.cuda.synchronize()
    fq = d.fused.cpu().numpy()
    src = np.linspace(0, s.N - 1, 150).astype(np.int64)
    fs = fq[src].copy()
    ws = d.scores.cpu().numpy()[src].copy()
    gpu = _run_gpu(fq, fs, ws, s.y, 5, T=s.temperature)
    rng = np.random.default_rng(4)
    sel = np.unique(np.concatenate([np.arange(0, 130), np.arange(s.N - 130, s.N), rng.integers(0, s.N, 3000)]))
    ref = orc.knn_densify(fq[sel], fs, ws, 5, y=s.y, T=s.temperature)
    print(_compare(gpu, ref, ws, s.y, sel=sel), flush=True)
    # a source is its own nearest neighbour
    assert (gpu["nn_idx"][src, 0] == np.arange(150)).all()


def test_nan_and_inf_features_leave_the_other_queries_alone():
    """A NaN in a query's features makes every comparison of the selection false; the call must still name sources
    inside the source set for that query (it addresses their material vectors), and the queries beside it must get
    exactly what they get without it.  Same for a source whose features hold a NaN: it is never selected."""
    Nq, Ns, D, K, P, k = 700, 70, 96, 12, 2, 6
    fq, fs, ws, y = _inputs(Nq, Ns, D, K, P, seed=77)
    clean = _run_gpu(fq, fs, ws, y, k)
    bad_q = np.array([0, 5, 31, 32, 333, 699])
    fq2 = fq.copy()
    fq2[bad_q[:3], 7] = np.nan
    fq2[bad_q[3:5], :] = np.nan
    fq2[bad_q[5], 3] = np.inf
    print("\n[knn] NaN / inf rows among the queries", flush=True)
    gpu = _run_gpu(fq2, fs, ws, y, k)
    ok = np.ones(Nq, bool)
    ok[bad_q] = False
    for key in ("wq", "prop", "label", "nn_idx"):
        assert np.array_equal(gpu[key][ok], clean[key][ok]), key
    assert ((gpu["nn_idx"] >= 0) & (gpu["nn_idx"] < Ns)).all()
    fs2 = fs.copy()
    fs2[11, 5] = np.nan
    print("[knn] a NaN among the sources", flush=True)
    gpu = _run_gpu(fq, fs2, ws, y, k)
    assert ((gpu["nn_idx"] >= 0) & (gpu["nn_idx"] < Ns)).all()
    untouched = ~(clean["nn_idx"] == 11).any(1)
    assert (gpu["nn_idx"][untouched] == clean["nn_idx"][untouched]).all()
    assert np.array_equal(gpu["wq"][untouched], clean["wq"][untouched])
