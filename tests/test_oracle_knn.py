"""Pins for the oracle's feature-space k-NN densification (Sec. 3.4.1, Eq. 5).

Expectations: hand-worked cases (tests/golden/knn_cases.txt), a numpy evaluation of the definition built
from library routines (normalised matmul, stable argsort), closed forms and invariants.  None comes from
the oracle or from the GPU library.
"""
import os

import numpy as np
import pytest
from scipy.special import softmax

GOLD = os.path.join(os.path.dirname(__file__), "golden", "knn_cases.txt")


def _vecs(text):
    return np.array([[float(x) for x in part.split()] for part in text.split(";")], np.float64)


def test_hand_worked_cases(orc):
    rows = [l for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 8
    for line in rows:
        k, q, fs, ws, want, order = [c.strip() for c in line.split("|")]
        r = orc.knn_densify(_vecs(q), _vecs(fs), _vecs(ws), int(k))
        assert np.allclose(r["wq"][0], _vecs(want)[0], rtol=1e-13, atol=1e-13), line
        picked = [int(x) - 1 for x in order.split()]
        assert list(r["nn_idx"][0][:len(picked)]) == picked, line
        assert (r["nn_idx"][0][len(picked):] == -1).all()


def _numpy_reference(fq, fs, ws, k):
    """The definition with library routines: cosine matrix, stable sort, weighted mean."""
    qn = fq / np.linalg.norm(fq, axis=1, keepdims=True)
    sn = fs / np.linalg.norm(fs, axis=1, keepdims=True)
    phi = qn @ sn.T
    idx = np.argsort(-phi, axis=1, kind="stable")[:, :k]
    w = np.take_along_axis(phi, idx, 1)
    return (w[:, :, None] * ws[idx]).sum(1) / w.sum(1, keepdims=True), idx, w


@pytest.mark.parametrize("Nq,Ns,D,K,k", [(200, 37, 16, 5, 1), (300, 150, 64, 12, 5), (64, 8, 3, 2, 8), (50, 200, 32, 33, 16)])
def test_matches_numpy_evaluation_of_the_definition(orc, Nq, Ns, D, K, k):
    rng = np.random.default_rng(Nq + Ns)
    # clustered features, all in the positive orthant: similarities are positive as for parts of one object
    fs = np.abs(rng.standard_normal((Ns, D))) + 0.1
    fq = np.abs(fs[rng.integers(0, Ns, Nq)] + 0.3 * rng.standard_normal((Nq, D))) + 0.05
    ws = rng.uniform(-1, 1, (Ns, K))
    r = orc.knn_densify(fq, fs, ws, k)
    want, idx, w = _numpy_reference(fq, fs, ws, k)
    assert np.array_equal(r["nn_idx"], idx)
    assert np.allclose(r["nn_sim"], w, rtol=0, atol=1e-14)
    assert np.allclose(r["wq"], want, rtol=1e-12, atol=1e-13)
    # the gap is the margin to the best source left out
    if k < Ns:
        qn = fq / np.linalg.norm(fq, axis=1, keepdims=True)
        sn = fs / np.linalg.norm(fs, axis=1, keepdims=True)
        srt = -np.sort(-(qn @ sn.T), axis=1)
        assert np.allclose(r["gap"], srt[:, k - 1] - srt[:, k], atol=1e-14)
    else:
        assert np.isinf(r["gap"]).all()


def test_special_cases_and_invariants(orc):
    rng = np.random.default_rng(3)
    Ns, D, K = 40, 24, 6
    fs = np.abs(rng.standard_normal((Ns, D))) + 0.1
    ws = rng.uniform(0, 1, (Ns, K))
    fq = np.abs(rng.standard_normal((100, D))) + 0.1
    base = orc.knn_densify(fq, fs, ws, 4)
    # a query that IS a source, k = 1: that source's vector, similarity 1
    r = orc.knn_densify(fs[[7, 23]], fs, ws, 1)
    assert list(r["nn_idx"][:, 0]) == [7, 23] and np.allclose(r["nn_sim"], 1.0, atol=1e-15)
    assert np.array_equal(r["wq"], ws[[7, 23]])
    # cosine: positive scaling of any feature vector changes nothing
    r = orc.knn_densify(fq * rng.uniform(0.1, 9, (100, 1)), fs * rng.uniform(0.1, 9, (Ns, 1)), ws, 4)
    assert np.array_equal(r["nn_idx"], base["nn_idx"]) and np.allclose(r["wq"], base["wq"], rtol=1e-12)
    # permuting the sources permutes the indices, nothing else (no ties in random data)
    perm = rng.permutation(Ns)
    r = orc.knn_densify(fq, fs[perm], ws[perm], 4)
    assert np.array_equal(perm[r["nn_idx"]], base["nn_idx"]) and np.allclose(r["wq"], base["wq"], rtol=1e-12)
    # positive similarities: a convex combination, inside the neighbours' range per component
    nb = ws[base["nn_idx"]]
    assert (base["wq"] <= nb.max(1) + 1e-12).all() and (base["wq"] >= nb.min(1) - 1e-12).all()
    # all sources carry the same vector: it is reproduced whatever the weights
    r = orc.knn_densify(fq, fs, np.tile(ws[:1], (Ns, 1)), 5)
    assert np.allclose(r["wq"], ws[0], rtol=1e-13)
    # the material vectors enter linearly
    r2 = orc.knn_densify(fq, fs, 3.0 * ws + 1.0, 4)
    assert np.allclose(r2["wq"], 3.0 * base["wq"] + 1.0, rtol=1e-12)
    # duplicate sources: equal similarity, the lower index first
    fs2 = np.concatenate([fs, fs[:3]])
    ws2 = np.concatenate([ws, ws[:3] + 5.0])
    r = orc.knn_densify(fs[:3], fs2, ws2, 2)
    assert np.array_equal(r["nn_idx"], np.array([[0, Ns], [1, Ns + 1], [2, Ns + 2]]))
    assert np.allclose(r["wq"], ws[:3] + 2.5)
    # zero query: every similarity is 0, the first k sources by index, the sum of weights vanishes -> nearest source's vector
    r = orc.knn_densify(np.zeros((1, D)), fs, ws, 3)
    assert list(r["nn_idx"][0]) == [0, 1, 2] and np.array_equal(r["wq"][0], ws[0])


def test_eq4_on_the_interpolated_vector(orc):
    rng = np.random.default_rng(8)
    Ns, D, K, P = 30, 16, 7, 2
    fs = np.abs(rng.standard_normal((Ns, D))) + 0.1
    fq = np.abs(rng.standard_normal((80, D))) + 0.1
    ws = rng.uniform(-0.2, 0.4, (Ns, K))
    y = rng.uniform(100, 8000, (K, P)).astype(np.float32)
    r = orc.knn_densify(fq, fs, ws, 3, y=y, T=0.1)
    want = softmax(r["wq"] / np.float64(np.float32(0.1)), axis=1) @ y.astype(np.float64)
    assert np.allclose(r["prop"], want, rtol=1e-12)
    assert np.array_equal(r["label"], r["wq"].argmax(1))
