"""Pins for the WMD / WCD / pruning oracle (CPU only): hand-evaluated values, closed forms, other library routines
on special cases, bounds that the mathematics fixes, and brute force on small inputs."""
import os

import numpy as np
import pytest
import scipy.optimize
from scipy.spatial.distance import cdist

import oracle
from paper_1711_07227_amd import synth
from test_oracle_pins import csr_from_docs, docs_from_csr, small_problem

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_wmd.txt")


def test_hand_worked_wmd_and_wcd():
    E = np.array([[0, 0], [3, 0], [0, 4], [3, 4], [6, 8]], np.float32)
    docs = {"A": {0: 0.5, 1: 0.5}, "B": {2: 0.25, 3: 0.75}, "C": {0: 0.125, 4: 0.875}}
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 4
    for first, second, wmd, wcd in rows:
        a, b = csr_from_docs([docs[first]]), csr_from_docs([docs[second]])
        assert oracle.wmd_pair(E, a, b, 0, 0) == pytest.approx(float(wmd), abs=1e-9)
        assert oracle.wmd_pair(E, b, a, 0, 0) == pytest.approx(float(wmd), abs=1e-9)
        assert oracle.wcd(E, a, b)[0, 0] == pytest.approx(float(wcd), abs=1e-12)


def test_cost_matrix_against_cdist_and_orientation():
    rng = np.random.default_rng(0)
    A, B = rng.standard_normal((5, 7)), rng.standard_normal((3, 7))
    C = oracle.cost_matrix(A, B)
    assert C.shape == (5, 3)
    assert np.allclose(C, cdist(A, B), rtol=1e-13, atol=0)


def test_emd_one_word_against_closed_form():
    """All mass sits on one word: every flow is forced, EMD = sum_q x2[q] c[0, q]; and the transposed case."""
    rng = np.random.default_rng(1)
    c = rng.random((1, 9)) + 0.1
    x2 = rng.random(9)
    x2 /= x2.sum()
    assert oracle.emd([1.0], x2, c) == pytest.approx(float(c[0] @ x2), rel=1e-12)
    assert oracle.emd(x2, [1.0], c.T) == pytest.approx(float(c[0] @ x2), rel=1e-12)


def test_emd_two_by_two_closed_form():
    """One free parameter t = y[0,0] in [max(0, a+b-1), min(a, b)]; the cost is linear in t."""
    rng = np.random.default_rng(2)
    for _ in range(20):
        a, b = rng.uniform(0.05, 0.95, 2)
        c = rng.random((2, 2))
        ends = [max(0.0, a + b - 1.0), min(a, b)]
        best = min(t * c[0, 0] + (a - t) * c[0, 1] + (b - t) * c[1, 0] + (1 - a - b + t) * c[1, 1] for t in ends)
        assert oracle.emd([a, 1 - a], [b, 1 - b], c) == pytest.approx(best, rel=1e-10, abs=1e-12)


def test_emd_uniform_weights_against_assignment_solver():
    """Equal weights 1/h on both sides: an optimal flow is a permutation (Birkhoff), so EMD = assignment cost / h."""
    rng = np.random.default_rng(3)
    for h in (2, 5, 17):
        c = rng.random((h, h))
        r, s = scipy.optimize.linear_sum_assignment(c)
        x = np.full(h, 1.0 / h)
        assert oracle.emd(x, x, c) == pytest.approx(c[r, s].sum() / h, rel=1e-10)
    # a transposed cost matrix must change the answer when the weights are not symmetric: guards the variable order
    c = np.array([[0.0, 1.0, 5.0], [2.0, 0.0, 1.0]])
    x1, x2 = np.array([0.7, 0.3]), np.array([0.1, 0.2, 0.7])
    # rows: word 0 sends 0.1 to q0 (0), 0.2 to q1 (1), 0.4 to q2 (5): alternatives checked by the LP; closed value below
    # feasible flows: y = [[0.1, s, 0.6 - s], [0, 0.2 - s, 0.1 + s]] with y[1,0] = 0 optimal since c[1,0] > c[0,0]
    best = min(0.1 * 0 + s * 1 + (0.6 - s) * 5 + (0.2 - s) * 0 + (0.1 + s) * 1 for s in (0.0, 0.2))
    assert oracle.emd(x1, x2, c) == pytest.approx(best, rel=1e-10)


def emd_on_a_line(xa, fa, xb, fb):
    """Textbook closed form in one dimension with cost |x - y|: the area between the two cumulative distributions."""
    pts = np.unique(np.concatenate([xa, xb]))
    Fa = np.array([fa[xa <= t].sum() for t in pts])
    Fb = np.array([fb[xb <= t].sum() for t in pts])
    return float(np.sum(np.abs(Fa - Fb)[:-1] * np.diff(pts)))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_wmd_on_a_line_against_cdf_area(seed):
    rng = np.random.default_rng(seed)
    v = 30
    E = rng.uniform(-3, 3, (v, 1)).astype(np.float32)
    docs = []
    for _ in range(4):
        h = int(rng.integers(2, 9))
        words = rng.choice(v, h, replace=False)
        w = rng.random(h) + 0.05
        docs.append({int(a): float(b) for a, b in zip(words, (w / w.sum()).astype(np.float32))})
    csr = csr_from_docs(docs)
    dd = docs_from_csr(csr)
    for i in range(4):
        for j in range(4):
            (pa, fa), (pb, fb) = dd[i], dd[j]
            ref = emd_on_a_line(E[pa, 0].astype(np.float64), fa / fa.sum(), E[pb, 0].astype(np.float64), fb / fb.sum())
            assert oracle.wmd_pair(E, csr, csr, i, j) == pytest.approx(ref, rel=1e-9, abs=1e-12)


def test_wmd_bounds_symmetry_and_triangle_inequality():
    E, db, qs = small_problem(5, v=60, m=6, n=6, q=5, hmax=7)
    R, R12, R21 = oracle.rwmd_bruteforce(E, db, qs, parts=True)
    W = np.array([[oracle.wmd_pair(E, db, qs, i, j) for j in range(5)] for i in range(6)])
    Wt = np.array([[oracle.wmd_pair(E, qs, db, j, i) for j in range(5)] for i in range(6)])
    assert np.allclose(W, Wt, rtol=1e-9)                                    # EMD with a symmetric ground distance
    # Sec. III: RWMD <= WMD.  RWMD uses the weights as stored (mass 1 up to fp32 rounding), WMD renormalises them
    slack = W * 1e-6
    assert np.all(R <= W + slack) and np.all(R12 <= W + slack) and np.all(R21 <= W + slack)
    assert np.all(oracle.wcd(E, db, qs) <= W + slack)                      # WCD is a lower bound as well
    assert np.any(R < W - 1e-6)                                             # and the relaxation is not always tight
    # the independent coupling y = x1 x2^T is feasible, so it bounds WMD from above
    ddb, dq = docs_from_csr(db), docs_from_csr(qs)
    for i, (pa, fa) in enumerate(ddb):
        for j, (pb, fb) in enumerate(dq):
            up = (fa / fa.sum()) @ cdist(E[pa].astype(np.float64), E[pb].astype(np.float64)) @ (fb / fb.sum())
            assert W[i, j] <= up + 1e-9
    # metric: WMD(a, c) <= WMD(a, b) + WMD(b, c) within one set
    S = np.array([[oracle.wmd_pair(E, db, db, i, j) for j in range(6)] for i in range(6)])
    assert np.allclose(np.diag(S), 0, atol=1e-12)
    for a in range(6):
        for b in range(6):
            for c in range(6):
                assert S[a, c] <= S[a, b] + S[b, c] + 1e-9


def test_wmd_does_not_depend_on_the_scale_of_the_stored_weights():
    """Weights are renormalised in fp64, so a histogram stored with mass 1 - 3e-8 or 2.0 gives the same distance."""
    E, db, qs = small_problem(7)
    ptr, col, val = db
    scaled = (ptr, col, (val * np.float32(2.0)).astype(np.float32))
    for j in range(3):
        assert oracle.wmd_pair(E, scaled, qs, 1, j) == pytest.approx(oracle.wmd_pair(E, db, qs, 1, j), rel=1e-12)


def test_wcd_against_numpy_centroids(tiny):
    sub = synth.csr_rows(*tiny["db"], np.arange(40))
    got = oracle.wcd(tiny["E"], sub, tiny["queries"])
    ptr, col, val = sub
    X = np.zeros((40, tiny["E"].shape[0]))
    for i in range(40):
        X[i, col[ptr[i]:ptr[i + 1]]] = val[ptr[i]:ptr[i + 1]]
    qp, qc, qv = tiny["queries"]
    Q = np.zeros((10, tiny["E"].shape[0]))
    for j in range(10):
        Q[j, qc[qp[j]:qp[j + 1]]] = qv[qp[j]:qp[j + 1]]
    E64 = tiny["E"].astype(np.float64)
    assert np.allclose(got, cdist(X @ E64, Q @ E64), rtol=1e-12, atol=1e-14)


def test_pruned_topk_equals_exhaustive_topk_and_prunes():
    """Sec. III, 'Speeding-up WMD using RWMD': the cut-off never loses a true neighbour."""
    rng = np.random.default_rng(11)
    v, m, n, q, k = 80, 4, 40, 4, 3
    E = rng.standard_normal((v, m)).astype(np.float32)
    db = synth.corpus(n, v, 2, 7, 1.0, 12)
    qs = synth.corpus(q, v, 2, 7, 1.0, 13)
    R = oracle.rwmd_bruteforce(E, db, qs)
    W = np.array([[oracle.wmd_pair(E, db, qs, i, j) for j in range(q)] for i in range(n)])
    idx, dist, evaluated = oracle.wmd_topk_pruned(E, db, qs, k, R)
    for j in range(q):
        order = np.lexsort((np.arange(n), W[:, j]))[:k]
        assert np.array_equal(idx[j], order)
        assert np.allclose(dist[j], W[order, j], rtol=1e-12)
        L = W[np.lexsort((np.arange(n), R[:, j]))[:k], j].max()
        assert evaluated[j] == len(set(np.nonzero(R[:, j] < L)[0]) | set(np.lexsort((np.arange(n), R[:, j]))[:k]))
    assert evaluated.sum() < n * q                     # something was pruned
    assert np.all(evaluated >= k)
