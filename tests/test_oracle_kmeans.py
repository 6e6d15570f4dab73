"""Pins for the oracle's coarse k-means (Section "Architecture", Indexing: k-means on unit-sphere
data, centroids L2-normalised; read as Euclidean Lloyd iterations on the normalised rows).

Nothing here calls the oracle to produce an expected value:
  * a planted case on the unit circle whose memberships after every iteration are derived by hand
    (written out below) and whose centres are the normalised sums of those explicit sets;
  * a pure-Python Lloyd loop written from the definition (squared distances as sum (x - m)^2,
    means as sums divided by counts) on a small set whose cluster means have very different lengths;
  * the fixed point at convergence; the empty-cell rule; and planted mistakes that these pins reject.
"""
import math

import numpy as np
import pytest

from oracle import ivftq_oracle as orc


def _circle(deg):
    a = np.deg2rad(np.asarray(deg, dtype=np.float64))
    return np.stack([np.cos(a), np.sin(a)], axis=1)


def _unit(v):
    v = np.asarray(v, dtype=np.float64)
    return v / np.linalg.norm(v)


# ---------------------------------------------------------------- hand-computable case

# Six points on the unit circle at these angles; both initial centres sit in the first group.
ANGLES = [0.0, 8.0, 20.0, 100.0, 110.0, 120.0]
INIT = [0, 2]       # centres start at 0 deg and 20 deg
# Iteration 1 (centres 0 deg and 20 deg, both of length 1, so the nearest is the smaller angle):
#   0 -> A, 8 -> A (8 < 12), 20 -> B, 100/110/120 -> B.        A1 = {0, 1}, B1 = {2, 3, 4, 5}
#   mean A = cos(4 deg) * u(4 deg); mean B = (sum cos, sum sin)/4 = (-0.01900, 0.78314), length 0.78337
# Iteration 2 (Euclidean distance to those means): the point at 20 deg is 0.2780 from mean A and
#   1.055 from mean B, so it moves to A; the others stay.        A2 = {0, 1, 2}, B2 = {3, 4, 5}
# Iteration 3: nothing moves (A's mean points to 9.33 deg, B's to 110 deg).
MEMBERS = {1: ([0, 1], [2, 3, 4, 5]), 2: ([0, 1, 2], [3, 4, 5]), 3: ([0, 1, 2], [3, 4, 5])}


def test_hand_case_memberships_are_what_the_comment_says():
    """The derivation above, checked with explicit distances (no oracle call)."""
    P = _circle(ANGLES)
    centres = [P[INIT[0]].copy(), P[INIT[1]].copy()]
    for it in (1, 2, 3):
        sets = ([], [])
        for i, p in enumerate(P):
            d0 = sum((p[j] - centres[0][j]) ** 2 for j in range(2))
            d1 = sum((p[j] - centres[1][j]) ** 2 for j in range(2))
            sets[0 if d0 <= d1 else 1].append(i)
        assert (sets[0], sets[1]) == MEMBERS[it]
        centres = [P[s].sum(axis=0) / len(s) for s in sets]
    assert abs(math.degrees(math.atan2(centres[0][1], centres[0][0])) - 9.326) < 1e-3
    assert abs(math.degrees(math.atan2(centres[1][1], centres[1][0])) - 110.0) < 1e-9


@pytest.mark.parametrize("niter", [1, 2, 3, 7])
def test_hand_case_centres(niter):
    P = _circle(ANGLES)
    # the inputs are scaled row by row: training normalises them first
    X = P * np.array([[3.0], [0.5], [1.0], [7.0], [0.1], [2.0]])
    C, inertia = orc.train_coarse(X, 2, niter, np.array(INIT))
    A, B = MEMBERS[min(niter, 3)]
    np.testing.assert_allclose(C[0], _unit(P[A].sum(axis=0)), atol=1e-12)
    np.testing.assert_allclose(C[1], _unit(P[B].sum(axis=0)), atol=1e-12)
    # closed forms: after one iteration A points to 4 deg; from the second on B points to 110 deg
    if niter == 1:
        np.testing.assert_allclose(C[0], _circle([4.0])[0], atol=1e-12)
    else:
        np.testing.assert_allclose(C[1], _circle([110.0])[0], atol=1e-12)
    # objective of the last assignment step = sum of squared distances to the centres it used
    if niter == 1:
        prev = [P[INIT[0]], P[INIT[1]]]
    else:
        pa, pb = MEMBERS[min(niter - 1, 3)]
        prev = [P[pa].mean(axis=0), P[pb].mean(axis=0)]
    want = sum(float(np.sum((P[i] - prev[0]) ** 2)) for i in A) + sum(float(np.sum((P[i] - prev[1]) ** 2)) for i in B)
    assert inertia == pytest.approx(want, abs=1e-12)


def test_hand_case_objective_strictly_drops_until_the_fixed_point():
    P = _circle(ANGLES)
    obj = [orc.train_coarse(P, 2, it, np.array(INIT))[1] for it in (1, 2, 3, 4)]
    assert obj[0] > obj[1] > obj[2]          # the move of the 20-degree point pays
    assert obj[3] == pytest.approx(obj[2], abs=1e-14)


def test_zero_iterations_return_the_normalised_initial_rows():
    P = _circle(ANGLES) * 4.0
    C, inertia = orc.train_coarse(P, 2, 0, np.array(INIT))
    np.testing.assert_allclose(C, _circle([0.0, 20.0]), atol=1e-15)
    assert math.isnan(inertia)


# ---------------------------------------------------------------- brute force from the definition


def _spread_set(seed=5, n=360, d=4):
    """Unit vectors in groups of very different spread, so that the cluster means have very
    different lengths and 'nearest mean' differs from 'largest cosine' and from 'largest dot product'."""
    rs = np.random.Generator(np.random.Philox(key=[seed, 7]))
    dirs = rs.standard_normal((5, d))
    dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
    spread = np.array([0.03, 0.9, 0.15, 1.4, 0.4])
    comp = rs.integers(0, 5, size=n)
    X = dirs[comp] + spread[comp][:, None] * rs.standard_normal((n, d)) / math.sqrt(d)
    return X * rs.uniform(0.2, 5.0, size=(n, 1))        # raw norms vary: training must normalise


def _lloyd_by_definition(X, init, niter, assign_rule="euclid", update=True):
    """Plain loops.  assign_rule: 'euclid' (the reading), 'cosine' (spherical k-means), 'dot' (largest
    inner product with the un-normalised mean).  Returns (normalised centres, last objective)."""
    n, d = X.shape
    Xn = [[float(v) / math.sqrt(sum(float(u) ** 2 for u in row)) for v in row] for row in X]
    C = [list(Xn[i]) for i in init]
    L = len(C)
    obj = float("nan")
    for _ in range(niter):
        members = [[] for _ in range(L)]
        obj = 0.0
        for i, x in enumerate(Xn):
            dist = [sum((x[j] - c[j]) ** 2 for j in range(d)) for c in C]
            if assign_rule == "euclid":
                key = [-v for v in dist]
            elif assign_rule == "cosine":
                key = [sum(x[j] * c[j] for j in range(d)) / math.sqrt(sum(v * v for v in c)) for c in C]
            else:
                key = [sum(x[j] * c[j] for j in range(d)) for c in C]
            best = max(range(L), key=lambda l: (key[l], -l))      # ties: smallest index
            members[best].append(i)
            obj += dist[best]
        if update:
            for l in range(L):
                assert members[l], "the brute-force sets are chosen so that no cell empties"
                C[l] = [sum(Xn[i][j] for i in members[l]) / len(members[l]) for j in range(d)]
    out = np.array([[v / math.sqrt(sum(u * u for u in c)) for v in c] for c in C])
    return out, obj


@pytest.mark.parametrize("niter", [1, 2, 4, 9])
def test_matches_lloyd_written_from_the_definition(niter):
    X = _spread_set()
    init = np.array([3, 50, 111, 200, 301])
    want, want_obj = _lloyd_by_definition(X, init, niter)
    C, obj = orc.train_coarse(X, 5, niter, init)
    np.testing.assert_allclose(C, want, atol=1e-12)
    assert obj == pytest.approx(want_obj, rel=1e-12)


@pytest.mark.parametrize("mistake", ["no_update", "cosine", "dot"])
def test_planted_mistakes_fail_the_brute_force_pin(mistake):
    """A k-means that never moves its centres, assigns by cosine (spherical k-means) or by the raw
    inner product must not pass for the reading: each gives other centres on this set."""
    X = _spread_set()
    init = np.array([3, 50, 111, 200, 301])
    C, _ = orc.train_coarse(X, 5, 4, init)
    if mistake == "no_update":
        wrong, _ = _lloyd_by_definition(X, init, 4, update=False)
    else:
        wrong, _ = _lloyd_by_definition(X, init, 4, assign_rule=mistake)
    assert np.max(np.abs(C - wrong)) > 1e-3


# ---------------------------------------------------------------- fixed point, empty cells


def test_fixed_point_at_convergence():
    """Well-separated blobs: after convergence every centre is the normalised mean of the points that
    are nearest to it, and no point is nearer to another centre."""
    rs = np.random.Generator(np.random.Philox(key=[11, 3]))
    d, L = 6, 4
    dirs = np.eye(d)[:L] * 2.0 - 0.3
    dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
    comp = np.repeat(np.arange(L), 40)
    X = dirs[comp] + 0.05 * rs.standard_normal((len(comp), d))
    init = np.array([0, 40, 80, 120])
    C, obj = orc.train_coarse(X, L, 25, init)
    C2, obj2 = orc.train_coarse(X, L, 26, init)
    np.testing.assert_allclose(C2, C, atol=1e-14)              # converged
    assert obj2 == pytest.approx(obj, abs=1e-13)
    Xn = X / np.linalg.norm(X, axis=1, keepdims=True)
    d2 = ((Xn[:, None, :] - C[None, :, :]) ** 2).sum(axis=2)
    near = d2.argmin(axis=1)
    assert np.array_equal(near, comp)                            # each blob is one cell
    for l in range(L):
        np.testing.assert_allclose(C[l], _unit(Xn[near == l].sum(axis=0)), atol=1e-12)
        others = np.delete(d2[near == l], l, axis=1)
        assert np.all(others.min(axis=1) > d2[near == l, l])
    # the objective equals the within-cell scatter about the un-normalised means
    scatter = sum(float(((Xn[near == l] - Xn[near == l].mean(axis=0)) ** 2).sum()) for l in range(L))
    assert obj == pytest.approx(scatter, rel=1e-12)


def test_empty_cell_is_reseeded_from_the_largest_cell():
    """Two initial rows are the same vector: ties go to the smaller index, the second cell gets no
    point and must come back as a member of the largest cell, not as a stale or undefined centre."""
    P = _circle([0.0, 0.0, 5.0, 10.0, 180.0, 185.0, 90.0])
    X = P.copy()
    X[1] *= 2.0                                   # same direction as row 0, another raw norm
    C, _ = orc.train_coarse(X, 3, 1, np.array([0, 1, 4]))
    # iteration 1: cell 0 takes 0, 0, 5, 10 and 90 (five points: the largest), cell 1 nothing, cell 2 takes 180, 185
    np.testing.assert_allclose(C[0], _unit(P[[0, 1, 2, 3, 6]].sum(axis=0)), atol=1e-12)
    np.testing.assert_allclose(C[2], _unit(P[[4, 5]].sum(axis=0)), atol=1e-12)
    members = P[[0, 1, 2, 3, 6]]
    assert np.min(np.abs(members - C[1][None, :]).max(axis=1)) < 1e-12
