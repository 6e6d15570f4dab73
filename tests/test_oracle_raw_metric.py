"""Pins for the oracle's raw-metric search (inner product and squared L2 distance of un-normalised
vectors from the stored norm and the estimate of <q~, x~>).  The paper has no such mode; what fixes it
is the mathematics: with the exact cosine in place of the estimate the values are the metric's
definition, written out here in plain loops, and with fine codes the ranking is the exact one."""
import math

import numpy as np
import pytest

from oracle import ivftq_oracle as orc
from workloads import synth


def _problem(n=1500, nq=12, d=24, L=8, b=8, seed=4):
    rs = np.random.Generator(np.random.Philox(key=[seed, 31]))
    means = rs.standard_normal((6, d))
    X = means[rs.integers(0, 6, n)] + 0.5 * rs.standard_normal((n, d))
    X *= rs.uniform(0.2, 6.0, size=(n, 1))                   # lengths vary by a factor of 30
    Q = means[rs.integers(0, 6, nq)] + 0.5 * rs.standard_normal((nq, d))
    Q *= rs.uniform(0.5, 3.0, size=(nq, 1))
    cent, _ = orc.train_coarse(X, L, 4, synth.kmeans_init_indices(seed, n, L))
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(seed, d))
    c, tau = orc.lloyd_max_codebook(b, d)
    idx = orc.ListIndex(cent, Pi, c, tau)
    idx.add(X)
    return X, Q, idx, orc.raw_norms_fp32(X)


def test_identities_with_the_exact_cosine_reproduce_the_definitions():
    rs = np.random.Generator(np.random.Philox(key=[1, 2]))
    for _ in range(50):
        d = int(rs.integers(2, 9))
        x = rs.standard_normal(d) * rs.uniform(0.1, 9.0)
        q = rs.standard_normal(d) * rs.uniform(0.1, 9.0)
        nx = math.sqrt(sum(v * v for v in x))
        nq = math.sqrt(sum(v * v for v in q))
        cos = sum((a / nx) * (b / nq) for a, b in zip(x, q))
        ip = sum(a * b for a, b in zip(x, q))
        l2 = sum((a - b) ** 2 for a, b in zip(x, q))
        assert orc.metric_value(cos, nx, nq, "ip") == pytest.approx(ip, abs=1e-10)
        assert orc.metric_value(cos, nx, nq, "l2") == pytest.approx(l2, abs=1e-10)
    with pytest.raises(ValueError):
        orc.metric_value(0.0, 1.0, 1.0, "cosine")


def test_stored_norm_is_the_float32_of_the_double_norm():
    X = np.array([[3.0, 4.0], [1e-3, 0.0], [1.0, 1.0]])
    n = orc.raw_norms_fp32(X)
    assert n.dtype == np.float32
    np.testing.assert_array_equal(n, np.array([5.0, 1e-3, math.sqrt(2.0)], dtype=np.float32))


@pytest.mark.parametrize("metric", ["ip", "l2"])
def test_fine_codes_and_every_cell_probed_give_the_exact_ranking(metric):
    """8-bit codes, nprobe = nlist: the estimate is within 1e-3 of the cosine, so the values are within a
    small multiple of |q||x| of the exact metric and nearly all of the exact top 10 are found."""
    X, Q, idx, xnorm = _problem()
    L = idx.centroids.shape[0]
    vals, ids, _, _, everything = orc.search_raw(idx, xnorm, Q, L, 10, metric, return_all=True)
    t_vals, t_ids = orc.exact_topk_raw(X, Q, 10, metric)
    assert orc.recall_at_k(ids, t_ids) > 0.9
    Xd = np.asarray(X, dtype=np.float64)
    for qi in range(len(Q)):
        cid, val = everything[qi]
        assert len(cid) == len(X)                                        # every vector is a candidate
        q = np.asarray(Q[qi], dtype=np.float64)
        exact = Xd[cid] @ q if metric == "ip" else np.sum((Xd[cid] - q) ** 2, axis=1)
        scale = np.linalg.norm(q) * np.linalg.norm(Xd[cid], axis=1)
        assert np.max(np.abs(val - exact) / scale) < 0.02
        order = np.argsort(-vals[qi]) if metric == "ip" else np.argsort(vals[qi])
        np.testing.assert_array_equal(order, np.arange(10))              # best first


def test_ranking_by_raw_metric_differs_from_cosine_when_lengths_vary():
    """A planted pair: the same direction at two lengths.  Cosine cannot tell them apart; the inner product
    prefers the long one, the distance the one whose length is nearer the query's."""
    d = 16
    e = np.zeros(d)
    e[0] = 1.0
    rs = np.random.Generator(np.random.Philox(key=[9, 9]))
    noise = rs.standard_normal((40, d))
    X = np.vstack([0.5 * e, 20.0 * e, noise])
    q = (1.0 * e)[None, :]
    cent = orc.normalize_rows(np.vstack([e, -e, noise[0], noise[1]]))
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(3, d))
    c, tau = orc.lloyd_max_codebook(6, d)
    idx = orc.ListIndex(cent, Pi, c, tau)
    idx.add(X)
    xn = orc.raw_norms_fp32(X)
    _, ids_ip, _, _ = orc.search_raw(idx, xn, q, 4, 2, "ip")
    _, ids_l2, _, _ = orc.search_raw(idx, xn, q, 4, 2, "l2")
    s_cos, ids_cos, _, _ = orc.search(idx, q, 4, 2)
    assert ids_ip[0, 0] == 1                        # <q, 20 e> = 20 beats <q, 0.5 e> = 0.5
    assert ids_l2[0, 0] == 0                        # |q - 0.5 e|^2 = 0.25 beats |q - 20 e|^2 = 361
    assert set(ids_cos[0]) == {0, 1} and abs(s_cos[0, 0] - s_cos[0, 1]) < 1e-12
    v_l2, _, _, _ = orc.search_raw(idx, xn, q, 4, 2, "l2")
    assert v_l2[0, 0] == pytest.approx(0.25, abs=0.05)


@pytest.mark.parametrize("mistake", ["drop_x2", "norm_not_squared", "sign", "unit_query"])
def test_planted_mistakes_break_the_definition_pin(mistake):
    def wrong(s_hat, xn, qn, metric):
        if mistake == "drop_x2":
            return qn * qn - 2.0 * qn * xn * s_hat
        if mistake == "norm_not_squared":
            return qn * qn + xn - 2.0 * qn * xn * s_hat
        if mistake == "sign":
            return qn * qn + xn * xn + 2.0 * qn * xn * s_hat
        return 1.0 + xn * xn - 2.0 * xn * s_hat
    x, q = np.array([3.0, 4.0, 0.0]), np.array([0.0, 2.0, 2.0])
    nx, nq = 5.0, math.sqrt(8.0)
    cos = float(x @ q) / (nx * nq)
    exact = float(np.sum((x - q) ** 2))
    assert orc.metric_value(cos, nx, nq, "l2") == pytest.approx(exact, abs=1e-12)
    assert abs(wrong(cos, nx, nq, "l2") - exact) > 0.5


def test_padding_and_ties():
    X, Q, idx, xnorm = _problem(n=40, nq=3, L=8, b=4)
    for metric, worst in (("ip", -np.inf), ("l2", np.inf)):
        vals, ids, probes, _ = orc.search_raw(idx, xnorm, Q, 1, 30, metric)
        for qi in range(3):
            n_real = len(idx.ids[probes[qi, 0]])
            assert np.all(ids[qi, n_real:] == -1) and np.all(vals[qi, n_real:] == worst)
            assert np.all(ids[qi, :n_real] >= 0)
