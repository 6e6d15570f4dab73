"""Pins for the oracle's encode, search, reconstruction and ground truth (CPU only).

The encode/search arithmetic is checked against (i) identities the paper states,
(ii) pure-Python re-derivations through a different route (reconstruct the vector in
the original frame, then take the inner product), (iii) brute force on tiny inputs,
(iv) the paper's printed numbers, and (v) planted mistakes that each pin must catch.
"""
import math

import numpy as np
import pytest

from oracle import ivftq_oracle as orc
from workloads import synth


def _small_problem(n=600, d=16, L=6, b=3, nq=12, seed=5):
    rng = np.random.default_rng(seed)
    means = rng.normal(size=(L, d))
    X = (means[rng.integers(0, L, n)] + 0.4 * rng.normal(size=(n, d))).astype(np.float32)
    Q = (means[rng.integers(0, L, nq)] + 0.4 * rng.normal(size=(nq, d))).astype(np.float32)
    init = synth.kmeans_init_indices(seed, n, L)
    C, _ = orc.train_coarse(X, L, 5, init)
    C = C.astype(np.float32)
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(seed, d)).astype(np.float32)
    c, tau = orc.codebook_fp32(b, d)
    return X, Q, C, Pi, c, tau


# ---------------------------------------------------------------- paper's printed numbers


def test_bit_accounting_worked_examples(paper_numbers):
    assert orc.bits_per_vector(4, 96, True) == paper_numbers["bits_deep_b4_sign"]
    assert orc.bits_per_vector(4, 128, True) == paper_numbers["bits_sift_b4_sign"]
    assert orc.bits_per_vector(4, 200, True) == paper_numbers["bits_t2i_b4_sign"]
    # Stage-1-only storage at B bits has the same total as (B-1)+sign: the matched-memory column
    for key, d in (("sift1m", 128), ("deep1m", 96)):
        for B in (4, 5, 6):
            mib = (1_000_000 * orc.bits_per_vector(B, d, False) / 8 + 1000 * d * 4) / 2 ** 20
            assert abs(mib - paper_numbers[f"mem_mb_{key}_B{B}"]) <= 0.6
            assert orc.bits_per_vector(B, d, False) == orc.bits_per_vector(B - 1, d, True)
    assert abs(1000 * 128 * 4 / 2 ** 20 - paper_numbers["centroid_table_mb_L1000_d128"]) < 0.02


def test_theorem_two_term_by_term(paper_numbers):
    p = paper_numbers
    D, bias, rand, tail = orc.theorem2_terms(p["t2_D4"], 4, 128, 1e-2)
    assert abs(math.sqrt(2 * 4 * math.log(2)) - p["t2_M"]) < 1e-3
    assert abs(math.log(2 / 1e-2) - p["t2_log2delta"]) < 1e-3
    assert abs(math.log(3 * 128) - p["t2_log3d"]) < 1e-3
    assert abs(bias - p["t2_bias"]) < 5e-3
    assert abs(rand - p["t2_random"]) < 1e-3
    assert abs(tail - p["t2_tail"]) < 5e-4
    assert abs(D + bias + rand + tail - p["t2_total"]) < 6e-3
    cs = orc.theorem1_bound(p["t2_D4"], 0.0, 128, 1e-2)
    assert abs(cs - p["cs_total"]) < 5e-3
    assert abs(cs - math.sqrt(p["t2_D4"]) - p["cs_conc"]) < 1e-3


# ---------------------------------------------------------------- quantiser on the sphere


@pytest.mark.parametrize("b,d", [(2, 64), (4, 64), (4, 128)])
def test_flat_tq_error_matches_distortion_and_bounds(b, d):
    """E||v^ - v||^2 = D_b(f_d) and E<v, v^> = 1 - D_b over the rotation; Theorems 1 and 2 hold."""
    c, tau = orc.lloyd_max_codebook(b, d)
    D = orc.codebook_distortion(c, tau, d)
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(11, d))
    V = synth.random_unit_vectors(1, 4000, d)
    Vh = orc.tq_reconstruct(V, Pi, c, tau)
    err2 = np.sum((Vh - V) ** 2, axis=1)
    assert abs(err2.mean() - D) < 4 * err2.std() / math.sqrt(len(V)) + 1e-4
    ip = np.sum(Vh * V, axis=1)
    assert abs(ip.mean() - (1.0 - D)) < 4 * ip.std() / math.sqrt(len(V)) + 1e-4
    # Lemma 2: per-coordinate error at most half the widest bin (outer bins end at +-1)
    edges = np.concatenate(([-1.0], tau, [1.0]))
    U = V @ Pi.T
    assert np.max(np.abs(U - c[orc.quantize(U, tau)])) <= np.max(np.diff(edges))
    # Theorem 1 (delta = 1e-2, R_d >= 0): no violation expected among 4000 vectors
    assert np.all(np.sqrt(err2) <= orc.theorem1_bound(D, 0.0, d, 1e-2))
    # Theorem 2: |<q,v> - <q,v^>| under the printed bound for random unit queries
    Qs = synth.random_unit_vectors(2, 64, d, stream=101)
    gap = np.abs(Qs @ (V - Vh).T)
    assert gap.max() <= sum(orc.theorem2_terms(D, b, d, 1e-2))


# ---------------------------------------------------------------- encode


def test_encode_identities():
    X, Q, C, Pi, c, tau = _small_problem()
    enc = orc.encode(X, C, Pi, tau)
    Xn = orc.normalize_rows(X)
    Cd = C.astype(np.float64)
    # assignment = brute-force argmax of the inner product, smallest index on ties
    for i in range(0, len(X), 37):
        best, arg = -np.inf, -1
        for l in range(C.shape[0]):
            s = float(np.dot(Xn[i], Cd[l]))
            if s > best:
                best, arg = s, l
        assert arg == enc["assign"][i]
        assert abs(best - enc["coarse"][i]) < 1e-15
    # for unit vectors ||x - c||^2 = 2 - 2<x,c>  (the amplification identity, per vector)
    cn = np.linalg.norm(Cd, axis=1)
    g2 = 1.0 + cn[enc["assign"]] ** 2 - 2.0 * enc["coarse"]
    np.testing.assert_allclose(enc["gamma"] ** 2, g2, atol=1e-12)
    assert np.all(enc["gamma"] <= 2.0 + 1e-6)
    # rho is a unit vector and is the rotated residual direction
    np.testing.assert_allclose(np.linalg.norm(enc["rho"], axis=1), 1.0, atol=1e-12)
    r = Xn - Cd[enc["assign"]]
    back = enc["rho"] @ Pi.astype(np.float64) * enc["gamma"][:, None]      # Pi^T (gamma rho) = r
    np.testing.assert_allclose(back, r, atol=1e-6)                         # Pi is fp32-rounded
    # codes: rho_j lies in [tau_{code-1}, tau_code)
    t = np.concatenate(([-np.inf], tau.astype(np.float64), [np.inf]))
    assert np.all(enc["rho"] >= t[enc["codes"]]) and np.all(enc["rho"] < t[enc["codes"].astype(int) + 1])
    # float16 norm is the nearest representable value
    g16 = enc["gamma16"].astype(np.float64)
    up = np.nextafter(enc["gamma16"], np.float16(np.inf)).astype(np.float64)
    dn = np.nextafter(enc["gamma16"], np.float16(-np.inf)).astype(np.float64)
    assert np.all(np.abs(g16 - enc["gamma"]) <= np.abs(up - enc["gamma"]))
    assert np.all(np.abs(g16 - enc["gamma"]) <= np.abs(dn - enc["gamma"]))
    # distance to the nearest boundary
    assert np.all(enc["bdist"] >= 0) and enc["bdist"].max() <= 1.0
    assert np.all(enc["gap"] >= 0)


def test_zero_residual_and_zero_norm_rows():
    X, Q, C, Pi, c, tau = _small_problem()
    enc = orc.encode(C[:2] * 3.0, C, Pi, tau)     # inputs that are centroids themselves (scaled)
    assert list(enc["assign"]) == [0, 1]
    assert np.all(enc["gamma"] < 1e-7)
    with pytest.raises(ValueError):
        orc.encode(np.zeros((1, C.shape[1]), np.float32), C, Pi, tau)


def test_reconstruction_error_is_gamma_squared_times_distortion():
    """||x^ - x~||^2 = gamma^2 ||C(rho) - rho||^2, on average gamma^2 D_b: fails for a transposed
    rotation, a wrong residual sign or a mis-indexed codebook."""
    w = synth.scaled(synth.config_tiny(), 4000, 10)
    X = synth.database(w, 0, 4000)
    d, b = w.d, 4
    init = synth.kmeans_init_indices(0, len(X), 32)
    C, _ = orc.train_coarse(X, 32, 6, init)
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(0, d))
    c, tau = orc.lloyd_max_codebook(b, d)
    D = orc.codebook_distortion(c, tau, d)
    idx = orc.ListIndex(C, Pi, c, tau)
    enc = idx.add(X)
    Xn = orc.normalize_rows(X)
    num, den = 0.0, 0.0
    for l in range(32):
        if len(idx.ids[l]) == 0:
            continue
        xh = orc.reconstruct(idx, l)
        num += np.sum((xh - Xn[idx.ids[l]]) ** 2)
        den += np.sum(idx.gamma16[l].astype(np.float64) ** 2)
    assert abs(num / den - D) < 0.08 * D
    # amplification: E||r||^2 = 2 (1 - E<x~, c~>)
    assert abs(np.mean(enc["gamma"] ** 2) - 2 * (1 - np.mean(enc["coarse"]))) < 1e-12


# ---------------------------------------------------------------- search


def _python_search(X, Q, C, Pi, c, tau, lists, nprobe, k):
    """Search re-derived in the original frame with explicit loops:
    score = <q~, c~_l + gamma16 * Pi^T c[code]>."""
    Qn = orc.normalize_rows(Q)
    Cd, Pid, cd = C.astype(np.float64), Pi.astype(np.float64), c.astype(np.float64)
    out = []
    for q in Qn:
        coarse = [(float(np.dot(q, Cd[l])), l) for l in range(len(Cd))]
        coarse.sort(key=lambda t: (-t[0], t[1]))
        cand = []
        for _, l in coarse[:nprobe]:
            ids, codes, g16 = lists[l]
            for i in range(len(ids)):
                xhat = Cd[l] + float(g16[i]) * (Pid.T @ cd[codes[i]])
                cand.append((float(np.dot(q, xhat)), int(ids[i])))
        cand.sort(key=lambda t: (-t[0], t[1]))
        out.append(cand[:k])
    return out


def test_search_matches_original_frame_rederivation():
    X, Q, C, Pi, c, tau = _small_problem()
    idx = orc.ListIndex(C, Pi, c, tau)
    idx.add(X)
    assert idx.ntotal == len(X) and sum(len(i) for i in idx.ids) == len(X)
    sc, ids, probes, S = orc.search(idx, Q, nprobe=3, k=7)
    ref = _python_search(X, Q, C, Pi, c, tau,
                         [(idx.ids[l], idx.codes[l], idx.gamma16[l]) for l in range(len(idx.ids))], 3, 7)
    for qi, row in enumerate(ref):
        assert [r[1] for r in row] == list(ids[qi])
        np.testing.assert_allclose([r[0] for r in row], sc[qi], atol=1e-6)
    assert np.all(np.diff(sc, axis=1) <= 0)


def test_decomposition_is_exact_with_unquantised_residual():
    """s_l + gamma <Pi q~, rho> = <q~, x~>: only the quantiser makes the estimate approximate."""
    X, Q, C, Pi, c, tau = _small_problem(d=32)
    Pi64 = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(5, 32))
    enc = orc.encode(X, C, Pi64, tau)
    Xn, Qn = orc.normalize_rows(X), orc.normalize_rows(Q)
    Z = Qn @ Pi64.T
    S = Qn @ C.astype(np.float64).T
    est = S[:, enc["assign"]] + (Z @ enc["rho"].T) * enc["gamma"][None, :]
    np.testing.assert_allclose(est, Qn @ Xn.T, atol=1e-12)


def test_search_padding_and_small_lists():
    X, Q, C, Pi, c, tau = _small_problem()
    idx = orc.ListIndex(C, Pi, c, tau)
    idx.add(X[:5], ids=[10, 11, 12, 13, 14])
    sc, ids, probes, _ = orc.search(idx, Q, nprobe=C.shape[0], k=8)
    assert np.all(ids[:, 5:] == -1) and np.all(np.isneginf(sc[:, 5:]))
    assert all(sorted(row[:5]) == [10, 11, 12, 13, 14] for row in ids)
    assert np.all(np.sort(probes, axis=1) == np.arange(C.shape[0]))


def test_recall_rises_with_probes_and_bits_and_reaches_ground_truth():
    w = synth.scaled(synth.config_tiny(), 5000, 60)
    X, Q = synth.database(w, 0, 5000), synth.queries(w, 60)
    L = 32
    C, _ = orc.train_coarse(X, L, 8, synth.kmeans_init_indices(0, len(X), L))
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(0, w.d))
    gt_sc, gt = orc.exact_topk(X, Q, 10)
    rec = {}
    for b in (2, 4, 6):
        c, tau = orc.lloyd_max_codebook(b, w.d)
        idx = orc.ListIndex(C, Pi, c, tau)
        idx.add(X)
        for p in (1, 4, L):
            _, ids, _, _ = orc.search(idx, Q, p, 10)
            rec[b, p] = orc.recall_at_k(ids, gt)
    for b in (2, 4, 6):
        assert rec[b, 1] <= rec[b, 4] <= rec[b, L]
    assert rec[2, L] < rec[4, L] < rec[6, L]
    # isotropic 64-d clusters make near neighbours almost equidistant, so recall is modest
    assert rec[6, L] > 0.85
    assert rec[4, L] > 0.6


def test_exact_topk_against_python_loops():
    rng = np.random.default_rng(3)
    X = rng.normal(size=(70, 5)).astype(np.float32)
    Q = rng.normal(size=(4, 5)).astype(np.float32)
    sc, ids = orc.exact_topk(X, Q, 6)
    for qi in range(4):
        qn = Q[qi].astype(np.float64) / math.sqrt(sum(float(v) ** 2 for v in Q[qi]))
        rows = []
        for i in range(70):
            xn = X[i].astype(np.float64) / math.sqrt(sum(float(v) ** 2 for v in X[i]))
            rows.append((-sum(a * b for a, b in zip(qn, xn)), i))
        rows.sort()
        assert [r[1] for r in rows[:6]] == list(ids[qi])
    assert orc.recall_at_k(ids, ids) == 1.0
    assert orc.recall_at_k(np.full_like(ids, -1), ids) == 0.0


# ---------------------------------------------------------------- k-means invariants


def test_kmeans_invariants():
    w = synth.scaled(synth.config_tiny(), 3000, 1)
    X = synth.database(w, 0, 3000)
    init = synth.kmeans_init_indices(0, len(X), 16)
    prev = None
    for it in (1, 3, 6):
        C, inertia = orc.train_coarse(X, 16, it, init)
        np.testing.assert_allclose(np.linalg.norm(C, axis=1), 1.0, atol=1e-12)
        if prev is not None:
            assert inertia <= prev + 1e-9          # Lloyd iterations never increase the objective
        prev = inertia
    # an initial centre that captures nothing is re-seeded rather than left empty
    far = np.vstack([X, -X[:1]])
    C, _ = orc.train_coarse(far, 4, 3, np.array([0, 1, 2, len(far) - 1]))
    assert np.all(np.isfinite(C))


# ---------------------------------------------------------------- planted mistakes


@pytest.mark.parametrize("mistake", ["transpose_pi", "residual_sign", "codebook_shift", "drop_coarse"])
def test_pins_catch_planted_mistakes(mistake):
    """Each plausible slip must break the original-frame re-derivation pin."""
    X, Q, C, Pi, c, tau = _small_problem()
    idx = orc.ListIndex(C, Pi, c, tau)
    idx.add(X)
    lists = [(idx.ids[l], idx.codes[l], idx.gamma16[l]) for l in range(len(idx.ids))]
    bad = orc.ListIndex(C, Pi, c, tau)
    for l, (i, cd, g) in enumerate(lists):
        bad.set_list(l, i, cd, g)
    if mistake == "transpose_pi":
        bad.Pi = bad.Pi.T.copy()
    elif mistake == "residual_sign":
        bad.gamma16 = [(-g.astype(np.float32)).astype(np.float16) for g in bad.gamma16]
    elif mistake == "codebook_shift":
        bad.c = np.roll(bad.c, 1)
    elif mistake == "drop_coarse":
        bad.centroids = bad.centroids * 0.0
    sc, ids, _, _ = orc.search(bad, Q, nprobe=3, k=7)
    ref = _python_search(X, Q, C, Pi, c, tau, lists, 3, 7)
    same = all([r[1] for r in row] == list(ids[qi]) for qi, row in enumerate(ref))
    close = all(np.allclose([r[0] for r in row], sc[qi], atol=1e-6) for qi, row in enumerate(ref))
    assert not (same and close)


# ---------------------------------------------------------------- adaptive coarse refresh


def test_stratified_positions_cover_lists_proportionally():
    sizes = [0, 1, 7, 100, 1000, 3]
    pos = orc.stratified_positions(sizes, 111)
    assert [len(p) for p in pos] == [0, 1, 1, 10, 100, 1]          # round(111 * n_l / 1111), at least 1 when non-empty
    for n_l, p in zip(sizes, pos):
        assert np.all(np.diff(p) > 0) and (len(p) == 0 or (p[0] == 0 and p[-1] < n_l))
    np.testing.assert_array_equal(pos[3], np.arange(10) * 10)        # evenly spaced in storage order
    # asking for more than is stored takes everything once
    assert [len(p) for p in orc.stratified_positions([5, 0, 2], 1000)] == [5, 0, 2]


def test_refresh_recovers_a_stale_partition_without_raw_vectors():
    """Index built on centroids that ignore the data (random directions): the refresh re-clusters the
    reconstructions and re-encodes everything from them.  Labels survive as a permutation, the
    residuals shrink (E gamma^2 = 2(1 - E<x~, c~>)) and recall against the raw vectors' exact
    neighbours goes up; the rotation and the codebook are untouched."""
    w = synth.scaled(synth.config_tiny(), 6000, 60)
    X, Q = synth.database(w, 0, 6000), synth.queries(w, 60)
    d, L, b = w.d, 32, 4
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(0, d))
    c, tau = orc.lloyd_max_codebook(b, d)
    stale = synth.random_unit_vectors(3, L, d)
    idx = orc.ListIndex(stale, Pi, c, tau)
    labels = np.arange(6000, dtype=np.int64) * 7 + 3
    idx.add(X, labels)
    _, truth = orc.exact_topk(X, Q, 10)
    truth = labels[truth]
    _, ids0, _, _ = orc.search(idx, Q, 4, 10)
    rec0 = orc.recall_at_k(ids0, truth)
    g0 = np.mean(np.concatenate([g.astype(np.float64) ** 2 for g in idx.gamma16]))

    fresh, xh, lab, sample = orc.refresh_coarse(idx, 2000, 8, synth.kmeans_init_indices(0, 2000, L))
    assert fresh.Pi is idx.Pi and fresh.c is idx.c and fresh.tau is idx.tau
    assert 1990 <= len(sample) <= 2010 and xh.shape == (6000, d)
    np.testing.assert_array_equal(np.sort(np.concatenate([np.asarray(i) for i in fresh.ids])), np.sort(labels))
    np.testing.assert_array_equal(np.sort(lab), np.sort(labels))
    # reconstructions are close to the unit vectors they stand for
    Xn = orc.normalize_rows(X)
    err = np.linalg.norm(xh - Xn[(lab - 3) // 7], axis=1)
    assert np.mean(err ** 2) < 0.03
    g1 = np.mean(np.concatenate([g.astype(np.float64) ** 2 for g in fresh.gamma16 if len(g)]))
    _, ids1, _, _ = orc.search(fresh, Q, 4, 10)
    rec1 = orc.recall_at_k(ids1, truth)
    print(f"stale: recall {rec0:.3f}, E gamma^2 {g0:.3f}; refreshed: recall {rec1:.3f}, E gamma^2 {g1:.3f}")
    assert g1 < 0.5 * g0
    assert rec1 > rec0 + 0.15


def test_refresh_with_the_same_centroids_keeps_almost_every_assignment():
    w = synth.scaled(synth.config_tiny(), 3000, 10)
    X = synth.database(w, 0, 3000)
    C, _ = orc.train_coarse(X, 16, 5, synth.kmeans_init_indices(0, 3000, 16))
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(0, w.d))
    c, tau = orc.lloyd_max_codebook(4, w.d)
    idx = orc.ListIndex(C, Pi, c, tau)
    idx.add(X)
    fresh, _, _, _ = orc.refresh_coarse(idx, 500, 0, new_centroids=C)
    moved = sum(len(set(np.asarray(fresh.ids[l]).tolist()) - set(np.asarray(idx.ids[l]).tolist())) for l in range(16))
    assert moved < 0.03 * 3000


# ---------------------------------------------------------------- re-ranking on raw vectors


def test_rerank_is_exact_on_its_candidates_and_lifts_recall():
    w = synth.scaled(synth.config_tiny(), 5000, 50)
    X, Q = synth.database(w, 0, 5000), synth.queries(w, 50)
    C, _ = orc.train_coarse(X, 32, 5, synth.kmeans_init_indices(0, 5000, 32))
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(0, w.d))
    c, tau = orc.lloyd_max_codebook(2, w.d)                    # coarse codes: the estimate alone ranks poorly
    idx = orc.ListIndex(C, Pi, c, tau)
    idx.add(X)
    t_sc, truth = orc.exact_topk(X, Q, 10)
    # with every row as a candidate the re-rank is the exact search itself
    everything = np.tile(np.arange(5000), (3, 1))
    sc, ids = orc.rerank(X, Q[:3], everything, 10)
    np.testing.assert_array_equal(ids, truth[:3])
    np.testing.assert_allclose(sc, t_sc[:3], atol=1e-12)
    # top-50 by estimate, re-ranked: recall@10 cannot drop and here rises clearly
    _, ids10, _, _ = orc.search(idx, Q, 8, 10)
    _, ids50, _, _ = orc.search(idx, Q, 8, 50)
    r_sc, r_ids = orc.rerank(X, Q, ids50, 10)
    rec10, rec_rr = orc.recall_at_k(ids10, truth), orc.recall_at_k(r_ids, truth)
    print(f"recall@10: estimate {rec10:.3f}, top-50 re-ranked {rec_rr:.3f}")
    assert rec_rr > rec10 + 0.1
    # re-ranked scores are exact inner products of the returned rows, sorted, duplicates and -1 ignored
    Xn, Qn = orc.normalize_rows(X), orc.normalize_rows(Q)
    for qi in range(5):
        np.testing.assert_allclose(r_sc[qi], Xn[r_ids[qi]] @ Qn[qi], atol=1e-12)
        assert np.all(np.diff(r_sc[qi]) <= 0)
    dup = np.array([[7, 7, -1, 3, 3, 9]])
    s2, i2 = orc.rerank(X, Q[:1], dup, 4)
    assert sorted(i2[0][:3].tolist()) == [3, 7, 9] and i2[0][3] == -1 and np.isneginf(s2[0][3])


# ---------------------------------------------------------------- cascade (Appendix "Cascade search")


@pytest.mark.parametrize("b,d,beta", [(4, 32, 2), (5, 96, 4), (3, 16, 1)])
def test_coarsened_codebook_is_the_conditional_mean_of_the_merged_bins(b, d, beta):
    from scipy import integrate
    c, tau = orc.lloyd_max_codebook(b, d)
    cc = orc.coarsened_codebook(c, tau, d, beta)
    assert cc.shape == (1 << beta,) and np.all(np.diff(cc) > 0)
    np.testing.assert_allclose(cc, -cc[::-1], atol=1e-12)          # the density is even
    # straight from the definition: E[T | T in the union of the 2^(b-beta) bins], by adaptive quadrature
    # on the density formula itself (the oracle goes through per-bin masses and the level table)
    kappa = math.gamma(d / 2) / (math.sqrt(math.pi) * math.gamma((d - 1) / 2))
    f = lambda t: kappa * (1 - t * t) ** ((d - 3) / 2)
    edges = np.concatenate(([-1.0], tau, [1.0]))
    g = 1 << (b - beta)
    for i in range(1 << beta):
        lo, hi = edges[i * g], edges[(i + 1) * g]
        m0 = integrate.quad(f, lo, hi, epsabs=1e-14, epsrel=1e-12)[0]
        m1 = integrate.quad(lambda t: t * f(t), lo, hi, epsabs=1e-14, epsrel=1e-12)[0]
        assert abs(cc[i] - m1 / m0) < 1e-9
        # ordinality: a merged value lies between its outermost member levels
        assert c[i * g] <= cc[i] <= c[(i + 1) * g - 1]
    # all bits kept: nothing is merged
    np.testing.assert_allclose(orc.coarsened_codebook(c, tau, d, b), c, atol=1e-12)
    # one bit: the two half-line means +-E|T|, in closed form kappa / ((d-1)/2) ... = 2*kappa/(d-1)
    np.testing.assert_allclose(orc.coarsened_codebook(c, tau, d, 1), [-2 * kappa / (d - 1), 2 * kappa / (d - 1)], rtol=1e-9)


def test_cascade_reduces_to_the_plain_search_and_keeps_recall():
    w = synth.scaled(synth.config_tiny(), 6000, 60)
    X, Q = synth.database(w, 0, 6000), synth.queries(w, 60)
    C, _ = orc.train_coarse(X, 24, 5, synth.kmeans_init_indices(0, 6000, 24))
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(0, w.d))
    c, tau = orc.lloyd_max_codebook(4, w.d)
    idx = orc.ListIndex(C, Pi, c, tau)
    idx.add(X)
    base_sc, base_ids, _, _, everything = orc.search(idx, Q, 6, 10, return_all=True)
    # (i) pass 1 keeps everything: pass 2 alone decides, so the result is the plain search's
    sc, ids = orc.cascade_search(idx, Q, 6, 10, 2, 10 ** 6, orc.coarsened_codebook(c, tau, w.d, 2))
    np.testing.assert_array_equal(ids, base_ids)
    np.testing.assert_allclose(sc, base_sc, atol=1e-12)
    # (ii) all bits in pass 1: its ranking is the final one, any n_keep >= k gives the plain search
    sc, ids = orc.cascade_search(idx, Q, 6, 10, 4, 10, c)
    np.testing.assert_array_equal(ids, base_ids)
    # (iii) the kept set is the pass-1 top n_keep, and every returned score is the full-code score of its id
    cc = orc.coarsened_codebook(c, tau, w.d, 3)
    sc, ids, kept = orc.cascade_search(idx, Q, 6, 10, 3, 100, cc, return_kept=True)
    for qi in range(5):
        cid, s1, keep_ids = kept[qi]
        assert len(keep_ids) == min(100, len(cid))
        cut = np.sort(s1)[::-1][len(keep_ids) - 1]
        assert np.all(s1[np.isin(cid, keep_ids)] >= cut)
        full = dict(zip(everything[qi][0].tolist(), everything[qi][1].tolist()))
        for s, i in zip(sc[qi], ids[qi]):
            assert abs(full[int(i)] - s) < 1e-12 and int(i) in set(keep_ids.tolist())
    # (iv) the appendix's observation: top bits + 100 kept preserve recall@10 (there: 5+1 bits, beta 4, N 100)
    _, truth = orc.exact_topk(X, Q, 10)
    r_base, r_casc = orc.recall_at_k(base_ids, truth), orc.recall_at_k(ids, truth)
    print(f"recall@10 plain {r_base:.4f}, cascade beta=3 N=100 {r_casc:.4f}")
    assert abs(r_casc - r_base) <= 0.01
    # and a pass 1 that is too coarse with too few kept does lose recall (the pin is not vacuous)
    _, ids_bad = orc.cascade_search(idx, Q, 6, 10, 1, 10, orc.coarsened_codebook(c, tau, w.d, 1))
    assert orc.recall_at_k(ids_bad, truth) < r_base - 0.02


def test_cascade_on_the_refined_table_uses_primary_bits():
    """With the sign bit stored, the merged (b+1)-bit code's top beta bits are the primary's top beta bits."""
    b, d = 3, 24
    c, tau = orc.lloyd_max_codebook(b, d)
    levels, bnd = orc.refined_tables(c, tau, d)
    for beta in (1, 2, 3):
        np.testing.assert_allclose(orc.coarsened_codebook(levels, bnd, d, beta),
                                   orc.coarsened_codebook(c, tau, d, beta), atol=1e-12)
