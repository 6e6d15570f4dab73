"""Parity at the benchmark's full size (1M x 128, nlist 1024, b=4, 10,000 queries, nprobe 32, k 10),
in the launch configuration bench.py times, on outputs the oracle can compute one by one:
sampled rows of the encode, every returned (label, score) of sampled queries, and the complete
result of a few queries whose probed lists the oracle encodes itself."""
import numpy as np
import pytest

import parity
from oracle import ivftq_oracle as orc
from workloads import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

NPROBE, K = 32, 10


@pytest.fixture(scope="module")
def full():
    import paper_2605_17415_amd as pkg
    w = synth.config_1m()
    print("[fullsize] generating 1M x 128", flush=True)
    X, Q = synth.database(w), synth.queries(w)
    rows = synth.train_sample_indices(w)
    print("[fullsize] oracle k-means (3 iterations on the 100k sample)", flush=True)
    cent, _ = orc.train_coarse(X[rows], w.nlist, 3, synth.kmeans_init_indices(w.seed, len(rows), w.nlist))
    cent = cent.astype(np.float32)
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(w.seed, w.d)).astype(np.float32)
    c, tau = orc.codebook_fp32(w.b, w.d)
    print("[fullsize] oracle coarse assignment of every row", flush=True)
    C64 = cent.astype(np.float64)
    o_assign = np.empty(w.n, np.int32)
    o_gap = np.empty(w.n)
    for s in range(0, w.n, 1 << 16):
        sc = orc.normalize_rows(X[s:s + (1 << 16)]) @ C64.T
        a = np.argmax(sc, axis=1)
        top2 = np.partition(sc, -2, axis=1)[:, -2:]
        o_assign[s:s + len(a)] = a
        o_gap[s:s + len(a)] = top2[:, 1] - top2[:, 0]
    ix = pkg.Index(w.d, w.b, w.nlist)
    ix.set_coarse(cent)
    ix.set_rotation(Pi)
    dev = torch.device("cuda:0")
    xd = torch.from_numpy(X).to(dev)
    print("[fullsize] GPU encode_add of 1M rows and search of 10k queries", flush=True)
    ix.encode_add(xd)
    scores, ids = ix.search(torch.from_numpy(Q).to(dev), NPROBE, K)
    g_assign, _, _ = ix.encode_only(xd, want_codes=False)
    torch.cuda.synchronize()
    yield dict(g_assign=g_assign.cpu().numpy(), w=w, X=X, Q=Q, cent=cent, Pi=Pi, c=c, tau=tau, o_assign=o_assign, o_gap=o_gap, ix=ix, xd=xd,
               scores=scores.cpu().numpy(), ids=ids.cpu().numpy())
    ix.close()


def test_fullsize_encode_sampled_rows(full):
    w, ix = full["w"], full["ix"]
    assign, codes, gamma = ix.encode_only(full["xd"])
    torch.cuda.synchronize()
    g_assign = assign.cpu().numpy()
    # every assignment against the oracle's
    bad = np.flatnonzero(g_assign != full["o_assign"])
    assert np.all(full["o_gap"][bad] < parity.BOUNDARY_TOL), "assignment differs away from a near-tie"
    print(f"assignments: {len(bad)} near-tie differences of {w.n}; "
          f"{int(np.sum(full['o_gap'] < parity.BOUNDARY_TOL))} near-ties in all", flush=True)
    # sampled rows, including the last partial tile: full encode against the oracle
    rng = np.random.default_rng(1)
    sample = np.unique(np.concatenate([rng.choice(w.n, 4000, replace=False), np.arange(w.n - 70, w.n), np.arange(200)]))
    enc = orc.encode(full["X"][sample], full["cent"], full["Pi"], full["tau"])
    rep = parity.compare_encode(enc, g_assign[sample], codes[torch.from_numpy(sample).to(codes.device)].cpu().numpy(),
                                gamma[torch.from_numpy(sample).to(gamma.device)].cpu().numpy())
    print("sampled encode:", rep, flush=True)
    # the stored lists hold exactly the rows assigned to them, in arrival order
    sizes = np.array([ix.list_size(l) for l in range(w.nlist)])
    np.testing.assert_array_equal(sizes, np.bincount(g_assign, minlength=w.nlist))
    for l in (0, 517, w.nlist - 1):
        ids_l, codes_l, gam_l = ix.export_list(l)
        members = np.flatnonzero(g_assign == l)
        np.testing.assert_array_equal(ids_l, members)
        sel = torch.from_numpy(members).to(codes.device)
        np.testing.assert_array_equal(codes_l, codes[sel].cpu().numpy())
        np.testing.assert_array_equal(gam_l.view(np.uint16), gamma[sel].cpu().numpy().view(np.uint16))


def _oracle_score(full, q_row, label):
    """Estimated inner product of one stored vector for one query, from the oracle's own encode."""
    enc = orc.encode(full["X"][label:label + 1], full["cent"], full["Pi"], full["tau"])
    qn = orc.normalize_rows(full["Q"][q_row:q_row + 1])[0]
    z = full["Pi"].astype(np.float64) @ qn
    l = enc["assign"][0]
    s_l = float(qn @ full["cent"][l].astype(np.float64))
    dot = float(np.sum(z * full["c"].astype(np.float64)[enc["codes"][0]]))
    return s_l + float(enc["gamma16"][0]) * dot, enc


def test_fullsize_returned_scores_one_by_one(full):
    rng = np.random.default_rng(2)
    checked = near = 0
    for q_row in rng.choice(full["w"].nq, 40, replace=False):
        assert np.all(np.diff(full["scores"][q_row]) <= 0)
        assert len(set(full["ids"][q_row].tolist())) == K
        for lab, sc in zip(full["ids"][q_row], full["scores"][q_row]):
            ref, enc = _oracle_score(full, q_row, int(lab))
            if enc["bdist"].min() < parity.BOUNDARY_TOL or enc["gap"][0] < parity.BOUNDARY_TOL:
                near += 1          # a code of this vector sits on a decision boundary: may differ by one bin
                continue
            assert abs(sc - ref) <= parity.SCORE_RTOL * abs(ref) + parity.SCORE_ATOL, (q_row, lab, sc, ref)
            checked += 1
    print(f"returned scores checked one by one: {checked}, skipped near a boundary: {near}", flush=True)
    assert checked > 300


def test_fullsize_complete_results_of_sampled_queries(full):
    """For a few queries the oracle encodes every vector of the probed lists itself and searches them."""
    w = full["w"]
    qsel = [3, 4242, 9999, 17, 2500, 7001, 123, 8888, 5555, 64]
    Qs = full["Q"][qsel]
    S = orc.normalize_rows(Qs) @ full["cent"].astype(np.float64).T
    gap = parity.probe_cut_gap(S, NPROBE)
    probes = np.argsort(-S, axis=1, kind="stable")[:, :NPROBE]
    lists = np.unique(probes)
    members = np.flatnonzero(np.isin(full["o_assign"], lists))
    print(f"[fullsize] oracle encodes {len(members)} vectors of {len(lists)} lists", flush=True)
    enc = orc.encode(full["X"][members], full["cent"], full["Pi"], full["tau"])
    ref = orc.ListIndex(full["cent"], full["Pi"], full["c"], full["tau"])
    ref.add_encoded(enc["assign"], members.astype(np.int64), enc["codes"], enc["gamma16"])
    o_sc, o_ids, _, _, o_all = orc.search(ref, Qs, NPROBE, K, return_all=True)
    # vectors whose code or cell may legitimately differ between the two encodes
    shaky = set(members[(enc["bdist"].min(axis=1) < parity.BOUNDARY_TOL) | (enc["gap"] < parity.BOUNDARY_TOL)].tolist())
    shaky |= set(np.flatnonzero(full["g_assign"] != full["o_assign"]).tolist())   # near-tie cells (checked elsewhere)
    strict = 0
    for i, q_row in enumerate(qsel):
        g_ids, g_sc = full["ids"][q_row], full["scores"][q_row]
        if not ((set(g_ids.tolist()) | set(o_ids[i].tolist())) & shaky):
            rep = parity.compare_search(full["scores"][q_row:q_row + 1], full["ids"][q_row:q_row + 1], o_sc[i:i + 1],
                                        o_ids[i:i + 1], o_all[i:i + 1], gap[i:i + 1])
            print(f"query {q_row}:", rep, flush=True)
            strict += 1
            continue
        # a vector with a code on a decision boundary is among the results: its score may differ by one
        # bin's worth, so it is left out and everything else is held to the usual rules
        lookup = dict(zip(o_all[i][0].tolist(), o_all[i][1].tolist()))
        kth_o, kth_g = o_sc[i, K - 1], g_sc[K - 1]
        tol = 2 * (parity.SCORE_RTOL * abs(kth_o) + parity.SCORE_ATOL)
        for lab, sc in zip(g_ids.tolist(), g_sc.tolist()):
            if lab in shaky:
                continue
            assert abs(sc - lookup[lab]) <= parity.SCORE_RTOL * abs(lookup[lab]) + parity.SCORE_ATOL
        for lab in o_ids[i].tolist():
            if lab not in shaky and lab not in set(g_ids.tolist()):
                assert lookup[lab] <= kth_g + tol, f"query {q_row}: oracle result {lab} missing"
        print(f"query {q_row}: compared without its boundary vectors", flush=True)
    assert strict >= 2
