"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

import gpu_cases
import parity
from oracle import ivftq_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _pkg():
    import paper_2605_17415_amd as pkg
    return pkg


def _dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch.device("cuda:0")


def _make_index(cs):
    ix = _pkg().Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit)
    ix.set_coarse(cs.cent)
    ix.set_rotation(cs.Pi)
    # the library's own (b, d) codebook must be the oracle's, bit for bit: both sides quantise against
    # the same float32 boundaries and reconstruct from the same float32 levels
    c, tau = ix.get_codebook()
    np.testing.assert_array_equal(c, cs.c.astype(np.float32))
    np.testing.assert_array_equal(tau, cs.tau.astype(np.float32))
    return ix


@pytest.mark.parametrize("name", gpu_cases.ALL_CASES)
def test_encode_matches_oracle(name):
    cs = gpu_cases.get_case(name)
    enc = gpu_cases.oracle_encode(name)
    print(f"[case {name}] n={len(cs.X)} d={cs.d} L={cs.nlist} b={cs.b}", flush=True)
    ix = _make_index(cs)
    x = torch.from_numpy(cs.X).to(_dev())
    assign, codes, gamma = ix.encode_only(x)
    torch.cuda.synchronize()
    rep = parity.compare_encode(enc, assign.cpu().numpy(), codes.cpu().numpy(), gamma.cpu().numpy())
    print("encode_only:", rep, flush=True)
    assert rep["code_near_boundary_mismatch"] <= rep["code_near_boundary_total"]

    # the stored index holds the same thing, list by list, in arrival order
    ix.encode_add(x)
    assert ix.ntotal() == len(cs.X)
    ga, gc, gg = assign.cpu().numpy(), codes.cpu().numpy(), gamma.cpu().numpy()
    total = 0
    for l in range(cs.nlist):
        ids, lc, lg = ix.export_list(l)
        members = np.flatnonzero(ga == l)
        np.testing.assert_array_equal(ids, members)              # stable: arrival order, default labels
        np.testing.assert_array_equal(lc, gc[members])
        np.testing.assert_array_equal(lg.view(np.uint16), gg[members].view(np.uint16))
        total += len(ids)
    assert total == len(cs.X)
    ix.close()


BATCHED_CASES = ["tiny", "d128", "d96_b2", "d96_b3", "d96_b4", "d200", "d96_b3s", "d128_b4s", "d100_b5"]    # shapes the batched scan covers
SEARCH_CASES = [(n, 1) for n in gpu_cases.ALL_CASES] + [(n, 2) for n in BATCHED_CASES]


@pytest.mark.parametrize("name,mode", SEARCH_CASES)
def test_search_matches_oracle_on_the_same_codes(name, mode):
    """mode 1: streaming scan; mode 2: query-batched matrix-core scan."""
    cs = gpu_cases.get_case(name)
    enc = gpu_cases.oracle_encode(name)
    oidx = gpu_cases.oracle_index(name)
    print(f"[case {name}] mode={mode} nq={len(cs.Q)} nprobe={cs.nprobe} k={cs.k}", flush=True)
    dev = _dev()
    ix = _make_index(cs)
    ix.set_search_mode(mode)
    ix.add_encoded(torch.from_numpy(enc["assign"]).to(dev), torch.from_numpy(enc["codes"]).to(dev),
                   torch.from_numpy(enc["gamma16"]).to(dev))
    for l in range(0, cs.nlist, max(1, cs.nlist // 7)):          # storage round trip
        ids, lc, lg = ix.export_list(l)
        np.testing.assert_array_equal(ids, oidx.ids[l])
        np.testing.assert_array_equal(lc, oidx.codes[l])
        np.testing.assert_array_equal(lg.view(np.uint16), oidx.gamma16[l].view(np.uint16))

    q = torch.from_numpy(cs.Q).to(dev)
    o_sc, o_ids, o_probe, S, o_all = orc.search(oidx, cs.Q, cs.nprobe, cs.k, return_all=True)
    gap = parity.probe_cut_gap(S, cs.nprobe)

    probe, coarse = ix.coarse_probe(q, cs.nprobe)
    torch.cuda.synchronize()
    probe, coarse = probe.cpu().numpy(), coarse.cpu().numpy()
    rows = np.arange(len(cs.Q))[:, None]
    np.testing.assert_allclose(coarse, S[rows, probe], rtol=1e-5, atol=1e-6)   # exact coarse term
    assert np.all(np.diff(coarse, axis=1) <= 0)
    for qi in range(len(cs.Q)):
        if not np.array_equal(probe[qi], o_probe[qi]):
            ordered = np.sort(S[qi])[::-1]
            close = np.min(np.abs(np.diff(ordered[:cs.nprobe + 1]))) < parity.BOUNDARY_TOL
            assert close and set(probe[qi]) ^ set(o_probe[qi]) <= set(np.argsort(-S[qi])[:cs.nprobe + 1]), \
                f"query {qi}: probe list differs from the oracle's away from a near-tie"

    scores, ids = ix.search(q, cs.nprobe, cs.k)
    torch.cuda.synchronize()
    rep = parity.compare_search(scores.cpu().numpy(), ids.cpu().numpy(), o_sc, o_ids, o_all, gap)
    print("search:", rep, flush=True)
    assert rep["probe_near_tie_excused"] <= max(1, len(cs.Q) // 20)
    ix.close()


def test_batched_scan_overflow_falls_back_to_the_exact_scan():
    """More candidates beat the nearest list's k-th score than the per-query candidate list holds:
    the query must be redone by the streaming scan and still match the oracle."""
    cs = gpu_cases.get_case("tiny")
    dev = _dev()
    K = 1 << cs.b
    qn = orc.normalize_rows(cs.Q[:3])
    S = qn @ cs.cent.astype(np.float64).T
    z = qn @ cs.Pi.astype(np.float64).T
    order = np.argsort(-S[0])
    rng = np.random.default_rng(0)
    assign, codes, gamma = [], [], []
    # the two nearest cells of query 0 (the prefix its threshold comes from): 20 and 100 vectors whose
    # residual estimate is as negative as it can be
    worst = np.where(z[0] > 0, 0, K - 1).astype(np.uint8)
    for l, count in ((order[0], 20), (order[1], 100)):
        for _ in range(count):
            assign.append(l); codes.append(worst); gamma.append(1.0)
    # next cells: 300 vectors each with zero residual norm, so every score equals the coarse term
    for l in order[2:8]:
        for _ in range(300):
            assign.append(l); codes.append(rng.integers(0, K, cs.d).astype(np.uint8)); gamma.append(0.0)
    assign = np.array(assign, np.int32)
    codes = np.stack(codes)
    gamma = np.array(gamma, np.float16)
    ref = orc.ListIndex(cs.cent, cs.Pi, cs.c, cs.tau)
    ref.add_encoded(assign, np.arange(len(assign), dtype=np.int64), codes, gamma)
    o_sc, o_ids, _, S_all, o_all = orc.search(ref, cs.Q[:3], 8, 10, return_all=True)
    for mode in (1, 2):
        ix = _make_index(cs)
        ix.set_search_mode(mode)
        ix.add_encoded(torch.from_numpy(assign).to(dev), torch.from_numpy(codes).to(dev), torch.from_numpy(gamma).to(dev))
        sc, ids = ix.search(torch.from_numpy(cs.Q[:3]).to(dev), 8, 10)
        torch.cuda.synchronize()
        rep = parity.compare_search(sc.cpu().numpy(), ids.cpu().numpy(), o_sc, o_ids, o_all,
                                    parity.probe_cut_gap(S_all, 8))
        print(f"mode {mode}:", rep, flush=True)
        ix.close()


def test_many_overflowing_queries_take_turns_in_the_full_length_rows():
    """Under a small workspace limit the batched path keeps short score rows (dense prefix) for all queries of
    a pass and only a few full-length rows for the queries it has to redo exactly: nine queries overflow here
    and three rows are available, so the exact pass runs in several turns.  Every query must match the oracle."""
    cs = gpu_cases.get_case("tiny")
    dev = _dev()
    K = 1 << cs.b
    Q = np.concatenate([np.repeat(cs.Q[:1], 9, axis=0), cs.Q[1:4]]).astype(np.float32)
    Q[1:9] *= np.linspace(0.5, 3.0, 8, dtype=np.float32)[:, None]     # same direction: same answer after normalising
    qn = orc.normalize_rows(Q[:1])
    S = qn @ cs.cent.astype(np.float64).T
    z = qn @ cs.Pi.astype(np.float64).T
    order = np.argsort(-S[0])
    rng = np.random.default_rng(1)
    worst = np.where(z[0] > 0, 0, K - 1).astype(np.uint8)
    assign = [np.full(20, order[0]), np.full(100, order[1])]
    codes = [np.tile(worst, (120, 1))]
    gamma = [np.ones(120)]
    per_list = 12000                       # zero residual norm: every score equals the coarse term
    for l in order[2:8]:
        assign.append(np.full(per_list, l))
        codes.append(rng.integers(0, K, (per_list, cs.d)).astype(np.uint8))
        gamma.append(np.zeros(per_list))
    assign = np.concatenate(assign).astype(np.int32)
    codes = np.concatenate(codes)
    gamma = np.concatenate(gamma).astype(np.float16)
    ref = orc.ListIndex(cs.cent, cs.Pi, cs.c, cs.tau)
    ref.add_encoded(assign, np.arange(len(assign), dtype=np.int64), codes, gamma)
    o_sc, o_ids, _, S_all, o_all = orc.search(ref, Q, 8, 10, return_all=True)
    ix = _make_index(cs)
    ix.set_search_mode(2)                  # the batched scan, although the call brings only twelve queries
    ix.add_encoded(torch.from_numpy(assign).to(dev), torch.from_numpy(codes).to(dev), torch.from_numpy(gamma).to(dev))
    ix.set_workspace_limit(1 << 20)        # 3 rows of 8 lists' length, 12 queries in one pass
    print("[turns] search", flush=True)
    sc, ids = ix.search(torch.from_numpy(Q).to(dev), 8, 10)
    torch.cuda.synchronize()
    rep = parity.compare_search(sc.cpu().numpy(), ids.cpu().numpy(), o_sc, o_ids, o_all, parity.probe_cut_gap(S_all, 8))
    print("turns:", rep, flush=True)
    ix.set_workspace_limit(1 << 32)        # one turn: same bits
    sc2, ids2 = ix.search(torch.from_numpy(Q).to(dev), 8, 10)
    torch.cuda.synchronize()
    assert torch.equal(sc, sc2) and torch.equal(ids, ids2)
    ix.close()


@pytest.mark.parametrize("name", ["d128", "d96_b3"])
def test_batched_scan_with_duplicated_vectors_ranks_ties_by_label(name):
    """Every stored vector three times under different labels: the batched scan's threshold pass works
    on upper bounds and the merge re-scores what may still matter, so equal scores must come out as one
    run in ascending label order and the label set must be the oracle's."""
    cs = gpu_cases.get_case(name)
    enc = gpu_cases.oracle_encode(name)
    dev = _dev()
    n = len(cs.X)
    ref = orc.ListIndex(cs.cent, cs.Pi, cs.c, cs.tau)
    ix = _make_index(cs)
    ix.set_search_mode(2)
    for rep in range(3):
        labels = np.arange(n, dtype=np.int64) * 3 + (2 - rep)          # later copies get the smaller labels
        ref.add_encoded(enc["assign"], labels, enc["codes"], enc["gamma16"])
        ix.add_encoded(torch.from_numpy(enc["assign"]).to(dev), torch.from_numpy(enc["codes"]).to(dev),
                       torch.from_numpy(enc["gamma16"]).to(dev), torch.from_numpy(labels).to(dev))
    k = 12
    o_sc, o_ids, _, S, o_all = orc.search(ref, cs.Q, cs.nprobe, k, return_all=True)
    sc, ids = ix.search(torch.from_numpy(cs.Q).to(dev), cs.nprobe, k)
    torch.cuda.synchronize()
    g_sc, g_ids = sc.cpu().numpy(), ids.cpu().numpy()
    rep = parity.compare_search(g_sc, g_ids, o_sc, o_ids, o_all, parity.probe_cut_gap(S, cs.nprobe))
    print("duplicates:", rep, flush=True)
    for qi in range(len(cs.Q)):
        for i in range(k - 1):
            if g_sc[qi, i] == g_sc[qi, i + 1]:
                assert g_ids[qi, i] < g_ids[qi, i + 1], f"query {qi}: equal scores not in label order"
        # the three copies of a vector score identically, so whole triples appear (except at the cut)
        full = g_ids[qi][: (k // 3) * 3] // 3
        assert np.all(full.reshape(-1, 3) == full.reshape(-1, 3)[:, :1]) or rep["tie_swaps"] > 0
    ix.close()


def test_end_to_end_recall_matches_oracle_pipeline():
    """GPU encode + GPU search against oracle encode + oracle search and exact ground truth."""
    cs = gpu_cases.get_case("tiny")
    oidx = gpu_cases.oracle_index("tiny")
    dev = _dev()
    ix = _make_index(cs)
    ix.encode_add(torch.from_numpy(cs.X).to(dev))
    scores, ids = ix.search(torch.from_numpy(cs.Q).to(dev), cs.nprobe, cs.k)
    torch.cuda.synchronize()
    _, gt = orc.exact_topk(cs.X, cs.Q, cs.k)
    _, o_ids, _, _ = orc.search(oidx, cs.Q, cs.nprobe, cs.k)
    r_gpu = orc.recall_at_k(ids.cpu().numpy(), gt)
    r_orc = orc.recall_at_k(o_ids, gt)
    print(f"recall@10 gpu={r_gpu:.4f} oracle={r_orc:.4f}", flush=True)
    assert abs(r_gpu - r_orc) <= 0.005
    overlap = np.mean([len(set(a) & set(b)) / cs.k for a, b in zip(ids.cpu().numpy(), o_ids)])
    assert overlap > 0.995
    ix.close()
