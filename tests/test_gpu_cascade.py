"""GPU: the two-pass cascade search (Appendix "Cascade search via Lloyd-Max bin ordinality") through the
C ABI against the oracle's cascade on the same stored codes.

What is unique is compared exactly: returned scores are the full-code scores of their labels, and the
label set is the oracle's, up to ties at the k-th full score.  Where a query's pass-1 cut is itself a
near-tie (the n_keep-th and the next pass-1 score closer than 1e-5, the decision-boundary rule of the
other comparisons) either side may be kept;
such queries are only checked for valid scores and are counted.
"""
import numpy as np
import pytest

import gpu_cases
import parity
from oracle import ivftq_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _index(cs, mode, plane_beta=0):
    import paper_2605_17415_amd as pkg
    enc = gpu_cases.oracle_encode(cs.name)
    ix = pkg.Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit)
    ix.set_coarse(cs.cent)
    ix.set_rotation(cs.Pi)
    ix.set_search_mode(mode)
    ix.set_cascade_plane(plane_beta)
    dev = torch.device("cuda:0")
    ix.add_encoded(torch.from_numpy(enc["assign"]).to(dev), torch.from_numpy(enc["codes"]).to(dev),
                   torch.from_numpy(enc["gamma16"]).to(dev))
    return ix


CASES = [("tiny", 1, 2, 40), ("d128", 1, 3, 100), ("d128", 2, 2, 100), ("d96_b3s", 1, 2, 64),
         ("d128_b4s", 2, 3, 100), ("d100_b5", 1, 4, 100), ("d200", 2, 1, 30)]


@pytest.mark.parametrize("plane", [False, True])
@pytest.mark.parametrize("name,mode,beta,n_keep", CASES)
def test_cascade_matches_oracle_on_the_same_codes(name, mode, beta, n_keep, plane):
    """plane: the index keeps the top beta bits of every code in a plane of their own and pass 1 reads that."""
    import paper_2605_17415_amd as pkg
    cs = gpu_cases.get_case(name)
    if plane and beta >= cs.b:
        pytest.skip("a plane of all stored bits would be the codes themselves")
    oidx = gpu_cases.oracle_index(name)
    k = min(cs.k, n_keep)
    print(f"[cascade {name}] mode={mode} beta={beta} n_keep={n_keep} k={k} nq={len(cs.Q)}", flush=True)
    # the library's coarsened table against the oracle's
    c1, tau1 = orc.lloyd_max_codebook(cs.b_stage1, cs.d)
    cc = orc.coarsened_codebook(c1, tau1, cs.d, beta)
    np.testing.assert_allclose(pkg.ivftq_build_coarsened_codebook(cs.b_stage1, cs.d, beta, cs.sign_bit), cc,
                               rtol=0, atol=3e-8)
    o_sc, o_ids, kept = orc.cascade_search(oidx, cs.Q, cs.nprobe, k, beta, n_keep, cc, return_kept=True)
    _, _, _, S, o_all = orc.search(oidx, cs.Q, cs.nprobe, k, return_all=True)
    gap = parity.probe_cut_gap(S, cs.nprobe)

    ix = _index(cs, mode, beta if plane else 0)
    q = torch.from_numpy(cs.Q).to("cuda:0")
    scores, ids = ix.search_cascade(q, cs.nprobe, k, beta, n_keep)
    torch.cuda.synchronize()
    g_sc, g_ids = scores.cpu().numpy(), ids.cpu().numpy()
    if plane:
        # the plane holds the top beta bits of the stored codes, and reading it changes nothing in the result
        for l in (0, cs.nlist // 2, cs.nlist - 1):
            np.testing.assert_array_equal(ix.export_cascade_plane(l), ix.export_list(l)[1] >> (cs.b - beta))
        flat = _index(cs, mode, 0)
        f_sc, f_ids = flat.search_cascade(q, cs.nprobe, k, beta, n_keep)
        torch.cuda.synchronize()
        assert torch.equal(f_ids, ids) and torch.equal(f_sc, scores)
        assert ix.index_bytes() == flat.index_bytes() + len(cs.X) * 4 * ((beta * cs.d + 31) // 32)
        flat.close()

    strict, loose = [], []
    for qi in range(len(cs.Q)):
        cid, s1, keep_ids = kept[qi]
        if len(cid) > len(keep_ids):
            order = np.sort(s1)[::-1]
            cut_gap = order[len(keep_ids) - 1] - order[len(keep_ids)]
            (loose if cut_gap < parity.BOUNDARY_TOL else strict).append(qi)
        else:
            strict.append(qi)
    # strict queries: the oracle's kept set is the only valid one; compare like any search over those candidates
    full = [dict(zip(o_all[qi][0].tolist(), o_all[qi][1].tolist())) for qi in range(len(cs.Q))]
    sub_all = []
    for qi in strict:
        keep_ids = kept[qi][2]
        sub_all.append((keep_ids, np.array([full[qi][int(i)] for i in keep_ids])))
    if strict:
        rep = parity.compare_search(g_sc[strict], g_ids[strict], o_sc[strict], o_ids[strict], sub_all, gap[strict])
        print("cascade:", rep, "loose queries:", len(loose), flush=True)
        assert rep["probe_near_tie_excused"] <= max(1, len(cs.Q) // 20)
    # loose queries: every returned label is a candidate and carries its full-code score, in order
    for qi in loose:
        real = g_ids[qi] >= 0
        assert np.all(np.diff(g_sc[qi][real]) <= 0)
        for lab, sc in zip(g_ids[qi][real].tolist(), g_sc[qi][real].tolist()):
            if lab in full[qi]:
                assert abs(sc - full[qi][lab]) <= parity.SCORE_RTOL * abs(full[qi][lab]) + parity.SCORE_ATOL
            else:
                assert gap[qi] < parity.BOUNDARY_TOL
    assert len(loose) <= max(2, len(cs.Q) // 10)

    # reductions: everything kept, or every Stage-1 bit used in pass 1 -> the plain search
    p_sc, p_ids = ix.search(q, cs.nprobe, k)
    a_sc, a_ids = ix.search_cascade(q, cs.nprobe, k, cs.b_stage1, max(k, 16))
    torch.cuda.synchronize()
    if not cs.sign_bit:        # with a sign bit, pass 1 on all Stage-1 bits is still coarser than the stored code
        rep2 = parity.compare_search(a_sc.cpu().numpy(), a_ids.cpu().numpy(), p_sc.cpu().numpy().astype(np.float64),
                                     p_ids.cpu().numpy(), o_all, gap)
        print("cascade with all bits vs plain search:", rep2, flush=True)
    ix.close()


def test_cascade_argument_checks():
    import paper_2605_17415_amd as pkg
    cs = gpu_cases.get_case("tiny")
    ix = _index(cs, 1)
    q = torch.from_numpy(cs.Q).to("cuda:0")
    for kwargs in (dict(k=5, beta=0, n_keep=10), dict(k=5, beta=cs.b_stage1 + 1, n_keep=10),
                   dict(k=11, beta=1, n_keep=10), dict(k=5, beta=1, n_keep=4096)):
        with pytest.raises(pkg.IvftqError):
            ix.search_cascade(q, cs.nprobe, **kwargs)
    # an empty index returns padding
    ix.reset()
    sc, ids = ix.search_cascade(q, cs.nprobe, 5, 1, 10)
    torch.cuda.synchronize()
    assert torch.all(ids == -1) and torch.all(torch.isinf(sc))
    ix.close()


@pytest.mark.parametrize("name,beta", [("d96_b4", 3), ("d128", 2), ("d96_b3s", 3), ("d70_b6", 4), ("d200", 1)])
def test_plane_written_by_encode_add_and_kept_through_growth(name, beta):
    """The encode kernel fills the plane itself: after several appends (the pool grows and is copied) the
    plane still is the top beta bits of the stored codes, list by list, and the plain search ignores it."""
    import paper_2605_17415_amd as pkg
    cs = gpu_cases.get_case(name)
    dev = torch.device("cuda:0")
    x = torch.from_numpy(cs.X).to(dev)
    q = torch.from_numpy(cs.Q).to(dev)
    with_plane = pkg.Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit)
    plain = pkg.Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit)
    for ix in (with_plane, plain):
        ix.set_coarse(cs.cent)
        ix.set_rotation(cs.Pi)
    with_plane.set_cascade_plane(beta)
    cuts = [0, 1, 700, 5000, len(cs.X)]
    for a, b in zip(cuts[:-1], cuts[1:]):
        with_plane.encode_add(x[a:b])
    plain.encode_add(x)
    for l in range(cs.nlist):
        ids, codes, gamma = with_plane.export_list(l)
        ids0, codes0, gamma0 = plain.export_list(l)
        np.testing.assert_array_equal(ids, ids0)
        np.testing.assert_array_equal(codes, codes0)
        np.testing.assert_array_equal(with_plane.export_cascade_plane(l), codes >> (cs.b - beta))
    s1, i1 = with_plane.search(q, cs.nprobe, cs.k)
    s0, i0 = plain.search(q, cs.nprobe, cs.k)
    c1 = with_plane.search_cascade(q, cs.nprobe, cs.k, beta, 4 * cs.k)
    c0 = plain.search_cascade(q, cs.nprobe, cs.k, beta, 4 * cs.k)
    torch.cuda.synchronize()
    assert torch.equal(i1, i0) and torch.equal(s1, s0)
    assert torch.equal(c1[1], c0[1]) and torch.equal(c1[0], c0[0])
    # layout changes are refused once vectors are stored; bad widths always
    with pytest.raises(pkg.IvftqError) as e:
        with_plane.set_cascade_plane(0)
    assert e.value.status == pkg.binding.BAD_STATE
    empty = pkg.Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit)
    for bad in (-1, cs.b_stage1 + 1, cs.b):
        with pytest.raises(pkg.IvftqError):
            empty.set_cascade_plane(bad)
    with pytest.raises(pkg.IvftqError):
        plain.export_cascade_plane(0)
    for ix in (with_plane, plain, empty):
        ix.close()
