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


def _index(cs, mode):
    import paper_2605_17415_amd as pkg
    enc = gpu_cases.oracle_encode(cs.name)
    ix = pkg.Index(cs.d, cs.b_stage1, cs.nlist, sign_bit=cs.sign_bit)
    ix.set_coarse(cs.cent)
    ix.set_rotation(cs.Pi)
    ix.set_search_mode(mode)
    dev = torch.device("cuda:0")
    ix.add_encoded(torch.from_numpy(enc["assign"]).to(dev), torch.from_numpy(enc["codes"]).to(dev),
                   torch.from_numpy(enc["gamma16"]).to(dev))
    return ix


CASES = [("tiny", 1, 2, 40), ("d128", 1, 3, 100), ("d128", 2, 2, 100), ("d96_b3s", 1, 2, 64),
         ("d128_b4s", 2, 3, 100), ("d100_b5", 1, 4, 100), ("d200", 2, 1, 30)]


@pytest.mark.parametrize("name,mode,beta,n_keep", CASES)
def test_cascade_matches_oracle_on_the_same_codes(name, mode, beta, n_keep):
    import paper_2605_17415_amd as pkg
    cs = gpu_cases.get_case(name)
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

    ix = _index(cs, mode)
    q = torch.from_numpy(cs.Q).to("cuda:0")
    scores, ids = ix.search_cascade(q, cs.nprobe, k, beta, n_keep)
    torch.cuda.synchronize()
    g_sc, g_ids = scores.cpu().numpy(), ids.cpu().numpy()

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
