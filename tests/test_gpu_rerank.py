"""Re-ranking on raw vectors through the C ABI against the oracle.  The candidate lists given to both
sides come from the oracle's own search (nothing the HIP path produced is an oracle input)."""
import numpy as np
import pytest

import gpu_cases
import parity
from oracle import ivftq_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("name,r,k", [("tiny", 50, 10), ("d96_b2", 64, 10), ("d200", 100, 20), ("d70_b6", 7, 3)])
def test_rerank_matches_oracle(name, r, k):
    import paper_2605_17415_amd as pkg
    cs = gpu_cases.get_case(name)
    ref = gpu_cases.oracle_index(name)
    _, cand, _, _ = orc.search(ref, cs.Q, cs.nprobe, r)              # -1 padded where fewer than r exist
    cand = cand.copy()
    cand[0, :3] = cand[0, 3]                                          # repeats count once
    cand[1, 0] = len(cs.X) + 5                                        # a label outside the matrix is skipped
    cand[2, :] = -1                                                   # no candidate at all
    o_sc, o_ids = orc.rerank(cs.X, cs.Q, np.where(cand < len(cs.X), cand, -1), k)
    g_sc, g_ids = pkg.ivftq_rerank(torch.from_numpy(cs.Q).to(DEV), torch.from_numpy(cs.X).to(DEV),
                                   torch.from_numpy(cand).to(DEV), k)
    torch.cuda.synchronize()
    g_sc, g_ids = g_sc.cpu().numpy(), g_ids.cpu().numpy()
    assert np.all(g_ids[2] == -1) and np.all(np.isneginf(g_sc[2]))
    swaps = 0
    for q in range(len(cs.Q)):
        real = o_ids[q] >= 0
        assert np.array_equal(g_ids[q] >= 0, real), f"query {q}: different number of results"
        np.testing.assert_allclose(g_sc[q][real], o_sc[q][real], rtol=0, atol=2e-6)
        assert np.all(np.diff(g_sc[q][real]) <= 0) and len(set(g_ids[q][real].tolist())) == int(real.sum())
        if not np.array_equal(g_ids[q], o_ids[q]):                    # only exact-score neighbours may swap or differ at the cut
            swaps += 1
            qn = orc.normalize_rows(cs.Q[q:q + 1])[0]
            for gid, osc in zip(g_ids[q][real], o_sc[q][real]):
                s = float(orc.normalize_rows(cs.X[gid:gid + 1])[0] @ qn)
                assert abs(s - osc) <= 2e-6, f"query {q}: label {gid} is not tied with the oracle's result at its rank"
    print(f"[{name}] r={r} k={k}: {swaps} queries with tie swaps", flush=True)


def test_rerank_argument_errors():
    import paper_2605_17415_amd as pkg
    q = torch.zeros((2, 16), device=DEV)
    x = torch.ones((10, 16), device=DEV)
    c = torch.zeros((2, 4), dtype=torch.int64, device=DEV)
    with pytest.raises(pkg.IvftqError) as e:
        pkg.ivftq_rerank(q, x, c, 5)                                  # k > r
    assert e.value.status == 1
    sc, ids = pkg.ivftq_rerank(q, x, c, 2)                            # zero-norm queries: nothing can be scored
    torch.cuda.synchronize()
    assert np.all(ids.cpu().numpy() == -1)
