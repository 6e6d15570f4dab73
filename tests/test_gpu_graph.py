"""GPU: ivftq_search recorded into a HIP graph (after eager calls of every shape the program uses, which
size the workspace; the search makes no allocation, no host synchronisation and no memset after that) and
replayed.  Every replay is compared with the eager result for the same queries, with eager searches of
other shapes and new query values between the replays.  (A call that makes the workspace grow moves it,
which invalidates graphs recorded before: hence the sizing calls come first.)"""
import numpy as np
import pytest

import gpu_cases

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nq,mode", [(1, 0), (48, 0), (48, 2), (1, 2), (130, 0)])
def test_search_replays_from_a_graph(nq, mode):
    """mode 0 takes the streaming scan for calls of this size and the batched scan for large ones; mode 2 the
    batched scan at any size."""
    import paper_2605_17415_amd as pkg
    cs = gpu_cases.get_case("d128")
    dev = torch.device("cuda:0")
    ix = pkg.Index(cs.d, cs.b, len(cs.cent))
    ix.set_coarse(cs.cent)
    ix.set_rotation(cs.Pi)
    ix.encode_add(torch.from_numpy(cs.X).to(dev))
    ix.set_search_mode(mode)
    Q = torch.from_numpy(cs.Q).to(dev)
    q = Q[:nq].clone()
    out_s = torch.empty((nq, cs.k), dtype=torch.float32, device=dev)
    out_i = torch.empty((nq, cs.k), dtype=torch.int64, device=dev)
    ix.search(Q[:200], max(1, cs.nprobe // 2), cs.k)                     # eager, every shape used below: sizes the workspace
    ix.search(q, cs.nprobe, cs.k, out_scores=out_s, out_ids=out_i)
    torch.cuda.synchronize()
    print(f"[graph] capture nq={nq} mode={mode}", flush=True)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ix.search(q, cs.nprobe, cs.k, out_scores=out_s, out_ids=out_i, stream=torch.cuda.current_stream())
    for rep in range(4):
        lo = (rep * nq) % (len(cs.Q) - nq)
        q.copy_(Q[lo:lo + nq])                                          # new query values, same buffers
        ref_s, ref_i = ix.search(q, cs.nprobe, cs.k)                     # eager result for these queries
        ix.search(Q[:200], max(1, cs.nprobe // 2), cs.k)                 # eager work of another shape in between
        torch.cuda.synchronize()
        out_s.fill_(-7.0)
        out_i.fill_(-7)
        print(f"[graph] replay {rep}", flush=True)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_i, ref_i), f"replay {rep}: labels differ from the eager search"
        assert torch.equal(out_s, ref_s), f"replay {rep}: scores differ from the eager search"
    ix.close()
