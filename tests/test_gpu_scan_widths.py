"""The streaming list scan (Appendix "Why cascade does not yield a speedup": per-query table of z_j * C[e],
one lookup per stored code) at every code width b = 1 ... 8, with rows of whole 32-coordinate chunks only,
of chunks plus a short rest, and shorter than one chunk: codes that sit in the lowest bits of a packed word,
that straddle two words (b = 3, 5, 6, 7) and that end a row are all on the path.  Search results against the
oracle on the oracle's own codes, by the same rules as the fixed cases."""
import numpy as np
import pytest

import parity
from oracle import ivftq_oracle as orc
from workloads import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d", [20, 64, 72, 200, 256])
@pytest.mark.parametrize("b", range(1, 9))
def test_streaming_scan_every_width(b, d):
    import paper_2605_17415_amd as pkg
    L, n, nq, nprobe, k = 8, 2500, 24, 4, 10
    print(f"[scan widths] b={b} d={d}", flush=True)
    rng = np.random.default_rng(1000 * b + d)
    means = rng.standard_normal((L, d))
    X = (means[rng.integers(0, L, n)] + 0.5 * rng.standard_normal((n, d))).astype(np.float32)
    Q = (means[rng.integers(0, L, nq)] + 0.5 * rng.standard_normal((nq, d))).astype(np.float32)
    cent, _ = orc.train_coarse(X, L, 2, synth.kmeans_init_indices(b, n, L))
    cent = cent.astype(np.float32)
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(b, d)).astype(np.float32)
    c, tau = orc.codebook_fp32(b, d)
    enc = orc.encode(X, cent, Pi, tau)
    oidx = orc.ListIndex(cent, Pi, c, tau)
    oidx.add_encoded(enc["assign"], np.arange(n, dtype=np.int64), enc["codes"], enc["gamma16"])
    o_sc, o_ids, _, S, o_all = orc.search(oidx, Q, nprobe, k, return_all=True)
    gap = parity.probe_cut_gap(S, nprobe)

    dev = torch.device("cuda:0")
    ix = pkg.Index(d, b, L)
    ix.set_coarse(cent)
    ix.set_rotation(Pi)
    ix.add_encoded(torch.from_numpy(enc["assign"]).to(dev), torch.from_numpy(enc["codes"]).to(dev),
                   torch.from_numpy(enc["gamma16"]).to(dev))
    ix.set_search_mode(1)
    sc, ids = ix.search(torch.from_numpy(Q).to(dev), nprobe, k)
    torch.cuda.synchronize()
    rs = parity.compare_search(sc.cpu().numpy(), ids.cpu().numpy(), o_sc, o_ids, o_all, gap)
    print("search:", rs, flush=True)
    assert rs["probe_near_tie_excused"] <= 2
    ix.close()
