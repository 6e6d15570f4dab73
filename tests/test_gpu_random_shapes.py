"""GPU parity on seeded random shapes: dimension, list count, bit width, probe count and k drawn at
random (including every residue of d modulo 4 and 16, list counts around the kernels' 32/64/128-centroid
stages, nprobe = 1 and nprobe = nlist), encode and search compared with the oracle by the same rules as the
fixed cases."""
import numpy as np
import pytest

import parity
from oracle import ivftq_oracle as orc
from workloads import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _shape(seed):
    rng = np.random.default_rng(9000 + seed)
    d = int(rng.choice([8, 12, 17, 24, 31, 32, 33, 48, 63, 64, 65, 90, 96, 97, 127, 128, 129, 160, 190, 201, 224, 255, 256]))
    L = int(rng.choice([1, 2, 5, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 200]))
    b = int(rng.integers(1, 9))
    n = int(rng.integers(300, 4000))
    nq = int(rng.integers(1, 70))
    nprobe = int(rng.choice([1, min(L, 3), min(L, 8), L]))
    k = int(rng.choice([1, 3, 10, 40]))
    return d, L, b, n, nq, nprobe, k


@pytest.mark.parametrize("seed", range(14))
def test_random_shape_matches_oracle(seed):
    import paper_2605_17415_amd as pkg
    d, L, b, n, nq, nprobe, k = _shape(seed)
    print(f"[random shape {seed}] d={d} L={L} b={b} n={n} nq={nq} nprobe={nprobe} k={k}", flush=True)
    rng = np.random.default_rng(100 + seed)
    means = rng.standard_normal((max(2, L // 2), d))
    X = (means[rng.integers(0, len(means), n)] + 0.4 * rng.standard_normal((n, d))).astype(np.float32)
    Q = (means[rng.integers(0, len(means), nq)] + 0.4 * rng.standard_normal((nq, d))).astype(np.float32)
    cent, _ = orc.train_coarse(X, L, 2, synth.kmeans_init_indices(seed, n, L))
    cent = cent.astype(np.float32)
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(seed, d)).astype(np.float32)
    c, tau = orc.codebook_fp32(b, d)
    enc = orc.encode(X, cent, Pi, tau)
    oidx = orc.ListIndex(cent, Pi, c, tau)
    oidx.add_encoded(enc["assign"], np.arange(n, dtype=np.int64), enc["codes"], enc["gamma16"])

    dev = torch.device("cuda:0")
    ix = pkg.Index(d, b, L)
    ix.set_coarse(cent)
    ix.set_rotation(Pi)
    x = torch.from_numpy(X).to(dev)
    assign, codes, gamma = ix.encode_only(x)
    torch.cuda.synchronize()
    # with a few hundred rows in up to 200 cells some cells hold a single row, which then is its own centroid
    # (zero residual): at most one such row per cell
    rep = parity.compare_encode(enc, assign.cpu().numpy(), codes.cpu().numpy(), gamma.cpu().numpy(), max_excused=L)
    print("encode:", rep, flush=True)

    # search on the oracle's codes, both scan strategies
    o_sc, o_ids, _, S, o_all = orc.search(oidx, Q, nprobe, k, return_all=True)
    gap = parity.probe_cut_gap(S, nprobe)
    ix.add_encoded(torch.from_numpy(enc["assign"]).to(dev), torch.from_numpy(enc["codes"]).to(dev),
                   torch.from_numpy(enc["gamma16"]).to(dev))
    q = torch.from_numpy(Q).to(dev)
    for mode in (2, 1):
        ix.set_search_mode(mode)
        sc, ids = ix.search(q, nprobe, k)
        torch.cuda.synchronize()
        rs = parity.compare_search(sc.cpu().numpy(), ids.cpu().numpy(), o_sc, o_ids, o_all, gap)
        print(f"search mode {mode}:", rs, flush=True)
        assert rs["probe_near_tie_excused"] <= max(1, nq // 10)
    ix.close()


@pytest.mark.parametrize("d,b,L,n", [(32, 4, 5, 700), (64, 8, 33, 2100), (64, 4, 64, 4097), (96, 8, 31, 1500), (100, 4, 20, 2500),
                                     (128, 8, 64, 3000), (128, 4, 129, 5000), (70, 4, 17, 900), (200, 8, 40, 1800), (160, 4, 9, 1000),
                                     (96, 3, 32, 2000), (96, 5, 32, 2000), (255, 4, 12, 640), (24, 8, 3, 333)])
def test_encode_add_stores_what_encode_only_returns(d, b, L, n):
    """Every way the encode-and-store kernels put codes together (words assembled in registers for 4 and 8
    bits, with the rotation resident in LDS up to 128 dimensions and streamed beyond, through LDS for other
    bit widths; 16-byte and scalar row reads; padded last tiles) must store, list by list and in arrival
    order, exactly the cell, codes and norm that `ivftq_encode_only` returns for the same rows, which the test
    above holds against the oracle; two batches, the second ragged."""
    import paper_2605_17415_amd as pkg
    print(f"[encode_add vs encode_only] d={d} b={b} L={L} n={n}", flush=True)
    rng = np.random.default_rng(d * 1000 + b * 10 + L)
    means = rng.standard_normal((max(2, L), d))
    X = (means[rng.integers(0, len(means), n)] + 0.5 * rng.standard_normal((n, d))).astype(np.float32)
    cent, _ = orc.train_coarse(X, L, 1, synth.kmeans_init_indices(d + b, n, L))
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(d + b, d)).astype(np.float32)
    c, tau = orc.codebook_fp32(b, d)
    enc = orc.encode(X, cent.astype(np.float32), Pi, tau)
    dev = torch.device("cuda:0")
    ix = pkg.Index(d, b, L)
    ix.set_coarse(cent.astype(np.float32))
    ix.set_rotation(Pi)
    x = torch.from_numpy(X).to(dev)
    assign, codes, gamma = ix.encode_only(x)
    torch.cuda.synchronize()
    assign, codes, gamma = assign.cpu().numpy(), codes.cpu().numpy(), gamma.cpu().numpy()
    print("encode:", parity.compare_encode(enc, assign, codes, gamma, max_excused=L), flush=True)
    cut = n // 2 + 13
    ix.encode_add(x[:cut])
    ix.encode_add(x[cut:])
    assert ix.ntotal() == n
    seen = 0
    for l in range(L):
        ids, lc, lg = ix.export_list(l)
        want = np.flatnonzero(assign == l)
        np.testing.assert_array_equal(ids, want)                        # arrival order
        np.testing.assert_array_equal(lc, codes[want])
        np.testing.assert_array_equal(lg.view(np.uint16), gamma[want].view(np.uint16))
        seen += len(ids)
    assert seen == n
    ix.close()
