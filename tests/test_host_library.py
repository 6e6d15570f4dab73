"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host-side constants (codebook, rotation) agree with the oracle and with the mathematics.
No kernel is launched here."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import paper_2605_17415_amd as pkg
from oracle import ivftq_oracle as orc
from workloads import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_symbols():
    text = open(os.path.join(ROOT, "include", "ivftq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ivftq_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = pkg.load_library()
    declared = _header_symbols()
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in ivftq.h but not exported"
    assert sorted(pkg.declared_symbols()) == declared       # the binding covers the whole header
    assert pkg.ivftq_version().startswith("ivftq")


@pytest.mark.parametrize("b,d", [(1, 64), (2, 96), (3, 96), (4, 64), (4, 96), (4, 128), (4, 200), (5, 128), (6, 8), (7, 70), (8, 8),
                                 (8, 256)])
def test_codebook_matches_oracle(b, d):
    c, tau = pkg.ivftq_build_codebook(b, d)
    oc, otau = orc.lloyd_max_codebook(b, d)
    assert c.dtype == np.float32 and c.shape == (1 << b,) and tau.shape == ((1 << b) - 1,)
    np.testing.assert_allclose(c, oc, rtol=6e-8, atol=2e-8)       # float32 rounding of a float64 value
    np.testing.assert_allclose(tau, otau, rtol=6e-8, atol=2e-8)
    # ... and the float32 tables both sides work with are the same bits
    oc32, otau32 = orc.codebook_fp32(b, d)
    np.testing.assert_array_equal(c, oc32)
    np.testing.assert_array_equal(tau, otau32)
    assert np.all(np.diff(c) > 0)
    assert tau[len(tau) // 2] == 0.0                        # the middle boundary is exactly zero
    np.testing.assert_array_equal(c, -c[::-1])


def test_one_bit_codebook_closed_form():
    for d in (64, 96, 128, 200):
        c, tau = pkg.ivftq_build_codebook(1, d)
        closed = math.exp(math.lgamma(d / 2) - 0.5 * math.log(math.pi) - math.lgamma((d + 1) / 2))
        assert abs(c[1] - closed) < 1e-8 and abs(c[0] + closed) < 1e-8


def test_codebook_argument_errors():
    lib = pkg.load_library()
    buf = np.empty(256, np.float32)
    p = buf.ctypes.data_as(ctypes.c_void_p)
    assert lib.ivftq_build_codebook(0, 64, p, p) == 1
    assert lib.ivftq_build_codebook(9, 64, p, p) == 1
    assert lib.ivftq_build_codebook(4, 2, p, p) == 1
    assert lib.ivftq_build_codebook(4, 64, None, None) == 1
    assert b"b" in lib.ivftq_last_error() or len(lib.ivftq_last_error()) > 0
    with pytest.raises(pkg.IvftqError):
        pkg.ivftq_build_codebook(0, 64)


@pytest.mark.parametrize("d", (8, 64, 200))
def test_rotation_from_shared_gaussian_matches_oracle(d):
    G = synth.gaussian_matrix(7, d)
    Pi = pkg.ivftq_haar_from_gaussian(G)
    ref = orc.haar_rotation_from_gaussian(G)
    np.testing.assert_allclose(Pi, ref, atol=2e-7)


def test_own_rotation_is_orthogonal_and_seeded():
    d = 96
    P1, P2, P3 = pkg.ivftq_haar_rotation(d, 1), pkg.ivftq_haar_rotation(d, 1), pkg.ivftq_haar_rotation(d, 2)
    np.testing.assert_array_equal(P1, P2)
    assert np.max(np.abs(P1 - P3)) > 0.01
    P = P1.astype(np.float64)
    assert np.max(np.abs(P @ P.T - np.eye(d))) < 1e-6
    # entries of a Haar matrix have variance 1/d and are far from a permutation or identity
    assert abs(P.var() - 1.0 / d) < 0.05 / d
    assert np.max(np.abs(P)) < 0.6
    cols = np.array([pkg.ivftq_haar_rotation(16, s)[:, 0] for s in range(300)], dtype=np.float64)
    assert abs(cols.mean()) < 0.02 and abs(cols.var() - 1 / 16) < 0.1 / 16


def test_create_rejects_bad_arguments_before_touching_a_device():
    lib = pkg.load_library()
    h = ctypes.c_void_p()
    assert lib.ivftq_create(64, 0, 8, 0, None, None, None, ctypes.byref(h)) == 1       # b out of range
    assert lib.ivftq_create(4, 4, 8, 0, None, None, None, ctypes.byref(h)) == 1        # d too small
    assert lib.ivftq_create(64, 4, 0, 0, None, None, None, ctypes.byref(h)) == 1       # nlist too small
    assert lib.ivftq_create(64, 4, 8, 0, None, None, None, None) == 1                  # NULL out pointer
    assert lib.ivftq_create(4096, 4, 8, 0, None, None, None, ctypes.byref(h)) == 6     # d beyond the limit
    assert lib.ivftq_create(64, 4, 1 << 20, 0, None, None, None, ctypes.byref(h)) == 6 # nlist beyond the limit
    assert not h.value
    assert lib.ivftq_ntotal(None) == -1
    assert lib.ivftq_destroy(None) == 0


@pytest.mark.parametrize("b,d", [(1, 64), (2, 96), (3, 96), (4, 8), (4, 128), (4, 200), (5, 100), (6, 70), (7, 96), (8, 8),
                                 (8, 256)])
def test_quantiser_grid_counts_boundaries_exactly(b, d):
    """The table the encode kernel quantises through gives code = #{i : v >= tau_i} (bins
    [tau_i, tau_{i+1})) for every float32 value: at, just below and just above every boundary, at the
    cell edges of the grid itself, far outside, and for random values; also when the cell number is
    off by the rounding of its float32 computation."""
    _, tau = pkg.ivftq_build_codebook(b, d)
    cells, scale, offset, boundary, index = pkg.ivftq_quantiser_grid(b, d)
    assert 1 <= cells <= 4096 and boundary.shape == (cells,) and index.shape == (cells,)
    rng = np.random.default_rng(b * 1000 + d)
    vals = [tau, np.nextafter(tau, np.float32(-2)), np.nextafter(tau, np.float32(2)),
            np.float32([-1.0, 1.0, 0.0, -0.0, -3.0, 3.0, 1e-30, -1e-30]),
            (rng.standard_normal(20000) / math.sqrt(d)).astype(np.float32),
            rng.uniform(-1, 1, 20000).astype(np.float32)]
    if cells > 1:
        edges = ((np.arange(cells + 1, dtype=np.float64) - float(offset)) / float(scale)).astype(np.float32)
        vals += [edges, np.nextafter(edges, np.float32(-2)), np.nextafter(edges, np.float32(2))]
    v = np.concatenate(vals).astype(np.float32)
    want = np.searchsorted(tau, v, side="right")            # number of boundaries <= v
    x = v * scale + offset                                   # float32 arithmetic, as on the device
    assert x.dtype == np.float32
    for nudge in (0.0, -0.2, 0.2):                           # a fifth of a cell of slack either way
        cell = np.clip(np.trunc(x.astype(np.float64) + nudge), 0, cells - 1).astype(np.int64)
        got = index[cell] + (v >= boundary[cell])
        np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("b,d", [(1, 64), (2, 96), (3, 128), (4, 8), (4, 96), (4, 200), (7, 256)])
def test_refined_codebook_matches_oracle_and_its_grid_counts_exactly(b, d):
    """Stage 1 + sign bit as one quantiser: levels and boundaries against the oracle, and the lookup
    table built over the merged boundaries still counts them exactly."""
    lv, bd = pkg.ivftq_build_refined_codebook(b, d)
    olv, obd = orc.refined_codebook_fp32(b, d)
    np.testing.assert_array_equal(bd, obd)                  # float32 Stage-1 centroids and boundaries, interleaved
    np.testing.assert_array_equal(lv, olv)                  # the same float32 levels, bit for bit
    assert np.all(np.diff(bd) > 0) and np.all(np.diff(lv) > 0)
    c, tau = pkg.ivftq_build_codebook(b, d)
    np.testing.assert_array_equal(bd[0::2], c)
    np.testing.assert_array_equal(bd[1::2], tau)
    cells, scale, offset, boundary, index = pkg.ivftq_quantiser_grid(b, d, sign_bit=True)
    assert 1 <= cells <= 4096
    rng = np.random.default_rng(b + d)
    v = np.concatenate([bd, np.nextafter(bd, np.float32(-2)), np.nextafter(bd, np.float32(2)),
                        (rng.standard_normal(20000) / math.sqrt(d)).astype(np.float32), np.float32([-1, 1, 0])]).astype(np.float32)
    x = v * scale + offset
    for nudge in (0.0, -0.2, 0.2):
        cell = np.clip(np.trunc(x.astype(np.float64) + nudge), 0, cells - 1).astype(np.int64)
        np.testing.assert_array_equal(index[cell] + (v >= boundary[cell]), np.searchsorted(bd, v, side="right"))


@pytest.mark.parametrize("b,d,beta,sign_bit", [(4, 128, 2, False), (5, 96, 4, True), (3, 16, 1, False), (4, 96, 4, False)])
def test_coarsened_codebook_matches_oracle(b, d, beta, sign_bit):
    """Cascade pass-1 table (Appendix "Cascade search"): conditional means of the merged bins."""
    import paper_2605_17415_amd as pkg
    c, tau = orc.lloyd_max_codebook(b, d)
    want = orc.coarsened_codebook(c, tau, d, beta)
    got = pkg.ivftq_build_coarsened_codebook(b, d, beta, sign_bit)
    np.testing.assert_allclose(got, want, rtol=0, atol=3e-8)
    with pytest.raises(pkg.IvftqError):
        pkg.ivftq_build_coarsened_codebook(b, d, b + 1, sign_bit)
    with pytest.raises(pkg.IvftqError):
        pkg.ivftq_build_coarsened_codebook(b, d, 0, sign_bit)


def test_create_reports_oom_when_the_allocator_callback_refuses():
    """No device is touched before the first allocation, so this runs without a GPU: a callback that
    returns NULL gives IVFTQ_OOM and no handle; giving only one of the two callbacks is an argument error."""
    lib = pkg.load_library()
    calls = []

    def refuse(nbytes, ctx):
        calls.append(int(nbytes))
        return None

    freed = []
    alloc_cb = pkg.ALLOC_FN(refuse)
    free_cb = pkg.FREE_FN(lambda p, ctx: freed.append(p))
    handle = ctypes.c_void_p(12345)
    status = lib.ivftq_create(96, 4, 64, 1, ctypes.cast(alloc_cb, ctypes.c_void_p), ctypes.cast(free_cb, ctypes.c_void_p),
                              None, ctypes.byref(handle))
    assert status == pkg.binding.OOM and handle.value is None
    assert len(calls) == 1 and calls[0] == 64 * 96 * 4 and freed == []
    assert b"memory" in lib.ivftq_last_error().lower() or len(lib.ivftq_last_error()) > 0
    status = lib.ivftq_create(96, 4, 64, 1, ctypes.cast(alloc_cb, ctypes.c_void_p), None, None, ctypes.byref(handle))
    assert status == pkg.binding.INVALID_ARG and handle.value is None
    with pytest.raises(pkg.IvftqError) as e:
        pkg.Index(96, 4, 64, allocator=(alloc_cb, free_cb))
    assert e.value.status == pkg.binding.OOM
