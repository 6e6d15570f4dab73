"""CPU oracle for the IVF-TQ hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, double-precision statement of what the method computes, written
from the paper (arxiv 2605.17415) so that the HIP kernels can be checked against
it.  Only tests, the smoke check and the benchmark's CPU-baseline leg may use
this module; the product path never does, and this module never imports the
product package.

Every function follows the paper's steps in the paper's order:

  codebook      Appendix "Proofs of the rate-distortion bounds", Setup and
                Lemma 1 (coordinate density of a Haar-rotated unit vector);
                Lloyd-Max = alternate "boundaries are centroid midpoints" and
                "centroids are bin conditional means" (proof of Lemma 2).
  rotation      Setup of the same appendix: Pi ~ Haar(O(d)).
  coarse train  Section "Architecture", Indexing: k-means on unit-sphere data,
                centroids re-normalised.
  encode        Section "Architecture", Indexing and Bit accounting.
  search        Section "Architecture", Search; Section "IVF amplifies
                codebook-free quantization" (decomposition <q,x>=<q,c>+<q,r>).
  bin rule      Appendix "Sign-bit refinement": bins are [tau_i, tau_{i+1}).

Readings taken where the paper is silent (each is also listed in the design
notes): ties go to the smallest index; a zero residual encodes as rho = 0;
fewer than k candidates pad with id -1 and score -inf; the stored norm is the
norm of r (not of Pi r), rounded to nearest-even float16; the reconstruction
uses the plain centroid values with no de-biasing factor.

  raw metrics   not in the paper (it keeps every vector on the unit sphere):
                <q,x> = |q||x|<q~,x~> and |q-x|^2 = |q|^2+|x|^2-2|q||x|<q~,x~>
                applied to the estimate of <q~,x~>, with |x| stored as float32.

Parity status: codebook, rotation, k-means, encode, search, raw-metric search,
reconstruction and exact k-NN are pinned by tests/test_oracle_*.py against
closed forms, hand-derived cases, invariants and brute force.  The reading of
k-means (Euclidean Lloyd iterations from given rows, empty cells re-seeded from
the largest cell) is the build's: the paper only names k-means.
"""
from __future__ import annotations

import math

import numpy as np

# --------------------------------------------------------------------------
# Codebook (b, d)
# --------------------------------------------------------------------------


def sphere_coord_density(t, d: int):
    """f_d(t) = Gamma(d/2) / (sqrt(pi) Gamma((d-1)/2)) (1-t^2)^((d-3)/2) on [-1,1] (Lemma 1)."""
    t = np.asarray(t, dtype=np.float64)
    logk = math.lgamma(d / 2.0) - 0.5 * math.log(math.pi) - math.lgamma((d - 1) / 2.0)
    base = np.clip(1.0 - t * t, 0.0, None)
    with np.errstate(divide="ignore"):
        val = np.exp(logk + 0.5 * (d - 3) * np.log(base))
    return np.where(np.abs(t) <= 1.0, val, 0.0)


def gauss_coord_density(t, d: int):
    """N(0, 1/d) density: the Gaussian the paper's text names as the design source."""
    t = np.asarray(t, dtype=np.float64)
    return math.sqrt(d / (2.0 * math.pi)) * np.exp(-0.5 * d * t * t)


_GL_X, _GL_W = np.polynomial.legendre.leggauss(96)
_PIECES = 4


def _integrate_bins(fn, edges):
    """Integral of fn over each [edges[i], edges[i+1]]: composite Gauss-Legendre quadrature."""
    edges = np.asarray(edges, dtype=np.float64)
    frac = np.arange(_PIECES + 1) / _PIECES
    sub = edges[:-1, None] + (edges[1:] - edges[:-1])[:, None] * frac[None, :]   # [bins, pieces+1]
    a, b = sub[:, :-1], sub[:, 1:]
    x = 0.5 * (b - a)[..., None] * _GL_X + 0.5 * (b + a)[..., None]              # [bins, pieces, nodes]
    return np.sum(0.5 * (b - a) * np.sum(_GL_W * fn(x), axis=-1), axis=-1)


def _support(density: str, d: int):
    if density == "sphere":
        return -1.0, 1.0
    s = 12.0 / math.sqrt(d)  # Gaussian mass beyond 12 sigma is below 1e-32
    return -s, s


def _pdf(density: str, d: int):
    if density == "sphere":
        return lambda t: sphere_coord_density(t, d)
    if density == "gauss":
        return lambda t: gauss_coord_density(t, d)
    raise ValueError(density)


def lloyd_max_codebook(b: int, d: int, density: str = "sphere",
                       tol: float = 1e-13, max_iter: int = 20000):
    """K = 2^b Lloyd-Max centroids (ascending) and K-1 interior boundaries, float64.

    Fixed point of: tau_i = (c_{i-1} + c_i)/2 ;  c_i = int_bin t f / int_bin f,
    with the outer bin edges at the ends of the support.
    """
    if not (1 <= b <= 8) or d < 3:
        raise ValueError("need 1 <= b <= 8 and d >= 3")
    K = 1 << b
    pdf = _pdf(density, d)
    lo, hi = _support(density, d)
    sd = 1.0 / math.sqrt(d)
    # start from a uniform grid over +-3 standard deviations, cut to the support of the density
    # (for small d three standard deviations reach beyond [-1, 1], where every bin would be empty)
    half_width = min(3.0 * sd, hi)
    c = ((np.arange(K) + 0.5) / K * 2.0 - 1.0) * half_width
    def lloyd_step(c):
        tau = 0.5 * (c[:-1] + c[1:])
        edges = np.concatenate(([lo], tau, [hi]))
        mass = _integrate_bins(pdf, edges)
        first = _integrate_bins(lambda t: t * pdf(t), edges)
        return first / mass, mass, edges

    converged = False
    for _ in range(min(max_iter, 3000)):
        new, _, _ = lloyd_step(c)
        delta = float(np.max(np.abs(new - c)))
        c = new
        if delta < tol:
            converged = True
            break
    # For large K the Lloyd map contracts very slowly (rate -> 1), so what is left is removed by
    # Newton's method on the same stationarity conditions c = T(c).  With m_i the mass of bin i and
    # e_i, e_{i+1} its edges, dT_i/de_i = f(e_i)(T_i - e_i)/m_i and dT_i/de_{i+1} = f(e_{i+1})(e_{i+1} - T_i)/m_i,
    # and an interior edge is the mean of the two centroids beside it.
    for _ in range(0 if converged else 100):
        T, mass, edges = lloyd_step(c)
        resid = T - c
        if float(np.max(np.abs(resid))) < tol:
            converged = True
            c = T
            break
        fe = pdf(edges)
        d_lower = fe[:-1] * (T - edges[:-1]) / mass
        d_upper = fe[1:] * (edges[1:] - T) / mass
        d_lower[0] = 0.0      # the outer edges are fixed at the ends of the support
        d_upper[-1] = 0.0
        J = np.diag(0.5 * (d_lower + d_upper)) + np.diag(0.5 * d_lower[1:], -1) + np.diag(0.5 * d_upper[:-1], 1)
        step = np.linalg.solve(np.eye(K) - J, resid)
        trial = c + step
        c = trial if np.all(np.diff(trial) > 0) and np.all(np.abs(trial) < max(abs(lo), abs(hi))) else T
        c = 0.5 * (c - c[::-1])
    if not converged:
        raise RuntimeError("Lloyd-Max conditions not met")
    c = 0.5 * (c - c[::-1])  # the density is even: impose c_i = -c_{K-1-i} exactly
    tau = 0.5 * (c[:-1] + c[1:])
    return c, tau


def codebook_fp32(b: int, d: int, density: str = "sphere"):
    """The codebook as stored: float32 centroids and float32 boundaries."""
    c, tau = lloyd_max_codebook(b, d, density)
    return c.astype(np.float32), tau.astype(np.float32)


def codebook_distortion(c, tau, d: int, density: str = "sphere") -> float:
    """D = d * E[(C(T) - T)^2] under the given coordinate density."""
    pdf = _pdf(density, d)
    lo, hi = _support(density, d)
    edges = np.concatenate(([lo], np.asarray(tau, dtype=np.float64), [hi]))
    c = np.asarray(c, dtype=np.float64)
    per_bin = _integrate_bins(lambda t: (t - c[:, None, None]) ** 2 * pdf(t), edges)
    return d * float(np.sum(per_bin))


def bin_masses(tau, d: int, density: str = "sphere"):
    pdf = _pdf(density, d)
    lo, hi = _support(density, d)
    edges = np.concatenate(([lo], np.asarray(tau, dtype=np.float64), [hi]))
    return _integrate_bins(pdf, edges)


# --------------------------------------------------------------------------
# Stage 2: sign-bit refinement (Appendix "Sign-bit refinement")
# --------------------------------------------------------------------------
#
# One more bit per coordinate says on which side of its bin's centroid the value lies,
# s = 1[v >= c_i]; reconstruction uses the mean of the half-bin.  The half-bin means are taken
# under the same coordinate density the codebook is designed for (the appendix writes
# N(0, 1/d) there as it does for the codebook itself).


def half_bin_means(c, tau, d: int, density: str = "sphere"):
    """m[i, s] = E[T | T in half-bin (i, s)]: s = 0 is [tau_i, c_i), s = 1 is [c_i, tau_{i+1}).

    Also returns the probability mass of every half-bin, same shape [K, 2]."""
    pdf = _pdf(density, d)
    lo, hi = _support(density, d)
    c = np.asarray(c, dtype=np.float64)
    edges = np.concatenate(([lo], np.asarray(tau, dtype=np.float64), [hi]))
    K = len(c)
    means = np.empty((K, 2))
    mass = np.empty((K, 2))
    for i in range(K):
        for s, (a, b) in enumerate(((edges[i], c[i]), (c[i], edges[i + 1]))):
            m0 = _integrate_bins(pdf, np.array([a, b]))[0]
            m1 = _integrate_bins(lambda t: t * pdf(t), np.array([a, b]))[0]
            mass[i, s] = m0
            means[i, s] = m1 / m0
    return means, mass


def sign_bits(rho, codes, c):
    """s_j = 1[rho_j >= c_{code_j}] for every coordinate (the stored refinement bit)."""
    c = np.asarray(c)
    return (np.asarray(rho) >= c[np.asarray(codes, dtype=np.int64)]).astype(np.uint8)


def refined_tables(c, tau, d: int, density: str = "sphere"):
    """The same refinement written as one quantiser with 2K levels: its 2K-1 boundaries are the
    bin boundaries and the centroids interleaved (c_0 < tau_1 < c_1 < ...), its level 2i+s is the
    mean of half-bin (i, s); then  #{boundaries <= v} = 2*code + s."""
    means, _ = half_bin_means(c, tau, d, density)
    c = np.asarray(c, dtype=np.float64)
    tau = np.asarray(tau, dtype=np.float64)
    K = len(c)
    bnd = np.empty(2 * K - 1)
    bnd[0::2] = c
    bnd[1::2] = tau
    return means.reshape(2 * K), bnd


def refined_codebook_fp32(b: int, d: int, density: str = "sphere"):
    """Stage 1 at b bits plus the sign bit, as stored: 2^(b+1) float32 levels and 2^(b+1) - 1
    float32 boundaries.  Boundaries are the float32 Stage-1 centroids and boundaries themselves."""
    c, tau = lloyd_max_codebook(b, d, density)
    levels, _ = refined_tables(c, tau, d, density)
    c32, tau32 = c.astype(np.float32), tau.astype(np.float32)
    bnd = np.empty(2 * len(c) - 1, np.float32)
    bnd[0::2] = c32
    bnd[1::2] = tau32
    return levels.astype(np.float32), bnd


# --------------------------------------------------------------------------
# Rotation
# --------------------------------------------------------------------------


def haar_rotation_from_gaussian(G):
    """Haar-distributed orthogonal Pi from a d x d iid N(0,1) matrix.

    QR-factorise G and multiply column j of Q by sign(R_jj): with that sign
    convention Q is Haar on O(d).  Pi acts as u = Pi @ r.
    """
    G = np.asarray(G, dtype=np.float64)
    Q, R = np.linalg.qr(G)
    s = np.sign(np.diag(R))
    s[s == 0] = 1.0
    return Q * s[None, :]


# --------------------------------------------------------------------------
# Coarse partition
# --------------------------------------------------------------------------


def normalize_rows(X):
    X = np.asarray(X, dtype=np.float64)
    nrm = np.sqrt(np.sum(X * X, axis=1, keepdims=True))
    if np.any(nrm == 0):
        raise ValueError("zero-norm input row")
    return X / nrm


def train_coarse(X, nlist: int, niter: int, init_idx, rng_seed: int = 0):
    """Lloyd k-means on the normalised rows of X; final centroids L2-normalised.

    init_idx: nlist distinct rows used as initial centres.  Each iteration assigns
    every point to its nearest mean (Euclidean) and replaces each mean by the average
    of its points; an empty cell takes a seeded random member of the largest cell.
    Returns (unit centroids [nlist, d] float64, inertia of the last assignment step).
    """
    Xn = normalize_rows(X)
    C = Xn[np.asarray(init_idx)].copy()
    rs = np.random.Generator(np.random.Philox(key=[int(rng_seed), 99]))
    inertia = float("nan")
    for _ in range(niter):
        # ||x - m||^2 = 1 - 2<x,m> + ||m||^2 for unit x
        score = Xn @ C.T - 0.5 * np.sum(C * C, axis=1)[None, :]
        a = np.argmax(score, axis=1)
        inertia = float(np.sum(1.0 - 2.0 * score[np.arange(len(a)), a]))
        counts = np.bincount(a, minlength=nlist)
        sums = np.zeros_like(C)
        np.add.at(sums, a, Xn)
        for l in range(nlist):
            if counts[l] > 0:
                C[l] = sums[l] / counts[l]
            else:
                big = int(np.argmax(counts))
                members = np.flatnonzero(a == big)
                C[l] = Xn[members[rs.integers(0, len(members))]]
    return normalize_rows(C), inertia


# --------------------------------------------------------------------------
# Encode
# --------------------------------------------------------------------------


def quantize(rho, tau):
    """code = number of boundaries tau_i with rho >= tau_i  (bin [tau_i, tau_{i+1}))."""
    rho = np.asarray(rho, dtype=np.float64)
    tau = np.asarray(tau, dtype=np.float64)
    return np.sum(rho[..., None] >= tau, axis=-1).astype(np.uint8)


def encode(X, centroids, Pi, tau, chunk: int = 8192):
    """Encode rows of X.  Returns a dict:

      assign   [n] int32   coarse cell l = argmax_l <x~, c~_l>  (ties -> smallest l)
      codes    [n, d] u8   Lloyd-Max bin index of each coordinate of rho
      gamma16  [n] f16     ||x~ - c~_l||_2 rounded to nearest-even float16
      gamma    [n] f64     the same norm before rounding
      rho      [n, d] f64  Pi r / ||Pi r||
      bdist    [n, d] f64  distance of rho_j to its nearest decision boundary
      gap      [n] f64     best minus second-best coarse score
      coarse   [n] f64     <x~, c~_l>
    """
    X = np.asarray(X)
    C = np.asarray(centroids, dtype=np.float64)
    Pi = np.asarray(Pi, dtype=np.float64)
    tau = np.asarray(tau, dtype=np.float64)
    n, d = X.shape
    out = dict(assign=np.empty(n, np.int32), codes=np.empty((n, d), np.uint8),
               gamma16=np.empty(n, np.float16), gamma=np.empty(n), rho=np.empty((n, d)),
               bdist=np.empty((n, d)), gap=np.empty(n), coarse=np.empty(n))
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        xt = normalize_rows(X[s:e])
        sc = xt @ C.T
        a = np.argmax(sc, axis=1)                       # first maximum = smallest l
        best = sc[np.arange(e - s), a]
        if C.shape[0] > 1:
            second = np.partition(sc, -2, axis=1)[:, -2]
        else:
            second = np.full(e - s, -np.inf)
        r = xt - C[a]
        gamma = np.sqrt(np.sum(r * r, axis=1))
        u = r @ Pi.T
        un = np.sqrt(np.sum(u * u, axis=1))
        rho = np.where(un[:, None] > 1e-30, u / np.maximum(un, 1e-300)[:, None], 0.0)
        out["assign"][s:e] = a
        out["coarse"][s:e] = best
        out["gap"][s:e] = best - second
        out["gamma"][s:e] = gamma
        out["gamma16"][s:e] = gamma.astype(np.float16)
        out["rho"][s:e] = rho
        out["codes"][s:e] = quantize(rho, tau)
        out["bdist"][s:e] = np.min(np.abs(rho[..., None] - tau), axis=-1)
    return out


class ListIndex:
    """Inverted lists as the paper stores them: per list, ids, codes and float16 norms."""

    def __init__(self, centroids, Pi, c, tau):
        self.centroids = np.asarray(centroids, dtype=np.float64)
        self.Pi = np.asarray(Pi, dtype=np.float64)
        self.c = np.asarray(c, dtype=np.float64)
        self.tau = np.asarray(tau, dtype=np.float64)
        L = self.centroids.shape[0]
        self.ids = [np.empty(0, np.int64) for _ in range(L)]
        self.codes = [np.empty((0, self.centroids.shape[1]), np.uint8) for _ in range(L)]
        self.gamma16 = [np.empty(0, np.float16) for _ in range(L)]
        self.ntotal = 0

    def add(self, X, ids=None):
        enc = encode(X, self.centroids, self.Pi, self.tau)
        n = len(enc["assign"])
        ids = np.arange(self.ntotal, self.ntotal + n, dtype=np.int64) if ids is None \
            else np.asarray(ids, dtype=np.int64)
        self.add_encoded(enc["assign"], ids, enc["codes"], enc["gamma16"])
        return enc

    def add_encoded(self, assign, ids, codes, gamma16):
        """Append already-encoded vectors in input order (streaming append)."""
        order = np.argsort(assign, kind="stable")
        a_sorted = np.asarray(assign)[order]
        bounds = np.searchsorted(a_sorted, np.arange(len(self.ids) + 1))
        for l in range(len(self.ids)):
            sel = order[bounds[l]:bounds[l + 1]]
            if len(sel):
                self.ids[l] = np.concatenate([self.ids[l], np.asarray(ids)[sel]])
                self.codes[l] = np.concatenate([self.codes[l], np.asarray(codes)[sel]])
                self.gamma16[l] = np.concatenate([self.gamma16[l], np.asarray(gamma16)[sel]])
        self.ntotal += len(assign)

    def set_list(self, l, ids, codes, gamma16):
        """Load one list verbatim (used to search the index a device path stored)."""
        self.ntotal += len(ids) - len(self.ids[l])
        self.ids[l] = np.asarray(ids, np.int64)
        self.codes[l] = np.asarray(codes, np.uint8)
        self.gamma16[l] = np.asarray(gamma16, np.float16)


def search(index: ListIndex, Q, nprobe: int, k: int, return_all: bool = False):
    """For each query: exact coarse term plus residual estimate over the probed lists.

      s_l   = <q~, c~_l>                      for every cell l
      P     = nprobe cells with the largest s_l (ties -> smaller l)
      z     = Pi q~
      score = s_l + float(gamma16_i) * sum_j z_j * c[code_ij]   for i in list l, l in P
      result: k largest scores (ties -> smaller id), padded with (-1, -inf)

    Returns (scores [nq,k] f64, ids [nq,k] i64, probes [nq,nprobe] i32, coarse scores
    [nq, L] f64) and, when return_all, a per-query list of (ids, scores) of every
    scanned candidate.
    """
    Qn = normalize_rows(Q)
    nq = Qn.shape[0]
    S = Qn @ index.centroids.T
    Z = Qn @ index.Pi.T
    scores = np.full((nq, k), -np.inf)
    ids = np.full((nq, k), -1, dtype=np.int64)
    probes = np.empty((nq, nprobe), dtype=np.int32)
    everything = []
    L = index.centroids.shape[0]
    for qi in range(nq):
        order = np.lexsort((np.arange(L), -S[qi]))[:nprobe]
        probes[qi] = order
        cand_ids, cand_sc = [], []
        for l in order:
            if len(index.ids[l]) == 0:
                continue
            recon = index.c[index.codes[l]]                       # [n_l, d] centroid values
            est = S[qi, l] + index.gamma16[l].astype(np.float64) * (recon @ Z[qi])
            cand_ids.append(index.ids[l])
            cand_sc.append(est)
        if cand_ids:
            cid = np.concatenate(cand_ids)
            csc = np.concatenate(cand_sc)
        else:
            cid = np.empty(0, np.int64)
            csc = np.empty(0)
        top = np.lexsort((cid, -csc))[:k]
        scores[qi, :len(top)] = csc[top]
        ids[qi, :len(top)] = cid[top]
        if return_all:
            everything.append((cid, csc))
    if return_all:
        return scores, ids, probes, S, everything
    return scores, ids, probes, S


# --------------------------------------------------------------------------
# Raw metrics: inner product and squared L2 distance of un-normalised vectors
# --------------------------------------------------------------------------
#
# The paper normalises everything, so that cosine, inner product and L2 rank alike.  For inputs whose
# lengths matter one more number per vector is kept, |x| as float32, and the estimate s^ of <q~, x~>
# is turned into the metric by the identities of the header.  Probing is unchanged.


def raw_norms_fp32(X):
    """|x| of every row, computed in double and rounded to the float32 that is stored."""
    X = np.asarray(X, dtype=np.float64)
    return np.sqrt(np.sum(X * X, axis=1)).astype(np.float32)


def metric_value(s_hat, xnorm, qnorm, metric: str):
    """Estimated <q, x> ('ip') or |q - x|^2 ('l2') from the estimate s_hat of <q~, x~>."""
    s_hat = np.asarray(s_hat, dtype=np.float64)
    xnorm = np.asarray(xnorm, dtype=np.float64)
    if metric == "ip":
        return qnorm * xnorm * s_hat
    if metric == "l2":
        return qnorm * qnorm + xnorm * xnorm - 2.0 * qnorm * xnorm * s_hat
    raise ValueError(metric)


def search_raw(index: ListIndex, xnorm_by_id, Q, nprobe: int, k: int, metric: str, return_all: bool = False):
    """Search of a raw-metric index.  xnorm_by_id[label] = stored float32 |x| of that vector.  Candidates are
    those of `search` (same probes, same estimates); they are ranked by the metric value, best first
    (ip: largest, l2: smallest; ties -> smaller id), padded with (-1, -inf) or (-1, +inf).
    Returns (values [nq, k], ids [nq, k], probes, coarse scores[, per-query (ids, values)])."""
    Q = np.asarray(Q)
    nq = Q.shape[0]
    qnorm = np.sqrt(np.sum(np.asarray(Q, dtype=np.float64) ** 2, axis=1))
    _, _, probes, S, everything = search(index, Q, nprobe, 1, return_all=True)
    worst = -np.inf if metric == "ip" else np.inf
    values = np.full((nq, k), worst)
    ids = np.full((nq, k), -1, dtype=np.int64)
    all_out = []
    for qi in range(nq):
        cid, s_hat = everything[qi]
        val = metric_value(s_hat, np.asarray(xnorm_by_id)[cid], qnorm[qi], metric) if len(cid) else np.empty(0)
        key = -val if metric == "ip" else val
        top = np.lexsort((cid, key))[:k]
        values[qi, :len(top)] = val[top]
        ids[qi, :len(top)] = cid[top]
        all_out.append((cid, val))
    if return_all:
        return values, ids, probes, S, all_out
    return values, ids, probes, S


def exact_topk_raw(X, Q, k: int, metric: str):
    """Exact k best of the raw metric, straight from its definition (ties -> smaller id)."""
    X = np.asarray(X, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    ids = np.empty((Q.shape[0], k), dtype=np.int64)
    vals = np.empty((Q.shape[0], k))
    for qi in range(Q.shape[0]):
        if metric == "ip":
            v = X @ Q[qi]
            key = -v
        else:
            diff = X - Q[qi][None, :]
            v = np.sum(diff * diff, axis=1)
            key = v
        top = np.lexsort((np.arange(len(v)), key))[:k]
        ids[qi], vals[qi] = top, v[top]
    return vals, ids


# --------------------------------------------------------------------------
# Cascade search (Appendix "Cascade search via Lloyd-Max bin ordinality")
# --------------------------------------------------------------------------
#
# Pass 1 scores every candidate from the top beta bits of each stored code alone, with a codebook of
# 2^beta values; the n_keep best go to pass 2, which scores them with the full codes.  The appendix
# does not spell the coarsened codebook out.  Reading taken here: dropping the low bits of a code
# merges 2^(bits-beta) neighbouring bins into one, and the value of a merged bin is what a Lloyd-Max
# codebook would put there, the mean of the coordinate density over it, i.e. the mass-weighted mean
# of the member levels (each of which is the mean of its own bin).


def coarsened_codebook(levels, boundaries, d: int, beta: int, density: str = "sphere"):
    """2^beta values for the top beta bits of a code whose full table is (levels, boundaries)."""
    levels = np.asarray(levels, dtype=np.float64)
    K = len(levels)
    bits = int(round(np.log2(K)))
    if not (1 <= beta <= bits) or (1 << bits) != K:
        raise ValueError("beta must lie between 1 and the stored bits")
    mass = bin_masses(boundaries, d, density)
    group = 1 << (bits - beta)
    m = mass.reshape(-1, group)
    return (m * levels.reshape(-1, group)).sum(axis=1) / m.sum(axis=1)


def cascade_search(index: ListIndex, Q, nprobe: int, k: int, beta: int, n_keep: int, c_coarse,
                   return_kept: bool = False):
    """Two-pass search.  Probes as in search(); then per query

      pass 1: s1 = s_l + float(gamma16_i) * sum_j z_j * c_coarse[code_ij >> (bits - beta)]
              keep the n_keep candidates with the largest s1 (ties -> smaller id)
      pass 2: score = s_l + float(gamma16_i) * sum_j z_j * c[code_ij]  for the kept ones
      result: k largest scores (ties -> smaller id), padded with (-1, -inf)

    return_kept adds, per query, (ids, pass-1 scores) of every candidate and the kept ids.
    """
    c_coarse = np.asarray(c_coarse, dtype=np.float64)
    bits = int(round(np.log2(len(index.c))))
    shift = bits - beta
    assert len(c_coarse) == 1 << beta
    Qn = normalize_rows(Q)
    nq = Qn.shape[0]
    S = Qn @ index.centroids.T
    Z = Qn @ index.Pi.T
    L = index.centroids.shape[0]
    scores = np.full((nq, k), -np.inf)
    ids = np.full((nq, k), -1, dtype=np.int64)
    kept_all = []
    for qi in range(nq):
        order = np.lexsort((np.arange(L), -S[qi]))[:nprobe]
        cid, s1, s2 = [], [], []
        for l in order:
            if len(index.ids[l]) == 0:
                continue
            g = index.gamma16[l].astype(np.float64)
            cid.append(index.ids[l])
            s1.append(S[qi, l] + g * (c_coarse[index.codes[l] >> shift] @ Z[qi]))
            s2.append(S[qi, l] + g * (index.c[index.codes[l]] @ Z[qi]))
        if not cid:
            kept_all.append((np.empty(0, np.int64), np.empty(0), np.empty(0, np.int64)))
            continue
        cid, s1, s2 = np.concatenate(cid), np.concatenate(s1), np.concatenate(s2)
        keep = np.lexsort((cid, -s1))[:n_keep]
        top = keep[np.lexsort((cid[keep], -s2[keep]))[:k]]
        scores[qi, :len(top)] = s2[top]
        ids[qi, :len(top)] = cid[top]
        kept_all.append((cid, s1, cid[keep]))
    if return_kept:
        return scores, ids, kept_all
    return scores, ids


def reconstruct(index: ListIndex, l: int):
    """x^ = c~_l + gamma * Pi^T c[code]  for every vector of list l (Adaptive refresh, Sec. 3.3)."""
    recon = index.c[index.codes[l]]
    return index.centroids[l][None, :] + index.gamma16[l].astype(np.float64)[:, None] * (recon @ index.Pi)


def stratified_positions(sizes, sample_n: int):
    """Which stored vectors a refresh samples: list l contributes round(sample_n * n_l / N) of its n_l
    vectors (at least one when it is not empty, never more than it holds), evenly spaced in storage
    order: position floor(t * n_l / s_l), t = 0 .. s_l - 1.  Returns a list of position arrays."""
    sizes = np.asarray(sizes, dtype=np.int64)
    total = int(sizes.sum())
    out = []
    for n_l in sizes:
        n_l = int(n_l)
        if n_l == 0 or total == 0:
            out.append(np.empty(0, np.int64))
            continue
        s_l = int(min(n_l, max(1, (2 * sample_n * n_l + total) // (2 * total))))   # round half up
        out.append((np.arange(s_l, dtype=np.int64) * n_l) // s_l)
    return out


def refresh_coarse(index: ListIndex, sample_n: int, niter: int, init_idx=None, new_centroids=None):
    """Adaptive coarse refresh (Section "Adaptive coarse refresh", Algorithm and Refresh
    self-containedness): sample the stored vectors stratified across partitions, reconstruct them as
    x^ = c~_old + gamma * Pi^T rho^, re-cluster the sample, then re-assign and re-encode every stored
    vector from its reconstruction against the new centroids with the unchanged (Pi, C_b).

    init_idx: rows of the sample used as initial k-means centres.  new_centroids: skip the clustering
    and use these (lets a test give both implementations the same partition).
    Returns (new index, reconstructions [N, d] in storage order, labels [N], sample [S, d])."""
    L = len(index.ids)
    recon = [reconstruct(index, l) if len(index.ids[l]) else np.empty((0, index.centroids.shape[1])) for l in range(L)]
    pos = stratified_positions([len(index.ids[l]) for l in range(L)], sample_n)
    sample = np.concatenate([recon[l][pos[l]] for l in range(L)], axis=0)
    if new_centroids is None:
        new_centroids, _ = train_coarse(sample, L, niter, init_idx)
    xh = np.concatenate(recon, axis=0)
    labels = np.concatenate([np.asarray(index.ids[l], dtype=np.int64) for l in range(L)])
    fresh = ListIndex(new_centroids, index.Pi, index.c, index.tau)
    fresh.add(xh, labels)
    return fresh, xh, labels, sample


def tq_reconstruct(V, Pi, c, tau):
    """v^ = Pi^T C_b(Pi v) for rows v (flat TQ; Theorem 1 setup)."""
    U = np.asarray(V, dtype=np.float64) @ np.asarray(Pi, dtype=np.float64).T
    return np.asarray(c, dtype=np.float64)[quantize(U, tau)] @ np.asarray(Pi, dtype=np.float64)


# --------------------------------------------------------------------------
# Ground truth
# --------------------------------------------------------------------------


def exact_topk(X, Q, k: int, chunk: int = 256):
    """Exact k nearest by inner product of normalised rows (ties -> smaller id)."""
    Xn = normalize_rows(X)
    Qn = normalize_rows(Q)
    ids = np.empty((Qn.shape[0], k), dtype=np.int64)
    sc = np.empty((Qn.shape[0], k))
    for s in range(0, Qn.shape[0], chunk):
        S = Qn[s:s + chunk] @ Xn.T
        for r in range(S.shape[0]):
            top = np.lexsort((np.arange(S.shape[1]), -S[r]))[:k]
            ids[s + r] = top
            sc[s + r] = S[r, top]
    return sc, ids


def rerank(X, Q, cand_ids, k: int):
    """Re-ranking on raw vectors (Section "Architecture", Search: optional; "Bits vs. re-ranking"):
    the candidates' exact inner products <q~, x~> replace the estimates and the k best are kept
    (ties -> smaller id).  cand_ids: [nq, r] row numbers of X, -1 = no candidate."""
    X = np.asarray(X)
    Qn = normalize_rows(Q)
    cand_ids = np.asarray(cand_ids, dtype=np.int64)
    nq = cand_ids.shape[0]
    scores = np.full((nq, k), -np.inf)
    ids = np.full((nq, k), -1, dtype=np.int64)
    for qi in range(nq):
        c = np.unique(cand_ids[qi][cand_ids[qi] >= 0])
        if len(c) == 0:
            continue
        s = normalize_rows(X[c]) @ Qn[qi]
        top = np.lexsort((c, -s))[:k]
        scores[qi, :len(top)] = s[top]
        ids[qi, :len(top)] = c[top]
    return scores, ids


def recall_at_k(found_ids, true_ids) -> float:
    k = true_ids.shape[1]
    hits = 0
    for f, t in zip(found_ids, true_ids):
        hits += len(set(int(x) for x in f if x >= 0) & set(int(x) for x in t))
    return hits / (k * len(true_ids))


# --------------------------------------------------------------------------
# Bounds the paper states (used as checks, not by the method)
# --------------------------------------------------------------------------


def theorem1_bound(D_b: float, R_d: float, d: int, delta: float) -> float:
    """sqrt(D_b) + R_d + sqrt(8 log(2/delta) / (d-2))   (Theorem 1)."""
    return math.sqrt(D_b) + R_d + math.sqrt(8.0 * math.log(2.0 / delta) / (d - 2))


def theorem2_terms(D_b: float, b: int, d: int, delta: float, c_marg: float = 0.0):
    """The four terms of the uniform inner-product bound (Theorem 2, appendix form)."""
    bias = (math.sqrt(2.0 * b * math.log(2.0)) + 1.0) * math.sqrt(2.0 * math.log(2.0 / delta) / (d - 2)) \
        + c_marg / d
    rand = math.sqrt(2.0 * D_b * (d * math.log(3.0 * d) + math.log(2.0 / delta)) / (d - 1))
    return D_b, bias, rand, 2.0 / d


def bits_per_vector(b: int, d: int, sign_bit: bool) -> int:
    """b*d code bits (+ d sign bits) + 32 bits of centroid id and float16 norm (Bit accounting)."""
    return b * d + (d if sign_bit else 0) + 32
