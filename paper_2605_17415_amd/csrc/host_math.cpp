// Host-side constants of IVF-TQ: the (b, d) Lloyd-Max codebook and the Haar rotation.
// Both depend on no data (Section "TurboQuant: data-independent scalar quantization";
// Appendix "Proofs of the rate-distortion bounds", Setup and Lemma 1).  Double precision.
#include "host_math.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

namespace ivftq {

namespace {

// Nodes and weights of n-point Gauss-Legendre quadrature on [-1, 1] by Newton iteration on P_n.
void gauss_legendre(int n, std::vector<double>& x, std::vector<double>& w) {
    x.assign(n, 0.0);
    w.assign(n, 0.0);
    const double pi = 3.14159265358979323846;
    for (int i = 0; i < (n + 1) / 2; ++i) {
        double z = std::cos(pi * (i + 0.75) / (n + 0.5));
        double pp = 0.0;
        for (int it = 0; it < 100; ++it) {
            double p1 = 1.0, p2 = 0.0;
            for (int j = 0; j < n; ++j) {
                double p3 = p2;
                p2 = p1;
                p1 = ((2.0 * j + 1.0) * z * p2 - j * p3) / (j + 1.0);
            }
            pp = n * (z * p1 - p2) / (z * z - 1.0);
            double dz = p1 / pp;
            z -= dz;
            if (std::fabs(dz) < 1e-16) break;
        }
        x[i] = -z;
        x[n - 1 - i] = z;
        w[i] = w[n - 1 - i] = 2.0 / ((1.0 - z * z) * pp * pp);
    }
}

// With t = sin(theta) the sphere-coordinate density becomes kappa * cos^(d-2)(theta) d(theta),
// which is smooth on the whole interval; integrate it there.
struct SphereMarginal {
    int d;
    double log_kappa;
    std::vector<double> gx, gw;
    explicit SphereMarginal(int d_) : d(d_) {
        log_kappa = std::lgamma(0.5 * d) - 0.5 * std::log(3.14159265358979323846) - std::lgamma(0.5 * (d - 1));
        gauss_legendre(48, gx, gw);
    }
    // P(a <= T <= b)
    double mass(double a, double b) const {
        double ta = std::asin(std::max(-1.0, std::min(1.0, a)));
        double tb = std::asin(std::max(-1.0, std::min(1.0, b)));
        const int pieces = 6;
        double total = 0.0;
        for (int p = 0; p < pieces; ++p) {
            double lo = ta + (tb - ta) * p / pieces, hi = ta + (tb - ta) * (p + 1) / pieces;
            double half = 0.5 * (hi - lo), mid = 0.5 * (hi + lo), s = 0.0;
            for (size_t i = 0; i < gx.size(); ++i) {
                double c = std::cos(mid + half * gx[i]);
                s += gw[i] * std::exp(log_kappa + (d - 2) * std::log(std::max(c, 1e-300)));
            }
            total += half * s;
        }
        return total;
    }
    double pdf(double t) const {
        const double c2 = 1.0 - t * t;
        return c2 > 0.0 ? std::exp(log_kappa + 0.5 * (d - 3) * std::log(c2)) : 0.0;
    }
    // E[T ; a <= T <= b] in closed form: kappa/(d-1) * [(1-a^2)^((d-1)/2) - (1-b^2)^((d-1)/2)]
    double first_moment(double a, double b) const {
        double k = std::exp(log_kappa) / (d - 1);
        return k * (std::pow(std::max(0.0, 1.0 - a * a), 0.5 * (d - 1)) -
                    std::pow(std::max(0.0, 1.0 - b * b), 0.5 * (d - 1)));
    }
};

}  // namespace

// One Lloyd step T(c): boundaries at the midpoints, centroids at the conditional means.  Only the
// upper half is integrated (the density is even).  Also returns, per bin, the probability mass.
static void lloyd_step(const SphereMarginal& f, const std::vector<double>& cent, std::vector<double>& edge,
                       std::vector<double>& next, std::vector<double>& mass) {
    const int K = (int)cent.size();
    edge[0] = -1.0;
    edge[K] = 1.0;
    for (int i = 1; i < K; ++i) edge[i] = 0.5 * (cent[i - 1] + cent[i]);
    for (int i = K / 2; i < K; ++i) {
        mass[i] = f.mass(edge[i], edge[i + 1]);
        next[i] = f.first_moment(edge[i], edge[i + 1]) / mass[i];
        mass[K - 1 - i] = mass[i];
        next[K - 1 - i] = -next[i];
    }
}

bool build_codebook(int b, int d, std::vector<double>& cent, std::vector<double>& bnd) {
    if (b < 1 || b > 8 || d < 3) return false;
    const int K = 1 << b;
    SphereMarginal f(d);
    cent.resize(K);
    bnd.resize(K - 1);
    const double sd = 1.0 / std::sqrt((double)d);
    // start from a uniform grid over three standard deviations, kept inside the support (-1, 1)
    const double span = std::min(3.0 * sd, 1.0);
    for (int i = 0; i < K; ++i) cent[i] = ((i + 0.5) / K * 2.0 - 1.0) * span;
    std::vector<double> edge(K + 1), next(K), mass(K);
    // The Lloyd-Max quantiser is the solution of c = T(c).  Plain Lloyd iteration c <- T(c) converges
    // linearly with a rate that approaches 1 as K grows (hundreds of thousands of steps at K = 256),
    // so after a short warm-up the same equations are solved by Newton's method: the Jacobian of T is
    // tridiagonal, dT_i/d(edge) = f(edge) * |T_i - edge| / mass_i at either edge of bin i, and each
    // interior edge moves by half of either neighbouring centroid.
    for (int it = 0; it < 64; ++it) {
        lloyd_step(f, cent, edge, next, mass);
        cent = next;
    }
    std::vector<double> lo(K), di(K), up(K), rhs(K), trial(K);
    double resid = 1e300;
    for (int it = 0; it < 200; ++it) {
        lloyd_step(f, cent, edge, next, mass);
        double r = 0.0;
        for (int i = 0; i < K; ++i) r = std::max(r, std::fabs(next[i] - cent[i]));
        if (r < 1e-14 || (r < 1e-12 && r >= resid)) { cent = next; break; }   // at the rounding floor of the quadrature
        resid = r;
        // (I - J_T) delta = T(c) - c
        for (int i = 0; i < K; ++i) {
            const double dl = i > 0 ? f.pdf(edge[i]) * (next[i] - edge[i]) / mass[i] : 0.0;
            const double du = i < K - 1 ? f.pdf(edge[i + 1]) * (edge[i + 1] - next[i]) / mass[i] : 0.0;
            lo[i] = -0.5 * dl;
            up[i] = -0.5 * du;
            di[i] = 1.0 - 0.5 * (dl + du);
            rhs[i] = next[i] - cent[i];
        }
        for (int i = 1; i < K; ++i) {                 // Thomas algorithm
            const double m = lo[i] / di[i - 1];
            di[i] -= m * up[i - 1];
            rhs[i] -= m * rhs[i - 1];
        }
        trial[K - 1] = rhs[K - 1] / di[K - 1];
        for (int i = K - 2; i >= 0; --i) trial[i] = (rhs[i] - up[i] * trial[i + 1]) / di[i];
        bool ordered = true;
        for (int i = 0; i < K; ++i) {
            trial[i] += cent[i];
            if (!std::isfinite(trial[i]) || std::fabs(trial[i]) >= 1.0 || (i > 0 && !(trial[i] > trial[i - 1]))) ordered = false;
        }
        cent = ordered ? trial : next;               // a Newton step that leaves the ordered cone is replaced by a Lloyd step
        for (int i = 0; i < K / 2; ++i) {             // T is evaluated on the upper half only: keep c exactly antisymmetric
            const double v = 0.5 * (cent[K - 1 - i] - cent[i]);
            cent[K - 1 - i] = v;
            cent[i] = -v;
        }
    }
    for (int i = 0; i < K / 2; ++i) {                 // exact antisymmetry
        const double v = 0.5 * (cent[K - 1 - i] - cent[i]);
        cent[K - 1 - i] = v;
        cent[i] = -v;
    }
    for (int i = 1; i < K; ++i) bnd[i - 1] = 0.5 * (cent[i - 1] + cent[i]);
    for (int i = 0; i < K; ++i)
        if (!std::isfinite(cent[i]) || (i > 0 && !(cent[i] > cent[i - 1]))) return false;
    // the result must satisfy the Lloyd-Max conditions themselves
    lloyd_step(f, cent, edge, next, mass);
    for (int i = 0; i < K; ++i)
        if (std::fabs(next[i] - cent[i]) > 1e-12) return false;
    return true;
}

bool build_refined_codebook(int b, int d, std::vector<double>& levels, std::vector<double>& boundaries) {
    std::vector<double> cent, bnd;
    if (b < 1 || b > 7 || !build_codebook(b, d, cent, bnd)) return false;
    const int K = 1 << b;
    SphereMarginal f(d);
    levels.resize(2 * (size_t)K);
    boundaries.resize(2 * (size_t)K - 1);
    for (int i = 0; i < K; ++i) {
        const double lo = i == 0 ? -1.0 : bnd[i - 1], hi = i == K - 1 ? 1.0 : bnd[i];
        const double edge[3] = {lo, cent[i], hi};
        for (int s = 0; s < 2; ++s) {
            const double m = f.mass(edge[s], edge[s + 1]);
            if (!(m > 0.0)) return false;
            levels[2 * i + s] = f.first_moment(edge[s], edge[s + 1]) / m;
        }
        boundaries[2 * i] = cent[i];
        if (i < K - 1) boundaries[2 * i + 1] = bnd[i];
    }
    for (size_t i = 1; i < levels.size(); ++i)
        if (!(levels[i] > levels[i - 1])) return false;
    return true;
}

bool build_coarsened_levels(int d, const std::vector<double>& levels, const std::vector<double>& boundaries,
                            int beta, std::vector<double>& out) {
    const size_t K = levels.size();
    int bits = 0;
    while (((size_t)1 << bits) < K) ++bits;
    if (K < 2 || ((size_t)1 << bits) != K || boundaries.size() != K - 1 || beta < 1 || beta > bits || d < 3) return false;
    SphereMarginal f(d);
    const size_t group = (size_t)1 << (bits - beta);
    out.assign((size_t)1 << beta, 0.0);
    for (size_t g = 0; g < out.size(); ++g) {
        double m0 = 0.0, m1 = 0.0;
        for (size_t i = g * group; i < (g + 1) * group; ++i) {
            const double lo = i == 0 ? -1.0 : boundaries[i - 1], hi = i == K - 1 ? 1.0 : boundaries[i];
            const double m = f.mass(lo, hi);
            m0 += m;
            m1 += m * levels[i];
        }
        if (!(m0 > 0.0)) return false;
        out[g] = m1 / m0;
    }
    return true;
}

// ---- random numbers for the rotation draw ------------------------------------------------

static inline uint64_t splitmix64(uint64_t& s) {
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

void gaussian_matrix(int d, uint64_t seed, std::vector<double>& g) {
    g.resize((size_t)d * d);
    uint64_t s = seed ^ 0xD1B54A32D192ED03ull;
    const double two_pi = 6.28318530717958647692;
    for (size_t i = 0; i < g.size(); i += 2) {
        double u1 = ((splitmix64(s) >> 11) + 1.0) * (1.0 / 9007199254740993.0);  // (0,1)
        double u2 = (splitmix64(s) >> 11) * (1.0 / 9007199254740992.0);          // [0,1)
        double r = std::sqrt(-2.0 * std::log(u1));
        g[i] = r * std::cos(two_pi * u2);
        if (i + 1 < g.size()) g[i + 1] = r * std::sin(two_pi * u2);
    }
}

// Householder QR of the d x d row-major matrix g; returns Q with column j multiplied by
// sign(R_jj), the factor of the unique QR decomposition with positive diagonal.
bool haar_from_gaussian(int d, const double* g, std::vector<double>& q) {
    std::vector<double> a(g, g + (size_t)d * d);       // becomes R
    std::vector<std::vector<double>> vs(d);
    std::vector<double> rdiag(d);
    for (int k = 0; k < d; ++k) {
        double nrm = 0.0;
        for (int i = k; i < d; ++i) nrm += a[(size_t)i * d + k] * a[(size_t)i * d + k];
        nrm = std::sqrt(nrm);
        if (nrm == 0.0) return false;
        double alpha = a[(size_t)k * d + k] >= 0 ? -nrm : nrm;
        std::vector<double> v(d - k);
        for (int i = k; i < d; ++i) v[i - k] = a[(size_t)i * d + k];
        v[0] -= alpha;
        double vn = 0.0;
        for (double t : v) vn += t * t;
        vn = std::sqrt(vn);
        if (vn > 0) for (double& t : v) t /= vn;
        for (int j = k; j < d; ++j) {                  // a <- (I - 2 v v^T) a
            double dot = 0.0;
            for (int i = k; i < d; ++i) dot += v[i - k] * a[(size_t)i * d + j];
            for (int i = k; i < d; ++i) a[(size_t)i * d + j] -= 2.0 * v[i - k] * dot;
        }
        rdiag[k] = a[(size_t)k * d + k];
        vs[k] = std::move(v);
    }
    q.assign((size_t)d * d, 0.0);
    for (int i = 0; i < d; ++i) q[(size_t)i * d + i] = 1.0;
    for (int k = d - 1; k >= 0; --k) {                 // Q = H_0 H_1 ... H_{d-1}
        const std::vector<double>& v = vs[k];
        for (int j = 0; j < d; ++j) {
            double dot = 0.0;
            for (int i = k; i < d; ++i) dot += v[i - k] * q[(size_t)i * d + j];
            for (int i = k; i < d; ++i) q[(size_t)i * d + j] -= 2.0 * v[i - k] * dot;
        }
    }
    for (int j = 0; j < d; ++j)
        if (rdiag[j] < 0)
            for (int i = 0; i < d; ++i) q[(size_t)i * d + j] = -q[(size_t)i * d + j];
    return true;
}

double orthogonality_defect(int d, const float* pi) {
    double sum = 0.0;
    for (int i = 0; i < d; ++i)
        for (int j = i; j < d; ++j) {
            double dot = 0.0;
            for (int k = 0; k < d; ++k) dot += (double)pi[(size_t)i * d + k] * (double)pi[(size_t)j * d + k];
            const double e = dot - (i == j ? 1.0 : 0.0);
            sum += (i == j ? 1.0 : 2.0) * e * e;
        }
    return std::sqrt(sum);
}

bool build_quantiser_grid(const std::vector<float>& tau, int max_cells, QuantiserGrid& grid) {
    const int nb = (int)tau.size();
    if (nb < 1) return false;
    if (nb == 1) {
        grid.cells = 1;
        grid.scale = 0.f;
        grid.offset = 0.f;
        grid.boundary.assign(1, tau[0]);
        grid.index.assign(1, 0);
        return true;
    }
    double gap = 1e300;
    for (int i = 1; i < nb; ++i) {
        if (!(tau[i] > tau[i - 1])) return false;
        gap = std::min(gap, (double)tau[i] - (double)tau[i - 1]);
    }
    const double w = 0.5 * gap;
    const double lo = (double)tau[0] - w;
    const int cells = (int)std::ceil(((double)tau[nb - 1] + w - lo) / w) + 1;
    if (cells > max_cells) return false;
    grid.cells = cells;
    grid.scale = (float)(1.0 / w);
    grid.offset = (float)(-lo / w);
    grid.boundary.resize(cells);
    grid.index.resize(cells);
    int near = 0;
    for (int i = 0; i < cells; ++i) {
        const double mid = lo + (i + 0.5) * w;
        while (near + 1 < nb && std::fabs((double)tau[near + 1] - mid) < std::fabs((double)tau[near] - mid)) ++near;
        grid.boundary[i] = tau[near];
        grid.index[i] = near;
    }
    return true;
}

}  // namespace ivftq
