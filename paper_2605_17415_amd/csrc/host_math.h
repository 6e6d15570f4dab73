// Host-side constants of IVF-TQ (double precision): codebook and rotation.
#pragma once
#include <cstdint>
#include <vector>

namespace ivftq {

// K = 2^b Lloyd-Max centroids (ascending) and K-1 midpoints for the sphere-coordinate density.
bool build_codebook(int b, int d, std::vector<double>& centroids, std::vector<double>& boundaries);

// Stage 1 at b bits plus the sign-bit refinement (Appendix "Sign-bit refinement") written as one
// quantiser of 2K levels: boundaries[2K-1] = the Stage-1 centroids and boundaries interleaved
// (c_0 < tau_1 < c_1 < ...), levels[2i + s] = E[T | T in half-bin (i, s)] under the same density, so
// that #{boundaries <= v} = 2*code + 1[v >= c_code].
bool build_refined_codebook(int b, int d, std::vector<double>& levels, std::vector<double>& boundaries);

// Codebook for the top beta bits of a code whose full table is (levels, boundaries), 2^bits levels
// (Appendix "Cascade search via Lloyd-Max bin ordinality", pass 1): dropping the low bits merges
// 2^(bits-beta) neighbouring bins, and a merged bin takes the mean of the sphere-coordinate density
// over it, the mass-weighted mean of its members' levels.  out has 2^beta entries.
bool build_coarsened_levels(int d, const std::vector<double>& levels, const std::vector<double>& boundaries,
                            int beta, std::vector<double>& out);

// d x d iid N(0,1), row-major, from a 64-bit seed.
void gaussian_matrix(int d, uint64_t seed, std::vector<double>& g);

// Orthogonal factor of g with the sign convention diag(R) > 0 (Haar when g is Gaussian).
bool haar_from_gaussian(int d, const double* g, std::vector<double>& q);

// Frobenius norm of pi * pi^T - I for a d x d row-major matrix.
double orthogonality_defect(int d, const float* pi);

// Uniform-grid index over the ascending quantiser boundaries tau (K-1 of them, K-1 >= 1).  The real
// line is cut into `cells` intervals of equal width (the two outermost ones open-ended); entry i
// holds the boundary nearest to the middle of cell i and that boundary's index, so that for a value v
// falling in cell i  #{j : v >= tau_j} = index_i + (v >= boundary_i).  The cell width is half the
// smallest gap between boundaries, which makes the identity hold also for values up to a quarter
// cell outside the cell they were put in (rounding of the cell computation).
//   cell(v) = clamp(int(v * scale + offset), 0, cells - 1)
struct QuantiserGrid {
    std::vector<float> boundary;   // [cells]
    std::vector<int32_t> index;    // [cells]
    float scale = 0.f, offset = 0.f;
    int cells = 0;
};
bool build_quantiser_grid(const std::vector<float>& tau, int max_cells, QuantiserGrid& grid);

}  // namespace ivftq
