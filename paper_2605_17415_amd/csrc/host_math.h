// Host-side constants of IVF-TQ (double precision): codebook and rotation.
#pragma once
#include <cstdint>
#include <vector>

namespace ivftq {

// K = 2^b Lloyd-Max centroids (ascending) and K-1 midpoints for the sphere-coordinate density.
bool build_codebook(int b, int d, std::vector<double>& centroids, std::vector<double>& boundaries);

// d x d iid N(0,1), row-major, from a 64-bit seed.
void gaussian_matrix(int d, uint64_t seed, std::vector<double>& g);

// Orthogonal factor of g with the sign convention diag(R) > 0 (Haar when g is Gaussian).
bool haar_from_gaussian(int d, const double* g, std::vector<double>& q);

}  // namespace ivftq
