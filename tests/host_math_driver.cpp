// Driver for the sanitizer build of the host-side constants (tests/test_host_sanitizer.py): runs every
// function of host_math.h over a range of (b, d) and prints a checksum.  Built with g++ and
// -fsanitize=address,undefined; any report from the sanitizers fails the test.
#include <cmath>
#include <cstdio>
#include <vector>

#include "host_math.h"

int main() {
    using namespace ivftq;
    double sum = 0.0;
    const int ds[] = {3, 8, 17, 64, 96, 128, 200, 256};
    for (int d : ds) {
        for (int b = 1; b <= 8; ++b) {
            std::vector<double> c, t, lv, bd, co;
            if (!build_codebook(b, d, c, t)) { std::printf("codebook failed b=%d d=%d\n", b, d); return 1; }
            // Stage 1 + sign bit is stored in at most 8 bits: b <= 7
            if (b <= 7 && !build_refined_codebook(b, d, lv, bd)) { std::printf("refined failed b=%d d=%d\n", b, d); return 1; }
            for (int beta = 1; beta <= b; ++beta) {
                if (!build_coarsened_levels(d, c, t, beta, co)) { std::printf("coarsened failed\n"); return 1; }
                sum += co.front();
            }
            std::vector<float> tau(t.begin(), t.end());
            if (!tau.empty()) {
                QuantiserGrid g;
                if (!build_quantiser_grid(tau, 4096, g)) { std::printf("grid failed b=%d d=%d\n", b, d); return 1; }
                sum += g.cells + g.boundary[g.cells / 2] + g.index[g.cells - 1];
            }
            if (b <= 7) {
                std::vector<float> tau2(bd.begin(), bd.end());
                QuantiserGrid g2;
                if (!build_quantiser_grid(tau2, 4096, g2)) { std::printf("refined grid failed b=%d d=%d\n", b, d); return 1; }
                sum += lv.front() + g2.cells;
            }
            sum += c.back();
        }
        std::vector<double> g, q;
        gaussian_matrix(d, 1234 + d, g);
        if (!haar_from_gaussian(d, g.data(), q)) { std::printf("rotation failed d=%d\n", d); return 1; }
        std::vector<float> qf(q.begin(), q.end());
        const double defect = orthogonality_defect(d, qf.data());
        if (!(defect < 1e-5)) { std::printf("rotation not orthogonal d=%d defect=%g\n", d, defect); return 1; }
        sum += q[0] + defect;
    }
    std::printf("ok %.6f\n", sum);
    return std::isfinite(sum) ? 0 : 1;
}
