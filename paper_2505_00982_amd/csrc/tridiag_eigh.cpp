// Host eigen-solver for the symmetric tridiagonal matrix B of Algorithm 1
// (needed for Eq. 8).  Implicit-shift QR iteration with Wilkinson shifts:
// each sweep chases one bulge down the active block with plane rotations,
// which are also applied to the accumulated eigenvector matrix.  float64
// throughout; m is at most a few hundred, so this costs microseconds to a few
// milliseconds and never touches the GPU.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

namespace fosi {

int tridiag_eigh(int m, const double* alpha, const double* beta, double* evals, double* evecs) {
    if (m < 1) return 1;
    std::vector<double> d(alpha, alpha + m), e(m, 0.0);
    for (int i = 0; i + 1 < m; ++i) e[i] = beta[i];
    std::vector<double> Z;
    const bool want_vecs = evecs != nullptr;
    if (want_vecs) {
        Z.assign((size_t)m * m, 0.0);
        for (int i = 0; i < m; ++i) Z[(size_t)i * m + i] = 1.0;   // column-major identity
    }
    const double eps = 2.220446049250313e-16;
    int hi = m - 1;
    long budget = 80L * m + 200;
    while (hi > 0) {
        // deflate converged trailing entries
        if (std::fabs(e[hi - 1]) <= eps * (std::fabs(d[hi - 1]) + std::fabs(d[hi]))) {
            e[hi - 1] = 0.0;
            --hi;
            continue;
        }
        int lo = hi - 1;
        while (lo > 0 && std::fabs(e[lo - 1]) > eps * (std::fabs(d[lo - 1]) + std::fabs(d[lo]))) --lo;
        if (lo > 0) e[lo - 1] = 0.0;
        if (--budget < 0) return 2;
        // Wilkinson shift: eigenvalue of the trailing 2x2 closer to d[hi]
        const double delta = 0.5 * (d[hi - 1] - d[hi]);
        const double eh = e[hi - 1];
        const double denom = delta + (delta >= 0.0 ? 1.0 : -1.0) * std::hypot(delta, eh);
        const double mu = d[hi] - (denom != 0.0 ? eh * eh / denom : 0.0);
        double x = d[lo] - mu;
        double z = e[lo];
        for (int k = lo; k < hi; ++k) {
            const double r = std::hypot(x, z);
            double c = 1.0, s = 0.0;
            if (r != 0.0) { c = x / r; s = z / r; }
            if (k > lo) e[k - 1] = r;
            const double a = d[k], b = e[k], cc = d[k + 1];
            d[k] = c * c * a + 2.0 * c * s * b + s * s * cc;
            d[k + 1] = s * s * a - 2.0 * c * s * b + c * c * cc;
            e[k] = (c * c - s * s) * b + c * s * (cc - a);
            if (k + 1 < hi) {
                z = s * e[k + 1];
                e[k + 1] = c * e[k + 1];
                x = e[k];
            }
            if (want_vecs) {
                double* zk = &Z[(size_t)k * m];
                double* zk1 = zk + m;
                for (int i = 0; i < m; ++i) {
                    const double p = zk[i], q = zk1[i];
                    zk[i] = c * p + s * q;
                    zk1[i] = c * q - s * p;
                }
            }
        }
    }
    std::vector<int> order(m);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int i, int j) { return d[i] < d[j]; });
    for (int j = 0; j < m; ++j) {
        evals[j] = d[order[j]];
        if (want_vecs) std::copy(&Z[(size_t)order[j] * m], &Z[(size_t)order[j] * m] + m, evecs + (size_t)j * m);
    }
    return 0;
}

}  // namespace fosi
