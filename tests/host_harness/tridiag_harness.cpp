// Host harness for the tridiagonal eigen-solver, built with AddressSanitizer and UndefinedBehaviorSanitizer by
// tests/test_host_sanitizers.py.  Solves a family of matrices (sizes 1..255, wide dynamic range, decoupled blocks,
// repeated and zero entries) and checks T Z = Z diag(u), Z^T Z = I and the ordering; any sanitizer report aborts.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

namespace fosi { int tridiag_eigh(int m, const double* alpha, const double* beta, double* evals, double* evecs); }

static unsigned long long state = 88172645463325252ull;
static double uniform() {                       // xorshift64, values in [0, 1)
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0;
}

static int check(int m, const std::vector<double>& a, const std::vector<double>& b, bool vectors) {
    std::vector<double> u(m), Z(vectors ? (size_t)m * m : 0);
    if (fosi::tridiag_eigh(m, a.data(), m > 1 ? b.data() : nullptr, u.data(), vectors ? Z.data() : nullptr) != 0) return 1;
    double scale = 0.0;
    for (int i = 0; i < m; ++i) scale = std::fmax(scale, std::fabs(a[i]) + (i + 1 < m ? std::fabs(b[i]) : 0.0));
    if (scale == 0.0) scale = 1.0;
    for (int i = 1; i < m; ++i) if (u[i] < u[i - 1]) return 2;
    if (!vectors) return 0;
    for (int j = 0; j < m; ++j) {
        for (int i = 0; i < m; ++i) {             // residual of column j, row i
            double r = a[i] * Z[(size_t)j * m + i] - u[j] * Z[(size_t)j * m + i];
            if (i > 0) r += b[i - 1] * Z[(size_t)j * m + i - 1];
            if (i + 1 < m) r += b[i] * Z[(size_t)j * m + i + 1];
            if (std::fabs(r) > 1e-10 * scale * m) return 3;
        }
        for (int k = 0; k <= j; ++k) {            // orthonormality
            double d = 0.0;
            for (int i = 0; i < m; ++i) d += Z[(size_t)j * m + i] * Z[(size_t)k * m + i];
            if (std::fabs(d - (j == k ? 1.0 : 0.0)) > 1e-10 * m) return 4;
        }
    }
    return 0;
}

int main() {
    int cases = 0;
    const int sizes[] = {1, 2, 3, 4, 7, 16, 33, 61, 80, 100, 101, 128, 255};
    for (int m : sizes) {
        for (int kind = 0; kind < 6; ++kind) {
            std::vector<double> a(m), b(m > 1 ? m - 1 : 1);
            for (int i = 0; i < m; ++i) {
                const double mag = kind == 1 ? std::pow(10.0, 8.0 * uniform() - 4.0) : 1.0;
                a[i] = kind == 4 ? 2.0 : (2.0 * uniform() - 1.0) * mag;
                if (i + 1 < m) {
                    b[i] = kind == 2 && i % 5 == 4 ? 0.0 : kind == 4 ? 1.0 : uniform() * mag;
                    if (kind == 3) b[i] *= 1e-300;       // off-diagonal at the underflow edge
                }
            }
            if (kind == 5) { for (auto& x : a) x = 0.0; for (auto& x : b) x = 0.0; }
            for (int vec = 0; vec < 2; ++vec) {
                const int rc = check(m, a, b, vec != 0);
                if (rc != 0) { std::printf("FAILED m=%d kind=%d vectors=%d rc=%d\n", m, kind, vec, rc); return 1; }
                ++cases;
            }
        }
    }
    std::printf("tridiag harness ok: %d cases\n", cases);
    return 0;
}
