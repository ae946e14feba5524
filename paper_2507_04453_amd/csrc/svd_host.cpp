// One-sided (Hestenes) Jacobi thin SVD in fp64, used once per LoRA factor at set-up time
// (paper: Algorithm 1, SVD-init step).  Host only.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "essa_internal.h"

void essa_host_thin_svd(const double* G, int m, int r, double* U, double* s, double* V) {
    // work on columns stored contiguously: W[j] = column j of G
    std::vector<double> W((size_t)r * m), Vc((size_t)r * r, 0.0);
    for (int j = 0; j < r; ++j) {
        for (int i = 0; i < m; ++i) W[(size_t)j * m + i] = G[(size_t)i * r + j];
        Vc[(size_t)j * r + j] = 1.0;   // Vc[j] = column j of V
    }
    const double eps = 1e-15;
    for (int sweep = 0; sweep < 60; ++sweep) {
        bool rotated = false;
        for (int p = 0; p < r - 1; ++p) {
            for (int q = p + 1; q < r; ++q) {
                double* wp = &W[(size_t)p * m];
                double* wq = &W[(size_t)q * m];
                double a = 0, b = 0, g = 0;
                for (int i = 0; i < m; ++i) { a += wp[i] * wp[i]; b += wq[i] * wq[i]; g += wp[i] * wq[i]; }
                if (std::fabs(g) <= eps * std::sqrt(a * b) || g == 0.0) continue;
                rotated = true;
                double zeta = (b - a) / (2.0 * g);
                double t = (zeta >= 0 ? 1.0 : -1.0) / (std::fabs(zeta) + std::sqrt(1.0 + zeta * zeta));
                double c = 1.0 / std::sqrt(1.0 + t * t), sn = c * t;
                for (int i = 0; i < m; ++i) {
                    double x = wp[i], y = wq[i];
                    wp[i] = c * x - sn * y;
                    wq[i] = sn * x + c * y;
                }
                double* vp = &Vc[(size_t)p * r];
                double* vq = &Vc[(size_t)q * r];
                for (int i = 0; i < r; ++i) {
                    double x = vp[i], y = vq[i];
                    vp[i] = c * x - sn * y;
                    vq[i] = sn * x + c * y;
                }
            }
        }
        if (!rotated) break;
    }
    std::vector<double> norms(r);
    for (int j = 0; j < r; ++j) {
        double a = 0;
        for (int i = 0; i < m; ++i) a += W[(size_t)j * m + i] * W[(size_t)j * m + i];
        norms[j] = std::sqrt(a);
    }
    std::vector<int> idx(r);
    std::iota(idx.begin(), idx.end(), 0);
    std::stable_sort(idx.begin(), idx.end(), [&](int x, int y) { return norms[x] > norms[y]; });
    for (int jj = 0; jj < r; ++jj) {
        int j = idx[jj];
        s[jj] = norms[j];
        double inv = norms[j] > 0 ? 1.0 / norms[j] : 0.0;   // a null direction gets a zero vector
        for (int i = 0; i < m; ++i) U[(size_t)i * r + jj] = W[(size_t)j * m + i] * inv;
        for (int i = 0; i < r; ++i) V[(size_t)i * r + jj] = Vc[(size_t)j * r + i];
    }
}
