// Principal axes for the improved k-means (Sec. 3.2, step 1: "PCA space of {x'}"): eigen-decomposition of the
// D x D covariance matrix.  Host code, fp64: the matrix is tiny next to the data (D <= 4096) and the work is
// serial by nature -- Householder reduction to tridiagonal form, then implicit-shift QR sweeps (Wilkinson shift)
// on the tridiagonal matrix with every plane rotation applied to the accumulated transformation.  The
// transformation is kept TRANSPOSED (row i = i-th basis vector), so a rotation works on two contiguous rows and
// the result already has the axes as rows, which is how the rotation kernels take R.
#pragma once
#include <math.h>
#include <stddef.h>
#include <algorithm>
#include <numeric>
#include <vector>

namespace hclae {

// A: n x n symmetric, row-major; destroyed.  On return w[0] >= ... >= w[n-1] are the eigenvalues and row i of
// Vt (n x n, row-major) is a unit eigenvector of w[i], signed so that its entry of largest magnitude (the
// first one among equals) is positive.  Returns 0, or -1 when the iteration did not converge (never seen).
inline int symmetric_eigen(double *A, int n, double *w, double *Vt)
{
    if (n <= 0) return 0;
    std::vector<double> d(n), e(n > 1 ? n - 1 : 1, 0.0), beta(n, 0.0), p(n), u(n);
    auto row = [&](int i) { return A + (size_t)i * n; };

    // ---- Householder reduction: H_k = I - beta_k v_k v_k^T acts on coordinates k+1..n-1 and clears column k
    // below the sub-diagonal.  v_k is kept in row k of A (columns k+1..), which is no longer needed then.
    for (int k = 0; k + 2 < n; ++k) {
        double *x = row(k) + k + 1;                                 // = column k below the diagonal, by symmetry
        const int len = n - k - 1;
        double tail = 0.0;
        for (int i = 1; i < len; ++i) tail += x[i] * x[i];
        d[k] = row(k)[k];
        if (tail == 0.0) {                                          // already tridiagonal here
            e[k] = x[0];
            beta[k] = 0.0;
            continue;
        }
        const double norm = sqrt(x[0] * x[0] + tail);
        const double alpha = x[0] > 0.0 ? -norm : norm;
        e[k] = alpha;
        x[0] -= alpha;                                              // x is v from here on
        const double vv = x[0] * x[0] + tail;
        const double b = 2.0 / vv;
        beta[k] = b;
        // trailing block B = A[k+1.., k+1..]:  B <- B - v q^T - q v^T  with  pv = b B v,  q = pv - (b/2)(v.pv) v
        double vp = 0.0;
        for (int i = 0; i < len; ++i) {
            const double *bi = row(k + 1 + i) + k + 1;
            double s = 0.0;
            for (int j = 0; j < len; ++j) s += bi[j] * x[j];
            p[i] = b * s;
            vp += x[i] * p[i];
        }
        const double kc = 0.5 * b * vp;
        for (int i = 0; i < len; ++i) p[i] -= kc * x[i];
        for (int i = 0; i < len; ++i) {
            double *bi = row(k + 1 + i) + k + 1;
            const double vi = x[i], qi = p[i];
            for (int j = 0; j < len; ++j) bi[j] -= vi * p[j] + qi * x[j];
        }
    }
    if (n >= 2) {
        d[n - 2] = row(n - 2)[n - 2];
        e[n - 2] = row(n - 2)[n - 1];
    }
    d[n - 1] = row(n - 1)[n - 1];

    // ---- Q = H_0 H_1 ... H_{n-3}, accumulated from the last reflector backwards into Vt (the part of Q that
    // is not yet the identity is the trailing block, so each step touches only that block); then transposed.
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) Vt[(size_t)i * n + j] = (i == j) ? 1.0 : 0.0;
    for (int k = n - 3; k >= 0; --k) {
        if (beta[k] == 0.0) continue;
        const double *v = row(k) + k + 1;
        const int len = n - k - 1;
        for (int j = 0; j < len; ++j) u[j] = 0.0;
        for (int i = 0; i < len; ++i) {
            const double *qi = Vt + (size_t)(k + 1 + i) * n + k + 1;
            const double vi = v[i];
            for (int j = 0; j < len; ++j) u[j] += vi * qi[j];
        }
        for (int i = 0; i < len; ++i) {
            double *qi = Vt + (size_t)(k + 1 + i) * n + k + 1;
            const double bv = beta[k] * v[i];
            for (int j = 0; j < len; ++j) qi[j] -= bv * u[j];
        }
    }
    for (int i = 0; i < n; ++i)
        for (int j = i + 1; j < n; ++j) std::swap(Vt[(size_t)i * n + j], Vt[(size_t)j * n + i]);

    // ---- implicit-shift QR on the tridiagonal matrix (d, e); rotation of the plane (k, k+1) turns rows k, k+1 of Vt
    const double eps = 2.220446049250313e-16;
    int budget = 64 * n;
    for (;;) {
        for (int i = 0; i + 1 < n; ++i)
            if (fabs(e[i]) <= eps * (fabs(d[i]) + fabs(d[i + 1]))) e[i] = 0.0;
        int hi = n - 1;
        while (hi > 0 && e[hi - 1] == 0.0) --hi;
        if (hi == 0) break;
        int lo = hi - 1;
        while (lo > 0 && e[lo - 1] != 0.0) --lo;
        if (--budget < 0) return -1;
        // Wilkinson shift: the eigenvalue of the trailing 2 x 2 block nearer to d[hi]
        const double dd = 0.5 * (d[hi - 1] - d[hi]), off = e[hi - 1];
        const double den = dd + (dd >= 0.0 ? 1.0 : -1.0) * hypot(dd, off);
        const double mu = d[hi] - (den != 0.0 ? off * off / den : 0.0);
        double x = d[lo] - mu, z = e[lo];
        for (int k = lo; k < hi; ++k) {
            // c, s with [c s; -s c]^T [x; z] = [r; 0]
            const double r = hypot(x, z);
            const double c = r != 0.0 ? x / r : 1.0, s = r != 0.0 ? -z / r : 0.0;
            if (k > lo) e[k - 1] = r;
            const double a = d[k], b = e[k], g = d[k + 1];
            d[k] = c * c * a - 2.0 * c * s * b + s * s * g;
            d[k + 1] = s * s * a + 2.0 * c * s * b + c * c * g;
            e[k] = c * s * (a - g) + (c * c - s * s) * b;
            if (k + 1 < hi) {
                x = e[k];
                z = -s * e[k + 1];                                  // the bulge at (k, k+2)
                e[k + 1] = c * e[k + 1];
            }
            double *rk = Vt + (size_t)k * n, *rk1 = rk + n;
            for (int j = 0; j < n; ++j) {
                const double t0 = rk[j], t1 = rk1[j];
                rk[j] = c * t0 - s * t1;
                rk1[j] = s * t0 + c * t1;
            }
        }
    }

    // ---- descending order (equal values keep their order), sign convention
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return d[a] > d[b]; });
    std::vector<double> tmp((size_t)n * n);
    for (int i = 0; i < n; ++i) {
        w[i] = d[order[i]];
        const double *src = Vt + (size_t)order[i] * n;
        double big = 0.0;
        int at = 0;
        for (int j = 0; j < n; ++j)
            if (fabs(src[j]) > big) { big = fabs(src[j]); at = j; }
        const double sg = src[at] < 0.0 ? -1.0 : 1.0;
        for (int j = 0; j < n; ++j) tmp[(size_t)i * n + j] = sg * src[j];
    }
    std::copy(tmp.begin(), tmp.end(), Vt);
    return 0;
}

}  // namespace hclae
