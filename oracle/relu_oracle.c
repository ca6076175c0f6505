/*
 * CPU oracle for the ReLU block (forward and backward).
 *
 * THIS IS TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
 * CPU-baseline leg may call it; the product path never does, and it shares no
 * code with the GPU path.
 *
 * What it follows (MatConvNet manual, arXiv 1412.4564):
 *   - Sec. 4.4 "Activation functions": y_ijd = max{0, x_ijd};
 *   - Sec. 6.4.1: dz/dx = diag(s) dz/dy with s = [x > 0], an indicator (so
 *     the derivative at x = 0 is taken as 0).
 * The block acts element by element, so arrays are plain vectors here.
 * Arithmetic: double.
 */
#include <stdint.h>
#include <stddef.h>

int orr_forward(const double *x, double *y, int64_t n) {
    if (!x || !y || n < 0) return 1;
    for (int64_t e = 0; e < n; ++e) y[e] = x[e] > 0.0 ? x[e] : 0.0;
    return 0;
}

int orr_backward(const double *x, const double *dzdy, double *dzdx, int64_t n) {
    if (!x || !dzdy || !dzdx || n < 0) return 1;
    for (int64_t e = 0; e < n; ++e) dzdx[e] = x[e] > 0.0 ? dzdy[e] : 0.0;
    return 0;
}
