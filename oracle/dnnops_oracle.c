/*
 * CPU oracle for the paper's other memory-bound operators: the Mish activation
 * (section "Evaluation", Mish paragraph: mish(x) = x*tanh(softplus(x)), backward
 * recomputed from x alone), layer normalisation (section "Statistical
 * Normalization": gamma*(x-E[x])/sqrt(Var(x)+eps)+beta over the last dimension)
 * and softmax over the last dimension (section "Softmax": subtract the row
 * maximum, exponentiate, divide by the row sum).
 *
 * TEST INFRASTRUCTURE ONLY: it exists to check the HIP library and to serve as
 * the timed CPU baseline; nothing in the product path may call it and it shares
 * no code with the HIP path.  Everything is fp64 and every loop is the textbook
 * definition; OpenMP only over independent rows / elements.
 *
 * Pins (tests marked "not gpu"): Mish special values, its odd/even
 * decomposition limits, central finite differences and PyTorch fp64 autograd;
 * layer normalisation row invariants (zero mean, variance var/(var+eps)),
 * shift invariance, the affine case, PyTorch fp64 autograd for all three
 * gradients; softmax rows summing to one, shift invariance, the two-element
 * closed form (a sigmoid), PyTorch fp64 autograd.
 */
#include <math.h>
#include <stddef.h>

/* mish(x) = x * tanh(log(1 + e^x)) */
double orc_mish(double x) { return x * tanh(log1p(exp(x))); }

/* d/dx mish = tanh(sp) + x * (1 - tanh(sp)^2) * sigmoid(x), sp = softplus(x) */
double orc_mish_grad(double x)
{
    const double t = tanh(log1p(exp(x)));
    const double s = 1.0 / (1.0 + exp(-x));
    return t + x * (1.0 - t * t) * s;
}

void orc_mish_fwd(size_t n, const double *x, double *y)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i)
        y[i] = orc_mish(x[i]);
}

/* Nothing but x is kept from the forward pass: dx = dy * mish'(x). */
void orc_mish_bwd(size_t n, const double *x, const double *dy, double *dx)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i)
        dx[i] = dy[i] * orc_mish_grad(x[i]);
}

/* Layer normalisation of each row of x[rows][cols] over its cols entries (biased variance). */
void orc_layernorm_fwd(int rows, int cols, const double *x, const double *gamma,
                       const double *beta, double eps, double *y, double *mean, double *rstd)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const double *xr = x + (size_t)r * cols;
        double s = 0.0;
        for (int c = 0; c < cols; ++c)
            s += xr[c];
        const double mu = s / cols;
        double s2 = 0.0;
        for (int c = 0; c < cols; ++c)
            s2 += (xr[c] - mu) * (xr[c] - mu);
        const double rs = 1.0 / sqrt(s2 / cols + eps);
        mean[r] = mu;
        rstd[r] = rs;
        for (int c = 0; c < cols; ++c)
            y[(size_t)r * cols + c] = gamma[c] * ((xr[c] - mu) * rs) + beta[c];
    }
}

/* dbeta[c] = sum_r dy, dgamma[c] = sum_r dy*xhat,
 * dx = rstd * (g - mean_c(g) - xhat * mean_c(g*xhat)) with g = dy*gamma, per row. */
void orc_layernorm_bwd(int rows, int cols, const double *x, const double *dy, const double *gamma,
                       const double *mean, const double *rstd, double *dx, double *dgamma,
                       double *dbeta)
{
    for (int c = 0; c < cols; ++c) {
        double sb = 0.0, sg = 0.0;
        for (int r = 0; r < rows; ++r) {
            const double xh = (x[(size_t)r * cols + c] - mean[r]) * rstd[r];
            sb += dy[(size_t)r * cols + c];
            sg += dy[(size_t)r * cols + c] * xh;
        }
        dbeta[c] = sb;
        dgamma[c] = sg;
    }
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const size_t o = (size_t)r * cols;
        double a = 0.0, b = 0.0;
        for (int c = 0; c < cols; ++c) {
            const double g = dy[o + c] * gamma[c];
            const double xh = (x[o + c] - mean[r]) * rstd[r];
            a += g;
            b += g * xh;
        }
        a /= cols;
        b /= cols;
        for (int c = 0; c < cols; ++c) {
            const double g = dy[o + c] * gamma[c];
            const double xh = (x[o + c] - mean[r]) * rstd[r];
            dx[o + c] = rstd[r] * (g - a - xh * b);
        }
    }
}

/* y[r][c] = exp(x[r][c] - max_c x[r]) / sum_c exp(x[r][c] - max_c x[r]) */
void orc_softmax_fwd(int rows, int cols, const double *x, double *y)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const double *xr = x + (size_t)r * cols;
        double m = xr[0];
        for (int c = 1; c < cols; ++c)
            m = xr[c] > m ? xr[c] : m;
        double s = 0.0;
        for (int c = 0; c < cols; ++c) {
            const double e = exp(xr[c] - m);
            y[(size_t)r * cols + c] = e;
            s += e;
        }
        for (int c = 0; c < cols; ++c)
            y[(size_t)r * cols + c] /= s;
    }
}

/* dx = y * (dy - sum_c dy*y), per row */
void orc_softmax_bwd(int rows, int cols, const double *y, const double *dy, double *dx)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const size_t o = (size_t)r * cols;
        double s = 0.0;
        for (int c = 0; c < cols; ++c)
            s += dy[o + c] * y[o + c];
        for (int c = 0; c < cols; ++c)
            dx[o + c] = y[o + c] * (dy[o + c] - s);
    }
}
