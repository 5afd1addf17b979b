/*
 * CPU oracle for one training step (forward + backward) of an EfficientNet
 * MBConv block.  TEST INFRASTRUCTURE ONLY: it exists to check the HIP library
 * and to serve as the timed CPU baseline.  Nothing in the product path may
 * call it, and it shares no code, header, table or helper with the HIP path.
 *
 * Everything is fp64, every loop nest is the textbook definition of the
 * operation (no blocking, no fusion, no algebraic shortcuts).  OpenMP is used
 * only on outermost loops whose iterations are independent.
 *
 * What is computed (the block is the one optimised in the paper's EfficientNet
 * guided case study, section "Guided Optimization Case Study: EfficientNet";
 * the paper does not define the block itself, it cites EfficientNet):
 *   1x1 expansion conv -> BN(batch statistics) -> Swish ->
 *   kxk depthwise conv -> BN -> Swish -> squeeze-and-excitation ->
 *   1x1 projection conv -> BN -> optional residual.
 * The MobileNet-V2 inverted-residual block, which the paper also times (table
 * "Automatic optimization results"), is the same chain with ReLU6 in place of
 * Swish and no squeeze-and-excitation stage (desc.activation = 1, has_se = 0).
 * Batch normalisation follows the paper's formula in section "Statistical
 * Normalization": gamma*(x-E[x])/sqrt(Var(x)+eps)+beta, with E and Var taken
 * over (N,H,W) per channel, and the running mean/variance written back as that
 * section says training-mode BN does.
 * The backward pass is the hand-derived vector-Jacobian product of each step
 * (the paper obtains the same thing by symbolic reverse-mode AD, section
 * "Symbolic Automatic Differentiation").
 *
 * Pins (tests marked "not gpu"): 1x1 conv against a library contraction,
 * depthwise conv against a brute-force loop over an explicitly zero-padded
 * copy plus the delta-kernel and all-ones closed forms, BN mean/variance
 * invariants and the running-statistics closed form, Swish closed forms,
 * SE on a spatially constant input, residual with gamma3 = 0, central finite
 * differences for every gradient, linearity of backward in dOut, and an
 * independently assembled PyTorch-CPU fp64 autograd block.  Evaluation mode:
 * the evaluation-mode block fed with a training batch's own (biased) statistics
 * reproduces the training-mode output, the single-value closed form of
 * orc_bn_eval, and the same PyTorch block in eval() mode.
 * Parity unpinned: whether the conventions chosen where the paper is silent
 * (eps, momentum, SE activation and biases, symmetric padding) are those of
 * the model source the paper's authors ran; nothing numeric in the paper
 * fixes any value of this block.
 *
 * All tensors are NCHW, contiguous, W fastest.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int N, Cin, H, W;
    int Cexp, Cse, Cout;
    int k, stride, pad;
    int has_expand, residual;
    double eps, momentum;
    int activation; /* 0: Swish (EfficientNet MBConv), 1: ReLU6 (MobileNet-V2 inverted residual) */
    int has_se;     /* 0: no squeeze-and-excitation stage (sc = a2); Cse and the SE parameters are ignored */
} orc_desc;

typedef struct {
    const double *w_expand;             /* [Cexp,Cin] */
    const double *bn1_gamma, *bn1_beta; /* [Cexp] */
    const double *w_dw;                 /* [Cexp,k,k] */
    const double *bn2_gamma, *bn2_beta; /* [Cexp] */
    const double *se_w1, *se_b1;        /* [Cse,Cexp],[Cse] */
    const double *se_w2, *se_b2;        /* [Cexp,Cse],[Cexp] */
    const double *w_proj;               /* [Cout,Cexp] */
    const double *bn3_gamma, *bn3_beta; /* [Cout] */
} orc_params;

typedef struct {
    double *w_expand, *bn1_gamma, *bn1_beta, *w_dw, *bn2_gamma, *bn2_beta;
    double *se_w1, *se_b1, *se_w2, *se_b2, *w_proj, *bn3_gamma, *bn3_beta;
} orc_grads;

typedef struct {
    double *bn1_mean, *bn1_var, *bn2_mean, *bn2_var, *bn3_mean, *bn3_var;
} orc_running;

/* Every intermediate of the forward pass, caller-allocated. */
typedef struct {
    double *e, *xhat1, *y1, *a1;      /* [N,Cexp,H,W]  (a1 == x when !has_expand) */
    double *d, *xhat2, *y2, *a2, *sc; /* [N,Cexp,Ho,Wo] */
    double *z, *t, *g;                /* [N,Cexp] */
    double *q, *r;                    /* [N,Cse] */
    double *p, *xhat3;                /* [N,Cout,Ho,Wo] */
    double *mean1, *var1, *mean2, *var2; /* [Cexp], biased batch variance */
    double *mean3, *var3;             /* [Cout] */
} orc_tape;

/* ---- scalar functions ---------------------------------------------------- */

double orc_sigmoid(double t) { return 1.0 / (1.0 + exp(-t)); }

/* Swish(t) = t * sigmoid(t). */
double orc_swish(double t) { return t * orc_sigmoid(t); }

/* d/dt Swish(t) = sigmoid(t) * (1 + t * (1 - sigmoid(t))). */
double orc_swish_grad(double t)
{
    double s = orc_sigmoid(t);
    return s * (1.0 + t * (1.0 - s));
}

/* ReLU6(t) = min(max(t, 0), 6), the activation of the MobileNet-V2 inverted-residual block
 * (one of the networks the paper times, table "Automatic optimization results"); its
 * derivative is 1 strictly inside (0, 6) and 0 elsewhere, kinks included. */
double orc_relu6(double t) { return t < 0.0 ? 0.0 : (t > 6.0 ? 6.0 : t); }
double orc_relu6_grad(double t) { return (t > 0.0 && t < 6.0) ? 1.0 : 0.0; }

/* The block's two activations (after BN1 and after BN2); the SE stage keeps its own Swish
 * and sigmoid. */
static double orc_act(int activation, double t)
{
    return activation == 1 ? orc_relu6(t) : orc_swish(t);
}
static double orc_act_grad(int activation, double t)
{
    return activation == 1 ? orc_relu6_grad(t) : orc_swish_grad(t);
}

/* ---- 1x1 convolution: y[n,o,q] = sum_i W[o,i] x[n,i,q] ------------------- */
/* A 1x1 convolution in NCHW is a per-image matrix product (the paper lowers
 * convolutions to matrix products in section "ONNX on SDFG"; for a 1x1 filter
 * no im2col copy is involved). */

void orc_conv1x1(int N, int Ci, int Co, int HW, const double *Wt, const double *x, double *y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < Co; ++o) {
            double *yr = y + ((size_t)n * Co + o) * HW;
            for (int q = 0; q < HW; ++q) {
                double acc = 0.0;
                for (int i = 0; i < Ci; ++i)
                    acc += Wt[(size_t)o * Ci + i] * x[((size_t)n * Ci + i) * HW + q];
                yr[q] = acc;
            }
        }
}

/* dx[n,i,q] = sum_o W[o,i] dy[n,o,q] */
void orc_conv1x1_bwd_input(int N, int Ci, int Co, int HW, const double *Wt, const double *dy,
                           double *dx)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < Ci; ++i) {
            double *dr = dx + ((size_t)n * Ci + i) * HW;
            for (int q = 0; q < HW; ++q) {
                double acc = 0.0;
                for (int o = 0; o < Co; ++o)
                    acc += Wt[(size_t)o * Ci + i] * dy[((size_t)n * Co + o) * HW + q];
                dr[q] = acc;
            }
        }
}

/* dW[o,i] = sum_{n,q} dy[n,o,q] x[n,i,q] */
void orc_conv1x1_bwd_weight(int N, int Ci, int Co, int HW, const double *x, const double *dy,
                            double *dW)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int o = 0; o < Co; ++o)
        for (int i = 0; i < Ci; ++i) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n) {
                const double *dr = dy + ((size_t)n * Co + o) * HW;
                const double *xr = x + ((size_t)n * Ci + i) * HW;
                for (int q = 0; q < HW; ++q)
                    acc += dr[q] * xr[q];
            }
            dW[(size_t)o * Ci + i] = acc;
        }
}

/* ---- batch normalisation, training mode ---------------------------------- */
/* Per channel c over the m = N*HW values: mean, biased variance (two passes),
 * xhat = (x-mean)/sqrt(var+eps), y = gamma*xhat+beta.  Running statistics:
 * run <- (1-momentum)*run + momentum*batch, the variance entering the running
 * update being the unbiased estimate var*m/(m-1). */

void orc_bn_fwd(int N, int C, int HW, const double *x, const double *gamma, const double *beta,
                double eps, double momentum, double *mean, double *var, double *run_mean,
                double *run_var, double *xhat, double *y)
{
    const double m = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double s = 0.0;
        for (int n = 0; n < N; ++n) {
            const double *xr = x + ((size_t)n * C + c) * HW;
            for (int q = 0; q < HW; ++q)
                s += xr[q];
        }
        const double mu = s / m;
        double s2 = 0.0;
        for (int n = 0; n < N; ++n) {
            const double *xr = x + ((size_t)n * C + c) * HW;
            for (int q = 0; q < HW; ++q) {
                double dlt = xr[q] - mu;
                s2 += dlt * dlt;
            }
        }
        const double v = s2 / m;
        const double rstd = 1.0 / sqrt(v + eps);
        mean[c] = mu;
        var[c] = v;
        for (int n = 0; n < N; ++n) {
            const size_t off = ((size_t)n * C + c) * HW;
            for (int q = 0; q < HW; ++q) {
                double xh = (x[off + q] - mu) * rstd;
                xhat[off + q] = xh;
                y[off + q] = gamma[c] * xh + beta[c];
            }
        }
        if (run_mean)
            run_mean[c] = (1.0 - momentum) * run_mean[c] + momentum * mu;
        if (run_var) {
            const double unbiased = (m > 1.0) ? v * m / (m - 1.0) : v;
            run_var[c] = (1.0 - momentum) * run_var[c] + momentum * unbiased;
        }
    }
}

/* dbeta = sum dy, dgamma = sum dy*xhat,
 * dx = gamma*rstd*(dy - dbeta/m - xhat*dgamma/m). */
void orc_bn_bwd(int N, int C, int HW, const double *dy, const double *xhat, const double *gamma,
                const double *var, double eps, double *dx, double *dgamma, double *dbeta)
{
    const double m = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double sb = 0.0, sg = 0.0;
        for (int n = 0; n < N; ++n) {
            const size_t off = ((size_t)n * C + c) * HW;
            for (int q = 0; q < HW; ++q) {
                sb += dy[off + q];
                sg += dy[off + q] * xhat[off + q];
            }
        }
        dbeta[c] = sb;
        dgamma[c] = sg;
        const double rstd = 1.0 / sqrt(var[c] + eps);
        for (int n = 0; n < N; ++n) {
            const size_t off = ((size_t)n * C + c) * HW;
            for (int q = 0; q < HW; ++q)
                dx[off + q] = gamma[c] * rstd * (dy[off + q] - sb / m - xhat[off + q] * sg / m);
        }
    }
}

/* ---- depthwise convolution (cross-correlation, zero padding, no bias) ---- */
/* d[n,c,i,j] = sum_{u,v<k} w[c,u,v] * a[n,c,i*s+u-p,j*s+v-p], taps that fall
 * outside the image contribute nothing.  Ho = (H+2p-k)/s+1. */

void orc_depthwise_fwd(int N, int C, int H, int W, int k, int s, int p, const double *w,
                       const double *a, double *d)
{
    const int Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            const double *ap = a + ((size_t)n * C + c) * H * W;
            double *dp = d + ((size_t)n * C + c) * Ho * Wo;
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    double acc = 0.0;
                    for (int u = 0; u < k; ++u)
                        for (int v = 0; v < k; ++v) {
                            int h = i * s + u - p, x = j * s + v - p;
                            if (h >= 0 && h < H && x >= 0 && x < W)
                                acc += w[((size_t)c * k + u) * k + v] * ap[(size_t)h * W + x];
                        }
                    dp[(size_t)i * Wo + j] = acc;
                }
        }
}

/* da[n,c,h,x] = sum over (u,v) and output pixels (i,j) with i*s+u-p == h and
 * j*s+v-p == x of w[c,u,v]*dd[n,c,i,j].  Written as a scatter over the forward
 * loop nest, which is the transpose of the forward definition by inspection;
 * each (n,c) plane is owned by one thread so no update races. */
void orc_depthwise_bwd_input(int N, int C, int H, int W, int k, int s, int p, const double *w,
                             const double *dd, double *da)
{
    const int Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double *ap = da + ((size_t)n * C + c) * H * W;
            const double *dp = dd + ((size_t)n * C + c) * Ho * Wo;
            for (int q = 0; q < H * W; ++q)
                ap[q] = 0.0;
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j)
                    for (int u = 0; u < k; ++u)
                        for (int v = 0; v < k; ++v) {
                            int h = i * s + u - p, x = j * s + v - p;
                            if (h >= 0 && h < H && x >= 0 && x < W)
                                ap[(size_t)h * W + x] +=
                                    w[((size_t)c * k + u) * k + v] * dp[(size_t)i * Wo + j];
                        }
        }
}

/* dw[c,u,v] = sum_{n,i,j} dd[n,c,i,j] * a[n,c,i*s+u-p,j*s+v-p] */
void orc_depthwise_bwd_weight(int N, int C, int H, int W, int k, int s, int p, const double *a,
                              const double *dd, double *dw)
{
    const int Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c)
        for (int u = 0; u < k; ++u)
            for (int v = 0; v < k; ++v) {
                double acc = 0.0;
                for (int n = 0; n < N; ++n) {
                    const double *ap = a + ((size_t)n * C + c) * H * W;
                    const double *dp = dd + ((size_t)n * C + c) * Ho * Wo;
                    for (int i = 0; i < Ho; ++i)
                        for (int j = 0; j < Wo; ++j) {
                            int h = i * s + u - p, x = j * s + v - p;
                            if (h >= 0 && h < H && x >= 0 && x < W)
                                acc += dp[(size_t)i * Wo + j] * ap[(size_t)h * W + x];
                        }
                }
                dw[((size_t)c * k + u) * k + v] = acc;
            }
}

/* ---- squeeze-and-excitation ---------------------------------------------- */
/* z[n,c] = mean_{ij} a2; q = W1 z + b1; r = swish(q); t = W2 r + b2;
 * g = sigmoid(t); sc[n,c,i,j] = a2[n,c,i,j] * g[n,c]. */

void orc_se_fwd(int N, int C, int Cse, int HW, const double *a2, const double *W1,
                const double *b1, const double *W2, const double *b2, double *z, double *q,
                double *r, double *t, double *g, double *sc)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < C; ++c) {
            double s = 0.0;
            const double *ap = a2 + ((size_t)n * C + c) * HW;
            for (int i = 0; i < HW; ++i)
                s += ap[i];
            z[(size_t)n * C + c] = s / (double)HW;
        }
        for (int j = 0; j < Cse; ++j) {
            double acc = b1[j];
            for (int c = 0; c < C; ++c)
                acc += W1[(size_t)j * C + c] * z[(size_t)n * C + c];
            q[(size_t)n * Cse + j] = acc;
            r[(size_t)n * Cse + j] = orc_swish(acc);
        }
        for (int c = 0; c < C; ++c) {
            double acc = b2[c];
            for (int j = 0; j < Cse; ++j)
                acc += W2[(size_t)c * Cse + j] * r[(size_t)n * Cse + j];
            t[(size_t)n * C + c] = acc;
            g[(size_t)n * C + c] = orc_sigmoid(acc);
            const double *ap = a2 + ((size_t)n * C + c) * HW;
            double *sp = sc + ((size_t)n * C + c) * HW;
            for (int i = 0; i < HW; ++i)
                sp[i] = ap[i] * g[(size_t)n * C + c];
        }
    }
}

/* Given dsc, returns da2 and the four FC gradients.
 * dg = sum_{ij} dsc*a2; dt = dg*g*(1-g); dW2 = sum_n dt r^T; db2 = sum_n dt;
 * dr = W2^T dt; dq = dr*swish'(q); dW1 = sum_n dq z^T; db1 = sum_n dq;
 * dz = W1^T dq; da2 = dsc*g + dz/HW. */
void orc_se_bwd(int N, int C, int Cse, int HW, const double *a2, const double *W1,
                const double *W2, const double *z, const double *q, const double *r,
                const double *g, const double *dsc, double *da2, double *dW1, double *db1,
                double *dW2, double *db2)
{
    double *dt = (double *)malloc(sizeof(double) * (size_t)N * C);
    double *dq = (double *)malloc(sizeof(double) * (size_t)N * Cse);
    double *dz = (double *)malloc(sizeof(double) * (size_t)N * C);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < C; ++c) {
            const size_t off = ((size_t)n * C + c) * HW;
            double dg = 0.0;
            for (int i = 0; i < HW; ++i)
                dg += dsc[off + i] * a2[off + i];
            const double gv = g[(size_t)n * C + c];
            dt[(size_t)n * C + c] = dg * gv * (1.0 - gv);
        }
        for (int j = 0; j < Cse; ++j) {
            double dr = 0.0;
            for (int c = 0; c < C; ++c)
                dr += W2[(size_t)c * Cse + j] * dt[(size_t)n * C + c];
            dq[(size_t)n * Cse + j] = dr * orc_swish_grad(q[(size_t)n * Cse + j]);
        }
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int j = 0; j < Cse; ++j)
                acc += W1[(size_t)j * C + c] * dq[(size_t)n * Cse + j];
            dz[(size_t)n * C + c] = acc;
            const size_t off = ((size_t)n * C + c) * HW;
            const double gv = g[(size_t)n * C + c];
            for (int i = 0; i < HW; ++i)
                da2[off + i] = dsc[off + i] * gv + acc / (double)HW;
        }
    }
    for (int c = 0; c < C; ++c) {
        double sb = 0.0;
        for (int n = 0; n < N; ++n)
            sb += dt[(size_t)n * C + c];
        db2[c] = sb;
        for (int j = 0; j < Cse; ++j) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n)
                acc += dt[(size_t)n * C + c] * r[(size_t)n * Cse + j];
            dW2[(size_t)c * Cse + j] = acc;
        }
    }
    for (int j = 0; j < Cse; ++j) {
        double sb = 0.0;
        for (int n = 0; n < N; ++n)
            sb += dq[(size_t)n * Cse + j];
        db1[j] = sb;
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n)
                acc += dq[(size_t)n * Cse + j] * z[(size_t)n * C + c];
            dW1[(size_t)j * C + c] = acc;
        }
    }
    free(dt);
    free(dq);
    free(dz);
}

/* ---- the block ------------------------------------------------------------ */

static int desc_ok(const orc_desc *D)
{
    if (!D || D->N < 1 || D->Cin < 1 || D->H < 1 || D->W < 1 || D->Cexp < 1 ||
        (D->has_se && D->Cse < 1) || D->Cout < 1 || D->k < 1 || D->stride < 1 || D->pad < 0)
        return 0;
    if (D->activation != 0 && D->activation != 1)
        return 0;
    if (!D->has_expand && D->Cexp != D->Cin)
        return 0;
    if (D->residual && (D->stride != 1 || D->Cin != D->Cout))
        return 0;
    if (D->H + 2 * D->pad < D->k || D->W + 2 * D->pad < D->k)
        return 0;
    return 1;
}

int orc_mbconv_forward(const orc_desc *D, const orc_params *P, orc_running *R, const double *x,
                       double *out, orc_tape *T)
{
    if (!desc_ok(D))
        return -1;
    const int N = D->N, HW = D->H * D->W;
    const int Ho = (D->H + 2 * D->pad - D->k) / D->stride + 1;
    const int Wo = (D->W + 2 * D->pad - D->k) / D->stride + 1;
    const int HWo = Ho * Wo;
    const size_t nE = (size_t)N * D->Cexp * HW, nD = (size_t)N * D->Cexp * HWo;
    const size_t nP = (size_t)N * D->Cout * HWo;

    /* expansion: 1x1 conv, BN1, Swish (absent when the expand ratio is 1) */
    if (D->has_expand) {
        orc_conv1x1(N, D->Cin, D->Cexp, HW, P->w_expand, x, T->e);
        orc_bn_fwd(N, D->Cexp, HW, T->e, P->bn1_gamma, P->bn1_beta, D->eps, D->momentum, T->mean1,
                   T->var1, R ? R->bn1_mean : NULL, R ? R->bn1_var : NULL, T->xhat1, T->y1);
#pragma omp parallel for schedule(static)
        for (size_t i = 0; i < nE; ++i)
            T->a1[i] = orc_act(D->activation, T->y1[i]);
    } else {
        memcpy(T->a1, x, sizeof(double) * nE);
    }
    /* depthwise conv, BN2, activation */
    orc_depthwise_fwd(N, D->Cexp, D->H, D->W, D->k, D->stride, D->pad, P->w_dw, T->a1, T->d);
    orc_bn_fwd(N, D->Cexp, HWo, T->d, P->bn2_gamma, P->bn2_beta, D->eps, D->momentum, T->mean2,
               T->var2, R ? R->bn2_mean : NULL, R ? R->bn2_var : NULL, T->xhat2, T->y2);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < nD; ++i)
        T->a2[i] = orc_act(D->activation, T->y2[i]);
    /* squeeze-and-excitation (absent in the MobileNet-V2 block: sc = a2) */
    if (D->has_se)
        orc_se_fwd(N, D->Cexp, D->Cse, HWo, T->a2, P->se_w1, P->se_b1, P->se_w2, P->se_b2, T->z,
                   T->q, T->r, T->t, T->g, T->sc);
    else
        memcpy(T->sc, T->a2, sizeof(double) * nD);
    /* projection: 1x1 conv, BN3 (no activation), optional residual */
    orc_conv1x1(N, D->Cexp, D->Cout, HWo, P->w_proj, T->sc, T->p);
    orc_bn_fwd(N, D->Cout, HWo, T->p, P->bn3_gamma, P->bn3_beta, D->eps, D->momentum, T->mean3,
               T->var3, R ? R->bn3_mean : NULL, R ? R->bn3_var : NULL, T->xhat3, out);
    if (D->residual)
        for (size_t i = 0; i < nP; ++i)
            out[i] += x[i];
    return 0;
}

/* ---- evaluation mode ------------------------------------------------------- */
/* The paper notes that batch normalisation behaves differently in training and in
 * inference (section "Background and Related Work", paragraph "Training vs. inference
 * compilation"): training normalises with the batch statistics and stores running
 * statistics; inference normalises with those stored statistics,
 *   y = gamma*(x - run_mean)/sqrt(run_var + eps) + beta,
 * so no reduction over the batch is involved and nothing is written back. */
void orc_bn_eval(int N, int C, int HW, const double *x, const double *gamma, const double *beta,
                 double eps, const double *run_mean, const double *run_var, double *y)
{
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        const double rstd = 1.0 / sqrt(run_var[c] + eps);
        for (int n = 0; n < N; ++n) {
            const size_t off = ((size_t)n * C + c) * HW;
            for (int q = 0; q < HW; ++q)
                y[off + q] = gamma[c] * ((x[off + q] - run_mean[c]) * rstd) + beta[c];
        }
    }
}

/* The block of orc_mbconv_forward with every BN in evaluation mode.  R is read only. */
int orc_mbconv_forward_eval(const orc_desc *D, const orc_params *P, const orc_running *R,
                            const double *x, double *out)
{
    if (!desc_ok(D) || !R)
        return -1;
    const int N = D->N, HW = D->H * D->W;
    const int Ho = (D->H + 2 * D->pad - D->k) / D->stride + 1;
    const int Wo = (D->W + 2 * D->pad - D->k) / D->stride + 1;
    const int HWo = Ho * Wo;
    const size_t nE = (size_t)N * D->Cexp * HW, nD = (size_t)N * D->Cexp * HWo;
    const size_t nP = (size_t)N * D->Cout * HWo;
    double *a1 = (double *)malloc(sizeof(double) * nE);
    double *e = (double *)malloc(sizeof(double) * nE);
    double *d = (double *)malloc(sizeof(double) * nD);
    double *a2 = (double *)malloc(sizeof(double) * nD);
    double *sc = (double *)malloc(sizeof(double) * nD);
    double *p = (double *)malloc(sizeof(double) * nP);
    double *z = (double *)malloc(sizeof(double) * (size_t)N * D->Cexp);
    double *t = (double *)malloc(sizeof(double) * (size_t)N * D->Cexp);
    double *g = (double *)malloc(sizeof(double) * (size_t)N * D->Cexp);
    const size_t nQ = (size_t)N * (D->has_se ? D->Cse : 1);
    double *q = (double *)malloc(sizeof(double) * nQ);
    double *r = (double *)malloc(sizeof(double) * nQ);
    if (!a1 || !e || !d || !a2 || !sc || !p || !z || !t || !g || !q || !r)
        return -2;
    if (D->has_expand) {
        orc_conv1x1(N, D->Cin, D->Cexp, HW, P->w_expand, x, e);
        orc_bn_eval(N, D->Cexp, HW, e, P->bn1_gamma, P->bn1_beta, D->eps, R->bn1_mean, R->bn1_var, a1);
#pragma omp parallel for schedule(static)
        for (size_t i = 0; i < nE; ++i)
            a1[i] = orc_act(D->activation, a1[i]);
    } else {
        memcpy(a1, x, sizeof(double) * nE);
    }
    orc_depthwise_fwd(N, D->Cexp, D->H, D->W, D->k, D->stride, D->pad, P->w_dw, a1, d);
    orc_bn_eval(N, D->Cexp, HWo, d, P->bn2_gamma, P->bn2_beta, D->eps, R->bn2_mean, R->bn2_var, a2);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < nD; ++i)
        a2[i] = orc_act(D->activation, a2[i]);
    if (D->has_se)
        orc_se_fwd(N, D->Cexp, D->Cse, HWo, a2, P->se_w1, P->se_b1, P->se_w2, P->se_b2, z, q, r, t,
                   g, sc);
    else
        memcpy(sc, a2, sizeof(double) * nD);
    orc_conv1x1(N, D->Cexp, D->Cout, HWo, P->w_proj, sc, p);
    orc_bn_eval(N, D->Cout, HWo, p, P->bn3_gamma, P->bn3_beta, D->eps, R->bn3_mean, R->bn3_var, out);
    if (D->residual)
        for (size_t i = 0; i < nP; ++i)
            out[i] += x[i];
    free(a1);
    free(e);
    free(d);
    free(a2);
    free(sc);
    free(p);
    free(z);
    free(t);
    free(g);
    free(q);
    free(r);
    return 0;
}

int orc_mbconv_backward(const orc_desc *D, const orc_params *P, const double *x,
                        const double *dout, const orc_tape *T, double *dx, orc_grads *G)
{
    if (!desc_ok(D))
        return -1;
    const int N = D->N, HW = D->H * D->W;
    const int Ho = (D->H + 2 * D->pad - D->k) / D->stride + 1;
    const int Wo = (D->W + 2 * D->pad - D->k) / D->stride + 1;
    const int HWo = Ho * Wo;
    const size_t nX = (size_t)N * D->Cin * HW;
    const size_t nE = (size_t)N * D->Cexp * HW, nD = (size_t)N * D->Cexp * HWo;
    const size_t nP = (size_t)N * D->Cout * HWo;

    double *dp = (double *)malloc(sizeof(double) * nP);
    double *dsc = (double *)malloc(sizeof(double) * nD);
    double *da2 = (double *)malloc(sizeof(double) * nD);
    double *dy2 = (double *)malloc(sizeof(double) * nD);
    double *dd = (double *)malloc(sizeof(double) * nD);
    double *da1 = (double *)malloc(sizeof(double) * nE);
    if (!dp || !dsc || !da2 || !dy2 || !dd || !da1)
        return -2;

    /* BN3 backward (dy3 = dOut, the residual branch is added at the end) */
    orc_bn_bwd(N, D->Cout, HWo, dout, T->xhat3, P->bn3_gamma, T->var3, D->eps, dp, G->bn3_gamma,
               G->bn3_beta);
    /* projection conv */
    orc_conv1x1_bwd_input(N, D->Cexp, D->Cout, HWo, P->w_proj, dp, dsc);
    orc_conv1x1_bwd_weight(N, D->Cexp, D->Cout, HWo, T->sc, dp, G->w_proj);
    /* squeeze-and-excitation */
    if (D->has_se)
        orc_se_bwd(N, D->Cexp, D->Cse, HWo, T->a2, P->se_w1, P->se_w2, T->z, T->q, T->r, T->g, dsc,
                   da2, G->se_w1, G->se_b1, G->se_w2, G->se_b2);
    else
        memcpy(da2, dsc, sizeof(double) * nD);
    /* activation, BN2 */
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < nD; ++i)
        dy2[i] = da2[i] * orc_act_grad(D->activation, T->y2[i]);
    orc_bn_bwd(N, D->Cexp, HWo, dy2, T->xhat2, P->bn2_gamma, T->var2, D->eps, dd, G->bn2_gamma,
               G->bn2_beta);
    /* depthwise conv */
    orc_depthwise_bwd_weight(N, D->Cexp, D->H, D->W, D->k, D->stride, D->pad, T->a1, dd, G->w_dw);
    orc_depthwise_bwd_input(N, D->Cexp, D->H, D->W, D->k, D->stride, D->pad, P->w_dw, dd, da1);

    if (D->has_expand) {
        double *dy1 = (double *)malloc(sizeof(double) * nE);
        double *de = (double *)malloc(sizeof(double) * nE);
        if (!dy1 || !de)
            return -2;
#pragma omp parallel for schedule(static)
        for (size_t i = 0; i < nE; ++i)
            dy1[i] = da1[i] * orc_act_grad(D->activation, T->y1[i]);
        orc_bn_bwd(N, D->Cexp, HW, dy1, T->xhat1, P->bn1_gamma, T->var1, D->eps, de,
                   G->bn1_gamma, G->bn1_beta);
        orc_conv1x1_bwd_weight(N, D->Cin, D->Cexp, HW, x, de, G->w_expand);
        orc_conv1x1_bwd_input(N, D->Cin, D->Cexp, HW, P->w_expand, de, dx);
        free(dy1);
        free(de);
    } else {
        memcpy(dx, da1, sizeof(double) * nX);
    }
    if (D->residual)
        for (size_t i = 0; i < nX; ++i)
            dx[i] += dout[i];

    free(dp);
    free(dsc);
    free(da2);
    free(dy2);
    free(dd);
    free(da1);
    return 0;
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
