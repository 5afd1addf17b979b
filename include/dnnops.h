/*
 * dnnops.h - C ABI of the paper's other memory-bound operators on one AMD MI355X (gfx950),
 * exported by the same shared library as mbconv.h: the Mish activation (forward, and a
 * backward that recomputes everything from x: the paper's scalar-level recomputation, section
 * "Evaluation", Mish paragraph), layer normalisation over the last dimension (section
 * "Statistical Normalization") and softmax over the last dimension (section "Softmax").
 *
 * Conventions
 *   - fp32 tensors, row-major, contiguous; every pointer is a DEVICE pointer owned by the
 *     caller and must be 16-byte aligned.  The library allocates nothing, keeps no state and
 *     never synchronises: all work is enqueued on the hipStream_t passed as `hip_stream`
 *     (NULL = the default stream).
 *   - Every argument check happens on the host before the first launch and returns a negative
 *     status without touching device memory.  A failed launch returns DNNOPS_EHIP.
 *   - Reductions run in a fixed order without floating-point atomics: results are bitwise
 *     repeatable.
 */
#ifndef DNNOPS_H
#define DNNOPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DNNOPS_OK = 0,
    DNNOPS_EINVAL = -1,       /* NULL pointer, non-positive size */
    DNNOPS_EUNSUPPORTED = -2, /* cols > DNNOPS_MAX_COLS */
    DNNOPS_ESCRATCH = -3,     /* the shape needs more scratch than the library's static buffer holds */
    DNNOPS_EALIGN = -4,       /* pointer not 16-byte aligned */
    DNNOPS_EHIP = -5          /* a launch failed */
} dnnops_status;

/* Longest row the row-wise operators accept. */
#define DNNOPS_MAX_COLS 8192

/* y[i] = x[i] * tanh(log(1 + exp(x[i]))), i < n.  x and y may be the same buffer. */
dnnops_status dnnops_mish_forward(const float *x, float *y, size_t n, void *hip_stream);

/* dx[i] = dy[i] * mish'(x[i]) with mish'(x) = tanh(sp) + x*(1 - tanh(sp)^2)*sigmoid(x),
 * sp = log(1 + exp(x)): nothing but x is kept from the forward pass.  dx may alias dy. */
dnnops_status dnnops_mish_backward(const float *x, const float *dy, float *dx, size_t n,
                                   void *hip_stream);

/* Layer normalisation of each row of x[rows][cols]:
 *   y = gamma*(x - mean)/sqrt(var + eps) + beta, mean and (biased) var over the row.
 * Also writes mean[rows] and rstd[rows] = 1/sqrt(var + eps) for the backward call. */
dnnops_status dnnops_layernorm_forward(const float *x, const float *gamma, const float *beta,
                                       float eps, int32_t rows, int32_t cols, float *y, float *mean,
                                       float *rstd, void *hip_stream);

/* Host-only: bytes of scratch dnnops_layernorm_backward needs for this shape (0 on bad sizes). */
size_t dnnops_layernorm_backward_scratch_bytes(int32_t rows, int32_t cols);

/* Backward of dnnops_layernorm_forward (same x, gamma, mean, rstd):
 *   dx[rows][cols]; dgamma[c] = sum_r dy*xhat; dbeta[c] = sum_r dy (both overwritten).
 * scratch: at least dnnops_layernorm_backward_scratch_bytes(rows, cols), overwritten. */
dnnops_status dnnops_layernorm_backward(const float *x, const float *dy, const float *gamma,
                                        const float *mean, const float *rstd, int32_t rows,
                                        int32_t cols, float *dx, float *dgamma, float *dbeta,
                                        void *scratch, void *hip_stream);

/* The same backward pass for callers that cannot allocate device memory or pass a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and kernels as dnnops_layernorm_backward without `scratch`: the partial
 * sums live in a buffer of dnnops_layernorm_backward_noalloc_max_scratch_bytes() (8 MiB) that is
 * part of the library's device code, one copy per GPU, held until the process ends.  The call
 * allocates and frees nothing.  A shape for which dnnops_layernorm_backward_scratch_bytes(rows,
 * cols) exceeds that size is rejected with DNNOPS_ESCRATCH on the host, before any launch (every
 * shape with cols <= 2048 fits, whatever rows is).  All calls on one GPU share that GPU's buffer:
 * the buffer keeps the previous call's contents, every value a call reads it has written itself
 * first, and calls that overlap on one GPU (different streams, or threads) race: serialise them. */
size_t dnnops_layernorm_backward_noalloc_max_scratch_bytes(void);
dnnops_status dnnops_layernorm_backward_noalloc(const float *x, const float *dy, const float *gamma,
                                                const float *mean, const float *rstd, int32_t rows,
                                                int32_t cols, float *dx, float *dgamma,
                                                float *dbeta, void *hip_stream);

/* y[r][c] = exp(x[r][c] - max_c x[r][.]) / sum_c exp(x[r][c] - max_c x[r][.]).  y may alias x. */
dnnops_status dnnops_softmax_forward(const float *x, float *y, int32_t rows, int32_t cols,
                                     void *hip_stream);

/* dx = y * (dy - sum_c dy*y) per row, y the forward result.  dx may alias dy. */
dnnops_status dnnops_softmax_backward(const float *y, const float *dy, float *dx, int32_t rows,
                                      int32_t cols, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DNNOPS_H */
