// Small kernels: batch-norm statistics finalisation (forward and backward), the
// squeeze-and-excitation fully connected layers and their gradients, and the fixed-order
// second stage of the split reductions.  All of them touch O(N*C) values.
#include "mbconv_dev.h"
#include "mbconv_launch.h"

namespace mbk {

__device__ __forceinline__ double wave_sum_d(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o, kWave);
    return v;
}

// One wavefront per channel.  Partials are fp32 sums over at most a plane or a GEMM tile;
// they are combined in fp64 so that var = E[x^2]-E[x]^2 loses nothing in this stage.
// BN formula and running statistics: section "Statistical Normalization".
__global__ __launch_bounds__(256) void bn_finalize_kernel(int C, int NP, double m,
                                                          const float *__restrict__ psum,
                                                          const float *__restrict__ psq,
                                                          const float *__restrict__ gamma,
                                                          const float *__restrict__ beta, float eps,
                                                          float momentum, float *run_mean,
                                                          float *run_var, float *bn)
{
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (c >= C)
        return;
    double s = 0.0, s2 = 0.0;
    for (int i = lane; i < NP; i += kWave) {
        s += (double)psum[(size_t)c * NP + i];
        s2 += (double)psq[(size_t)c * NP + i];
    }
    s = wave_sum_d(s);
    s2 = wave_sum_d(s2);
    if (lane == 0) {
        const double mean = s / m;
        double var = s2 / m - mean * mean;
        if (var < 0.0)
            var = 0.0;
        const double rstd = 1.0 / sqrt(var + (double)eps);
        const double scale = (double)gamma[c] * rstd;
        bn[c] = (float)scale;
        bn[C + c] = (float)((double)beta[c] - mean * scale);
        bn[2 * C + c] = (float)mean;
        bn[3 * C + c] = (float)rstd;
        if (run_mean)
            run_mean[c] = (float)((1.0 - (double)momentum) * (double)run_mean[c] + (double)momentum * mean);
        if (run_var) {
            const double unbiased = m > 1.0 ? var * m / (m - 1.0) : var;
            run_var[c] = (float)((1.0 - (double)momentum) * (double)run_var[c] + (double)momentum * unbiased);
        }
    }
}

hipError_t launch_bn_finalize(int C, int NP, double m, const float *psum, const float *psq,
                              const float *gamma, const float *beta, float eps, float momentum,
                              float *run_mean, float *run_var, float *bn, hipStream_t st)
{
    hipLaunchKernelGGL(bn_finalize_kernel, dim3((C + 3) / 4), dim3(256), 0, st, C, NP, m, psum, psq,
                       gamma, beta, eps, momentum, run_mean, run_var, bn);
    return hipGetLastError();
}

// dx = gamma*rstd*(dy - dbeta/m - xhat*dgamma/m) with xhat = (raw-mean)*rstd, rewritten as
// c0*dy + c1*raw + c2 so the consumer's prologue is two fused multiply-adds.
__device__ __forceinline__ void bn_bwd_coef(int C, int c, double m, double dgamma, double dbeta,
                                            float gamma, const float *bn, float *coef)
{
    const double mean = bn[2 * C + c], rstd = bn[3 * C + c];
    const double c0 = (double)gamma * rstd;
    const double c1 = -c0 * rstd * dgamma / m;
    const double c2 = -c0 * dbeta / m - c1 * mean;
    coef[c] = (float)c0;
    coef[C + c] = (float)c1;
    coef[2 * C + c] = (float)c2;
}

__global__ __launch_bounds__(256) void bn_bwd_finalize_kernel(int C, int NP, double m,
                                                              const float *__restrict__ psb,
                                                              const float *__restrict__ psr,
                                                              const float *__restrict__ gamma,
                                                              const float *__restrict__ bn,
                                                              float *dgamma, float *dbeta,
                                                              float *coef)
{
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (c >= C)
        return;
    double sb = 0.0, sr = 0.0;
    for (int i = lane; i < NP; i += kWave) {
        sb += (double)psb[(size_t)c * NP + i];
        sr += (double)psr[(size_t)c * NP + i];
    }
    sb = wave_sum_d(sb);
    sr = wave_sum_d(sr);
    if (lane == 0) {
        if (dbeta)
            dbeta[c] = (float)sb;
        if (dgamma)
            dgamma[c] = (float)sr;
        bn_bwd_coef(C, c, m, sr, sb, gamma[c], bn, coef);
    }
}

hipError_t launch_bn_bwd_finalize(int C, int NP, double m, const float *psb, const float *psr,
                                  const float *gamma, const float *bn, float *dgamma,
                                  float *dbeta, float *coef, hipStream_t st)
{
    hipLaunchKernelGGL(bn_bwd_finalize_kernel, dim3((C + 3) / 4), dim3(256), 0, st, C, NP, m, psb,
                       psr, gamma, bn, dgamma, dbeta, coef);
    return hipGetLastError();
}

// ---- squeeze-and-excitation --------------------------------------------------------------------
// One workgroup per image.  q = W1 z + b1 (a wavefront per output, lanes stride over C),
// r = swish(q), g = sigmoid(W2 r + b2) (a thread per channel).

__global__ __launch_bounds__(256) void se_fwd_kernel(int C, int Cse, const float *__restrict__ z,
                                                     const float *__restrict__ w1,
                                                     const float *__restrict__ b1,
                                                     const float *__restrict__ w2,
                                                     const float *__restrict__ b2, float *q,
                                                     float *g)
{
    extern __shared__ float lds[];
    float *zs = lds, *rs = lds + C;
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int c = tid; c < C; c += 256)
        zs[c] = z[(size_t)n * C + c];
    __syncthreads();
    for (int j = wave; j < Cse; j += 4) {
        float acc = 0.f;
        for (int c = lane; c < C; c += kWave)
            acc = fmaf(w1[(size_t)j * C + c], zs[c], acc);
        acc = wave_sum(acc);
        if (lane == 0) {
            const float qv = acc + b1[j];
            q[(size_t)n * Cse + j] = qv;
            rs[j] = swishf(qv);
        }
    }
    __syncthreads();
    for (int c = tid; c < C; c += 256) {
        float acc = b2[c];
        for (int j = 0; j < Cse; ++j)
            acc = fmaf(w2[(size_t)c * Cse + j], rs[j], acc);
        g[(size_t)n * C + c] = sigmoidf_fast(acc);
    }
}

hipError_t launch_se_fwd(int N, int C, int Cse, const float *z, const float *w1, const float *b1,
                         const float *w2, const float *b2, float *q, float *g, hipStream_t st)
{
    hipLaunchKernelGGL(se_fwd_kernel, dim3(N), dim3(256), sizeof(float) * (C + Cse), st, C, Cse, z,
                       w1, b1, w2, b2, q, g);
    return hipGetLastError();
}

// Backward, per image: dt = dg*g*(1-g); dq = (W2^T dt)*swish'(q); dzs = (W1^T dq)/HW.
__global__ __launch_bounds__(256) void se_bwd_image_kernel(SeBwdArgs a)
{
    extern __shared__ float lds[];
    float *dts = lds, *dqs = lds + a.C;
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int C = a.C, Cse = a.Cse;
    for (int c = tid; c < C; c += 256) {
        const float gv = a.g[(size_t)n * C + c];
        const float v = a.dg[(size_t)n * C + c] * gv * (1.f - gv);
        dts[c] = v;
        a.dt[(size_t)n * C + c] = v;
    }
    __syncthreads();
    for (int j = wave; j < Cse; j += 4) {
        float acc = 0.f;
        for (int c = lane; c < C; c += kWave)
            acc = fmaf(a.w2[(size_t)c * Cse + j], dts[c], acc);
        acc = wave_sum(acc);
        if (lane == 0) {
            float val, grad;
            swish_both(a.q[(size_t)n * Cse + j], val, grad);
            const float v = acc * grad;
            dqs[j] = v;
            a.dq[(size_t)n * Cse + j] = v;
        }
    }
    __syncthreads();
    const float inv = 1.f / (float)a.HW;
    for (int c = tid; c < C; c += 256) {
        float acc = 0.f;
        for (int j = 0; j < Cse; ++j)
            acc = fmaf(a.w1[(size_t)j * C + c], dqs[j], acc);
        a.dzs[(size_t)n * C + c] = acc * inv;
    }
}

// Sums over the batch.  Each output element is owned by 32 consecutive lanes: lane l adds
// the images l, l+32, ... and the 32 partial sums are combined by a fixed butterfly, so the
// result does not depend on scheduling.  Output elements in order:
//   [0, C*Cse)            dW2[c,j] = sum_n dt[n,c]*swish(q[n,j])
//   [C*Cse, 2*C*Cse)      dW1[j,c] = sum_n dq[n,j]*z[n,c]
//   next C                db2[c], and BN2's dbeta/dgamma/coef from the plane sums:
//                         dbeta2 = sum_n g*A1 + dzs*s3,  dgamma2 = sum_n g*A2 + dzs*s4
//   next Cse              db1[j]
__device__ __forceinline__ double half_wave_sum_d(double v)
{
#pragma unroll
    for (int o = 16; o > 0; o >>= 1)
        v += __shfl_xor(v, o, kWave);
    return v;
}

__global__ __launch_bounds__(256) void se_bwd_batch_kernel(SeBwdArgs a)
{
    const int C = a.C, Cse = a.Cse, N = a.N;
    const int ln = threadIdx.x & 31;
    int i = blockIdx.x * 8 + (threadIdx.x >> 5);
    if (i < C * Cse) {
        const int c = i / Cse, j = i - c * Cse;
        float acc = 0.f;
        for (int n = ln; n < N; n += 32)
            acc = fmaf(a.dt[(size_t)n * C + c], swishf(a.q[(size_t)n * Cse + j]), acc);
        acc = half_wave_sum(acc);
        if (ln == 0)
            a.dw2[i] = acc;
        return;
    }
    i -= C * Cse;
    if (i < C * Cse) {
        const int j = i / C, c = i - j * C;
        float acc = 0.f;
        for (int n = ln; n < N; n += 32)
            acc = fmaf(a.dq[(size_t)n * Cse + j], a.z[(size_t)n * C + c], acc);
        acc = half_wave_sum(acc);
        if (ln == 0)
            a.dw1[i] = acc;
        return;
    }
    i -= C * Cse;
    if (i < C) {
        const int c = i;
        float sb = 0.f;
        double dbeta = 0.0, dgamma = 0.0;
        for (int n = ln; n < N; n += 32) {
            const size_t o = (size_t)n * C + c;
            sb += a.dt[o];
            dbeta += (double)a.g[o] * a.A1[o] + (double)a.dzs[o] * a.s3[o];
            dgamma += (double)a.g[o] * a.A2[o] + (double)a.dzs[o] * a.s4[o];
        }
        sb = half_wave_sum(sb);
        dbeta = half_wave_sum_d(dbeta);
        dgamma = half_wave_sum_d(dgamma);
        if (ln == 0) {
            a.db2[c] = sb;
            a.dbeta2[c] = (float)dbeta;
            a.dgamma2[c] = (float)dgamma;
            bn_bwd_coef(C, c, (double)N * a.HW, dgamma, dbeta, a.gamma2[c], a.bn2, a.coef2);
        }
        return;
    }
    i -= C;
    if (i < Cse) {
        float sb = 0.f;
        for (int n = ln; n < N; n += 32)
            sb += a.dq[(size_t)n * Cse + i];
        sb = half_wave_sum(sb);
        if (ln == 0)
            a.db1[i] = sb;
    }
}

hipError_t launch_se_bwd(const SeBwdArgs &a, hipStream_t st)
{
    hipLaunchKernelGGL(se_bwd_image_kernel, dim3(a.N), dim3(256), sizeof(float) * (a.C + a.Cse), st,
                       a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    const int total = 2 * a.C * a.Cse + a.C + a.Cse;
    hipLaunchKernelGGL(se_bwd_batch_kernel, dim3((total + 7) / 8), dim3(256), 0, st, a);
    return hipGetLastError();
}

// out[c*inner+i] = sum_n in[(c*N+n)*inner+i]
__global__ void reduce_planes_kernel(const float *__restrict__ in, int C, int N, int inner,
                                     float *__restrict__ out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= C * inner)
        return;
    const int c = i / inner, t = i - c * inner;
    float s = 0.f;
    for (int n = 0; n < N; ++n)
        s += in[((size_t)c * N + n) * inner + t];
    out[i] = s;
}

hipError_t launch_reduce_planes(const float *in, int C, int N, int inner, float *out,
                                hipStream_t st)
{
    const int total = C * inner;
    hipLaunchKernelGGL(reduce_planes_kernel, dim3((total + 255) / 256), dim3(256), 0, st, in, C, N,
                       inner, out);
    return hipGetLastError();
}

} // namespace mbk
