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
                                                          float *run_var, float *bn, float *ones,
                                                          size_t ones_count)
{
    // a block without squeeze-and-excitation has its gate buffer set to one here, by the launch
    // that precedes the gate's first reader anyway
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < ones_count; i += (size_t)gridDim.x * 256)
        ones[i] = 1.0f;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (c >= C)
        return;
    // everything the last step needs is requested up front, and the partials are read four
    // strides at a time, so the kernel costs a few memory round trips whatever NP is
    const float gm = gamma[c], bt = beta[c];
    // (a null running-stat pointer reads gamma instead: no branch in front of the loads)
    const float rm = (run_mean ? run_mean : gamma)[c], rv = (run_var ? run_var : gamma)[c];
    const float *ps = psum + (size_t)c * NP, *pq = psq + (size_t)c * NP;
    double s = 0.0, s2 = 0.0;
    for (int i0 = lane; i0 < NP; i0 += 4 * kWave) {
        float a0[4], a1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = min(i0 + kWave * u, NP - 1); // unconditional loads, masked below
            a0[u] = ps[i];
            a1[u] = pq[i];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (i0 + kWave * u < NP) {
                s += (double)a0[u];
                s2 += (double)a1[u];
            }
        }
    }
    s = wave_sum_d(s);
    s2 = wave_sum_d(s2);
    if (lane == 0) {
        const double mean = s / m;
        double var = s2 / m - mean * mean;
        if (var < 0.0)
            var = 0.0;
        const double rstd = 1.0 / sqrt(var + (double)eps);
        const double scale = (double)gm * rstd;
        bn[c] = (float)scale;
        bn[C + c] = (float)((double)bt - mean * scale);
        bn[2 * C + c] = (float)mean;
        bn[3 * C + c] = (float)rstd;
        if (run_mean)
            run_mean[c] = (float)((1.0 - (double)momentum) * (double)rm + (double)momentum * mean);
        if (run_var) {
            const double unbiased = m > 1.0 ? var * m / (m - 1.0) : var;
            run_var[c] = (float)((1.0 - (double)momentum) * (double)rv + (double)momentum * unbiased);
        }
    }
}

hipError_t launch_bn_finalize(int C, int NP, double m, const float *psum, const float *psq,
                              const float *gamma, const float *beta, float eps, float momentum,
                              float *run_mean, float *run_var, float *bn, hipStream_t st,
                              float *ones, size_t ones_count)
{
    hipLaunchKernelGGL(bn_finalize_kernel, dim3((C + 3) / 4), dim3(256), 0, st, C, NP, m, psum, psq,
                       gamma, beta, eps, momentum, run_mean, run_var, bn, ones, ones ? ones_count : 0);
    return hipGetLastError();
}

// Evaluation mode: the same {scale, shift, mean, rstd} blocks from the stored running
// statistics, for up to three normalisations in one launch (a batch-norm layer with fixed
// statistics is an affine map per channel; section "Background and Related Work", paragraph
// "Training vs. inference compilation": BN behaves differently in inference).
struct BnEvalOne {
    int C;
    const float *gamma, *beta, *run_mean, *run_var;
    float *bn;
};
struct BnEvalArgs {
    BnEvalOne b[3];
    float eps;
};
__global__ __launch_bounds__(256) void bn_eval_coef_kernel(BnEvalArgs a)
{
    int i = blockIdx.x * 256 + threadIdx.x;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const BnEvalOne &b = a.b[k];
        if (i >= 0 && i < b.C) {
            const double mean = (double)b.run_mean[i];
            const double rstd = 1.0 / sqrt((double)b.run_var[i] + (double)a.eps);
            const double scale = (double)b.gamma[i] * rstd;
            b.bn[i] = (float)scale;
            b.bn[b.C + i] = (float)((double)b.beta[i] - mean * scale);
            b.bn[2 * b.C + i] = (float)mean;
            b.bn[3 * b.C + i] = (float)rstd;
        }
        i -= b.C;
    }
}

hipError_t launch_bn_eval_coef(int C1, const float *gamma1, const float *beta1, const float *rm1,
                               const float *rv1, float *bn1, int C2, const float *gamma2,
                               const float *beta2, const float *rm2, const float *rv2, float *bn2,
                               int C3, const float *gamma3, const float *beta3, const float *rm3,
                               const float *rv3, float *bn3, float eps, hipStream_t st)
{
    BnEvalArgs a;
    a.b[0] = {C1, gamma1, beta1, rm1, rv1, bn1};
    a.b[1] = {C2, gamma2, beta2, rm2, rv2, bn2};
    a.b[2] = {C3, gamma3, beta3, rm3, rv3, bn3};
    a.eps = eps;
    const int total = C1 + C2 + C3;
    hipLaunchKernelGGL(bn_eval_coef_kernel, dim3((total + 255) / 256), dim3(256), 0, st, a);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_kernel(float *out, float value, size_t count)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count)
        out[i] = value;
}

hipError_t launch_fill(float *out, float value, size_t count, hipStream_t st)
{
    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, out,
                       value, count);
    return hipGetLastError();
}

// dx = gamma*rstd*(dy - dbeta/m - xhat*dgamma/m) with xhat = (raw-mean)*rstd, rewritten as
// c0*dy + c1*raw + c2 so the consumer's prologue is two fused multiply-adds.
__device__ __forceinline__ void bn_bwd_coef_vals(int C, int c, double m, double dgamma, double dbeta,
                                                 float gamma, double mean, double rstd, float *coef)
{
    const double c0 = (double)gamma * rstd;
    const double c1 = -c0 * rstd * dgamma / m;
    const double c2 = -c0 * dbeta / m - c1 * mean;
    coef[c] = (float)c0;
    coef[C + c] = (float)c1;
    coef[2 * C + c] = (float)c2;
}
__device__ __forceinline__ void bn_bwd_coef(int C, int c, double m, double dgamma, double dbeta,
                                            float gamma, const float *bn, float *coef)
{
    bn_bwd_coef_vals(C, c, m, dgamma, dbeta, gamma, bn[2 * C + c], bn[3 * C + c], coef);
}

__device__ __forceinline__ void bn_bwd_finalize_body(int block, int C, int NP, double m,
                                                     const float *__restrict__ psb,
                                                     const float *__restrict__ psr,
                                                     const float *__restrict__ gamma,
                                                     const float *__restrict__ bn, float *dgamma,
                                                     float *dbeta, float *coef)
{
    const int c = block * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (c >= C)
        return;
    const float gm = gamma[c], mean = bn[2 * C + c], rstd = bn[3 * C + c]; // requested up front
    const float *pb = psb + (size_t)c * NP, *pr = psr + (size_t)c * NP;
    double sb = 0.0, sr = 0.0;
    for (int i0 = lane; i0 < NP; i0 += 4 * kWave) {
        float a0[4], a1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = min(i0 + kWave * u, NP - 1); // unconditional loads, masked below
            a0[u] = pb[i];
            a1[u] = pr[i];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (i0 + kWave * u < NP) {
                sb += (double)a0[u];
                sr += (double)a1[u];
            }
        }
    }
    sb = wave_sum_d(sb);
    sr = wave_sum_d(sr);
    if (lane == 0) {
        if (dbeta)
            dbeta[c] = (float)sb;
        if (dgamma)
            dgamma[c] = (float)sr;
        bn_bwd_coef_vals(C, c, m, sr, sb, gm, mean, rstd, coef);
    }
}

__global__ __launch_bounds__(256) void bn_bwd_finalize_kernel(int C, int NP, double m,
                                                              const float *__restrict__ psb,
                                                              const float *__restrict__ psr,
                                                              const float *__restrict__ gamma,
                                                              const float *__restrict__ bn,
                                                              float *dgamma, float *dbeta,
                                                              float *coef)
{
    bn_bwd_finalize_body(blockIdx.x, C, NP, m, psb, psr, gamma, bn, dgamma, dbeta, coef);
}

// Block without squeeze-and-excitation: one wavefront per channel adds the plane sums of the
// batch in a fixed order (lane l takes images l, l+64, ...; fp64 butterfly), writes BN2's
// parameter gradients and backward coefficients, and zeroes the channel's column of dzs.
__global__ __launch_bounds__(256) void bn2_bwd_nose_kernel(int N, int C, double m,
                                                           const float *__restrict__ A1,
                                                           const float *__restrict__ A2,
                                                           const float *__restrict__ gamma,
                                                           const float *__restrict__ bn,
                                                           float *dgamma, float *dbeta, float *coef,
                                                           float *dzs)
{
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (c >= C)
        return;
    double sb = 0.0, sr = 0.0;
    for (int n = lane; n < N; n += kWave) {
        sb += (double)A1[(size_t)n * C + c];
        sr += (double)A2[(size_t)n * C + c];
        dzs[(size_t)n * C + c] = 0.f;
    }
    sb = wave_sum_d(sb);
    sr = wave_sum_d(sr);
    if (lane == 0) {
        dbeta[c] = (float)sb;
        dgamma[c] = (float)sr;
        bn_bwd_coef(C, c, m, sr, sb, gamma[c], bn, coef);
    }
}

hipError_t launch_bn2_bwd_nose(int N, int C, double m, const float *A1, const float *A2,
                               const float *gamma, const float *bn, float *dgamma, float *dbeta,
                               float *coef, float *dzs, hipStream_t st)
{
    hipLaunchKernelGGL(bn2_bwd_nose_kernel, dim3((C + 3) / 4), dim3(256), 0, st, N, C, m, A1, A2,
                       gamma, bn, dgamma, dbeta, coef, dzs);
    return hipGetLastError();
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

// The same for wide blocks (hundreds of channels): a workgroup per (image, channel slice).
// Every workgroup of an image recomputes the whole of q (Cse dot products of length C: cheap,
// and it keeps the kernel free of a grid-wide dependency), then produces g for its slice.
// A dependent global load costs about a microsecond here, so every phase issues all of its
// loads before it consumes any: loops are unrolled over compile-time bounds (CI*256 >= C,
// Cse <= 64) with guards.  Requires Cse % 4 == 0.
template <int CI>
__global__ __launch_bounds__(256) void se_fwd_wide_kernel(int C, int Cse, int slice,
                                                          const float *__restrict__ z,
                                                          const float *__restrict__ w1,
                                                          const float *__restrict__ b1,
                                                          const float *__restrict__ w2,
                                                          const float *__restrict__ b2, float *q,
                                                          float *g)
{
    __shared__ float part[4][64];
    __shared__ float rs[64];
    const int n = blockIdx.x, sl = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float zv[CI];
#pragma unroll
    for (int i = 0; i < CI; ++i) {
        const int c = tid + 256 * i;
        zv[i] = c < C ? z[(size_t)n * C + c] : 0.f;
    }
    for (int jb = 0; jb < Cse; jb += 16) {
        float wv[16][CI];
        // unconditional loads from clamped indices: rows past Cse repeat the last row (their
        // sums are never read), columns past C meet zv = 0
#pragma unroll
        for (int u = 0; u < 16; ++u)
#pragma unroll
            for (int i = 0; i < CI; ++i) {
                const int c = min(tid + 256 * i, C - 1);
                wv[u][i] = w1[(size_t)min(jb + u, Cse - 1) * C + c];
            }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < CI; ++i)
                acc = fmaf(wv[u][i], zv[i], acc);
            acc = wave_sum(acc);
            if (lane == 0)
                part[wave][jb + u] = acc;
        }
    }
    __syncthreads();
    if (tid < Cse) {
        const float qv = (part[0][tid] + part[1][tid]) + (part[2][tid] + part[3][tid]) + b1[tid];
        if (sl == 0)
            q[(size_t)n * Cse + tid] = qv;
        rs[tid] = swishf(qv);
    }
    __syncthreads();
    const int cend = min(C, (sl + 1) * slice);
    for (int c = sl * slice + tid; c < cend; c += 256) {
        const float4 *row = reinterpret_cast<const float4 *>(w2 + (size_t)c * Cse);
        // unconditional loads (a quad past the end re-reads the last one and is masked): a
        // branch around each load would make every load wait for the previous one
        const int lastq = (Cse >> 2) - 1;
        float4 w[16];
#pragma unroll
        for (int jj = 0; jj < 16; ++jj)
            w[jj] = row[min(jj, lastq)];
        float acc = b2[c];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const bool ok = jj <= lastq;
            const int j4 = 4 * min(jj, lastq);
            acc = fmaf(ok ? w[jj].x : 0.f, rs[j4], acc);
            acc = fmaf(ok ? w[jj].y : 0.f, rs[j4 + 1], acc);
            acc = fmaf(ok ? w[jj].z : 0.f, rs[j4 + 2], acc);
            acc = fmaf(ok ? w[jj].w : 0.f, rs[j4 + 3], acc);
        }
        g[(size_t)n * C + c] = sigmoidf_fast(acc);
    }
}

// channel slices per image so that a wide block launches a few hundred workgroups
static int se_slices(int N, int C)
{
    int G = (512 + N - 1) / N;
    const int maxG = (C + 63) / 64;
    if (G > maxG)
        G = maxG;
    if (G > 8)
        G = 8;
    return G < 1 ? 1 : G;
}
static bool se_wide(int C, int Cse)
{
    return C >= 256 && C <= 2048 && C % 4 == 0 && Cse % 4 == 0 && Cse <= 64;
}

hipError_t launch_se_fwd(int N, int C, int Cse, const float *z, const float *w1, const float *b1,
                         const float *w2, const float *b2, float *q, float *g, hipStream_t st)
{
    if (se_wide(C, Cse)) {
        const int G = se_slices(N, C), slice = (C + G - 1) / G;
        if (C <= 768)
            hipLaunchKernelGGL(se_fwd_wide_kernel<3>, dim3(N, G), dim3(256), 0, st, C, Cse, slice, z,
                               w1, b1, w2, b2, q, g);
        else if (C <= 1280)
            hipLaunchKernelGGL(se_fwd_wide_kernel<5>, dim3(N, G), dim3(256), 0, st, C, Cse, slice, z,
                               w1, b1, w2, b2, q, g);
        else
            hipLaunchKernelGGL(se_fwd_wide_kernel<8>, dim3(N, G), dim3(256), 0, st, C, Cse, slice, z,
                               w1, b1, w2, b2, q, g);
        return hipGetLastError();
    }
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

// Wide-block variants of the two SE backward kernels (Cse % 4 == 0, Cse <= 64).
// Per (image, channel slice): dt for every channel, dq by a [C x Cse] sweep of W2 with float4
// loads (a thread owns four consecutive j of every RP-th row; row groups are combined in LDS in
// a fixed order), then dzs for the slice.
__global__ __launch_bounds__(256) void se_bwd_image_wide_kernel(SeBwdArgs a, int slice)
{
    extern __shared__ float lds[];
    const int C = a.C, Cse = a.Cse;
    float *dts = lds, *dqs = lds + C, *red = dqs + Cse; // red: [RP][Cse]
    const int n = blockIdx.x, part = blockIdx.y, tid = threadIdx.x;
    for (int c = tid; c < C; c += 256) {
        const float gv = a.g[(size_t)n * C + c];
        const float v = a.dg[(size_t)n * C + c] * gv * (1.f - gv);
        dts[c] = v;
        if (part == 0)
            a.dt[(size_t)n * C + c] = v;
    }
    __syncthreads();
    const int JQ = Cse >> 2, RP = 256 / JQ;
    const int jq = tid % JQ, r0 = tid / JQ;
    if (r0 < RP) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int cb = r0; cb < C; cb += 16 * RP) { // 16 independent loads per round
            float4 w[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int c = cb + u * RP;
                w[u] = c < C ? *reinterpret_cast<const float4 *>(a.w2 + (size_t)c * Cse + 4 * jq)
                             : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int c = cb + u * RP;
                const float d = c < C ? dts[c] : 0.f;
                acc.x = fmaf(w[u].x, d, acc.x);
                acc.y = fmaf(w[u].y, d, acc.y);
                acc.z = fmaf(w[u].z, d, acc.z);
                acc.w = fmaf(w[u].w, d, acc.w);
            }
        }
        *reinterpret_cast<float4 *>(red + (size_t)r0 * Cse + 4 * jq) = acc;
    }
    __syncthreads();
    if (tid < Cse) {
        float s = 0.f;
        for (int r = 0; r < RP; ++r)
            s += red[(size_t)r * Cse + tid];
        float val, grad;
        swish_both(a.q[(size_t)n * Cse + tid], val, grad);
        const float v = s * grad;
        dqs[tid] = v;
        if (part == 0)
            a.dq[(size_t)n * Cse + tid] = v;
    }
    __syncthreads();
    const float inv = 1.f / (float)a.HW;
    const int cend = min(C, (part + 1) * slice);
    for (int c = part * slice + tid; c < cend; c += 256) {
        float acc = 0.f;
        for (int j0 = 0; j0 < Cse; j0 += 16) { // sixteen unconditional loads per round
            float w[16];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                w[u] = a.w1[(size_t)min(j0 + u, Cse - 1) * C + c];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 16; ++u)
                acc = fmaf(j0 + u < Cse ? w[u] : 0.f, dqs[min(j0 + u, Cse - 1)], acc);
        }
        a.dzs[(size_t)n * C + c] = acc * inv;
    }
}

// Sums over the batch for a tile of 16 channels: thread (c, jq) owns dW2[c][4jq..4jq+3] and
// dW1[4jq..4jq+3][c]; the batch is walked 32 images at a time through LDS, always in the same
// order, and the j-contiguous operands are read as one 16-byte LDS access per image.  The
// per-channel sums (db2, BN2's dbeta/dgamma/coef) are split over the 16 jq groups and combined
// in a fixed order.  The three kinds of sums are independent chains of memory round trips and
// there are far fewer channel tiles than compute units, so each kind has workgroups of its own
// (blockIdx.y: 0 the weight gradients, 1 the per-channel sums, 2 db1 in one workgroup) and the
// launch lasts as long as the longest chain, not their sum.
__global__ __launch_bounds__(256) void se_bwd_batch_wide_kernel(SeBwdArgs a)
{
    constexpr int TC = 16, TN = 32, JQ = 16; // Cse <= 4*JQ
    __shared__ float dtL[TN][TC], zL[TN][TC];
    __shared__ __attribute__((aligned(16))) float rL[TN][4 * JQ], dqL[TN][4 * JQ];
    __shared__ float sbL[JQ][TC];
    __shared__ double dbL[JQ][TC], dgL[JQ][TC];
    const int C = a.C, Cse = a.Cse, N = a.N;
    const int tid = threadIdx.x, cl = tid & 15, jq = tid >> 4;
    const int c0 = blockIdx.x * TC, c = c0 + cl;
    const int role = blockIdx.y;
    if (role == 0) {
        float acc2[4] = {0.f, 0.f, 0.f, 0.f}, acc1[4] = {0.f, 0.f, 0.f, 0.f};
        // A round's loads (all in flight together, clamped addresses and masks instead of branches)
        // are issued one round ahead: they travel while the previous round is multiplied.
        float t0[2], t1[2], t2[8], t3[8];
        const auto fetch = [&](int n0) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int i = tid + 256 * u, nn = i >> 4, cc = i & 15;
                const bool ok = n0 + nn < N && c0 + cc < C;
                const size_t at = ok ? (size_t)(n0 + nn) * C + c0 + cc : 0;
                t0[u] = and_mask(a.dt[at], ok ? 0xffffffffu : 0u);
                t1[u] = and_mask(a.z[at], ok ? 0xffffffffu : 0u);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = tid + 256 * u, nn = i >> 6, j = i & 63;
                const bool ok = n0 + nn < N && j < Cse;
                const size_t at = ok ? (size_t)(n0 + nn) * Cse + j : 0;
                t2[u] = and_mask(a.q[at], ok ? 0xffffffffu : 0u);
                t3[u] = and_mask(a.dq[at], ok ? 0xffffffffu : 0u);
            }
        };
        fetch(0);
        for (int n0 = 0; n0 < N; n0 += TN) {
            __syncthreads();
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int i = tid + 256 * u;
                dtL[i >> 4][i & 15] = t0[u];
                zL[i >> 4][i & 15] = t1[u];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = tid + 256 * u;
                rL[i >> 6][i & 63] = (i & 63) < Cse ? swishf(t2[u]) : 0.f;
                dqL[i >> 6][i & 63] = t3[u];
            }
            if (n0 + TN < N)
                fetch(n0 + TN);
            __syncthreads();
#pragma unroll 8
            for (int nn = 0; nn < TN; ++nn) {
                const float dtv = dtL[nn][cl], zv = zL[nn][cl];
                const float4 r4 = *reinterpret_cast<const float4 *>(&rL[nn][4 * jq]);
                const float4 q4 = *reinterpret_cast<const float4 *>(&dqL[nn][4 * jq]);
                acc2[0] = fmaf(dtv, r4.x, acc2[0]);
                acc2[1] = fmaf(dtv, r4.y, acc2[1]);
                acc2[2] = fmaf(dtv, r4.z, acc2[2]);
                acc2[3] = fmaf(dtv, r4.w, acc2[3]);
                acc1[0] = fmaf(q4.x, zv, acc1[0]);
                acc1[1] = fmaf(q4.y, zv, acc1[1]);
                acc1[2] = fmaf(q4.z, zv, acc1[2]);
                acc1[3] = fmaf(q4.w, zv, acc1[3]);
            }
        }
        if (c < C) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = 4 * jq + u;
                if (j < Cse) {
                    a.dw2[(size_t)c * Cse + j] = acc2[u];
                    a.dw1[(size_t)j * C + c] = acc1[u];
                }
            }
        }
    } else if (role == 1) {
        // per-channel sums: the 16 thread groups take every 16th image, then group 0 adds the
        // partial sums in order
        float sb = 0.f;
        double dbeta = 0.0, dgamma = 0.0;
        if (c < C) {
#pragma unroll 8
            for (int n = jq; n < N; n += JQ) {
                const size_t o = (size_t)n * C + c;
                const float dtv = a.dt[o], gv = a.g[o], a1 = a.A1[o], a2 = a.A2[o];
                const float dz = a.dzs[o], s3 = a.s3[o], s4 = a.s4[o];
                sb += dtv;
                dbeta += (double)gv * a1 + (double)dz * s3;
                dgamma += (double)gv * a2 + (double)dz * s4;
            }
        }
        sbL[jq][cl] = sb;
        dbL[jq][cl] = dbeta;
        dgL[jq][cl] = dgamma;
        __syncthreads();
        if (jq == 0 && c < C) {
            sb = 0.f;
            dbeta = dgamma = 0.0;
            for (int u = 0; u < JQ; ++u) {
                sb += sbL[u][cl];
                dbeta += dbL[u][cl];
                dgamma += dgL[u][cl];
            }
            a.db2[c] = sb;
            a.dbeta2[c] = (float)dbeta;
            a.dgamma2[c] = (float)dgamma;
            bn_bwd_coef(C, c, (double)N * a.HW, dgamma, dbeta, a.gamma2[c], a.bn2, a.coef2);
        }
    } else if (blockIdx.x == 0) {
        // db1[j] = sum_n dq[n][j]: four thread groups take every fourth image (sixteen loads in
        // flight each: a plain loop would pay one memory round trip per image), combined in a
        // fixed order
        __shared__ float db1L[4][64];
        const int j = tid & 63, part = tid >> 6;
        float s = 0.f;
        if (j < Cse) {
#pragma unroll 16
            for (int n = part; n < N; n += 4)
                s += a.dq[(size_t)n * Cse + j];
        }
        db1L[part][j] = s;
        __syncthreads();
        if (tid < Cse)
            a.db1[tid] = (db1L[0][tid] + db1L[1][tid]) + (db1L[2][tid] + db1L[3][tid]);
    }
}

hipError_t launch_se_bwd(const SeBwdArgs &a, hipStream_t st)
{
    if (se_wide(a.C, a.Cse)) {
        const int G = se_slices(a.N, a.C), slice = (a.C + G - 1) / G;
        const int RP = 256 / (a.Cse / 4);
        const size_t lds = sizeof(float) * ((size_t)a.C + a.Cse + (size_t)RP * a.Cse);
        hipLaunchKernelGGL(se_bwd_image_wide_kernel, dim3(a.N, G), dim3(256), lds, st, a, slice);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
        hipLaunchKernelGGL(se_bwd_batch_wide_kernel, dim3((a.C + 15) / 16, 3), dim3(256), 0, st, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(se_bwd_image_kernel, dim3(a.N), dim3(256), sizeof(float) * (a.C + a.Cse), st,
                       a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    const int total = 2 * a.C * a.Cse + a.C + a.Cse;
    hipLaunchKernelGGL(se_bwd_batch_kernel, dim3((total + 7) / 8), dim3(256), 0, st, a);
    return hipGetLastError();
}

// out[c*inner+i] = sum_n in[(c*N+n)*inner+i].  Eight lanes share an output: lane s adds
// the images s, s+8, ... and the eight partial sums are combined by a fixed butterfly.
__device__ __forceinline__ void reduce_planes_body(int block, const float *__restrict__ in, int C,
                                                   int N, int inner, float *__restrict__ out)
{
    const int gid = block * 256 + threadIdx.x;
    const int i = gid >> 3, sub = gid & 7;
    float s = 0.f;
    if (i < C * inner) {
        const int c = i / inner, t = i - c * inner;
        const float *src = in + (size_t)c * N * inner + t;
        float s0 = 0.f, s1 = 0.f;
        int n = sub;
        for (; n + 8 < N; n += 16) {
            s0 += src[(size_t)n * inner];
            s1 += src[(size_t)(n + 8) * inner];
        }
        if (n < N)
            s0 += src[(size_t)n * inner];
        s = s0 + s1;
    }
    s += __shfl_xor(s, 4, kWave);
    s += __shfl_xor(s, 2, kWave);
    s += __shfl_xor(s, 1, kWave);
    if (sub == 0 && i < C * inner)
        out[i] = s;
}

__global__ __launch_bounds__(256) void reduce_planes_kernel(const float *__restrict__ in, int C,
                                                            int N, int inner,
                                                            float *__restrict__ out)
{
    reduce_planes_body(blockIdx.x, in, C, N, inner, out);
}

// The two second stages that follow the fused depthwise backward, in one launch: the first nb1
// workgroups add the filter-gradient partials, the others finalise BN1's backward.
__global__ __launch_bounds__(256) void dw_bwd_finalize_kernel(int nb1, const float *__restrict__ pdw,
                                                              int C, int NP, int inner,
                                                              float *__restrict__ dw, double m,
                                                              const float *__restrict__ psb,
                                                              const float *__restrict__ psr,
                                                              const float *__restrict__ gamma,
                                                              const float *__restrict__ bn,
                                                              float *dgamma, float *dbeta,
                                                              float *coef)
{
    if ((int)blockIdx.x < nb1)
        reduce_planes_body(blockIdx.x, pdw, C, NP, inner, dw);
    else
        bn_bwd_finalize_body(blockIdx.x - nb1, C, NP, m, psb, psr, gamma, bn, dgamma, dbeta, coef);
}

hipError_t launch_dw_bwd_finalize(const float *pdw, int C, int NP, int inner, float *dw, double m,
                                  const float *psb, const float *psr, const float *gamma,
                                  const float *bn, float *dgamma, float *dbeta, float *coef,
                                  hipStream_t st)
{
    const long long total = (long long)C * inner * 8;
    const int nb1 = (int)((total + 255) / 256), nb2 = (C + 3) / 4;
    hipLaunchKernelGGL(dw_bwd_finalize_kernel, dim3((unsigned)(nb1 + nb2)), dim3(256), 0, st, nb1, pdw,
                       C, NP, inner, dw, m, psb, psr, gamma, bn, dgamma, dbeta, coef);
    return hipGetLastError();
}

hipError_t launch_reduce_planes(const float *in, int C, int N, int inner, float *out,
                                hipStream_t st)
{
    const long long total = (long long)C * inner * 8;
    hipLaunchKernelGGL(reduce_planes_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       in, C, N, inner, out);
    return hipGetLastError();
}

} // namespace mbk
