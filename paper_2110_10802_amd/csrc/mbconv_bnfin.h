// Batch-norm statistics finalised by the kernel that consumes them (device side).
#pragma once
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

// A group of TPP consecutive threads (lane index `lt` within the group) that works on channel c
// reduces that channel's partial sums itself and derives {scale, shift, mean, rstd}: the
// normalisation's finalise step costs no launch of its own.  Every group of the channel adds the
// same numbers in the same order, so all of them arrive at the same bits; the group for which
// `writer` holds also stores the block to f.bn_out and updates the running statistics.
// Partials are fp32 sums over at most a plane or a GEMM tile, combined in fp64.
// BN formula and running statistics: section "Statistical Normalization".
//
// Two phases, so that the caller can put its own loads between them: bn_fin_issue requests the
// partial sums (the first 4*TPP of them), bn_fin_finish consumes them.  Loads return in order,
// so the reduction waits for the partial sums only and runs while the caller's loads, issued
// after them, are still in flight.
// TPP > 64: one group per workgroup, every thread of the workgroup calls bn_fin_finish (it
// synchronises); `redd` is LDS scratch of 2*TPP/64 doubles.  TPP == 64: no LDS, no barrier.
// (Measured on the 56x56 block: leaving the reduction to the group's first wavefront and
// handing the coefficients over through LDS is slower than every wavefront taking a quarter of
// the partial sums: the chain behind the loads gets longer.)
struct BnFinRegs {
    float a0[4], a1[4];
    float gm, bt, rm, rv;
};

template <int TPP>
__device__ __forceinline__ void bn_fin_issue(const BnFin &f, int c, int lt, BnFinRegs &r)
{
    const float *ps = f.psum + (size_t)c * f.NP, *pq = f.psq + (size_t)c * f.NP;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = min(lt + TPP * u, f.NP - 1); // unconditional loads, masked when summed
        r.a0[u] = ps[i];
        r.a1[u] = pq[i];
    }
    r.gm = f.gamma[c];
    r.bt = f.beta[c];
    // (a null running-stat pointer reads gamma instead: no branch in front of the loads)
    r.rm = (f.run_mean ? f.run_mean : f.gamma)[c];
    r.rv = (f.run_var ? f.run_var : f.gamma)[c];
}

template <int TPP>
__device__ __forceinline__ void bn_fin_finish(const BnFin &f, int C, int c, int lt, bool writer,
                                              double *redd, const BnFinRegs &r, float &sc,
                                              float &sh, float &mu, float &rs)
{
    static_assert(TPP == 64 || TPP % 256 == 0, "one wavefront, or a whole workgroup");
    double s = 0.0, s2 = 0.0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (lt + TPP * u < f.NP) {
            s += (double)r.a0[u];
            s2 += (double)r.a1[u];
        }
    }
    if (f.NP > 4 * TPP) { // more partial sums than the first round holds
        const float *ps = f.psum + (size_t)c * f.NP, *pq = f.psq + (size_t)c * f.NP;
        for (int i0 = lt + 4 * TPP; i0 < f.NP; i0 += 4 * TPP) {
            float a0[4], a1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = min(i0 + TPP * u, f.NP - 1);
                a0[u] = ps[i];
                a1[u] = pq[i];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (i0 + TPP * u < f.NP) {
                    s += (double)a0[u];
                    s2 += (double)a1[u];
                }
            }
        }
    }
    s = wave_sum_d(s);
    s2 = wave_sum_d(s2);
    if (TPP > 64) {
        const int wv = lt >> 6;
        if ((lt & 63) == 0) {
            redd[2 * wv] = s;
            redd[2 * wv + 1] = s2;
        }
        __syncthreads();
        s = 0.0;
        s2 = 0.0;
#pragma unroll
        for (int w = 0; w < TPP / 64; ++w) {
            s += redd[2 * w];
            s2 += redd[2 * w + 1];
        }
    }
    const double mean = s * f.inv_m;
    double var = s2 * f.inv_m - mean * mean;
    if (var < 0.0)
        var = 0.0;
    // 1/sqrt: the hardware estimate and one Newton step (the result is rounded to fp32); for
    // eps = 0 and a constant channel the estimate is already the answer (inf, as 1/sqrt(0) in
    // the separate finalisation kernel) and the step would turn it into inf * 0
    const double xv = var + (double)f.eps;
    double rstd = __builtin_amdgcn_rsq(xv);
    if (xv > 0.0)
        rstd = rstd * (1.5 - 0.5 * xv * rstd * rstd);
    const double scale = (double)r.gm * rstd;
    sc = (float)scale;
    sh = (float)((double)r.bt - mean * scale);
    mu = (float)mean;
    rs = (float)rstd;
    if (writer && lt == 0) {
        f.bn_out[c] = sc;
        f.bn_out[C + c] = sh;
        f.bn_out[2 * C + c] = mu;
        f.bn_out[3 * C + c] = rs;
        if (f.run_mean)
            f.run_mean[c] = (float)((1.0 - (double)f.momentum) * (double)r.rm + (double)f.momentum * mean);
        if (f.run_var) {
            const double unbiased = var * f.unbias; // m/(m-1), or 1 when m == 1
            f.run_var[c] = (float)((1.0 - (double)f.momentum) * (double)r.rv + (double)f.momentum * unbiased);
        }
    }
}

} // namespace mbk
