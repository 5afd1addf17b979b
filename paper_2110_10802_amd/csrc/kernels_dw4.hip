// Vectorised depthwise chain for stride 1 and plane width a multiple of 4 (the 112, 56, 28
// and 14 wide EfficientNet stages).
//
// Same plan as kernels_dw.hip (whole plane in LDS with a zero border, BN + Swish evaluated
// once per input element while staging, no atomics), restructured so that every global and
// LDS access is 16 bytes per lane and every thread keeps the element positions it staged:
//   - a thread owns up to NG runs of four consecutive pixels; it loads them as float4,
//     applies BN + Swish and writes the run to LDS with one ds_write_b128 (the interior of a
//     tile row starts at column 4, so runs are 16-byte aligned);
//   - the k x k stencil of a run reads, per filter row, one ds_read_b128 plus the (k-1)
//     neighbours, i.e. about one LDS instruction per output instead of k*k;
//   - backward keeps y1 and sigmoid(y1) of its own runs in registers between staging and the
//     Swish' multiplication, so the expansion output e is read once (recompute without a second
//     load; section "Backpropagation and Data Movement" of the paper).
#include "mbconv_dev.h"
#include "mbconv_launch.h"
#include "mbconv_bnfin.h"

namespace mbk {

typedef float float4v __attribute__((ext_vector_type(4)));

template <typename T>
__device__ __forceinline__ void gload4(const T *p, size_t i, float (&v)[4]);
template <>
__device__ __forceinline__ void gload4<float>(const float *p, size_t i, float (&v)[4])
{
    const float4v t = *reinterpret_cast<const float4v *>(p + i);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
}
template <>
__device__ __forceinline__ void gload4<bf16_t>(const bf16_t *p, size_t i, float (&v)[4])
{
    const uint2 t = *reinterpret_cast<const uint2 *>(&p[i]);
    v[0] = bf16_bits_to_float(t.x & 0xffffu);
    v[1] = bf16_bits_to_float(t.x >> 16);
    v[2] = bf16_bits_to_float(t.y & 0xffffu);
    v[3] = bf16_bits_to_float(t.y >> 16);
}
template <typename T>
__device__ __forceinline__ void gstore4(T *p, size_t i, const float (&v)[4]);
template <>
__device__ __forceinline__ void gstore4<float>(float *p, size_t i, const float (&v)[4])
{
    float4v t = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<float4v *>(p + i) = t;
}
template <>
__device__ __forceinline__ void gstore4<bf16_t>(bf16_t *p, size_t i, const float (&v)[4])
{
    uint2 t;
    t.x = bf16_pack2(v[0], v[1]);
    t.y = bf16_pack2(v[2], v[3]);
    *reinterpret_cast<uint2 *>(&p[i]) = t;
}

struct Dw4Args {
    int N, C, H, W;
    int WP;      // tile pitch = W + 8
    int groups;  // H*W/4
    FastDiv divC, divW4; // W/4
    // forward
    const void *e;
    const float *bn1;
    const void *w;
    void *d;
    float *psum, *psq;
    BnFin fin; // fin.psum non-null: bn1 is derived in the forward kernel from the partial sums
    int PL;    // forward, planes per workgroup (images n0..n0+PL-1 of one channel), 1: a plane each
    // backward
    const void *G;
    const float *g, *dzs, *bn2, *coef2;
    void *dy1_out;
    const void *res;
    float *pdw, *psb, *psr;
};

template <int TPP>
__device__ __forceinline__ bool plane_of(const Dw4Args &a, size_t &plane, int &n, int &c)
{
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    constexpr int PPB = BLOCK / TPP;
    const size_t pl = (size_t)blockIdx.x * PPB + threadIdx.x / TPP;
    const bool active = pl < (size_t)a.N * a.C;
    plane = active ? pl : 0;
    n = (int)fdiv((uint32_t)plane, a.divC);
    c = (int)(plane - (size_t)n * a.C);
    return active;
}

// Zero the border of a tile: the two 4-column pads of every row, and the P top/bottom rows.
template <int P, int TPP>
__device__ __forceinline__ void zero_border(float *tile, int H, int W, int WP, int lt)
{
    const float4v z = {0.f, 0.f, 0.f, 0.f};
    const int rows = H + 2 * P;
    for (int r = lt; r < rows; r += TPP) {
        *reinterpret_cast<float4v *>(tile + r * WP) = z;
        *reinterpret_cast<float4v *>(tile + r * WP + 4 + W) = z;
    }
    const int w4 = W >> 2;
    for (int i = lt; i < 2 * P * w4; i += TPP) {
        const int rr = i / w4, cc = i - rr * w4;
        const int r = rr < P ? rr : H + rr; // rows 0..P-1 and H+P..H+2P-1
        *reinterpret_cast<float4v *>(tile + r * WP + 4 + 4 * cc) = z;
    }
}

// One row of a (K+3)-wide window starting at column (4 + w - P) of tile row `row`.
template <int K>
__device__ __forceinline__ void read_window_row(const float *tile, int row, int WP, int w,
                                                float (&o)[K + 3])
{
    constexpr int P = (K - 1) / 2;
    const float *p = tile + row * WP + 4 + w;
    const float4v m = *reinterpret_cast<const float4v *>(p);
    if (P == 1) {
        o[0] = p[-1];
        o[5] = p[4];
    } else {
        const float2 l = *reinterpret_cast<const float2 *>(p - 2);
        const float2 r = *reinterpret_cast<const float2 *>(p + 4);
        o[0] = l.x;
        o[1] = l.y;
        o[K + 1] = r.x;
        o[K + 2] = r.y;
    }
    o[P] = m.x;
    o[P + 1] = m.y;
    o[P + 2] = m.z;
    o[P + 3] = m.w;
}

// ---- forward ---------------------------------------------------------------------------------

template <typename T, int K, int TPP, int NG, bool EXPAND>
__global__ __launch_bounds__(TPP > 256 ? TPP : 256) void dw4_fwd_kernel(Dw4Args a)
{
    constexpr int P = (K - 1) / 2;
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    constexpr int PPB = BLOCK / TPP;
    extern __shared__ float lds[];
    const int H = a.H, W = a.W, WP = a.WP;
    const int tileElems = (H + 2 * P) * WP;
    const int lt = threadIdx.x % TPP;
    float *tile = lds + (threadIdx.x / TPP) * tileElems;
    float *red = lds + PPB * tileElems;
    __shared__ double redd[2 * (BLOCK / 64)];
    size_t plane;
    int n, c;
    const bool active = plane_of<TPP>(a, plane, n, c);

    float wt[K * K];
    if (active) { // (TPP > 64: one plane per workgroup, always active)
        // BN1's coefficients are requested first (or the partial sums they are finalised from),
        // then the plane: loads return in order, so the finalisation runs while the plane's data
        // is still on its way
        float scale = 1.f, shift = 0.f;
        BnFinRegs fr;
        if (EXPAND) {
            if (a.fin.psum) {
                bn_fin_issue<TPP>(a.fin, c, lt, fr);
            } else {
                scale = a.bn1[c];
                shift = a.bn1[a.C + c];
            }
        }
#pragma unroll
        for (int t = 0; t < K * K; ++t)
            wt[t] = ld<T>((const T *)a.w, (size_t)c * K * K + t);
        __builtin_amdgcn_sched_barrier(0);
        zero_border<P, TPP>(tile, H, W, WP, lt);
        const size_t base = plane * (size_t)H * W;
        // all runs of the thread are loaded before any is transformed (one memory round trip,
        // not one per run; the fence keeps the scheduler from re-pairing load and use)
        float ev[NG][4];
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int gidx = lt + TPP * i;
            gload4<T>((const T *)a.e, base + 4 * (size_t)(gidx < a.groups ? gidx : 0), ev[i]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (EXPAND && a.fin.psum) {
            float mu, rs;
            bn_fin_finish<TPP>(a.fin, a.C, c, lt, n == 0, redd, fr, scale, shift, mu, rs);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int gidx = lt + TPP * i;
            if (gidx < a.groups) {
                const int h = (int)fdiv((uint32_t)gidx, a.divW4);
                const int w = 4 * (gidx - h * (W >> 2));
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    v[r] = ev[i][r];
                if (EXPAND) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        v[r] = actf(fmaf(v[r], scale, shift));
                }
                float4v t4 = {v[0], v[1], v[2], v[3]};
                *reinterpret_cast<float4v *>(tile + (h + P) * WP + 4 + w) = t4;
            }
        }
    }
    __syncthreads();
    float acc2[2] = {0.f, 0.f};
    if (active) {
        const size_t base = plane * (size_t)H * W;
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int gidx = lt + TPP * i;
            if (gidx < a.groups) {
                const int h = (int)fdiv((uint32_t)gidx, a.divW4);
                const int w = 4 * (gidx - h * (W >> 2));
                float o[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int u = 0; u < K; ++u) {
                    float row[K + 3];
                    read_window_row<K>(tile, h + u, WP, w, row);
#pragma unroll
                    for (int v = 0; v < K; ++v)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            o[r] = fmaf(wt[u * K + v], row[r + v], o[r]);
                }
                gstore4<T>((T *)a.d, base + 4 * (size_t)gidx, o);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float sv = as_stored<T>(o[r]);
                    acc2[0] += sv;
                    acc2[1] = fmaf(sv, sv, acc2[1]);
                }
            }
        }
    }
    group_sum<2, TPP>(acc2, red);
    if (active && lt == 0) {
        a.psum[(size_t)c * a.N + n] = acc2[0];
        a.psq[(size_t)c * a.N + n] = acc2[1];
    }
}

// The same for a workgroup of 256 threads that walks PL images of one channel: the filter, the
// BN1 constants (or their finalisation from the partial sums), and the tile's zero border are set
// up once, and the next plane's loads are issued before the current plane is convolved, so they
// travel under the arithmetic.
template <typename T, int K, int NG, bool EXPAND>
__global__ __launch_bounds__(256) void dw4_fwd_multi_kernel(Dw4Args a)
{
    constexpr int P = (K - 1) / 2, TPP = 256;
    extern __shared__ float lds[];
    const int H = a.H, W = a.W, WP = a.WP;
    const int tileElems = (H + 2 * P) * WP;
    const int lt = threadIdx.x;
    float *tile = lds;
    float *red = lds + tileElems;
    __shared__ double redd[2 * (TPP / 64)];
    const int ngrp = (int)fdiv(blockIdx.x, a.divC), c = (int)blockIdx.x - ngrp * a.C;
    const int n0 = ngrp * a.PL, n1 = min(a.N, n0 + a.PL);
    const size_t HW = (size_t)H * W;

    float wt[K * K];
    float scale = 1.f, shift = 0.f;
    BnFinRegs fr;
    if (EXPAND) {
        if (a.fin.psum) {
            bn_fin_issue<TPP>(a.fin, c, lt, fr);
        } else {
            scale = a.bn1[c];
            shift = a.bn1[a.C + c];
        }
    }
#pragma unroll
    for (int t = 0; t < K * K; ++t)
        wt[t] = ld<T>((const T *)a.w, (size_t)c * K * K + t);
    __builtin_amdgcn_sched_barrier(0);
    zero_border<P, TPP>(tile, H, W, WP, lt);
    float ev[NG][4];
    const auto fetch = [&](int n) {
        const size_t base = ((size_t)n * a.C + c) * HW;
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int gidx = lt + TPP * i;
            gload4<T>((const T *)a.e, base + 4 * (size_t)(gidx < a.groups ? gidx : 0), ev[i]);
        }
    };
    fetch(n0);
    __builtin_amdgcn_sched_barrier(0);
    if (EXPAND && a.fin.psum) {
        float mu, rs;
        bn_fin_finish<TPP>(a.fin, a.C, c, lt, n0 == 0, redd, fr, scale, shift, mu, rs);
    }
    __builtin_amdgcn_sched_barrier(0);
    for (int n = n0; n < n1; ++n) {
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int gidx = lt + TPP * i;
            if (gidx < a.groups) {
                const int h = (int)fdiv((uint32_t)gidx, a.divW4);
                const int w = 4 * (gidx - h * (W >> 2));
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    v[r] = EXPAND ? actf(fmaf(ev[i][r], scale, shift)) : ev[i][r];
                float4v t4 = {v[0], v[1], v[2], v[3]};
                *reinterpret_cast<float4v *>(tile + (h + P) * WP + 4 + w) = t4;
            }
        }
        __syncthreads();
        if (n + 1 < n1)
            fetch(n + 1);
        float acc2[2] = {0.f, 0.f};
        const size_t base = ((size_t)n * a.C + c) * HW;
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int gidx = lt + TPP * i;
            if (gidx < a.groups) {
                const int h = (int)fdiv((uint32_t)gidx, a.divW4);
                const int w = 4 * (gidx - h * (W >> 2));
                float o[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int u = 0; u < K; ++u) {
                    float row[K + 3];
                    read_window_row<K>(tile, h + u, WP, w, row);
#pragma unroll
                    for (int v = 0; v < K; ++v)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            o[r] = fmaf(wt[u * K + v], row[r + v], o[r]);
                }
                gstore4<T>((T *)a.d, base + 4 * (size_t)gidx, o);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float sv = as_stored<T>(o[r]);
                    acc2[0] += sv;
                    acc2[1] = fmaf(sv, sv, acc2[1]);
                }
            }
        }
        // (two barriers inside: every read of this plane's tile precedes the next plane's stores)
        group_sum<2, TPP>(acc2, red);
        if (lt == 0) {
            a.psum[(size_t)c * a.N + n] = acc2[0];
            a.psq[(size_t)c * a.N + n] = acc2[1];
        }
    }
}

// ---- backward ----------------------------------------------------------------------------------

// (3x3, up to 256 threads per plane: register allocation held to six wavefronts per SIMD, which
// the single LDS tile allows; no spills, 0.5 us on the 56x56 plane.  3x3 without BN1 on 1024
// threads per plane: held to 64 registers so that two of these 16-wavefront workgroups share a
// CU, as the kernel needs no more than 61 when the allocator is asked to be frugal)
template <typename T, int K, int TPP, int NG, bool EXPAND>
__global__ __launch_bounds__(TPP > 256 ? TPP : 256, (K == 3 && TPP <= 256) ? 6 : ((K == 3 && !EXPAND) ? 8 : 1)) void dw4_bwd_kernel(Dw4Args a)
{
    constexpr int P = (K - 1) / 2;
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    constexpr int PPB = BLOCK / TPP;
    constexpr int NV = K * K + 2;
    extern __shared__ float lds[];
    const int H = a.H, W = a.W, WP = a.WP, C = a.C;
    const int tileElems = (H + 2 * P) * WP;
    const int lt = threadIdx.x % TPP;
    // Only dd lives in LDS.  The filter gradient dW[u][v] = sum_p dd[p] * a1[p + (u,v) - P] is
    // summed over q = p + (u,v) - P instead: sum_q a1[q] * dd[q - (u,v) + P], which pairs each
    // thread's own a1 values (registers) with exactly the dd window elements the input gradient
    // reads anyway; the zero border of the dd tile supplies the out-of-plane terms.  (An a1 tile
    // would double the LDS footprint and the window reads.)
    float *ddt = lds + (threadIdx.x / TPP) * tileElems;
    float *red = lds + PPB * tileElems;
    size_t plane;
    int n, c;
    const bool active = plane_of<TPP>(a, plane, n, c);

    float wt[K * K];
    float rawk[NG][4], sgk[NG][4]; // e (and sigmoid(y1) with an expansion) of the runs this thread staged
    float mean1 = 0.f, rstd1 = 0.f, scale1 = 1.f, shift1 = 0.f;
    if (active) {
#pragma unroll
        for (int t = 0; t < K * K; ++t)
            wt[t] = ld<T>((const T *)a.w, (size_t)c * K * K + t);
        if (EXPAND) {
            scale1 = a.bn1[c];
            shift1 = a.bn1[C + c];
            mean1 = a.bn1[2 * C + c];
            rstd1 = a.bn1[3 * C + c];
        }
        const float scale2 = a.bn2[c], shift2 = a.bn2[C + c];
        const float c0 = a.coef2[c], c1 = a.coef2[C + c], c2 = a.coef2[2 * C + c];
        const float gate = a.g[plane], dzs = a.dzs[plane];
        zero_border<P, TPP>(ddt, H, W, WP, lt);
        const size_t base = plane * (size_t)H * W;
        float evA[NG][4], GvA[NG][4], dvA[NG][4]; // all loads first (see the forward kernel)
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int gidx = lt + TPP * i;
            const size_t at = base + 4 * (size_t)(gidx < a.groups ? gidx : 0);
            gload4<T>((const T *)a.e, at, evA[i]);
            gload4<T>((const T *)a.G, at, GvA[i]);
            gload4<T>((const T *)a.d, at, dvA[i]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int gidx = lt + TPP * i;
            if (gidx < a.groups) {
                const int h = (int)fdiv((uint32_t)gidx, a.divW4);
                const int w = 4 * (gidx - h * (W >> 2));
                float ddv[4];
                const float(&ev)[4] = evA[i];
                const float(&Gv)[4] = GvA[i];
                const float(&dv)[4] = dvA[i];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    rawk[i][r] = ev[r];
                    if (EXPAND)
                        sgk[i][r] = act_aux(fmaf(ev[r], scale1, shift1));
                    const float y2 = fmaf(dv[r], scale2, shift2);
                    const float s2 = act_aux(y2);
                    const float grad2 = act_grad(y2, s2);
                    const float dy2 = fmaf(Gv[r], gate, dzs) * grad2;
                    ddv[r] = fmaf(c0, dy2, fmaf(c1, dv[r], c2));
                }
                float4v u4 = {ddv[0], ddv[1], ddv[2], ddv[3]};
                *reinterpret_cast<float4v *>(ddt + (h + P) * WP + 4 + w) = u4;
            }
        }
    }
    __syncthreads();

    float acc[NV];
#pragma unroll
    for (int t = 0; t < NV; ++t)
        acc[t] = 0.f;
    if (active) {
        const size_t base = plane * (size_t)H * W;
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int gidx = lt + TPP * i;
            if (gidx < a.groups) {
                const int h = (int)fdiv((uint32_t)gidx, a.divW4);
                const int w = 4 * (gidx - h * (W >> 2));
                float da[4] = {0.f, 0.f, 0.f, 0.f};
                // this thread's a1 values (the depthwise conv's input at its own four pixels)
                float a1c[4], y1[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    y1[r] = fmaf(rawk[i][r], scale1, shift1);
                    a1c[r] = EXPAND ? act_val(y1[r], sgk[i][r]) : rawk[i][r];
                }
                // input gradient  da[r]     = sum_{u,v} wt[u][v] * ddwin[K-1-u][r+K-1-v]
                // filter gradient acc[u][v] += sum_r   a1c[r]   * ddwin[K-1-u][r+K-1-v]
#pragma unroll
                for (int rr = 0; rr < K; ++rr) {
                    float row[K + 3];
                    read_window_row<K>(ddt, h + rr, WP, w, row);
                    const int u = K - 1 - rr;
#pragma unroll
                    for (int v = 0; v < K; ++v)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            da[r] = fmaf(wt[u * K + v], row[r + K - 1 - v], da[r]);
                            acc[u * K + v] = fmaf(a1c[r], row[r + K - 1 - v], acc[u * K + v]);
                        }
                }
                float o[4];
                if (EXPAND) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float raw = rawk[i][r], sg = sgk[i][r];
                        const float y = y1[r];
                        o[r] = da[r] * act_grad(y, sg);
                        const float sv = as_stored<T>(o[r]);
                        acc[K * K] += sv;
                        acc[K * K + 1] = fmaf(sv, (raw - mean1) * rstd1, acc[K * K + 1]);
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[r] = da[r];
                    if (a.res) {
                        float rv[4];
                        gload4<T>((const T *)a.res, base + 4 * (size_t)gidx, rv);
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            o[r] += rv[r];
                    }
                }
                gstore4<T>((T *)a.dy1_out, base + 4 * (size_t)gidx, o);
            }
        }
    }
    group_sum<NV, TPP>(acc, red);
    if (active && lt == 0) {
        float *dst = a.pdw + ((size_t)c * a.N + n) * (K * K);
#pragma unroll
        for (int t = 0; t < K * K; ++t)
            dst[t] = acc[t];
        if (EXPAND) {
            a.psb[(size_t)c * a.N + n] = acc[K * K];
            a.psr[(size_t)c * a.N + n] = acc[K * K + 1];
        }
    }
}

// ---- dispatch ---------------------------------------------------------------------------------

// Thread-group shape for a plane of `groups` float4 runs: (threads per plane, runs per thread).
static bool dw4_shape(int groups, int *tpp, int *ng)
{
    if (groups <= 64) {
        *tpp = 64;
        *ng = 1;
    } else if (groups <= 256) {
        *tpp = 64;
        *ng = 4;
    } else if (groups <= 1024) {
        *tpp = 256;
        *ng = 4;
    } else if (groups <= 4096) {
        *tpp = 1024;
        *ng = 4;
    } else {
        return false;
    }
    return true;
}

bool dw4_supported(const DwShape &s)
{
    int tpp, ng;
    return s.s == 1 && (s.W % 4) == 0 && (s.k == 3 || s.k == 5) && s.Ho == s.H && s.Wo == s.W &&
           dw4_shape(s.H * s.W / 4, &tpp, &ng);
}

static size_t dw4_lds(const DwShape &s, int tiles, int nv)
{
    int tpp, ng;
    dw4_shape(s.H * s.W / 4, &tpp, &ng);
    const int block = tpp > 256 ? tpp : 256;
    const int ppb = block / tpp;
    const int p = (s.k - 1) / 2;
    return sizeof(float) * ((size_t)ppb * tiles * (s.H + 2 * p) * (s.W + 8) + (size_t)(block / 64) * nv);
}

static Dw4Args dw4_args(const DwShape &s)
{
    Dw4Args a = {};
    a.N = s.N;
    a.C = s.C;
    a.H = s.H;
    a.W = s.W;
    a.WP = s.W + 8;
    a.groups = s.H * s.W / 4;
    a.divC = make_div((uint32_t)s.C);
    a.divW4 = make_div((uint32_t)(s.W / 4));
    return a;
}

template <typename KERN>
static hipError_t dw4_launch(KERN kern, const Dw4Args &a, int block, int ppb, size_t lds,
                             hipStream_t st)
{
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds);
    if (e != hipSuccess)
        return e;
    const size_t planes = (size_t)a.N * a.C;
    const unsigned grid = (unsigned)((planes + ppb - 1) / ppb);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(block), lds, st, a);
    return hipGetLastError();
}

#define MBK_DW4_SHAPES(KERNEL, T, K, EXP)                                                         \
    if (tpp == 64 && ng == 1)                                                                     \
        return dw4_launch(KERNEL<T, K, 64, 1, EXP>, a, 256, 4, lds, st);                          \
    if (tpp == 64 && ng == 4)                                                                     \
        return dw4_launch(KERNEL<T, K, 64, 4, EXP>, a, 256, 4, lds, st);                          \
    if (tpp == 256)                                                                               \
        return dw4_launch(KERNEL<T, K, 256, 4, EXP>, a, 256, 1, lds, st);                         \
    return dw4_launch(KERNEL<T, K, 1024, 4, EXP>, a, 1024, 1, lds, st);

template <typename T, int K, bool EXP>
static hipError_t dw4_fwd_go(const Dw4Args &a, int tpp, int ng, size_t lds, hipStream_t st)
{
    MBK_DW4_SHAPES(dw4_fwd_kernel, T, K, EXP)
}
template <typename T, int K, bool EXP>
static hipError_t dw4_bwd_go(const Dw4Args &a, int tpp, int ng, size_t lds, hipStream_t st)
{
    MBK_DW4_SHAPES(dw4_bwd_kernel, T, K, EXP)
}

hipError_t launch_dw4_fwd(bool bf16, const DwShape &s, const void *e, const float *bn1,
                          const void *w_dw, void *d, float *psum, float *psq, const BnFin *fin,
                          hipStream_t st)
{
    Dw4Args a = dw4_args(s);
    if (fin)
        a.fin = *fin;
    a.e = e;
    a.bn1 = bn1;
    a.w = w_dw;
    a.d = d;
    a.psum = psum;
    a.psq = psq;
    int tpp, ng;
    dw4_shape(a.groups, &tpp, &ng);
    const size_t lds = dw4_lds(s, 1, 2);
    const bool ex = bn1 != nullptr;
    // 56x56-class planes (a workgroup of 256 threads per plane): two images of a channel per
    // workgroup where that still leaves eight workgroups per CU (config 1: 26.4 us against 29.5
    // for the step; four images 26.6, eight 29.5)
    a.PL = (tpp == 256 && ng == 4 && (long long)a.C * ((a.N + 1) / 2) >= 2048) ? 2 : 1;
    if (a.PL > 1) {
        const unsigned grid = (unsigned)(a.C * ((a.N + a.PL - 1) / a.PL));
#define MBK_MULTI(T, K, EXP)                                                                      \
    {                                                                                             \
        auto kern = dw4_fwd_multi_kernel<T, K, 4, EXP>;                                           \
        hipError_t e_ = hipFuncSetAttribute((const void *)kern,                                   \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e_ != hipSuccess)                                                                     \
            return e_;                                                                            \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, a);                              \
        return hipGetLastError();                                                                 \
    }
#define MBK_MULTI_K(T, EXP)                                                                       \
    {                                                                                             \
        if (s.k == 3)                                                                             \
            MBK_MULTI(T, 3, EXP)                                                                  \
        MBK_MULTI(T, 5, EXP)                                                                      \
    }
        if (bf16) {
            if (ex)
                MBK_MULTI_K(bf16_t, true)
            MBK_MULTI_K(bf16_t, false)
        }
        if (ex)
            MBK_MULTI_K(float, true)
        MBK_MULTI_K(float, false)
#undef MBK_MULTI_K
#undef MBK_MULTI
    }
#define MBK_GO(T, K)                                                                              \
    return ex ? dw4_fwd_go<T, K, true>(a, tpp, ng, lds, st) : dw4_fwd_go<T, K, false>(a, tpp, ng, lds, st);
    if (bf16) {
        if (s.k == 3)
            MBK_GO(bf16_t, 3)
        MBK_GO(bf16_t, 5)
    }
    if (s.k == 3)
        MBK_GO(float, 3)
    MBK_GO(float, 5)
#undef MBK_GO
}

hipError_t launch_dw4_bwd(bool bf16, const DwBwdArgs &h, hipStream_t st)
{
    Dw4Args a = dw4_args(h.s);
    a.e = h.e;
    a.bn1 = h.bn1;
    a.w = h.w_dw;
    a.d = const_cast<void *>(h.d); // read-only in backward
    a.G = h.G;
    a.g = h.g;
    a.dzs = h.dzs;
    a.bn2 = h.bn2;
    a.coef2 = h.coef2;
    a.dy1_out = h.dy1_out;
    a.res = h.res;
    a.pdw = h.pdw;
    a.psb = h.psb;
    a.psr = h.psr;
    int tpp, ng;
    dw4_shape(a.groups, &tpp, &ng);
    const size_t lds = dw4_lds(h.s, 1, h.s.k * h.s.k + 2);
    const bool ex = h.bn1 != nullptr;
#define MBK_GO(T, K)                                                                              \
    return ex ? dw4_bwd_go<T, K, true>(a, tpp, ng, lds, st) : dw4_bwd_go<T, K, false>(a, tpp, ng, lds, st);
    if (bf16) {
        if (h.s.k == 3)
            MBK_GO(bf16_t, 3)
        MBK_GO(bf16_t, 5)
    }
    if (h.s.k == 3)
        MBK_GO(float, 3)
    MBK_GO(float, 5)
#undef MBK_GO
}

} // namespace mbk
