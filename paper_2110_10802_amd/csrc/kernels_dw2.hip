// Vectorised depthwise chain for stride 2 (the down-sampling blocks), even input height and
// width (16-byte global accesses when the width is a multiple of 4, else masked pairs).  Same plan as the stride-1 kernels in kernels_dw4.hip: the whole input plane is staged
// into LDS with a zero border, BN + Swish evaluated once per input element, every thread keeps
// the runs of four pixels it staged; the output plane is a quarter of the input, so a thread
// owns up to four input runs and one output run.
//   forward      an output run (4 columns) reads, per filter row, the K+6 consecutive input
//                columns it touches as two 16-byte LDS reads plus the edge values;
//   input grad   an input pixel only meets the taps u = (h+P) mod 2, v = (x+P) mod 2 (section
//                "Backpropagation and Data Movement": the transposed stencil).  Inside a run
//                the column parity is fixed by the position and a thread's runs alternate
//                between even and odd rows, so both the column and the row taps are
//                compile-time;
//   filter grad  summed over the input position: the thread's own a1 values times the dd
//                elements the input gradient reads (no a1 tile in the backward kernel).
// Partial sums per (channel, image); no atomics.
#include "mbconv_dev.h"
#include "mbconv_launch.h"

namespace mbk {

typedef float float4v __attribute__((ext_vector_type(4)));

struct Dw2Args {
    int N, C, H, W, Ho, Wo;
    int WP;      // a1 tile pitch  = 8*Wo4 + 8 (>= W + 8), interior at column 4
    int WQ;      // dd tile pitch  = 4*Wo4 + 8, interior at column 4
    int Wo4;     // output runs per row = ceil(Wo/4)
    int W4;      // input runs per row = ceil(W/4)
    int inRuns;  // H*W4
    int outRuns; // Ho*Wo4
    FastDiv divC, divW4, divWo4;
    const void *e;
    const float *bn1;
    const void *w;
    void *d;
    float *psum, *psq;
    const void *G;
    const float *g, *dzs, *bn2, *coef2;
    void *dy1_out;
    float *pdw, *psb, *psr;
};

constexpr int kDw2PB = 2; // zero rows above and below the dd tile

template <typename T>
__device__ __forceinline__ void d2_load4(const T *p, size_t i, float (&v)[4]);
template <>
__device__ __forceinline__ void d2_load4<float>(const float *p, size_t i, float (&v)[4])
{
    const float4v t = *reinterpret_cast<const float4v *>(p + i);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
}
template <>
__device__ __forceinline__ void d2_load4<bf16_t>(const bf16_t *p, size_t i, float (&v)[4])
{
    const uint2 t = *reinterpret_cast<const uint2 *>(&p[i]);
    v[0] = bf16_bits_to_float(t.x & 0xffffu);
    v[1] = bf16_bits_to_float(t.x >> 16);
    v[2] = bf16_bits_to_float(t.y & 0xffffu);
    v[3] = bf16_bits_to_float(t.y >> 16);
}
template <typename T>
__device__ __forceinline__ void d2_store4(T *p, size_t i, const float (&v)[4]);
template <>
__device__ __forceinline__ void d2_store4<float>(float *p, size_t i, const float (&v)[4])
{
    float4v t = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<float4v *>(p + i) = t;
}
template <>
__device__ __forceinline__ void d2_store4<bf16_t>(bf16_t *p, size_t i, const float (&v)[4])
{
    uint2 t;
    t.x = bf16_pack2(v[0], v[1]);
    t.y = bf16_pack2(v[2], v[3]);
    *reinterpret_cast<uint2 *>(&p[i]) = t;
}

// An input run of four columns x0..x0+3; GVI = 4: the width is a multiple of 4; GVI = 2: it is
// even, so the run is two pairs of which the second may lie past the end.
template <typename T, int GVI>
__device__ __forceinline__ void d2_in_load(const T *p, size_t idx, int x0, int W, float (&v)[4])
{
    if (GVI == 4) {
        d2_load4<T>(p, idx, v);
    } else {
        v[0] = ld<T>(p, idx);
        v[1] = ld<T>(p, idx + 1);
        const bool hi = x0 + 2 < W;
        v[2] = hi ? ld<T>(p, idx + 2) : 0.f;
        v[3] = hi ? ld<T>(p, idx + 3) : 0.f;
    }
}
template <typename T, int GVI>
__device__ __forceinline__ void d2_in_store(T *p, size_t idx, int x0, int W, const float (&v)[4])
{
    if (GVI == 4) {
        d2_store4<T>(p, idx, v);
    } else {
        st<T>(p, idx, v[0]);
        st<T>(p, idx + 1, v[1]);
        if (x0 + 2 < W) {
            st<T>(p, idx + 2, v[2]);
            st<T>(p, idx + 3, v[3]);
        }
    }
}

// An output run of four columns j0..j0+3 (those >= Wo masked); Wo is even, so pairs are whole.
template <typename T, int GVO>
__device__ __forceinline__ void d2_out_load(const T *p, size_t idx, int j0, int Wo, float (&v)[4])
{
    if (GVO == 4) {
        d2_load4<T>(p, idx, v);
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = j0 + r < Wo ? ld<T>(p, idx + r) : 0.f;
    }
}
template <typename T, int GVO>
__device__ __forceinline__ void d2_out_store(T *p, size_t idx, int j0, int Wo, const float (&v)[4])
{
    if (GVO == 4) {
        d2_store4<T>(p, idx, v);
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (j0 + r < Wo)
                st<T>(p, idx + r, v[r]);
    }
}

template <int TPP>
__device__ __forceinline__ bool d2_plane(const Dw2Args &a, size_t &plane, int &n, int &c)
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

// Zero everything of a tile except the W interior columns of its `rows` interior rows
// (top border `top` rows, bottom border `bot` rows, pitch a multiple of 4).
template <int TPP>
__device__ __forceinline__ void d2_zero_border(float *tile, int rows, int top, int bot, int W,
                                               int pitch, int lt)
{
    const float4v z = {0.f, 0.f, 0.f, 0.f};
    const int p4 = pitch >> 2, w4 = W >> 2; // interior quads: columns 4 .. 4+W-1 (W % 4 == 0)
    for (int i = lt; i < (top + bot) * p4; i += TPP) {
        const int rr = i / p4, cc = i - rr * p4;
        const int r = rr < top ? rr : rows + rr;
        *reinterpret_cast<float4v *>(tile + r * pitch + 4 * cc) = z;
    }
    const int side = p4 - w4; // pad quads per interior row: one on the left, the rest right
    for (int i = lt; i < rows * side; i += TPP) {
        const int rr = i / side, cc = i - rr * side;
        const int col = cc == 0 ? 0 : 4 + W + 4 * (cc - 1);
        *reinterpret_cast<float4v *>(tile + (top + rr) * pitch + col) = z;
    }
}

// The K+6 input columns 2*j0-P .. 2*j0+5+P+... of tile row `row` that an output run touches.
template <int K>
__device__ __forceinline__ void d2_window(const float *tile, int row, int WP, int j0, float (&o)[K + 6])
{
    constexpr int P = (K - 1) / 2;
    const float *p = tile + row * WP + 4 + 2 * j0;
    const float4v m0 = *reinterpret_cast<const float4v *>(p);
    const float4v m1 = *reinterpret_cast<const float4v *>(p + 4);
    if (P == 1) {
        o[0] = p[-1];
    } else {
        const float2 l = *reinterpret_cast<const float2 *>(p - 2);
        o[0] = l.x;
        o[1] = l.y;
        o[K + 5] = p[8];
    }
    o[P] = m0.x;
    o[P + 1] = m0.y;
    o[P + 2] = m0.z;
    o[P + 3] = m0.w;
    o[P + 4] = m1.x;
    o[P + 5] = m1.y;
    o[P + 6] = m1.z;
    o[P + 7] = m1.w;
}

// ---- forward ---------------------------------------------------------------------------------
template <typename T, int K, int TPP, bool EXPAND, int GVO, int GVI>
__global__ __launch_bounds__(TPP > 256 ? TPP : 256) void dw2_fwd_kernel(Dw2Args a)
{
    constexpr int P = (K - 1) / 2, NGI = 4;
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    constexpr int PPB = BLOCK / TPP;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int H = a.H, W = a.W, WP = a.WP;
    const int tileElems = (H + 2 * P) * WP;
    const int lt = threadIdx.x % TPP;
    float *tile = lds + (threadIdx.x / TPP) * tileElems;
    float *red = lds + PPB * tileElems;
    size_t plane;
    int n, c;
    const bool active = d2_plane<TPP>(a, plane, n, c);

    float wt[K * K];
    if (active) {
        float scale = 1.f, shift = 0.f;
        if (EXPAND) {
            scale = a.bn1[c];
            shift = a.bn1[a.C + c];
        }
#pragma unroll
        for (int t = 0; t < K * K; ++t)
            wt[t] = ld<T>((const T *)a.w, (size_t)c * K * K + t);
        d2_zero_border<TPP>(tile, H, P, P, 4 * a.W4, WP, lt);
        const size_t base = plane * (size_t)H * W;
        float ev[NGI][4]; // all loads first, then the arithmetic (one memory round trip)
#pragma unroll
        for (int i = 0; i < NGI; ++i) {
            const int gidx = lt + TPP * i < a.inRuns ? lt + TPP * i : 0;
            const int h = (int)fdiv((uint32_t)gidx, a.divW4);
            const int x0 = 4 * (gidx - h * a.W4);
            d2_in_load<T, GVI>((const T *)a.e, base + (size_t)h * W + x0, x0, W, ev[i]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NGI; ++i) {
            const int gidx = lt + TPP * i;
            if (gidx < a.inRuns) {
                const int h = (int)fdiv((uint32_t)gidx, a.divW4);
                const int x0 = 4 * (gidx - h * a.W4);
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    // straight-line code for all four elements (a branch per element would run
                    // the four exp/rcp chains one after the other); whole runs need no mask
                    const float t = EXPAND ? actf(fmaf(ev[i][r], scale, shift)) : ev[i][r];
                    v[r] = GVI == 4 ? t : and_mask(t, x0 + r < W ? 0xffffffffu : 0u);
                }
                *reinterpret_cast<float4v *>(tile + (h + P) * WP + 4 + x0) =
                    float4v{v[0], v[1], v[2], v[3]};
            }
        }
    }
    __syncthreads();
    float acc2[2] = {0.f, 0.f};
    if (active && lt < a.outRuns) {
        const int i = (int)fdiv((uint32_t)lt, a.divWo4);
        const int j0 = 4 * (lt - i * a.Wo4);
        float o[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < K; ++u) {
            float win[K + 6];
            d2_window<K>(tile, 2 * i + u, WP, j0, win);
#pragma unroll
            for (int v = 0; v < K; ++v)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    o[r] = fmaf(wt[u * K + v], win[2 * r + v], o[r]);
        }
        d2_out_store<T, GVO>((T *)a.d, plane * (size_t)a.Ho * a.Wo + (size_t)i * a.Wo + j0, j0, a.Wo, o);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (GVO == 4 || j0 + r < a.Wo) {
                const float sv = as_stored<T>(o[r]);
                acc2[0] += sv;
                acc2[1] = fmaf(sv, sv, acc2[1]);
            }
        }
    }
    group_sum<2, TPP>(acc2, red);
    if (active && lt == 0) {
        a.psum[(size_t)c * a.N + n] = acc2[0];
        a.psq[(size_t)c * a.N + n] = acc2[1];
    }
}

// ---- backward (the fused kernel described in mbconv_launch.h, DwBwdArgs) -----------------------
// Backward.  Only dd (a quarter of the input plane) lives in LDS.  The filter gradient
// dW[u][v] = sum_{i,j} dd[i][j] * a1[2i+u-P][2j+v-P] is summed over the input position instead:
// an input pixel (h, x) meets exactly the taps and the dd elements its input gradient meets
// (u = (h+P) mod 2 + 2t, v = (x+P) mod 2 + 2s), so each thread multiplies its own a1 values
// (registers) by the dd elements it reads anyway and no a1 tile exists.  A thread's four input
// runs alternate between even and odd rows (run i lies in row 2*rp + (i & 1)), which makes the
// row parity, like the column parity inside a run, a compile-time property: the filter rows
// and the accumulators a run touches are fixed, nothing is selected at run time.
// (3x3 with 1024 threads per plane: register allocation held to 64, i.e. eight wavefronts per
// SIMD, so that two of these 16-wavefront workgroups share a CU: 65 registers allowed one.
// 112x112 planes, 64 x 96 of them: 213 -> 164 us.)
template <typename T, int K, int TPP, bool EXPAND, int GVO, int GVI>
__global__ __launch_bounds__(TPP > 256 ? TPP : 256, (TPP > 256 && K == 3) ? 8 : 1) void dw2_bwd_kernel(Dw2Args a)
{
    constexpr int P = (K - 1) / 2, NGI = 4, PB = kDw2PB;
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    constexpr int PPB = BLOCK / TPP;
    constexpr int NV = K * K + 2;
    constexpr int NT = (K + 1) / 2; // row taps of the input gradient
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int H = a.H, W = a.W, Ho = a.Ho, Wo = a.Wo, WQ = a.WQ, C = a.C;
    const int ddElems = (Ho + 2 * PB) * WQ;
    const int lt = threadIdx.x % TPP;
    float *ddt = lds + (threadIdx.x / TPP) * ddElems;
    float *red = lds + PPB * ddElems;
    size_t plane;
    int n, c;
    const bool active = d2_plane<TPP>(a, plane, n, c);

    float wt[K * K];
    float rawk[NGI][4], sgk[NGI][4]; // e and sigmoid(y1) of the input runs this thread staged
    float ddv[4] = {0.f, 0.f, 0.f, 0.f}; // dd of the output run this thread staged
    float mean1 = 0.f, rstd1 = 0.f, scale1 = 1.f, shift1 = 0.f;
    const bool has_out = lt < a.outRuns;
    const int oi = has_out ? (int)fdiv((uint32_t)lt, a.divWo4) : 0;
    const int oj0 = has_out ? 4 * (lt - oi * a.Wo4) : 0;
    // input run i of this thread: slot lt + TPP*(i/2) among the runs of the rows of parity i & 1
    // (H is even: each parity class holds inRuns/2 runs)
    const int halfRuns = a.inRuns >> 1;
    int rh[NGI], rx[NGI];
    bool rok[NGI];
#pragma unroll
    for (int i = 0; i < NGI; ++i) {
        const int slot = lt + TPP * (i >> 1);
        rok[i] = slot < halfRuns;
        const int sl = rok[i] ? slot : 0;
        const int rp = (int)fdiv((uint32_t)sl, a.divW4);
        rh[i] = 2 * rp + (i & 1);
        rx[i] = 4 * (sl - rp * a.W4);
    }
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
        // the dd tile is small: clear all of it, the interior is written after the barrier
        for (int i = lt; i < ddElems / 4; i += TPP)
            reinterpret_cast<float4v *>(ddt)[i] = float4v{0.f, 0.f, 0.f, 0.f};
        const size_t ebase = plane * (size_t)H * W;
        const size_t dbase = plane * (size_t)Ho * Wo + (size_t)oi * Wo + oj0;
        float Gv[4], dv[4]; // all loads first (one memory round trip)
#pragma unroll
        for (int i = 0; i < NGI; ++i)
            d2_in_load<T, GVI>((const T *)a.e, ebase + (size_t)rh[i] * W + rx[i], rx[i], W, rawk[i]);
        d2_out_load<T, GVO>((const T *)a.G, dbase, has_out ? oj0 : Wo, Wo, Gv);
        d2_out_load<T, GVO>((const T *)a.d, dbase, has_out ? oj0 : Wo, Wo, dv);
        __builtin_amdgcn_sched_barrier(0);
        if (EXPAND) {
#pragma unroll
            for (int i = 0; i < NGI; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    sgk[i][r] = act_aux(fmaf(rawk[i][r], scale1, shift1));
        }
        if (has_out) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float y2 = fmaf(dv[r], scale2, shift2);
                const float s2 = act_aux(y2);
                const float grad2 = act_grad(y2, s2);
                const float dy2 = fmaf(Gv[r], gate, dzs) * grad2;
                ddv[r] = (GVO == 4 || oj0 + r < Wo) ? fmaf(c0, dy2, fmaf(c1, dv[r], c2)) : 0.f;
            }
        }
    }
    __syncthreads(); // the dd tile has been cleared
    if (active && has_out)
        *reinterpret_cast<float4v *>(ddt + (oi + PB) * WQ + 4 + oj0) =
            float4v{ddv[0], ddv[1], ddv[2], ddv[3]};
    __syncthreads();

    float acc[NV];
#pragma unroll
    for (int t = 0; t < NV; ++t)
        acc[t] = 0.f;
    if (active) {
        const size_t ebase = plane * (size_t)H * W;
#pragma unroll
        for (int i = 0; i < NGI; ++i) {
            if (rok[i]) {
                const int h = rh[i], x0 = rx[i];
                const int ph = ((i & 1) + P) & 1; // (h + P) mod 2, known at compile time after unrolling
                const int hh = (h + P - ph) >> 1; // row tap t reads dd row hh - t with filter row ph + 2t
                const int cq = x0 >> 1;
                // this thread's a1 values at the run (zero in the pad columns of a ragged row)
                float a1c[4], y1[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    y1[r] = fmaf(rawk[i][r], scale1, shift1);
                    const float v = EXPAND ? act_val(y1[r], sgk[i][r]) : rawk[i][r];
                    a1c[r] = (GVI == 4 || x0 + r < W) ? v : 0.f;
                }
                float da[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int u = ph + 2 * t;
                    if (u < K) { // (the odd parity has one row tap fewer)
                        const float *wr = &wt[u * K];
                        float *ar = &acc[u * K];
                        const float *q = ddt + (hh - t + PB) * WQ + 4 + cq;
                        const float2 qm = *reinterpret_cast<const float2 *>(q); // columns cq, cq+1
                        const float q2 = q[2];
                        if (K == 3) {
                            // x even meets v = 1 (column x/2); x odd meets v = 0 ((x+1)/2) and v = 2 ((x-1)/2)
                            da[0] = fmaf(wr[1], qm.x, da[0]);
                            da[1] = fmaf(wr[0], qm.y, fmaf(wr[2], qm.x, da[1]));
                            da[2] = fmaf(wr[1], qm.y, da[2]);
                            da[3] = fmaf(wr[0], q2, fmaf(wr[2], qm.y, da[3]));
                            ar[1] = fmaf(a1c[0], qm.x, fmaf(a1c[2], qm.y, ar[1]));
                            ar[0] = fmaf(a1c[1], qm.y, fmaf(a1c[3], q2, ar[0]));
                            ar[2] = fmaf(a1c[1], qm.x, fmaf(a1c[3], qm.y, ar[2]));
                        } else {
                            // x even meets v = 0, 2, 4 (columns x/2+1, x/2, x/2-1); x odd v = 1, 3
                            const float qn = q[-1];
                            da[0] = fmaf(wr[0], qm.y, fmaf(wr[2], qm.x, fmaf(wr[4], qn, da[0])));
                            da[1] = fmaf(wr[1], qm.y, fmaf(wr[3], qm.x, da[1]));
                            da[2] = fmaf(wr[0], q2, fmaf(wr[2], qm.y, fmaf(wr[4], qm.x, da[2])));
                            da[3] = fmaf(wr[1], q2, fmaf(wr[3], qm.y, da[3]));
                            ar[0] = fmaf(a1c[0], qm.y, fmaf(a1c[2], q2, ar[0]));
                            ar[2] = fmaf(a1c[0], qm.x, fmaf(a1c[2], qm.y, ar[2]));
                            ar[4] = fmaf(a1c[0], qn, fmaf(a1c[2], qm.x, ar[4]));
                            ar[1] = fmaf(a1c[1], qm.y, fmaf(a1c[3], q2, ar[1]));
                            ar[3] = fmaf(a1c[1], qm.x, fmaf(a1c[3], qm.y, ar[3]));
                        }
                    }
                }
                float o[4];
                if (EXPAND) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float raw = rawk[i][r], sg = sgk[i][r];
                        o[r] = da[r] * act_grad(y1[r], sg);
                        if (GVI == 4 || x0 + r < W) {
                            const float sv = as_stored<T>(o[r]);
                            acc[K * K] += sv;
                            acc[K * K + 1] = fmaf(sv, (raw - mean1) * rstd1, acc[K * K + 1]);
                        }
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[r] = da[r];
                }
                d2_in_store<T, GVI>((T *)a.dy1_out, ebase + (size_t)h * W + x0, x0, W, o);
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

// ---- host side ---------------------------------------------------------------------------------

static bool dw2_shape(const DwShape &s, int *tpp)
{
    const int inRuns = s.H * ((s.W + 3) / 4), outRuns = s.Ho * ((s.Wo + 3) / 4);
    // (16 threads per plane: the 14x14 -> 7x7 planes of the late stages, four planes per
    // wavefront with nearly every lane busy; with 64 threads 28 of them had input runs)
    for (int t : {16, 64, 256, 1024}) {
        if (inRuns <= 4 * t && outRuns <= t) {
            *tpp = t;
            return true;
        }
    }
    return false;
}

bool dw2_supported(const DwShape &s)
{
    int tpp;
    return s.s == 2 && (s.k == 3 || s.k == 5) && s.W % 2 == 0 && s.H % 2 == 0 && s.Ho == s.H / 2 &&
           s.Wo == s.W / 2 && dw2_shape(s, &tpp);
}

static Dw2Args dw2_args(const DwShape &s)
{
    Dw2Args a = {};
    a.N = s.N;
    a.C = s.C;
    a.H = s.H;
    a.W = s.W;
    a.Ho = s.Ho;
    a.Wo = s.Wo;
    a.Wo4 = (s.Wo + 3) / 4;
    a.WP = 8 * a.Wo4 + 8;
    a.WQ = 4 * a.Wo4 + 8;
    a.W4 = (s.W + 3) / 4;
    a.inRuns = s.H * a.W4;
    a.outRuns = s.Ho * a.Wo4;
    a.divC = make_div((uint32_t)s.C);
    a.divW4 = make_div((uint32_t)a.W4);
    a.divWo4 = make_div((uint32_t)a.Wo4);
    return a;
}

static size_t dw2_lds(const Dw2Args &a, int k, int tpp, bool bwd)
{
    const int p = (k - 1) / 2;
    const int block = tpp > 256 ? tpp : 256, ppb = block / tpp;
    // forward: the a1 tile; backward: the dd tile only
    const size_t per = bwd ? (size_t)(a.Ho + 2 * kDw2PB) * a.WQ : (size_t)(a.H + 2 * p) * a.WP;
    const int nv = bwd ? k * k + 2 : 2;
    return sizeof(float) * (ppb * per + (size_t)(block / 64) * nv);
}

template <typename KERN>
static hipError_t dw2_launch(KERN kern, const Dw2Args &a, int tpp, size_t lds, hipStream_t st)
{
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds);
    if (e != hipSuccess)
        return e;
    const int block = tpp > 256 ? tpp : 256, ppb = block / tpp;
    const size_t planes = (size_t)a.N * a.C;
    hipLaunchKernelGGL(kern, dim3((unsigned)((planes + ppb - 1) / ppb)), dim3(block), lds, st, a);
    return hipGetLastError();
}

#define MBK_DW2_TPP(KERNEL, T, K, EXP, GVO)                                                       \
    {                                                                                             \
        if (s.W % 4 != 0) /* ragged rows: only the small planes of the late stages */             \
            return tpp == 16   ? dw2_launch(KERNEL<T, K, 16, EXP, 1, 2>, a, tpp, lds, st)         \
                   : tpp == 64 ? dw2_launch(KERNEL<T, K, 64, EXP, 1, 2>, a, tpp, lds, st)         \
                               : dw2_launch(KERNEL<T, K, 256, EXP, 1, 2>, a, tpp, lds, st);       \
        if (tpp == 16)                                                                            \
            return dw2_launch(KERNEL<T, K, 16, EXP, GVO, 4>, a, tpp, lds, st);                    \
        if (tpp == 64)                                                                            \
            return dw2_launch(KERNEL<T, K, 64, EXP, GVO, 4>, a, tpp, lds, st);                    \
        if (tpp == 256)                                                                           \
            return dw2_launch(KERNEL<T, K, 256, EXP, GVO, 4>, a, tpp, lds, st);                   \
        return dw2_launch(KERNEL<T, K, 1024, EXP, GVO, 4>, a, tpp, lds, st);                      \
    }
#define MBK_DW2_GO(KERNEL, T, K)                                                                  \
    {                                                                                             \
        if (ex && gvo == 4)                                                                       \
            MBK_DW2_TPP(KERNEL, T, K, true, 4)                                                    \
        if (ex)                                                                                   \
            MBK_DW2_TPP(KERNEL, T, K, true, 1)                                                    \
        if (gvo == 4)                                                                             \
            MBK_DW2_TPP(KERNEL, T, K, false, 4)                                                   \
        MBK_DW2_TPP(KERNEL, T, K, false, 1)                                                       \
    }

hipError_t launch_dw2_fwd(bool bf16, const DwShape &s, const void *e, const float *bn1,
                          const void *w_dw, void *d, float *psum, float *psq, hipStream_t st)
{
    Dw2Args a = dw2_args(s);
    a.e = e;
    a.bn1 = bn1;
    a.w = w_dw;
    a.d = d;
    a.psum = psum;
    a.psq = psq;
    int tpp;
    if (!dw2_shape(s, &tpp))
        return hipErrorInvalidValue;
    const size_t lds = dw2_lds(a, s.k, tpp, false);
    const bool ex = bn1 != nullptr;
    const int gvo = s.Wo % 4 == 0 ? 4 : 1;
    if (bf16) {
        if (s.k == 3)
            MBK_DW2_GO(dw2_fwd_kernel, bf16_t, 3)
        MBK_DW2_GO(dw2_fwd_kernel, bf16_t, 5)
    }
    if (s.k == 3)
        MBK_DW2_GO(dw2_fwd_kernel, float, 3)
    MBK_DW2_GO(dw2_fwd_kernel, float, 5)
}

hipError_t launch_dw2_bwd(bool bf16, const DwBwdArgs &h, hipStream_t st)
{
    const DwShape &s = h.s;
    Dw2Args a = dw2_args(s);
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
    a.pdw = h.pdw;
    a.psb = h.psb;
    a.psr = h.psr;
    int tpp;
    if (!dw2_shape(s, &tpp) || h.res)
        return hipErrorInvalidValue;
    const size_t lds = dw2_lds(a, s.k, tpp, true);
    const bool ex = h.bn1 != nullptr;
    const int gvo = s.Wo % 4 == 0 ? 4 : 1;
    if (bf16) {
        if (s.k == 3)
            MBK_DW2_GO(dw2_bwd_kernel, bf16_t, 3)
        MBK_DW2_GO(dw2_bwd_kernel, bf16_t, 5)
    }
    if (s.k == 3)
        MBK_DW2_GO(dw2_bwd_kernel, float, 3)
    MBK_DW2_GO(dw2_bwd_kernel, float, 5)
}
#undef MBK_DW2_GO
#undef MBK_DW2_TPP

} // namespace mbk
