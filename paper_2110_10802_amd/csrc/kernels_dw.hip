// The memory-bound depthwise chain: one (image, channel) plane at a time.
//
// A whole plane (at most 112x112 fp32 = 49 KB) fits in the 160 KB LDS of a gfx950 CU,
// so a group of threads stages the plane once, applying BN + Swish on the way in (each
// activation is evaluated once per input element, not once per filter tap), with the
// zero padding materialised as a border in LDS (the paper's Pad+Conv fusion, section
// "Coarse-Grained Transformations"; MapTiling + LocalStorage, section "Local Data
// Movement Reduction").  The activation a1 = Swish(BN1(e)) therefore never exists in
// HBM: forward reads e and writes d, backward re-derives everything it needs from the
// pre-normalisation tensors (recomputation instead of load/store, section "Guided
// Optimization Case Study: EfficientNet", step "Full fusion and vectorization").
//
// Every reduction (BN partial sums, filter gradients) is a fixed-order tree inside the
// plane's thread group followed by a fixed-order sum over images in a later kernel; no
// atomics anywhere (the same section's "Map fission" step).
#include "mbconv_dev.h"
#include "mbconv_launch.h"
#include "mbconv_bnfin.h"

#include <algorithm>

namespace mbk {

// kernels_dw4.hip: vectorised variants for stride 1 and W % 4 == 0
bool dw4_supported(const DwShape &s);
hipError_t launch_dw4_fwd(bool bf16, const DwShape &s, const void *e, const float *bn1,
                          const void *w_dw, void *d, float *psum, float *psq, const BnFin *fin,
                          hipStream_t st);
hipError_t launch_dw4_bwd(bool bf16, const DwBwdArgs &h, hipStream_t st);
// kernels_dw2.hip
bool dw2_supported(const DwShape &s);
hipError_t launch_dw2_fwd(bool bf16, const DwShape &s, const void *e, const float *bn1,
                          const void *w_dw, void *d, float *psum, float *psq, hipStream_t st);
hipError_t launch_dw2_bwd(bool bf16, const DwBwdArgs &h, hipStream_t st);
// kernels_dwr.hip
bool dwr_supported(const DwShape &s);
int dwr_num_partials(const DwShape &s);
hipError_t launch_dwr_fwd(bool bf16, const DwShape &s, const void *e, const float *bn1,
                          const void *w_dw, void *d, float *psum, float *psq, const BnFin *fin,
                          hipStream_t st);
hipError_t launch_dwr_bwd(bool bf16, const DwBwdArgs &h, hipStream_t st);

int dw_num_partials(const DwShape &s, bool stores_a1)
{
    if (!stores_a1 && !dw4_supported(s) && dwr_supported(s))
        return dwr_num_partials(s);
    return s.N;
}

// Threads per plane: a wavefront for planes up to 16x16, a 256-thread workgroup up to
// 64x64, 1024 threads above.
static int pick_tpp(int plane_elems) { return plane_elems <= 256 ? 64 : plane_elems <= 4096 ? 256 : 1024; }
// The plane reductions and the final elementwise pass give a plane of at most 256 elements to
// 16 lanes (a DPP row): four planes per wavefront share the per-plane overhead (index
// arithmetic, coefficient loads, the reduction), which is most of the work on 14x14 and 7x7 planes.
static int pick_tpp_plane(int plane_elems)
{
    return plane_elems <= 256 ? 16 : plane_elems <= 1024 ? 64 : pick_tpp(plane_elems);
}

struct PlaneId {
    bool active;
    int n, c;
    size_t plane;
};

template <int TPP>
__device__ __forceinline__ PlaneId plane_of_group(int N, int C, FastDiv divC)
{
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    constexpr int PPB = BLOCK / TPP;
    PlaneId p;
    const size_t plane = (size_t)blockIdx.x * PPB + threadIdx.x / TPP;
    p.active = plane < (size_t)N * C;
    p.plane = p.active ? plane : 0;
    p.n = (int)fdiv((uint32_t)p.plane, divC);
    p.c = (int)(p.plane - (size_t)p.n * C);
    return p;
}

// ---- forward: d = depthwise(swish(bn1(e))) + BN2 partial statistics ------------------------

struct DwFwdDev {
    DwShape s;
    FastDiv divC, divWp, divWo;
    const void *e;
    const float *bn1;
    const void *w;
    void *d;
    float *psum, *psq;
    void *a1_store;
};

template <typename T, int K, int S, int TPP>
__global__ __launch_bounds__(TPP > 256 ? TPP : 256) void dw_fwd_kernel(DwFwdDev a)
{
    constexpr int P = (K - 1) / 2;
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    constexpr int PPB = BLOCK / TPP;
    extern __shared__ float lds[];
    const int H = a.s.H, W = a.s.W, Ho = a.s.Ho, Wo = a.s.Wo, C = a.s.C, N = a.s.N;
    const int Hp = H + 2 * P, Wp = W + 2 * P;
    const int lt = threadIdx.x % TPP;
    float *tile = lds + (threadIdx.x / TPP) * (Hp * Wp);
    float *red = lds + PPB * (Hp * Wp);
    const PlaneId pl = plane_of_group<TPP>(N, C, a.divC);

    float w[K * K];
    float scale = 1.f, shift = 0.f;
    const bool bn = a.bn1 != nullptr;
    if (pl.active) {
#pragma unroll
        for (int t = 0; t < K * K; ++t)
            w[t] = ld<T>((const T *)a.w, (size_t)pl.c * K * K + t);
        if (bn) {
            scale = a.bn1[pl.c];
            shift = a.bn1[C + pl.c];
        }
        const size_t base = pl.plane * (size_t)H * W;
        for (int idx = lt; idx < Hp * Wp; idx += TPP) {
            const int hp = (int)fdiv((uint32_t)idx, a.divWp);
            const int wp = idx - hp * Wp;
            const int h = hp - P, x = wp - P;
            float v = 0.f;
            if (h >= 0 && h < H && x >= 0 && x < W) {
                v = ld<T>((const T *)a.e, base + (size_t)h * W + x);
                if (bn)
                    v = actf(fmaf(v, scale, shift));
                if (a.a1_store)
                    st<T>((T *)a.a1_store, base + (size_t)h * W + x, v);
            }
            tile[idx] = v;
        }
    }
    __syncthreads();
    float acc2[2] = {0.f, 0.f};
    if (pl.active) {
        const size_t obase = pl.plane * (size_t)Ho * Wo;
        for (int idx = lt; idx < Ho * Wo; idx += TPP) {
            const int i = (int)fdiv((uint32_t)idx, a.divWo);
            const int j = idx - i * Wo;
            const float *t0 = tile + (i * S) * Wp + j * S;
            float acc = 0.f;
#pragma unroll
            for (int u = 0; u < K; ++u)
#pragma unroll
                for (int v = 0; v < K; ++v)
                    acc = fmaf(w[u * K + v], t0[u * Wp + v], acc);
            st<T>((T *)a.d, obase + idx, acc);
            const float sv = as_stored<T>(acc);
            acc2[0] += sv;
            acc2[1] += sv * sv;
        }
    }
    group_sum<2, TPP>(acc2, red);
    if (pl.active && lt == 0) {
        a.psum[(size_t)pl.c * N + pl.n] = acc2[0];
        a.psq[(size_t)pl.c * N + pl.n] = acc2[1];
    }
}

size_t dw_fwd_lds_bytes(const DwShape &s)
{
    const int tpp = pick_tpp(s.H * s.W);
    const int block = tpp > 256 ? tpp : 256;
    const int ppb = block / tpp;
    const int p = (s.k - 1) / 2;
    return sizeof(float) * ((size_t)ppb * (s.H + 2 * p) * (s.W + 2 * p) + (block / 64) * 2);
}

template <typename T, int K, int S>
static hipError_t dw_fwd_tpp(const DwFwdDev &a, hipStream_t st)
{
    const DwShape &s = a.s;
    const int tpp = pick_tpp(s.H * s.W);
    const size_t lds = dw_fwd_lds_bytes(s);
    const size_t planes = (size_t)s.N * s.C;
#define MBK_LAUNCH(TPP)                                                                           \
    {                                                                                             \
        constexpr int BLOCK = TPP > 256 ? TPP : 256;                                              \
        auto kern = dw_fwd_kernel<T, K, S, TPP>;                                                  \
        hipError_t e = hipFuncSetAttribute((const void *)kern,                                    \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess)                                                                      \
            return e;                                                                             \
        const unsigned grid = (unsigned)((planes + BLOCK / TPP - 1) / (BLOCK / TPP));             \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(BLOCK), lds, st, a);                            \
        return hipGetLastError();                                                                 \
    }
    if (tpp == 64)
        MBK_LAUNCH(64)
    if (tpp == 256)
        MBK_LAUNCH(256)
    MBK_LAUNCH(1024)
#undef MBK_LAUNCH
}

template <typename T>
static hipError_t dw_fwd_ks(const DwFwdDev &a, hipStream_t st)
{
    const int k = a.s.k, s = a.s.s;
    if (k == 3 && s == 1)
        return dw_fwd_tpp<T, 3, 1>(a, st);
    if (k == 3 && s == 2)
        return dw_fwd_tpp<T, 3, 2>(a, st);
    if (k == 5 && s == 1)
        return dw_fwd_tpp<T, 5, 1>(a, st);
    if (k == 5 && s == 2)
        return dw_fwd_tpp<T, 5, 2>(a, st);
    return hipErrorInvalidValue;
}

// A consumer finalises a normalisation itself where its planes are large enough that the extra
// reduction per plane (overlapped with the plane's first loads) costs less than a launch.
bool plane_finalize_pays(int HW) { return HW >= 1024; }

bool dw_fwd_finalizes_bn1(const DwShape &s, bool stores_a1)
{
    if (stores_a1)
        return false;
    if (dw4_supported(s)) // (launch_dw_fwd's order of preference)
        return plane_finalize_pays(s.H * s.W);
    return dwr_supported(s); // a wavefront per channel and image range: once per wavefront
}

hipError_t launch_dw_fwd(bool bf16, const DwShape &s, const void *e, const float *bn1,
                         const void *w_dw, void *d, float *psum, float *psq, void *a1_store,
                         const BnFin *fin, hipStream_t st)
{
    if (fin && !dw_fwd_finalizes_bn1(s, a1_store != nullptr))
        return hipErrorInvalidValue;
    if (!a1_store && dw4_supported(s))
        return launch_dw4_fwd(bf16, s, e, bn1, w_dw, d, psum, psq, fin, st);
    if (!a1_store && dwr_supported(s))
        return launch_dwr_fwd(bf16, s, e, bn1, w_dw, d, psum, psq, fin, st);
    if (!a1_store && dw2_supported(s))
        return launch_dw2_fwd(bf16, s, e, bn1, w_dw, d, psum, psq, st);
    DwFwdDev a;
    a.s = s;
    a.divC = make_div((uint32_t)s.C);
    a.divWp = make_div((uint32_t)(s.W + 2 * s.p));
    a.divWo = make_div((uint32_t)s.Wo);
    a.e = e;
    a.bn1 = bn1;
    a.w = w_dw;
    a.d = d;
    a.psum = psum;
    a.psq = psq;
    a.a1_store = a1_store;
    return bf16 ? dw_fwd_ks<bf16_t>(a, st) : dw_fwd_ks<float>(a, st);
}

// ---- backward ---------------------------------------------------------------------------------

struct DwBwdDev {
    DwShape s;
    FastDiv divC, divWp, divWq, divWo, divW;
    FastDiv divWc0, divWc1; // stride 2: columns per parity class starting at column 0 / 1
    const void *G, *d, *e;
    const float *g, *dzs, *bn2, *coef2, *bn1;
    const void *w;
    const void *a1_saved;
    void *dy1_out;
    const void *res;
    float *pdw, *psb, *psr;
};

template <typename T, int K, int S, int TPP>
__global__ __launch_bounds__(TPP > 256 ? TPP : 256, (K == 3 && TPP == 1024) ? 8 : 1) void dw_bwd_kernel(DwBwdDev a)
{
    constexpr int P = (K - 1) / 2;
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    constexpr int PPB = BLOCK / TPP;
    constexpr int NV = K * K + 2;
    extern __shared__ float lds[];
    const int H = a.s.H, W = a.s.W, Ho = a.s.Ho, Wo = a.s.Wo, C = a.s.C, N = a.s.N;
    const int Hp = H + 2 * P, Wp = W + 2 * P;    // a1 tile, border P
    const int Hq = Ho + 2 * P, Wq = Wo + 2 * P;  // dd tile, border P
    const int lt = threadIdx.x % TPP, grp = threadIdx.x / TPP;
    float *a1t = lds + grp * (Hp * Wp + Hq * Wq);
    float *ddt = a1t + Hp * Wp;
    float *red = lds + PPB * (Hp * Wp + Hq * Wq);
    const PlaneId pl = plane_of_group<TPP>(N, C, a.divC);
    const bool bn = a.bn1 != nullptr;

    float w[K * K];
    float scale1 = 1.f, shift1 = 0.f, mean1 = 0.f, rstd1 = 0.f;
    if (pl.active) {
#pragma unroll
        for (int t = 0; t < K * K; ++t)
            w[t] = ld<T>((const T *)a.w, (size_t)pl.c * K * K + t);
        if (bn) {
            scale1 = a.bn1[pl.c];
            shift1 = a.bn1[C + pl.c];
            mean1 = a.bn1[2 * C + pl.c];
            rstd1 = a.bn1[3 * C + pl.c];
        }
        // depthwise input a1 with a zero border
        const size_t ebase = pl.plane * (size_t)H * W;
        for (int idx = lt; idx < Hp * Wp; idx += TPP) {
            const int hp = (int)fdiv((uint32_t)idx, a.divWp);
            const int wp = idx - hp * Wp;
            const int h = hp - P, x = wp - P;
            float v = 0.f;
            if (h >= 0 && h < H && x >= 0 && x < W) {
                if (a.a1_saved) {
                    v = ld<T>((const T *)a.a1_saved, ebase + (size_t)h * W + x);
                } else {
                    v = ld<T>((const T *)a.e, ebase + (size_t)h * W + x);
                    if (bn)
                        v = actf(fmaf(v, scale1, shift1));
                }
            }
            a1t[idx] = v;
        }
        // gradient w.r.t. the depthwise output, dd, with a zero border
        const float scale2 = a.bn2[pl.c], shift2 = a.bn2[C + pl.c];
        const float c0 = a.coef2[pl.c], c1 = a.coef2[C + pl.c], c2 = a.coef2[2 * C + pl.c];
        const float gate = a.g[pl.plane], dzs = a.dzs[pl.plane];
        const size_t dbase = pl.plane * (size_t)Ho * Wo;
        for (int idx = lt; idx < Hq * Wq; idx += TPP) {
            const int ip = (int)fdiv((uint32_t)idx, a.divWq);
            const int jp = idx - ip * Wq;
            const int i = ip - P, j = jp - P;
            float v = 0.f;
            if (i >= 0 && i < Ho && j >= 0 && j < Wo) {
                const float Gv = ld<T>((const T *)a.G, dbase + (size_t)i * Wo + j);
                const float dv = ld<T>((const T *)a.d, dbase + (size_t)i * Wo + j);
                float val, grad;
                act_both(fmaf(dv, scale2, shift2), val, grad);
                const float dy2 = fmaf(Gv, gate, dzs) * grad;
                v = fmaf(c0, dy2, fmaf(c1, dv, c2));
            }
            ddt[idx] = v;
        }
    }
    __syncthreads();

    float acc[NV];
#pragma unroll
    for (int t = 0; t < NV; ++t)
        acc[t] = 0.f;
    if (pl.active) {
        // filter gradient: dw[u,v] += dd[i,j] * a1[i*S+u-P, j*S+v-P]
        for (int idx = lt; idx < Ho * Wo; idx += TPP) {
            const int i = (int)fdiv((uint32_t)idx, a.divWo);
            const int j = idx - i * Wo;
            const float ddv = ddt[(i + P) * Wq + j + P];
            const float *t0 = a1t + (i * S) * Wp + j * S;
#pragma unroll
            for (int u = 0; u < K; ++u)
#pragma unroll
                for (int v = 0; v < K; ++v)
                    acc[u * K + v] = fmaf(ddv, t0[u * Wp + v], acc[u * K + v]);
        }
        // input gradient: da1[h,x] = sum_{u,v} w[u,v]*dd[(h+P-u)/S, (x+P-v)/S] over the taps
        // for which both quotients are exact; in border coordinates the row is
        // (h+P-u+S*P)/S, always non-negative.
        const size_t ebase = pl.plane * (size_t)H * W;
        auto finish = [&](int idx, float da) { // Swish', store, BN1 partial sums
            if (bn) {
                const float raw = ld<T>((const T *)a.e, ebase + idx);
                float val, grad;
                act_both(fmaf(raw, scale1, shift1), val, grad);
                const float dy1 = da * grad;
                st<T>((T *)a.dy1_out, ebase + idx, dy1);
                const float sv = as_stored<T>(dy1);
                acc[K * K] += sv;
                acc[K * K + 1] = fmaf(sv, (raw - mean1) * rstd1, acc[K * K + 1]);
            } else {
                if (a.res)
                    da += ld<T>((const T *)a.res, ebase + idx);
                st<T>((T *)a.dy1_out, ebase + idx, da);
            }
        };
        if (S == 1) {
            for (int idx = lt; idx < H * W; idx += TPP) {
                const int h = (int)fdiv((uint32_t)idx, a.divW);
                const int x = idx - h * W;
                float da = 0.f;
#pragma unroll
                for (int u = 0; u < K; ++u)
#pragma unroll
                    for (int v = 0; v < K; ++v)
                        da = fmaf(w[u * K + v], ddt[(h + 2 * P - u) * Wq + x + 2 * P - v], da);
                finish(idx, da);
            }
        } else {
            // stride 2: an input pixel only meets the taps u = ph (mod 2), v = pw (mod 2) with
            // ph = (h+P)&1, pw = (x+P)&1.  The four parity classes are walked one after the
            // other so that the tap set, and hence the weight registers, are compile-time.
#pragma unroll
            for (int ph = 0; ph < 2; ++ph)
#pragma unroll
                for (int pw = 0; pw < 2; ++pw) {
                    const int hs = ph ^ (P & 1), xs = pw ^ (P & 1); // first row / column of the class
                    const int Hc = (H - hs + 1) >> 1, Wc = (W - xs + 1) >> 1;
                    const FastDiv dv = xs ? a.divWc1 : a.divWc0;
                    for (int idx = lt; idx < Hc * Wc; idx += TPP) {
                        const int hh = (int)fdiv((uint32_t)idx, dv);
                        const int h = hs + 2 * hh, x = xs + 2 * (idx - hh * Wc);
                        const int r0 = ((h + P - ph) >> 1) + P, c0 = ((x + P - pw) >> 1) + P;
                        float da = 0.f;
#pragma unroll
                        for (int ua = 0; ph + 2 * ua < K; ++ua)
#pragma unroll
                            for (int vb = 0; pw + 2 * vb < K; ++vb)
                                da = fmaf(w[(ph + 2 * ua) * K + pw + 2 * vb],
                                          ddt[(r0 - ua) * Wq + c0 - vb], da);
                        finish(h * W + x, da);
                    }
                }
        }
    }
    group_sum<NV, TPP>(acc, red);
    if (pl.active && lt == 0) {
        float *dst = a.pdw + ((size_t)pl.c * N + pl.n) * (K * K);
#pragma unroll
        for (int t = 0; t < K * K; ++t)
            dst[t] = acc[t];
        if (bn) {
            a.psb[(size_t)pl.c * N + pl.n] = acc[K * K];
            a.psr[(size_t)pl.c * N + pl.n] = acc[K * K + 1];
        }
    }
}

size_t dw_bwd_lds_bytes(const DwShape &s)
{
    const int tpp = pick_tpp(s.H * s.W);
    const int block = tpp > 256 ? tpp : 256;
    const int ppb = block / tpp;
    const int p = (s.k - 1) / 2;
    const size_t per = (size_t)(s.H + 2 * p) * (s.W + 2 * p) + (size_t)(s.Ho + 2 * p) * (s.Wo + 2 * p);
    return sizeof(float) * (ppb * per + (size_t)(block / 64) * (s.k * s.k + 2));
}

template <typename T, int K, int S>
static hipError_t dw_bwd_tpp(const DwBwdDev &a, hipStream_t st)
{
    const DwShape &s = a.s;
    const int tpp = pick_tpp(s.H * s.W);
    const size_t lds = dw_bwd_lds_bytes(s);
    const size_t planes = (size_t)s.N * s.C;
#define MBK_LAUNCH(TPP)                                                                           \
    {                                                                                             \
        constexpr int BLOCK = TPP > 256 ? TPP : 256;                                              \
        auto kern = dw_bwd_kernel<T, K, S, TPP>;                                                  \
        hipError_t e = hipFuncSetAttribute((const void *)kern,                                    \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess)                                                                      \
            return e;                                                                             \
        const unsigned grid = (unsigned)((planes + BLOCK / TPP - 1) / (BLOCK / TPP));             \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(BLOCK), lds, st, a);                            \
        return hipGetLastError();                                                                 \
    }
    if (tpp == 64)
        MBK_LAUNCH(64)
    if (tpp == 256)
        MBK_LAUNCH(256)
    MBK_LAUNCH(1024)
#undef MBK_LAUNCH
}

template <typename T>
static hipError_t dw_bwd_ks(const DwBwdDev &a, hipStream_t st)
{
    const int k = a.s.k, s = a.s.s;
    if (k == 3 && s == 1)
        return dw_bwd_tpp<T, 3, 1>(a, st);
    if (k == 3 && s == 2)
        return dw_bwd_tpp<T, 3, 2>(a, st);
    if (k == 5 && s == 1)
        return dw_bwd_tpp<T, 5, 1>(a, st);
    if (k == 5 && s == 2)
        return dw_bwd_tpp<T, 5, 2>(a, st);
    return hipErrorInvalidValue;
}

hipError_t launch_dw_bwd(bool bf16, const DwBwdArgs &h, hipStream_t st)
{
    if (!h.a1_saved && dw4_supported(h.s))
        return launch_dw4_bwd(bf16, h, st);
    if (!h.a1_saved && dwr_supported(h.s))
        return launch_dwr_bwd(bf16, h, st);
    if (!h.a1_saved && !h.res && dw2_supported(h.s))
        return launch_dw2_bwd(bf16, h, st);
    DwBwdDev a;
    a.s = h.s;
    const int p = h.s.p;
    a.divC = make_div((uint32_t)h.s.C);
    a.divWp = make_div((uint32_t)(h.s.W + 2 * p));
    a.divWq = make_div((uint32_t)(h.s.Wo + 2 * p));
    a.divWo = make_div((uint32_t)h.s.Wo);
    a.divW = make_div((uint32_t)h.s.W);
    a.divWc0 = make_div((uint32_t)std::max(1, (h.s.W + 1) / 2));
    a.divWc1 = make_div((uint32_t)std::max(1, h.s.W / 2));
    a.G = h.G;
    a.d = h.d;
    a.e = h.e;
    a.g = h.g;
    a.dzs = h.dzs;
    a.bn2 = h.bn2;
    a.coef2 = h.coef2;
    a.bn1 = h.bn1;
    a.w = h.w_dw;
    a.a1_saved = h.a1_saved;
    a.dy1_out = h.dy1_out;
    a.res = h.res;
    a.pdw = h.pdw;
    a.psb = h.psb;
    a.psr = h.psr;
    return bf16 ? dw_bwd_ks<bf16_t>(a, st) : dw_bwd_ks<float>(a, st);
}

// ---- per-plane reductions and the final elementwise pass --------------------------------------

struct PlaneArgs {
    int N, C, HW;
    FastDiv divC;
    const void *t0, *t1;
    const float *bn; // {scale, shift, mean, rstd}[C]
    float *o0, *o1, *o2;
    int layoutCN; // 1: outputs indexed [c][n]; 0: [n][c]
    float o0_scale; // multiplies the first output (1/HW turns a plane sum into a mean)
    void *out;    // elementwise output (bn_apply)
    const void *res;
    BnFin fin;    // bn_apply, fin.psum non-null: `bn` is derived there from the partial sums
};

// Four consecutive elements at once (16 bytes per lane for fp32, 8 for bf16).
template <typename T>
__device__ __forceinline__ void ldvec4(const T *p, size_t i, float (&v)[4]);
template <>
__device__ __forceinline__ void ldvec4<float>(const float *p, size_t i, float (&v)[4])
{
    const float4 t = *reinterpret_cast<const float4 *>(p + i);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
}
template <>
__device__ __forceinline__ void ldvec4<bf16_t>(const bf16_t *p, size_t i, float (&v)[4])
{
    const uint2 t = *reinterpret_cast<const uint2 *>(&p[i]);
    v[0] = bf16_bits_to_float(t.x & 0xffffu);
    v[1] = bf16_bits_to_float(t.x >> 16);
    v[2] = bf16_bits_to_float(t.y & 0xffffu);
    v[3] = bf16_bits_to_float(t.y >> 16);
}
template <typename T>
__device__ __forceinline__ void stvec4(T *p, size_t i, const float (&v)[4]);
template <>
__device__ __forceinline__ void stvec4<float>(float *p, size_t i, const float (&v)[4])
{
    *reinterpret_cast<float4 *>(p + i) = make_float4(v[0], v[1], v[2], v[3]);
}
template <>
__device__ __forceinline__ void stvec4<bf16_t>(bf16_t *p, size_t i, const float (&v)[4])
{
    uint2 t;
    t.x = bf16_pack2(v[0], v[1]);
    t.y = bf16_pack2(v[2], v[3]);
    *reinterpret_cast<uint2 *>(&p[i]) = t;
}

// z = mean swish(y), s3 = sum swish'(y), s4 = sum swish'(y)*xhat, y = BN(t0)
struct OpPool {
    static constexpr int NV = 3;
    static constexpr bool kTwo = false;
    static __device__ __forceinline__ void eval(float v, float, float sc, float sh, float mu,
                                                float rs, float (&acc)[NV])
    {
        float val, grad;
        act_both(fmaf(v, sc, sh), val, grad);
        acc[0] += val;
        acc[1] += grad;
        acc[2] = fmaf(grad, (v - mu) * rs, acc[2]);
    }
};
// sums of dy (t0) and dy*xhat(t1)
struct OpDot {
    static constexpr int NV = 2;
    static constexpr bool kTwo = true;
    static __device__ __forceinline__ void eval(float dy, float raw, float, float, float mu,
                                                float rs, float (&acc)[NV])
    {
        acc[0] += dy;
        acc[1] = fmaf(dy, (raw - mu) * rs, acc[1]);
    }
};
// G (t0) against a2, swish'(y2), swish'(y2)*dhat rebuilt from d (t1)
struct OpGate {
    static constexpr int NV = 3;
    static constexpr bool kTwo = true;
    static __device__ __forceinline__ void eval(float Gv, float v, float sc, float sh, float mu,
                                                float rs, float (&acc)[NV])
    {
        float val, grad;
        act_both(fmaf(v, sc, sh), val, grad);
        acc[0] = fmaf(Gv, val, acc[0]);
        acc[1] = fmaf(Gv, grad, acc[1]);
        acc[2] = fmaf(Gv * grad, (v - mu) * rs, acc[2]);
    }
};

template <typename T, int TPP, typename OP>
__global__ __launch_bounds__(TPP > 256 ? TPP : 256) void plane_reduce_kernel(PlaneArgs a)
{
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    __shared__ float red[(BLOCK / 64) * OP::NV];
    const int lt = threadIdx.x % TPP;
    const PlaneId pl = plane_of_group<TPP>(a.N, a.C, a.divC);
    float acc[OP::NV];
#pragma unroll
    for (int t = 0; t < OP::NV; ++t)
        acc[t] = 0.f;
    if (pl.active) {
        const float sc = a.bn[pl.c], sh = a.bn[a.C + pl.c];
        const float mu = a.bn[2 * a.C + pl.c], rs = a.bn[3 * a.C + pl.c];
        const size_t base = pl.plane * (size_t)a.HW;
        // Four strides of the plane per round: all loads of a round are issued before any of
        // them is consumed (the scheduler fence keeps the compiler from pairing each load with
        // its arithmetic, which would cost one memory round trip per stride).
        if ((a.HW & 3) == 0) {
            float v0[4][4], v1[4][4];
            const auto load_round = [&](int idx0) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int idx = idx0 + 4 * TPP * u;
                    // past the end: reread an element of the plane, masked when consumed
                    const int ic = idx < a.HW ? idx : (idx0 < a.HW ? idx0 : 0);
                    ldvec4<T>((const T *)a.t0, base + ic, v0[u]);
                    if (OP::kTwo)
                        ldvec4<T>((const T *)a.t1, base + ic, v1[u]);
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            int idx0 = 4 * lt;
            load_round(idx0);
            while (true) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (idx0 + 4 * TPP * u < a.HW) {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            OP::eval(v0[u][r], OP::kTwo ? v1[u][r] : 0.f, sc, sh, mu, rs, acc);
                    }
                }
                idx0 += 16 * TPP;
                if (idx0 >= a.HW)
                    break;
                load_round(idx0);
            }
        } else {
            for (int idx0 = lt; idx0 < a.HW; idx0 += 4 * TPP) {
                float v0[4], v1[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int idx = idx0 + TPP * u;
                    const int ic = idx < a.HW ? idx : idx0;
                    v0[u] = ld<T>((const T *)a.t0, base + ic);
                    v1[u] = OP::kTwo ? ld<T>((const T *)a.t1, base + ic) : 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (idx0 + TPP * u < a.HW)
                        OP::eval(v0[u], v1[u], sc, sh, mu, rs, acc);
            }
        }
    }
    group_sum<OP::NV, TPP>(acc, red);
    if (pl.active && lt == 0) {
        const size_t o = a.layoutCN ? (size_t)pl.c * a.N + pl.n : pl.plane;
        float *outs[3] = {a.o0, a.o1, a.o2};
#pragma unroll
        for (int t = 0; t < OP::NV; ++t)
            outs[t][o] = t == 0 ? acc[t] * a.o0_scale : acc[t];
    }
}

template <typename T, int TPP>
__global__ __launch_bounds__(TPP > 256 ? TPP : 256) void bn_apply_kernel(PlaneArgs a)
{
    constexpr int BLOCK = TPP > 256 ? TPP : 256;
    __shared__ double redd[2 * (BLOCK / 64)];
    const int lt = threadIdx.x % TPP;
    const PlaneId pl = plane_of_group<TPP>(a.N, a.C, a.divC);
    if (!pl.active) // (TPP > 64: one plane per workgroup, always active)
        return;
    float sc, sh;
    BnFinRegs fr;
    if (TPP >= 64 && a.fin.psum) { // (a 16-lane group never finalises: its planes are small)
        bn_fin_issue<TPP>(a.fin, pl.c, lt, fr);
    } else {
        sc = a.bn[pl.c];
        sh = a.bn[a.C + pl.c];
    }
    __builtin_amdgcn_sched_barrier(0);
    const auto coefs = [&]() {
        float mu, rs;
        if constexpr (TPP >= 64) {
            if (a.fin.psum)
                bn_fin_finish<TPP>(a.fin, a.C, pl.c, lt, pl.n == 0, redd, fr, sc, sh, mu, rs);
        }
    };
    const size_t base = pl.plane * (size_t)a.HW;
    if ((a.HW & 3) == 0) {
        // (coefficient requests in front of the first round's loads, as in plane_reduce_kernel)
        float v[4][4], rr[4][4];
        const auto load_round = [&](int idx0) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = idx0 + 4 * TPP * u;
                const int ic = idx < a.HW ? idx : (idx0 < a.HW ? idx0 : 0);
                ldvec4<T>((const T *)a.t0, base + ic, v[u]);
                if (a.res)
                    ldvec4<T>((const T *)a.res, base + ic, rr[u]);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        int idx0 = 4 * lt;
        load_round(idx0);
        coefs();
        __builtin_amdgcn_sched_barrier(0);
        while (true) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = idx0 + 4 * TPP * u;
                if (idx < a.HW) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        v[u][r] = fmaf(v[u][r], sc, sh);
                        if (a.res)
                            v[u][r] += rr[u][r];
                    }
                    stvec4<T>((T *)a.out, base + idx, v[u]);
                }
            }
            idx0 += 16 * TPP;
            if (idx0 >= a.HW)
                break;
            load_round(idx0);
        }
    } else {
        coefs();
        for (int idx = lt; idx < a.HW; idx += TPP) {
            float v = fmaf(ld<T>((const T *)a.t0, base + idx), sc, sh);
            if (a.res)
                v += ld<T>((const T *)a.res, base + idx);
            st<T>((T *)a.out, base + idx, v);
        }
    }
}

template <typename T, typename OP>
static hipError_t plane_reduce_launch(const PlaneArgs &a, hipStream_t st)
{
    const int tpp = pick_tpp_plane(a.HW);
    const size_t planes = (size_t)a.N * a.C;
#define MBK_LAUNCH(TPP)                                                                           \
    {                                                                                             \
        constexpr int BLOCK = TPP > 256 ? TPP : 256;                                              \
        const unsigned grid = (unsigned)((planes + BLOCK / TPP - 1) / (BLOCK / TPP));             \
        hipLaunchKernelGGL((plane_reduce_kernel<T, TPP, OP>), dim3(grid), dim3(BLOCK), 0, st, a); \
        return hipGetLastError();                                                                 \
    }
    if (tpp == 16)
        MBK_LAUNCH(16)
    if (tpp == 64)
        MBK_LAUNCH(64)
    if (tpp == 256)
        MBK_LAUNCH(256)
    MBK_LAUNCH(1024)
#undef MBK_LAUNCH
}

static PlaneArgs plane_args(int N, int C, int HW, const void *t0, const void *t1, const float *bn)
{
    PlaneArgs a = {};
    a.N = N;
    a.C = C;
    a.HW = HW;
    a.divC = make_div((uint32_t)C);
    a.t0 = t0;
    a.t1 = t1;
    a.bn = bn;
    a.o0_scale = 1.f;
    return a;
}

hipError_t launch_pool(bool bf16, int N, int C, int HW, const void *d, const float *bn2, float *z,
                       float *s3, float *s4, hipStream_t st)
{
    PlaneArgs a = plane_args(N, C, HW, d, nullptr, bn2);
    a.o0 = z;
    a.o1 = s3;
    a.o2 = s4;
    a.layoutCN = 0;
    a.o0_scale = 1.f / (float)HW;
    return bf16 ? plane_reduce_launch<bf16_t, OpPool>(a, st) : plane_reduce_launch<float, OpPool>(a, st);
}

hipError_t launch_plane_dot(bool bf16, int N, int C, int HW, const void *dy, const void *raw,
                            const float *bn, float *psb, float *psr, hipStream_t st)
{
    PlaneArgs a = plane_args(N, C, HW, dy, raw, bn);
    a.o0 = psb;
    a.o1 = psr;
    a.layoutCN = 1;
    return bf16 ? plane_reduce_launch<bf16_t, OpDot>(a, st) : plane_reduce_launch<float, OpDot>(a, st);
}

hipError_t launch_gate_sums(bool bf16, int N, int C, int HW, const void *G, const void *d,
                            const float *bn2, float *dg, float *A1, float *A2, hipStream_t st)
{
    PlaneArgs a = plane_args(N, C, HW, G, d, bn2);
    a.o0 = dg;
    a.o1 = A1;
    a.o2 = A2;
    a.layoutCN = 0;
    return bf16 ? plane_reduce_launch<bf16_t, OpGate>(a, st) : plane_reduce_launch<float, OpGate>(a, st);
}

hipError_t launch_bn_apply(bool bf16, int N, int C, int HW, const void *p, const float *bn3,
                           const void *res, void *out, const BnFin *fin, hipStream_t st)
{
    PlaneArgs a = plane_args(N, C, HW, p, nullptr, bn3);
    if (fin)
        a.fin = *fin;
    a.out = out;
    a.res = res;
    const int tpp = pick_tpp_plane(HW);
    const size_t planes = (size_t)N * C;
#define MBK_LAUNCH(TPP)                                                                           \
    {                                                                                             \
        constexpr int BLOCK = TPP > 256 ? TPP : 256;                                              \
        const unsigned grid = (unsigned)((planes + BLOCK / TPP - 1) / (BLOCK / TPP));             \
        if (bf16)                                                                                 \
            hipLaunchKernelGGL((bn_apply_kernel<bf16_t, TPP>), dim3(grid), dim3(BLOCK), 0, st, a);\
        else                                                                                      \
            hipLaunchKernelGGL((bn_apply_kernel<float, TPP>), dim3(grid), dim3(BLOCK), 0, st, a); \
        return hipGetLastError();                                                                 \
    }
    if (tpp == 16)
        MBK_LAUNCH(16)
    if (tpp == 64)
        MBK_LAUNCH(64)
    if (tpp == 256)
        MBK_LAUNCH(256)
    MBK_LAUNCH(1024)
#undef MBK_LAUNCH
}

} // namespace mbk
