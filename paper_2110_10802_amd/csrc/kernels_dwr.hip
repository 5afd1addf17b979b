// Depthwise chain for the small planes of the late stages (stride 1, any width; 14x14 and 7x7
// in EfficientNet-B0), where a plane is only a few dozen runs of four pixels.
//
// A wavefront owns one channel and a range of images and walks them in a software-pipelined
// loop: lane = (plane slot, run), with as many planes side by side as fit into 64 lanes
// (four 7x7 planes, one 14x14 plane).  The raw values of the next planes are loaded while the
// current ones are processed (a dependent global load costs about a microsecond on this chip,
// so nothing waits on a load issued in the same iteration); the filter, the BN constants and
// the border of the LDS tiles are set up once per wavefront; and the filter-gradient and
// BN-statistics accumulators stay in registers across all images of the range, so there is one
// wavefront reduction per range instead of one per plane.  Partial results are written per
// (channel, range) and added by the fixed-order second stage (no atomics).
//
// Rows are padded to a multiple of four columns inside LDS (pad columns hold zeros), so the
// k x k stencil uses the same 16-byte window reads as the wide-plane kernels; global accesses
// are 16, 8 or 4 bytes per lane depending on the divisibility of the width.
#include "mbconv_dev.h"
#include "mbconv_launch.h"
#include "mbconv_bnfin.h"

namespace mbk {

typedef float float4v __attribute__((ext_vector_type(4)));

struct DwrArgs {
    int N, C, H, W;
    int W4;   // runs per row = ceil(W/4)
    int WP;   // tile pitch = 4*W4 + 8 (interior starts at column 4)
    int runs; // H*W4
    int PW;   // planes side by side in one wavefront
    int nseg, nper; // image ranges per channel, images per range
    FastDiv divRuns, divW4, divNseg;
    const void *e;
    const float *bn1;
    const void *w;
    void *d;
    float *psum, *psq;
    BnFin fin; // forward, fin.psum non-null: bn1 is derived in the kernel from the partial sums
    const void *G;
    const float *g, *dzs, *bn2, *coef2;
    void *dy1_out;
    const void *res;
    float *pdw, *psb, *psr;
};

// ---- one run of four pixels (columns x0..x0+3, those >= W masked) ----------------------------
template <typename T, int GV>
__device__ __forceinline__ void run_load(const T *p, size_t idx, int x0, int W, float (&v)[4]);

template <>
__device__ __forceinline__ void run_load<float, 4>(const float *p, size_t idx, int, int, float (&v)[4])
{
    const float4v t = *reinterpret_cast<const float4v *>(p + idx);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
}
template <>
__device__ __forceinline__ void run_load<float, 2>(const float *p, size_t idx, int x0, int W, float (&v)[4])
{
    float2 a = make_float2(0.f, 0.f), b = make_float2(0.f, 0.f);
    if (x0 < W)
        a = *reinterpret_cast<const float2 *>(p + idx);
    if (x0 + 2 < W)
        b = *reinterpret_cast<const float2 *>(p + idx + 2);
    v[0] = a.x;
    v[1] = a.y;
    v[2] = b.x;
    v[3] = b.y;
}
template <>
__device__ __forceinline__ void run_load<float, 1>(const float *p, size_t idx, int x0, int W, float (&v)[4])
{
#pragma unroll
    for (int r = 0; r < 4; ++r)
        v[r] = x0 + r < W ? p[idx + r] : 0.f;
}
template <>
__device__ __forceinline__ void run_load<bf16_t, 4>(const bf16_t *p, size_t idx, int, int, float (&v)[4])
{
    const uint2 t = *reinterpret_cast<const uint2 *>(&p[idx]);
    v[0] = bf16_bits_to_float(t.x & 0xffffu);
    v[1] = bf16_bits_to_float(t.x >> 16);
    v[2] = bf16_bits_to_float(t.y & 0xffffu);
    v[3] = bf16_bits_to_float(t.y >> 16);
}
template <>
__device__ __forceinline__ void run_load<bf16_t, 2>(const bf16_t *p, size_t idx, int x0, int W, float (&v)[4])
{
    uint32_t a = 0, b = 0;
    if (x0 < W)
        a = *reinterpret_cast<const uint32_t *>(&p[idx]);
    if (x0 + 2 < W)
        b = *reinterpret_cast<const uint32_t *>(&p[idx + 2]);
    v[0] = bf16_bits_to_float(a & 0xffffu);
    v[1] = bf16_bits_to_float(a >> 16);
    v[2] = bf16_bits_to_float(b & 0xffffu);
    v[3] = bf16_bits_to_float(b >> 16);
}
template <>
__device__ __forceinline__ void run_load<bf16_t, 1>(const bf16_t *p, size_t idx, int x0, int W, float (&v)[4])
{
#pragma unroll
    for (int r = 0; r < 4; ++r)
        v[r] = x0 + r < W ? bf16_bits_to_float(p[idx + r].bits) : 0.f;
}

template <typename T, int GV>
__device__ __forceinline__ void run_store(T *p, size_t idx, int x0, int W, const float (&v)[4]);

template <>
__device__ __forceinline__ void run_store<float, 4>(float *p, size_t idx, int, int, const float (&v)[4])
{
    float4v t = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<float4v *>(p + idx) = t;
}
template <>
__device__ __forceinline__ void run_store<float, 2>(float *p, size_t idx, int x0, int W, const float (&v)[4])
{
    if (x0 < W)
        *reinterpret_cast<float2 *>(p + idx) = make_float2(v[0], v[1]);
    if (x0 + 2 < W)
        *reinterpret_cast<float2 *>(p + idx + 2) = make_float2(v[2], v[3]);
}
template <>
__device__ __forceinline__ void run_store<float, 1>(float *p, size_t idx, int x0, int W, const float (&v)[4])
{
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (x0 + r < W)
            p[idx + r] = v[r];
}
template <>
__device__ __forceinline__ void run_store<bf16_t, 4>(bf16_t *p, size_t idx, int, int, const float (&v)[4])
{
    uint2 t;
    t.x = bf16_pack2(v[0], v[1]);
    t.y = bf16_pack2(v[2], v[3]);
    *reinterpret_cast<uint2 *>(&p[idx]) = t;
}
template <>
__device__ __forceinline__ void run_store<bf16_t, 2>(bf16_t *p, size_t idx, int x0, int W, const float (&v)[4])
{
    if (x0 < W)
        *reinterpret_cast<uint32_t *>(&p[idx]) =
            bf16_pack2(v[0], v[1]);
    if (x0 + 2 < W)
        *reinterpret_cast<uint32_t *>(&p[idx + 2]) =
            bf16_pack2(v[2], v[3]);
}
template <>
__device__ __forceinline__ void run_store<bf16_t, 1>(bf16_t *p, size_t idx, int x0, int W, const float (&v)[4])
{
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (x0 + r < W)
            p[idx + r].bits = float_to_bf16_bits(v[r]);
}

// One row of a (K+3)-wide window starting at column (4 + x0 - P) of tile row `row`.
template <int K>
__device__ __forceinline__ void window_row(const float *tile, int row, int WP, int x0, float (&o)[K + 3])
{
    constexpr int P = (K - 1) / 2;
    const float *p = tile + row * WP + 4 + x0;
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

// Every wavefront of these kernels works on LDS tiles of its own, so no workgroup barrier is
// needed: a wavefront's LDS operations execute in order, and this fence keeps the compiler from
// moving the tile reads above the tile writes of other lanes.  The four wavefronts of a
// workgroup then run independently instead of at the pace of the slowest.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Lane geometry shared by forward and backward.
struct DwrLane {
    int c, seg;      // channel and image range of this wavefront
    bool wave_ok;    // the wavefront has a (channel, range)
    int pw, h, x0;   // plane slot, row and first column of this lane's run
    bool lane_ok;    // the lane has a run
    int n_begin, n_end, iters;
};
__device__ __forceinline__ DwrLane dwr_lane(const DwrArgs &a)
{
    DwrLane L;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int slot = blockIdx.x * 4 + wave;
    L.c = (int)fdiv((uint32_t)slot, a.divNseg);
    L.seg = slot - L.c * a.nseg;
    L.wave_ok = L.c < a.C;
    if (!L.wave_ok)
        L.c = 0;
    L.pw = (int)fdiv((uint32_t)lane, a.divRuns);
    const int r = lane - L.pw * a.runs;
    L.h = (int)fdiv((uint32_t)r, a.divW4);
    L.x0 = 4 * (r - L.h * a.W4);
    L.lane_ok = L.pw < a.PW;
    L.n_begin = L.seg * a.nper;
    L.n_end = min(a.N, L.n_begin + a.nper);
    L.iters = (a.nper + a.PW - 1) / a.PW;
    return L;
}

// ---- forward: d = depthwise(swish(bn1(e))), partial sums of d and d^2 per (channel, range) ----
template <typename T, int K, int GV, bool EXPAND>
__global__ __launch_bounds__(256) void dwr_fwd_kernel(DwrArgs a)
{
    constexpr int P = (K - 1) / 2;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int H = a.H, W = a.W, WP = a.WP;
    const int tileElems = (H + 2 * P) * WP;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const DwrLane L = dwr_lane(a);
    // per wavefront: two buffers of PW tiles
    float *mine = lds + wave * (2 * a.PW * tileElems);
    for (int i = lane; i < 2 * a.PW * tileElems / 4; i += 64)
        reinterpret_cast<float4v *>(mine)[i] = float4v{0.f, 0.f, 0.f, 0.f};

    float wt[K * K];
#pragma unroll
    for (int t = 0; t < K * K; ++t)
        wt[t] = ld<T>((const T *)a.w, (size_t)L.c * K * K + t);
    // BN1's coefficients: fetched, or finalised here from the expansion conv's partial sums.  A
    // wavefront owns a channel and a range of images, so the finalise step is paid once per
    // wavefront, not once per plane; the wavefront of the channel's first range stores the block.
    float scale = 1.f, shift = 0.f;
    BnFinRegs fr;
    const bool fuse = EXPAND && a.fin.psum != nullptr;
    if (EXPAND) {
        if (fuse) {
            bn_fin_issue<64>(a.fin, L.c, lane, fr);
        } else {
            scale = a.bn1[L.c];
            shift = a.bn1[a.C + L.c];
        }
    }
    const size_t hw = (size_t)H * W;
    const int off = L.h * W + L.x0;
    float pe[4] = {0.f, 0.f, 0.f, 0.f};
    auto prefetch = [&](int it) -> bool {
        const int n = L.n_begin + it * a.PW + L.pw;
        const bool ok = L.wave_ok && L.lane_ok && n < L.n_end;
        if (ok)
            run_load<T, GV>((const T *)a.e, ((size_t)n * a.C + L.c) * hw + off, L.x0, W, pe);
        return ok;
    };
    bool cur_ok = prefetch(0);
    if (fuse) {
        float mu, rs;
        bn_fin_finish<64>(a.fin, a.C, L.c, lane, L.wave_ok && L.seg == 0, nullptr, fr, scale, shift, mu, rs);
    }
    float acc0 = 0.f, acc1 = 0.f;
    wave_lds_sync();
    for (int it = 0; it < L.iters; ++it) {
        float *tile = mine + ((it & 1) * a.PW + (L.lane_ok ? L.pw : 0)) * tileElems;
        const int n = L.n_begin + it * a.PW + L.pw;
        const bool ok = cur_ok;
        if (L.lane_ok) {
            float av[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool m = ok && L.x0 + r < W;
                const float v = EXPAND ? actf(fmaf(pe[r], scale, shift)) : pe[r];
                av[r] = m ? v : 0.f;
            }
            *reinterpret_cast<float4v *>(tile + (L.h + P) * WP + 4 + L.x0) =
                float4v{av[0], av[1], av[2], av[3]};
        }
        if (it + 1 < L.iters)
            cur_ok = prefetch(it + 1);
        wave_lds_sync();
        if (ok) {
            float o[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < K; ++u) {
                float row[K + 3];
                window_row<K>(tile, L.h + u, WP, L.x0, row);
#pragma unroll
                for (int v = 0; v < K; ++v)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[r] = fmaf(wt[u * K + v], row[r + v], o[r]);
            }
            run_store<T, GV>((T *)a.d, ((size_t)n * a.C + L.c) * hw + off, L.x0, W, o);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (L.x0 + r < W) {
                    const float sv = as_stored<T>(o[r]);
                    acc0 += sv;
                    acc1 = fmaf(sv, sv, acc1);
                }
            }
        }
    }
    acc0 = wave_sum(acc0);
    acc1 = wave_sum(acc1);
    if (L.wave_ok && lane == 0) {
        a.psum[(size_t)L.c * a.nseg + L.seg] = acc0;
        a.psq[(size_t)L.c * a.nseg + L.seg] = acc1;
    }
}

// ---- backward (the fused kernel described in mbconv_launch.h, DwBwdArgs) -----------------------
template <typename T, int K, int GV, bool EXPAND>
__global__ __launch_bounds__(256) void dwr_bwd_kernel(DwrArgs a)
{
    constexpr int P = (K - 1) / 2;
    constexpr int NV = K * K + 2;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int H = a.H, W = a.W, WP = a.WP, C = a.C;
    const int tileElems = (H + 2 * P) * WP;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const DwrLane L = dwr_lane(a);
    // per wavefront: two buffers of PW dd tiles.  There is no a1 tile: the filter gradient
    // dW[u][v] = sum_p dd[p] * a1[p + (u,v) - P] is summed over q = p + (u,v) - P, which pairs each
    // lane's own a1 values (registers) with the dd window elements the input gradient reads anyway.
    float *mine = lds + wave * (2 * a.PW * tileElems);
    for (int i = lane; i < 2 * a.PW * tileElems / 4; i += 64)
        reinterpret_cast<float4v *>(mine)[i] = float4v{0.f, 0.f, 0.f, 0.f};

    float wt[K * K];
#pragma unroll
    for (int t = 0; t < K * K; ++t)
        wt[t] = ld<T>((const T *)a.w, (size_t)L.c * K * K + t);
    float scale1 = 1.f, shift1 = 0.f, mean1 = 0.f, rstd1 = 0.f;
    if (EXPAND) {
        scale1 = a.bn1[L.c];
        shift1 = a.bn1[C + L.c];
        mean1 = a.bn1[2 * C + L.c];
        rstd1 = a.bn1[3 * C + L.c];
    }
    const float scale2 = a.bn2[L.c], shift2 = a.bn2[C + L.c];
    const float c0 = a.coef2[L.c], c1 = a.coef2[C + L.c], c2 = a.coef2[2 * C + L.c];
    const size_t hw = (size_t)H * W;
    const int off = L.h * W + L.x0;

    float pe[4] = {0.f, 0.f, 0.f, 0.f}, pG[4] = {0.f, 0.f, 0.f, 0.f}, pd[4] = {0.f, 0.f, 0.f, 0.f};
    float pgate = 0.f, pdzs = 0.f;
    auto prefetch = [&](int it) -> bool {
        const int n = L.n_begin + it * a.PW + L.pw;
        const bool ok = L.wave_ok && L.lane_ok && n < L.n_end;
        if (ok) {
            const size_t plane = (size_t)n * C + L.c;
            run_load<T, GV>((const T *)a.e, plane * hw + off, L.x0, W, pe);
            run_load<T, GV>((const T *)a.G, plane * hw + off, L.x0, W, pG);
            run_load<T, GV>((const T *)a.d, plane * hw + off, L.x0, W, pd);
            pgate = a.g[plane];
            pdzs = a.dzs[plane];
        }
        return ok;
    };
    bool cur_ok = prefetch(0);
    float acc[NV];
#pragma unroll
    for (int t = 0; t < NV; ++t)
        acc[t] = 0.f;
    wave_lds_sync();
    for (int it = 0; it < L.iters; ++it) {
        float *ddt = mine + ((it & 1) * a.PW + (L.lane_ok ? L.pw : 0)) * tileElems;
        const int n = L.n_begin + it * a.PW + L.pw;
        const bool ok = cur_ok;
        float rawk[4], sgk[4], a1c[4];
        if (L.lane_ok) {
            float ddv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool m = ok && L.x0 + r < W;
                float v = pe[r];
                if (EXPAND) {
                    const float y = fmaf(pe[r], scale1, shift1);
                    const float sg = act_aux(y);
                    rawk[r] = pe[r];
                    sgk[r] = sg;
                    v = act_val(y, sg);
                }
                a1c[r] = m ? v : 0.f;
                const float y2 = fmaf(pd[r], scale2, shift2);
                const float s2 = act_aux(y2);
                const float grad2 = act_grad(y2, s2);
                const float dy2 = fmaf(pG[r], pgate, pdzs) * grad2;
                ddv[r] = m ? fmaf(c0, dy2, fmaf(c1, pd[r], c2)) : 0.f;
            }
            *reinterpret_cast<float4v *>(ddt + (L.h + P) * WP + 4 + L.x0) =
                float4v{ddv[0], ddv[1], ddv[2], ddv[3]};
        }
        if (it + 1 < L.iters)
            cur_ok = prefetch(it + 1);
        wave_lds_sync();
        if (ok) {
            float da[4] = {0.f, 0.f, 0.f, 0.f};
            // input gradient  da[r]     = sum_{u,v} wt[u][v] * ddwin[K-1-u][r+K-1-v]
            // filter gradient acc[u][v] += sum_r   a1c[r]   * ddwin[K-1-u][r+K-1-v]
#pragma unroll
            for (int rr = 0; rr < K; ++rr) {
                float row[K + 3];
                window_row<K>(ddt, L.h + rr, WP, L.x0, row);
                const int u = K - 1 - rr;
#pragma unroll
                for (int v = 0; v < K; ++v)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        da[r] = fmaf(wt[u * K + v], row[r + K - 1 - v], da[r]);
                        acc[u * K + v] = fmaf(a1c[r], row[r + K - 1 - v], acc[u * K + v]);
                    }
            }
            const size_t base = ((size_t)n * C + L.c) * hw + off;
            float o[4];
            if (EXPAND) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float raw = rawk[r], sg = sgk[r];
                    const float y = fmaf(raw, scale1, shift1);
                    o[r] = da[r] * act_grad(y, sg);
                    if (L.x0 + r < W) {
                        const float sv = as_stored<T>(o[r]);
                        acc[K * K] += sv;
                        acc[K * K + 1] = fmaf(sv, (raw - mean1) * rstd1, acc[K * K + 1]);
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    o[r] = da[r];
                if (a.res) {
                    float rv[4];
                    run_load<T, GV>((const T *)a.res, base, L.x0, W, rv);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[r] += rv[r];
                }
            }
            run_store<T, GV>((T *)a.dy1_out, base, L.x0, W, o);
        }
    }
#pragma unroll
    for (int t = 0; t < NV; ++t)
        acc[t] = wave_sum(acc[t]);
    if (L.wave_ok && lane == 0) {
        float *dst = a.pdw + ((size_t)L.c * a.nseg + L.seg) * (K * K);
#pragma unroll
        for (int t = 0; t < K * K; ++t)
            dst[t] = acc[t];
        if (EXPAND) {
            a.psb[(size_t)L.c * a.nseg + L.seg] = acc[K * K];
            a.psr[(size_t)L.c * a.nseg + L.seg] = acc[K * K + 1];
        }
    }
}

// ---- host side -----------------------------------------------------------------------------

bool dwr_supported(const DwShape &s)
{
    const int w4 = (s.W + 3) / 4;
    return s.s == 1 && (s.k == 3 || s.k == 5) && s.Ho == s.H && s.Wo == s.W && s.H * w4 <= 64;
}

static DwrArgs dwr_args(const DwShape &s)
{
    DwrArgs a = {};
    a.N = s.N;
    a.C = s.C;
    a.H = s.H;
    a.W = s.W;
    a.W4 = (s.W + 3) / 4;
    a.WP = 4 * a.W4 + 8;
    a.runs = s.H * a.W4;
    a.PW = 64 / a.runs;
    if (a.PW > s.N)
        a.PW = s.N;
    // image ranges: enough wavefronts to fill the chip, at least four pipeline steps each
    int nseg = (4096 + s.C - 1) / s.C;
    const int cap = s.N / (4 * a.PW) > 1 ? s.N / (4 * a.PW) : 1;
    if (nseg > cap)
        nseg = cap;
    a.nper = (s.N + nseg - 1) / nseg;
    a.nper = (a.nper + a.PW - 1) / a.PW * a.PW;
    a.nseg = (s.N + a.nper - 1) / a.nper;
    a.divRuns = make_div((uint32_t)a.runs);
    a.divW4 = make_div((uint32_t)a.W4);
    a.divNseg = make_div((uint32_t)a.nseg);
    return a;
}

int dwr_num_partials(const DwShape &s) { return dwr_args(s).nseg; }

static size_t dwr_lds(const DwrArgs &a, int k, int tiles)
{
    const int p = (k - 1) / 2;
    return sizeof(float) * 4 * (size_t)(2 * tiles * a.PW) * (a.H + 2 * p) * a.WP;
}

template <typename KERN>
static hipError_t dwr_launch(KERN kern, const DwrArgs &a, size_t lds, hipStream_t st)
{
    if (lds > 65536) {
        hipError_t e = hipFuncSetAttribute((const void *)kern,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
    }
    const long long slots = (long long)a.C * a.nseg;
    hipLaunchKernelGGL(kern, dim3((unsigned)((slots + 3) / 4)), dim3(256), lds, st, a);
    return hipGetLastError();
}

#define MBK_DWR_GO(KERNEL, T, K)                                                                  \
    {                                                                                             \
        if (gv == 4)                                                                              \
            return ex ? dwr_launch(KERNEL<T, K, 4, true>, a, lds, st)                             \
                      : dwr_launch(KERNEL<T, K, 4, false>, a, lds, st);                           \
        if (gv == 2)                                                                              \
            return ex ? dwr_launch(KERNEL<T, K, 2, true>, a, lds, st)                             \
                      : dwr_launch(KERNEL<T, K, 2, false>, a, lds, st);                           \
        return ex ? dwr_launch(KERNEL<T, K, 1, true>, a, lds, st)                                 \
                  : dwr_launch(KERNEL<T, K, 1, false>, a, lds, st);                               \
    }

hipError_t launch_dwr_fwd(bool bf16, const DwShape &s, const void *e, const float *bn1,
                          const void *w_dw, void *d, float *psum, float *psq, const BnFin *fin,
                          hipStream_t st)
{
    DwrArgs a = dwr_args(s);
    if (fin)
        a.fin = *fin;
    a.e = e;
    a.bn1 = bn1;
    a.w = w_dw;
    a.d = d;
    a.psum = psum;
    a.psq = psq;
    const size_t lds = dwr_lds(a, s.k, 1);
    const bool ex = bn1 != nullptr;
    const int gv = s.W % 4 == 0 ? 4 : (s.W % 2 == 0 ? 2 : 1);
    if (bf16) {
        if (s.k == 3)
            MBK_DWR_GO(dwr_fwd_kernel, bf16_t, 3)
        MBK_DWR_GO(dwr_fwd_kernel, bf16_t, 5)
    }
    if (s.k == 3)
        MBK_DWR_GO(dwr_fwd_kernel, float, 3)
    MBK_DWR_GO(dwr_fwd_kernel, float, 5)
}

hipError_t launch_dwr_bwd(bool bf16, const DwBwdArgs &h, hipStream_t st)
{
    DwrArgs a = dwr_args(h.s);
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
    const DwShape &s = h.s;
    const size_t lds = dwr_lds(a, s.k, 1);
    const bool ex = h.bn1 != nullptr;
    const int gv = s.W % 4 == 0 ? 4 : (s.W % 2 == 0 ? 2 : 1);
    if (bf16) {
        if (s.k == 3)
            MBK_DWR_GO(dwr_bwd_kernel, bf16_t, 3)
        MBK_DWR_GO(dwr_bwd_kernel, bf16_t, 5)
    }
    if (s.k == 3)
        MBK_DWR_GO(dwr_bwd_kernel, float, 3)
    MBK_DWR_GO(dwr_bwd_kernel, float, 5)
}
#undef MBK_DWR_GO

} // namespace mbk
